"""Benchmark of the block-aggregation hot path on one MI355X.

One "step" = one pass of the whole hot path over one sampled mini-batch of the
products-shaped 3-layer GCN workload: build the bookkeeping (plans) of the
mini-batch's blocks, run the forward aggregation of every layer, then the
backward aggregation of every layer in reverse order.  All inputs are synthetic, seeded
and already resident in HBM when the timed region starts.

Prints ONE JSON line:
  value     aggregated GEdges/s = 2 * sum(E_layer) / step time (plan build included)
  roofline  achieved HBM GB/s of the dominant kernel from compulsory bytes
            (indptr + indices + unique source rows + output) against 8 TB/s
  cpu_baseline  the CPU oracle's parallel variant timed on the host cores
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
METRIC = "aggregated GEdges/s (fwd+bwd) and achieved HBM GB/s vs peak, 1 MI355X"

# HBM-side bytes per launch of the dominant kernel, from two rocprofv3 --pmc runs
# of this file (FETCH_SIZE, then WRITE_SIZE), each scaled by what the same counter
# reads for a plain 1 GiB copy (`--calibrate`): FETCH_SIZE counts 2 KiB units,
# WRITE_SIZE 1 KiB units on this stack.  Summary: profiles/pull_rows_config2_traffic.md.
# Key: (config, direction, layer).  Re-measure when the kernel's access pattern changes.
MEASURED_TRAFFIC_BYTES = {(2, "fwd", 0): int(632334.8 * 2048 + 208647.1 * 1024)}


def compulsory_bytes(rowptr_rows, nnz, used_in_rows, out_rows, feat, elem):
    """indptr + indices + each referenced input row once + every output row once."""
    return 4 * (rowptr_rows + 1) + 4 * nnz + used_in_rows * feat * elem + out_rows * feat * elem


MFMA_BF16_PEAK_TFLOPS = 2500.0     # dense bf16 matrix-core peak; an fp32 product costs six bf16 piece products
HIDDEN, CLASSES = 256, 47          # hidden width of the benchmark's configs; class count of the products-shaped stand-in


def idmap_leg(args, w, B, bg, torch, np, with_cpu):
    """Extra leg (not the headline metric): the ID map of the sample phase (paper Section 2.2;
    Section 4.3, Algorithm 2) for every hop of the same mini-batch: destination global IDs + sampled
    neighbour global IDs (scrambled 40-bit IDs) -> the block's `indices` and its source-node list."""
    dev = torch.device("cuda:0")
    hops = []
    for i, blk in enumerate(w.blocks):
        dst, nbr = bg.hop_global_ids(blk, w.seed + i)
        h = dict(dst=torch.from_numpy(dst).to(dev), nbr=torch.from_numpy(nbr).to(dev), host=(dst, nbr), blk=blk)
        n = dst.size + nbr.size
        h["ws"] = torch.empty(B.fastgl_idmap_workspace_bytes(dst.size, nbr.size), dtype=torch.uint8, device=dev)
        h["local"] = torch.empty(nbr.size, dtype=torch.int32, device=dev)
        h["uniq"] = torch.empty(n, dtype=torch.int64, device=dev)
        h["res"] = torch.empty(2, dtype=torch.int32, device=dev)
        # table fill + one entry touched per ID + IDs in + slot array out and in + indices out + source list out
        h["bytes"] = 16 * B.fastgl_idmap_table_slots(n) + 16 * n + 8 * n + 8 * n + 4 * nbr.size + 8 * blk.num_src
        hops.append(h)
    n_ids = sum(h["dst"].numel() + h["nbr"].numel() for h in hops)
    out = {"what": "global -> local IDs of every hop of the mini-batch (64-bit IDs, hash table with "
                   "compare-and-swap insertion); 'ordered' numbers by first appearance (reproducible), "
                   "'fused' by a counter as the paper's Algorithm 2 does",
           "ids_per_step": n_ids}
    reps = max(5, args.steps // 2)
    for mode in ("ordered", "fused"):
        def run():
            for h in hops:
                B.fastgl_idmap(h["dst"], h["nbr"], mode, h["local"], h["uniq"], h["res"], h["ws"])
        for _ in range(3):
            run()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(reps):
            run()
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / reps
        for h in hops:                       # the result of the last run must be a clean map of the right size
            U, bad = (int(x) for x in h["res"].cpu().numpy())
            assert bad == 0 and U == h["blk"].num_src, (mode, U, bad)
        out[mode] = {"ms": round(ms, 4), "gids_per_s": round(n_ids / ms / 1e6, 3),
                     "hbm_gbps_algorithmic": round(sum(h["bytes"] for h in hops) / ms / 1e6, 1),
                     "hbm_frac_of_peak": round(sum(h["bytes"] for h in hops) / ms / 1e6 / HBM_PEAK_GBPS, 4)}
    if with_cpu:
        import oracle
        t0 = time.perf_counter()
        for h in hops:
            oracle.idmap(*h["host"])
        dt = time.perf_counter() - t0
        out["cpu_oracle"] = {"gids_per_s": round(n_ids / dt / 1e9, 5), "cores": 1, "kind": "oracle",
                             "sample": f"one pass over all {len(hops)} hops (sort-based definition), {dt:.1f} s"}
    return out


def match_leg(args, w, B, bg, torch, np, with_cpu=False):
    """Extra leg (not the headline metric): the Match process and the Greedy Reorder Strategy (paper
    Section 4.1) over several mini-batches sampled from ONE products-shaped graph.  The raw features
    sit in a device-resident table; with Match only the rows that the last mini-batch does not hold
    are gathered from it, the rest is copied from the last mini-batch's feature matrix."""
    dev = torch.device("cuda:0")
    nb, feat, n_nodes = args.match_batches, w.widths[0], 2_400_000
    t0 = time.time()
    sets = bg.minibatch_node_sets(nb, w.seed)
    gen_s = time.time() - t0
    sizes = [len(x) for x in sets]
    offsets = [0] + [int(x) for x in np.cumsum(sizes)]
    allg = torch.from_numpy(np.concatenate(sets)).to(dev)
    gids = [allg[offsets[i]:offsets[i + 1]] for i in range(nb)]
    g = torch.Generator(device="cuda")
    g.manual_seed(w.seed + 2)
    table = torch.empty((n_nodes, feat), device=dev)
    for lo in range(0, n_nodes, 600_000):
        table[lo:lo + 600_000] = torch.randn((min(600_000, n_nodes - lo), feat), generator=g, device=dev)
    reps = max(5, args.steps // 2)

    def timed(fn):
        for _ in range(2):
            fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    ows = torch.empty(B.fastgl_overlap_workspace_bytes(allg.numel()), dtype=torch.uint8, device=dev)
    counts, viol = B.fastgl_overlap_counts(allg, offsets, ows)
    overlap_ms = timed(lambda: B.fastgl_overlap_counts(allg, offsets, ows))
    O = counts.cpu().numpy()
    assert int(viol.cpu()[0]) == 0
    order = B.fastgl_greedy_reorder(O.tolist(), sizes)

    def loaded(seq):
        return sizes[seq[0]] + sum(sizes[b] - int(O[a, b]) for a, b in zip(seq[:-1], seq[1:]))
    plain = list(range(nb))
    needed = sum(sizes)

    # one transition of the reordered list, timed step by step
    a, b = order[0], order[1]
    mws = torch.empty(B.fastgl_match_workspace_bytes(sizes[a], sizes[b]), dtype=torch.uint8, device=dev)
    src_row, load_pos, load_gid, res = B.fastgl_match(gids[a], gids[b], workspace=mws)
    n_load, bad = (int(x) for x in res.cpu().numpy())
    assert bad == 0 and n_load == sizes[b] - int(O[a, b])
    X_prev = B.fastgl_gather_rows(table, gids[a])
    X_load = torch.empty((sizes[b], feat), device=dev)
    X_new = torch.empty((sizes[b], feat), device=dev)
    match_ms = timed(lambda: B.fastgl_match(gids[a], gids[b], src_row, load_pos, load_gid, res, mws))
    gather_load_ms = timed(lambda: B.fastgl_gather_rows(table, load_gid[:n_load], out=X_load[:n_load]))
    assemble_ms = timed(lambda: B.fastgl_assemble_rows(X_prev, X_load, src_row, n_load, out=X_new))
    gather_all_ms = timed(lambda: B.fastgl_gather_rows(table, gids[b], out=X_new))
    B.fastgl_assemble_rows(X_prev, X_load, src_row, n_load, out=X_new)
    ref = B.fastgl_gather_rows(table, gids[b])
    assert torch.equal(X_new, ref), "Match + assemble must equal loading every row"
    row_bytes = feat * 4
    asm_bytes = 2 * sizes[b] * row_bytes + 4 * sizes[b]
    cpu = None
    if with_cpu:
        import oracle
        t0 = time.perf_counter()
        oracle.match(sets[a], sets[b])
        dt = time.perf_counter() - t0
        cpu = {"match_gids_per_s": round((sizes[a] + sizes[b]) / dt / 1e9, 5), "cores": 1, "kind": "oracle",
               "sample": f"the same transition (sort + binary search), {dt:.2f} s"}
    return {
        "cpu_oracle": cpu,
        "what": f"{nb} mini-batches sampled from one products-shaped graph; features ({feat} x f32) in a device table",
        "nodes_per_minibatch": sizes, "gen_seconds": round(gen_s, 1),
        "match_degree_mean": round(float(np.mean([O[i, j] / min(sizes[i], sizes[j]) for i in range(nb)
                                                  for j in range(i)])), 4),
        "rows_needed": needed, "rows_loaded_sampled_order": loaded(plain), "rows_loaded_reordered": loaded(order),
        "load_fraction_sampled_order": round(loaded(plain) / needed, 4),
        "load_fraction_reordered": round(loaded(order) / needed, 4),
        "order": order,
        "overlap_counts_ms": round(overlap_ms, 4),
        "overlap_gids_per_s": round(allg.numel() / overlap_ms / 1e6, 3),
        "transition": {"from": a, "to": b, "n_new": sizes[b], "n_load": n_load,
                       "match_ms": round(match_ms, 4),
                       "match_gids_per_s": round((sizes[a] + sizes[b]) / match_ms / 1e6, 3),
                       "gather_loaded_rows_ms": round(gather_load_ms, 4),
                       "assemble_ms": round(assemble_ms, 4),
                       "assemble_hbm_gbps": round(asm_bytes / assemble_ms / 1e6, 1),
                       "assemble_hbm_frac_of_peak": round(asm_bytes / assemble_ms / 1e6 / HBM_PEAK_GBPS, 4),
                       "with_match_ms": round(match_ms + gather_load_ms + assemble_ms, 4),
                       "gather_every_row_ms": round(gather_all_ms, 4)},
    }


def edge_leg(args, w, layers, workspace, B, torch, np, with_cpu=False):
    """Extra leg (not the headline metric): one attention-style pass over the input-layer block with
    learned edge weights - the attention logits of a GAT head from per-node terms, their softmax over
    every destination's incoming edges, the aggregation weighted by it (SUM mode), and the backward
    pass: dL/dw per edge (sampled dot products), the softmax backward, the gradients of the per-node
    terms, the weighted backward aggregation."""
    L = layers[0]
    blk, feat, dev = L["blk"], L["feat"], L["X"].device
    g = torch.Generator(device="cuda")
    g.manual_seed(w.seed + 3)
    el = torch.randn(blk.num_dst, generator=g, device=dev)
    er = torch.randn(blk.num_src, generator=g, device=dev)
    score = torch.empty(blk.num_edges, device=dev)
    g_el, g_er = torch.empty_like(el), torch.empty_like(er)
    alpha, gw, gs = torch.empty_like(score), torch.empty_like(score), torch.empty_like(score)
    ews = torch.empty(B.fastgl_edge_workspace_bytes(blk.num_dst, blk.num_edges), dtype=torch.uint8, device=dev)
    plan = B.fastgl_block_plan_create(L["indptr"], L["indices"], blk.num_src, B.PLAN_ALL | B.PLAN_PERM)
    reps = max(5, args.steps // 2)

    def timed(fn):
        for _ in range(2):
            fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps
    t = {
        "score_fwd": timed(lambda: B.fastgl_edge_score_fwd(L["indptr"], L["indices"], el, er, 0.2, score)),
        "softmax_fwd": timed(lambda: B.fastgl_edge_softmax_fwd(L["indptr"], score, alpha, ews)),
        "aggregate_fwd_weighted": timed(lambda: B.fastgl_block_aggregate_fwd(
            L["indptr"], L["indices"], alpha, blk.num_src, "sum", L["X"], out=L["out"], plan=plan, workspace=workspace)),
        "edge_weight_grad": timed(lambda: B.fastgl_edge_weight_grad(
            L["indptr"], L["indices"], blk.num_src, "sum", L["X"], L["G"], grad_w=gw, workspace=ews)),
        "softmax_bwd": timed(lambda: B.fastgl_edge_softmax_bwd(L["indptr"], alpha, gw, gs, ews)),
        "score_bwd": timed(lambda: B.fastgl_edge_score_bwd(L["indptr"], L["indices"], el, er, 0.2, gs, plan=plan,
                                                               grad_el=g_el, grad_er=g_er)),
        "aggregate_bwd_weighted": timed(lambda: B.fastgl_block_aggregate_bwd(
            L["indptr"], L["indices"], alpha, blk.num_src, "sum", L["G"], grad_X=L["dX"], plan=plan, workspace=workspace)),
    }
    # compulsory bytes of the weight gradient: CSR + every referenced X row once + every grad row once + E results
    byt = L["bytes_fwd"] + 4 * blk.num_edges
    ach = byt / t["edge_weight_grad"] / 1e6
    cpu = None
    if with_cpu:
        import oracle
        rows = min(blk.num_dst, 100_000)                 # a bounded sample: the first rows of the block
        ne = int(blk.indptr[rows])
        Xh, Gh = L["X"].cpu().numpy(), L["G"][:rows].cpu().numpy()
        t0 = time.perf_counter()
        oracle.edge_weight_grad(blk.indptr[:rows + 1], blk.indices[:ne], blk.num_src, "sum", "f32", Xh, Gh)
        oracle.edge_softmax_fwd(blk.indptr[:rows + 1], score[:ne].cpu().numpy())
        dt = time.perf_counter() - t0
        cpu = {"gedges_per_s": round(2 * ne / dt / 1e9, 5), "cores": 1, "kind": "oracle",
               "sample": f"weight gradient + softmax forward over the first {rows} rows ({ne} edges), {dt:.2f} s"}
    return {"cpu_oracle": cpu, "what": f"input-layer block (E={blk.num_edges}, F={feat}, f32), SUM mode with learned weights",
            "ms": {k: round(v, 4) for k, v in t.items()}, "total_ms": round(sum(t.values()), 4),
            "gedges_per_s": round(len(t) * blk.num_edges / sum(t.values()) / 1e6, 3),
            "roofline": {"bound": "hbm", "kernel": "k_edge_dot (dL/dw per edge)", "achieved": round(ach, 1),
                         "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(ach / HBM_PEAK_GBPS, 4), "traffic": None,
                         "launch_ms": round(t["edge_weight_grad"], 4), "algorithmic_bytes": int(byt)}}


def locality_leg(args, w, layers, workspace, B, bg, torch, np):
    """Extra leg (not the headline metric): the input-layer block with the same sizes and row lengths
    but its neighbours re-drawn inside a band around the diagonal (blockgen.banded_like), i.e. a block
    with the locality that a graph with community structure has under a locality-preserving node
    order.  Same kernels, same launch shapes; shows what the aggregation reaches when the gathered
    rows can be reused out of L2, which the Chung-Lu workload cannot offer."""
    L = layers[0]
    blk, feat, dev = L["blk"], L["feat"], L["X"].device
    elem = L["X"].element_size()
    res = {"what": f"input-layer block, neighbours re-drawn within a band of W source rows (E={blk.num_edges}, F={feat})",
           "bands": []}
    reps = max(5, args.steps // 2)
    for window in (1024, 16384, 262144):
        bb = bg.banded_like(blk, window, w.seed + 17)
        ip, ix = torch.from_numpy(bb.indptr).to(dev), torch.from_numpy(bb.indices).to(dev)
        dout = np.bincount(bb.indices, minlength=bb.num_src)
        byt_f = compulsory_bytes(bb.num_dst, bb.num_edges, int((dout > 0).sum()), bb.num_dst, feat, elem)
        byt_b = compulsory_bytes(bb.num_src, bb.num_edges, int((np.diff(bb.indptr) > 0).sum()), bb.num_src, feat, elem)
        plan = B.fastgl_block_plan_create(ip, ix, bb.num_src, B.PLAN_ALL, L["plan_mem"])

        def timed(fn):
            for _ in range(2):
                fn()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            e0.record()
            for _ in range(reps):
                fn()
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / reps
        f = timed(lambda: B.fastgl_block_aggregate_fwd(ip, ix, None, bb.num_src, w.mode, L["X"], out=L["out"], plan=plan,
                                                       workspace=workspace))
        b = timed(lambda: B.fastgl_block_aggregate_bwd(ip, ix, None, bb.num_src, w.mode, L["G"], grad_X=L["dX"], plan=plan,
                                                       workspace=workspace))
        res["bands"].append({"W": window, "unique_src_rows": int((dout > 0).sum()), "fwd_ms": round(f, 4), "bwd_ms": round(b, 4),
                             "fwd_gbps_compulsory": round(byt_f / f / 1e6, 1), "fwd_frac_of_peak": round(byt_f / f / 1e6 / HBM_PEAK_GBPS, 4),
                             "bwd_gbps_compulsory": round(byt_b / b / 1e6, 1), "bwd_frac_of_peak": round(byt_b / b / 1e6 / HBM_PEAK_GBPS, 4)})
    return res


def gcn_step_leg(args, w, layers, workspace, make_plans, B, torch, np, with_cpu=False):
    """Extra leg (not the headline metric): one training step of the whole sampled GCN on the same
    mini-batch - per layer aggregate (Eq. 1) then update (Eq. 2, Y = act(H W + b)), ReLU between
    layers, a synthetic upstream gradient at the class scores, then the backward pass: gradients of
    every W and b, and of every layer input except the raw features."""
    dev, tdt = layers[0]["X"].device, layers[0]["X"].dtype      # bf16 workloads keep bf16 activations and weights
    g = torch.Generator(device="cuda")
    g.manual_seed(w.seed + 1)
    n = len(layers)
    outs = [HIDDEN] * (n - 1) + [CLASSES]
    P = []
    for i, L in enumerate(layers):
        M, K, N = L["blk"].num_dst, L["feat"], outs[i]
        if i + 1 < n:
            assert layers[i + 1]["feat"] == N and layers[i + 1]["blk"].num_src == M
        p = dict(M=M, K=K, N=N, relu=i + 1 < n)
        p["W"] = (torch.randn((K, N), generator=g, device=dev) / K ** 0.5).to(tdt)
        p["b"] = torch.randn((N,), generator=g, device=dev) * 0.1
        p["H"] = torch.empty((M, K), device=dev, dtype=tdt)
        p["Y"] = torch.empty((M, N), device=dev, dtype=tdt)
        p["dW"], p["db"] = torch.empty((K, N), device=dev), torch.empty((N,), device=dev)
        p["dH"] = torch.empty((M, K), device=dev, dtype=tdt) if i > 0 else None
        p["dX"] = torch.empty((L["blk"].num_src, K), device=dev, dtype=tdt) if i > 0 else None
        p["ws"] = torch.empty(max(256, B.fastgl_update_bwd_workspace_bytes(M, K, N)), dtype=torch.uint8, device=dev)
        P.append(p)
    dlogits = torch.randn((P[-1]["M"], CLASSES), generator=g, device=dev).to(tdt)
    ev = {}

    def mark(key, fn, record):
        if not record:
            return fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        fn()
        e1.record()
        ev.setdefault(key, []).append((e0, e1))

    side = None

    def step(record=False):
        plans = None

        def build():
            nonlocal plans
            plans = make_plans()
        mark("plan", build, record)
        x = layers[0]["X"]
        for i, (L, p) in enumerate(zip(layers, P)):
            mark(f"agg_fwd{i}", lambda: B.fastgl_block_aggregate_fwd(
                L["indptr"], L["indices"], None, L["blk"].num_src, w.mode, x, out=p["H"], plan=plans[i],
                workspace=workspace), record)
            mark(f"upd_fwd{i}", lambda: B.fastgl_update_fwd(p["H"], p["W"], p["b"], p["relu"], p["Y"]), record)
            x = p["Y"]
        grad = dlogits
        for i in reversed(range(n)):
            L, p = layers[i], P[i]
            if i > 0 and side is not None and not record:
                # dW/db of this layer do not feed the rest of the backward pass: they run on a second
                # stream next to the backward aggregation (matrix-core bound next to bandwidth bound)
                ready = torch.cuda.Event()
                ready.record()
                B.fastgl_update_bwd(p["H"], p["W"], p["Y"] if p["relu"] else None, grad, p["relu"], want=(),
                                    dH=p["dH"], workspace=p["ws"])
                with torch.cuda.stream(side):
                    side.wait_event(ready)
                    B.fastgl_update_bwd(p["H"], p["W"], p["Y"] if p["relu"] else None, grad, p["relu"], want=(),
                                        dW=p["dW"], db=p["db"], workspace=p["ws"])
            else:
                mark(f"upd_bwd{i}", lambda: B.fastgl_update_bwd(
                    p["H"], p["W"], p["Y"] if p["relu"] else None, grad, p["relu"], want=(), dH=p["dH"], dW=p["dW"],
                    db=p["db"], workspace=p["ws"]), record)
            if i > 0:
                mark(f"agg_bwd{i}", lambda: B.fastgl_block_aggregate_bwd(
                    L["indptr"], L["indices"], None, L["blk"].num_src, w.mode, p["dH"], grad_X=p["dX"],
                    plan=plans[i], workspace=workspace), record)
                grad = p["dX"]
        if side is not None and not record:
            torch.cuda.current_stream().wait_stream(side)

    for _ in range(max(2, args.warmup // 2)):
        step()
    torch.cuda.synchronize()
    steps = max(5, args.steps // 2)
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    # the same step with the weight gradients of the inner layers on a second stream
    side = torch.cuda.Stream()
    for _ in range(2):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    ms_two = (time.perf_counter() - t0) * 1e3 / steps
    side = None
    for _ in range(steps):
        step(record=True)
    torch.cuda.synchronize()
    parts = {k: float(np.mean([a.elapsed_time(b) for a, b in v])) for k, v in ev.items()}
    flops_fwd = [2.0 * p["M"] * p["K"] * p["N"] for p in P]
    flops = sum(flops_fwd) + sum(f * (2 if i > 0 else 1) for i, f in enumerate(flops_fwd))
    upd_ms = sum(v for k, v in parts.items() if k.startswith("upd"))
    agg_ms = sum(v for k, v in parts.items() if k.startswith("agg"))
    dom_ms = parts["upd_fwd0"]
    ach = flops_fwd[0] / (dom_ms * 1e-3) / 1e12
    pieces = 1 if tdt == torch.bfloat16 else 6
    cpu = None
    if with_cpu and tdt == torch.float32:
        import oracle
        rows = min(P[0]["M"], 4000)                      # a bounded sample: the first rows of the input layer
        Hh, Wh, bh = P[0]["H"][:rows].cpu().numpy(), P[0]["W"].cpu().numpy(), P[0]["b"].cpu().numpy()
        t0 = time.perf_counter()
        oracle.update_fwd(Hh, Wh, bh, True)
        dt = time.perf_counter() - t0
        cpu = {"update_tflops": round(2.0 * rows * P[0]["K"] * P[0]["N"] / dt / 1e12, 6), "cores": 1, "kind": "oracle",
               "sample": f"forward update of the first {rows} rows of the input layer (fp64 triple loop), {dt:.2f} s"}
    return {
        "cpu_oracle": cpu,
        "what": "plans + per layer [aggregate, act(H W + b)] forward, then backward (dW, db every layer; "
                "dH and the backward aggregation for every layer but the input one); widths "
                f"{[p['K'] for p in P]} -> {outs}",
        "ms_per_step": round(ms, 4),
        "ms_per_step_two_streams": round(ms_two, 4),
        "parts_ms": {k: round(v, 4) for k, v in parts.items()},
        "aggregation_ms": round(agg_ms, 4), "update_ms": round(upd_ms, 4), "plan_ms": round(parts["plan"], 4),
        "update_flops_per_step": flops,
        "update_tflops": round(flops / (upd_ms * 1e-3) / 1e12, 2),
        "roofline": {"bound": "mfma", "kernel": "k_update_gemm, forward of the input layer "
                                                  f"(M={P[0]['M']}, K={P[0]['K']}, N={P[0]['N']}; bf16 MFMA, "
                                                  f"{pieces} piece product(s) per element product)",
                     "achieved": round(ach, 2), "peak": round(MFMA_BF16_PEAK_TFLOPS / pieces, 1), "unit": "TFLOP/s",
                     "frac": round(ach * pieces / MFMA_BF16_PEAK_TFLOPS, 4), "traffic": None,
                     "mfma_tflops_executed": round(ach * pieces, 1),
                     "launch_ms": round(dom_ms, 4), "algorithmic_flops": flops_fwd[0]},
    }


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=2, help="workload 1..5 (2 = the headline)")
    ap.add_argument("--width", type=int, default=32, help="feature width of config 5")
    ap.add_argument("--fanout-order", default="A", choices=["A", "B"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-idmap", action="store_true",
                    help="skip the extra leg that times the ID map (global -> local IDs) of the mini-batch's hops")
    ap.add_argument("--no-match", action="store_true",
                    help="skip the extra leg that times Match / Reorder over several mini-batches of one graph")
    ap.add_argument("--match-batches", type=int, default=4)
    ap.add_argument("--no-edge", action="store_true",
                    help="skip the extra leg that times the learned-edge-weight path (edge softmax, weight gradient)")
    ap.add_argument("--locality", action="store_true",
                    help="also run the aggregation on banded copies of the input-layer block (neighbours re-drawn "
                         "near the diagonal): what the kernels reach when gathered rows can be reused out of L2")
    ap.add_argument("--no-gcn-step", action="store_true",
                    help="skip the extra leg that times the whole sampled GCN (aggregation + update phase)")
    ap.add_argument("--verbose", action="store_true")
    ap.add_argument("--calibrate", action="store_true",
                    help="only run a plain 1 GiB device copy a few times (reference for rocprofv3 byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU; --gpus must be 1 "
              "(data-parallel training gives every GPU its own mini-batch and needs no "
              "communication in the aggregation path)", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    import blockgen as bg
    from paper_2409_14939_amd import binding as B

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")

    if args.calibrate:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)     # 1 GiB
        dst = torch.empty_like(src)
        for _ in range(4):
            dst.copy_(src)                                             # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        print(json.dumps({"calibrate": "4 device copies of 1 GiB (1073741824 bytes read and written each)"}))
        return 0

    t0 = time.time()
    w = bg.make_config(args.config, fanout_order=args.fanout_order, width=args.width)
    gen_s = time.time() - t0
    tdt = torch.float32 if w.dtype == "f32" else torch.bfloat16
    elem = 4 if w.dtype == "f32" else 2

    layers = []
    g = torch.Generator(device="cuda")
    g.manual_seed(w.seed)
    ws_bytes = 0
    for blk, feat in zip(w.blocks, w.widths):
        L = dict(blk=blk, feat=feat)
        L["indptr"] = torch.from_numpy(blk.indptr).to(dev)
        L["indices"] = torch.from_numpy(blk.indices).to(dev)
        L["X"] = torch.randn((blk.num_src, feat), generator=g, device=dev, dtype=torch.float32).to(tdt)
        L["G"] = torch.randn((blk.num_dst, feat), generator=g, device=dev, dtype=torch.float32).to(tdt)
        L["out"] = torch.empty((blk.num_dst, feat), device=dev, dtype=tdt)
        L["dX"] = torch.empty((blk.num_src, feat), device=dev, dtype=tdt)
        L["plan_mem"] = torch.empty(B.fastgl_block_plan_bytes(blk.num_dst, blk.num_src, blk.num_edges),
                                    dtype=torch.uint8, device=dev)
        ws_bytes = max(ws_bytes, B.fastgl_block_workspace_bytes(blk.num_dst, blk.num_src, blk.num_edges,
                                                                feat, w.dtype))
        din = np.diff(blk.indptr)
        dout = np.bincount(blk.indices, minlength=blk.num_src)
        L["bytes_fwd"] = compulsory_bytes(blk.num_dst, blk.num_edges, int((dout > 0).sum()), blk.num_dst, feat, elem)
        L["bytes_bwd"] = compulsory_bytes(blk.num_src, blk.num_edges, int((din > 0).sum()), blk.num_src, feat, elem)
        layers.append(L)
    workspace = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
    table = gid = None
    gather_bytes = 0
    if w.src_gid is not None:
        # config 4: the raw features sit in a device-resident table and are gathered by global id
        feat0 = w.widths[0]
        table = torch.empty((w.table_rows, feat0), dtype=tdt, device=dev)
        for lo in range(0, w.table_rows, 8_000_000):
            hi = min(w.table_rows, lo + 8_000_000)
            table[lo:hi] = torch.randn((hi - lo, feat0), generator=g, device=dev, dtype=torch.float32).to(tdt)
        gid = torch.from_numpy(w.src_gid).to(dev)
        gather_bytes = 8 * gid.numel() + 2 * gid.numel() * feat0 * elem
    total_edges = w.total_edges()
    bytes_step = sum(L["bytes_fwd"] + L["bytes_bwd"] for L in layers) + gather_bytes

    def make_plans():
        """Bookkeeping of every block of the mini-batch (transpose CSR, degrees, scale
        factors, degree buckets), built together: each stage is one launch for all layers."""
        return B.fastgl_block_plan_create_many([(L["indptr"], L["indices"], L["blk"].num_src) for L in layers],
                                               B.PLAN_ALL, [L["plan_mem"] for L in layers])

    def fwd(L, plan):
        B.fastgl_block_aggregate_fwd(L["indptr"], L["indices"], None, L["blk"].num_src, w.mode, L["X"],
                                     out=L["out"], plan=plan, workspace=workspace)

    def bwd(L, plan):
        B.fastgl_block_aggregate_bwd(L["indptr"], L["indices"], None, L["blk"].num_src, w.mode, L["G"],
                                     grad_X=L["dX"], plan=plan, workspace=workspace)

    # the dominant kernel: forward pull over the input-layer block
    dom = max(range(len(layers)), key=lambda i: layers[i]["bytes_fwd"])
    dom_ev = []

    def step(timed_dom=False):
        if table is not None:
            B.fastgl_gather_rows(table, gid, out=layers[0]["X"])
        plans = make_plans()
        for i, L in enumerate(layers):
            if timed_dom and i == dom:
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                fwd(L, plans[i])
                e1.record()
                dom_ev.append((e0, e1))
            else:
                fwd(L, plans[i])
        for L, p in zip(reversed(layers), reversed(plans)):
            bwd(L, p)
        return plans

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(timed_dom=True)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_step = wall * 1e3 / args.steps
    dom_ms = float(np.mean([a.elapsed_time(b) for a, b in dom_ev]))

    # breakdown (not part of the headline): plan / forward / backward, and a step
    # with plans built once ("cached plan")
    def timed(fn, reps):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    reps = max(5, args.steps // 2)
    plans = make_plans()
    plan_ms = timed(make_plans, reps)
    fwd_ms = timed(lambda: [fwd(L, p) for L, p in zip(layers, plans)], reps)
    bwd_ms = timed(lambda: [bwd(L, p) for L, p in zip(reversed(layers), reversed(plans))], reps)
    per_layer = []
    for i, (L, p) in enumerate(zip(layers, plans)):
        f = timed(lambda: fwd(L, p), reps)
        b = timed(lambda: bwd(L, p), reps)
        per_layer.append(dict(layer=i, num_dst=L["blk"].num_dst, num_src=L["blk"].num_src,
                              E=L["blk"].num_edges, feat=L["feat"],
                              fwd_ms=round(f, 4), bwd_ms=round(b, 4),
                              fwd_gbps=round(L["bytes_fwd"] / f / 1e6, 1),
                              bwd_gbps=round(L["bytes_bwd"] / b / 1e6, 1)))

    value = 2.0 * total_edges / (ms_step * 1e-3) / 1e9
    domL = layers[dom]
    achieved = domL["bytes_fwd"] / (dom_ms * 1e-3) / 1e9
    traffic = MEASURED_TRAFFIC_BYTES.get((args.config, "fwd", dom))
    result = {
        "metric": METRIC,
        "value": round(value, 4),
        "unit": "GEdges/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32" if w.dtype == "f32" else "bf16",
        "data": "synthetic",
        "config": {"workload": w.name, "config_id": args.config, "seed": w.seed,
                   "fanout_order": args.fanout_order, "mode": w.mode, "widths": w.widths,
                   "total_edges": total_edges, "accumulate": "f64" if w.dtype == "f32" else "f32",
                   "step": "plans of all layers (one batched call); forward per layer; backward per layer (reverse)"},
        "hbm_gbps_compulsory": round(bytes_step / (ms_step * 1e-3) / 1e9, 1),
        "hbm_frac_of_peak": round(bytes_step / (ms_step * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
        "compulsory_bytes_per_step": int(bytes_step),
        "breakdown_ms": {"plan": round(plan_ms, 4), "fwd": round(fwd_ms, 4), "bwd": round(bwd_ms, 4),
                         "cached_plan_step": round(fwd_ms + bwd_ms, 4)},
        "value_cached_plan": round(2.0 * total_edges / ((fwd_ms + bwd_ms) * 1e-3) / 1e9, 4),
        "hbm_frac_cached_plan": round(bytes_step / ((fwd_ms + bwd_ms) * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
        "layers": per_layer,
        "roofline": {"bound": "hbm", "kernel": f"forward aggregation call, layer {dom} (k_pull_rows)",
                     "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": traffic,
                     "launch_ms": round(dom_ms, 4), "algorithmic_bytes": int(domL["bytes_fwd"])},
        "gen_seconds": round(gen_s, 2),
    }

    if not args.no_idmap:
        result["idmap"] = idmap_leg(args, w, B, bg, torch, np, with_cpu=not args.no_cpu_baseline)
    if not args.no_match and args.config == 2:
        result["match_reorder"] = match_leg(args, w, B, bg, torch, np, with_cpu=not args.no_cpu_baseline)
    if not args.no_edge and w.dtype == "f32":
        result["edge_weights"] = edge_leg(args, w, layers, workspace, B, torch, np,
                                          with_cpu=not args.no_cpu_baseline)
    if args.locality and args.config == 2:
        result["locality_probe"] = locality_leg(args, w, layers, workspace, B, bg, torch, np)
    if not args.no_gcn_step and len(layers) > 1:
        result["gcn_step"] = gcn_step_leg(args, w, layers, workspace, make_plans, B, torch, np,
                                          with_cpu=not args.no_cpu_baseline)

    if not args.no_cpu_baseline:
        import oracle
        # bounded sample: whole passes over the same workload, layer by layer, repeated
        # until about 12 s of CPU work (at least one full pass over every layer)
        budget, spent, edges_done, passes = 12.0, 0.0, 0, 0
        host = []
        for L in layers:
            if w.dtype == "f32":
                host.append((L["X"].cpu().numpy(), L["G"].cpu().numpy()))
            else:
                host.append((L["X"].view(torch.int16).cpu().numpy().view(np.uint16),
                             L["G"].view(torch.int16).cpu().numpy().view(np.uint16)))
        while spent < budget:
            for L, (Xh, Gh) in zip(layers, host):
                blk = L["blk"]
                t0 = time.perf_counter()
                oracle.par_aggregate_fwd(blk.indptr, blk.indices, None, blk.num_src, w.mode, w.dtype, Xh)
                oracle.par_aggregate_bwd(blk.indptr, blk.indices, None, blk.num_src, w.mode, w.dtype, Gh)
                spent += time.perf_counter() - t0
                edges_done += 2 * blk.num_edges
            passes += 1
        sample = f"{passes} full fwd+bwd passes over all {len(layers)} layers"
        result["cpu_baseline"] = {
            "value": round(edges_done / spent / 1e9, 5), "unit": "GEdges/s",
            "cores": oracle.num_threads(), "kind": "oracle",
            "sample": f"parallel oracle variant (fp32 accumulate, OpenMP over rows, backward through its own "
                      f"transpose): {sample} of the same workload, {spent:.1f} s of CPU time",
        }
    if args.verbose:
        print(json.dumps(result, indent=1), file=sys.stderr)
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
