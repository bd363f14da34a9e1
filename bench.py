"""Benchmark of the block-aggregation hot path on one MI355X.

One "step" = one pass of the whole hot path over one sampled mini-batch of the
products-shaped 3-layer GCN workload: build the bookkeeping (plans) of the
mini-batch's blocks, run the forward aggregation of every layer, then the
backward aggregation of every layer in reverse order.  All inputs are synthetic, seeded
and already resident in HBM when the timed region starts.

Timing: every step is bracketed by a pair of HIP events on the launch stream; `ms_per_step` is
the median of the timed steps (>= 50 by default), `ms_per_step_wall` the wall-clock mean of the
same steps between two device synchronisations.  Repetitions are cache-cold: a workload whose
buffers (features, outputs, gradients) take less than 512 MB (twice the 256 MB Infinity Cache)
rotates over up to 8 independent copies of them, and if that is still less it runs an untimed
512 MB fill between the steps.

Prints ONE JSON line:
  value     aggregated GEdges/s = 2 * sum(E_layer) / step time (plan build included)
  roofline  achieved HBM GB/s of the dominant kernel from compulsory bytes
            (indptr + indices + unique source rows + output) against 8 TB/s
  cpu_baseline  the CPU oracle's parallel variant timed on the host cores
  other_configs  the same measurement, shorter, for the other four workloads
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

# HBM-side bytes per launch are not measured in this run (byte counters need rocprofv3): they are
# read from a tracked table of earlier rocprofv3 --pmc runs of this file (FETCH_SIZE, then
# WRITE_SIZE, each scaled by what the same counter reads for a plain 1 GiB copy, `--calibrate`).
# A launch without an entry reports null.  Re-measure when a kernel's access pattern changes.
TRAFFIC_TABLE = os.path.join(ROOT, "profiles", "traffic_counters.txt")
FETCH_UNIT, WRITE_UNIT = 2048, 1024     # bytes per count of FETCH_SIZE / WRITE_SIZE on this stack


def load_traffic_table():
    """Lines: config width layer direction FETCH_SIZE WRITE_SIZE (counter means per dispatch)."""
    table = {}
    try:
        with open(TRAFFIC_TABLE) as f:
            for line in f:
                line = line.split("#", 1)[0].split()
                if len(line) == 6:
                    cfg, width, layer, direction, fetch, write = line
                    table[(int(cfg), int(width), int(layer), direction)] = int(float(fetch) * FETCH_UNIT +
                                                                               float(write) * WRITE_UNIT)
    except OSError:
        pass
    return table


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
        # (entries: 16 bytes in the ordered mode, 8-byte key + 4-byte local ID in the fused one)
        h["bytes"] = {mode: per * B.fastgl_idmap_table_slots(n) + per * n + 8 * n + 8 * n + 4 * nbr.size + 8 * blk.num_src
                      for mode, per in (("ordered", 16), ("fused", 12))}
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
                     "hbm_gbps_algorithmic": round(sum(h["bytes"][mode] for h in hops) / ms / 1e6, 1),
                     "hbm_frac_of_peak": round(sum(h["bytes"][mode] for h in hops) / ms / 1e6 / HBM_PEAK_GBPS, 4)}
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
        # the bandwidth-bound kernel of this leg; the match and overlap kernels are bound by random
        # accesses into the hash table (one 128-byte line per ID for 16 useful bytes), not by bytes
        "roofline": {"bound": "hbm", "kernel": "k_assemble_rows (new feature matrix from reused and loaded rows)",
                     "achieved": round(asm_bytes / assemble_ms / 1e6, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(asm_bytes / assemble_ms / 1e6 / HBM_PEAK_GBPS, 4), "traffic": None,
                     "launch_ms": round(assemble_ms, 4), "algorithmic_bytes": int(asm_bytes)},
        "match_lines_per_s": {"what": "hash-table lines touched per second by k_match_insert_prev + k_match_probe "
                                      "(one 128-byte line per ID of either mini-batch)",
                              "glines_per_s": round((sizes[a] + sizes[b]) / match_ms / 1e6, 3),
                              "line_gbps": round((sizes[a] + sizes[b]) * 128 / match_ms / 1e6, 1)},
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
    fuse_last = B.fastgl_layer_fwd_fuses(P[-1]["K"], P[-1]["N"], "f32" if tdt == torch.float32 else "bf16")
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
            if fuse_last and i == n - 1:
                # the class-score layer: aggregation and update in one kernel (H kept for the backward pass)
                mark(f"layer_fwd{i}", lambda: B.fastgl_layer_fwd(
                    L["indptr"], L["indices"], None, L["blk"].num_src, w.mode, x, p["W"], p["b"], p["relu"],
                    H=p["H"], Y=p["Y"], plan=plans[i], workspace=workspace), record)
            else:
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
    parts = {k: float(np.median([a.elapsed_time(b) for a, b in v])) for k, v in ev.items()}
    flops_fwd = [2.0 * p["M"] * p["K"] * p["N"] for p in P]
    flops = sum(flops_fwd) + sum(f * (2 if i > 0 else 1) for i, f in enumerate(flops_fwd))
    upd_ms = sum(v for k, v in parts.items() if k.startswith("upd"))
    agg_ms = sum(v for k, v in parts.items() if k.startswith("agg") or k.startswith("layer"))
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
                f"{[p['K'] for p in P]} -> {outs}" + ("; the last layer's forward is one fused kernel "
                                                      "(fastgl_layer_fwd, counted with the aggregation)" if fuse_last else ""),
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


def measure_copy_gbps(torch):
    """Plain device copy of 1 GiB (read + write), the practical streaming ceiling of this GPU."""
    src = torch.ones(1 << 28, dtype=torch.float32, device="cuda:0")
    dst = torch.empty_like(src)
    for _ in range(2):
        dst.copy_(src)
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(7)]
    for a, b in ev:
        a.record()
        dst.copy_(src)
        b.record()
    torch.cuda.synchronize()
    ms = sorted(a.elapsed_time(b) for a, b in ev)[len(ev) // 2]
    return 2.0 * src.numel() * 4 / (ms * 1e-3) / 1e9


class Workload:
    """Device buffers of one configuration: index arrays, plan memory, and `nsets` independent
    copies of (X, G, out, dX) per layer that the timed loops rotate over."""

    def __init__(self, cfg, width, fanout_order, B, bg, torch, np, max_sets=8):
        self.cfg, self.width = cfg, width
        t0 = time.time()
        self.w = w = bg.make_config(cfg, fanout_order=fanout_order, width=width)
        self.gen_s = time.time() - t0
        dev = torch.device("cuda:0")
        self.tdt = tdt = torch.float32 if w.dtype == "f32" else torch.bfloat16
        self.elem = elem = 4 if w.dtype == "f32" else 2
        foot = sum((2 * b.num_src + 2 * b.num_dst) * f * elem for b, f in zip(w.blocks, w.widths))
        self.footprint = foot
        self.nsets = nsets = max(1, min(max_sets, -(-(512 << 20) // foot)))
        self.flush = torch.empty(512 << 20, dtype=torch.uint8, device=dev) if nsets * foot < (512 << 20) else None
        g = torch.Generator(device="cuda")
        g.manual_seed(w.seed)
        self.layers, ws_bytes = [], 0
        for blk, feat in zip(w.blocks, w.widths):
            L = dict(blk=blk, feat=feat)
            L["indptr"] = torch.from_numpy(blk.indptr).to(dev)
            L["indices"] = torch.from_numpy(blk.indices).to(dev)
            L["Xs"] = [torch.randn((blk.num_src, feat), generator=g, device=dev, dtype=torch.float32).to(tdt)
                       for _ in range(nsets)]
            L["Gs"] = [torch.randn((blk.num_dst, feat), generator=g, device=dev, dtype=torch.float32).to(tdt)
                       for _ in range(nsets)]
            L["outs"] = [torch.empty((blk.num_dst, feat), device=dev, dtype=tdt) for _ in range(nsets)]
            L["dXs"] = [torch.empty((blk.num_src, feat), device=dev, dtype=tdt) for _ in range(nsets)]
            L["X"], L["G"], L["out"], L["dX"] = L["Xs"][0], L["Gs"][0], L["outs"][0], L["dXs"][0]
            L["plan_mem"] = torch.empty(B.fastgl_block_plan_bytes(blk.num_dst, blk.num_src, blk.num_edges),
                                        dtype=torch.uint8, device=dev)
            ws_bytes = max(ws_bytes, B.fastgl_block_workspace_bytes(blk.num_dst, blk.num_src, blk.num_edges,
                                                                    feat, w.dtype))
            din = np.diff(blk.indptr)
            dout = np.bincount(blk.indices, minlength=blk.num_src)
            L["bytes_fwd"] = compulsory_bytes(blk.num_dst, blk.num_edges, int((dout > 0).sum()), blk.num_dst, feat, elem)
            L["bytes_bwd"] = compulsory_bytes(blk.num_src, blk.num_edges, int((din > 0).sum()), blk.num_src, feat, elem)
            # L2-level demand: every gathered row + every output row (indices apart)
            L["gathered_fwd"] = (blk.num_edges + blk.num_dst) * feat * elem
            L["gathered_bwd"] = (blk.num_edges + blk.num_src) * feat * elem
            self.layers.append(L)
        self.workspace = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
        self.table = self.gid = None
        self.gather_bytes = 0
        if w.src_gid is not None:
            # config 4: the raw features sit in a device-resident table and are gathered by global id
            feat0 = w.widths[0]
            self.table = torch.empty((w.table_rows, feat0), dtype=tdt, device=dev)
            for lo in range(0, w.table_rows, 8_000_000):
                hi = min(w.table_rows, lo + 8_000_000)
                self.table[lo:hi] = torch.randn((hi - lo, feat0), generator=g, device=dev, dtype=torch.float32).to(tdt)
            self.gid = torch.from_numpy(w.src_gid).to(dev)
            self.gather_bytes = 8 * self.gid.numel() + 2 * self.gid.numel() * feat0 * elem
        self.total_edges = w.total_edges()
        self.bytes_step = sum(L["bytes_fwd"] + L["bytes_bwd"] for L in self.layers) + self.gather_bytes
        self.gathered_step = sum(L["gathered_fwd"] + L["gathered_bwd"] for L in self.layers) + self.gather_bytes
        self.B, self.torch = B, torch

    def make_plans(self):
        """Bookkeeping of every block of the mini-batch (transpose CSR, degrees, scale
        factors, degree buckets), built together: each stage is one launch for all layers."""
        B = self.B
        # sampled blocks (configs 1-4): the fan-out bounds every destination row far below the long-row
        # threshold, which the sampler knows and passes on as a hint; config 5 takes all neighbours
        parts = B.PLAN_ALL | (B.PLAN_SHORT_DST_ROWS if self.cfg != 5 else 0)
        return B.fastgl_block_plan_create_many([(L["indptr"], L["indices"], L["blk"].num_src) for L in self.layers],
                                               parts, [L["plan_mem"] for L in self.layers])

    def fwd(self, L, plan, k=0):
        self.B.fastgl_block_aggregate_fwd(L["indptr"], L["indices"], None, L["blk"].num_src, self.w.mode, L["Xs"][k],
                                          out=L["outs"][k], plan=plan, workspace=self.workspace)

    def bwd(self, L, plan, k=0):
        self.B.fastgl_block_aggregate_bwd(L["indptr"], L["indices"], None, L["blk"].num_src, self.w.mode, L["Gs"][k],
                                          grad_X=L["dXs"][k], plan=plan, workspace=self.workspace)

    def cold(self):
        """Between timed repetitions of a workload too small to rotate out of the cache."""
        if self.flush is not None:
            self.flush.fill_(1)


DOM_EVERY = 4   # timed steps per step that also times its dominant launch
GATHER_CEILING_GBPS = 7000.0   # random row gathers by a bare probe kernel: 6.4-7.6 TB/s, see profiles/


def median_ms(pairs):
    t = sorted(a.elapsed_time(b) for a, b in pairs)
    return float(t[len(t) // 2])


def headline(W, steps, warmup, np, traffic_table, copy_gbps, per_layer_reps):
    """Timed steps of one workload (plans + forward + backward of all layers) and its breakdown."""
    torch, layers, w = W.torch, W.layers, W.w
    dom = max(range(len(layers)), key=lambda i: layers[i]["bytes_fwd"])
    dom_ev, step_ev = [], []

    def step(i, timed=False):
        k = i % W.nsets
        if timed:
            W.cold()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
        if W.table is not None:
            W.B.fastgl_gather_rows(W.table, W.gid, out=layers[0]["Xs"][k])
        plans = W.make_plans()
        for j, L in enumerate(layers):
            if timed and j == dom and i % DOM_EVERY == 0:
                # two more events on the stream cost the step about 6 us each: only every fourth
                # timed step carries them, so the median step is one without
                d0, d1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                d0.record()
                W.fwd(L, plans[j], k)
                d1.record()
                dom_ev.append((d0, d1))
            else:
                W.fwd(L, plans[j], k)
        for L, p in zip(reversed(layers), reversed(plans)):
            W.bwd(L, p, k)
        if timed:
            e1.record()
            step_ev.append((e0, e1))

    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        step(i, timed=True)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / steps
    ms_step = median_ms(step_ev)
    dom_ms = float(np.mean([a.elapsed_time(b) for a, b in dom_ev]))

    # breakdown (not part of the headline): plan / forward / backward, every layer and pass
    def timed(fn, reps):
        ev = []
        for i in range(reps):
            W.cold()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            fn(i % W.nsets)
            b.record()
            ev.append((a, b))
        torch.cuda.synchronize()
        return median_ms(ev)

    reps = per_layer_reps
    plans = W.make_plans()
    plan_ms = timed(lambda k: W.make_plans(), reps)
    fwd_ms = timed(lambda k: [W.fwd(L, p, k) for L, p in zip(layers, plans)], reps)
    bwd_ms = timed(lambda k: [W.bwd(L, p, k) for L, p in zip(reversed(layers), reversed(plans))], reps)
    per_layer = []
    for i, (L, p) in enumerate(zip(layers, plans)):
        f = timed(lambda k: W.fwd(L, p, k), reps)
        b = timed(lambda k: W.bwd(L, p, k), reps)
        rec = dict(layer=i, num_dst=L["blk"].num_dst, num_src=L["blk"].num_src, E=L["blk"].num_edges, feat=L["feat"])
        for name, ms, byt, gat in (("fwd", f, L["bytes_fwd"], L["gathered_fwd"]), ("bwd", b, L["bytes_bwd"], L["gathered_bwd"])):
            gbps = byt / ms / 1e6
            rec[name] = {"ms": round(ms, 4), "compulsory_bytes": int(byt), "gbps_compulsory": round(gbps, 1),
                         "frac_of_peak": round(gbps / HBM_PEAK_GBPS, 4),
                         "frac_of_copy_bw": round(gbps / copy_gbps, 4),
                         "gbps_gathered": round(gat / ms / 1e6, 1),
                         "traffic_bytes": traffic_table.get((W.cfg, L["feat"], i, name))}
        per_layer.append(rec)
    gather_ms = None
    if W.table is not None:
        gather_ms = timed(lambda k: W.B.fastgl_gather_rows(W.table, W.gid, out=layers[0]["Xs"][k]), reps)

    value = 2.0 * W.total_edges / (ms_step * 1e-3) / 1e9
    domL = layers[dom]
    achieved = domL["bytes_fwd"] / (dom_ms * 1e-3) / 1e9
    gbps_step = W.bytes_step / (ms_step * 1e-3) / 1e9
    cached = fwd_ms + bwd_ms + (gather_ms or 0.0)
    res = {
        "value": round(value, 4),
        "ms_per_step": round(ms_step, 4),
        "ms_per_step_wall": round(wall_ms, 4),
        "timing": f"median of {steps} steps, each between two HIP events on the launch stream (every "
                  f"{DOM_EVERY}th of them with two more events around the dominant launch: roofline.launch_ms is the "
                  f"mean of those {len(dom_ev)}); wall = mean of the "
                  f"same steps between two device synchronisations; cold cache by "
                  + (f"rotating {W.nsets} copies of the feature / gradient buffers" if W.nsets > 1 else
                     "the step's own footprint") + (" and an untimed 512 MB fill before every step" if W.flush is not None else ""),
        "config": {"workload": w.name, "config_id": W.cfg, "seed": w.seed, "mode": w.mode, "widths": w.widths,
                   "total_edges": W.total_edges, "accumulate": "f64" if w.dtype == "f32" else "f32",
                   "buffer_footprint_bytes": int(W.footprint), "buffer_sets": W.nsets,
                   "step": ("table gather; " if W.table is not None else "") +
                           "plans of all layers (one batched call); forward per layer; backward per layer (reverse)"},
        "dtype": "f32" if w.dtype == "f32" else "bf16",
        "hbm_gbps_compulsory": round(gbps_step, 1),
        "hbm_frac_of_peak": round(gbps_step / HBM_PEAK_GBPS, 4),
        "frac_of_copy_bw": round(gbps_step / copy_gbps, 4),
        "gathered_gbps": round(W.gathered_step / (ms_step * 1e-3) / 1e9, 1),
        "compulsory_bytes_per_step": int(W.bytes_step),
        "breakdown_ms": {"plan": round(plan_ms, 4), "fwd": round(fwd_ms, 4), "bwd": round(bwd_ms, 4),
                         "table_gather": None if gather_ms is None else round(gather_ms, 4),
                         "cached_plan_step": round(cached, 4)},
        "value_cached_plan": round(2.0 * W.total_edges / (cached * 1e-3) / 1e9, 4),
        "hbm_frac_cached_plan": round(W.bytes_step / (cached * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
        "layers": per_layer,
        "roofline": {"bound": "hbm", "kernel": f"forward aggregation call, layer {dom} (k_pull_rows)",
                     "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBPS, 4),
                     "traffic": traffic_table.get((W.cfg, domL["feat"], dom, "fwd")),
                     "traffic_source": "profiles/traffic_counters.txt (rocprofv3 --pmc runs of this file; not measured in this run)",
                     "frac_of_copy_bw": round(achieved / copy_gbps, 4),
                     "launch_ms": round(dom_ms, 4), "algorithmic_bytes": int(domL["bytes_fwd"])},
        "gen_seconds": round(W.gen_s, 2),
    }
    moved = res["roofline"]["traffic"]
    if moved:
        # the same launch in MOVED bytes (the counter table) against what a bare kernel of random row
        # gathers reaches on this GPU (profiles/pull_rows_config2_traffic.md: 6.4-6.8 TB/s out of HBM,
        # 7.2-7.6 TB/s out of a cache-resident table)
        res["roofline"]["moved_gbps"] = round(moved / (dom_ms * 1e-3) / 1e9, 1)
        res["roofline"]["gather_ceiling_gbps"] = GATHER_CEILING_GBPS
        res["roofline"]["moved_frac_of_gather_ceiling"] = round(moved / (dom_ms * 1e-3) / 1e9 / GATHER_CEILING_GBPS, 4)
    return res


def cpu_baseline(W, np, budget_s=12.0, single_budget_s=5.0):
    """The oracle on the host cores, on a bounded sample of the same workload: the parallel variant
    (fp32 accumulate, OpenMP over rows, -O3 -march=native build) for about budget_s seconds, and the
    single-thread fp64 definitional oracle (the one parity is checked against) on the smallest layers."""
    import oracle
    torch, layers, w = W.torch, W.layers, W.w
    host = []
    for L in layers:
        if w.dtype == "f32":
            host.append((L["X"].cpu().numpy(), L["G"].cpu().numpy()))
        else:
            host.append((L["X"].view(torch.int16).cpu().numpy().view(np.uint16),
                         L["G"].view(torch.int16).cpu().numpy().view(np.uint16)))
    oracle.timed_lib()                      # compiled before the clock starts
    spent, edges_done, passes = 0.0, 0, 0
    while spent < budget_s:
        for L, (Xh, Gh) in zip(layers, host):
            blk = L["blk"]
            t0 = time.perf_counter()
            oracle.par_aggregate_fwd(blk.indptr, blk.indices, None, blk.num_src, w.mode, w.dtype, Xh, timed=True)
            oracle.par_aggregate_bwd(blk.indptr, blk.indices, None, blk.num_src, w.mode, w.dtype, Gh, timed=True)
            spent += time.perf_counter() - t0
            edges_done += 2 * blk.num_edges
        passes += 1
    res = {"value": round(edges_done / spent / 1e9, 5), "unit": "GEdges/s",
           "cores": oracle.num_threads(), "kind": "oracle",
           "sample": f"parallel oracle variant (fp32 accumulate, OpenMP over rows, backward through its own "
                     f"transpose; gcc {' '.join(oracle.TIMED_FLAGS)}): {passes} full fwd+bwd passes over all "
                     f"{len(layers)} layers of the same workload, {spent:.1f} s"}
    # the definitional oracle, one thread, smallest layers first until its budget is used
    spent1, edges1, done = 0.0, 0, []
    for i in sorted(range(len(layers)), key=lambda i: layers[i]["blk"].num_edges * layers[i]["feat"]):
        blk, (Xh, Gh) = layers[i]["blk"], host[i]
        if done and spent1 + 2.5e-9 * blk.num_edges * layers[i]["feat"] * 2 > single_budget_s:
            break
        t0 = time.perf_counter()
        oracle.aggregate_fwd(blk.indptr, blk.indices, None, blk.num_src, w.mode, w.dtype, Xh)
        oracle.aggregate_bwd(blk.indptr, blk.indices, None, blk.num_src, w.mode, w.dtype, Gh)
        spent1 += time.perf_counter() - t0
        edges1 += 2 * blk.num_edges
        done.append(i)
    res["single_thread_definitional"] = {
        "value": round(edges1 / spent1 / 1e9, 5), "unit": "GEdges/s", "cores": 1,
        "sample": f"fp64 definitional oracle (the parity reference), one fwd+bwd pass over layer(s) {sorted(done)}, {spent1:.2f} s"}
    return res


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
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
    ap.add_argument("--no-other-configs", action="store_true",
                    help="skip the shorter runs of the other four workloads (object `other_configs`)")
    ap.add_argument("--only-headline", action="store_true",
                    help="the timed steps and their breakdown only: no extra legs, no CPU baseline, no other workloads "
                         "(what the rocprofv3 summaries under profiles/ are taken from)")
    ap.add_argument("--verbose", action="store_true")
    ap.add_argument("--calibrate", action="store_true",
                    help="only run a plain 1 GiB device copy a few times (reference for rocprofv3 byte counters)")
    args = ap.parse_args()
    if args.only_headline:
        args.no_cpu_baseline = args.no_idmap = args.no_match = args.no_edge = args.no_gcn_step = True
        args.no_other_configs = True
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

    traffic_table = load_traffic_table()
    copy_gbps = measure_copy_gbps(torch)
    W = Workload(args.config, args.width, args.fanout_order, B, bg, torch, np)
    w, layers, workspace = W.w, W.layers, W.workspace
    head = headline(W, args.steps, args.warmup, np, traffic_table, copy_gbps, per_layer_reps=max(20, args.steps))
    head["config"]["fanout_order"] = args.fanout_order
    result = {
        "metric": METRIC,
        "value": head.pop("value"),
        "unit": "GEdges/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": head.pop("ms_per_step"),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": head.pop("dtype"),
        "data": "synthetic",
        "config": head.pop("config"),
        "copy_gbps_measured": round(copy_gbps, 1),
    }
    result.update(head)
    make_plans = W.make_plans

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
        result["cpu_baseline"] = cpu_baseline(W, np)

    if not args.no_other_configs:
        # the other workloads, same measurement with fewer repetitions (their own invocation,
        # `--config N [--width 256]`, gives the full record)
        del W, layers, workspace, head
        torch.cuda.empty_cache()
        others = []
        for cfg, width in ((1, 32), (3, 32), (4, 32), (5, 32), (5, 256)):
            if cfg == args.config and (cfg != 5 or width == args.width):
                continue
            Wo = Workload(cfg, width, args.fanout_order, B, bg, torch, np)
            r = headline(Wo, max(50, args.steps), args.warmup, np, traffic_table, copy_gbps, per_layer_reps=20)
            r["unit"] = "GEdges/s"
            others.append(r)
            del Wo
            torch.cuda.empty_cache()
        result["other_configs"] = others

    if args.verbose:
        print(json.dumps(result, indent=1), file=sys.stderr)
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
