"""The pieces chained the way a training iteration uses them, on the GPU and through the oracle:
sampled hops with global IDs -> ID map (block indices + source-node list) -> feature rows gathered
from a device table (with Match against the previous mini-batch's rows) -> plans -> two GCN layers
forward (aggregate, update) -> backward (update, aggregate).  Every hand-over between the entry
points is exercised; integer stages are compared bit for bit, every floating-point link element by
element within its own tolerance plus the earlier links' bounds pushed through it (chain_check.py;
the GPU feeds its own intermediates forward, the ReLU gate of the backward pass is the oracle's)."""
import numpy as np
import pytest
import torch

import blockgen as bg
import chain_check
import oracle
from paper_2409_14939_amd import binding as B

pytestmark = pytest.mark.gpu


def sampled_hops(seed):
    """Two hops of a small mini-batch with 40-bit global IDs: (dst_gid, indptr, nbr_gid) per hop,
    input-layer hop first; hop 1's destinations are the seeds, hop 0's are hop 1's sources."""
    rng = np.random.default_rng(seed)
    n_nodes = 5000
    gid_of = np.unique(rng.integers(0, 2 ** 40, size=2 * n_nodes))[:n_nodes]
    rng.shuffle(gid_of)
    hops = []
    dst = rng.choice(n_nodes, size=120, replace=False)
    for fanout in (6, 4):                                   # from the seeds outwards
        deg = rng.integers(0, fanout + 1, size=dst.size)
        indptr = np.concatenate([[0], np.cumsum(deg)]).astype(np.int32)
        pop = (rng.random(int(indptr[-1])) ** 3 * n_nodes).astype(np.int64)      # skewed: some nodes are hubs
        hops.append((gid_of[dst], indptr, gid_of[pop]))
        _, uniq = oracle.idmap(gid_of[dst], gid_of[pop])
        inv = {int(g): i for i, g in enumerate(gid_of)}
        dst = np.array([inv[int(g)] for g in uniq])         # next hop's destinations = this hop's sources
    hops.reverse()
    return hops, gid_of


def test_iteration_chain_against_oracle():
    hops, gid_of = sampled_hops(11)
    rng = np.random.default_rng(12)
    feat, hidden, classes = 100, 64, 10
    table = rng.standard_normal((gid_of.size, feat)).astype(np.float32)          # row r holds node gid_of[r]
    row_of = {int(g): r for r, g in enumerate(gid_of)}
    Ws = [(rng.standard_normal((feat, hidden)) / 10).astype(np.float32),
          (rng.standard_normal((hidden, classes)) / 8).astype(np.float32)]
    bs = [(0.1 * rng.standard_normal(hidden)).astype(np.float32), (0.1 * rng.standard_normal(classes)).astype(np.float32)]
    dlogits = rng.standard_normal((hops[1][0].size, classes)).astype(np.float32)
    # the previous mini-batch held these nodes' rows already (Match reuses them)
    prev_rows = rng.choice(gid_of.size, size=1500, replace=False)
    print("case iteration chain: idmap -> match/gather/assemble -> plans -> 2 GCN layers fwd+bwd", flush=True)

    # ---------------- oracle chain
    o_blocks = []
    for dst_gid, indptr, nbr_gid in hops:
        local, uniq = oracle.idmap(dst_gid, nbr_gid)
        o_blocks.append((indptr, local, uniq))
    assert np.array_equal(o_blocks[1][2], hops[0][0])                             # layer chain: sources of hop 1 = destinations of hop 0
    src_gid = o_blocks[0][2]
    o_X = table[[row_of[int(g)] for g in src_gid]]
    csr = [(indptr, local, uniq.size) for indptr, local, uniq in o_blocks]
    R = chain_check.oracle_chain(csr, "gcn", o_X, Ws, bs, dlogits)

    # ---------------- HIP chain
    dev = lambda a, dt=None: torch.from_numpy(np.ascontiguousarray(a if dt is None else a.astype(dt))).cuda()
    g_blocks = []
    for (dst_gid, indptr, nbr_gid), (o_ip, o_local, o_uniq) in zip(hops, o_blocks):
        local, uniq, res = B.fastgl_idmap(dev(dst_gid), dev(nbr_gid), "ordered")
        torch.cuda.synchronize()
        U, bad = (int(v) for v in res.cpu().numpy())
        assert bad == 0 and U == o_uniq.size
        assert np.array_equal(local.cpu().numpy(), o_local) and np.array_equal(uniq.cpu().numpy()[:U], o_uniq)
        g_blocks.append((dev(indptr), local, uniq[:U].contiguous(), U))
    # the sources of one hop are the destinations of the next (the layer chain)
    assert np.array_equal(g_blocks[0][2][:hops[0][0].size].cpu().numpy(), hops[0][0])
    assert np.array_equal(g_blocks[1][2].cpu().numpy(), hops[0][0])
    # features: global ID -> table row is the caller's business (here a dict); Match decides what to load
    src = g_blocks[0][2]
    prev_gid = dev(gid_of[prev_rows])
    X_prev = dev(table[prev_rows])
    src_row, load_pos, load_gid, mres = B.fastgl_match(prev_gid, src)
    torch.cuda.synchronize()
    n_load, bad = (int(v) for v in mres.cpu().numpy())
    assert bad == 0
    m_ref, lp_ref, lg_ref = oracle.match(gid_of[prev_rows], src.cpu().numpy())
    assert n_load == lp_ref.size and np.array_equal(load_gid.cpu().numpy()[:n_load], lg_ref)
    load_rows = dev(np.array([row_of[int(g)] for g in load_gid.cpu().numpy()[:n_load]], np.int64))
    X_load = B.fastgl_gather_rows(dev(table), load_rows)
    X = B.fastgl_assemble_rows(X_prev, X_load, src_row, n_load)
    torch.cuda.synchronize()
    assert np.array_equal(X.cpu().numpy(), o_X)                                  # bytes moved, nothing computed

    plans = B.fastgl_block_plan_create_many([(ip, loc, U) for ip, loc, _, U in g_blocks])
    xd, G = X, {}
    for i, relu in enumerate([True, False]):
        ip, loc, _, U = g_blocks[i]
        G[f"H{i}"] = B.fastgl_block_aggregate_fwd(ip, loc, None, U, "gcn", xd, plan=plans[i])
        G[f"Y{i}"] = xd = B.fastgl_update_fwd(G[f"H{i}"], dev(Ws[i]), dev(bs[i]), relu)
    G["dH1"], G["dW1"], G["db1"] = B.fastgl_update_bwd(G["H1"], dev(Ws[1]), None, dev(dlogits), False)
    ip, loc, _, U = g_blocks[1]
    G["dY0"] = B.fastgl_block_aggregate_bwd(ip, loc, None, U, "gcn", G["dH1"], plan=plans[1])
    _, G["dW0"], G["db0"] = B.fastgl_update_bwd(G["H0"], dev(Ws[0]), dev(R["Y0"]), G["dY0"], True, want=("dW", "db"))
    torch.cuda.synchronize()
    chain_check.compare(csr, "gcn", o_X, Ws, bs, dlogits, R, {k: v.cpu().numpy() for k, v in G.items()},
                        B.fastgl_update_slab_rows)
