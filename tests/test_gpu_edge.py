"""GPU parity of the edge-weight gradient and the edge softmax against the CPU oracle, through the
C ABI.  Tolerances are the task's for this path: fp32 1e-5 relative + 1e-6 absolute (the kernels sum
in fp64), bf16 inputs 2e-2 relative (+1e-5 absolute; fp32 sums, fp32 output)."""
import numpy as np
import pytest
import torch

import blockgen as bg
import oracle
from paper_2409_14939_amd import binding as B
from gpu_util import dev_feat, dev_i32, make_inputs

pytestmark = pytest.mark.gpu
MODES = ["sum", "mean", "gcn"]


def close(got, ref, rtol, atol, what):
    got, ref = got.astype(np.float64), ref.astype(np.float64)
    bad = np.abs(got - ref) > atol + rtol * np.abs(ref)
    assert not bad.any(), (what, int(bad.sum()), got[bad][:3], ref[bad][:3])


def ragged_block(seed=31):
    return bg.random_block(np.random.default_rng(seed), 1237, 3001, 6.0, empty_frac=0.15, hub_rows=5, hub_deg=1500)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("feat", [1, 3, 6, 32, 100, 128, 256, 602])
def test_edge_weight_grad_ragged(dtype, mode, feat):
    blk = ragged_block()
    rng = np.random.default_rng(feat)
    X, G = make_inputs(rng, blk.num_src, feat, dtype), make_inputs(rng, blk.num_dst, feat, dtype)
    print(f"case edge grad mode={mode} dtype={dtype} F={feat} E={blk.num_edges}", flush=True)
    ip, ix = dev_i32(blk.indptr), dev_i32(blk.indices)
    plan = B.fastgl_block_plan_create(ip, ix, blk.num_src, B.PLAN_FWD | B.PLAN_SRC_DEG) if mode == "gcn" else None
    gw = B.fastgl_edge_weight_grad(ip, ix, blk.num_src, mode, dev_feat(X, dtype), dev_feat(G, dtype), plan=plan)
    torch.cuda.synchronize()
    ref = oracle.edge_weight_grad(blk.indptr, blk.indices, blk.num_src, mode, dtype, X, G)
    # bf16 inputs are exact in both; only the summation differs (fp32 on the GPU): relative to the sum of magnitudes
    if dtype == "f32":
        close(gw.cpu().numpy(), ref, 1e-5, 1e-6, "grad_w")
    else:
        close(gw.cpu().numpy(), ref, 2e-2, 1e-5 * max(1.0, np.sqrt(feat)), "grad_w")


def test_edge_weight_grad_degenerate():
    print("case edge grad degenerate", flush=True)
    ip = dev_i32(np.array([0, 0, 0], np.int32))
    ix = dev_i32(np.zeros(0, np.int32))
    gw = B.fastgl_edge_weight_grad(ip, ix, 4, "sum", torch.ones((4, 8), device="cuda"), torch.ones((2, 8), device="cuda"))
    assert gw.numel() == 0
    # one edge, one feature
    ip, ix = dev_i32(np.array([0, 1], np.int32)), dev_i32(np.array([2], np.int32))
    X = torch.tensor([[1.0], [2.0], [3.0]], device="cuda")
    G = torch.tensor([[-4.0]], device="cuda")
    gw = B.fastgl_edge_weight_grad(ip, ix, 3, "sum", X, G)
    torch.cuda.synchronize()
    assert gw.cpu().tolist() == [-12.0]


def softmax_case(blk, seed, what):
    rng = np.random.default_rng(seed)
    score = (4 * rng.standard_normal(blk.num_edges)).astype(np.float32)
    da = rng.standard_normal(blk.num_edges).astype(np.float32)
    print(f"case edge softmax {what} dst={blk.num_dst} E={blk.num_edges} max row={int(np.diff(blk.indptr).max())}",
          flush=True)
    ip = dev_i32(blk.indptr)
    alpha = B.fastgl_edge_softmax_fwd(ip, torch.from_numpy(score).cuda())
    torch.cuda.synchronize()
    ref = oracle.edge_softmax_fwd(blk.indptr, score)
    close(alpha.cpu().numpy(), ref, 1e-5, 1e-9, "alpha")
    ds = B.fastgl_edge_softmax_bwd(ip, torch.from_numpy(ref).cuda(), torch.from_numpy(da).cuda())
    torch.cuda.synchronize()
    close(ds.cpu().numpy(), oracle.edge_softmax_bwd(blk.indptr, ref, da), 1e-5, 1e-6, "grad_score")
    # run to run identical although long rows are queued in any order
    again = B.fastgl_edge_softmax_fwd(ip, torch.from_numpy(score).cuda())
    torch.cuda.synchronize()
    assert torch.equal(alpha, again)


def test_edge_softmax_ragged_with_long_rows():
    assert B.fastgl_edge_softmax_long_row() < 1500        # the hub rows below take the workgroup-per-row pass
    softmax_case(ragged_block(), 1, "ragged")
    blk = bg.random_block(np.random.default_rng(2), 300, 900, 3.0, empty_frac=0.3, hub_rows=40, hub_deg=5000)
    softmax_case(blk, 3, "many long rows")                 # mean row length > 96: 64 lanes per row
    blk = bg.random_block(np.random.default_rng(4), 2000, 5000, 50.0, empty_frac=0.1, hub_rows=3, hub_deg=1200)
    softmax_case(blk, 5, "medium rows")                    # mean row length 24..96: 32 lanes per row


def test_edge_softmax_degenerate():
    print("case edge softmax degenerate", flush=True)
    ip = dev_i32(np.array([0, 0, 1, 1, 3], np.int32))
    score = torch.tensor([7.0, 1000.0, 1000.0], device="cuda")
    alpha = B.fastgl_edge_softmax_fwd(ip, score)
    torch.cuda.synchronize()
    assert alpha.cpu().tolist() == [1.0, 0.5, 0.5]
    empty = B.fastgl_edge_softmax_fwd(dev_i32(np.array([0, 0], np.int32)), torch.empty(0, device="cuda"))
    assert empty.numel() == 0


def test_edge_paths_on_the_sampled_workload():
    """The input-layer block of the products-shaped workload (2.56 M edges, F = 100) in the launch
    shape the benchmark times; the oracle is fast enough to check every edge."""
    w = bg.make_config(2)
    blk, feat = w.blocks[0], w.widths[0]
    rng = np.random.default_rng(4)
    X, G = bg.features_f32(rng, blk.num_src, feat), bg.features_f32(rng, blk.num_dst, feat)
    print(f"case edge paths config2 input layer E={blk.num_edges} F={feat}", flush=True)
    ip, ix = dev_i32(blk.indptr), dev_i32(blk.indices)
    plan = B.fastgl_block_plan_create(ip, ix, blk.num_src, B.PLAN_FWD | B.PLAN_SRC_DEG)
    gw = B.fastgl_edge_weight_grad(ip, ix, blk.num_src, "gcn", torch.from_numpy(X).cuda(), torch.from_numpy(G).cuda(),
                                   plan=plan)
    torch.cuda.synchronize()
    close(gw.cpu().numpy(), oracle.edge_weight_grad(blk.indptr, blk.indices, blk.num_src, "gcn", "f32", X, G),
          1e-5, 1e-6, "grad_w")
    softmax_case(blk, 5, "config2 input layer")
    score_case(blk, 6, 0.2, "config2 input layer")


def test_edge_random_block_sweep():
    """Seeded sweep over block shapes and widths (lane-group sizes 1..64, 2/4/8/16-byte pieces)."""
    rng = np.random.default_rng(77)
    for case in range(16):
        nd, ns = int(rng.integers(1, 400)), int(rng.integers(1, 600))
        blk = bg.random_block(rng, nd, ns, float(rng.uniform(0.5, 9)), empty_frac=0.2,
                              hub_rows=int(rng.integers(0, 3)), hub_deg=int(rng.integers(100, 3000)))
        feat = int(rng.choice([1, 2, 3, 4, 5, 8, 12, 17, 32, 48, 64, 100, 129, 200, 300, 514]))
        dtype = "f32" if case % 2 == 0 else "bf16"
        mode = MODES[case % 3]
        X, G = make_inputs(rng, ns, feat, dtype), make_inputs(rng, nd, feat, dtype)
        print(f"case edge sweep {case} dst={nd} src={ns} E={blk.num_edges} F={feat} {dtype} {mode}", flush=True)
        ip, ix = dev_i32(blk.indptr), dev_i32(blk.indices)
        plan = B.fastgl_block_plan_create(ip, ix, ns, B.PLAN_FWD | B.PLAN_SRC_DEG) if mode == "gcn" else None
        gw = B.fastgl_edge_weight_grad(ip, ix, ns, mode, dev_feat(X, dtype), dev_feat(G, dtype), plan=plan)
        torch.cuda.synchronize()
        ref = oracle.edge_weight_grad(blk.indptr, blk.indices, ns, mode, dtype, X, G)
        if dtype == "f32":
            close(gw.cpu().numpy(), ref, 1e-5, 1e-6, "grad_w")
        else:
            close(gw.cpu().numpy(), ref, 2e-2, 1e-5 * max(1.0, np.sqrt(feat)), "grad_w")
        if blk.num_edges:
            softmax_case(blk, 500 + case, f"sweep {case}")


def score_case(blk, seed, slope, what):
    """Attention logits and their gradients.  The sum el + er is exact in fp64 on both sides and the
    result is rounded once, so the forward pass is compared bit for bit; the gradients are fp64 sums
    taken in different orders: 1e-6 relative to the sum of magnitudes is far above that noise."""
    rng = np.random.default_rng(seed)
    el = rng.standard_normal(blk.num_dst).astype(np.float32)
    er = rng.standard_normal(blk.num_src).astype(np.float32)
    ds = rng.standard_normal(blk.num_edges).astype(np.float32)
    print(f"case edge score {what} dst={blk.num_dst} src={blk.num_src} E={blk.num_edges} slope={slope}", flush=True)
    ip, ix = dev_i32(blk.indptr), dev_i32(blk.indices)
    eld, erd = torch.from_numpy(el).cuda(), torch.from_numpy(er).cuda()
    s = B.fastgl_edge_score_fwd(ip, ix, eld, erd, slope)
    torch.cuda.synchronize()
    assert np.array_equal(s.cpu().numpy(), oracle.edge_score_fwd(blk.indptr, blk.indices, el, er, slope))
    plan = B.fastgl_block_plan_create(ip, ix, blk.num_src, B.PLAN_ALL | B.PLAN_PERM)
    g_el, g_er = B.fastgl_edge_score_bwd(ip, ix, eld, erd, slope, torch.from_numpy(ds).cuda(), plan=plan)
    torch.cuda.synchronize()
    r_el, r_er = oracle.edge_score_bwd(blk.indptr, blk.indices, el, er, slope, ds)
    rows = np.repeat(np.arange(blk.num_dst), np.diff(blk.indptr))
    mag_el = np.bincount(rows, np.abs(ds).astype(np.float64), blk.num_dst)
    mag_er = np.bincount(blk.indices, np.abs(ds).astype(np.float64), blk.num_src)
    assert (np.abs(g_el.cpu().numpy().astype(np.float64) - r_el) <= 2.0 ** -23 * np.abs(r_el) + 1e-12 * mag_el).all()
    assert (np.abs(g_er.cpu().numpy().astype(np.float64) - r_er) <= 2.0 ** -23 * np.abs(r_er) + 1e-12 * mag_er).all()
    only_el, none = B.fastgl_edge_score_bwd(ip, ix, eld, erd, slope, torch.from_numpy(ds).cuda(), want=("el",))
    torch.cuda.synchronize()
    assert none is None and torch.equal(only_el, g_el)


def test_edge_score_ragged_and_degenerate():
    score_case(ragged_block(), 41, 0.2, "ragged")                          # 8 lanes per row, hub rows of 1500
    blk = bg.random_block(np.random.default_rng(2), 300, 900, 3.0, empty_frac=0.3, hub_rows=40, hub_deg=5000)
    score_case(blk, 42, 0.2, "many long rows")                             # 64 lanes per row
    blk = bg.random_block(np.random.default_rng(4), 2000, 5000, 50.0, empty_frac=0.1, hub_rows=3, hub_deg=1200)
    score_case(blk, 43, 0.01, "medium rows")                               # 32 lanes per row
    score_case(ragged_block(7), 44, 0.0, "slope 0")
    score_case(ragged_block(8), 45, 1.0, "slope 1")
    print("case edge score degenerate", flush=True)
    ip, ix = dev_i32(np.array([0, 0, 0], np.int32)), dev_i32(np.zeros(0, np.int32))
    el, er = torch.ones(2, device="cuda"), torch.ones(3, device="cuda")
    assert B.fastgl_edge_score_fwd(ip, ix, el, er, 0.2).numel() == 0
    plan = B.fastgl_block_plan_create(ip, ix, 3, B.PLAN_ALL | B.PLAN_PERM)
    g_el, g_er = B.fastgl_edge_score_bwd(ip, ix, el, er, 0.2, torch.empty(0, device="cuda"), plan=plan)
    torch.cuda.synchronize()
    assert g_el.cpu().tolist() == [0, 0] and g_er.cpu().tolist() == [0, 0, 0]
    with pytest.raises(B.FastglError):                                     # grad_er without the transposed block
        B.fastgl_edge_score_bwd(ip, ix, el, er, 0.2, torch.empty(0, device="cuda"))


def test_gat_heads_forward_and_backward_against_the_oracle():
    """Two attention heads of a GAT layer on one ragged block, head-major arrays, every step through
    the library: Z = X W (update phase without bias), el = Z a_l and er = Z a_r (the same call with
    one output column), logits, edge softmax, weighted aggregation; then the whole chain backwards
    down to dW, da_l and da_r.  The oracle runs the same chain; each side feeds its own intermediate
    results forward, so the comparison is of the chain, with tolerances widened accordingly."""
    blk = ragged_block(51)
    rng = np.random.default_rng(52)
    heads, fin, fout, slope = 2, 24, 16, 0.2
    X = bg.features_f32(rng, blk.num_src, fin)
    G = bg.features_f32(rng, blk.num_dst, fout)
    ip, ix = dev_i32(blk.indptr), dev_i32(blk.indices)
    plan = B.fastgl_block_plan_create(ip, ix, blk.num_src, B.PLAN_ALL | B.PLAN_PERM)
    Xd, Gd = torch.from_numpy(X).cuda(), torch.from_numpy(G).cuda()
    for h in range(heads):
        W = (rng.standard_normal((fin, fout)) / np.sqrt(fin)).astype(np.float32)
        al = (rng.standard_normal((fout, 1)) / 4).astype(np.float32)
        ar = (rng.standard_normal((fout, 1)) / 4).astype(np.float32)
        print(f"case gat head {h} dst={blk.num_dst} src={blk.num_src} E={blk.num_edges}", flush=True)
        Wd, ald, ard = (torch.from_numpy(a).cuda() for a in (W, al, ar))
        # forward (destinations are a prefix of the sources)
        Z = B.fastgl_update_fwd(Xd, Wd, None, False)
        el = B.fastgl_update_fwd(Z[:blk.num_dst].contiguous(), ald, None, False).reshape(-1)
        er = B.fastgl_update_fwd(Z, ard, None, False).reshape(-1)
        score = B.fastgl_edge_score_fwd(ip, ix, el, er, slope)
        alpha = B.fastgl_edge_softmax_fwd(ip, score)
        out = B.fastgl_block_aggregate_fwd(ip, ix, alpha, blk.num_src, "sum", Z, plan=plan)
        # backward
        dalpha = B.fastgl_edge_weight_grad(ip, ix, blk.num_src, "sum", Z, Gd)
        dZ = B.fastgl_block_aggregate_bwd(ip, ix, alpha, blk.num_src, "sum", Gd, plan=plan)
        dscore = B.fastgl_edge_softmax_bwd(ip, alpha, dalpha)
        del_, der = B.fastgl_edge_score_bwd(ip, ix, el, er, slope, dscore, plan=plan)
        _, dal, _ = B.fastgl_update_bwd(Z[:blk.num_dst].contiguous(), ald, None, del_.reshape(-1, 1), False, want=("dH", "dW"))
        dZl, _, _ = B.fastgl_update_bwd(Z[:blk.num_dst].contiguous(), ald, None, del_.reshape(-1, 1), False, want=("dH",))
        dZr, dar, _ = B.fastgl_update_bwd(Z, ard, None, der.reshape(-1, 1), False, want=("dH", "dW"))
        dZ = dZ + dZr
        dZ[:blk.num_dst] += dZl
        _, dW, _ = B.fastgl_update_bwd(Xd, Wd, None, dZ, False, want=("dW",))
        torch.cuda.synchronize()

        # the same chain through the oracle
        Zr = oracle.update_fwd(X, W, None, False)
        elr = oracle.update_fwd(Zr[:blk.num_dst], al, None, False).reshape(-1)
        err = oracle.update_fwd(Zr, ar, None, False).reshape(-1)
        sr = oracle.edge_score_fwd(blk.indptr, blk.indices, elr, err, slope)
        ar_ = oracle.edge_softmax_fwd(blk.indptr, sr)
        outr = oracle.aggregate_fwd(blk.indptr, blk.indices, ar_, blk.num_src, "sum", "f32", Zr)
        dar_ = oracle.edge_weight_grad(blk.indptr, blk.indices, blk.num_src, "sum", "f32", Zr, G)
        dZr_ = oracle.aggregate_bwd(blk.indptr, blk.indices, ar_, blk.num_src, "sum", "f32", G)
        dsr = oracle.edge_softmax_bwd(blk.indptr, ar_, dar_)
        delr, derr = oracle.edge_score_bwd(blk.indptr, blk.indices, elr, err, slope, dsr)
        dZl_r, dal_r, _ = oracle.update_bwd(Zr[:blk.num_dst], al, None, delr.reshape(-1, 1), False)
        dZr_r, dar_r, _ = oracle.update_bwd(Zr, ar, None, derr.reshape(-1, 1), False)
        dZt = dZr_.astype(np.float64) + dZr_r
        dZt[:blk.num_dst] += dZl_r
        _, dWr, _ = oracle.update_bwd(X, W, None, dZt.astype(np.float32), False)

        close(out.cpu().numpy(), outr, 1e-4, 1e-5, "head output")
        close(alpha.cpu().numpy(), ar_, 1e-4, 1e-7, "attention")
        close(dal.cpu().numpy(), dal_r, 1e-3, 1e-4, "grad a_l")
        close(dar.cpu().numpy(), dar_r, 1e-3, 1e-4, "grad a_r")
        close(dW.cpu().numpy(), dWr, 1e-3, 1e-3, "grad W")
