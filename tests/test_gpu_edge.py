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
