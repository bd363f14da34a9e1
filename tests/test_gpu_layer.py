"""fastgl_layer_fwd (aggregation, Eq. 1, then update, Eq. 2, in one call; one kernel for narrow
layers) against the oracle's chain aggregate_fwd -> update_fwd, through the C ABI, element by element.

Tolerances: H is what the aggregation call stores (1e-5 relative + 1e-6 absolute).  Y is formed from
the GPU's own H, so its bound is the update phase's rounding bound - (L + 4) u sum|h w| + u |y| with
L = K + 1 for an fp32 chain in any order, which covers both the one-kernel path (fp32 multiply-adds in
ascending k) and the matrix-core path - plus H's bound pushed through |W|."""
import numpy as np
import pytest
import torch

import blockgen as bg
import chain_check as cc
import oracle
from paper_2409_14939_amd import binding as B
from gpu_util import dev_i32

pytestmark = pytest.mark.gpu


def dev(a):
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()


def check_layer(blk, mode, K, N, relu, weighted, with_H, use_plan, seed, what):
    rng = np.random.default_rng(seed)
    X = bg.features_f32(rng, blk.num_src, K)
    W = (rng.standard_normal((K, N)) / np.sqrt(K)).astype(np.float32)
    b = (0.1 * rng.standard_normal(N)).astype(np.float32) if seed % 2 else None
    ew = rng.standard_normal(blk.num_edges).astype(np.float32) if weighted else None
    fused = B.fastgl_layer_fwd_fuses(K, N, "f32")
    print(f"case layer {what}: mode={mode} K={K} N={N} relu={relu} weighted={weighted} H={with_H} plan={use_plan} "
          f"fused={fused} dst={blk.num_dst} src={blk.num_src} E={blk.num_edges}", flush=True)
    ip, ix = dev_i32(blk.indptr), dev_i32(blk.indices)
    plan = B.fastgl_block_plan_create(ip, ix, blk.num_src, B.PLAN_FWD | B.PLAN_SRC_DEG) if use_plan else None
    Hd, Yd = B.fastgl_layer_fwd(ip, ix, dev(ew), blk.num_src, mode, dev(X), dev(W), dev(b), relu, want_H=with_H, plan=plan)
    torch.cuda.synchronize()
    Href = oracle.aggregate_fwd(blk.indptr, blk.indices, ew, blk.num_src, mode, "f32", X)
    Yref = oracle.update_fwd(Href, W, b, relu)
    aH = np.abs(Href).astype(np.float64)
    e_H = cc.agg_tol(aH)
    if with_H:
        cc.assert_within(what + " H", Hd.cpu().numpy(), Href, e_H)
    else:
        assert Hd is None
    aW = np.abs(W).astype(np.float64)
    absprod = (aH + e_H) @ aW + (0 if b is None else np.abs(b))
    bound = e_H @ aW + cc.gemm_tol(absprod, K + 1, np.abs(Yref).astype(np.float64) + e_H @ aW)
    cc.assert_within(what + " Y", Yd.cpu().numpy(), Yref, bound)
    return Hd, Yd


def small_block(seed, nd=1237, ns=3001, hubs=0):
    rng = np.random.default_rng(seed)
    return bg.random_block(rng, nd, ns, 9.0, empty_frac=0.1, hub_rows=hubs, hub_deg=700)


@pytest.mark.parametrize("mode,K,N,relu,weighted", [
    ("gcn", 256, 47, False, False),      # the class-score layer of the products-shaped GCN
    ("mean", 100, 64, True, False),
    ("sum", 64, 1, True, True),
    ("gcn", 4, 3, False, True),
    ("sum", 252, 33, True, False),
])
def test_layer_fused_shapes(mode, K, N, relu, weighted):
    assert B.fastgl_layer_fwd_fuses(K, N, "f32")
    blk = small_block(K + N)
    check_layer(blk, mode, K, N, relu, weighted, True, True, 1 + K, "fused")
    check_layer(blk, mode, K, N, relu, weighted, False, False, 2 + K, "fused, H not written, no plan")


def test_layer_fused_rows_that_are_long_and_ragged_tail():
    # rows far above the long-row threshold are walked by one wavefront here; 1237 rows leave a
    # partial last workgroup and a partial last wavefront
    check_layer(small_block(5, hubs=4), "gcn", 128, 47, True, False, True, True, 9, "fused, hub rows")
    check_layer(small_block(6, nd=3, ns=40), "mean", 32, 8, False, True, True, False, 10, "fused, 3 rows")
    check_layer(bg.random_block(np.random.default_rng(2), 50, 80, 0.0, empty_frac=1.0), "gcn", 16, 4, True, False,
                True, False, 11, "fused, no edges")


@pytest.mark.parametrize("mode,K,N", [("gcn", 602, 47), ("mean", 256, 100), ("sum", 30, 16)])
def test_layer_shapes_that_run_as_two_kernels(mode, K, N):
    assert not B.fastgl_layer_fwd_fuses(K, N, "f32")
    blk = small_block(K + N, hubs=2)
    check_layer(blk, mode, K, N, True, False, True, True, 3 + K, "two kernels")
    with pytest.raises(B.FastglError):          # no H to hand over between the two kernels
        check_layer(blk, mode, K, N, True, False, False, True, 3 + K, "two kernels, H missing")


def test_layer_fused_equals_separate_calls_in_H_and_full_size_output_layer():
    """The output layer of the products-shaped workload at full size (8 000 seeds, 256 -> 47): H of the
    fused call equals the aggregation call's bit for bit; Y against the oracle chain."""
    w = bg.make_config(2)
    blk = w.blocks[2]
    Hd, Yd = check_layer(blk, "gcn", 256, 47, False, False, True, True, 77, "config 2 output layer")
    rng = np.random.default_rng(77)
    X = bg.features_f32(rng, blk.num_src, 256)
    ip, ix = dev_i32(blk.indptr), dev_i32(blk.indices)
    H2 = B.fastgl_block_aggregate_fwd(ip, ix, None, blk.num_src, "gcn", dev(X))
    torch.cuda.synchronize()
    assert torch.equal(Hd.view(torch.int32), H2.view(torch.int32))
