"""Out-of-bounds stores: every output of the ragged and degenerate cases sits between two guard bands
of a sentinel bit pattern, in ONE allocation, and the bands must be untouched afterwards (a kernel
that writes a row too many, or a slice past the end of a row, lands in a band).  The results between
the bands are checked against the oracle as usual, so that a band is not intact simply because
nothing ran.  Covers aggregation forward / backward (plan and no plan, long rows, empty blocks),
row gather, row assembly, the update phase, the one-call layer, and the plan buffer (everything the
bookkeeping kernels write lies inside the caller's buffer of fastgl_block_plan_bytes bytes)."""
import numpy as np
import pytest
import torch

import blockgen as bg
import oracle
from paper_2409_14939_amd import binding as B
from gpu_util import assert_close, dev_feat, dev_i32, host_feat, make_inputs, read_i32

pytestmark = pytest.mark.gpu
GUARD_ROWS = 3
SENTINEL = {torch.float32: 0x7FC5A5A5, torch.bfloat16: 0x7FC5}      # NaN patterns no kernel here produces


class Guarded:
    """rows x cols matrix of `dtype` in the middle of a larger allocation filled with a sentinel."""

    def __init__(self, rows, cols, dtype):
        self.rows, self.cols, self.dtype = rows, cols, dtype
        self.it = torch.int32 if dtype == torch.float32 else torch.int16
        self.band = max(GUARD_ROWS * cols, 64)                      # elements before and after
        self.raw = torch.full((2 * self.band + rows * cols,), SENTINEL[dtype], dtype=self.it, device="cuda")
        self.t = self.raw[self.band:self.band + rows * cols].view(dtype).view(rows, cols)
        assert self.t.is_contiguous()

    def check(self, what):
        torch.cuda.synchronize()
        s = SENTINEL[self.dtype]
        lo, hi = self.raw[:self.band], self.raw[self.band + self.rows * self.cols:]
        assert bool((lo == s).all()), f"{what}: store below the output"
        assert bool((hi == s).all()), f"{what}: store above the output"


def tdt(dtype):
    return torch.float32 if dtype == "f32" else torch.bfloat16


def blocks():
    rng = np.random.default_rng(12)
    yield "ragged", bg.random_block(rng, 1237, 3001, 6.0, empty_frac=0.15, hub_rows=5, hub_deg=1500)
    yield "no-edges", bg.random_block(rng, 9, 17, 0.0, empty_frac=1.0)
    yield "one-by-one", bg.Block(np.array([0, 1], np.int32), np.array([0], np.int32), 1, 1)
    yield "single-hub", bg.random_block(rng, 1, 50, 0.0, empty_frac=0.0, hub_rows=1, hub_deg=5000)
    yield "threshold+1", bg.random_block(rng, 3, 40, 0.0, empty_frac=0.0, hub_rows=3,
                                         hub_deg=B.fastgl_long_row_threshold() + 1)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("feat", [1, 7, 100, 256, 602])
def test_aggregation_outputs_between_guard_bands(dtype, feat):
    rng = np.random.default_rng(feat)
    for name, blk in blocks():
        for mode, use_plan in (("gcn", True), ("mean", False)):
            print(f"guard bands: {name} mode={mode} dtype={dtype} F={feat} plan={use_plan}", flush=True)
            X, G = make_inputs(rng, blk.num_src, feat, dtype), make_inputs(rng, blk.num_dst, feat, dtype)
            ip, ix = dev_i32(blk.indptr), dev_i32(blk.indices)
            plan = B.fastgl_block_plan_create(ip, ix, blk.num_src) if use_plan else None
            out, dX = Guarded(blk.num_dst, feat, tdt(dtype)), Guarded(blk.num_src, feat, tdt(dtype))
            B.fastgl_block_aggregate_fwd(ip, ix, None, blk.num_src, mode, dev_feat(X, dtype), out=out.t, plan=plan)
            B.fastgl_block_aggregate_bwd(ip, ix, None, blk.num_src, mode, dev_feat(G, dtype), grad_X=dX.t, plan=plan)
            out.check(f"{name} forward")
            dX.check(f"{name} backward")
            assert_close(host_feat(out.t, dtype), oracle.aggregate_fwd(blk.indptr, blk.indices, None, blk.num_src, mode, dtype, X),
                         dtype, name + " fwd")
            assert_close(host_feat(dX.t, dtype), oracle.aggregate_bwd(blk.indptr, blk.indices, None, blk.num_src, mode, dtype, G),
                         dtype, name + " bwd")


@pytest.mark.parametrize("dtype,feat", [("f32", 100), ("bf16", 128), ("bf16", 7), ("f32", 602)])
def test_gather_and_assemble_between_guard_bands(dtype, feat):
    rng = np.random.default_rng(3 + feat)
    T = make_inputs(rng, 700, feat, dtype)
    ids = rng.integers(0, 700, size=333)
    out = Guarded(ids.size, feat, tdt(dtype))
    B.fastgl_gather_rows(dev_feat(T, dtype), torch.from_numpy(ids).cuda(), out=out.t)
    out.check("gather")
    assert np.array_equal(host_feat(out.t, dtype), oracle.gather_rows(T, ids, dtype))
    # assembly of a new feature matrix from reused and loaded rows
    prev = np.unique(rng.integers(0, 10 ** 9, size=500))
    new = np.concatenate([rng.choice(prev, size=200, replace=False), np.unique(rng.integers(10 ** 9, 2 * 10 ** 9, size=150))])
    rng.shuffle(new)
    src_row, load_pos, load_gid, res = B.fastgl_match(torch.from_numpy(prev).cuda(), torch.from_numpy(new).cuda())
    torch.cuda.synchronize()
    n_load = int(res.cpu()[0])
    Xp, Xl = make_inputs(rng, prev.size, feat, dtype), make_inputs(rng, n_load, feat, dtype)
    Xn = Guarded(new.size, feat, tdt(dtype))
    B.fastgl_assemble_rows(dev_feat(Xp, dtype), dev_feat(Xl, dtype), src_row, n_load, out=Xn.t)
    Xn.check("assemble")
    m_ref, _, _ = oracle.match(prev, new)
    assert np.array_equal(host_feat(Xn.t, dtype), oracle.assemble(Xp, Xl, m_ref))


@pytest.mark.parametrize("M,K,N", [(300, 100, 256), (2500, 256, 47), (257, 17, 130), (1, 40, 5), (129, 1, 1)])
def test_update_outputs_between_guard_bands(M, K, N):
    rng = np.random.default_rng(M + K + N)
    f = lambda *s: rng.standard_normal(s).astype(np.float32)
    H, W, b, dY = f(M, K), (f(K, N) / np.sqrt(K)).astype(np.float32), f(N), f(M, N)
    dev = lambda a: torch.from_numpy(a).cuda()
    Y, dH = Guarded(M, N, torch.float32), Guarded(M, K, torch.float32)
    dW, db = Guarded(K, N, torch.float32), Guarded(1, N, torch.float32)
    print(f"guard bands: update M={M} K={K} N={N}", flush=True)
    B.fastgl_update_fwd(dev(H), dev(W), dev(b), True, Y.t)
    Yref = oracle.update_fwd(H, W, b, True)
    B.fastgl_update_bwd(dev(H), dev(W), dev(Yref), dev(dY), True, dH=dH.t, dW=dW.t, db=db.t.view(N))
    for g, what in ((Y, "Y"), (dH, "dH"), (dW, "dW"), (db, "db")):
        g.check("update " + what)
    dHr, dWr, dbr = oracle.update_bwd(H, W, Yref, dY, True)
    for got, ref, what in ((Y.t, Yref, "Y"), (dH.t, dHr, "dH"), (dW.t, dWr, "dW"), (db.t.view(N), dbr, "db")):
        np.testing.assert_allclose(got.cpu().numpy(), ref, rtol=2e-4, atol=2e-4 * max(1.0, float(np.abs(ref).max())), err_msg=what)


@pytest.mark.parametrize("K,N", [(256, 47), (100, 64), (64, 1), (602, 47)])
def test_layer_outputs_between_guard_bands(K, N):
    rng = np.random.default_rng(K * N)
    blk = bg.random_block(rng, 1237, 3001, 6.0, empty_frac=0.15, hub_rows=2, hub_deg=600)
    X = bg.features_f32(rng, blk.num_src, K)
    W = (rng.standard_normal((K, N)) / np.sqrt(K)).astype(np.float32)
    b = rng.standard_normal(N).astype(np.float32)
    H, Y = Guarded(blk.num_dst, K, torch.float32), Guarded(blk.num_dst, N, torch.float32)
    print(f"guard bands: layer K={K} N={N} fused={B.fastgl_layer_fwd_fuses(K, N, 'f32')}", flush=True)
    B.fastgl_layer_fwd(dev_i32(blk.indptr), dev_i32(blk.indices), None, blk.num_src, "gcn", torch.from_numpy(X).cuda(),
                       torch.from_numpy(W).cuda(), torch.from_numpy(b).cuda(), True, H=H.t, Y=Y.t)
    H.check("layer H")
    Y.check("layer Y")
    Href = oracle.aggregate_fwd(blk.indptr, blk.indices, None, blk.num_src, "gcn", "f32", X)
    assert_close(H.t.cpu().numpy(), Href, "f32", "layer H")
    np.testing.assert_allclose(Y.t.cpu().numpy(), oracle.update_fwd(Href, W, b, True), rtol=2e-4, atol=2e-4)


def test_plan_buffer_between_guard_bands():
    """The bookkeeping kernels (both transposes, every array of a plan and their scratch) write inside
    the plan buffer: a buffer of exactly fastgl_block_plan_bytes bytes between two 64 KiB bands."""
    rng = np.random.default_rng(77)
    band = 1 << 16
    cases = list(blocks()) + [
        ("few-sources", bg.random_block(rng, 70000, 300, 3.0)),                 # one bucket in several parts
        ("three-buckets", bg.random_block(rng, 20000, 5000, 12.0)),
        ("ten-bit-split", bg.random_block(rng, 2000, 600_000, 100.0)),
        ("radix-sort", bg.random_block(rng, 3000, 2_500_000, 20.0)),            # more than 2^21 sources
    ]
    for name, blk in cases:
        for parts in (B.PLAN_ALL | B.PLAN_PERM, B.PLAN_ALL, B.PLAN_FWD | B.PLAN_SRC_DEG):
            print(f"guard bands: plan of {name} parts={parts} dst={blk.num_dst} src={blk.num_src} E={blk.num_edges}",
                  flush=True)
            need = B.fastgl_block_plan_bytes(blk.num_dst, blk.num_src, blk.num_edges)
            raw = torch.zeros(need + 2 * band, dtype=torch.uint8, device="cuda")
            raw[:band] = 0xA5
            raw[band + need:] = 0xA5
            ip, ix = dev_i32(blk.indptr), dev_i32(blk.indices)
            plan = B.fastgl_block_plan_create(ip, ix, blk.num_src, parts, raw[band:band + need])
            torch.cuda.synchronize()
            assert bool((raw[:band] == 0xA5).all()), f"{name}: store below the plan buffer"
            assert bool((raw[band + need:] == 0xA5).all()), f"{name}: store above the plan buffer"
            v = plan.export()
            din, dout = oracle.degrees(blk.indptr, blk.indices, blk.num_src)
            assert np.array_equal(read_i32(plan, v.dout, blk.num_src), dout), f"{name}: out-degrees"
            assert np.array_equal(read_i32(plan, v.din, blk.num_dst), din), f"{name}: in-degrees"
            plan.destroy()
