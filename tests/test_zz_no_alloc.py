"""The entry point that allocates nothing (fastgl_block_aggregate_fwd_static: scratch in a static
device array) against the entry point it is a variant of (fastgl_block_aggregate_fwd with a caller's
workspace), through the C ABI: two calls in a row on one GPU, the second on a smaller block, so the
array still holds the first call's bookkeeping and partial sums when the second call starts."""
import numpy as np
import pytest
import torch

import blockgen as bg
import oracle
from paper_2409_14939_amd import binding as B
from gpu_util import assert_close, dev_feat, dev_i32, host_feat, make_inputs

pytestmark = pytest.mark.gpu


def blocks():
    rng = np.random.default_rng(77)
    # rows above the long-row threshold in both (their partial sums live in the scratch array),
    # empty rows, a ragged tail; the second block is smaller in every dimension
    big = bg.random_block(rng, 4099, 9001, 7.0, empty_frac=0.1, hub_rows=6, hub_deg=2100)
    small = bg.random_block(rng, 517, 1201, 3.0, empty_frac=0.2, hub_rows=2, hub_deg=700)
    return big, small


@pytest.mark.parametrize("dtype,mode,feat,weighted", [("f32", "gcn", 100, False), ("f32", "mean", 37, True),
                                                      ("bf16", "sum", 128, True), ("f32", "sum", 256, False)])
def test_static_scratch_matches_workspace_entry_point(dtype, mode, feat, weighted):
    rng = np.random.default_rng(5 + feat)
    for which, blk in zip(("first call", "second call, smaller block"), blocks()):
        print(f"no-alloc {which}: dtype={dtype} mode={mode} F={feat} weighted={weighted} dst={blk.num_dst} "
              f"src={blk.num_src} E={blk.num_edges}", flush=True)
        ip, ix = dev_i32(blk.indptr), dev_i32(blk.indices)
        w = rng.standard_normal(blk.num_edges).astype(np.float32) if weighted else None
        wd = None if w is None else torch.from_numpy(w).cuda()
        X = make_inputs(rng, blk.num_src, feat, dtype)
        Xd = dev_feat(X, dtype)
        ref = B.fastgl_block_aggregate_fwd(ip, ix, wd, blk.num_src, mode, Xd)         # caller's workspace
        out = torch.full_like(ref, float("nan"))
        B.fastgl_block_aggregate_fwd_static(ip, ix, wd, blk.num_src, mode, Xd, out)   # static scratch array
        torch.cuda.synchronize()
        got, want = host_feat(out, dtype), host_feat(ref, dtype)
        assert_close(got, want, dtype, which + " vs workspace entry point")
        assert np.array_equal(got, want), "same kernels, same order of additions: the bits must agree"
        assert_close(got, oracle.aggregate_fwd(blk.indptr, blk.indices, w, blk.num_src, mode, dtype, X), dtype,
                     which + " vs oracle")


def test_static_scratch_refuses_a_block_beyond_its_array():
    # bookkeeping alone (12 bytes per destination, 8 per source) passes 64 MiB; refused on the host
    n = 6_000_000
    ip = torch.zeros(n + 1, dtype=torch.int32, device="cuda")
    ix = torch.zeros(0, dtype=torch.int32, device="cuda")
    X = torch.zeros((1, 4), device="cuda")
    out = torch.empty((n, 4), device="cuda")
    with pytest.raises(B.FastglError) as e:
        B.fastgl_block_aggregate_fwd_static(ip, ix, None, 1, "sum", X, out)
    assert e.value.status == B.FASTGL_ERR_WORKSPACE and "static scratch" in str(e.value)
