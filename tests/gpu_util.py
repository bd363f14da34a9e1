"""Helpers for the GPU parity tests: move numpy inputs to the device, call the
C ABI through the binding, bring results back."""
import numpy as np
import torch

import blockgen as bg
from paper_2409_14939_amd import binding as B

F32_TOL = dict(rtol=1e-5, atol=1e-6)     # the tolerance the benchmark spec states for fp32
BF16_TOL = dict(rtol=2e-2, atol=1e-5)    # 2e-2 relative for bf16; atol absorbs fp32-accumulation noise


def dev_i32(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).cuda()


def dev_feat(a, dtype):
    if dtype == "f32":
        return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.uint16).view(np.int16)).cuda().view(torch.bfloat16)


def host_feat(t, dtype):
    if dtype == "f32":
        return t.cpu().numpy()
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


def as_f64(a, dtype):
    return a.astype(np.float64) if dtype == "f32" else bg.bf16_bits_to_f32(a).astype(np.float64)


def make_inputs(rng, rows, feat, dtype):
    x = bg.features_f32(rng, rows, feat)
    return x if dtype == "f32" else bg.to_bf16_bits(x)


def assert_close(got, ref, dtype, what=""):
    tol = F32_TOL if dtype == "f32" else BF16_TOL
    g, r = as_f64(got, dtype), as_f64(ref, dtype)
    assert g.shape == r.shape, (what, g.shape, r.shape)
    err = np.abs(g - r)
    lim = tol["atol"] + tol["rtol"] * np.abs(r)
    bad = err > lim
    if bad.any():
        i = np.unravel_index(np.argmax(err - lim), err.shape)
        raise AssertionError(f"{what}: {bad.sum()} of {bad.size} elements out of tolerance; worst at {i}: "
                             f"got {g[i]!r} ref {r[i]!r}")


def read_i32(plan, ptr, n):
    """n int32 at a device address inside the plan's own buffer (plan views)."""
    if n == 0:
        return np.zeros(0, np.int32)
    off = ptr - plan.mem.data_ptr()
    assert 0 <= off and off + 4 * n <= plan.mem.numel()
    torch.cuda.synchronize()
    return plan.mem[off:off + 4 * n].view(torch.int32).cpu().numpy()


def read_f32(plan, ptr, n):
    return read_i32(plan, ptr, n).view(np.float32)
