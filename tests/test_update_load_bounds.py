"""Host-side model of every global load address of the update kernel (csrc/update.hip: PlaneMover
init / nvalid / fetch and run_steps), checked against the extents of the operands: no lane of any
workgroup may read outside [0, numel) of the matrix it loads from, including the masked lanes (which
load the first element of the tile's first step) and the look-ahead fetch of the step after the
last one.  The model mirrors the kernel's index arithmetic line by line; it has to be changed with
it."""
import random

import numpy as np

K_TILE, K_STEP = 128, 16


def clamp4(n):
    return np.clip(n, 0, 4)


def slab_rows(M, K, N):
    tiles = (max((K + 127) // 128, 1) if K > 0 else 1) * ((N + 127) // 128)
    best, best_cost = 32, None
    for rows in range(32, 2049, 32):
        nslab = (max(M, 1) + rows - 1) // rows
        rounds = (nslab * tiles + 767) // 768
        cost = rounds * (rows * 156250 + 20000000) + nslab * (K * N + N) * 2
        if best_cost is None or cost < best_cost:
            best, best_cost = rows, cost
    return best


def operand_in_bounds(col, vec, numel, ld, o0, omax, kbeg, kend, inside, origin_of_missing_step=0):
    t = np.arange(256)
    length = max(kend - kbeg, 0)
    nstep = (length + K_STEP - 1) // K_STEP if length > 0 else 1
    n_plain = max(0, min(length // K_STEP - 1 if inside else 0, nstep - 1))
    fetches = [(kbeg, True)] + [(kbeg + K_STEP * (i + 1), i >= n_plain) for i in range(nstep)]
    for k, mask in fetches:
        kf = k if k < kend else origin_of_missing_step
        origin = kf * ld + o0 if col else o0 * ld + kf
        for s in range(2):
            if not col:
                dr = t // 4 + 64 * s
                off = dr * ld + 4 * (t % 4)
                nv = np.where(o0 + dr < omax, clamp4(kend - (k + 4 * (t % 4))), 0) if mask else np.full(256, 4)
            else:
                off = (2 * (t >> 5) + s) * ld + 4 * (t & 31)
                nv = np.where(k + 2 * (t >> 5) + s < kend, clamp4(omax - (o0 + 4 * (t & 31))), 0) if mask else np.full(256, 4)
            if vec:                       # one 16-byte load at off, or at 0 when the quad is masked
                lo = origin + np.where(nv >= 4, off, 0)
                hi = lo + 3
            else:                         # element i < nv at off + i, the others at 0
                lo = np.minimum(origin + np.where(nv > 0, off, 0), origin)
                hi = np.maximum(origin + np.where(nv > 0, off + nv - 1, 0), origin)
            if lo.min() < 0 or hi.max() >= numel:
                return False
    return True


def gemm_in_bounds(a_col, b_col, R, C, Kc, lda, ldb, numel_a, numel_b, slab=None, **kw):
    if R == 0 or Kc == 0:                 # the host hands the kernel readable pointers; every lane is masked
        return True
    tiles_r, tiles_c = (R + 127) // 128, (C + 127) // 128
    vec = lda % 4 == 0 and ldb % 4 == 0
    ranges = [(0, Kc)] if not slab else [(b, min(b + slab, Kc)) for b in range(0, Kc, slab)]
    ranges = [ranges[0], ranges[-1]]
    ok = True
    for kb, ke in ranges:
        for tr in {0, tiles_r - 1}:
            for tc in {0, tiles_c - 1}:
                r0, c0 = tr * 128, tc * 128
                inside = vec and r0 + 128 <= R and c0 + 128 <= C
                ok &= operand_in_bounds(a_col, vec, numel_a, lda, r0, R, kb, ke, inside, **kw)
                ok &= operand_in_bounds(b_col, vec, numel_b, ldb, c0, C, kb, ke, inside, **kw)
    return ok


def all_products_in_bounds(M, K, N, **kw):
    fwd = gemm_in_bounds(False, True, M, N, K, K, N, M * K, K * N, **kw)
    dh = gemm_in_bounds(False, False, M, K, N, N, N, M * N, K * N, **kw)
    dw = gemm_in_bounds(True, True, K, N, M, K, N, M * K, M * N, slab=slab_rows(M, K, N), **kw)
    return fwd and dh and dw


SHAPES = [(512345, 100, 256), (91331, 256, 256), (8000, 256, 47), (91331, 1024, 256), (1, 1, 1), (5, 3, 2),
          (129, 17, 130), (300, 100, 47), (1000, 33, 64), (128, 16, 128), (128, 32, 128), (256, 48, 256), (77, 80, 4),
          (4096, 64, 128)]


def test_every_load_of_the_update_kernel_stays_inside_its_operand():
    rng = random.Random(1)
    shapes = SHAPES + [(rng.randint(1, 700), rng.randint(1, 300), rng.randint(1, 300)) for _ in range(200)]
    for M, K, N in shapes:
        assert all_products_in_bounds(M, K, N), (M, K, N)


def test_the_model_sees_a_fetch_past_the_last_step():
    """The mistake the model exists for: taking the origin of a step beyond the range from that
    step's own index reads past the end of a "col" operand (the weight matrix of the forward pass)."""
    t = np.arange(256)
    M, K, N = 512345, 100, 256
    bad = operand_in_bounds(True, True, K * N, N, 0, N, 0, K, True, origin_of_missing_step=112)
    assert not bad
