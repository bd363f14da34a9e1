"""Pins for the CPU oracle: it is checked against things other than itself.

Dense A.X / A^T.G built independently in numpy fp64 (Eq. 1 / Eq. 5 as matrix
products), closed forms, invariants, finite differences, brute force loops.
Each pin is chosen so that a plausible mistake (dropped term, wrong sign or
index, transposed operand, wrong degree in a scale) fails at least one.
"""
import numpy as np
import pytest

import blockgen as bg
import oracle

MODES = ["sum", "mean", "gcn"]


def dense_A(blk, edge_w, mode):
    """A[u,v] = sum over parallel edges of w_uv, built with plain numpy."""
    A = np.zeros((blk.num_dst, blk.num_src), dtype=np.float64)
    din = np.diff(blk.indptr).astype(np.float64)
    dout = np.bincount(blk.indices, minlength=blk.num_src).astype(np.float64)
    rows = np.repeat(np.arange(blk.num_dst), np.diff(blk.indptr))
    w = np.ones(blk.num_edges) if edge_w is None else edge_w.astype(np.float64)
    if mode == "mean":
        w = w / np.maximum(din[rows], 1.0)
    elif mode == "gcn":
        w = w / np.sqrt(np.maximum(din[rows], 1.0) * np.maximum(dout[blk.indices], 1.0))
    np.add.at(A, (rows, blk.indices), w)
    return A


def small_blocks():
    rng = np.random.default_rng(7)
    out = []
    for nd, ns, deg in [(1, 1, 1.0), (5, 9, 2.0), (17, 40, 3.5), (64, 128, 6.0), (33, 7, 4.0)]:
        out.append(bg.random_block(rng, nd, ns, deg))
    out.append(bg.random_block(rng, 8, 16, 0.0, empty_frac=1.0))       # no edges at all
    out.append(bg.random_block(rng, 12, 30, 2.0, hub_rows=2, hub_deg=90))
    return out


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("feat", [1, 3, 32, 100])
@pytest.mark.parametrize("weighted", [False, True])
def test_p1_dense_forward_and_backward(mode, feat, weighted):
    rng = np.random.default_rng(11)
    for blk in small_blocks():
        w = rng.standard_normal(blk.num_edges).astype(np.float32) if weighted else None
        A = dense_A(blk, w, mode)
        X = bg.features_f32(rng, blk.num_src, feat)
        G = bg.features_f32(rng, blk.num_dst, feat)
        out = oracle.aggregate_fwd(blk.indptr, blk.indices, w, blk.num_src, mode, "f32", X)
        dX = oracle.aggregate_bwd(blk.indptr, blk.indices, w, blk.num_src, mode, "f32", G)
        ref_out = (A @ X.astype(np.float64)).astype(np.float32)
        ref_dX = (A.T @ G.astype(np.float64)).astype(np.float32)
        # both are fp64 sums rounded once; only the order of the fp64 adds differs
        np.testing.assert_allclose(out, ref_out, rtol=2e-7, atol=1e-12)
        np.testing.assert_allclose(dX, ref_dX, rtol=2e-7, atol=1e-12)


def test_p2_all_ones_gives_degree_counts():
    rng = np.random.default_rng(3)
    blk = bg.random_block(rng, 50, 80, 5.0, hub_rows=1, hub_deg=300)
    din, dout = oracle.degrees(blk.indptr, blk.indices, blk.num_src)
    assert np.array_equal(din, np.diff(blk.indptr))
    assert np.array_equal(dout, np.bincount(blk.indices, minlength=blk.num_src))
    assert din.sum() == dout.sum() == blk.num_edges
    X = np.ones((blk.num_src, 4), np.float32)
    out = oracle.aggregate_fwd(blk.indptr, blk.indices, None, blk.num_src, "sum", "f32", X)
    assert np.array_equal(out, np.repeat(din[:, None], 4, 1).astype(np.float32))
    G = np.ones((blk.num_dst, 4), np.float32)
    dX = oracle.aggregate_bwd(blk.indptr, blk.indices, None, blk.num_src, "sum", "f32", G)
    assert np.array_equal(dX, np.repeat(dout[:, None], 4, 1).astype(np.float32))
    # bf16 holds integers exactly up to 256
    Xb = bg.to_bf16_bits(np.ones((blk.num_src, 4), np.float32))
    outb = oracle.aggregate_fwd(blk.indptr, blk.indices, None, blk.num_src, "sum", "bf16", Xb)
    small = din <= 256
    assert np.array_equal(bg.bf16_bits_to_f32(outb)[small], out[small])


def test_p3_mean_preserves_constants_and_zero_rows_are_zero():
    rng = np.random.default_rng(4)
    blk = bg.random_block(rng, 40, 60, 4.0, empty_frac=0.3)
    din = np.diff(blk.indptr)
    c = np.float32(2.71875)
    X = np.full((blk.num_src, 5), c, np.float32)
    out = oracle.aggregate_fwd(blk.indptr, blk.indices, None, blk.num_src, "mean", "f32", X)
    np.testing.assert_allclose(out[din > 0], c, rtol=1e-7)
    assert np.all(out[din == 0] == 0.0) and (din == 0).any()
    for mode in MODES:
        G = bg.features_f32(rng, blk.num_dst, 5)
        dX = oracle.aggregate_bwd(blk.indptr, blk.indices, None, blk.num_src, mode, "f32", G)
        dout = np.bincount(blk.indices, minlength=blk.num_src)
        assert (dout == 0).any() and np.all(dX[dout == 0] == 0.0)


def test_p4_gcn_closed_form():
    rng = np.random.default_rng(5)
    blk = bg.random_block(rng, 30, 45, 5.0)
    din = np.diff(blk.indptr).astype(np.float64)
    dout = np.bincount(blk.indices, minlength=blk.num_src).astype(np.float64)
    X = np.repeat(np.sqrt(np.maximum(dout, 1.0))[:, None], 3, 1).astype(np.float32)
    out = oracle.aggregate_fwd(blk.indptr, blk.indices, None, blk.num_src, "gcn", "f32", X)
    # sum_v dout^-1/2 * sqrt(dout) / sqrt(din) = din / sqrt(din) = sqrt(din)
    np.testing.assert_allclose(out[:, 0], np.sqrt(din), rtol=3e-7)
    G = np.repeat(np.sqrt(np.maximum(din, 1.0))[:, None], 3, 1).astype(np.float32)
    dX = oracle.aggregate_bwd(blk.indptr, blk.indices, None, blk.num_src, "gcn", "f32", G)
    np.testing.assert_allclose(dX[:, 0], np.sqrt(dout), rtol=3e-7)


@pytest.mark.parametrize("mode", MODES)
def test_p5_finite_differences(mode):
    """L(X) = <fwd(X), G> is linear, so a central difference is exact up to
    rounding; the derivative w.r.t. X[v,j] must equal bwd(G)[v,j]."""
    rng = np.random.default_rng(6)
    blk = bg.random_block(rng, 9, 12, 3.0)
    w = rng.standard_normal(blk.num_edges).astype(np.float32)
    X = bg.features_f32(rng, blk.num_src, 3)
    G = bg.features_f32(rng, blk.num_dst, 3)
    dX = oracle.aggregate_bwd(blk.indptr, blk.indices, w, blk.num_src, mode, "f32", G)

    def loss(Xp):
        o = oracle.aggregate_fwd(blk.indptr, blk.indices, w, blk.num_src, mode, "f32", Xp)
        return float((o.astype(np.float64) * G.astype(np.float64)).sum())

    h = np.float32(0.25)
    for v in range(blk.num_src):
        for j in range(3):
            Xp, Xm = X.copy(), X.copy()
            Xp[v, j] += h
            Xm[v, j] -= h
            fd = (loss(Xp) - loss(Xm)) / (float(Xp[v, j]) - float(Xm[v, j]))
            assert abs(fd - float(dX[v, j])) <= 2e-5 * max(1.0, abs(fd))


@pytest.mark.parametrize("mode", MODES)
def test_p6_adjoint_identity_medium(mode):
    rng = np.random.default_rng(8)
    blk = bg.random_block(rng, 3000, 9000, 8.0, hub_rows=3, hub_deg=2500)
    w = rng.standard_normal(blk.num_edges).astype(np.float32)
    X = bg.features_f32(rng, blk.num_src, 16)
    G = bg.features_f32(rng, blk.num_dst, 16)
    out = oracle.aggregate_fwd(blk.indptr, blk.indices, w, blk.num_src, mode, "f32", X)
    dX = oracle.aggregate_bwd(blk.indptr, blk.indices, w, blk.num_src, mode, "f32", G)
    lhs = (out.astype(np.float64) * G).sum()
    rhs = (X.astype(np.float64) * dX).sum()
    scale = np.abs(out.astype(np.float64) * G).sum()
    assert abs(lhs - rhs) <= 1e-6 * scale   # fp32 rounding of out/dX only


def test_p8_transpose_structure():
    rng = np.random.default_rng(9)
    for blk in small_blocks() + [bg.random_block(rng, 500, 300, 7.0, hub_rows=2, hub_deg=700)]:
        pT, iT, perm = oracle.transpose(blk.indptr, blk.indices, blk.num_src)
        e = blk.num_edges
        assert pT[0] == 0 and pT[-1] == e and np.all(np.diff(pT) >= 0)
        assert np.array_equal(np.diff(pT), np.bincount(blk.indices, minlength=blk.num_src))
        assert np.array_equal(np.sort(perm), np.arange(e))
        rows = np.repeat(np.arange(blk.num_dst), np.diff(blk.indptr))
        assert np.array_equal(iT, rows[perm])
        # sorted by source, ties by ascending edge id  == numpy's stable argsort
        assert np.array_equal(perm, np.argsort(blk.indices, kind="stable"))
        # transposing twice gives the original graph with every row stably sorted by source
        p2, i2, _ = oracle.transpose(pT, iT, blk.num_dst)
        assert np.array_equal(p2, blk.indptr)
        for u in range(blk.num_dst):
            seg = blk.indices[blk.indptr[u]:blk.indptr[u + 1]]
            assert np.array_equal(i2[p2[u]:p2[u + 1]], np.sort(seg, kind="stable"))


def test_long_row_buckets():
    ptr = np.array([0, 3, 3, 600, 601, 1700, 1700, 2212], np.int32)
    rows, cptr = oracle.long_rows(ptr, 512, 256)
    # lengths 3,0,597,1,1099,0,512 -> rows 2 and 4 exceed 512; chunks ceil(597/256)=3, ceil(1099/256)=5
    assert rows.tolist() == [2, 4] and cptr.tolist() == [0, 3, 8]
    rows, cptr = oracle.long_rows(ptr, 2 ** 30, 256)
    assert rows.size == 0 and cptr.tolist() == [0]


def test_work_split_covers_rows_with_bounded_work():
    rng = np.random.default_rng(14)
    for blk in small_blocks() + [bg.random_block(rng, 700, 300, 9.0, hub_rows=3, hub_deg=500)]:
        ptr = blk.indptr.astype(np.int64)
        n, work = blk.num_dst, 64
        sp = oracle.work_split(blk.indptr, work)
        assert sp[0] == 0 and sp[-1] == n and np.all(np.diff(sp) >= 0)
        assert sp.shape[0] == -(-(n + blk.num_edges) // work) + 1
        w = ptr + np.arange(n + 1)          # work before row r
        for g in range(sp.shape[0] - 1):
            a, b = sp[g], sp[g + 1]
            if a < b:                        # all rows of the set start inside its work window
                assert g * work <= w[a] and w[b - 1] < (g + 1) * work
        # independent definition: searchsorted on the work prefix
        assert np.array_equal(sp, np.searchsorted(w, np.arange(sp.shape[0]) * work, side="left").clip(max=n))


@pytest.mark.parametrize("mode", MODES)
def test_p9_metamorphic(mode):
    rng = np.random.default_rng(10)
    blk = bg.random_block(rng, 25, 40, 4.0)
    X = bg.features_f32(rng, blk.num_src, 7)
    Y = bg.features_f32(rng, blk.num_src, 7)
    f = lambda Z: oracle.aggregate_fwd(blk.indptr, blk.indices, None, blk.num_src, mode, "f32", Z)
    base = f(X)
    # linearity
    np.testing.assert_allclose(f((2 * X - 3 * Y).astype(np.float32)), 2.0 * base - 3.0 * f(Y),
                               rtol=1e-5, atol=1e-5)
    # relabel sources consistently
    p = rng.permutation(blk.num_src)
    inv = np.empty_like(p)
    inv[p] = np.arange(blk.num_src)
    out2 = oracle.aggregate_fwd(blk.indptr, inv[blk.indices].astype(np.int32), None, blk.num_src,
                                mode, "f32", X[p])
    np.testing.assert_allclose(out2, base, rtol=1e-6, atol=1e-7)
    # shuffle edges inside each row
    idx = blk.indices.copy()
    for u in range(blk.num_dst):
        seg = idx[blk.indptr[u]:blk.indptr[u + 1]]
        rng.shuffle(seg)
    out3 = oracle.aggregate_fwd(blk.indptr, idx, None, blk.num_src, mode, "f32", X)
    np.testing.assert_allclose(out3, base, rtol=1e-6, atol=1e-7)


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_p10_brute_force_python_loops(mode, dtype):
    rng = np.random.default_rng(12)
    blk = bg.random_block(rng, 7, 10, 2.5)
    w = rng.standard_normal(blk.num_edges).astype(np.float32)
    Xf = bg.features_f32(rng, blk.num_src, 4)
    Gf = bg.features_f32(rng, blk.num_dst, 4)
    if dtype == "bf16":
        Xs, Gs = bg.to_bf16_bits(Xf), bg.to_bf16_bits(Gf)
        Xf, Gf = bg.bf16_bits_to_f32(Xs), bg.bf16_bits_to_f32(Gs)
    else:
        Xs, Gs = Xf, Gf
    dout = [0] * blk.num_src
    for v in blk.indices:
        dout[v] += 1
    out = [[0.0] * 4 for _ in range(blk.num_dst)]
    dX = [[0.0] * 4 for _ in range(blk.num_src)]
    for u in range(blk.num_dst):
        b, e = int(blk.indptr[u]), int(blk.indptr[u + 1])
        n = max(e - b, 1)
        for k in range(b, e):
            v = int(blk.indices[k])
            wt = float(w[k])
            if mode == "mean":
                wt /= n
            if mode == "gcn":
                wt /= (n * max(dout[v], 1)) ** 0.5
            for j in range(4):
                out[u][j] += wt * float(Xf[v, j])
                dX[v][j] += wt * float(Gf[u, j])
    o = oracle.aggregate_fwd(blk.indptr, blk.indices, w, blk.num_src, mode, dtype, Xs)
    d = oracle.aggregate_bwd(blk.indptr, blk.indices, w, blk.num_src, mode, dtype, Gs)
    if dtype == "bf16":
        o, d = bg.bf16_bits_to_f32(o), bg.bf16_bits_to_f32(d)
        tol = dict(rtol=2 ** -8, atol=1e-30)   # one bf16 rounding: half ulp = 2^-9 relative
    else:
        tol = dict(rtol=2e-7, atol=1e-12)
    np.testing.assert_allclose(o, np.array(out), **tol)
    np.testing.assert_allclose(d, np.array(dX), **tol)


def test_bf16_rounding_is_nearest_even_in_one_step():
    f = oracle.double_to_bf16
    assert f(1.0) == 0x3F80 and f(-2.0) == 0xC000 and f(0.0) == 0
    assert f(1.0 + 2 ** -8) == 0x3F80            # exact tie -> even (down)
    assert f(1.0 + 3 * 2 ** -8) == 0x3F82        # exact tie -> even (up)
    assert f(1.0 + 2 ** -8 + 2 ** -40) == 0x3F81  # just above the tie: a fp32 detour would lose this
    assert f(float(np.float32(3.389e38))) == 0x7F7F
    assert f(3.4e38) == 0x7F80 and f(float("inf")) == 0x7F80
    assert f(2.0 ** -133) == 0x0001 and f(2.0 ** -134) == 0x0000 and f(1.5 * 2.0 ** -133) == 0x0002
    # agrees with the input generator's fp32->bf16 on random fp32 values
    x = np.random.default_rng(1).standard_normal(2000).astype(np.float32)
    got = np.array([f(float(v)) for v in x], dtype=np.uint16)
    assert np.array_equal(got, bg.to_bf16_bits(x))


def test_gather_rows_is_fancy_indexing():
    rng = np.random.default_rng(2)
    T = bg.features_f32(rng, 100, 6)
    ids = rng.integers(0, 100, size=37)
    assert np.array_equal(oracle.gather_rows(T, ids, "f32"), T[ids])
    Tb = bg.to_bf16_bits(T)
    assert np.array_equal(oracle.gather_rows(Tb, ids, "bf16"), Tb[ids])


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_parallel_variant_matches_definitional(mode, dtype):
    rng = np.random.default_rng(13)
    blk = bg.random_block(rng, 400, 700, 6.0, hub_rows=2, hub_deg=900)
    w = rng.standard_normal(blk.num_edges).astype(np.float32)
    X = bg.features_f32(rng, blk.num_src, 20)
    G = bg.features_f32(rng, blk.num_dst, 20)
    if dtype == "bf16":
        X, G = bg.to_bf16_bits(X), bg.to_bf16_bits(G)
    cv = (lambda a: bg.bf16_bits_to_f32(a)) if dtype == "bf16" else (lambda a: a)
    tol = dict(rtol=2e-2, atol=1e-3) if dtype == "bf16" else dict(rtol=1e-4, atol=1e-4)
    a = oracle.aggregate_fwd(blk.indptr, blk.indices, w, blk.num_src, mode, dtype, X)
    b = oracle.par_aggregate_fwd(blk.indptr, blk.indices, w, blk.num_src, mode, dtype, X)
    np.testing.assert_allclose(cv(b), cv(a), **tol)
    a = oracle.aggregate_bwd(blk.indptr, blk.indices, w, blk.num_src, mode, dtype, G)
    b = oracle.par_aggregate_bwd(blk.indptr, blk.indices, w, blk.num_src, mode, dtype, G)
    np.testing.assert_allclose(cv(b), cv(a), **tol)


def test_paper_traffic_model_bytes():
    """Eq. 3 / Eq. 4 numerators (Section 4.2): partial sums read |N|-1 times, weights, features."""
    import os
    path = os.path.join(os.path.dirname(__file__), "golden", "eq3_eq4_bytes.txt")
    for line in open(path):
        if line.startswith("#") or not line.strip():
            continue
        n, d, naive, ma_s, ma_g = map(int, line.split())
        assert 4 * (n - 1) * d + 4 * n * d + 4 * n * d == naive
        assert 4 * (n - 1) * d + 4 * n * (d - 1) == ma_s
        assert 4 * n * d + 4 * n == ma_g
        # the feature bytes alone are what this build calls "gathered bytes" for one row
        assert 4 * n * d <= ma_g
