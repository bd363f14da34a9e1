"""Pins of the edge-weight oracle (Eq. 1 differentiated by its weights; the softmax over a target
node's incoming edges) against things other than itself: finite differences through the pinned
aggregation oracle, the dense form, hand-worked values, the softmax Jacobian written out."""
import numpy as np
import pytest

import blockgen as bg
import oracle

MODES = ["sum", "mean", "gcn"]


def small_block(seed, nd=9, ns=14, deg=3.0):
    return bg.random_block(np.random.default_rng(seed), nd, ns, deg, empty_frac=0.2, hub_rows=1, hub_deg=11)


@pytest.mark.parametrize("mode", MODES)
def test_e1_finite_differences_through_the_aggregation(mode):
    # L(w) = <aggregate(w, X), G> is linear in w: a central difference is exact up to rounding
    blk = small_block(1)
    rng = np.random.default_rng(2)
    X = bg.features_f32(rng, blk.num_src, 5)
    G = bg.features_f32(rng, blk.num_dst, 5)
    w = rng.standard_normal(blk.num_edges).astype(np.float32)
    gw = oracle.edge_weight_grad(blk.indptr, blk.indices, blk.num_src, mode, "f32", X, G)

    def loss(wv):
        out = oracle.aggregate_fwd(blk.indptr, blk.indices, wv, blk.num_src, mode, "f32", X)
        return float((out.astype(np.float64) * G).sum())
    for e in range(blk.num_edges):
        wp, wm = w.copy(), w.copy()
        wp[e] += 1.0
        wm[e] -= 1.0
        assert abs((loss(wp) - loss(wm)) / 2 - gw[e]) <= 2e-5 * (1 + abs(gw[e])), e


@pytest.mark.parametrize("mode", MODES)
def test_e2_dense_form(mode):
    blk = small_block(3, nd=12, ns=20)
    rng = np.random.default_rng(4)
    X = rng.standard_normal((blk.num_src, 7)).astype(np.float32)
    G = rng.standard_normal((blk.num_dst, 7)).astype(np.float32)
    din = np.maximum(np.diff(blk.indptr), 1).astype(np.float64)
    dout = np.maximum(np.bincount(blk.indices, minlength=blk.num_src), 1).astype(np.float64)
    c = {"sum": np.ones_like(din), "mean": 1 / din, "gcn": din ** -0.5}[mode]
    s = dout ** -0.5 if mode == "gcn" else np.ones_like(dout)
    dense = (c[:, None] * (G.astype(np.float64) @ X.astype(np.float64).T)) * s[None, :]     # dL/dA[u, v]
    rows = np.repeat(np.arange(blk.num_dst), np.diff(blk.indptr))
    gw = oracle.edge_weight_grad(blk.indptr, blk.indices, blk.num_src, mode, "f32", X, G)
    assert np.array_equal(gw, dense[rows, blk.indices].astype(np.float32))


def test_e3_bf16_inputs_are_read_exactly():
    blk = small_block(5)
    rng = np.random.default_rng(6)
    Xb = bg.to_bf16_bits(bg.features_f32(rng, blk.num_src, 4))
    Gb = bg.to_bf16_bits(bg.features_f32(rng, blk.num_dst, 4))
    got = oracle.edge_weight_grad(blk.indptr, blk.indices, blk.num_src, "sum", "bf16", Xb, Gb)
    ref = oracle.edge_weight_grad(blk.indptr, blk.indices, blk.num_src, "sum", "f32", bg.bf16_bits_to_f32(Xb),
                                  bg.bf16_bits_to_f32(Gb))
    assert np.array_equal(got, ref)


def test_e4_softmax_hand_worked():
    # rows: [0, ln 3] -> (1/4, 3/4); one edge -> 1; empty row; [5, 5, 5] -> thirds
    indptr = np.array([0, 2, 3, 3, 6], np.int32)
    score = np.array([0.0, np.log(3.0), -7.5, 5, 5, 5], np.float32)
    a = oracle.edge_softmax_fwd(indptr, score)
    np.testing.assert_allclose(a, [0.25, 0.75, 1.0, 1 / 3, 1 / 3, 1 / 3], rtol=3e-7)
    # huge scores do not overflow (the row maximum is subtracted)
    a = oracle.edge_softmax_fwd(np.array([0, 2], np.int32), np.array([1000.0, 1000.0], np.float32))
    assert a.tolist() == [0.5, 0.5]


def test_e5_softmax_properties_and_jacobian():
    blk = small_block(7, nd=15, ns=15, deg=4.0)
    rng = np.random.default_rng(8)
    score = (3 * rng.standard_normal(blk.num_edges)).astype(np.float32)
    da = rng.standard_normal(blk.num_edges).astype(np.float32)
    alpha = oracle.edge_softmax_fwd(blk.indptr, score)
    ds = oracle.edge_softmax_bwd(blk.indptr, alpha, da)
    shifted = oracle.edge_softmax_fwd(blk.indptr, score + np.float32(2.0))
    for u in range(blk.num_dst):
        b, e = blk.indptr[u], blk.indptr[u + 1]
        if b == e:
            continue
        a64 = alpha[b:e].astype(np.float64)
        assert abs(a64.sum() - 1) < 1e-6 and (a64 > 0).all()
        s64 = score[b:e].astype(np.float64)
        ref = np.exp(s64 - s64.max()) / np.exp(s64 - s64.max()).sum()               # numpy, row by row
        np.testing.assert_allclose(a64, ref, rtol=2e-7)
        np.testing.assert_allclose(shifted[b:e], alpha[b:e], rtol=2e-6)              # shift invariance
        J = np.diag(a64) - np.outer(a64, a64)                                       # d alpha / d score
        np.testing.assert_allclose(ds[b:e], J.T @ da[b:e].astype(np.float64), rtol=1e-5, atol=1e-7)
        assert abs(ds[b:e].astype(np.float64).sum()) < 1e-5                          # gradients of a row cancel


def test_e6_softmax_backward_finite_differences():
    indptr = np.array([0, 4, 4, 7], np.int32)
    rng = np.random.default_rng(9)
    score = rng.standard_normal(7)
    da = rng.standard_normal(7).astype(np.float32)

    def loss(s):
        # fp64 softmax written here, not the oracle's
        out = 0.0
        for b, e in ((0, 4), (4, 7)):
            z = np.exp(s[b:e] - s[b:e].max())
            out += float((z / z.sum() * da[b:e]).sum())
        return out
    alpha = oracle.edge_softmax_fwd(indptr, score.astype(np.float32))
    ds = oracle.edge_softmax_bwd(indptr, alpha, da)
    s32 = score.astype(np.float32).astype(np.float64)
    for k in range(7):
        sp, sm = s32.copy(), s32.copy()
        sp[k] += 1e-5
        sm[k] -= 1e-5
        assert abs((loss(sp) - loss(sm)) / 2e-5 - ds[k]) < 1e-5, k


def test_e7_attention_logits_hand_worked():
    # rows: u0 <- {v0, v2}, u1 <- {}, u2 <- {v1}; el = (1, 5, -3), er = (0.5, 1, -4); slope 0.2
    indptr, indices = np.array([0, 2, 2, 3], np.int32), np.array([0, 2, 1], np.int32)
    el, er = np.array([1, 5, -3], np.float32), np.array([0.5, 1, -4], np.float32)
    s = oracle.edge_score_fwd(indptr, indices, el, er, 0.2)
    # 1 + 0.5 = 1.5;  1 - 4 = -3 -> 0.2 * -3 = -0.6;  -3 + 1 = -2 -> -0.4
    assert np.array_equal(s, np.array([1.5, np.float32(0.2 * -3.0), np.float32(0.2 * -2.0)], np.float32))
    ds = np.array([10, 100, 1000], np.float32)
    g_el, g_er = oracle.edge_score_bwd(indptr, indices, el, er, 0.2, ds)
    # g = (10, 0.2 * 100, 0.2 * 1000) = (10, 20, 200)
    assert np.allclose(g_el, [30, 0, 200], rtol=1e-7) and np.allclose(g_er, [10, 200, 20], rtol=1e-7)


def test_e8_attention_logits_dense_form_and_slope_one():
    blk = small_block(11, nd=13, ns=21)
    rng = np.random.default_rng(12)
    el, er = rng.standard_normal(blk.num_dst).astype(np.float32), rng.standard_normal(blk.num_src).astype(np.float32)
    rows = np.repeat(np.arange(blk.num_dst), np.diff(blk.indptr))
    dense = el.astype(np.float64)[:, None] + er.astype(np.float64)[None, :]
    for slope in (0.2, 0.0, 1.0):
        s = oracle.edge_score_fwd(blk.indptr, blk.indices, el, er, slope)
        ref = dense[rows, blk.indices]
        ref = np.where(ref > 0, ref, float(np.float32(slope)) * ref)      # the slope is an fp32 parameter
        assert np.array_equal(s, ref.astype(np.float32)), slope
    # slope 1: the identity, so the gradients are plain sums of grad_score over rows / over neighbours
    ds = rng.standard_normal(blk.num_edges).astype(np.float32)
    g_el, g_er = oracle.edge_score_bwd(blk.indptr, blk.indices, el, er, 1.0, ds)
    assert np.allclose(g_el, np.bincount(rows, ds.astype(np.float64), blk.num_dst), rtol=1e-6, atol=1e-7)
    assert np.allclose(g_er, np.bincount(blk.indices, ds.astype(np.float64), blk.num_src), rtol=1e-6, atol=1e-7)


def test_e9_attention_logits_finite_differences():
    blk = small_block(13, nd=10, ns=15)
    rng = np.random.default_rng(14)
    el, er = rng.standard_normal(blk.num_dst).astype(np.float32), rng.standard_normal(blk.num_src).astype(np.float32)
    ds = rng.standard_normal(blk.num_edges).astype(np.float32)
    g_el, g_er = oracle.edge_score_bwd(blk.indptr, blk.indices, el, er, 0.2, ds)
    rows = np.repeat(np.arange(blk.num_dst), np.diff(blk.indptr))

    def loss(a, b):         # an fp64 LeakyReLU written here; piecewise linear, so a small step is exact off the kinks
        x = a[rows] + b[blk.indices]
        return float((np.where(x > 0, x, 0.2 * x) * ds).sum())
    a0, b0 = el.astype(np.float64), er.astype(np.float64)
    h = 1e-6
    for u in range(blk.num_dst):
        d = np.zeros_like(a0); d[u] = h
        assert abs((loss(a0 + d, b0) - loss(a0 - d, b0)) / (2 * h) - g_el[u]) <= 1e-4 * (1 + abs(g_el[u])), u
    for v in range(blk.num_src):
        d = np.zeros_like(b0); d[v] = h
        assert abs((loss(a0, b0 + d) - loss(a0, b0 - d)) / (2 * h) - g_er[v]) <= 1e-4 * (1 + abs(g_er[v])), v
