"""Pins of the update-phase oracle (paper Section 2.1, Eq. 2, read as the GCN dense
transform Y = act(H W + b)) against things other than itself: a hand-worked example,
numpy's fp64 matmul, special cases, the adjoint identity and finite differences."""
import numpy as np
import pytest

import oracle


def _rand(rng, *shape):
    return rng.standard_normal(shape).astype(np.float32)


def test_u1_hand_worked_example():
    # H 2x3, W 3x2, worked by hand:
    #   row 0: [1,2,3]   . cols [1,0,-1] , [2,-1,0.5]  -> -2 , 1.5
    #   row 1: [-1,0,.5] . cols                         -> -1.5 , -1.75
    H = np.array([[1, 2, 3], [-1, 0, 0.5]], np.float32)
    W = np.array([[1, 2], [0, -1], [-1, 0.5]], np.float32)
    b = np.array([0.25, 2.0], np.float32)
    Z = np.array([[-2 + 0.25, 1.5 + 2.0], [-1.5 + 0.25, -1.75 + 2.0]], np.float32)
    assert np.array_equal(oracle.update_fwd(H, W, None, False), Z - b)
    assert np.array_equal(oracle.update_fwd(H, W, b, False), Z)
    Y = oracle.update_fwd(H, W, b, True)
    assert np.array_equal(Y, np.array([[0, 3.5], [0, 0.25]], np.float32))
    # backward with dY = [[1,10],[100,1000]]; the ReLU passes column 1 only
    dY = np.array([[1, 10], [100, 1000]], np.float32)
    dH, dW, db = oracle.update_bwd(H, W, Y, dY, True)
    # dZ = [[0,10],[0,1000]]; dH = dZ W^T: row0 = 10*[2,-1,.5], row1 = 1000*[2,-1,.5]
    assert np.array_equal(dH, np.array([[20, -10, 5], [2000, -1000, 500]], np.float32))
    # dW = H^T dZ: column 0 zero, column 1 = 10*H[0] + 1000*H[1]
    assert np.array_equal(dW, np.array([[0, -990], [0, 20], [0, 530]], np.float32))
    assert np.array_equal(db, np.array([0, 1010], np.float32))
    # identity activation: nothing is gated
    dH, dW, db = oracle.update_bwd(H, W, None, dY, False)
    assert np.array_equal(dH, (dY.astype(np.float64) @ W.T.astype(np.float64)).astype(np.float32))
    assert np.array_equal(db, np.array([101, 1010], np.float32))


@pytest.mark.parametrize("M,K,N", [(7, 5, 3), (33, 100, 47), (64, 17, 130)])
@pytest.mark.parametrize("relu", [False, True])
@pytest.mark.parametrize("bias", [False, True])
def test_u2_numpy_fp64_matmul(M, K, N, relu, bias):
    rng = np.random.default_rng(M * 1000 + K * 10 + N)
    H, W, dY = _rand(rng, M, K), _rand(rng, K, N), _rand(rng, M, N)
    b = _rand(rng, N) if bias else None
    Z = H.astype(np.float64) @ W.astype(np.float64)
    if bias:
        Z = Z + b.astype(np.float64)
    Yd = np.maximum(Z, 0.0) if relu else Z
    Y = oracle.update_fwd(H, W, b, relu)
    # one rounding of an fp64 sum: within half an fp32 ulp of numpy's fp64 result (whose own
    # summation order differs by a few fp64 ulps)
    np.testing.assert_allclose(Y, Yd, rtol=2.0 ** -23, atol=1e-12)
    dZ = dY.astype(np.float64) * ((Y > 0) if relu else 1.0)
    dH, dW, db = oracle.update_bwd(H, W, Y, dY, relu)
    np.testing.assert_allclose(dH, dZ @ W.T.astype(np.float64), rtol=2.0 ** -23, atol=1e-10)
    np.testing.assert_allclose(dW, H.T.astype(np.float64) @ dZ, rtol=2.0 ** -23, atol=1e-10)
    np.testing.assert_allclose(db, dZ.sum(axis=0), rtol=2.0 ** -23, atol=1e-10)


def test_u3_special_cases():
    rng = np.random.default_rng(3)
    H = _rand(rng, 19, 6)
    eye = np.eye(6, dtype=np.float32)
    assert np.array_equal(oracle.update_fwd(H, eye, None, False), H)            # identity weights
    assert np.array_equal(oracle.update_fwd(H, eye, None, True), np.maximum(H, 0))
    b = _rand(rng, 4)
    Y0 = oracle.update_fwd(H, np.zeros((6, 4), np.float32), b, False)            # zero weights -> bias rows
    assert np.array_equal(Y0, np.broadcast_to(b, (19, 4)))
    # a permutation matrix permutes columns exactly
    perm = rng.permutation(6)
    P = np.zeros((6, 6), np.float32)
    P[perm, np.arange(6)] = 1.0
    assert np.array_equal(oracle.update_fwd(H, P, None, False), H[:, perm])
    # empty shapes
    assert oracle.update_fwd(np.zeros((0, 6), np.float32), eye, None, True).shape == (0, 6)
    Yk0 = oracle.update_fwd(np.zeros((3, 0), np.float32), np.zeros((0, 4), np.float32), b, False)
    assert np.array_equal(Yk0, np.broadcast_to(b, (3, 4)))
    # parts can be skipped
    dH, dW, db = oracle.update_bwd(H, eye, None, H, False, want=("dW",))
    assert dH is None and db is None and dW.shape == (6, 6)


@pytest.mark.parametrize("relu", [False, True])
def test_u4_adjoint_identity(relu):
    """<dY, J_H v> = <dH, v> and <dY, J_W V> = <dW, V> with J the Jacobian at fixed gates."""
    rng = np.random.default_rng(11)
    M, K, N = 40, 23, 31
    H, W, b, dY = _rand(rng, M, K), _rand(rng, K, N), _rand(rng, N), _rand(rng, M, N)
    Y = oracle.update_fwd(H, W, b, relu)
    gate = (Y > 0) if relu else np.ones_like(Y, bool)
    dH, dW, db = oracle.update_bwd(H, W, Y, dY, relu)
    v, V, vb = _rand(rng, M, K), _rand(rng, K, N), _rand(rng, N)
    f8 = np.float64
    lhs_h = np.sum(dY.astype(f8) * gate * (v.astype(f8) @ W.astype(f8)))
    lhs_w = np.sum(dY.astype(f8) * gate * (H.astype(f8) @ V.astype(f8)))
    lhs_b = np.sum(dY.astype(f8) * gate * vb.astype(f8))
    assert abs(lhs_h - np.sum(dH.astype(f8) * v)) <= 1e-5 * np.sum(np.abs(dH.astype(f8) * v))
    assert abs(lhs_w - np.sum(dW.astype(f8) * V)) <= 1e-5 * np.sum(np.abs(dW.astype(f8) * V))
    assert abs(lhs_b - np.sum(db.astype(f8) * vb)) <= 1e-5 * np.sum(np.abs(db.astype(f8) * vb))


def test_u5_finite_differences_through_relu():
    """d/dtheta of L = sum(C * relu(H W + b)) by central differences in fp64 (numpy) against the
    oracle's gradients; pre-activations are kept away from the kink."""
    rng = np.random.default_rng(5)
    M, K, N = 6, 5, 4
    H, W, b, C = _rand(rng, M, K), _rand(rng, K, N), _rand(rng, N), _rand(rng, M, N)
    Z = H.astype(np.float64) @ W.astype(np.float64) + b
    assert np.min(np.abs(Z)) > 1e-3

    def loss(Hx, Wx, bx):
        return float(np.sum(C * np.maximum(Hx @ Wx + bx, 0.0)))

    Y = oracle.update_fwd(H, W, b, True)
    dH, dW, db = oracle.update_bwd(H, W, Y, C, True)
    eps = 1e-5
    H8, W8, b8 = H.astype(np.float64), W.astype(np.float64), b.astype(np.float64)
    for (i, k) in [(0, 0), (2, 3), (5, 4)]:
        Hp, Hm = H8.copy(), H8.copy()
        Hp[i, k] += eps
        Hm[i, k] -= eps
        assert abs((loss(Hp, W8, b8) - loss(Hm, W8, b8)) / (2 * eps) - dH[i, k]) < 1e-4
    for (k, j) in [(0, 0), (4, 3), (2, 1)]:
        Wp, Wm = W8.copy(), W8.copy()
        Wp[k, j] += eps
        Wm[k, j] -= eps
        assert abs((loss(H8, Wp, b8) - loss(H8, Wm, b8)) / (2 * eps) - dW[k, j]) < 1e-4
    for j in range(N):
        bp, bm = b8.copy(), b8.copy()
        bp[j] += eps
        bm[j] -= eps
        assert abs((loss(H8, W8, bp) - loss(H8, W8, bm)) / (2 * eps) - db[j]) < 1e-4


def test_u9_bf16_storage():
    """bf16 storage: inputs are read exactly, results are the fp64 sums rounded once to bf16 (Y, dH)
    or fp32 (dW, db).  Pinned by small integers (exact in every format), by the fp32 oracle on the
    same values (identical sums before the final rounding) and by numpy fp64."""
    import blockgen as bg
    # small integers: everything is exact, the two storage types must agree bit for bit
    H = np.array([[1, 2, 3], [-1, 0, 4]], np.float32)
    W = np.array([[1, 2], [0, -1], [-1, 3]], np.float32)
    b = np.array([1.0, -2.0], np.float32)
    Yb = oracle.update_fwd_bf16(bg.to_bf16_bits(H), bg.to_bf16_bits(W), b, True)
    assert np.array_equal(bg.bf16_bits_to_f32(Yb), oracle.update_fwd(H, W, b, True))
    dY = np.array([[1, -2], [3, 5]], np.float32)
    dHb, dWb, dbb = oracle.update_bwd_bf16(bg.to_bf16_bits(H), bg.to_bf16_bits(W), Yb, bg.to_bf16_bits(dY), True)
    dH, dW, db = oracle.update_bwd(H, W, bg.bf16_bits_to_f32(Yb), dY, True)
    assert np.array_equal(bg.bf16_bits_to_f32(dHb), dH) and np.array_equal(dWb, dW) and np.array_equal(dbb, db)
    # random bf16 inputs: fp64 sums through numpy, one rounding to bf16
    rng = np.random.default_rng(0)
    Hb, Wb = bg.to_bf16_bits(_rand(rng, 23, 37)), bg.to_bf16_bits(_rand(rng, 37, 11))
    dYb = bg.to_bf16_bits(_rand(rng, 23, 11))
    H64, W64, dY64 = (bg.bf16_bits_to_f32(a).astype(np.float64) for a in (Hb, Wb, dYb))
    Z = H64 @ W64
    Yb = oracle.update_fwd_bf16(Hb, Wb, None, False)
    assert np.array_equal(Yb, np.array([[oracle.double_to_bf16(z) for z in row] for row in Z], np.uint16))
    dHb, dWb, dbb = oracle.update_bwd_bf16(Hb, Wb, None, dYb, False)
    ref_dH = dY64 @ W64.T
    assert np.array_equal(dHb, np.array([[oracle.double_to_bf16(z) for z in row] for row in ref_dH], np.uint16))
    np.testing.assert_allclose(dWb, (H64.T @ dY64).astype(np.float32), rtol=1e-6, atol=1e-6)
    np.testing.assert_allclose(dbb, dY64.sum(axis=0).astype(np.float32), rtol=1e-6, atol=1e-6)
    # the ReLU gate reads the bf16 forward output
    Yr = oracle.update_fwd_bf16(Hb, Wb, None, True)
    dHr, _, dbr = oracle.update_bwd_bf16(Hb, Wb, Yr, dYb, True)
    gate = bg.bf16_bits_to_f32(Yr) > 0
    np.testing.assert_allclose(dbr, (dY64 * gate).sum(axis=0).astype(np.float32), rtol=1e-6, atol=1e-6)
    assert np.array_equal(dHr, np.array([[oracle.double_to_bf16(z) for z in row] for row in (dY64 * gate) @ W64.T], np.uint16))
