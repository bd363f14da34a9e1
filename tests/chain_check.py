"""Element-by-element comparison of a chained two-layer GCN step (aggregate, update, ReLU; then the
backward pass) computed on the GPU, every link fed with the GPU's own previous result, against the
same chain of oracle calls.

Each link has its own tolerance (aggregation: the stated 1e-5 relative + 1e-6 absolute; update
phase: the rounding bound derived in test_gpu_update.py).  Because the GPU feeds its own slightly
different intermediates forward, the bound of a link's output is the link's own tolerance plus the
previous links' bounds pushed through the link with absolute values (every link is linear, the
ReLU is 1-Lipschitz).  The one place where a small difference could become a large one is the
ReLU gate of the backward pass (an element within rounding of zero may fall on the other side), so
the GPU's backward update of the gated layer takes the ORACLE's forward output as its gate.
All bounds are computed in fp64 from the oracle's values; a structural mistake (a dropped term, a
wrong sign, a transposed operand) is off by the size of the result, orders of magnitude above them."""
import numpy as np

import oracle

U = 2.0 ** -24
SLACK = 1.0 + 1e-5      # the error operators below round their own results


def agg_tol(ref_abs):
    return 1e-6 + 1e-5 * ref_abs


def gemm_tol(absprod, L, ref_abs):
    return (L + 4) * U * absprod + U * ref_abs + 1e-30


def agg_abs(blk, mode, e, backward=False):
    """The aggregation operator (its weights are non-negative) applied to a non-negative error matrix."""
    indptr, indices, num_src = blk
    f = oracle.aggregate_bwd if backward else oracle.aggregate_fwd
    e32 = np.ascontiguousarray(e * SLACK, dtype=np.float32)
    return f(indptr, indices, None, num_src, mode, "f32", e32).astype(np.float64) * SLACK


def assert_within(name, got, ref, bound):
    got, ref = np.asarray(got, np.float64), np.asarray(ref, np.float64)
    assert got.shape == ref.shape, (name, got.shape, ref.shape)
    err = np.abs(got - ref)
    bad = err > bound
    if bad.any():
        i = np.unravel_index(np.argmax(err - bound), err.shape)
        raise AssertionError(f"{name}: {int(bad.sum())} of {bad.size} elements beyond the propagated bound; worst at "
                             f"{i}: got {got[i]!r} ref {ref[i]!r} bound {bound[i]!r}")
    # the bound must stay a rounding-level statement, not grow into something that hides a mistake:
    # worst-case bounds grow with the chain lengths (a few 1e-3 of the result's size after two layers
    # with hub rows of hundreds of edges); a structural mistake is off by the size of the result
    scale = np.sqrt(np.mean(ref ** 2)) + 1e-30
    assert np.sqrt(np.mean(bound ** 2)) < 2e-2 * scale + 1e-5, (name, "bound too loose", np.sqrt(np.mean(bound ** 2)), scale)


def oracle_chain(blocks, mode, X, Ws, bs, dlogits):
    """blocks: [(indptr, indices, num_src)] input layer first.  Returns the oracle's intermediates."""
    R = {}
    x = X
    for i, (blk, W, b, relu) in enumerate(zip(blocks, Ws, bs, [True, False])):
        indptr, indices, num_src = blk
        R[f"H{i}"] = oracle.aggregate_fwd(indptr, indices, None, num_src, mode, "f32", x)
        R[f"Y{i}"] = x = oracle.update_fwd(R[f"H{i}"], W, b, relu)
    R["dH1"], R["dW1"], R["db1"] = oracle.update_bwd(R["H1"], Ws[1], None, dlogits, False)
    indptr, indices, num_src = blocks[1]
    R["dY0"] = oracle.aggregate_bwd(indptr, indices, None, num_src, mode, "f32", R["dH1"])
    _, R["dW0"], R["db0"] = oracle.update_bwd(R["H0"], Ws[0], R["Y0"], R["dY0"], True, want=("dW", "db"))
    return R


def compare(blocks, mode, X, Ws, bs, dlogits, R, G, slab_rows):
    """R: oracle_chain(...); G: the GPU chain's results under the same keys (numpy).  The GPU chain
    must have gated its layer-0 backward update with R["Y0"].  slab_rows(M, K, N) = the height of the
    slabs whose partial weight gradients the kernel adds in fp64 (the fp32 chain length of dW / db)."""
    f64 = lambda a: np.abs(np.asarray(a, np.float64))
    aW0, aW1, adl = f64(Ws[0]), f64(Ws[1]), f64(dlogits)
    K0, K1, N1 = Ws[0].shape[0], Ws[1].shape[0], Ws[1].shape[1]
    # ---- forward
    e_H0 = agg_tol(f64(R["H0"]))
    assert_within("H0", G["H0"], R["H0"], e_H0)
    aH0 = f64(R["H0"]) + e_H0
    e_Y0 = e_H0 @ aW0 + gemm_tol(aH0 @ aW0 + f64(bs[0]), K0 + 1, f64(R["Y0"]) + e_H0 @ aW0)
    assert_within("Y0", G["Y0"], R["Y0"], e_Y0)
    p = agg_abs(blocks[1], mode, e_Y0)
    e_H1 = p + agg_tol(f64(R["H1"]) + p)
    assert_within("H1", G["H1"], R["H1"], e_H1)
    aH1 = f64(R["H1"]) + e_H1
    e_Y1 = e_H1 @ aW1 + gemm_tol(aH1 @ aW1 + f64(bs[1]), K1 + 1, f64(R["Y1"]) + e_H1 @ aW1)
    assert_within("logits", G["Y1"], R["Y1"], e_Y1)
    # ---- backward
    M1, M0 = R["H1"].shape[0], R["H0"].shape[0]
    L1, L0 = min(M1, slab_rows(M1, K1, N1)), min(M0, slab_rows(M0, K0, Ws[0].shape[1]))
    e_dH1 = gemm_tol(adl @ aW1.T, N1, f64(R["dH1"]))
    assert_within("dH1", G["dH1"], R["dH1"], e_dH1)
    e_dW1 = e_H1.T @ adl + gemm_tol(aH1.T @ adl, L1, f64(R["dW1"]) + e_H1.T @ adl)
    assert_within("dW1", G["dW1"], R["dW1"], e_dW1)
    assert_within("db1", G["db1"], R["db1"], gemm_tol(adl.sum(axis=0), L1, f64(R["db1"])))
    p = agg_abs(blocks[1], mode, e_dH1, backward=True)
    e_dY0 = p + agg_tol(f64(R["dY0"]) + p)
    assert_within("dY0", G["dY0"], R["dY0"], e_dY0)
    gate = (np.asarray(R["Y0"]) > 0).astype(np.float64)
    adZ, e_dZ = f64(R["dY0"]) * gate, e_dY0 * gate
    prop = e_H0.T @ adZ + aH0.T @ e_dZ
    e_dW0 = prop + gemm_tol(aH0.T @ (adZ + e_dZ), L0, f64(R["dW0"]) + prop)
    assert_within("dW0", G["dW0"], R["dW0"], e_dW0)
    prop = e_dZ.sum(axis=0)
    assert_within("db0", G["db0"], R["db0"], prop + gemm_tol((adZ + e_dZ).sum(axis=0), L0, f64(R["db0"]) + prop))
