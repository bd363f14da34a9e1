"""The chained-step checker (chain_check.py) itself, on the CPU: a stand-in for the GPU chain computed
in numpy fp32 (each link rounds to fp32 and feeds the next) must pass, and the same chain with a
planted mistake in one link must fail at that link."""
import numpy as np
import pytest

import blockgen as bg
import chain_check


def dense(blk, mode):
    A = np.zeros((blk.num_dst, blk.num_src))
    din = np.maximum(np.diff(blk.indptr), 1)
    dout = np.maximum(np.bincount(blk.indices, minlength=blk.num_src), 1)
    for u in range(blk.num_dst):
        for e in range(blk.indptr[u], blk.indptr[u + 1]):
            v = blk.indices[e]
            A[u, v] += 1.0 / np.sqrt(din[u] * dout[v]) if mode == "gcn" else 1.0
    return A


def fp32_chain(As, X, Ws, bs, dlogits, gate_Y0, mistake=None):
    f = lambda a: np.asarray(a, np.float32)
    G = {}
    x = X
    for i, relu in enumerate([True, False]):
        G[f"H{i}"] = f(As[i] @ x.astype(np.float64))
        y = G[f"H{i}"].astype(np.float64) @ Ws[i] + bs[i]
        if mistake == f"bias{i}":
            y = y - bs[i]
        G[f"Y{i}"] = x = f(np.maximum(y, 0) if relu else y)
    G["dH1"] = f(dlogits.astype(np.float64) @ Ws[1].T.astype(np.float64))
    G["dW1"] = f(G["H1"].astype(np.float64).T @ dlogits)
    G["db1"] = f(dlogits.astype(np.float64).sum(axis=0))
    AT = As[1].T if mistake != "transpose" else As[1].T[::-1]
    G["dY0"] = f(AT @ G["dH1"].astype(np.float64))
    dZ = G["dY0"].astype(np.float64) * (gate_Y0 > 0)
    if mistake == "gate":
        dZ = G["dY0"].astype(np.float64)
    G["dW0"] = f(G["H0"].astype(np.float64).T @ dZ)
    G["db0"] = f(dZ.sum(axis=0))
    return G


def setup():
    rng = np.random.default_rng(3)
    b0 = bg.random_block(rng, 90, 200, 4.0, empty_frac=0.05, hub_rows=1, hub_deg=60)
    b1 = bg.random_block(rng, 30, 90, 5.0, empty_frac=0.05, hub_rows=1, hub_deg=40)
    X = bg.features_f32(rng, b0.num_src, 20)
    Ws = [(rng.standard_normal((20, 24)) / np.sqrt(20)).astype(np.float32),
          (rng.standard_normal((24, 7)) / np.sqrt(24)).astype(np.float32)]
    bs = [(0.1 * rng.standard_normal(24)).astype(np.float32), (0.1 * rng.standard_normal(7)).astype(np.float32)]
    dlogits = rng.standard_normal((b1.num_dst, 7)).astype(np.float32)
    csr = [(b.indptr, b.indices, b.num_src) for b in (b0, b1)]
    return [b0, b1], csr, X, Ws, bs, dlogits


def test_fp32_chain_passes_and_planted_mistakes_fail():
    blocks, csr, X, Ws, bs, dlogits = setup()
    R = chain_check.oracle_chain(csr, "gcn", X, Ws, bs, dlogits)
    As = [dense(b, "gcn") for b in blocks]
    slab = lambda M, K, N: 64
    chain_check.compare(csr, "gcn", X, Ws, bs, dlogits, R, fp32_chain(As, X, Ws, bs, dlogits, R["Y0"]), slab)
    for mistake, where in (("bias0", "Y0"), ("bias1", "logits"), ("transpose", "dY0"), ("gate", "dW0")):
        with pytest.raises(AssertionError, match=where):
            chain_check.compare(csr, "gcn", X, Ws, bs, dlogits, R,
                                fp32_chain(As, X, Ws, bs, dlogits, R["Y0"], mistake), slab)
