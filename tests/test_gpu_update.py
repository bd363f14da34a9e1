"""GPU parity of the update phase (paper Section 2.1, Eq. 2: Y = act(H W + b) and its gradients)
against the CPU oracle, through the C ABI.

Tolerance (derived from the arithmetic, not tuned): the kernels form every product a*b of fp32
elements from bf16 pieces on the matrix cores (each element is the exact sum of three pieces; six of
the nine piece products are kept, the dropped ones are at most 2 u |a b| together, u = 2^-24) and
accumulate in fp32; the oracle sums in fp64 and rounds once.  For a chain of L fp32 accumulations
the textbook bound is |err| <= (L+2) u sum_k |a_k b_k| + u |ref|, whatever the order of the sum;
with the dropped piece products |err| <= (L+4) u sum_k |a_k b_k| + u |ref|.  L is the contracted
length (K for Y, N for dH) and the slab height for dW / db, whose slab partials are added in fp64.
That bound is checked element by element; because it is loose (it is a worst case), the
root-mean-square error is also checked against the random-walk estimate 2 u sqrt(L) s, s = the
larger of rms(ref) and rms(sum|terms|)/sqrt(L) (the size of the partial sums), which a wrong or
dropped term breaks by orders of magnitude."""
import numpy as np
import pytest
import torch

import oracle
from paper_2409_14939_amd import binding as B

pytestmark = pytest.mark.gpu
U = 2.0 ** -24


def dev(a):
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()


def check(got, ref, absprod, L, what):
    got, ref = got.astype(np.float64), ref.astype(np.float64)
    assert got.shape == ref.shape, (what, got.shape, ref.shape)
    if ref.size == 0:
        return
    err = np.abs(got - ref)
    lim = (L + 4) * U * absprod + U * np.abs(ref) + 1e-30
    bad = err > lim
    if bad.any():
        i = np.unravel_index(np.argmax(err - lim), err.shape)
        raise AssertionError(f"{what}: {bad.sum()} of {bad.size} beyond the rounding bound; worst at {i}: "
                             f"got {got[i]!r} ref {ref[i]!r} bound {lim[i]!r}")
    # random-walk estimate: the partial sums of a chain of L terms are of the size of the result, or,
    # where the result cancels, of sum|terms| / sqrt(L)
    scale = max(np.sqrt(np.mean(ref ** 2)), np.sqrt(np.mean(np.broadcast_to(absprod, ref.shape) ** 2)) / np.sqrt(max(L, 1)))
    rms_err = np.sqrt(np.mean(err ** 2))
    assert rms_err <= 2 * U * np.sqrt(max(L, 1)) * scale + 1e-30, (what, rms_err, scale)


def run_case(M, K, N, relu, bias, seed, what):
    rng = np.random.default_rng(seed)
    H = rng.standard_normal((M, K)).astype(np.float32)
    W = (rng.standard_normal((K, N)) / np.sqrt(max(K, 1))).astype(np.float32)
    b = rng.standard_normal(N).astype(np.float32) if bias else None
    dY = rng.standard_normal((M, N)).astype(np.float32)
    print(f"case {what} M={M} K={K} N={N} relu={relu} bias={bias}", flush=True)
    Hd, Wd = dev(H), dev(W)
    Yd = B.fastgl_update_fwd(Hd, Wd, dev(b), relu)
    dHd, dWd, dbd = B.fastgl_update_bwd(Hd, Wd, Yd if relu else None, dev(dY), relu)
    torch.cuda.synchronize()
    Y = Yd.cpu().numpy()

    aH, aW = np.abs(H).astype(np.float64), np.abs(W).astype(np.float64)
    Yref = oracle.update_fwd(H, W, b, relu)
    check(Y, Yref, aH @ aW + (0 if b is None else np.abs(b)), K + 1, what + " Y")
    # The backward pass is gated by the forward OUTPUT.  Both sides get the oracle's Y where the two
    # forward results disagree about the sign of an element (possible only within the rounding bound
    # of zero); otherwise each side uses its own.
    if relu:
        flips = (Y > 0) != (Yref > 0)
        assert flips.sum() <= 1e-4 * Y.size + 2, flips.sum()
        if flips.any():
            dHd, dWd, dbd = B.fastgl_update_bwd(Hd, Wd, dev(Yref), dev(dY), relu)
            torch.cuda.synchronize()
    dHr, dWr, dbr = oracle.update_bwd(H, W, Yref if relu else None, dY, relu)
    dZ = np.abs(dY).astype(np.float64) * ((Yref > 0) if relu else 1.0)
    slab = B.fastgl_update_slab_rows(M, K, N)
    check(dHd.cpu().numpy(), dHr, dZ @ aW.T, N, what + " dH")
    check(dWd.cpu().numpy(), dWr, aH.T @ dZ, min(M, slab), what + " dW")
    check(dbd.cpu().numpy(), dbr, dZ.sum(axis=0), min(M, slab), what + " db")


@pytest.mark.parametrize("relu", [False, True])
@pytest.mark.parametrize("M,K,N", [
    (300, 100, 256),      # the input layer's widths, ragged row tail
    (1500, 256, 256),     # two slabs, three row tiles
    (2500, 256, 47),      # class scores: N not a multiple of 4 (scalar loads), three slabs
    (257, 17, 130),       # nothing aligned
    (129, 1, 1), (1, 40, 5), (64, 8, 128), (1024, 32, 32), (1025, 36, 260),
])
def test_update_parity(M, K, N, relu):
    run_case(M, K, N, relu, bias=(N % 2 == 0), seed=M + 7 * K + 13 * N, what="update")


def test_update_single_products_of_awkward_elements():
    """K = 1: every result is one product, so the error of a product formed from bf16 pieces shows
    undiluted: at most 2 u |a b| from the dropped piece products plus the final rounding.  Elements
    with all mantissa bits set, just above a power of two, with the two low bytes set, and spread
    over 60 binades (the pieces of one element then differ by up to 2^-16 in size)."""
    rng = np.random.default_rng(77)
    bits = np.array([0x3FFFFFFF, 0x3F800001, 0x3F80FFFF, 0x3F7FFFFF, 0x3FFF0001, 0x3F808080, 0x3FAAAAAA,
                     0x3FD55555], np.uint32)
    M, N = 300, 136
    H = bits[rng.integers(0, len(bits), (M, 1))].view(np.float32) * np.exp2(rng.integers(-30, 30, (M, 1))).astype(np.float32)
    H *= rng.choice([-1.0, 1.0], (M, 1)).astype(np.float32)
    W = bits[rng.integers(0, len(bits), (1, N))].view(np.float32) * np.exp2(rng.integers(-30, 30, (1, N))).astype(np.float32)
    print("case update single products", flush=True)
    Y = B.fastgl_update_fwd(dev(H), dev(W), None, False)
    torch.cuda.synchronize()
    ref = H.astype(np.float64) @ W.astype(np.float64)
    err = np.abs(Y.cpu().numpy().astype(np.float64) - ref)
    assert (err <= 3 * U * np.abs(ref)).all(), (err / np.abs(ref)).max() / U
    # random elements: same bound, and on average well inside it
    H = rng.standard_normal((M, 1)).astype(np.float32)
    W = rng.standard_normal((1, N)).astype(np.float32)
    Y = B.fastgl_update_fwd(dev(H), dev(W), None, False)
    torch.cuda.synchronize()
    ref = H.astype(np.float64) @ W.astype(np.float64)
    err = np.abs(Y.cpu().numpy().astype(np.float64) - ref)
    assert (err <= 3 * U * np.abs(ref)).all(), (err / np.abs(ref)).max() / U
    assert (err / np.abs(ref)).mean() <= U


def test_update_long_extents():
    """Extents far from the benchmark's: a very wide result (32 768 column tiles, a leading dimension of
    2^22 elements in the 32-bit lane offsets) and a very long contracted range (262 144 steps in one
    workgroup; 4 096 slabs for dW)."""
    run_case(3, 5, 1 << 22, True, bias=True, seed=901, what="wide N")
    run_case(2, 1 << 22, 3, False, bias=False, seed=902, what="long K")
    run_case((1 << 22) + 3, 2, 3, True, bias=True, seed=903, what="tall M")


def test_update_degenerate():
    # K = 0: Y = act(b); M = 0: gradients of the weights are zero; N = 0: dH is zero
    b = np.array([-1.0, 2.0, 0.5], np.float32)
    H0 = torch.empty((5, 0), dtype=torch.float32, device="cuda")
    W0 = torch.empty((0, 3), dtype=torch.float32, device="cuda")
    print("case update degenerate K=0", flush=True)
    Y = B.fastgl_update_fwd(H0, W0, dev(b), True)
    torch.cuda.synchronize()
    assert np.array_equal(Y.cpu().numpy(), np.tile(np.maximum(b, 0), (5, 1)))
    dY = np.arange(15, dtype=np.float32).reshape(5, 3)
    dH, dW, db = B.fastgl_update_bwd(H0, W0, Y, dev(dY), True)
    torch.cuda.synchronize()
    assert dH.shape == (5, 0) and dW.shape == (0, 3)
    assert np.array_equal(db.cpu().numpy(), np.array([0, dY[:, 1].sum(), dY[:, 2].sum()], np.float32))
    print("case update degenerate M=0", flush=True)
    He = torch.empty((0, 4), dtype=torch.float32, device="cuda")
    Wd = dev(np.ones((4, 3), np.float32))
    Ye = B.fastgl_update_fwd(He, Wd, None, False)
    dH, dW, db = B.fastgl_update_bwd(He, Wd, None, torch.empty((0, 3), dtype=torch.float32, device="cuda"), False)
    torch.cuda.synchronize()
    assert Ye.shape == (0, 3) and not dW.cpu().numpy().any() and not db.cpu().numpy().any()
    print("case update degenerate N=0", flush=True)
    Hn = dev(np.ones((6, 4), np.float32))
    Wn = torch.empty((4, 0), dtype=torch.float32, device="cuda")
    dH, dW, db = B.fastgl_update_bwd(Hn, Wn, None, torch.empty((6, 0), dtype=torch.float32, device="cuda"), False)
    torch.cuda.synchronize()
    assert dH.shape == (6, 4) and not dH.cpu().numpy().any()


def test_update_partial_requests_and_determinism():
    rng = np.random.default_rng(3)
    M, K, N = 2100, 100, 256
    H, W = dev(rng.standard_normal((M, K))), dev(rng.standard_normal((K, N)) / 10)
    dY = dev(rng.standard_normal((M, N)))
    print("case update partial requests", flush=True)
    Y = B.fastgl_update_fwd(H, W, None, True)
    full = B.fastgl_update_bwd(H, W, Y, dY, True)
    only_h = B.fastgl_update_bwd(H, W, Y, dY, True, want=("dH",))
    only_w = B.fastgl_update_bwd(H, W, Y, dY, True, want=("dW",))
    only_b = B.fastgl_update_bwd(H, W, Y, dY, True, want=("db",))
    again = B.fastgl_update_bwd(H, W, Y, dY, True)
    torch.cuda.synchronize()
    assert only_h[1] is None and only_h[2] is None and only_w[0] is None and only_b[1] is None
    assert torch.equal(full[0], only_h[0]) and torch.equal(full[1], only_w[1]) and torch.equal(full[2], only_b[2])
    for a, b in zip(full, again):          # fixed slabs, fixed order: bit-identical from run to run
        assert torch.equal(a, b)


def test_update_full_size_sampled():
    """The products-shaped input layer (M = 512 345 rows, 100 -> 256) in the launch shape the
    benchmark times; the oracle computes sampled rows of Y and dH and sampled columns of dW, db."""
    rng = np.random.default_rng(11)
    M, K, N = 512345, 100, 256
    H = rng.standard_normal((M, K), dtype=np.float32)
    W = (rng.standard_normal((K, N)) / 10).astype(np.float32)
    b = rng.standard_normal(N).astype(np.float32)
    dY = rng.standard_normal((M, N), dtype=np.float32)
    print(f"case update full size M={M} K={K} N={N}", flush=True)
    Hd, Wd, dYd = dev(H), dev(W), dev(dY)
    Yd = B.fastgl_update_fwd(Hd, Wd, dev(b), True)
    dHd, dWd, dbd = B.fastgl_update_bwd(Hd, Wd, Yd, dYd, True)
    torch.cuda.synchronize()
    rows = np.unique(np.concatenate([rng.integers(0, M, 600), [0, 127, 128, M - 2, M - 1]]))
    aW = np.abs(W).astype(np.float64)
    Y = Yd.cpu().numpy()
    Yref = oracle.update_fwd(H[rows], W, b, True)
    check(Y[rows], Yref, np.abs(H[rows]).astype(np.float64) @ aW + np.abs(b), K + 1, "full Y")
    Ygate = Y[rows]                        # gate the oracle with the GPU's own forward output
    dHr, _, _ = oracle.update_bwd(H[rows], W, Ygate, dY[rows], True, want=("dH",))
    dZ = np.abs(dY[rows]).astype(np.float64) * (Ygate > 0)
    check(dHd.cpu().numpy()[rows], dHr, dZ @ aW.T, N, "full dH")
    cols = np.array([0, 1, 63, 64, 127, 128, 200, 255])
    Yc, dYc = np.ascontiguousarray(Y[:, cols]), np.ascontiguousarray(dY[:, cols])
    _, dWr, dbr = oracle.update_bwd(H, np.ascontiguousarray(W[:, cols]), Yc, dYc, True, want=("dW", "db"))
    dZc = np.abs(dYc).astype(np.float64) * (Yc > 0)
    slab = B.fastgl_update_slab_rows(M, K, N)
    check(dWd.cpu().numpy()[:, cols], dWr, np.abs(H).astype(np.float64).T @ dZc, slab, "full dW")
    check(dbd.cpu().numpy()[cols], dbr, dZc.sum(axis=0), slab, "full db")


def test_gcn_layers_chain_against_oracle():
    """Two sampled GCN layers end to end - aggregate (Eq. 1), update (Eq. 2), ReLU, and the whole
    backward pass - as the benchmark's extra leg chains them, against the same chain of oracle
    calls.  The GPU feeds its own intermediate results forward; every link's output is compared
    element by element within its own tolerance plus the earlier links' bounds pushed through it
    (chain_check.py).  The backward pass through the ReLU is gated by the oracle's forward output."""
    import blockgen as bg
    import chain_check
    from gpu_util import dev_i32
    rng = np.random.default_rng(77)
    b0 = bg.random_block(rng, 700, 1500, 5.0, empty_frac=0.05, hub_rows=2, hub_deg=400)
    b1 = bg.random_block(rng, 200, 700, 8.0, empty_frac=0.05, hub_rows=1, hub_deg=300)
    widths, outs = [100, 256], [256, 47]
    X = bg.features_f32(rng, b0.num_src, widths[0])
    Ws = [(rng.standard_normal((k, n)) / np.sqrt(k)).astype(np.float32) for k, n in zip(widths, outs)]
    bs = [(0.1 * rng.standard_normal(n)).astype(np.float32) for n in outs]
    dlogits = rng.standard_normal((b1.num_dst, outs[1])).astype(np.float32)
    blocks, mode = [b0, b1], "gcn"
    print("case gcn chain: 2 layers, gcn mode", flush=True)
    csr = [(b.indptr, b.indices, b.num_src) for b in blocks]
    R = chain_check.oracle_chain(csr, mode, X, Ws, bs, dlogits)

    # HIP chain
    ips, ixs = [dev_i32(b.indptr) for b in blocks], [dev_i32(b.indices) for b in blocks]
    plans = B.fastgl_block_plan_create_many([(ips[i], ixs[i], blocks[i].num_src) for i in range(2)])
    xd, G = dev(X), {}
    for i, relu in enumerate([True, False]):
        G[f"H{i}"] = B.fastgl_block_aggregate_fwd(ips[i], ixs[i], None, blocks[i].num_src, mode, xd, plan=plans[i])
        G[f"Y{i}"] = xd = B.fastgl_update_fwd(G[f"H{i}"], dev(Ws[i]), dev(bs[i]), relu)
    G["dH1"], G["dW1"], G["db1"] = B.fastgl_update_bwd(G["H1"], dev(Ws[1]), None, dev(dlogits), False)
    G["dY0"] = B.fastgl_block_aggregate_bwd(ips[1], ixs[1], None, blocks[1].num_src, mode, G["dH1"], plan=plans[1])
    _, G["dW0"], G["db0"] = B.fastgl_update_bwd(G["H0"], dev(Ws[0]), dev(R["Y0"]), G["dY0"], True, want=("dW", "db"))
    torch.cuda.synchronize()
    chain_check.compare(csr, mode, X, Ws, bs, dlogits, R, {k: v.cpu().numpy() for k, v in G.items()},
                        B.fastgl_update_slab_rows)


def test_update_random_shape_sweep():
    """Seeded sweep over shapes that mix every edge path of the tiled kernel: contracted lengths
    around the stage size, rows and columns around the tile size, extents that are and are not
    multiples of 4 (16-byte or scalar loads), with and without the ReLU gate."""
    rng = np.random.default_rng(2024)
    picks_m = [1, 2, 63, 64, 65, 127, 128, 129, 255, 257, 1023, 1025, 2050]
    picks_k = [1, 2, 3, 4, 7, 8, 9, 15, 16, 17, 31, 33, 64, 100, 130]
    picks_n = [1, 2, 4, 5, 8, 31, 32, 33, 64, 127, 128, 129, 132, 200, 256]
    for case in range(24):
        M, K, N = int(rng.choice(picks_m)), int(rng.choice(picks_k)), int(rng.choice(picks_n))
        run_case(M, K, N, relu=bool(case % 2), bias=bool((case // 2) % 2), seed=9000 + case, what=f"sweep {case}")


# ---- bf16 storage ------------------------------------------------------------------------
def dev_bf16(bits):
    return torch.from_numpy(np.ascontiguousarray(bits, dtype=np.uint16).view(np.int16)).cuda().view(torch.bfloat16)


def host_bf16(t):
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


def close_bf16(got_bits, ref_bits, absprod, L, what):
    """bf16 results: the kernel sums in fp32 and rounds fp32 -> bf16, the oracle rounds the fp64 sum
    once: they agree up to one bf16 unit (2^-8 relative, the task's 2e-2 with room to spare) plus the
    fp32 accumulation bound where the sum cancels."""
    import blockgen as bg
    got, ref = bg.bf16_bits_to_f32(got_bits).astype(np.float64), bg.bf16_bits_to_f32(ref_bits).astype(np.float64)
    assert got.shape == ref.shape, (what, got.shape, ref.shape)
    lim = 2.0 ** -7 * np.abs(ref) + (L + 2) * U * absprod + 1e-30
    bad = np.abs(got - ref) > lim
    assert not bad.any(), (what, int(bad.sum()), got[bad][:3], ref[bad][:3])
    assert (got_bits == ref_bits).mean() > 0.97, (what, (got_bits == ref_bits).mean())     # almost always the same bits


@pytest.mark.parametrize("relu", [False, True])
@pytest.mark.parametrize("M,K,N", [(300, 128, 256), (1500, 256, 256), (2500, 256, 47), (257, 18, 130), (1, 40, 5),
                                   (1025, 36, 260)])
def test_update_parity_bf16(M, K, N, relu):
    import blockgen as bg
    rng = np.random.default_rng(M + K + N)
    Hb = bg.to_bf16_bits(rng.standard_normal((M, K)).astype(np.float32))
    Wb = bg.to_bf16_bits((rng.standard_normal((K, N)) / np.sqrt(K)).astype(np.float32))
    b = rng.standard_normal(N).astype(np.float32) if N % 2 == 0 else None
    dYb = bg.to_bf16_bits(rng.standard_normal((M, N)).astype(np.float32))
    print(f"case update bf16 M={M} K={K} N={N} relu={relu}", flush=True)
    Hd, Wd = dev_bf16(Hb), dev_bf16(Wb)
    Yd = B.fastgl_update_fwd(Hd, Wd, dev(b), relu)
    torch.cuda.synchronize()
    Yref = oracle.update_fwd_bf16(Hb, Wb, b, relu)
    aH, aW = np.abs(bg.bf16_bits_to_f32(Hb)).astype(np.float64), np.abs(bg.bf16_bits_to_f32(Wb)).astype(np.float64)
    close_bf16(host_bf16(Yd), Yref, aH @ aW + (0 if b is None else np.abs(b)), K + 1, "Y")
    # gate both backward passes with the oracle's forward output (a last-bit difference may flip a sign at 0)
    dHd, dWd, dbd = B.fastgl_update_bwd(Hd, Wd, dev_bf16(Yref) if relu else None, dev_bf16(dYb), relu)
    torch.cuda.synchronize()
    dHr, dWr, dbr = oracle.update_bwd_bf16(Hb, Wb, Yref if relu else None, dYb, relu)
    dZ = np.abs(bg.bf16_bits_to_f32(dYb)).astype(np.float64) * ((bg.bf16_bits_to_f32(Yref) > 0) if relu else 1.0)
    close_bf16(host_bf16(dHd), dHr, dZ @ aW.T, N, "dH")
    slab = B.fastgl_update_slab_rows(M, K, N)
    check(dWd.cpu().numpy(), dWr, aH.T @ dZ, min(M, slab), "dW (bf16 inputs)")
    check(dbd.cpu().numpy(), dbr, dZ.sum(axis=0), min(M, slab), "db (bf16 inputs)")
