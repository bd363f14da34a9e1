"""GPU parity of the Match process, the row assembly and the pairwise overlap counts (paper Section
4.1) against the CPU oracle, through the C ABI.  Integer and byte work: everything is compared bit
for bit."""
import numpy as np
import pytest
import torch

import blockgen as bg
import oracle
from paper_2409_14939_amd import binding as B

pytestmark = pytest.mark.gpu


def dev64(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int64)).cuda()


def run_match(prev, new):
    src_row, load_pos, load_gid, res = B.fastgl_match(dev64(prev), dev64(new))
    torch.cuda.synchronize()
    n_load, bad = (int(x) for x in res.cpu().numpy())
    return src_row.cpu().numpy(), load_pos.cpu().numpy()[:max(n_load, 0)], load_gid.cpu().numpy()[:max(n_load, 0)], \
        n_load, bad


def check_match(prev, new, what):
    prev, new = np.asarray(prev, np.int64), np.asarray(new, np.int64)
    print(f"case {what} n_prev={prev.size} n_new={new.size}", flush=True)
    mrow, lpos, lgid = oracle.match(prev, new)
    src_row, load_pos, load_gid, n_load, bad = run_match(prev, new)
    assert bad == 0 and n_load == lpos.size
    assert np.array_equal(load_pos, lpos) and np.array_equal(load_gid, lgid)
    expect = mrow.copy()
    expect[lpos] = -1 - np.arange(lpos.size, dtype=np.int32)        # misses carry their place in the load lists
    assert np.array_equal(src_row, expect)
    return src_row, n_load


def two_sets(rng, n_prev, n_new, shared, span):
    pool = np.unique(rng.integers(0, span, size=3 * (n_prev + n_new) + 16))
    rng.shuffle(pool)
    assert pool.size >= n_prev + n_new
    prev = pool[:n_prev]
    k = min(shared, n_prev, n_new)
    new = rng.permutation(np.concatenate([rng.choice(prev, k, replace=False) if k else pool[:0],
                                          pool[n_prev:n_prev + n_new - k]]))
    return prev, new


@pytest.mark.parametrize("n_prev,n_new,shared,span", [
    (0, 7, 0, 100), (9, 0, 0, 100), (5, 5, 5, 10 ** 6), (5, 5, 0, 10 ** 6), (300, 200, 120, 10 ** 4),
    (1025, 4099, 700, 10 ** 12), (70_001, 65_537, 40_000, 2 ** 40),
])
def test_match_random(n_prev, n_new, shared, span):
    rng = np.random.default_rng(n_prev + 7 * n_new)
    prev, new = two_sets(rng, n_prev, n_new, shared, span)
    check_match(prev, new, "random")


@pytest.mark.parametrize("dtype,feat", [("f32", 100), ("f32", 7), ("bf16", 128), ("bf16", 3), ("f32", 256)])
def test_assemble_rows(dtype, feat):
    rng = np.random.default_rng(feat)
    prev, new = two_sets(rng, 1500, 2100, 900, 10 ** 9)
    src_row, n_load = check_match(prev, new, f"assemble {dtype} F={feat}")
    npdt = np.float32 if dtype == "f32" else np.uint16
    def rows(n):
        return (rng.standard_normal((n, feat)).astype(np.float32) if dtype == "f32"
                else rng.integers(0, 2 ** 16, size=(n, feat)).astype(np.uint16))
    X_prev, X_load = rows(prev.size), rows(n_load)
    mrow, _, _ = oracle.match(prev, new)
    ref = oracle.assemble(X_prev, X_load, mrow)
    def to_dev(a):
        t = torch.from_numpy(a.view(np.int16) if dtype == "bf16" else a).cuda()
        return t.view(torch.bfloat16) if dtype == "bf16" else t
    # the load buffer may be larger than what is loaded (sized for the worst case)
    Xl = to_dev(np.concatenate([X_load, rows(5)]))
    out = B.fastgl_assemble_rows(to_dev(X_prev), Xl, torch.from_numpy(src_row).cuda(), n_load)
    torch.cuda.synchronize()
    got = out.view(torch.int16).cpu().numpy().view(np.uint16) if dtype == "bf16" else out.cpu().numpy()
    assert got.dtype == npdt and np.array_equal(got, ref)


def test_match_violations_are_counted():
    print("case match violations", flush=True)
    assert run_match([4, 9, 4], [1, 2])[4] > 0          # the last mini-batch repeats an ID
    assert run_match([4, 9], [1, -5])[4] > 0            # negative ID
    assert run_match([4, -1], [1])[4] > 0


def test_overlap_counts_and_reorder_on_sampled_minibatches():
    sets = bg.minibatch_node_sets(7, 5, n=300_000, avg=20.0, n_seeds=600, fanouts=(10, 5))
    sizes = [len(s) for s in sets]
    offsets = np.concatenate([[0], np.cumsum(sizes)])
    print(f"case overlap counts of {len(sets)} sampled mini-batches, sizes {sizes}", flush=True)
    counts, viol = B.fastgl_overlap_counts(dev64(np.concatenate(sets)), offsets.tolist())
    torch.cuda.synchronize()
    assert int(viol.cpu()[0]) == 0
    O = oracle.overlap_matrix(sets)
    assert np.array_equal(counts.cpu().numpy(), O)
    assert B.fastgl_greedy_reorder(counts.cpu().numpy().tolist(), sizes) == oracle.greedy_reorder(O, sizes).tolist()
    # degenerate shapes
    c, v = B.fastgl_overlap_counts(dev64([]), [0])
    torch.cuda.synchronize()
    assert c.shape == (0, 0) and int(v.cpu()[0]) == 0
    c, v = B.fastgl_overlap_counts(dev64([3, 4, 3]), [0, 0, 2, 3])          # an empty mini-batch, two that share 3
    torch.cuda.synchronize()
    assert c.cpu().numpy().tolist() == [[0, 0, 0], [0, 2, 1], [0, 1, 1]] and int(v.cpu()[0]) == 0
    c, v = B.fastgl_overlap_counts(dev64([3, 3]), [0, 2])                   # a mini-batch that repeats an ID
    torch.cuda.synchronize()
    assert int(v.cpu()[0]) > 0


def test_match_full_size_minibatches():
    """Two mini-batches of the products-shaped workload (1.15 M nodes each) in the launch shape the
    benchmark times."""
    a, b = bg.minibatch_node_sets(2, 2000)
    check_match(a, b, "config2 mini-batches")
