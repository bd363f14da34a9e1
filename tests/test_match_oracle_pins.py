"""Pins of the Match / Greedy-Reorder oracle (paper Section 4.1, Algorithm 1) against things other
than itself: the paper's worked example, Python sets, numpy set routines, brute-force search over
orders on tiny inputs, and invariants."""
import itertools
import os

import numpy as np
import pytest

import blockgen as bg
import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "match_reorder_example.txt")


def golden():
    d = {}
    for line in open(GOLDEN):
        if line.strip() and not line.startswith("#"):
            k, *v = line.split()
            d[k] = [int(x) for x in v]
    return d


def test_r1_paper_match_example():
    g = golden()
    mrow, lpos, lgid = oracle.match(g["subg1"], g["next"])
    assert lgid.tolist() == g["load"]
    assert [g["next"][i] for i in range(len(mrow)) if mrow[i] >= 0] == g["overlap"]
    assert [g["subg1"][r] for r in mrow if r >= 0] == g["overlap"]           # the rows point at the same nodes
    assert lpos.tolist() == [3, 4]
    assert oracle.match_degree(g["subg1"], g["next"]) == 3 / 5


def test_r2_paper_reorder_example():
    g = golden()
    # three mini-batches of 10 nodes; SubG_1 shares 2 nodes with SubG_2 and 5 with SubG_3
    s1 = list(range(0, 10))
    s2 = [0, 1] + list(range(100, 108))
    s3 = [2, 3, 4, 5, 6] + list(range(200, 205))
    O = oracle.overlap_matrix([s1, s2, s3])
    assert O[0, 2] > O[0, 1]
    order = oracle.greedy_reorder(O, [10, 10, 10])
    assert (order + 1).tolist() == g["reorder_when_m13_gt_m12"]
    # the other way round nothing moves
    assert oracle.greedy_reorder(oracle.overlap_matrix([s1, s3, s2]), [10, 10, 10]).tolist() == [0, 1, 2]


@pytest.mark.parametrize("seed", range(5))
def test_r3_match_against_python_sets(seed):
    rng = np.random.default_rng(seed)
    span = [30, 1000, 10 ** 12, 50, 5000][seed]
    n_prev, n_new = [(10, 12), (300, 200), (500, 700), (0, 5), (800, 0)][seed]
    pool = rng.choice(span, size=min(span, n_prev + n_new), replace=False) if span < 10 ** 7 else \
        np.unique(rng.integers(0, span, 2 * (n_prev + n_new)))
    rng.shuffle(pool)
    prev = pool[:n_prev]
    new = rng.permutation(np.concatenate([pool[n_prev // 2:n_prev], pool[n_prev:]])[:n_new]) if n_new else pool[:0]
    mrow, lpos, lgid = oracle.match(prev, new)
    where = {int(g): j for j, g in enumerate(prev)}
    assert mrow.tolist() == [where.get(int(g), -1) for g in new]
    assert lpos.tolist() == [i for i, g in enumerate(new) if int(g) not in where]
    assert np.array_equal(lgid, new[lpos])
    # numpy's set routines agree on the two ID sets and on N_o
    assert set(lgid.tolist()) == set(np.setdiff1d(new, prev).tolist())
    assert oracle.overlap(prev, new) == np.intersect1d(prev, new).size == int((mrow >= 0).sum())
    with pytest.raises(ValueError):
        oracle.match([1, 2, 1], [1])


def test_r4_assemble_is_a_row_selection():
    rng = np.random.default_rng(0)
    prev = rng.choice(1000, 60, replace=False)
    new = rng.permutation(np.concatenate([prev[10:40], 2000 + np.arange(25)]))
    table = {int(g): rng.standard_normal(7).astype(np.float32) for g in np.concatenate([prev, new])}
    X_prev = np.stack([table[int(g)] for g in prev])
    mrow, lpos, lgid = oracle.match(prev, new)
    X_load = np.stack([table[int(g)] for g in lgid])
    X_new = oracle.assemble(X_prev, X_load, mrow)
    assert np.array_equal(X_new, np.stack([table[int(g)] for g in new]))     # = loading every row afresh
    # 2-byte elements move the same way
    X16 = oracle.assemble(X_prev.view(np.uint16), X_load.view(np.uint16), mrow)
    assert np.array_equal(X16.view(np.float32), X_new)


def total_reuse(O, order):
    return sum(O[a, b] for a, b in zip(order[:-1], order[1:]))


@pytest.mark.parametrize("seed", range(8))
def test_r5_greedy_reorder_properties(seed):
    rng = np.random.default_rng(100 + seed)
    n = int(rng.integers(1, 8))
    sets = [rng.choice(60, size=int(rng.integers(5, 30)), replace=False) for _ in range(n)]
    sizes = [len(s) for s in sets]
    O = oracle.overlap_matrix(sets)
    assert np.array_equal(O, O.T) and np.array_equal(np.diag(O), sizes)
    order = oracle.greedy_reorder(O, sizes).tolist()
    assert sorted(order) == list(range(n)) and order[0] == 0                 # a permutation that starts with SubG_1
    M = np.array([[0 if i == j else O[i, j] / min(sizes[i], sizes[j]) for j in range(n)] for i in range(n)])
    left = set(range(1, n))
    for z, h in zip(order[:-1], order[1:]):                                  # every step takes the best that is left
        assert M[z, h] == max(M[z, k] for k in left)
        assert h == min(k for k in left if M[z, k] == M[z, h])               # ties: smallest index
        left.remove(h)


def test_r6_greedy_is_the_listing_not_the_optimum():
    # Greedy follows the best next step; an exhaustive search over orders may reuse more.  Both are
    # computed here so that the oracle cannot silently turn into something else.
    O = np.array([[9, 5, 4, 0], [5, 9, 0, 1], [4, 0, 9, 8], [0, 1, 8, 9]], np.int64)
    sizes = [9, 9, 9, 9]
    assert oracle.greedy_reorder(O, sizes).tolist() == [0, 1, 3, 2]          # 5 + 1 + 8 = 14
    best = max(([0] + list(p) for p in itertools.permutations([1, 2, 3])), key=lambda o: total_reuse(O, o))
    assert total_reuse(O, best) >= total_reuse(O, [0, 1, 3, 2])


def test_r7_sampled_minibatches_overlap_and_reorder_helps():
    sets = bg.minibatch_node_sets(6, 3, n=200_000, avg=20.0, n_seeds=500, fanouts=(10, 5))
    assert all(np.unique(s).size == s.size for s in sets)
    O = oracle.overlap_matrix(sets)
    degrees = [oracle.match_degree(sets[i], sets[j]) for i in range(6) for j in range(i)]
    assert 0.1 < min(degrees) <= max(degrees) < 0.9                          # hubs are shared, the rest is not
    order = oracle.greedy_reorder(O, [len(s) for s in sets]).tolist()
    assert total_reuse(O, order) >= total_reuse(O, list(range(6))) - 0       # never worse on this instance
    # loading with Match moves exactly the non-overlapping rows
    for a, b in zip(order[:-1], order[1:]):
        mrow, lpos, lgid = oracle.match(sets[a], sets[b])
        assert lpos.size == len(sets[b]) - O[a, b]
