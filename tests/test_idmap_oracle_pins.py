"""Pins of the ID-map oracle (paper Section 2.2 "ID map", Section 4.3 Algorithm 2) against things
other than itself: the paper's worked example, brute force with a Python dict, Algorithm 2 run
sequentially against the sort-based definition, numpy's unique, hand-worked probe chains, the
bijection invariants, and the block generator's own relabelling."""
import os

import numpy as np
import pytest

import blockgen as bg
import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "fused_map_example.txt")


def dict_idmap(dst, nbr):
    """Brute force in another language: a dict filled in list order."""
    seen, uniq = {}, []
    for g in list(dst) + list(nbr):
        if int(g) not in seen:
            seen[int(g)] = len(uniq)
            uniq.append(int(g))
    return np.array([seen[int(g)] for g in nbr], np.int32), np.array(uniq, np.int64)


def test_m1_paper_worked_example():
    rows = [l.split() for l in open(GOLDEN) if l.strip() and not l.startswith("#")]
    ids = []
    for step, gid, slot, local, counter in rows:
        ids.append(int(gid))
        key, value, loc, U = oracle.fused_map_sequential(ids, 5)
        assert key[int(slot)] == int(gid) and value[int(slot)] == int(local), step
        assert U == int(counter) and loc[-1] == int(local), step
        assert (key == -1).sum() == 5 - U            # nothing else was touched


def test_m2_hand_worked_probe_chains():
    # 3, 8, 13 all hash to slot 3 of 5: 3 stays, 8 probes to 4, 13 wraps to 0; 4 then finds 4 and 0
    # taken and lands in 1.  Worked by hand.
    key, value, local, U = oracle.fused_map_sequential([3, 3, 8, 13, 4, 8], 5)
    assert key.tolist() == [13, 4, -1, 3, 8] and value.tolist() == [2, 3, 0, 0, 1]
    assert local.tolist() == [0, 0, 1, 2, 3, 1] and U == 4
    # a full table still maps every ID; one more distinct ID cannot be placed
    key, value, local, U = oracle.fused_map_sequential([7, 2, 12, 17, 22], 5)
    assert U == 5 and sorted(key.tolist()) == [2, 7, 12, 17, 22] and local.tolist() == [0, 1, 2, 3, 4]
    with pytest.raises(RuntimeError):
        oracle.fused_map_sequential([7, 2, 12, 17, 22, 27], 5)
    # negative IDs other than the empty marker hash by the mathematical remainder
    key, _, local, U = oracle.fused_map_sequential([-7, -2, -7], 5)
    assert key[3] == -7 and key[4] == -2 and local.tolist() == [0, 1, 0] and U == 2


def test_m3_definition_small_by_hand():
    local, uniq = oracle.idmap([10, 20], [20, 30, 10, 30, 40])
    assert local.tolist() == [1, 2, 0, 2, 3] and uniq.tolist() == [10, 20, 30, 40]
    local, uniq = oracle.idmap([], [5, 5, 4])
    assert local.tolist() == [0, 0, 1] and uniq.tolist() == [5, 4]
    local, uniq = oracle.idmap([9, 8], [])
    assert local.size == 0 and uniq.tolist() == [9, 8]
    local, uniq = oracle.idmap([], [])
    assert local.size == 0 and uniq.size == 0
    with pytest.raises(ValueError):
        oracle.idmap([4, 4], [1])


@pytest.mark.parametrize("seed", range(6))
def test_m4_brute_force_and_algorithm2(seed):
    rng = np.random.default_rng(seed)
    n_dst, n_nbr, span = [(0, 50, 20), (7, 0, 100), (13, 200, 60), (64, 1000, 300), (1, 1, 2), (100, 5000, 10 ** 12)][seed]
    dst = rng.choice(span, size=n_dst, replace=False).astype(np.int64) if n_dst else np.zeros(0, np.int64)
    nbr = rng.integers(0, span, size=n_nbr).astype(np.int64)
    local, uniq = oracle.idmap(dst, nbr)
    bl, bu = dict_idmap(dst, nbr)
    assert np.array_equal(local, bl) and np.array_equal(uniq, bu)
    # Algorithm 2 in one thread numbers nodes in processing order = first appearance
    ids = np.concatenate([dst, nbr])
    for table in (len(ids) + 1, 2 * len(ids) + 3, 4096):
        if table < len(np.unique(ids)):
            continue
        key, value, loc, U = oracle.fused_map_sequential(ids, table)
        assert U == uniq.size
        assert np.array_equal(loc[n_dst:], local) and np.array_equal(loc[:n_dst], np.arange(n_dst))
        filled = key != -1
        assert filled.sum() == U and sorted(key[filled].tolist()) == sorted(uniq.tolist())
        assert np.array_equal(uniq[value[filled]], key[filled])      # value is the local ID of its key


def test_m5_numpy_unique_and_invariants():
    rng = np.random.default_rng(42)
    dst = rng.choice(10 ** 6, size=500, replace=False).astype(np.int64)
    nbr = np.concatenate([rng.integers(0, 10 ** 6, size=20000), rng.choice(dst, 3000)]).astype(np.int64)
    rng.shuffle(nbr)
    local, uniq = oracle.idmap(dst, nbr)
    ids = np.concatenate([dst, nbr])
    u, first = np.unique(ids, return_index=True)
    assert uniq.size == u.size and np.array_equal(np.sort(uniq), u)
    assert np.array_equal(uniq, ids[np.sort(first)])                 # ordered by first position
    assert np.array_equal(uniq[:500], dst)                           # destinations are a prefix
    assert np.array_equal(uniq[local], nbr)                          # the map inverts
    assert local.min() >= 0 and local.max() == uniq.size - 1


def test_m6_block_generator_relabelling_agrees():
    # the input generator numbers nodes the same way (its blocks are what the aggregation tests use)
    w = bg.make_config(1)
    rng = np.random.default_rng(3)
    dst = rng.choice(10 ** 5, size=300, replace=False).astype(np.int64)
    rows = np.sort(rng.integers(0, 300, size=2000))
    nbr = rng.integers(0, 10 ** 5, size=2000).astype(np.int64)
    blk, src_ids = bg._relabel(dst, rows, nbr)
    local, uniq = oracle.idmap(dst, nbr)
    assert np.array_equal(blk.indices, local) and np.array_equal(src_ids, uniq) and blk.num_src == uniq.size
    assert w.blocks[0].num_dst == 256
