"""Input generator: determinism and the structural facts the paper states
(Section 2.2: local ids consecutive from 0; each hop's destinations are the
previous hop's sources)."""
import numpy as np

import blockgen as bg


def test_same_seed_same_bytes_and_chain():
    a, b = bg.make_config(4), bg.make_config(4)
    for x, y in zip(a.blocks, b.blocks):
        assert x.indptr.tobytes() == y.indptr.tobytes() and x.indices.tobytes() == y.indices.tobytes()
    assert np.array_equal(a.src_gid, b.src_gid)
    assert bg.make_config(4, run=1).blocks[0].indices.tobytes() != a.blocks[0].indices.tobytes()
    for lo, hi in zip(a.blocks[:-1], a.blocks[1:]):
        assert lo.num_dst == hi.num_src
    assert a.blocks[-1].num_dst == 1024
    assert a.src_gid.shape[0] == a.blocks[0].num_src
    assert np.unique(a.src_gid).shape[0] == a.src_gid.shape[0]
    assert a.src_gid.min() >= 0 and a.src_gid.max() < a.table_rows


def test_config1_shape():
    w = bg.make_config(1)
    blk = w.blocks[0]
    blk.check()
    assert blk.num_dst == 256 and np.diff(blk.indptr).max() <= 5
    # every source id is referenced or is a destination (dst prefix + first-appearance numbering)
    seen = np.zeros(blk.num_src, bool)
    seen[:blk.num_dst] = True
    seen[blk.indices] = True
    assert seen.all()
    new = blk.indices[blk.indices >= blk.num_dst]
    _, first = np.unique(new, return_index=True)
    assert np.array_equal(new[np.sort(first)], np.arange(blk.num_dst, blk.num_src))


def test_fanout_caps_and_no_duplicates_config3():
    w = bg.make_config(3)
    caps = [10, 25]   # input-layer block is the last hop sampled
    for blk, cap in zip(w.blocks, caps):
        din = np.diff(blk.indptr)
        assert din.max() <= cap
        rows = np.repeat(np.arange(blk.num_dst), din)
        key = rows.astype(np.int64) * blk.num_src + blk.indices
        assert np.unique(key).shape[0] == key.shape[0]
        assert not np.any(blk.indices == rows)      # no self loops


def test_chung_lu_calibration():
    g = bg.ChungLu(1_000_000, 100.0, 1.8, 50_000.0, 1)
    r = np.arange(g.n)
    w = g.weight(r)
    assert abs(w.mean() - 100.0) < 1e-6 * 100 and abs(w[0] - 50_000.0) < 1e-3 * 50_000
    assert np.all(np.diff(w) <= 0)
    gid = g.global_id(r)
    assert np.unique(gid).shape[0] == g.n


def test_banded_copy_keeps_sizes_and_stays_near_the_diagonal():
    blk = bg.random_block(np.random.default_rng(3), 500, 1300, 4.0, empty_frac=0.2, hub_rows=2, hub_deg=300)
    band = bg.banded_like(blk, 64, 9)
    assert band.num_dst == blk.num_dst and band.num_src == blk.num_src
    assert np.array_equal(band.indptr, blk.indptr)
    rows = np.repeat(np.arange(blk.num_dst), np.diff(blk.indptr))
    centre = rows * blk.num_src // blk.num_dst
    assert (np.abs(band.indices.astype(np.int64) - centre) <= 32).all()
    assert np.array_equal(band.indices, bg.banded_like(blk, 64, 9).indices)          # same seed, same block
    assert not np.array_equal(band.indices, bg.banded_like(blk, 64, 10).indices)
