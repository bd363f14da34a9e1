"""GPU parity of the ID map (paper Section 2.2; Section 4.3, Algorithm 2) against the CPU oracle,
through the C ABI.  Integer work: the ordered mode is compared bit for bit; the fused mode (local
IDs handed out in the order threads claim slots) is compared in what is unique - the number and set
of distinct IDs, destination i keeping local ID i - and checked to be a valid bijection."""
import numpy as np
import pytest
import torch

import blockgen as bg
import oracle
from paper_2409_14939_amd import binding as B

pytestmark = pytest.mark.gpu


def run(dst, nbr, mode):
    d = torch.from_numpy(np.ascontiguousarray(dst, dtype=np.int64)).cuda()
    n = torch.from_numpy(np.ascontiguousarray(nbr, dtype=np.int64)).cuda()
    local, uniq, res = B.fastgl_idmap(d, n, mode)
    torch.cuda.synchronize()
    U, bad = (int(x) for x in res.cpu().numpy())
    return local.cpu().numpy(), uniq.cpu().numpy()[:max(U, 0)], U, bad


def check(dst, nbr, what):
    dst, nbr = np.asarray(dst, np.int64), np.asarray(nbr, np.int64)
    ref_local, ref_uniq = oracle.idmap(dst, nbr)
    print(f"case {what} n_dst={dst.size} n_nbr={nbr.size} U={ref_uniq.size} ordered", flush=True)
    local, uniq, U, bad = run(dst, nbr, "ordered")
    assert bad == 0 and U == ref_uniq.size
    assert np.array_equal(uniq, ref_uniq) and np.array_equal(local, ref_local)
    print(f"case {what} fused", flush=True)
    local, uniq, U, bad = run(dst, nbr, "fused")
    assert bad == 0 and U == ref_uniq.size
    assert np.array_equal(uniq[:dst.size], dst)                          # destination i keeps local ID i
    assert np.array_equal(np.sort(uniq), np.sort(ref_uniq))              # same set, each ID once
    if nbr.size:
        assert local.min() >= 0 and local.max() < U
        assert np.array_equal(uniq[local], nbr)                          # the map inverts: a bijection


@pytest.mark.parametrize("n_dst,n_nbr,span", [
    (0, 1, 5), (1, 0, 5), (3, 17, 10), (256, 1280, 10_000), (1000, 5000, 3000), (1237, 30011, 10 ** 12),
    (5, 70_000, 50),           # few distinct IDs, every slot hammered
    (4099, 262_147, 2 ** 40),  # several scan blocks, ragged tails, almost all distinct
])
def test_idmap_random(n_dst, n_nbr, span):
    rng = np.random.default_rng(n_dst + 3 * n_nbr)
    dst = rng.choice(span, size=n_dst, replace=False) if span < 10 ** 7 else \
        np.unique(rng.integers(0, span, size=2 * n_dst + 8))[:n_dst]
    rng.shuffle(dst)
    nbr = rng.integers(0, span, size=n_nbr)
    if n_dst and n_nbr:
        k = n_nbr // 3
        nbr[rng.choice(n_nbr, k, replace=False)] = rng.choice(dst, k)    # neighbours that are destinations
    check(dst, nbr, "random")


def test_idmap_empty():
    print("case idmap empty", flush=True)
    for mode in ("ordered", "fused"):
        local, uniq, U, bad = run([], [], mode)
        assert U == 0 and bad == 0 and local.size == 0


def test_idmap_sampled_hop_chain():
    """The hops of the tiny sampled workload, with scrambled 40-bit global IDs: the ordered map
    must give back the block's own indices (the generator numbers by first appearance too)."""
    w = bg.make_config(1)
    blk = w.blocks[0]
    dst, nbr = bg.hop_global_ids(blk, 9)
    check(dst, nbr, "config1 hop")
    local, uniq, U, bad = run(dst, nbr, "ordered")
    assert U == blk.num_src and np.array_equal(local, blk.indices)


def test_idmap_full_size_hop():
    """The input-layer hop of the products-shaped workload (0.5 M destinations, 2.6 M sampled
    neighbours) in the launch shape the benchmark times."""
    w = bg.make_config(2)
    blk = w.blocks[0]
    dst, nbr = bg.hop_global_ids(blk, 2)
    check(dst, nbr, "config2 input-layer hop")


def test_idmap_violations_are_counted():
    print("case idmap violations", flush=True)
    for mode in ("ordered", "fused"):
        _, _, _, bad = run([4, 9, 4], [1, 2], mode)          # repeated destination
        assert bad > 0
        _, _, _, bad = run([4, 9], [1, -5, 2], mode)         # negative ID
        assert bad > 0
        _, _, _, bad = run([4, -1], [1], mode)               # the empty marker itself
        assert bad > 0


def test_idmap_ordered_is_reproducible():
    rng = np.random.default_rng(1)
    dst = rng.choice(10 ** 6, 2000, replace=False)
    nbr = rng.integers(0, 10 ** 6, 100_000)
    print("case idmap reproducible", flush=True)
    a = run(dst, nbr, "ordered")
    b = run(dst, nbr, "ordered")
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])


def test_idmap_random_sweep():
    """Seeded sweep: sizes around the block sizes of the counting passes, spans from heavy repeats to
    all-distinct."""
    rng = np.random.default_rng(31)
    for case in range(12):
        n_dst = int(rng.choice([0, 1, 5, 255, 256, 1023, 1024, 1025, 3000]))
        n_nbr = int(rng.choice([0, 1, 7, 1023, 1024, 1025, 2048, 5000, 20000]))
        span = int(rng.choice([max(n_dst, 1) + 3, 10 ** 4, 10 ** 7, 2 ** 45]))
        pool = np.unique(rng.integers(0, span, size=4 * (n_dst + 4)))
        rng.shuffle(pool)
        if pool.size < n_dst:
            continue
        dst = pool[:n_dst]
        nbr = rng.integers(0, span, size=n_nbr)
        check(dst, nbr, f"sweep {case}")
