"""Seeded synthetic mini-batch blocks shaped like the paper's workloads.

This module only *makes inputs*: bipartite sampled blocks in CSR-by-destination
form, random feature / gradient matrices and sampled global IDs. It holds none
of the aggregation arithmetic, so both the CPU oracle's tests and the GPU
path's tests may draw the same bytes from it.

Block shape follows the paper's description of sampling-based training
(Section 2.2, "Sampling-based GNN Training"): starting from the seed nodes of
a mini-batch, every hop samples up to `fanout` neighbours of each destination
node uniformly without replacement, and global node IDs are mapped to local
IDs that are consecutive and start from 0.  The datasets of the paper's
Table 6 are not available, so the graphs are random models that take only
their node count, average degree and heavy-tailed degree shape.

Local ID convention (deterministic stand-in for the paper's atomic ID map):
destination nodes keep local IDs 0..num_dst-1 (they are a prefix of the source
nodes), and every other source node gets the next free ID in order of first
appearance when the edges are scanned row by row.
"""
from __future__ import annotations

import dataclasses
import math
from typing import List, Optional, Sequence

import numpy as np

__all__ = [
    "Block", "Workload", "ChungLu", "make_config", "CONFIG_NAMES",
    "random_block", "features_f32", "to_bf16_bits", "bf16_bits_to_f32",
    "hash_u01",
]


# ----------------------------------------------------------------------------
# containers
# ----------------------------------------------------------------------------
@dataclasses.dataclass
class Block:
    """One layer's bipartite block, CSR by destination row."""
    indptr: np.ndarray   # int32 [num_dst+1]
    indices: np.ndarray  # int32 [E], local source ids in [0, num_src)
    num_dst: int
    num_src: int

    @property
    def num_edges(self) -> int:
        return int(self.indices.shape[0])

    def check(self) -> None:
        assert self.indptr.dtype == np.int32 and self.indices.dtype == np.int32
        assert self.indptr.shape == (self.num_dst + 1,)
        assert self.indptr[0] == 0 and self.indptr[-1] == self.num_edges
        assert np.all(np.diff(self.indptr) >= 0)
        if self.num_edges:
            assert self.indices.min() >= 0 and self.indices.max() < self.num_src


@dataclasses.dataclass
class Workload:
    """A sampled multi-layer mini-batch: blocks[0] is the input-layer block
    (it reads raw features), blocks[-1] is the block whose destinations are
    the seed nodes."""
    name: str
    blocks: List[Block]
    widths: List[int]            # feature width each layer aggregates at
    mode: str                    # "sum" | "mean" | "gcn"
    dtype: str                   # "f32" | "bf16"
    seed: int
    src_gid: Optional[np.ndarray] = None   # int64 [blocks[0].num_src], config 4
    table_rows: int = 0                    # rows of the device feature table

    def total_edges(self) -> int:
        return sum(b.num_edges for b in self.blocks)


# ----------------------------------------------------------------------------
# small counter-based hash -> uniform(0,1), used for per-node degrees so that a
# node's degree does not depend on which hop asks for it
# ----------------------------------------------------------------------------
def _splitmix64(x: np.ndarray) -> np.ndarray:
    x = x.astype(np.uint64, copy=True)
    with np.errstate(over="ignore"):
        x += np.uint64(0x9E3779B97F4A7C15)
        x = (x ^ (x >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
        x = (x ^ (x >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
        x = x ^ (x >> np.uint64(31))
    return x


def hash_u01(ids: np.ndarray, seed: int) -> np.ndarray:
    """Deterministic uniform(0,1) per integer id."""
    with np.errstate(over="ignore"):
        h = _splitmix64(np.asarray(ids, dtype=np.uint64)
                        ^ (np.uint64(seed & 0xFFFFFFFF) << np.uint64(32)))
    return (h >> np.uint64(11)).astype(np.float64) * (1.0 / (1 << 53))


# ----------------------------------------------------------------------------
# implicit Chung-Lu power-law graph
# ----------------------------------------------------------------------------
class ChungLu:
    """Power-law random graph that is never materialised.

    Node "ranks" i = 0..N-1 carry expected degree
        w_i = c * integral_i^{i+1} (t + i0)^(-alpha) dt,   alpha = 1/(gamma-1),
    with (c, i0) solved so that mean(w) = avg_degree and w_0 = w_max.
    A node's degree is floor(w_i + hash_u01(i)); its neighbour list is that
    many endpoints drawn i.i.d. proportional to w (inverse CDF, closed form),
    with self loops and duplicates dropped.  Sampling `k` neighbours uniformly
    without replacement from such a list is distributed as drawing k endpoints
    proportional to w and dropping repeats, which is what `sample_hop` does.
    """

    def __init__(self, n: int, avg_degree: float, gamma: float, w_max: float, seed: int):
        self.n = int(n)
        self.avg = float(avg_degree)
        self.alpha = 1.0 / (gamma - 1.0)
        self.seed = int(seed)
        self.w_max = float(w_max)
        self._solve()

    # antiderivative of (t+i0)^(-alpha)
    def _H(self, t, i0):
        a = self.alpha
        if abs(a - 1.0) < 1e-12:
            return np.log(t + i0)
        return (t + i0) ** (1.0 - a) / (1.0 - a)

    def _Hinv(self, h, i0):
        a = self.alpha
        if abs(a - 1.0) < 1e-12:
            return np.exp(h) - i0
        return ((1.0 - a) * h) ** (1.0 / (1.0 - a)) - i0

    def _solve(self) -> None:
        n, avg, wmax = self.n, self.avg, self.w_max
        total = n * avg

        # w_0 = c * (H(1)-H(0)) = wmax  and  c * (H(n)-H(0)) = total
        def ratio(i0):
            return (self._H(1.0, i0) - self._H(0.0, i0)) / (self._H(float(n), i0) - self._H(0.0, i0))

        target = wmax / total
        lo, hi = 1e-9, float(n) * 1e3
        # ratio(i0) decreases from ~1 (i0 -> 0) to 1/n (i0 -> inf)
        for _ in range(400):
            mid = math.sqrt(lo * hi)
            if ratio(mid) > target:
                lo = mid
            else:
                hi = mid
        self.i0 = math.sqrt(lo * hi)
        self.c = total / (self._H(float(n), self.i0) - self._H(0.0, self.i0))
        self._h0 = float(self._H(0.0, self.i0))
        self._hn = float(self._H(float(n), self.i0))

    def weight(self, rank: np.ndarray) -> np.ndarray:
        r = np.asarray(rank, dtype=np.float64)
        return self.c * (self._H(r + 1.0, self.i0) - self._H(r, self.i0))

    def degree(self, rank: np.ndarray) -> np.ndarray:
        w = self.weight(rank)
        return np.floor(w + hash_u01(rank, self.seed)).astype(np.int64)

    def draw_endpoints(self, rng: np.random.Generator, count: int) -> np.ndarray:
        u = rng.random(count)
        t = self._Hinv(self._h0 + u * (self._hn - self._h0), self.i0)
        return np.clip(np.floor(t), 0, self.n - 1).astype(np.int64)

    def global_id(self, rank: np.ndarray) -> np.ndarray:
        """Bijective affine scramble rank -> node id so that id order carries
        no degree information."""
        a = 0x9E3779B1 % self.n
        while math.gcd(a, self.n) != 1:
            a += 1
        b = 0x85EBCA6B % self.n
        r = np.asarray(rank, dtype=np.int64)
        # a, r < 2^31 for every graph here except n > 2^31 (not used)
        return (a * r + b) % self.n

    def sample_hop(self, rng: np.random.Generator, dst_rank: np.ndarray, fanout: Optional[int]):
        """Rows = dst_rank; returns (row_of_edge, nbr_rank) in sampled order with
        self loops and per-row duplicates removed (first occurrence kept)."""
        deg = self.degree(dst_rank)
        k = deg if fanout is None else np.minimum(deg, fanout)
        total = int(k.sum())
        rows = np.repeat(np.arange(dst_rank.shape[0], dtype=np.int64), k)
        nbr = self.draw_endpoints(rng, total)
        keep = nbr != dst_rank[rows]
        rows, nbr = rows[keep], nbr[keep]
        key = rows * np.int64(self.n) + nbr
        _, first = np.unique(key, return_index=True)
        first.sort()
        return rows[first], nbr[first]


def _relabel(dst_ids: np.ndarray, rows: np.ndarray, nbr_ids: np.ndarray):
    """dst ids keep 0..nd-1, other ids numbered by first appearance in edge order.
    Returns (Block, src_ids) where src_ids[local] = original id."""
    nd = dst_ids.shape[0]
    allv = np.concatenate([dst_ids, nbr_ids])
    uniq, first, inv = np.unique(allv, return_index=True, return_inverse=True)
    order = np.argsort(first, kind="stable")
    newid = np.empty(uniq.shape[0], dtype=np.int64)
    newid[order] = np.arange(uniq.shape[0], dtype=np.int64)
    local = newid[inv]
    assert np.array_equal(local[:nd], np.arange(nd)), "destination ids must be distinct"
    src_ids = uniq[order]
    indptr = np.zeros(nd + 1, dtype=np.int64)
    np.cumsum(np.bincount(rows, minlength=nd), out=indptr[1:])
    assert indptr[-1] < 2 ** 31 and uniq.shape[0] < 2 ** 31
    blk = Block(indptr.astype(np.int32), local[nd:].astype(np.int32), int(nd), int(uniq.shape[0]))
    return blk, src_ids


def _sample_distinct(rng: np.random.Generator, n: int, k: int, exclude: Sequence[int] = ()) -> np.ndarray:
    """k distinct integers in [0,n), none in `exclude`, in random order."""
    got: list = []
    seen = set(int(x) for x in exclude)
    while len(got) < k:
        for x in rng.integers(0, n, size=(k - len(got)) * 2 + 16):
            x = int(x)
            if x not in seen:
                seen.add(x)
                got.append(x)
                if len(got) == k:
                    break
    return np.asarray(got, dtype=np.int64)


def _sampled_layers(g: ChungLu, rng, seeds: np.ndarray, fanouts_from_seeds: Sequence[Optional[int]]):
    """Hop h's destinations are hop h-1's sources.  Returns blocks in
    input-layer-first order and the rank of every source node of blocks[0]."""
    blocks = []
    dst = seeds
    for f in fanouts_from_seeds:
        rows, nbr = g.sample_hop(rng, dst, f)
        blk, src = _relabel(dst, rows, nbr)
        blk.check()
        blocks.append(blk)
        dst = src
    blocks.reverse()
    for a, b in zip(blocks[:-1], blocks[1:]):
        assert a.num_dst == b.num_src, "layer chain broken"
    return blocks, dst


# ----------------------------------------------------------------------------
# the five workloads
# ----------------------------------------------------------------------------
CONFIG_NAMES = {
    1: "tiny-er-1layer",
    2: "products-shaped-3layer-gcn",
    3: "reddit-shaped-2layer-mean",
    4: "papers100m-shaped-3layer-bf16-sum",
    5: "skew-stress-full-neighbourhood",
}


def _config1(seed: int) -> Workload:
    rng = np.random.Generator(np.random.PCG64(seed))
    n, avg, nseed, fanout = 10_000, 10.0, 256, 5
    p = avg / (n - 1)
    m = int(rng.binomial(n * (n - 1) // 2, p))
    a = rng.integers(0, n, size=m + m // 8)
    b = rng.integers(0, n, size=m + m // 8)
    ok = a != b
    lo, hi = np.minimum(a[ok], b[ok]), np.maximum(a[ok], b[ok])
    und = np.unique(lo * n + hi)[:m]
    lo, hi = und // n, und % n
    s = np.concatenate([lo, hi])
    d = np.concatenate([hi, lo])
    order = np.argsort(s, kind="stable")
    s, d = s[order], d[order]
    gptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(np.bincount(s, minlength=n), out=gptr[1:])
    seeds = _sample_distinct(rng, n, nseed)
    rows, nbrs = [], []
    for r, u in enumerate(seeds):
        nb = d[gptr[u]:gptr[u + 1]]
        if nb.shape[0] > fanout:
            nb = rng.permutation(nb)[:fanout]
        else:
            nb = rng.permutation(nb)
        rows.append(np.full(nb.shape[0], r, dtype=np.int64))
        nbrs.append(nb)
    blk, _ = _relabel(seeds, np.concatenate(rows), np.concatenate(nbrs))
    blk.check()
    return Workload(CONFIG_NAMES[1], [blk], [64], "mean", "f32", seed)


def _fanouts(order: str):
    # list is in sampling order starting from the seeds
    return [15, 10, 5] if order == "A" else [5, 10, 15]


def _config2(seed: int, order: str) -> Workload:
    rng = np.random.Generator(np.random.PCG64(seed))
    n, avg = 2_400_000, 50.0
    g = ChungLu(n, avg, 2.1, math.sqrt(n * avg), seed)
    seeds = _sample_distinct(rng, n, 8000)
    blocks, _ = _sampled_layers(g, rng, seeds, _fanouts(order))
    return Workload(CONFIG_NAMES[2], blocks, [100, 256, 256], "gcn", "f32", seed)


def _config3(seed: int) -> Workload:
    rng = np.random.Generator(np.random.PCG64(seed))
    n, avg = 233_000, 492.0
    g = ChungLu(n, avg, 2.1, 20_000.0, seed)
    seeds = _sample_distinct(rng, n, 1024)
    blocks, _ = _sampled_layers(g, rng, seeds, [25, 10])
    return Workload(CONFIG_NAMES[3], blocks, [602, 256], "mean", "f32", seed)


def _config4(seed: int, order: str) -> Workload:
    rng = np.random.Generator(np.random.PCG64(seed))
    n, avg = 111_000_000, 29.0
    g = ChungLu(n, avg, 2.0, math.sqrt(n * avg), seed)
    seeds = _sample_distinct(rng, n, 1024)
    blocks, src_rank = _sampled_layers(g, rng, seeds, _fanouts(order))
    gid = g.global_id(src_rank).astype(np.int64)
    return Workload(CONFIG_NAMES[4], blocks, [128, 256, 256], "sum", "bf16", seed,
                    src_gid=gid, table_rows=n)


def _config5(seed: int, width: int) -> Workload:
    rng = np.random.Generator(np.random.PCG64(seed))
    n, avg = 1_000_000, 100.0
    g = ChungLu(n, avg, 1.8, 50_000.0, seed)
    top = np.arange(16, dtype=np.int64)
    others = _sample_distinct(rng, n, 65_536 - 16, exclude=top)
    dst = rng.permutation(np.concatenate([top, others]))
    rows, nbr = g.sample_hop(rng, dst, None)
    blk, _ = _relabel(dst, rows, nbr)
    blk.check()
    assert int(np.diff(blk.indptr).max()) > 10_000, "skew config needs a hub row"
    return Workload(CONFIG_NAMES[5] + f"-F{width}", [blk], [width], "gcn", "f32", seed)


def make_config(cfg: int, run: int = 0, fanout_order: str = "A", width: int = 32) -> Workload:
    """Build one of the five workloads; seed = 1000*cfg + run."""
    seed = 1000 * cfg + run
    if cfg == 1:
        return _config1(seed)
    if cfg == 2:
        return _config2(seed, fanout_order)
    if cfg == 3:
        return _config3(seed)
    if cfg == 4:
        return _config4(seed, fanout_order)
    if cfg == 5:
        return _config5(seed, width)
    raise ValueError(f"unknown config {cfg}")


# ----------------------------------------------------------------------------
# small random blocks for unit / property tests
# ----------------------------------------------------------------------------
def random_block(rng: np.random.Generator, num_dst: int, num_src: int, avg_deg: float,
                 empty_frac: float = 0.2, hub_rows: int = 0, hub_deg: int = 0) -> Block:
    """Arbitrary CSR: unsorted rows, duplicate edges allowed, some empty rows,
    optionally a few very long rows. num_src may exceed the referenced ids."""
    if num_dst == 0 or num_src == 0:
        return Block(np.zeros(num_dst + 1, np.int32), np.zeros(0, np.int32), num_dst, num_src)
    deg = rng.poisson(avg_deg, size=num_dst).astype(np.int64)
    deg[rng.random(num_dst) < empty_frac] = 0
    if hub_rows:
        deg[rng.choice(num_dst, size=min(hub_rows, num_dst), replace=False)] = hub_deg
    indptr = np.zeros(num_dst + 1, dtype=np.int64)
    np.cumsum(deg, out=indptr[1:])
    e = int(indptr[-1])
    # skewed source popularity so that some source rows are hubs too
    r = rng.random(e)
    idx = np.minimum((r * r * num_src).astype(np.int64), num_src - 1)
    blk = Block(indptr.astype(np.int32), idx.astype(np.int32), num_dst, num_src)
    blk.check()
    return blk


def banded_like(blk: Block, window: int, seed: int) -> Block:
    """A block with the row lengths of `blk` whose neighbours are re-drawn near the diagonal:
    row u takes its neighbours uniformly from the `window` source rows around u * num_src / num_dst.
    Same sizes and degree sequence as `blk`, but with the locality a graph with community structure
    has after a locality-preserving node ordering (which a Chung-Lu graph cannot offer)."""
    rng = np.random.default_rng(seed)
    rows = np.repeat(np.arange(blk.num_dst, dtype=np.int64), np.diff(blk.indptr))
    centre = rows * blk.num_src // max(blk.num_dst, 1)
    idx = centre + rng.integers(-(window // 2), window // 2 + 1, size=rows.shape[0])
    idx = np.clip(idx, 0, blk.num_src - 1)
    out = Block(blk.indptr.copy(), idx.astype(np.int32), blk.num_dst, blk.num_src)
    out.check()
    return out


def minibatch_node_sets(n_batches: int, seed: int, n: int = 2_400_000, avg: float = 50.0, gamma: float = 2.1,
                        n_seeds: int = 8000, fanouts: Sequence[int] = (15, 10, 5)):
    """Node sets of several mini-batches sampled from ONE graph (the products-shaped Chung-Lu graph
    by default): for each mini-batch the global IDs of the source nodes of its input-layer block, in
    local-ID order (distinct).  These are the nodes whose features a mini-batch needs; consecutive
    mini-batches share many of them (the hubs), which is what the Match process exploits."""
    g = ChungLu(n, avg, gamma, math.sqrt(n * avg), seed)
    out = []
    for b in range(n_batches):
        rng = np.random.Generator(np.random.PCG64([seed, b]))
        seeds = _sample_distinct(rng, n, n_seeds)
        _, src_rank = _sampled_layers(g, rng, seeds, list(fanouts))
        out.append(g.global_id(src_rank).astype(np.int64))
    return out


def hop_global_ids(blk: Block, seed: int, bits: int = 40):
    """Global IDs for the nodes of a block: local ID l -> (l * A + C) mod 2^bits with A odd, which
    is one-to-one.  Returns (dst_gid int64[num_dst], nbr_gid int64[E]): what a sampler hands to
    the ID map for this hop (destinations first, then the sampled neighbours in edge order)."""
    rng = np.random.default_rng(seed)
    mask = (1 << bits) - 1
    a = (int(rng.integers(1, 1 << (bits - 1))) << 1 | 1) & mask
    c = int(rng.integers(0, 1 << bits))

    def to_gid(local):
        x = local.astype(np.uint64)
        return ((x * np.uint64(a) + np.uint64(c)) & np.uint64(mask)).astype(np.int64)
    return to_gid(np.arange(blk.num_dst)), to_gid(blk.indices)


# ----------------------------------------------------------------------------
# feature matrices
# ----------------------------------------------------------------------------
def features_f32(rng: np.random.Generator, rows: int, width: int) -> np.ndarray:
    return rng.standard_normal((rows, width), dtype=np.float32)


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bfloat16 bit patterns (uint16), round to nearest even.
    Input preparation only (the values handed to both sides are the bf16 ones)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = u + np.uint32(0x7FFF) + lsb
    return (r >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)
