// Per-block integer bookkeeping on the GPU: degrees, scale factors, a stable
// transpose of the CSR, equal-work row sets and degree buckets (ordered compaction of
// long rows).  Everything is integer work with a single valid answer: no float atomics,
// no order-dependent results, and (on the full-plan path) no global atomics at all.
//
// Why it exists: the backward pass (paper Section 4.2, Eq. 5) gathers along
// the reversed edges; pulling along a transposed CSR keeps one writer per
// output row, as the forward pass has (Section 4.2: a target's aggregation is
// completed by one owner).  Every sampled block is new, so this work is part of
// each iteration and is kept to a handful of launches.  The work of a plan is a
// sequence of STAGES; stage k of every plan built in one call shares one launch
// of k_plan_stage, whose workgroups look up which job they belong to.
//
// The transpose of a block with at most 2^21 source nodes (every sampled block of the
// paper's workloads) is BUCKETED: the edges are split, in order, into buckets of 2 048
// consecutive source ids, and a workgroup then finishes a bucket on chip.
//
//   stage 0   bucket histogram per workgroup      + destination-side row pass (degrees,
//             scale factors, edge -> row expansion, equal-work split, long-row counts)
//   stage 1   column prefix of the histograms     + destination-side long-row fill
//   stage 2   stable scatter of the edges into their buckets
//   stage 3   k_plan_bucket_counts: buckets of more than 7 680 edges are finished in sub-chunks;
//             edges per source of each sub-chunk
//             k_plan_buckets: per bucket (sub-chunk): out-degrees of its 2 048 sources, their row
//             starts (indptr_T), the source-side row pass, and the stable placement of its edges
//             (indices_T, the edge permutation)
//   stage 4   source-side long-row fill
//
// Six launches for the plans of all layers of a mini-batch.  Blocks with more source
// nodes take an LSD radix sort of the edges by source id instead (8-bit digits:
// histogram + scatter per pass, then row starts, row pass, fill: 9 launches at 3 passes).
// These stages are bound by latency and instruction issue, not by bytes: loads are written
// so that all loads of a phase are in flight together, and a launch holds enough workgroups
// to fill the compute units once.
#include <vector>

#include "internal.h"

namespace fastgl {

constexpr int kSortThreads = 1024;                   // 16 wavefronts per sort workgroup
constexpr int kSortWaves = kSortThreads / kWave;
constexpr int kMaxSortItems = 4;                     // keys per thread and step: 1, 2 or 4
constexpr int kMaxSortBlocks = 256;
constexpr int kSplitThreads = 512;                   // workgroup of the split into buckets (bucketed transpose)
constexpr int kMaxSplitBlocks = 512;                 // two of them per compute unit

// -------------------------------------------------- block-wide primitives ----
__device__ __forceinline__ int wave_incl_scan(int v)
{
    const int lane = threadIdx.x & (kWave - 1);
#pragma unroll
    for (int o = 1; o < kWave; o <<= 1) {
        int t = __shfl_up(v, o, kWave);
        if (lane >= o) v += t;
    }
    return v;
}

// Exclusive scan over all threads of the block (any multiple of 64 up to 1024);
// *total = block sum.  `lds` needs 16 ints and is free again on return.
__device__ __forceinline__ int block_excl_scan(int v, int *total, int *lds)
{
    const int lane = threadIdx.x & (kWave - 1), w = threadIdx.x / kWave, nw = blockDim.x / kWave;
    int inc = wave_incl_scan(v);
    if (lane == kWave - 1) lds[w] = inc;
    __syncthreads();
    int off = 0, tot = 0;
    for (int i = 0; i < nw; ++i) {
        int s = lds[i];
        if (i < w) off += s;
        tot += s;
    }
    __syncthreads();
    *total = tot;
    return off + inc - v;
}

// Block sums of two values at once.  `lds` needs 32 ints and is free again on return.
__device__ __forceinline__ void block_sum2(int &a, int &b, int *lds)
{
    const int lane = threadIdx.x & (kWave - 1), w = threadIdx.x / kWave, nw = blockDim.x / kWave;
#pragma unroll
    for (int o = kWave / 2; o > 0; o >>= 1) {
        a += __shfl_xor(a, o, kWave);
        b += __shfl_xor(b, o, kWave);
    }
    if (lane == 0) {
        lds[w] = a;
        lds[16 + w] = b;
    }
    __syncthreads();
    int sa = 0, sb = 0;
    for (int i = 0; i < nw; ++i) {
        sa += lds[i];
        sb += lds[16 + i];
    }
    __syncthreads();
    a = sa;
    b = sb;
}

// ---------------------------------------- degrees + long-row buckets (roles) ----
struct RowsArgs {
    const int32_t *rowptr;   // [n+1]
    int64_t n, per;          // block b owns rows [b*per, min(n,(b+1)*per))
    int nb;
    int32_t *len_out;        // [n] or NULL
    float *inv, *rsq;        // [n] or NULL: 1/max(len,1), 1/sqrt(max(len,1))
    int32_t *counts;         // [2*nb] per-block (long rows, chunks)
    int32_t *long_rows, *chunk_ptr, *totals;
    int32_t *edge_row;       // [nnz] or NULL: edge_row[e] = row that owns edge e
    int32_t *split;          // [nsets+1] or NULL: first row of every equal-work row set
    int64_t nsets;
};

// What one row contributes: its length and scale factors, the long-row counts, and the
// equal-work row sets that start right after it.  Called by every thread of a wavefront
// together (rows that start many sets are written by the whole wavefront); valid = the
// thread has a row.  e0 = first edge of row r, len = its length.
__device__ __forceinline__ void row_emit(const RowsArgs &A, int64_t r, bool valid, int e0, int len, int &nl,
                                         int &nc)
{
    const int lane = threadIdx.x & (kWave - 1);
    if (valid) {
        if (A.len_out) A.len_out[r] = len;
        double d = (double)(len < 1 ? 1 : len);
        if (A.inv) A.inv[r] = (float)(1.0 / d);
        if (A.rsq) A.rsq[r] = (float)(1.0 / sqrt(d));
        if (len > kLongThreshold) {
            nl += 1;
            nc += (len + kLongChunk - 1) / kLongChunk;
        }
    }
    if (A.split) {
        // Equal-work row sets: set g starts at the first row whose work prefix
        // W[r] = rowptr[r] + r reaches g * kWorkPerGroup.  Row r+1 is that row for
        // every g in (W[r]/work, W[r+1]/work]; the thread of row r writes them.
        int64_t g0 = 1, g1 = 0;   // empty
        if (valid) {
            g0 = ((int64_t)e0 + r) / kWorkPerGroup + 1;
            g1 = ((int64_t)e0 + len + r + 1) / kWorkPerGroup;
            if (r == 0) A.split[0] = 0;
            if (r == A.n - 1 && g1 < A.nsets) A.split[A.nsets] = (int32_t)A.n;   // partial last set
        }
        const bool big = g1 - g0 >= kWave;
        if (!big)
            for (int64_t g = g0; g <= g1; ++g) A.split[g] = (int32_t)(r + 1);
        unsigned long long m = __ballot(big);
        while (m) {
            const int leader = __ffsll((long long)m) - 1;
            const int64_t lg0 = __shfl(g0, leader, kWave), lg1 = __shfl(g1, leader, kWave);
            const int64_t lr = __shfl(r, leader, kWave);
            for (int64_t g = lg0 + lane; g <= lg1; g += kWave) A.split[g] = (int32_t)(lr + 1);
            m &= m - 1;
        }
    }
}

// Pass 1 over row pointers: row lengths, scale factors, per-block counts of long
// rows / their chunks, and (optionally) the row id of every edge.  A thread
// expands its own short rows; rows longer than a wavefront are expanded by the
// whole wavefront, one after the other.
__device__ __forceinline__ void rows_count(const RowsArgs &A, int b, int *lds)
{
    int64_t beg = b * A.per, end = beg + A.per < A.n ? beg + A.per : A.n;
    const int lane = threadIdx.x & (kWave - 1);
    int nl = 0, nc = 0;
    for (int64_t base = beg; base < end; base += blockDim.x) {
        const int64_t r = base + threadIdx.x;
        int e0 = 0, len = 0;
        if (r < end) {
            e0 = A.rowptr[r];
            len = A.rowptr[r + 1] - e0;
        }
        row_emit(A, r, r < end, e0, len, nl, nc);
        if (A.edge_row) {
            const bool big = len > kWave;
            if (!big)
                for (int k = 0; k < len; ++k) A.edge_row[e0 + k] = (int32_t)r;
            unsigned long long m = __ballot(big);
            while (m) {
                const int leader = __ffsll((long long)m) - 1;
                const int le0 = __shfl(e0, leader, kWave), ll = __shfl(len, leader, kWave);
                const int lr = __shfl((int)r, leader, kWave);
                for (int k = lane; k < ll; k += kWave) A.edge_row[le0 + k] = lr;
                m &= m - 1;
            }
        }
    }
    block_sum2(nl, nc, lds);
    if (threadIdx.x == 0) {
        A.counts[2 * b] = nl;
        A.counts[2 * b + 1] = nc;
    }
}

// Pass 2: ordered compaction.  long_rows ascending; chunk_ptr[i] = first chunk of
// the i-th long row; totals[0] = number of long rows, totals[1] = number of chunks.
__device__ __forceinline__ void rows_fill(const RowsArgs &A, int b, int *lds)
{
    // long rows and chunks in the blocks before this one; the loads go out together (past the end
    // they re-read the block's own pair)
    const int2 *cnt = reinterpret_cast<const int2 *>(A.counts);
    const int2 own = cnt[b];
    int cl = 0, cc = 0;
    constexpr int kBatch = 4;
    for (int i0 = threadIdx.x; i0 < b; i0 += kBatch * blockDim.x) {
        int2 v[kBatch];
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
            const int i = i0 + u * (int)blockDim.x;
            v[u] = cnt[i < b ? i : b];
        }
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
            if (i0 + u * (int)blockDim.x < b) {
                cl += v[u].x;
                cc += v[u].y;
            }
        }
    }
    block_sum2(cl, cc, lds);
    int64_t beg = b * A.per, end = beg + A.per < A.n ? beg + A.per : A.n;
    const bool any = own.x != 0;      // block-uniform: most blocks have no long row
    for (int64_t base = beg; any && base < end; base += blockDim.x) {
        int64_t r = base + threadIdx.x;
        int len = r < end ? A.rowptr[r + 1] - A.rowptr[r] : 0;
        int isl = len > kLongThreshold ? 1 : 0;
        int nch = isl ? (len + kLongChunk - 1) / kLongChunk : 0;
        int tl, tc;
        int el = block_excl_scan(isl, &tl, lds);
        int ec = block_excl_scan(nch, &tc, lds);
        if (isl) {
            A.long_rows[cl + el] = (int32_t)r;
            A.chunk_ptr[cl + el] = cc + ec;
        }
        cl += tl;
        cc += tc;
    }
    if (b == A.nb - 1 && threadIdx.x == 0) {
        A.chunk_ptr[cl] = cc;
        A.totals[0] = cl;
        A.totals[1] = cc;
    }
}

// ------------------------------------ bucketed transpose: sizes, workgroup map ----
constexpr int kBucketBits = 11;
constexpr int kBucketIds = 1 << kBucketBits;
constexpr int kMaxBuckets = 1024;                            // one thread per bucket in the histogram, two in the scatter's prologue
constexpr int kLocalThreads = 512;
constexpr int kLocalWaves = kLocalThreads / kWave;
constexpr int kSubRounds = 15;                               // rounds of 64 edges per wavefront
constexpr int kSubChunk = kLocalWaves * kSubRounds * kWave;  // 7 680 edges; below 65 536: 16-bit counts
constexpr int kLocalKeys = kBucketIds / kLocalThreads;       // consecutive sources per thread in the scans
constexpr int kLocalWords = kLocalKeys / 2;                  // = words of the count table per thread
static_assert(kMaxBuckets <= kSortThreads && kMaxBuckets <= kMaxScanBlocks, "bucket prologue, fill pass");
static_assert(kLocalKeys * kLocalThreads == kBucketIds && kLocalKeys % 2 == 0, "whole words per thread");
static_assert(kSubChunk < 65536, "per-wavefront counts are 16 bits wide");

struct BucketOfGroup {   // what workgroup g of k_plan_buckets works on
    int bucket;          // -1: nothing
    int sub;             // sub-chunk of the bucket
    int first_edge;      // of the bucket
    int edges;           // of the bucket
};

inline int64_t bucket_groups(int nbuckets, int64_t n) { return nbuckets + n / kSubChunk; }   // >= groups in use
// >= groups of buckets with several sub-chunks: such a bucket of e > kSubChunk edges takes ceil(e / kSubChunk) < 2e / kSubChunk
inline int64_t large_bucket_groups(int64_t n) { return n > kSubChunk ? 2 * n / kSubChunk + 1 : 0; }

// Bucket d takes max(1, ceil(tot[d] / kSubChunk)) workgroups.  Those of the buckets with several
// sub-chunks come first (they have the most to do, and workgroups start in this order), then one per
// remaining bucket.  Written by one workgroup of the scatter launch: a thread has PER consecutive
// buckets from d0 on, tv[] = their edges, ex[] = their first edges.
template <int PER>
__device__ __forceinline__ void write_bucket_map(BucketOfGroup *map, int cap, int nbuckets, int d0,
                                                 const int (&tv)[PER], const int (&ex)[PER], int *lds)
{
    int ns[PER], nl = 0, nsm = 0;
#pragma unroll
    for (int i = 0; i < PER; ++i) {
        ns[i] = d0 + i < nbuckets ? (tv[i] > kSubChunk ? (tv[i] + kSubChunk - 1) / kSubChunk : 1) : 0;
        nl += ns[i] > 1 ? ns[i] : 0;
        nsm += ns[i] == 1 ? 1 : 0;
    }
    int large, small;
    int wl = block_excl_scan(nl, &large, lds);
    int ws = large + block_excl_scan(nsm, &small, lds);
#pragma unroll
    for (int i = 0; i < PER; ++i) {
        int at = 0;
        if (ns[i] > 1) {
            at = wl;
            wl += ns[i];
        } else if (ns[i] == 1) {
            at = ws;
            ws += 1;
        }
        for (int q = 0; q < ns[i]; ++q) {
            BucketOfGroup m;
            m.bucket = d0 + i; m.sub = q; m.first_edge = ex[i]; m.edges = tv[i];
            if (at + q < cap) map[at + q] = m;
        }
    }
    for (int i = large + small + (int)threadIdx.x; i < cap; i += blockDim.x) map[i].bucket = -1;
}

// ------------------------------------------------- stable split by a digit ----
// One stable counting pass over (source id, destination row[, edge id]) triples: a pass of the
// LSD radix sort (digit = 8 bits of the key), or the split into buckets of kBucketIds consecutive
// source ids of the bucketed transpose (digit = key >> kBucketBits: 8 or 10 bits).
struct SortArgs {
    const int32_t *keys_in, *vals_in;   // vals: the destination row of the edge
    int32_t *keys_out, *vals_out;
    const int32_t *eid_in;              // second payload, the original edge id; NULL on the first pass = identity
    int32_t *eid_out;                   // NULL: the plan carries no edge permutation
    int64_t n, per;                     // block b owns keys [b*per, min(n,(b+1)*per))
    int nb, shift;
    int bits;                           // digit width: kRadixBits, or 10 for more than 256 buckets
    int nbins;                          // digits that occur = row length of cnt
    int32_t *cnt;                       // [nb][nbins] digit counts per block; after the column prefix of the
                                        // bucketed transpose: keys of that digit in earlier blocks
    const int32_t *tot;                 // bucketed transpose: [nbins] keys per digit; NULL: LSD pass
    struct BucketOfGroup *map;          // bucketed transpose: [map_cap] which bucket each workgroup of the next
    int map_cap;                        // stage finishes (written by workgroup 0)
    int items;                          // keys per thread and step: 1, 2 or 4
};

__device__ __forceinline__ int digit_of(const SortArgs &S, int32_t key) { return (key >> S.shift) & ((1 << S.bits) - 1); }

// Lanes of the wavefront whose `bits`-bit value equals this lane's (lanes with ok == false match
// nobody and nobody matches them).  One ballot per bit; lo / hi = the mask's halves.
template <int BITS>
__device__ __forceinline__ void match_lanes(int v, bool ok, unsigned &lo, unsigned &hi)
{
    const unsigned long long act = __ballot(ok);
    unsigned dlo = 0, dhi = 0;   // lanes that differ from this one in some bit
#pragma unroll
    for (int bit = 0; bit < BITS; ++bit) {
        const int neg = (int)((unsigned)v << (31 - bit)) >> 31;   // all ones where the bit is set
        const unsigned long long bl = __ballot(neg < 0);
        dlo |= (unsigned)bl ^ (unsigned)neg;
        dhi |= (unsigned)(bl >> 32) ^ (unsigned)neg;
    }
    lo = ok ? (unsigned)act & ~dlo : 0u;
    hi = ok ? (unsigned)(act >> 32) & ~dhi : 0u;
}

__device__ __forceinline__ int lanes_below(unsigned lo, unsigned hi)   // set bits of the mask below this lane
{
    return (int)__builtin_amdgcn_mbcnt_hi(hi, __builtin_amdgcn_mbcnt_lo(lo, 0u));
}

// Digit histogram of the block's key range.  h: 1 << bits counters.
__device__ __forceinline__ void sort_hist(const SortArgs &S, int b, int *h)
{
    for (int i = threadIdx.x; i < (1 << S.bits); i += kSortThreads) h[i] = 0;
    __syncthreads();
    const int64_t beg = b * S.per, end = beg + S.per < S.n ? beg + S.per : S.n;
    constexpr int kBatch = 8;   // loads in flight per thread (past the end they re-read the last key)
    for (int64_t i0 = beg + threadIdx.x; i0 < end; i0 += (int64_t)kBatch * kSortThreads) {
        int32_t key[kBatch];
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
            const int64_t i = i0 + (int64_t)u * kSortThreads;
            key[u] = S.keys_in[i < end ? i : end - 1];
        }
#pragma unroll
        for (int u = 0; u < kBatch; ++u)
            if (i0 + (int64_t)u * kSortThreads < end) atomicAdd(&h[digit_of(S, key[u])], 1);
    }
    __syncthreads();
    if (threadIdx.x < S.nbins) S.cnt[(int64_t)b * S.nbins + threadIdx.x] = h[threadIdx.x];
}

// Bucketed transpose, between histogram and scatter: cnt[b][d] becomes the number of keys of digit
// d in blocks before b, tot[d] the number in all blocks.  A workgroup takes 64 columns (one per
// lane); each wavefront sums a strip of rows, then walks it again with its running prefix.
struct ColScanArgs {
    int32_t *cnt, *tot;
    int nb, nbins;
};

__device__ __forceinline__ void col_scan(const ColScanArgs &A, int g, int *part)   // part: [kSortWaves][64]
{
    const int lane = threadIdx.x & (kWave - 1), w = threadIdx.x / kWave;
    const int c = g * kWave + lane;
    const bool ok = c < A.nbins;
    const int rp = (A.nb + kSortWaves - 1) / kSortWaves;
    const int r0 = w * rp < A.nb ? w * rp : A.nb, r1 = r0 + rp < A.nb ? r0 + rp : A.nb;
    int sum = 0;
    if (ok) {
#pragma unroll 4
        for (int r = r0; r < r1; ++r) sum += A.cnt[(int64_t)r * A.nbins + c];
    }
    part[w * kWave + lane] = sum;
    __syncthreads();
    int base = 0, total = 0;
#pragma unroll
    for (int k = 0; k < kSortWaves; ++k) {
        const int v = part[k * kWave + lane];
        if (k < w) base += v;
        total += v;
    }
    if (ok) {
        if (w == 0) A.tot[c] = total;
#pragma unroll 4
        for (int r = r0; r < r1; ++r) {
            int32_t *q = A.cnt + (int64_t)r * A.nbins + c;
            const int v = *q;
            *q = base;
            base += v;
        }
    }
}

// Stable scatter by one digit.  Output offsets of the block's digits: for an LSD pass every
// workgroup derives them from the [nb][256] count table (no separate scan launch),
//   base = sum_{d' < d} total[d'] + sum_{b' < b} cnt[b'][d];
// for the bucketed transpose the column prefix is already there and only tot[] is scanned.
// Within a step of 1024*ITEMS keys each wavefront owns 64*ITEMS consecutive keys and ranks
// them 64 at a time: lanes with equal digits find each other with one ballot per digit bit, the
// running per-wavefront digit counts live in LDS, and a column scan over the 16
// wavefronts plus a scan over the digits give each key its place in the step's
// sorted order.  The step is sorted into LDS first and written out from there.
// The payload is the edge's destination row and, if asked for, its original id.
template <int BITS, int NT>
struct SortShared {
    static constexpr int kBins = 1 << BITS;
    int running[kBins], lbase[kBins], gdelta[kBins];
    int wcnt[NT / kWave][kBins];
    int32_t skey[NT * kMaxSortItems], sval[NT * kMaxSortItems];
    int32_t seid[NT * kMaxSortItems];
};

// NT threads: 1024 for an LSD pass (its prologue is laid out for that), kSplitThreads for the split
// into buckets, where two or three smaller workgroups share a compute unit and fill each other's
// waits at the barriers.
template <int ITEMS, int BITS, int NT>
__device__ __forceinline__ void sort_scatter(const SortArgs &S, int b, SortShared<BITS, NT> &M, int *lds)
{
    constexpr int kBins = 1 << BITS, kWaves = NT / kWave;
    constexpr int kPer = kBins > NT ? kBins / NT : 1;   // consecutive digits per thread in the scans
    static_assert(kPer * NT >= kBins && (kWaves * kBins) % NT == 0, "digits and counters divide among the threads");
    int (&running)[kBins] = M.running, (&lbase)[kBins] = M.lbase, (&gdelta)[kBins] = M.gdelta;
    int (&wcnt)[kWaves][kBins] = M.wcnt;
    int32_t *skey = M.skey, *sval = M.sval, *seid = M.seid;
    const bool EID = S.eid_out != nullptr;
    const int t = threadIdx.x, lane = t & (kWave - 1), w = t / kWave;
    const int d0 = t * kPer;   // this thread's digits in the scans: d0 .. d0 + kPer - 1, those below kBins
    if (S.tot) {   // bucketed transpose: start of the bucket + keys of it in earlier blocks
        int tv[kPer], ex[kPer], sum = 0;
#pragma unroll
        for (int i = 0; i < kPer; ++i) {
            tv[i] = d0 + i < S.nbins ? S.tot[d0 + i] : 0;
            sum += tv[i];
        }
        int cb[kPer];
#pragma unroll
        for (int i = 0; i < kPer; ++i) cb[i] = d0 + i < S.nbins ? S.cnt[(int64_t)b * S.nbins + d0 + i] : 0;
        int dummy;
        int at = block_excl_scan(sum, &dummy, lds);
#pragma unroll
        for (int i = 0; i < kPer; ++i) {
            ex[i] = at;
            at += tv[i];
            if (d0 + i < kBins) running[d0 + i] = d0 + i < S.nbins ? ex[i] + cb[i] : 0;
        }
        if (b == 0) write_bucket_map<kPer>(S.map, S.map_cap, S.nbins, d0, tv, ex, lds);
        __syncthreads();
    } else if constexpr (BITS == kRadixBits && NT == kSortThreads) {   // LSD pass: offsets from the whole count table
        const int d = t & (kBins - 1), part = t / kBins;   // 4 parts share the blocks
        int below = 0, total = 0;
        constexpr int kParts = kSortThreads / kBins, kBatch = 16;
        for (int b0 = part; b0 < S.nb; b0 += kParts * kBatch) {
            int c[kBatch];
#pragma unroll
            for (int k = 0; k < kBatch; ++k) {   // independent loads first
                const int bb = b0 + k * kParts;
                c[k] = bb < S.nb ? S.cnt[(int64_t)bb * kBins + d] : 0;
            }
#pragma unroll
            for (int k = 0; k < kBatch; ++k) {
                total += c[k];
                if (b0 + k * kParts < b) below += c[k];
            }
        }
        wcnt[part][d] = below;
        wcnt[4 + part][d] = total;
        __syncthreads();
        int tot = 0, bel = 0;
        if (t < kBins) {
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                bel += wcnt[k][t];
                tot += wcnt[4 + k][t];
            }
        }
        int dummy;
        int ex = block_excl_scan(t < kBins ? tot : 0, &dummy, lds);   // threads >= 256 add 0 after the digits
        if (t < kBins) running[t] = ex + bel;
        __syncthreads();
    }
    const int64_t beg = b * S.per, end = beg + S.per < S.n ? beg + S.per : S.n;
    // the keys of a step are loaded while the step before it is worked on; the loads carry no
    // branch of their own (past the end they re-read the last key), so they go out together
    int32_t nkey[ITEMS], nval[ITEMS], neid[ITEMS];
    auto load_step = [&](int64_t step) {
#pragma unroll
        for (int i = 0; i < ITEMS; ++i) {
            const int64_t idx = step + (int64_t)w * (kWave * ITEMS) + i * kWave + lane;
            const int64_t at = idx < end ? idx : end - 1;
            nkey[i] = S.keys_in[at];
            nval[i] = S.vals_in[at];
            neid[i] = EID ? (S.eid_in ? S.eid_in[at] : (int32_t)at) : 0;
        }
    };
    if (beg < end) load_step(beg);
    for (int64_t step = beg; step < end; step += NT * ITEMS) {
#pragma unroll
        for (int k = 0; k < kWaves * kBins / NT; ++k)
            (&wcnt[0][0])[k * NT + t] = 0;
        __syncthreads();
        int32_t key[ITEMS], val[ITEMS], eid[ITEMS];
        int rank[ITEMS], dig[ITEMS];
        bool ok[ITEMS];
#pragma unroll
        for (int i = 0; i < ITEMS; ++i) {
            const int64_t idx = step + (int64_t)w * (kWave * ITEMS) + i * kWave + lane;
            ok[i] = idx < end;
            key[i] = nkey[i];
            val[i] = nval[i];
            eid[i] = neid[i];
            dig[i] = (key[i] >> S.shift) & (kBins - 1);
        }
        if (step + NT * ITEMS < end) load_step(step + NT * ITEMS);
#pragma unroll
        for (int i = 0; i < ITEMS; ++i) {
            unsigned mlo, mhi;
            match_lanes<BITS>(dig[i], ok[i], mlo, mhi);
            const int lower = lanes_below(mlo, mhi);
            const int prior = ok[i] ? wcnt[w][dig[i]] : 0;   // count from this wavefront's earlier rounds
            rank[i] = prior + lower;
            // the LDS read above is issued before this write by the same wavefront
            if (ok[i] && lower == 0) wcnt[w][dig[i]] = prior + __popc(mlo) + __popc(mhi);
        }
        __syncthreads();
        // column scan over the wavefronts, then a scan over the digits: position of
        // every key inside this step's sorted order
        int tot_d[kPer], tot_t = 0;
#pragma unroll
        for (int i = 0; i < kPer; ++i) {
            tot_d[i] = 0;
            if (d0 + i < kBins) {
#pragma unroll
                for (int k = 0; k < kWaves; ++k) {
                    int c = wcnt[k][d0 + i];
                    wcnt[k][d0 + i] = tot_d[i];
                    tot_d[i] += c;
                }
            }
            tot_t += tot_d[i];
        }
        int nvalid;
        int lb = block_excl_scan(tot_t, &nvalid, lds);
#pragma unroll
        for (int i = 0; i < kPer; ++i) {
            if (d0 + i < kBins) {
                lbase[d0 + i] = lb;
                gdelta[d0 + i] = running[d0 + i] - lb;   // global position = gdelta[digit] + position in the step
                running[d0 + i] += tot_d[i];
                lb += tot_d[i];
            }
        }
        __syncthreads();
#pragma unroll
        for (int i = 0; i < ITEMS; ++i) {
            if (!ok[i]) continue;
            const int lpos = lbase[dig[i]] + wcnt[w][dig[i]] + rank[i];
            skey[lpos] = key[i];
            sval[lpos] = val[i];
            if (EID) seid[lpos] = eid[i];
        }
        __syncthreads();
        // keys of one digit are now consecutive in LDS and go to consecutive global
        // slots: neighbouring threads write neighbouring addresses
#pragma unroll
        for (int i = 0; i < ITEMS; ++i) {
            const int j = i * NT + t;
            if (j >= nvalid) continue;
            const int32_t k = skey[j], v = sval[j];
            const int64_t pos = (int64_t)gdelta[(k >> S.shift) & (kBins - 1)] + j;
            if (pos < 0 || pos >= S.n) continue;   // only a source id outside [0, num_src) gets here
            S.keys_out[pos] = k;
            S.vals_out[pos] = v;
            if (EID) S.eid_out[pos] = seid[j];
        }
        __syncthreads();   // wcnt and the staging arrays are reused by the next step
    }
}

// ------------------------------------------- bucketed transpose: one bucket ----
// The edges of bucket d (source ids [d * kBucketIds, (d+1) * kBucketIds), in their original
// order) are finished by one workgroup of k_plan_buckets per sub-chunk of kSubChunk edges (most
// buckets are one sub-chunk).  The workgroup places its sub-chunk: each wavefront owns a run of
// consecutive edges and counts them per source (16-bit counters, two to a word), a column scan
// over the wavefronts turns the counts into offsets and yields the sub-chunk's edges per source,
// a scan over the sources gives the row starts, and a second walk ranks 64 edges at a time
// (equal sources find each other with one ballot per id bit).  Edges of one source thus keep
// their order: the transposed row lists its destination rows as a stable counting sort does.
// A bucket of several sub-chunks is first counted per source outside the own sub-chunk (all of
// it -> out-degrees and row starts; what precedes the sub-chunk -> where the own edges of a
// source begin).  The first sub-chunk's workgroup also writes what belongs to the bucket's rows:
// indptr_T, out-degrees, scale factors, row sets, long-row counts.
struct LocalArgs {
    const int32_t *keys, *vals, *eids;   // the bucketed edges: source id, destination row, edge id
    const BucketOfGroup *map;
    uint16_t *subcnt;                    // [large_groups][kBucketIds] edges per source of every sub-chunk of a bucket
    int large_groups;                    // that has several (workgroups 0 .. of the map, at most this many)
    int nbuckets;
    int64_t n, num_src;
    int32_t *indptr_T, *indices_T, *perm;   // perm NULL: not wanted (eids is not read then)
    RowsArgs rows;                       // source-side row outputs; counts[] is per bucket
};

struct LocalShared {
    int start[kBucketIds];                          // first edge (within the bucket) of a source's edges of this sub-chunk
    unsigned tab[kLocalWaves][kBucketIds / 2];      // per wavefront and source: count, then offset (16 bits each); while
                                                    // a large bucket is counted: edges elsewhere / before, per source
};

// This wavefront's run of the sub-chunk [c0, c1) of a bucket: seg consecutive edges per wavefront, a
// multiple of 64 and at most kSubRounds * 64.
__device__ __forceinline__ void wave_run(int c0, int c1, int w, int &s0, int &s1)
{
    const int len = c1 > c0 ? c1 - c0 : 0;
    const int seg = ((len + kLocalThreads - 1) / kLocalThreads) * kWave;
    s0 = c0 + w * seg < c1 ? c0 + w * seg : c1;
    s1 = s0 + seg < c1 ? s0 + seg : c1;
}

// The source ids of this lane's edges in the rounds of the run [s0, s1), as loaded: the loads carry
// no branch of their own (past the end they re-read the last edge; an empty run reads nothing), so all
// of them are in flight at once, and nothing here waits for them.
__device__ __forceinline__ void load_run(const int32_t *keys, int s0, int s1, int32_t (&raw)[kSubRounds])
{
    const int lane = threadIdx.x & (kWave - 1);
#pragma unroll
    for (int u = 0; u < kSubRounds; ++u) raw[u] = 0;
    if (s1 > s0) {   // same for the whole wavefront
#pragma unroll
        for (int u = 0; u < kSubRounds; ++u) {
            const int i = s0 + u * kWave + lane;
            raw[u] = keys[i < s1 ? i : s1 - 1];
        }
    }
}

// Edges per wavefront and source of the run (16-bit counts, two to a word), and the local source
// ids kk[] of the lane's edges (-1: no edge).  The table is zeroed while the loads are under way.
__device__ __forceinline__ void count_run(const int32_t (&raw)[kSubRounds], int s0, int s1, int32_t lo,
                                          int (&kk)[kSubRounds], LocalShared &M)
{
    const int t = threadIdx.x, lane = t & (kWave - 1), w = t / kWave;
    uint4 *z = reinterpret_cast<uint4 *>(&M.tab[0][0]);
#pragma unroll
    for (int k = 0; k < (int)(sizeof(M.tab) / sizeof(uint4)) / kLocalThreads; ++k)
        z[k * kLocalThreads + t] = make_uint4(0u, 0u, 0u, 0u);
    __syncthreads();
#pragma unroll
    for (int u = 0; u < kSubRounds; ++u) {
        kk[u] = s0 + u * kWave + lane < s1 ? (raw[u] - lo) & (kBucketIds - 1) : -1;
        if (kk[u] >= 0) atomicAdd(&M.tab[w][kk[u] >> 1], 1u << ((kk[u] & 1) * 16));
    }
    __syncthreads();
}

// Buckets with several sub-chunks, before they are finished: edges per source of every sub-chunk,
// so that each sub-chunk's workgroup can add up what the others hold.
__device__ __forceinline__ void bucket_count(const LocalArgs &L, int g, LocalShared &M)
{
    const int t = threadIdx.x, lane = t & (kWave - 1), w = t / kWave;
    if (g >= L.large_groups) return;
    const BucketOfGroup m = L.map[g];
    if (m.bucket < 0 || m.edges <= kSubChunk) return;   // same for every thread
    const int32_t lo = m.bucket * kBucketIds;
    const int c0 = m.sub * kSubChunk, c1 = c0 + kSubChunk < m.edges ? c0 + kSubChunk : m.edges;
    const int32_t *keys = L.keys + m.first_edge;
    int s0, s1;
    wave_run(c0, c1, w, s0, s1);
    int kk[kSubRounds];
    int32_t raw[kSubRounds];
    load_run(keys, s0, s1, raw);
    count_run(raw, s0, s1, lo, kk, M);
    unsigned run[kLocalWords] = {};   // two sources per word: no carry, a sub-chunk has < 65 536 edges
#pragma unroll
    for (int k = 0; k < kLocalWaves; ++k) {
#pragma unroll
        for (int i = 0; i < kLocalWords; ++i) run[i] += M.tab[k][kLocalWords * t + i];
    }
    unsigned *out = reinterpret_cast<unsigned *>(L.subcnt + (size_t)g * kBucketIds) + kLocalWords * t;
#pragma unroll
    for (int i = 0; i < kLocalWords; ++i) out[i] = run[i];
}

__device__ __forceinline__ void bucket_finish(const LocalArgs &L, int g, LocalShared &M, int *lds)
{
    const int t = threadIdx.x, lane = t & (kWave - 1), w = t / kWave;
    const BucketOfGroup m = L.map[g];
    if (m.bucket < 0) return;   // same for every thread
    const int d = m.bucket, sub = m.sub, nbk = m.edges;
    const int64_t B0 = m.first_edge;
    const int32_t lo = d * kBucketIds;
    const int c0 = sub * kSubChunk, c1 = c0 + kSubChunk < nbk ? c0 + kSubChunk : nbk;
    const int32_t *keys = L.keys + B0, *vals = L.vals + B0, *eids = L.perm ? L.eids + B0 : nullptr;
    // this wavefront's run of the sub-chunk: rounds of 64 consecutive edges, all loaded up front
    int s0, s1;
    wave_run(c0, c1, w, s0, s1);
    int kk[kSubRounds];
    int32_t vv[kSubRounds], raw[kSubRounds];
    load_run(keys, s0, s1, raw);
    if (s1 > s0) {   // in flight while the sub-chunk is counted
#pragma unroll
        for (int u = 0; u < kSubRounds; ++u) {
            const int i = s0 + u * kWave + lane;
            vv[u] = vals[i < s1 ? i : s1 - 1];
        }
    }
    int other[kLocalKeys] = {}, before[kLocalKeys] = {};
    if (nbk > kSubChunk && g < L.large_groups) {   // edges of the bucket's other sub-chunks, per source
        const int nsub = (nbk + kSubChunk - 1) / kSubChunk;
        const unsigned *c = reinterpret_cast<const unsigned *>(L.subcnt + (size_t)(g - sub) * kBucketIds) + kLocalWords * t;
#pragma unroll 4
        for (int j = 0; j < nsub; ++j) {
            unsigned v[kLocalWords];
#pragma unroll
            for (int i = 0; i < kLocalWords; ++i) v[i] = c[(size_t)j * (kBucketIds / 2) + i];
#pragma unroll
            for (int k = 0; k < kLocalKeys; ++k) {
                const int x = (int)((v[k >> 1] >> ((k & 1) * 16)) & 0xFFFFu);
                if (j != sub) other[k] += x;
                if (j < sub) before[k] += x;
            }
        }
    }
    count_run(raw, s0, s1, lo, kk, M);
    // column scan over the wavefronts, both halves of a word at once (no carry: len < 65 536); the
    // totals are the sub-chunk's edges of this thread's sources
    unsigned run[kLocalWords] = {};
#pragma unroll
    for (int k = 0; k < kLocalWaves; ++k) {
#pragma unroll
        for (int i = 0; i < kLocalWords; ++i) {
            unsigned *q = &M.tab[k][kLocalWords * t + i];
            const unsigned v = *q;
            *q = run[i];
            run[i] += v;
        }
    }
    int cnt[kLocalKeys], all = 0;
#pragma unroll
    for (int k = 0; k < kLocalKeys; ++k) {
        cnt[k] = (int)((run[k >> 1] >> ((k & 1) * 16)) & 0xFFFFu) + other[k];
        all += cnt[k];
    }
    int dummy;
    int e0[kLocalKeys];
    e0[0] = block_excl_scan(all, &dummy, lds);
#pragma unroll
    for (int k = 1; k < kLocalKeys; ++k) e0[k] = e0[k - 1] + cnt[k - 1];
#pragma unroll
    for (int k = 0; k < kLocalKeys; ++k) M.start[kLocalKeys * t + k] = e0[k] + before[k];
    __syncthreads();
    // place: rank the 64 edges of a round among each other, add what this wavefront placed of the
    // source in earlier rounds and what earlier wavefronts hold
#pragma unroll
    for (int u = 0; u < kSubRounds; ++u) {
        if (s0 + u * kWave >= s1) break;   // same for the whole wavefront
        const bool ok = kk[u] >= 0;
        const int k = ok ? kk[u] : 0;
        unsigned mlo, mhi;
        match_lanes<kBucketBits>(k, ok, mlo, mhi);
        const int lower = lanes_below(mlo, mhi);
        const int sh = (k & 1) * 16;
        const int prior = (int)((M.tab[w][k >> 1] >> sh) & 0xFFFFu);
        // the LDS read above is issued before this update by the same wavefront
        if (ok && lower == 0) atomicAdd(&M.tab[w][k >> 1], (unsigned)(__popc(mlo) + __popc(mhi)) << sh);
        const int64_t pos = B0 + M.start[k] + prior + lower;
        const bool put = ok && pos >= 0 && pos < L.n;
        if (put) L.indices_T[pos] = vv[u];
        vv[u] = put ? (int32_t)pos : -1;   // the edge's place, for its id below
    }
    if (L.perm) {   // the edge ids go to the same places
        int32_t ee[kSubRounds];
#pragma unroll
        for (int u = 0; u < kSubRounds; ++u) {
            if (kk[u] < 0) vv[u] = -1;   // rounds past the end of the run were not placed
            const int i = s0 + u * kWave + lane;
            ee[u] = s1 > s0 ? eids[i < s1 ? i : s1 - 1] : 0;   // no branch per load: they all go out together
        }
#pragma unroll
        for (int u = 0; u < kSubRounds; ++u)
            if (vv[u] >= 0) L.perm[vv[u]] = ee[u];
    }
    if (sub == 0) {   // the bucket's rows
        int nl = 0, nc = 0;
#pragma unroll
        for (int k = 0; k < kLocalKeys; ++k) {
            const int64_t r = (int64_t)lo + kLocalKeys * t + k;
            const bool valid = r < L.num_src;
            if (valid) L.indptr_T[r] = (int32_t)(B0 + e0[k]);
            row_emit(L.rows, r, valid, (int)(B0 + e0[k]), cnt[k], nl, nc);
        }
        if (d == L.nbuckets - 1 && t == 0) L.indptr_T[L.num_src] = (int32_t)L.n;
        block_sum2(nl, nc, lds);
        if (t == 0) {
            L.rows.counts[2 * d] = nl;
            L.rows.counts[2 * d + 1] = nc;
        }
    }
}

// indptr_T from the sorted source ids: position k starts every source id in
// (key[k-1], key[k]].  k == n closes the tail.  Gaps (sources without edges) are
// short in practice; a long one is filled by the whole wavefront together.
struct StartsArgs {
    const int32_t *keys;     // [n] sorted source ids
    int64_t n, num_src;
    int32_t *indptr_T;       // [num_src+1]
    int nb;
};

__device__ __forceinline__ void row_starts(const StartsArgs &A, int b)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t n = A.n;
    for (int64_t base = (int64_t)b * blockDim.x; base <= n; base += (int64_t)A.nb * blockDim.x) {
        const int64_t k = base + threadIdx.x;
        int64_t prev = 0, cur = -1;   // empty interval by default
        if (k <= n) {
            prev = k > 0 ? A.keys[k - 1] : -1;
            cur = k < n ? A.keys[k] : A.num_src;
        }
        const bool big = cur - prev > 4;
        if (!big)
            for (int64_t v = prev + 1; v <= cur; ++v) A.indptr_T[v] = (int32_t)k;
        unsigned long long m = __ballot(big);
        while (m) {
            const int leader = __ffsll((long long)m) - 1;
            const int64_t p = __shfl(prev, leader, kWave), c = __shfl(cur, leader, kWave);
            const int64_t kk = __shfl(k, leader, kWave);
            for (int64_t v = p + 1 + lane; v <= c; v += kWave) A.indptr_T[v] = (int32_t)kk;
            m &= m - 1;
        }
    }
}

// ------------------------------------------------------- the stage kernel ----
enum {
    JOB_ROWS_COUNT = 0, JOB_ROWS_FILL = 1, JOB_SORT_HIST = 2, JOB_SORT_SCATTER = 3, JOB_ROW_STARTS = 4,
    JOB_COL_SCAN = 5
};
constexpr int kMaxJobs = 16;

struct Job {
    int kind, nblocks;
    union {
        RowsArgs rows;
        SortArgs sort;
        StartsArgs starts;
        ColScanArgs cols;
    };
};

struct StageArgs {
    int njobs;
    int first[kMaxJobs + 1];   // first workgroup of each job
    Job job[kMaxJobs];
};

// LDS a job's workgroups use (the launch reserves the largest of its jobs).
static size_t job_lds_bytes(const Job &j)
{
    switch (j.kind) {
        case JOB_SORT_HIST: return sizeof(int) << j.sort.bits;
        case JOB_SORT_SCATTER:
            if (!j.sort.tot) return sizeof(SortShared<kRadixBits, kSortThreads>);
            return j.sort.bits == kRadixBits ? sizeof(SortShared<kRadixBits, kSplitThreads>)
                                             : sizeof(SortShared<10, kSplitThreads>);
        case JOB_COL_SCAN: return sizeof(int) * kSortWaves * kWave;
        default: return 0;
    }
}
constexpr size_t kMaxSplitLds = sizeof(SortShared<10, kSplitThreads>);

template <int BITS, int NT>
__device__ __forceinline__ void sort_scatter_any(const SortArgs &S, int b, unsigned char *dyn, int *lds)
{
    SortShared<BITS, NT> &M = *reinterpret_cast<SortShared<BITS, NT> *>(dyn);
    if (S.items == 1) sort_scatter<1, BITS, NT>(S, b, M, lds);
    else if (S.items == 2) sort_scatter<2, BITS, NT>(S, b, M, lds);
    else sort_scatter<4, BITS, NT>(S, b, M, lds);
}

// SCATTER: the launch holds passes of the LSD radix sort.  Their registers would otherwise cap
// every stage at one 1024-thread workgroup per compute unit; the light variant runs two.
template <bool SCATTER>
__global__ __launch_bounds__(kSortThreads, SCATTER ? 4 : 8) void k_plan_stage(StageArgs A)
{
    extern __shared__ __align__(16) unsigned char dyn[];
    __shared__ int lds[32];
    int j = 0;
    while (j + 1 < A.njobs && (int)blockIdx.x >= A.first[j + 1]) ++j;
    const int b = blockIdx.x - A.first[j];
    const Job &J = A.job[j];
    switch (J.kind) {
        case JOB_ROWS_COUNT: rows_count(J.rows, b, lds); break;
        case JOB_ROWS_FILL: rows_fill(J.rows, b, lds); break;
        case JOB_SORT_HIST: sort_hist(J.sort, b, reinterpret_cast<int *>(dyn)); break;
        case JOB_SORT_SCATTER:
            if constexpr (SCATTER) sort_scatter_any<kRadixBits, kSortThreads>(J.sort, b, dyn, lds);
            break;
        case JOB_COL_SCAN: col_scan(J.cols, b, reinterpret_cast<int *>(dyn)); break;
        default: row_starts(J.starts, b); break;
    }
}

// The split into buckets of every bucketed transpose of a stage (jobs of kind JOB_SORT_SCATTER
// with a bucket total array).
__global__ __launch_bounds__(kSplitThreads) void k_plan_split(StageArgs A)
{
    extern __shared__ __align__(16) unsigned char dyn[];
    __shared__ int lds[32];
    int j = 0;
    while (j + 1 < A.njobs && (int)blockIdx.x >= A.first[j + 1]) ++j;
    const int b = blockIdx.x - A.first[j];
    const SortArgs &S = A.job[j].sort;
    if (S.bits == kRadixBits) sort_scatter_any<kRadixBits, kSplitThreads>(S, b, dyn, lds);
    else sort_scatter_any<10, kSplitThreads>(S, b, dyn, lds);
}

// The buckets of every bucketed transpose of a stage: smaller workgroups than k_plan_stage's, three
// to a compute unit, so that (nearly) all buckets of a mini-batch are in flight at once.
struct BucketStageArgs {
    int njobs;
    int first[kMaxJobs + 1];
    LocalArgs job[kMaxJobs];
};

__global__ __launch_bounds__(kLocalThreads, 6) void k_plan_bucket_counts(BucketStageArgs A)
{
    __shared__ LocalShared M;
    int j = 0;
    while (j + 1 < A.njobs && (int)blockIdx.x >= A.first[j + 1]) ++j;
    bucket_count(A.job[j], blockIdx.x - A.first[j], M);
}

__global__ __launch_bounds__(kLocalThreads, 6) void k_plan_buckets(BucketStageArgs A)
{
    __shared__ LocalShared M;
    __shared__ int lds[32];
    int j = 0;
    while (j + 1 < A.njobs && (int)blockIdx.x >= A.first[j + 1]) ++j;
    bucket_finish(A.job[j], blockIdx.x - A.first[j], M, lds);
}

// --------------------------------------- forward-only GCN: out-degree histogram ----
__global__ __launch_bounds__(kBlock) void k_fill_i32(int32_t *p, int64_t n, int32_t v)
{
    for (int64_t i = blockIdx.x * (int64_t)kBlock + threadIdx.x; i < n; i += (int64_t)gridDim.x * kBlock)
        p[i] = v;
}

__global__ __launch_bounds__(kBlock) void k_hist(const int32_t *__restrict__ idx, int64_t n,
                                                 int32_t *__restrict__ cnt)
{
    for (int64_t i = blockIdx.x * (int64_t)kBlock + threadIdx.x; i < n; i += (int64_t)gridDim.x * kBlock)
        atomicAdd(&cnt[idx[i]], 1);
}

__global__ __launch_bounds__(kBlock) void k_rsqrt_deg(const int32_t *__restrict__ deg, int64_t n,
                                                      float *__restrict__ rsq)
{
    for (int64_t i = blockIdx.x * (int64_t)kBlock + threadIdx.x; i < n; i += (int64_t)gridDim.x * kBlock) {
        int d = deg[i];
        rsq[i] = (float)(1.0 / sqrt((double)(d < 1 ? 1 : d)));
    }
}

// -------------------------------------------------------------- validate ----
__global__ __launch_bounds__(kBlock) void k_validate(const int32_t *__restrict__ indptr,
                                                     const int32_t *__restrict__ indices, int64_t num_dst,
                                                     int64_t num_src, int64_t num_edges,
                                                     unsigned long long *bad)
{
    int64_t gid = blockIdx.x * (int64_t)kBlock + threadIdx.x, stride = (int64_t)gridDim.x * kBlock;
    unsigned long long c = 0;
    if (gid == 0) {
        if (indptr[0] != 0) ++c;
        if ((int64_t)indptr[num_dst] != num_edges) ++c;
    }
    for (int64_t r = gid; r < num_dst; r += stride)
        if (indptr[r + 1] < indptr[r]) ++c;
    for (int64_t e = gid; e < num_edges; e += stride) {
        int32_t v = indices[e];
        if (v < 0 || (int64_t)v >= num_src) ++c;
    }
    if (c) atomicAdd(bad, c);
}

// ------------------------------------------------------------- host side ----
static int grid_for(int64_t n, int per_thread)
{
    int64_t g = ceil_div(n, (int64_t)kBlock * per_thread);
    if (g < 1) g = 1;
    if (g > 4096) g = 4096;
    return (int)g;
}

static RowsArgs rows_args(const int32_t *rowptr, int64_t n, int32_t *len_out, float *inv, float *rsq,
                          int32_t *counts, int32_t *long_rows, int32_t *chunk_ptr, int32_t *totals,
                          int32_t *edge_row, int32_t *split, int64_t nnz)
{
    RowsArgs A;
    int64_t b = ceil_div(n, (int64_t)kSortThreads * 2);   // two rows per thread while that gives at most kMaxScanBlocks blocks
    if (b < 1) b = 1;
    if (b > kMaxScanBlocks) b = kMaxScanBlocks;
    A.rowptr = rowptr; A.n = n; A.nb = (int)b;
    A.per = n > 0 ? ceil_div(n, b) : 1;
    A.len_out = len_out; A.inv = inv; A.rsq = rsq;
    A.counts = counts; A.long_rows = long_rows; A.chunk_ptr = chunk_ptr; A.totals = totals;
    A.edge_row = edge_row;
    A.split = split;
    A.nsets = num_row_sets(n, nnz);
    return A;
}

// How the edges of a transpose are cut into workgroups, and which transpose is taken.
struct SortGeom {
    int items;        // keys per thread and step
    int64_t per;      // keys per workgroup (a multiple of the step)
    int nb;           // workgroups
    bool bucketed;    // bucketed transpose (else LSD radix sort)
    int nbuckets;     // bucketed: buckets of kBucketIds source ids
    int bits;         // bucketed: digit width of the split
};

// keys_per_group: 0, or how many keys a workgroup should take at least (plans built together share
// the compute units: see plans_build); the count table is laid out for keys_per_group == 0.
static SortGeom sort_geom(int64_t num_src, int64_t n, int64_t keys_per_group = 0)
{
    SortGeom g;
    g.bucketed = num_src <= (int64_t)kMaxBuckets * kBucketIds;
    const int threads = g.bucketed ? kSplitThreads : kSortThreads, most = g.bucketed ? kMaxSplitBlocks : kMaxSortBlocks;
    // one step per workgroup when the keys fit `most` workgroups x 4 keys per thread
    int64_t want = ceil_div(n, (int64_t)most);
    if (want < keys_per_group) want = keys_per_group;
    g.items = 1;
    while (g.items < kMaxSortItems && (int64_t)g.items * threads < want) g.items <<= 1;
    const int64_t step = (int64_t)g.items * threads;
    g.per = ceil_div(want, step) * step;
    if (g.per < step) g.per = step;
    g.nb = n > 0 ? (int)ceil_div(n, g.per) : 1;
    g.nbuckets = g.bucketed ? (int)(num_src > 0 ? ceil_div(num_src, (int64_t)kBucketIds) : 1) : 0;
    g.bits = g.nbuckets <= kRadixBins ? kRadixBits : 10;
    return g;
}

size_t plan_layout(fastgl_plan *p, void *base, int64_t num_dst, int64_t num_src, int64_t num_edges,
                   bool fwd_only)
{
    size_t off = 0;
    char *b = (char *)base;
    auto take = [&](size_t bytes) {
        char *q = b ? b + off : nullptr;
        off += align_up(bytes ? bytes : 4, 256);
        return (void *)q;
    };
    // arrays that only the transpose (a backward plan) needs take no room in a forward-only layout
    auto take_bwd = [&](size_t bytes) { return fwd_only ? nullptr : take(bytes); };
    const int64_t cl = cap_long_rows(num_edges);
    fastgl_plan tmp;
    fastgl_plan *q = p ? p : &tmp;
    q->din = (int32_t *)take(4 * (size_t)num_dst);
    q->dout = (int32_t *)take(4 * (size_t)num_src);
    q->indptr_T = (int32_t *)take_bwd(4 * ((size_t)num_src + 1));
    q->indices_T = (int32_t *)take_bwd(4 * (size_t)num_edges);
    q->perm = (int32_t *)take_bwd(4 * (size_t)num_edges);
    q->dst_inv = (float *)take(4 * (size_t)num_dst);
    q->dst_rsqrt = (float *)take(4 * (size_t)num_dst);
    q->src_rsqrt = (float *)take(4 * (size_t)num_src);
    q->long_dst = (int32_t *)take(4 * (size_t)cl);
    q->chunk_ptr_dst = (int32_t *)take(4 * ((size_t)cl + 1));
    q->long_src = (int32_t *)take_bwd(4 * (size_t)cl);
    q->chunk_ptr_src = (int32_t *)take_bwd(4 * ((size_t)cl + 1));
    q->split_dst = (int32_t *)take(4 * ((size_t)num_row_sets(num_dst, num_edges) + 1));
    q->split_src = (int32_t *)take_bwd(4 * ((size_t)num_row_sets(num_src, num_edges) + 1));
    q->counters = (int32_t *)take(4 * 4);
    const SortGeom sg = sort_geom(num_src, num_edges);
    // the split into buckets writes one set of (source id, destination row, edge id); the radix sort ping-pongs two
    for (int i = 0; i < 6; ++i)
        q->sort_buf[i] = i < 3 || !sg.bucketed ? (int32_t *)take_bwd(4 * (size_t)num_edges) : nullptr;
    q->edge_dst = (int32_t *)take_bwd(4 * (size_t)num_edges);
    q->radix_cnt = (int32_t *)take_bwd(4 * (size_t)sg.nb * (sg.bucketed ? sg.nbuckets : kRadixBins));
    q->bucket_tot = (int32_t *)take_bwd(4 * (size_t)kMaxBuckets);
    q->bucket_map = take_bwd(sg.bucketed ? sizeof(BucketOfGroup) * (size_t)bucket_groups(sg.nbuckets, num_edges) : 0);
    q->bucket_subcnt = take_bwd(sg.bucketed ? sizeof(uint16_t) * kBucketIds * (size_t)large_bucket_groups(num_edges) : 0);
    q->block_sums = (int32_t *)take(4 * 2 * (size_t)kMaxScanBlocks);
    q->block_sums2 = (int32_t *)take_bwd(4 * 2 * (size_t)kMaxScanBlocks);
    return off;
}

// ---- stages ----------------------------------------------------------------
struct BucketJob {
    LocalArgs args;
    int nblocks;
};
struct Stage {
    std::vector<Job> jobs;            // workgroups of k_plan_stage
    std::vector<Job> splits;          // workgroups of k_plan_split
    std::vector<BucketJob> buckets;   // workgroups of k_plan_buckets
};
using Stages = std::vector<Stage>;

static void add_job(Stages &st, size_t k, const Job &j)
{
    if (st.size() <= k) st.resize(k + 1);
    st[k].jobs.push_back(j);
}

static void add_split(Stages &st, size_t k, const Job &j)
{
    if (st.size() <= k) st.resize(k + 1);
    st[k].splits.push_back(j);
}

static void add_buckets(Stages &st, size_t k, const BucketJob &j)
{
    if (st.size() <= k) st.resize(k + 1);
    st[k].buckets.push_back(j);
}

static Job rows_job(int kind, const RowsArgs &A)
{
    Job j;
    j.kind = kind; j.nblocks = A.nb; j.rows = A;
    return j;
}

// Append the jobs of one plan.  Stage k of a plan only depends on its own
// earlier stages, so plans of different depth can share launches.
static void plan_stages(fastgl_plan *p, int parts, Stages &st, int64_t keys_per_group)
{
    p->parts = parts;
    const bool full = (parts & FASTGL_PLAN_BWD) != 0;
    if (!full) parts &= ~FASTGL_PLAN_PERM;
    p->parts = parts;
    RowsArgs dstA = rows_args(p->indptr, p->num_dst, p->din, p->dst_inv, p->dst_rsqrt, p->block_sums,
                              p->long_dst, p->chunk_ptr_dst, p->counters, full ? p->edge_dst : nullptr,
                              p->split_dst, p->num_edges);
    add_job(st, 0, rows_job(JOB_ROWS_COUNT, dstA));
    add_job(st, 1, rows_job(JOB_ROWS_FILL, dstA));
    if (!full) return;

    const int64_t n = p->num_edges;
    const bool want_perm = (parts & FASTGL_PLAN_PERM) != 0;
    const SortGeom sg = sort_geom(p->num_src, n, keys_per_group);
    SortArgs S;
    S.n = n;
    S.items = sg.items;
    S.per = sg.per;
    S.nb = sg.nb;
    S.cnt = p->radix_cnt;
    RowsArgs srcA = rows_args(p->indptr_T, p->num_src, p->dout, nullptr, p->src_rsqrt, p->block_sums2,
                              p->long_src, p->chunk_ptr_src, p->counters + 2, nullptr, p->split_src,
                              p->num_edges);
    if (sg.bucketed) {
        S.keys_in = p->indices; S.vals_in = p->edge_dst; S.eid_in = nullptr;
        S.keys_out = p->sort_buf[0]; S.vals_out = p->sort_buf[1];
        S.eid_out = want_perm ? p->sort_buf[2] : nullptr;
        S.shift = kBucketBits; S.bits = sg.bits; S.nbins = sg.nbuckets;
        S.tot = p->bucket_tot;
        S.map = reinterpret_cast<BucketOfGroup *>(p->bucket_map);
        S.map_cap = (int)bucket_groups(sg.nbuckets, n);
        Job j;
        j.nblocks = S.nb; j.sort = S;
        j.kind = JOB_SORT_HIST;
        add_job(st, 0, j);
        j.kind = JOB_SORT_SCATTER;
        add_split(st, 2, j);
        Job c;
        c.kind = JOB_COL_SCAN;
        c.cols.cnt = p->radix_cnt; c.cols.tot = p->bucket_tot; c.cols.nb = S.nb; c.cols.nbins = sg.nbuckets;
        c.nblocks = (int)ceil_div(sg.nbuckets, kWave);
        add_job(st, 1, c);
        // the source-side row pass runs per bucket; the fill pass then sees buckets as its blocks
        srcA.per = kBucketIds;
        srcA.nb = sg.nbuckets;
        BucketJob f;
        f.args.keys = S.keys_out; f.args.vals = S.vals_out; f.args.eids = S.eid_out;
        f.args.map = reinterpret_cast<const BucketOfGroup *>(p->bucket_map); f.args.nbuckets = sg.nbuckets;
        f.args.subcnt = reinterpret_cast<uint16_t *>(p->bucket_subcnt);
        // no more than the map holds: workgroups past the map's end must not read it
        f.args.large_groups = (int)(large_bucket_groups(n) < bucket_groups(sg.nbuckets, n) ? large_bucket_groups(n)
                                                                                          : bucket_groups(sg.nbuckets, n));
        f.args.n = n; f.args.num_src = p->num_src;
        f.args.indptr_T = p->indptr_T; f.args.indices_T = p->indices_T;
        f.args.perm = want_perm ? p->perm : nullptr;
        f.args.rows = srcA;
        f.nblocks = (int)bucket_groups(sg.nbuckets, n);
        add_buckets(st, 3, f);
        add_job(st, 4, rows_job(JOB_ROWS_FILL, srcA));
        return;
    }

    int bits = 1;
    while (bits < 31 && ((int64_t)1 << bits) < p->num_src) ++bits;
    const int npass = (bits + kRadixBits - 1) / kRadixBits;
    S.bits = kRadixBits; S.nbins = kRadixBins; S.tot = nullptr; S.map = nullptr; S.map_cap = 0;
    const int32_t *kin = p->indices, *vin = p->edge_dst, *ein = nullptr;
    for (int pass = 0; pass < npass; ++pass) {
        const bool last = pass == npass - 1;
        S.keys_in = kin; S.vals_in = vin; S.eid_in = ein; S.shift = pass * kRadixBits;
        S.keys_out = p->sort_buf[(pass & 1) * 3];
        S.vals_out = last ? p->indices_T : p->sort_buf[(pass & 1) * 3 + 1];
        S.eid_out = !want_perm ? nullptr : last ? p->perm : p->sort_buf[(pass & 1) * 3 + 2];
        Job j;
        j.nblocks = S.nb; j.sort = S;
        j.kind = JOB_SORT_HIST;
        add_job(st, 2 * pass, j);
        j.kind = JOB_SORT_SCATTER;
        add_job(st, 2 * pass + 1, j);
        kin = S.keys_out;
        vin = S.vals_out;
        ein = S.eid_out;
    }
    Job t;
    t.kind = JOB_ROW_STARTS;
    t.starts.keys = kin; t.starts.n = n; t.starts.num_src = p->num_src; t.starts.indptr_T = p->indptr_T;
    int64_t nb = ceil_div(n + 1, (int64_t)kSortThreads);
    if (nb > 1024) nb = 1024;
    t.starts.nb = (int)nb; t.nblocks = (int)nb;
    add_job(st, 2 * npass, t);
    add_job(st, 2 * npass + 1, rows_job(JOB_ROWS_COUNT, srcA));
    add_job(st, 2 * npass + 2, rows_job(JOB_ROWS_FILL, srcA));
}

static fastgl_status run_stages(const Stages &st, hipStream_t s)
{
    static_assert(sizeof(StageArgs) <= 4096 && sizeof(BucketStageArgs) <= 4096, "kernel arguments are passed by value");
    static bool raised = false;   // benign if two threads both do it
    if (!raised) {   // the scatter kernels take more LDS than a launch gets by default
        FASTGL_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_plan_stage<true>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)sizeof(SortShared<kRadixBits, kSortThreads>)));
        FASTGL_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_plan_split),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)kMaxSplitLds));
        raised = true;
    }
    for (const Stage &stage : st) {
        const auto &jobs = stage.jobs;
        for (size_t at = 0; at < jobs.size(); at += kMaxJobs) {
            StageArgs A;
            A.njobs = (int)(jobs.size() - at < (size_t)kMaxJobs ? jobs.size() - at : kMaxJobs);
            int blocks = 0;
            size_t lds = 0;
            for (int i = 0; i < A.njobs; ++i) {
                A.first[i] = blocks;
                A.job[i] = jobs[at + i];
                blocks += A.job[i].nblocks;
                const size_t need = job_lds_bytes(A.job[i]);
                if (need > lds) lds = need;
            }
            A.first[A.njobs] = blocks;
            bool scatter = false;
            for (int i = 0; i < A.njobs; ++i) scatter = scatter || A.job[i].kind == JOB_SORT_SCATTER;
            if (scatter) hipLaunchKernelGGL(k_plan_stage<true>, dim3(blocks), dim3(kSortThreads), lds, s, A);
            else hipLaunchKernelGGL(k_plan_stage<false>, dim3(blocks), dim3(kSortThreads), lds, s, A);
            FASTGL_LAUNCH_CHECK("k_plan_stage");
        }
        const auto &sp = stage.splits;
        for (size_t at = 0; at < sp.size(); at += kMaxJobs) {
            StageArgs A;
            A.njobs = (int)(sp.size() - at < (size_t)kMaxJobs ? sp.size() - at : kMaxJobs);
            int blocks = 0;
            size_t lds = 0;
            for (int i = 0; i < A.njobs; ++i) {
                A.first[i] = blocks;
                A.job[i] = sp[at + i];
                blocks += A.job[i].nblocks;
                const size_t need = job_lds_bytes(A.job[i]);
                if (need > lds) lds = need;
            }
            A.first[A.njobs] = blocks;
            hipLaunchKernelGGL(k_plan_split, dim3(blocks), dim3(kSplitThreads), lds, s, A);
            FASTGL_LAUNCH_CHECK("k_plan_split");
        }
        const auto &bk = stage.buckets;
        for (size_t at = 0; at < bk.size(); at += kMaxJobs) {
            BucketStageArgs A;
            A.njobs = (int)(bk.size() - at < (size_t)kMaxJobs ? bk.size() - at : kMaxJobs);
            int blocks = 0;   // first the per-source counts of the sub-chunks of large buckets (if there can be any)
            for (int i = 0; i < A.njobs; ++i) {
                A.first[i] = blocks;
                A.job[i] = bk[at + i].args;
                blocks += A.job[i].large_groups;
            }
            A.first[A.njobs] = blocks;
            if (blocks > 0) {
                hipLaunchKernelGGL(k_plan_bucket_counts, dim3(blocks), dim3(kLocalThreads), 0, s, A);
                FASTGL_LAUNCH_CHECK("k_plan_bucket_counts");
            }
            blocks = 0;
            for (int i = 0; i < A.njobs; ++i) {
                A.first[i] = blocks;
                blocks += bk[at + i].nblocks;
            }
            A.first[A.njobs] = blocks;
            hipLaunchKernelGGL(k_plan_buckets, dim3(blocks), dim3(kLocalThreads), 0, s, A);
            FASTGL_LAUNCH_CHECK("k_plan_buckets");
        }
    }
    return FASTGL_OK;
}

// Out-degrees by histogram for a forward-only plan of a GCN-normalised pass.
static fastgl_status src_degrees(fastgl_plan *p, hipStream_t s)
{
    p->parts |= FASTGL_PLAN_SRC_DEG;
    hipLaunchKernelGGL(k_fill_i32, dim3(grid_for(p->num_src, 4)), dim3(kBlock), 0, s, p->dout, p->num_src, 0);
    FASTGL_LAUNCH_CHECK("k_fill_i32");
    hipLaunchKernelGGL(k_hist, dim3(grid_for(p->num_edges, 4)), dim3(kBlock), 0, s, p->indices, p->num_edges,
                       p->dout);
    FASTGL_LAUNCH_CHECK("k_hist");
    hipLaunchKernelGGL(k_rsqrt_deg, dim3(grid_for(p->num_src, 4)), dim3(kBlock), 0, s, p->dout, p->num_src,
                       p->src_rsqrt);
    FASTGL_LAUNCH_CHECK("k_rsqrt_deg");
    return FASTGL_OK;
}

// Enqueue the bookkeeping of n plans; stage k of all of them shares a launch.
// parts[i]: FASTGL_PLAN_FWD or FASTGL_PLAN_ALL; src_deg[i] asks a forward-only
// plan for dout / src_rsqrt as well (GCN).
fastgl_status plans_build(fastgl_plan *const *plans, const int *parts, const bool *src_deg, int n, hipStream_t s)
{
    // The split of the edges runs two 512-thread workgroups per compute unit: the transposes of a
    // call share the (256) compute units, each workgroup taking about the same number of edges.
    int64_t edges = 0;
    for (int i = 0; i < n; ++i)
        if (parts[i] & FASTGL_PLAN_BWD) edges += plans[i]->num_edges;
    const int64_t keys_per_group = ceil_div(edges, (int64_t)kMaxSplitBlocks);
    Stages st;
    for (int i = 0; i < n; ++i) plan_stages(plans[i], parts[i], st, keys_per_group);
    fastgl_status rc = run_stages(st, s);
    if (rc != FASTGL_OK) return rc;
    for (int i = 0; i < n; ++i)
        if (src_deg[i] && !(parts[i] & FASTGL_PLAN_BWD)) {
            rc = src_degrees(plans[i], s);
            if (rc != FASTGL_OK) return rc;
        }
    return FASTGL_OK;
}

fastgl_status plan_build(fastgl_plan *p, int parts, bool need_src_degrees, hipStream_t s)
{
    return plans_build(&p, &parts, &need_src_degrees, 1, s);
}

fastgl_status validate_block(const int32_t *indptr, const int32_t *indices, int64_t num_dst,
                             int64_t num_src, int64_t num_edges, void *scratch, int64_t *n_violations,
                             hipStream_t s)
{
    unsigned long long *bad = (unsigned long long *)scratch;
    hipLaunchKernelGGL(k_fill_i32, dim3(1), dim3(kBlock), 0, s, (int32_t *)scratch, (int64_t)2, 0);
    FASTGL_LAUNCH_CHECK("k_fill_i32");
    int64_t m = num_dst > num_edges ? num_dst : num_edges;
    hipLaunchKernelGGL(k_validate, dim3(grid_for(m, 4)), dim3(kBlock), 0, s, indptr, indices, num_dst,
                       num_src, num_edges, bad);
    FASTGL_LAUNCH_CHECK("k_validate");
    unsigned long long host = 0;
    FASTGL_HIP(hipMemcpyAsync(&host, bad, sizeof(host), hipMemcpyDeviceToHost, s));
    FASTGL_HIP(hipStreamSynchronize(s));
    *n_violations = (int64_t)host;
    return FASTGL_OK;
}

}  // namespace fastgl
