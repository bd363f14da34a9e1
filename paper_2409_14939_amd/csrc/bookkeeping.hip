// Per-block integer bookkeeping on the GPU: degrees, scale factors, a stable
// transpose of the CSR (LSD radix sort of the edges by source id), equal-work row
// sets and degree buckets (ordered compaction of long rows).  Everything is integer work with
// a single valid answer: no float atomics, no order-dependent results, and (on
// the full-plan path) no global atomics at all.
//
// Why it exists: the backward pass (paper Section 4.2, Eq. 5) gathers along
// the reversed edges; pulling along a transposed CSR keeps one writer per
// output row, as the forward pass has (Section 4.2: a target's aggregation is
// completed by one owner).  Every sampled block is new, so this work is part of
// each iteration and is kept to a handful of launches.  The work of a plan is a
// sequence of STAGES; stage k of every plan built in one call shares one launch
// of k_plan_stage, whose workgroups look up which job they belong to:
//
//   stage 0        digit histogram of pass 0    + destination-side row pass (degrees,
//                  scale factors, edge -> row expansion, equal-work split, bucket counts)
//   stage 1        stable scatter of pass 0     + destination-side bucket fill
//   stage 2p,2p+1  histogram / scatter of radix pass p (8-bit digits)
//   then           row starts (indptr_T from the sorted keys),
//                  source-side row pass, source-side bucket fill
//
// A full plan with a 3-pass sort is 9 launches, and so are the plans of all
// layers of a mini-batch when they are built together.
#include <vector>

#include "internal.h"

namespace fastgl {

constexpr int kSortThreads = 1024;                   // 16 wavefronts per sort workgroup
constexpr int kSortWaves = kSortThreads / kWave;
constexpr int kMaxSortItems = 4;                     // keys per thread and step: 1, 2 or 4
constexpr int kMaxSortBlocks = 256;

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

__device__ __forceinline__ int block_sum(int v, int *lds)
{
    int tot;
    block_excl_scan(v, &tot, lds);
    return tot;
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
            if (A.len_out) A.len_out[r] = len;
            double d = (double)(len < 1 ? 1 : len);
            if (A.inv) A.inv[r] = (float)(1.0 / d);
            if (A.rsq) A.rsq[r] = (float)(1.0 / sqrt(d));
            if (len > kLongThreshold) {
                nl += 1;
                nc += (len + kLongChunk - 1) / kLongChunk;
            }
        }
        if (A.edge_row) {
            const bool big = len > kWave;
            if (!big)
                for (int k = 0; k < len; ++k) A.edge_row[e0 + k] = (int32_t)r;
            unsigned long long m = __ballot(big);
            while (m) {
                const int leader = __ffsll((long long)m) - 1;
                const int le0 = __shfl(e0, leader, kWave), ll = __shfl(len, leader, kWave);
                const int lr = (int)(base - beg) + (threadIdx.x - lane) + leader;   // row offset in block
                for (int k = lane; k < ll; k += kWave) A.edge_row[le0 + k] = (int32_t)(beg + lr);
                m &= m - 1;
            }
        }
        if (A.split) {
            // Equal-work row sets: set g starts at the first row whose work prefix
            // W[r] = rowptr[r] + r reaches g * kWorkPerGroup.  Row r+1 is that row for
            // every g in (W[r]/work, W[r+1]/work]; the thread of row r writes them.
            int64_t g0 = 1, g1 = 0;   // empty
            if (r < end) {
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
    nl = block_sum(nl, lds);
    nc = block_sum(nc, lds);
    if (threadIdx.x == 0) {
        A.counts[2 * b] = nl;
        A.counts[2 * b + 1] = nc;
    }
}

// Pass 2: ordered compaction.  long_rows ascending; chunk_ptr[i] = first chunk of
// the i-th long row; totals[0] = number of long rows, totals[1] = number of chunks.
__device__ __forceinline__ void rows_fill(const RowsArgs &A, int b, int *lds)
{
    int pl = 0, pc = 0;
    for (int i = threadIdx.x; i < A.nb; i += blockDim.x) {
        if (i < b) {
            pl += A.counts[2 * i];
            pc += A.counts[2 * i + 1];
        }
    }
    int cl = block_sum(pl, lds);
    int cc = block_sum(pc, lds);
    int64_t beg = b * A.per, end = beg + A.per < A.n ? beg + A.per : A.n;
    const bool any = A.counts[2 * b] != 0;      // block-uniform: most blocks have no long row
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

// ------------------------------------------------------------ radix sort ----
struct SortArgs {
    const int32_t *keys_in, *vals_in;   // vals: the destination row of the edge
    int32_t *keys_out, *vals_out;       // keys_out == NULL: not needed (never on this path: row starts read them)
    const int32_t *eid_in;              // second payload, the original edge id; NULL on the first pass = identity
    int32_t *eid_out;                   // NULL: the plan carries no edge permutation
    int64_t n, per;                     // block b owns keys [b*per, min(n,(b+1)*per))
    int nb, shift;
    int32_t *cnt;                       // [nb][256] digit counts per block
    int items;                          // keys per thread and step: 1, 2 or 4
};

// Digit histogram of the block's key range.
__device__ __forceinline__ void sort_hist(const SortArgs &S, int b, int *h)
{
    if (threadIdx.x < kRadixBins) h[threadIdx.x] = 0;
    __syncthreads();
    const int64_t beg = b * S.per, end = beg + S.per < S.n ? beg + S.per : S.n;
    for (int64_t i = beg + threadIdx.x; i < end; i += kSortThreads)
        atomicAdd(&h[(S.keys_in[i] >> S.shift) & (kRadixBins - 1)], 1);
    __syncthreads();
    if (threadIdx.x < kRadixBins) S.cnt[(int64_t)b * kRadixBins + threadIdx.x] = h[threadIdx.x];
}

// Stable scatter of one digit.  Every workgroup derives its own output offsets
// from the [nb][256] count table (no separate scan launch): for digit d,
//   base = sum_{d' < d} total[d'] + sum_{b' < b} cnt[b'][d].
// Within a step of 1024*ITEMS keys each wavefront owns 64*ITEMS consecutive keys and ranks
// them 64 at a time: lanes with equal digits find each other with 8 ballots, the
// running per-wavefront digit counts live in LDS, and a column scan over the 16
// wavefronts plus a scan over the digits give each key its place in the step's
// sorted order.  The step is sorted into LDS first and written out from there.
// The payload is the edge's destination row and, if asked for, its original id.
struct SortShared {
    int running[kRadixBins], lbase[kRadixBins], gdelta[kRadixBins];
    int wcnt[kSortWaves][kRadixBins];
    int32_t skey[kSortThreads * kMaxSortItems], sval[kSortThreads * kMaxSortItems];
    int32_t seid[kSortThreads * kMaxSortItems];
};

template <int ITEMS>
__device__ __forceinline__ void sort_scatter(const SortArgs &S, int b, SortShared &M, int *lds)
{
    int (&running)[kRadixBins] = M.running, (&lbase)[kRadixBins] = M.lbase, (&gdelta)[kRadixBins] = M.gdelta;
    int (&wcnt)[kSortWaves][kRadixBins] = M.wcnt;
    int32_t *skey = M.skey, *sval = M.sval, *seid = M.seid;
    const bool EID = S.eid_out != nullptr;
    const int t = threadIdx.x, lane = t & (kWave - 1), w = t / kWave;
    {   // offsets of this block's digits
        const int d = t & (kRadixBins - 1), part = t / kRadixBins;   // 4 parts share the blocks
        int below = 0, total = 0;
        constexpr int kParts = kSortThreads / kRadixBins, kBatch = 16;
        for (int b0 = part; b0 < S.nb; b0 += kParts * kBatch) {
            int c[kBatch];
#pragma unroll
            for (int k = 0; k < kBatch; ++k) {   // independent loads first
                const int bb = b0 + k * kParts;
                c[k] = bb < S.nb ? S.cnt[(int64_t)bb * kRadixBins + d] : 0;
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
        if (t < kRadixBins) {
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                bel += wcnt[k][t];
                tot += wcnt[4 + k][t];
            }
        }
        int dummy;
        int ex = block_excl_scan(t < kRadixBins ? tot : 0, &dummy, lds);   // threads >= 256 add 0 after the digits
        if (t < kRadixBins) running[t] = ex + bel;
        __syncthreads();
    }
    const int64_t beg = b * S.per, end = beg + S.per < S.n ? beg + S.per : S.n;
    for (int64_t step = beg; step < end; step += kSortThreads * ITEMS) {
#pragma unroll
        for (int k = 0; k < kSortWaves * kRadixBins / kSortThreads; ++k)
            (&wcnt[0][0])[k * kSortThreads + t] = 0;
        __syncthreads();
        int32_t key[ITEMS], val[ITEMS], eid[ITEMS];
        int rank[ITEMS], dig[ITEMS];
        bool ok[ITEMS];
#pragma unroll
        for (int i = 0; i < ITEMS; ++i) {
            const int64_t idx = step + (int64_t)w * (kWave * ITEMS) + i * kWave + lane;
            ok[i] = idx < end;
            key[i] = ok[i] ? S.keys_in[idx] : 0;
            val[i] = ok[i] ? S.vals_in[idx] : 0;
            eid[i] = EID && ok[i] ? (S.eid_in ? S.eid_in[idx] : (int32_t)idx) : 0;
            dig[i] = (key[i] >> S.shift) & (kRadixBins - 1);
        }
#pragma unroll
        for (int i = 0; i < ITEMS; ++i) {
            unsigned long long mask = __ballot(ok[i]);
#pragma unroll
            for (int bit = 0; bit < kRadixBits; ++bit) {
                const bool one = (dig[i] >> bit) & 1;
                const unsigned long long bl = __ballot(one);
                mask &= one ? bl : ~bl;
            }
            const int lower = __popcll(mask & ((1ull << lane) - 1ull));
            const int prior = ok[i] ? wcnt[w][dig[i]] : 0;   // count from this wavefront's earlier rounds
            rank[i] = prior + lower;
            // the LDS read above is issued before this write by the same wavefront
            if (ok[i] && lower == 0) wcnt[w][dig[i]] = prior + __popcll(mask);
        }
        __syncthreads();
        // column scan over the wavefronts, then a scan over the digits: position of
        // every key inside this step's sorted order
        int tot_t = 0;
        if (t < kRadixBins) {
#pragma unroll
            for (int k = 0; k < kSortWaves; ++k) {
                int c = wcnt[k][t];
                wcnt[k][t] = tot_t;
                tot_t += c;
            }
        }
        int nvalid;
        const int lb = block_excl_scan(tot_t, &nvalid, lds);
        if (t < kRadixBins) {
            lbase[t] = lb;
            gdelta[t] = running[t] - lb;   // global position = gdelta[digit] + position in the step
            running[t] += tot_t;
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
            const int j = i * kSortThreads + t;
            if (j >= nvalid) continue;
            const int32_t k = skey[j], v = sval[j];
            const int pos = gdelta[(k >> S.shift) & (kRadixBins - 1)] + j;
            S.keys_out[pos] = k;
            S.vals_out[pos] = v;
            if (EID) S.eid_out[pos] = seid[j];
        }
        __syncthreads();   // wcnt and the staging arrays are reused by the next step
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
enum { JOB_ROWS_COUNT = 0, JOB_ROWS_FILL = 1, JOB_SORT_HIST = 2, JOB_SORT_SCATTER = 3, JOB_ROW_STARTS = 4 };
constexpr int kMaxJobs = 16;

struct Job {
    int kind, nblocks;
    union {
        RowsArgs rows;
        SortArgs sort;
        StartsArgs starts;
    };
};

struct StageArgs {
    int njobs;
    int first[kMaxJobs + 1];   // first workgroup of each job
    Job job[kMaxJobs];
};

__global__ __launch_bounds__(kSortThreads) void k_plan_stage(StageArgs A)
{
    __shared__ SortShared M;
    __shared__ int lds[16];
    int j = 0;
    while (j + 1 < A.njobs && (int)blockIdx.x >= A.first[j + 1]) ++j;
    const int b = blockIdx.x - A.first[j];
    const Job &J = A.job[j];
    switch (J.kind) {
        case JOB_ROWS_COUNT: rows_count(J.rows, b, lds); break;
        case JOB_ROWS_FILL: rows_fill(J.rows, b, lds); break;
        case JOB_SORT_HIST: sort_hist(J.sort, b, M.running); break;
        case JOB_SORT_SCATTER:
            if (J.sort.items == 1) sort_scatter<1>(J.sort, b, M, lds);
            else if (J.sort.items == 2) sort_scatter<2>(J.sort, b, M, lds);
            else sort_scatter<4>(J.sort, b, M, lds);
            break;
        default: row_starts(J.starts, b); break;
    }
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
    int64_t b = ceil_div(n, (int64_t)kSortThreads * 4);
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
    for (int i = 0; i < 6; ++i) q->sort_buf[i] = (int32_t *)take_bwd(4 * (size_t)num_edges);
    q->edge_dst = (int32_t *)take_bwd(4 * (size_t)num_edges);
    q->radix_cnt = (int32_t *)take_bwd(4 * (size_t)kRadixBins * kMaxSortBlocks);
    q->block_sums = (int32_t *)take(4 * 2 * (size_t)kMaxScanBlocks);
    q->block_sums2 = (int32_t *)take_bwd(4 * 2 * (size_t)kMaxScanBlocks);
    return off;
}

// ---- stages ----------------------------------------------------------------
using Stages = std::vector<std::vector<Job>>;

static void add_job(Stages &st, size_t k, const Job &j)
{
    if (st.size() <= k) st.resize(k + 1);
    st[k].push_back(j);
}

static Job rows_job(int kind, const RowsArgs &A)
{
    Job j;
    j.kind = kind; j.nblocks = A.nb; j.rows = A;
    return j;
}

// Append the jobs of one plan.  Stage k of a plan only depends on its own
// earlier stages, so plans of different depth can share launches.
static void plan_stages(fastgl_plan *p, int parts, Stages &st)
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
    int bits = 1;
    while (bits < 31 && ((int64_t)1 << bits) < p->num_src) ++bits;
    const int npass = (bits + kRadixBits - 1) / kRadixBits;
    SortArgs S;
    S.n = n;
    // one step per workgroup when the keys fit 256 workgroups x 4 keys per thread
    int items = 1;
    while (items < kMaxSortItems && (int64_t)items * kSortThreads * kMaxSortBlocks < n) items <<= 1;
    const int64_t step = (int64_t)items * kSortThreads;
    int64_t per = ceil_div(ceil_div(n, (int64_t)kMaxSortBlocks), step) * step;
    if (per < step) per = step;
    S.items = items;
    S.per = per;
    S.nb = n > 0 ? (int)ceil_div(n, per) : 1;
    S.cnt = p->radix_cnt;
    const bool want_perm = (parts & FASTGL_PLAN_PERM) != 0;
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
    RowsArgs srcA = rows_args(p->indptr_T, p->num_src, p->dout, nullptr, p->src_rsqrt, p->block_sums2,
                              p->long_src, p->chunk_ptr_src, p->counters + 2, nullptr, p->split_src,
                              p->num_edges);
    add_job(st, 2 * npass + 1, rows_job(JOB_ROWS_COUNT, srcA));
    add_job(st, 2 * npass + 2, rows_job(JOB_ROWS_FILL, srcA));
}

static fastgl_status run_stages(const Stages &st, hipStream_t s)
{
    for (const auto &jobs : st) {
        for (size_t at = 0; at < jobs.size(); at += kMaxJobs) {
            StageArgs A;
            A.njobs = (int)(jobs.size() - at < (size_t)kMaxJobs ? jobs.size() - at : kMaxJobs);
            int blocks = 0;
            for (int i = 0; i < A.njobs; ++i) {
                A.first[i] = blocks;
                A.job[i] = jobs[at + i];
                blocks += A.job[i].nblocks;
            }
            A.first[A.njobs] = blocks;
            hipLaunchKernelGGL(k_plan_stage, dim3(blocks), dim3(kSortThreads), 0, s, A);
            FASTGL_LAUNCH_CHECK("k_plan_stage");
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
    Stages st;
    for (int i = 0; i < n; ++i) plan_stages(plans[i], parts[i], st);
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
