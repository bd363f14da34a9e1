// Per-block integer bookkeeping on the GPU: degrees, scale factors, a stable
// transpose of the CSR (LSD radix sort of (source id, edge id)), and degree
// buckets (ordered compaction of long rows).  Everything is integer work with
// a single valid answer, so no float atomics and no order-dependent results.
//
// Why it exists: the backward pass (paper Section 4.2, Eq. 5) gathers along
// the reversed edges; pulling along a transposed CSR keeps one writer per
// output row, as the forward pass has (Section 4.2: a target's aggregation is
// completed by one owner).
#include "internal.h"

namespace fastgl {

// ---------------------------------------------------------------- scans ----
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

// Exclusive scan over the 256 threads of a block; *total = block sum.
// `lds` needs kBlock / kWave ints and is free again on return.
__device__ __forceinline__ int block_excl_scan(int v, int *total, int *lds)
{
    const int lane = threadIdx.x & (kWave - 1), w = threadIdx.x / kWave;
    int inc = wave_incl_scan(v);
    if (lane == kWave - 1) lds[w] = inc;
    __syncthreads();
    int off = 0, tot = 0;
#pragma unroll
    for (int i = 0; i < kBlock / kWave; ++i) {
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

// Block b owns elements [b*per, min(n,(b+1)*per)).
__global__ __launch_bounds__(kBlock) void k_scan_partials(const int32_t *__restrict__ in, int64_t n,
                                                          int64_t per, int32_t *__restrict__ bsum)
{
    __shared__ int lds[kBlock / kWave];
    int64_t beg = blockIdx.x * per, end = beg + per < n ? beg + per : n;
    int s = 0;
    for (int64_t i = beg + threadIdx.x; i < end; i += kBlock) s += in[i];
    s = block_sum(s, lds);
    if (threadIdx.x == 0) bsum[blockIdx.x] = s;
}

// out[i] = sum of in[0..i) for i in [0,n]; optionally rsq[i] = 1/sqrt(max(in[i],1)).
// in and out may alias.
__global__ __launch_bounds__(kBlock) void k_scan_final(const int32_t *in, int64_t n, int64_t per,
                                                       const int32_t *__restrict__ bsum,
                                                       int32_t *out, float *__restrict__ rsq)
{
    __shared__ int lds[kBlock / kWave];
    const int b = blockIdx.x;
    int pre = 0;
    for (int i = threadIdx.x; i < b; i += kBlock) pre += bsum[i];
    int carry = block_sum(pre, lds);
    int64_t beg = b * per, end = beg + per < n ? beg + per : n;
    for (int64_t base = beg; base < end; base += kBlock) {
        int64_t i = base + threadIdx.x;
        int v = i < end ? in[i] : 0;
        int tot;
        int ex = block_excl_scan(v, &tot, lds);
        if (i < end) {
            out[i] = carry + ex;
            if (rsq) rsq[i] = (float)(1.0 / sqrt((double)(v < 1 ? 1 : v)));
        }
        carry += tot;
    }
    if (b == (int)gridDim.x - 1 && threadIdx.x == 0) out[n] = carry;
}

// ------------------------------------------------ degrees + long-row buckets ----
// Pass 1 over row pointers: row lengths, scale factors, and per-block counts of
// long rows / their chunks.
__global__ __launch_bounds__(kBlock) void k_rows_count(const int32_t *__restrict__ rowptr, int64_t n,
                                                       int64_t per, int32_t *__restrict__ len_out,
                                                       float *__restrict__ inv, float *__restrict__ rsq,
                                                       int32_t *__restrict__ counts)
{
    __shared__ int lds[kBlock / kWave];
    int64_t beg = blockIdx.x * per, end = beg + per < n ? beg + per : n;
    int nl = 0, nc = 0;
    for (int64_t r = beg + threadIdx.x; r < end; r += kBlock) {
        int len = rowptr[r + 1] - rowptr[r];
        if (len_out) len_out[r] = len;
        double d = (double)(len < 1 ? 1 : len);
        if (inv) inv[r] = (float)(1.0 / d);
        if (rsq) rsq[r] = (float)(1.0 / sqrt(d));
        if (len > kLongThreshold) {
            nl += 1;
            nc += (len + kLongChunk - 1) / kLongChunk;
        }
    }
    nl = block_sum(nl, lds);
    nc = block_sum(nc, lds);
    if (threadIdx.x == 0) {
        counts[2 * blockIdx.x] = nl;
        counts[2 * blockIdx.x + 1] = nc;
    }
}

// Pass 2: ordered compaction.  long_rows ascending; chunk_ptr[i] = first chunk of
// the i-th long row; totals[0] = number of long rows, totals[1] = number of chunks.
__global__ __launch_bounds__(kBlock) void k_rows_fill(const int32_t *__restrict__ rowptr, int64_t n,
                                                      int64_t per, const int32_t *__restrict__ counts,
                                                      int32_t *__restrict__ long_rows,
                                                      int32_t *__restrict__ chunk_ptr,
                                                      int32_t *__restrict__ totals)
{
    __shared__ int lds[kBlock / kWave];
    const int b = blockIdx.x;
    int pl = 0, pc = 0;
    for (int i = threadIdx.x; i < b; i += kBlock) {
        pl += counts[2 * i];
        pc += counts[2 * i + 1];
    }
    int cl = block_sum(pl, lds);
    int cc = block_sum(pc, lds);
    int64_t beg = b * per, end = beg + per < n ? beg + per : n;
    for (int64_t base = beg; base < end; base += kBlock) {
        int64_t r = base + threadIdx.x;
        int len = r < end ? rowptr[r + 1] - rowptr[r] : 0;
        int isl = len > kLongThreshold ? 1 : 0;
        int nch = isl ? (len + kLongChunk - 1) / kLongChunk : 0;
        int tl, tc;
        int el = block_excl_scan(isl, &tl, lds);
        int ec = block_excl_scan(nch, &tc, lds);
        if (isl) {
            long_rows[cl + el] = (int32_t)r;
            chunk_ptr[cl + el] = cc + ec;
        }
        cl += tl;
        cc += tc;
    }
    if (b == (int)gridDim.x - 1 && threadIdx.x == 0) {
        chunk_ptr[cl] = cc;
        totals[0] = cl;
        totals[1] = cc;
    }
}

// ------------------------------------------------------------ radix sort ----
__global__ __launch_bounds__(kBlock) void k_radix_hist(const int32_t *__restrict__ keys, int64_t n,
                                                       int64_t per, int shift,
                                                       int32_t *__restrict__ cnt)
{
    __shared__ int h[kRadixBins];
    h[threadIdx.x] = 0;
    __syncthreads();
    int64_t beg = blockIdx.x * per, end = beg + per < n ? beg + per : n;
    for (int64_t i = beg + threadIdx.x; i < end; i += kBlock)
        atomicAdd(&h[(keys[i] >> shift) & (kRadixBins - 1)], 1);
    __syncthreads();
    cnt[(int64_t)threadIdx.x * gridDim.x + blockIdx.x] = h[threadIdx.x];
}

// largest u with indptr[u] <= e  (the destination row that owns edge e)
__device__ __forceinline__ int32_t owner_row(const int32_t *__restrict__ indptr, int32_t num_rows, int32_t e)
{
    int32_t lo = 0, hi = num_rows;   // invariant: indptr[lo] <= e < indptr[hi]
    while (hi - lo > 1) {
        int32_t mid = lo + ((hi - lo) >> 1);
        if (indptr[mid] <= e) lo = mid; else hi = mid;
    }
    return lo;
}

// Stable scatter of one digit.  base[d*nb + b] = first output slot of digit d for
// block b.  vals_in == NULL means the identity (first pass).  LAST: write the
// final permutation and the destination row of every edge instead of keys.
template <bool LAST>
__global__ __launch_bounds__(kBlock) void k_radix_scatter(
    const int32_t *__restrict__ keys_in, const int32_t *__restrict__ vals_in, int64_t n, int64_t per,
    int shift, const int32_t *__restrict__ base, int32_t *__restrict__ keys_out,
    int32_t *__restrict__ vals_out, const int32_t *__restrict__ indptr, int32_t num_dst,
    int32_t *__restrict__ dst_out)
{
    __shared__ int running[kRadixBins];
    __shared__ int wcnt[kBlock / kWave][kRadixBins];
    const int t = threadIdx.x, lane = t & (kWave - 1), w = t / kWave;
    running[t] = base[(int64_t)t * gridDim.x + blockIdx.x];
    int64_t beg = blockIdx.x * per, end = beg + per < n ? beg + per : n;
    for (int64_t tile = beg; tile < end; tile += kSortTile) {
        int64_t i = tile + t;
        bool valid = i < end;
        int32_t key = valid ? keys_in[i] : 0;
        int32_t val = valid ? (vals_in ? vals_in[i] : (int32_t)i) : 0;
        int d = (key >> shift) & (kRadixBins - 1);
#pragma unroll
        for (int k = 0; k < kBlock / kWave; ++k) wcnt[k][t] = 0;
        __syncthreads();
        unsigned long long mask = __ballot(valid);
#pragma unroll
        for (int bit = 0; bit < kRadixBits; ++bit) {
            bool one = (d >> bit) & 1;
            unsigned long long bl = __ballot(one);
            mask &= one ? bl : ~bl;
        }
        int lower = __popcll(mask & ((1ull << lane) - 1ull));
        if (valid && lower == 0) wcnt[w][d] = __popcll(mask);
        __syncthreads();
        int pos = 0;
        if (valid) {
            pos = running[d] + lower;
            for (int k = 0; k < w; ++k) pos += wcnt[k][d];
        }
        __syncthreads();
        {
            int add = 0;
#pragma unroll
            for (int k = 0; k < kBlock / kWave; ++k) add += wcnt[k][t];
            running[t] += add;
        }
        if (valid) {
            if (LAST) {
                vals_out[pos] = val;
                dst_out[pos] = owner_row(indptr, num_dst, val);
            } else {
                keys_out[pos] = key;
                vals_out[pos] = val;
            }
        }
        // the zeroing of wcnt[*][t] at the top of the next step is done by the
        // same thread that just read it; readers of running[] wait at the barrier
        // that follows the zeroing.
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

static void scan_shape(int64_t n, int *nb, int64_t *per)
{
    int64_t b = ceil_div(n, (int64_t)kBlock * 8);
    if (b < 1) b = 1;
    if (b > kMaxScanBlocks) b = kMaxScanBlocks;
    *nb = (int)b;
    *per = n > 0 ? ceil_div(n, b) : 1;
}

size_t plan_layout(fastgl_plan *p, void *base, int64_t num_dst, int64_t num_src, int64_t num_edges)
{
    size_t off = 0;
    char *b = (char *)base;
    auto take = [&](size_t bytes) {
        char *q = b ? b + off : nullptr;
        off += align_up(bytes ? bytes : 4, 256);
        return (void *)q;
    };
    const int64_t cl = cap_long_rows(num_edges);
    fastgl_plan tmp;
    fastgl_plan *q = p ? p : &tmp;
    q->din = (int32_t *)take(4 * (size_t)num_dst);
    q->dout = (int32_t *)take(4 * (size_t)num_src);
    q->indptr_T = (int32_t *)take(4 * ((size_t)num_src + 1));
    q->indices_T = (int32_t *)take(4 * (size_t)num_edges);
    q->perm = (int32_t *)take(4 * (size_t)num_edges);
    q->dst_inv = (float *)take(4 * (size_t)num_dst);
    q->dst_rsqrt = (float *)take(4 * (size_t)num_dst);
    q->src_rsqrt = (float *)take(4 * (size_t)num_src);
    q->long_dst = (int32_t *)take(4 * (size_t)cl);
    q->chunk_ptr_dst = (int32_t *)take(4 * ((size_t)cl + 1));
    q->long_src = (int32_t *)take(4 * (size_t)cl);
    q->chunk_ptr_src = (int32_t *)take(4 * ((size_t)cl + 1));
    q->counters = (int32_t *)take(4 * 4);
    for (int i = 0; i < 4; ++i) q->sort_buf[i] = (int32_t *)take(4 * (size_t)num_edges);
    q->radix_cnt = (int32_t *)take(4 * ((size_t)kRadixBins * kMaxScanBlocks + 1));
    q->block_sums = (int32_t *)take(4 * 2 * (size_t)kMaxScanBlocks);
    return off;
}

static fastgl_status exclusive_scan(const int32_t *in, int64_t n, int32_t *out, float *rsq,
                                    int32_t *bsum, hipStream_t s)
{
    int nb;
    int64_t per;
    scan_shape(n, &nb, &per);
    hipLaunchKernelGGL(k_scan_partials, dim3(nb), dim3(kBlock), 0, s, in, n, per, bsum);
    FASTGL_LAUNCH_CHECK("k_scan_partials");
    hipLaunchKernelGGL(k_scan_final, dim3(nb), dim3(kBlock), 0, s, in, n, per, bsum, out, rsq);
    FASTGL_LAUNCH_CHECK("k_scan_final");
    return FASTGL_OK;
}

static fastgl_status bucket_rows(const int32_t *rowptr, int64_t n, int32_t *len_out, float *inv,
                                 float *rsq, int32_t *long_rows, int32_t *chunk_ptr, int32_t *totals,
                                 int32_t *bsum, hipStream_t s)
{
    int nb;
    int64_t per;
    scan_shape(n, &nb, &per);
    hipLaunchKernelGGL(k_rows_count, dim3(nb), dim3(kBlock), 0, s, rowptr, n, per, len_out, inv, rsq, bsum);
    FASTGL_LAUNCH_CHECK("k_rows_count");
    hipLaunchKernelGGL(k_rows_fill, dim3(nb), dim3(kBlock), 0, s, rowptr, n, per, bsum, long_rows,
                       chunk_ptr, totals);
    FASTGL_LAUNCH_CHECK("k_rows_fill");
    return FASTGL_OK;
}

static fastgl_status stable_transpose(fastgl_plan *p, hipStream_t s)
{
    const int64_t n = p->num_edges;
    int bits = 1;
    while (bits < 31 && ((int64_t)1 << bits) < p->num_src) ++bits;
    const int npass = (bits + kRadixBits - 1) / kRadixBits;
    int64_t nb64 = ceil_div(n, (int64_t)kSortTile * 8);
    if (nb64 < 1) nb64 = 1;
    if (nb64 > kMaxScanBlocks) nb64 = kMaxScanBlocks;
    const int nb = (int)nb64;
    const int64_t per = n > 0 ? ceil_div(n, (int64_t)nb) : 1;
    const int32_t *kin = p->indices, *vin = nullptr;
    for (int pass = 0; pass < npass; ++pass) {
        const int shift = pass * kRadixBits;
        const bool last = pass == npass - 1;
        int32_t *kout = p->sort_buf[(pass & 1) * 2], *vout = p->sort_buf[(pass & 1) * 2 + 1];
        hipLaunchKernelGGL(k_radix_hist, dim3(nb), dim3(kBlock), 0, s, kin, n, per, shift, p->radix_cnt);
        FASTGL_LAUNCH_CHECK("k_radix_hist");
        fastgl_status st = exclusive_scan(p->radix_cnt, (int64_t)kRadixBins * nb, p->radix_cnt, nullptr,
                                          p->block_sums, s);
        if (st != FASTGL_OK) return st;
        if (last) {
            hipLaunchKernelGGL(k_radix_scatter<true>, dim3(nb), dim3(kBlock), 0, s, kin, vin, n, per, shift,
                               p->radix_cnt, (int32_t *)nullptr, p->perm, p->indptr, (int32_t)p->num_dst,
                               p->indices_T);
        } else {
            hipLaunchKernelGGL(k_radix_scatter<false>, dim3(nb), dim3(kBlock), 0, s, kin, vin, n, per, shift,
                               p->radix_cnt, kout, vout, p->indptr, (int32_t)p->num_dst, (int32_t *)nullptr);
        }
        FASTGL_LAUNCH_CHECK("k_radix_scatter");
        kin = kout;
        vin = vout;
    }
    return FASTGL_OK;
}

// Enqueue the bookkeeping kernels for the requested parts.  need_src_degrees
// asks for dout / src_rsqrt even when only the forward part is built (GCN).
fastgl_status plan_build(fastgl_plan *p, int parts, bool need_src_degrees, hipStream_t s)
{
    fastgl_status st;
    p->parts = parts;
    if (parts & FASTGL_PLAN_FWD) {
        st = bucket_rows(p->indptr, p->num_dst, p->din, p->dst_inv, p->dst_rsqrt, p->long_dst,
                         p->chunk_ptr_dst, p->counters, p->block_sums, s);
        if (st != FASTGL_OK) return st;
    }
    if ((parts & FASTGL_PLAN_BWD) || need_src_degrees) {
        hipLaunchKernelGGL(k_fill_i32, dim3(grid_for(p->num_src, 4)), dim3(kBlock), 0, s, p->dout,
                           p->num_src, 0);
        FASTGL_LAUNCH_CHECK("k_fill_i32");
        hipLaunchKernelGGL(k_hist, dim3(grid_for(p->num_edges, 4)), dim3(kBlock), 0, s, p->indices,
                           p->num_edges, p->dout);
        FASTGL_LAUNCH_CHECK("k_hist");
        st = exclusive_scan(p->dout, p->num_src, p->indptr_T, p->src_rsqrt, p->block_sums, s);
        if (st != FASTGL_OK) return st;
    }
    if (parts & FASTGL_PLAN_BWD) {
        if (!(parts & FASTGL_PLAN_FWD)) {
            // backward gathers rows of grad_out scaled by the destination-side factors
            st = bucket_rows(p->indptr, p->num_dst, p->din, p->dst_inv, p->dst_rsqrt, p->long_dst,
                             p->chunk_ptr_dst, p->counters, p->block_sums, s);
            if (st != FASTGL_OK) return st;
        }
        st = bucket_rows(p->indptr_T, p->num_src, nullptr, nullptr, nullptr, p->long_src,
                         p->chunk_ptr_src, p->counters + 2, p->block_sums, s);
        if (st != FASTGL_OK) return st;
        st = stable_transpose(p, s);
        if (st != FASTGL_OK) return st;
    }
    return FASTGL_OK;
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
