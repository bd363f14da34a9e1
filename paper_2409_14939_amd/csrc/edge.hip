// Learned edge weights: gradient of Eq. 1 with respect to the weights (a sampled dense-dense
// product read at the block's edges) and the softmax over a destination's incoming edges.  See
// include/fastgl_edge.h for the contract.
//
// k_edge_dot: bound by HBM / fabric bandwidth like the aggregation itself - per edge one gathered row
// of X and one (cached, rows are consecutive) row of grad_out.  Work is dealt out per EDGE, not
// per row, so the degree distribution does not matter: a group of 2^k lanes covers the row pieces of
// one edge, several edges are in flight per group, and the lanes' partial dot products are added
// with cross-lane reads.  The destination of every edge comes from a small expansion pass.
//
// Softmax: a group of 8, 32 or 64 lanes (by the block's mean row length) walks one destination row
// three times (maximum, sum of exponentials, write); rows longer than kLongRow are queued and taken by whole workgroups afterwards.  exp and
// the sums are fp64, so the result is the correctly rounded quotient up to one unit in the last place.
#include <type_traits>

#include "fastgl_edge.h"
#include "internal.h"

namespace fastgl {
namespace {

constexpr int kLongRow = 1024;       // softmax rows longer than this go to the workgroup-per-row pass
constexpr int kLongGrid = 256;       // workgroups of that pass
constexpr int kEdgeUnroll = 4;       // edges in flight per lane group in k_edge_dot (reduce4 assumes 4)
constexpr int kEdgeSteps = 8;        // batches of that many edges per lane group

// ---------------------------------------------------------------- edge -> destination row
// A group of 8 lanes writes the row number over the edges of one row (rows of sampled blocks are
// short; a row of 10^4 edges costs one group ~10^3 steps).
__global__ __launch_bounds__(256) void k_edge_rows(const int32_t *__restrict__ indptr, int64_t num_dst, int64_t E,
                                                   int32_t *__restrict__ edge_row)
{
    (void)E;
    const int64_t u = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 3;
    if (u >= num_dst) return;
    const int b = indptr[u], e = indptr[u + 1];
    for (int k = b + (threadIdx.x & 7); k < e; k += 8) edge_row[k] = (int32_t)u;
}

// ---------------------------------------------------------------- dL/dw_e
template <typename ACC>
__device__ __forceinline__ ACC group_sum(ACC v, int lanes);

template <>
__device__ __forceinline__ double group_sum<double>(double v, int lanes)
{
    for (int d = lanes >> 1; d > 0; d >>= 1) v += __shfl_xor(v, d);
    return v;
}

template <>
__device__ __forceinline__ float group_sum<float>(float v, int lanes)
{
    for (int d = lanes >> 1; d > 0; d >>= 1) v += __shfl_xor(v, d);
    return v;
}

// Sums of four values over a group of `lanes` >= 4 lanes with 2 + 1 + (log2(lanes) - 2) exchanges
// instead of 4 log2(lanes): the first exchange leaves each half of the group with two of the four
// sums, the second each quarter with one, the rest finish that one.  Returns the sum of value
// number `which` (0..3, set here) - the same in every lane of a quarter.
template <typename ACC>
__device__ __forceinline__ ACC reduce4(const ACC (&v)[4], int l, int lanes, int &which)
{
    int d = lanes >> 1;
    const bool up = (l & d) != 0;
    const ACC r0 = (up ? v[2] : v[0]) + __shfl_xor(up ? v[0] : v[2], d);
    const ACC r1 = (up ? v[3] : v[1]) + __shfl_xor(up ? v[1] : v[3], d);
    d >>= 1;
    const bool up2 = (l & d) != 0;
    ACC r = (up2 ? r1 : r0) + __shfl_xor(up2 ? r0 : r1, d);
    for (d >>= 1; d > 0; d >>= 1) r += __shfl_xor(r, d);
    which = (up ? 2 : 0) + (up2 ? 1 : 0);
    return r;
}

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

// Dot product of one piece (PIECE bytes at byte offset `off` of both rows).
template <bool BF16, int PIECE, typename ACC>
__device__ __forceinline__ ACC piece_dot(const char *__restrict__ x, const char *__restrict__ g, int64_t off)
{
    ACC s = 0;
    if constexpr (!BF16) {
        if constexpr (PIECE == 16) {
            const float4 a = *reinterpret_cast<const float4 *>(x + off), b = *reinterpret_cast<const float4 *>(g + off);
            s += (ACC)a.x * (ACC)b.x;
            s += (ACC)a.y * (ACC)b.y;
            s += (ACC)a.z * (ACC)b.z;
            s += (ACC)a.w * (ACC)b.w;
        } else if constexpr (PIECE == 8) {
            const float2 a = *reinterpret_cast<const float2 *>(x + off), b = *reinterpret_cast<const float2 *>(g + off);
            s += (ACC)a.x * (ACC)b.x;
            s += (ACC)a.y * (ACC)b.y;
        } else {
            s += (ACC)(*reinterpret_cast<const float *>(x + off)) * (ACC)(*reinterpret_cast<const float *>(g + off));
        }
    } else {
        if constexpr (PIECE == 2) {
            const uint32_t wa = *reinterpret_cast<const uint16_t *>(x + off), wb = *reinterpret_cast<const uint16_t *>(g + off);
            s += (ACC)bf16_lo(wa) * (ACC)bf16_lo(wb);
        } else {
            constexpr int W = PIECE / 4;
            uint32_t a[W], b[W];
            if constexpr (W == 4) {
                const uint4 va = *reinterpret_cast<const uint4 *>(x + off), vb = *reinterpret_cast<const uint4 *>(g + off);
                a[0] = va.x; a[1] = va.y; a[2] = va.z; a[3] = va.w;
                b[0] = vb.x; b[1] = vb.y; b[2] = vb.z; b[3] = vb.w;
            } else if constexpr (W == 2) {
                const uint2 va = *reinterpret_cast<const uint2 *>(x + off), vb = *reinterpret_cast<const uint2 *>(g + off);
                a[0] = va.x; a[1] = va.y;
                b[0] = vb.x; b[1] = vb.y;
            } else {
                a[0] = *reinterpret_cast<const uint32_t *>(x + off);
                b[0] = *reinterpret_cast<const uint32_t *>(g + off);
            }
#pragma unroll
            for (int i = 0; i < W; ++i) {
                s += (ACC)bf16_lo(a[i]) * (ACC)bf16_lo(b[i]);
                s += (ACC)bf16_hi(a[i]) * (ACC)bf16_hi(b[i]);
            }
        }
    }
    return s;
}

struct DotArgs {
    const int32_t *indptr, *indices, *edge_row;
    const char *X, *G;
    const float *src_scale;      // [num_src] or NULL
    float *grad_w;
    int64_t E, row_bytes;
    int pieces;                  // row_bytes / PIECE
    int lanes;                   // lanes per edge group: power of two <= 64
    int mode;                    // 0 none, 1: 1/len, 2: 1/sqrt(len) of the destination row
};

// c_u * s_v of the aggregation mode.
__device__ __forceinline__ double edge_scale(const DotArgs &a, int32_t u, int32_t v)
{
    double scale = 1.0;
    if (a.mode) {
        const int len = a.indptr[u + 1] - a.indptr[u];
        const double d = len < 1 ? 1.0 : (double)len;
        scale = a.mode == 1 ? 1.0 / d : 1.0 / sqrt(d);
    }
    if (a.src_scale) scale *= (double)a.src_scale[v];
    return scale;
}

template <bool BF16, int PIECE>
__global__ __launch_bounds__(256) void k_edge_dot(const DotArgs a)
{
    using ACC = typename std::conditional<BF16, float, double>::type;
    const int lanes = a.lanes;
    const int groups_per_block = 256 / lanes;
    const int grp = threadIdx.x / lanes, l = threadIdx.x % lanes;
    // a group takes kEdgeSteps batches of kEdgeUnroll consecutive edges; the row and column of the
    // next batch's edges are fetched while the current batch's rows are in flight
    const int64_t first = ((int64_t)blockIdx.x * groups_per_block + grp) * (kEdgeUnroll * kEdgeSteps);
    int32_t u[kEdgeUnroll], v[kEdgeUnroll], un[kEdgeUnroll], vn[kEdgeUnroll];
#pragma unroll
    for (int k = 0; k < kEdgeUnroll; ++k) {
        const int64_t e = first + k < a.E ? first + k : a.E - 1;     // a clamped edge is computed and dropped
        un[k] = a.edge_row[e];
        vn[k] = a.indices[e];
    }
    for (int step = 0; step < kEdgeSteps; ++step) {
        const int64_t e0 = first + (int64_t)step * kEdgeUnroll;
        if (e0 >= a.E) break;                                        // uniform over the group
#pragma unroll
        for (int k = 0; k < kEdgeUnroll; ++k) {
            u[k] = un[k];
            v[k] = vn[k];
        }
        if (step + 1 < kEdgeSteps) {
#pragma unroll
            for (int k = 0; k < kEdgeUnroll; ++k) {
                const int64_t e = e0 + kEdgeUnroll + k < a.E ? e0 + kEdgeUnroll + k : a.E - 1;
                un[k] = a.edge_row[e];
                vn[k] = a.indices[e];
            }
        }
        ACC acc[kEdgeUnroll];
#pragma unroll
        for (int k = 0; k < kEdgeUnroll; ++k) acc[k] = 0;
        for (int p = l; p < a.pieces; p += lanes) {
            const int64_t off = (int64_t)p * PIECE;
#pragma unroll
            for (int k = 0; k < kEdgeUnroll; ++k)
                acc[k] += piece_dot<BF16, PIECE, ACC>(a.X + (int64_t)v[k] * a.row_bytes,
                                                      a.G + (int64_t)u[k] * a.row_bytes, off);
        }
        if (lanes >= 4) {
            int k;
            const ACC dot = reduce4<ACC>(acc, l, lanes, k);
            if ((l & (lanes / 4 - 1)) == 0 && e0 + k < a.E)          // first lane of each quarter
                a.grad_w[e0 + k] = (float)((double)dot * edge_scale(a, u[k], v[k]));
        } else {
#pragma unroll
            for (int k = 0; k < kEdgeUnroll; ++k) {
                const ACC dot = group_sum<ACC>(acc[k], lanes);
                if (l == 0 && e0 + k < a.E) a.grad_w[e0 + k] = (float)((double)dot * edge_scale(a, u[k], v[k]));
            }
        }
    }
}

// ---------------------------------------------------------------- softmax
struct SoftmaxArgs {
    const int32_t *indptr;
    int64_t num_dst;
    const float *in0;            // fwd: score;  bwd: alpha
    const float *in1;            // fwd: unused; bwd: grad_alpha
    float *out;
    int32_t *queue;              // rows longer than kLongRow
    int32_t *queue_len;
    int backward;
};

__device__ __forceinline__ double lanes_max(double v, int lanes)
{
    for (int d = lanes >> 1; d > 0; d >>= 1) v = fmax(v, __shfl_xor(v, d));
    return v;
}

// One row by `lanes` lanes starting at lane `l` of its group; every lane of the group returns.
__device__ __forceinline__ void softmax_row_fwd(const float *__restrict__ score, float *__restrict__ alpha, int b,
                                                int e, int l, int lanes)
{
    double m = -INFINITY;
    for (int k = b + l; k < e; k += lanes) m = fmax(m, (double)score[k]);
    m = lanes_max(m, lanes);
    double z = 0.0;
    for (int k = b + l; k < e; k += lanes) z += exp((double)score[k] - m);
    z = group_sum<double>(z, lanes);
    for (int k = b + l; k < e; k += lanes) alpha[k] = (float)(exp((double)score[k] - m) / z);
}

__device__ __forceinline__ void softmax_row_bwd(const float *__restrict__ alpha, const float *__restrict__ da,
                                                float *__restrict__ ds, int b, int e, int l, int lanes)
{
    double s = 0.0;
    for (int k = b + l; k < e; k += lanes) s += (double)alpha[k] * (double)da[k];
    s = group_sum<double>(s, lanes);
    for (int k = b + l; k < e; k += lanes) ds[k] = (float)((double)alpha[k] * ((double)da[k] - s));
}

template <int lanes>
__global__ __launch_bounds__(256) void k_edge_softmax_rows(const SoftmaxArgs a)
{
    const int64_t u = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) / lanes;
    const int l = threadIdx.x % lanes;
    int b = 0, e = 0;
    if (u < a.num_dst) {
        b = a.indptr[u];
        e = a.indptr[u + 1];
        if (e - b > kLongRow) {                   // queued for the workgroup-per-row pass
            if (l == 0) a.queue[atomicAdd(a.queue_len, 1)] = (int32_t)u;
            e = b;
        }
    }
    // all lanes of a group hold the same (b, e): the cross-lane sums below see whole groups
    if (a.backward)
        softmax_row_bwd(a.in0, a.in1, a.out, b, e, l, lanes);
    else
        softmax_row_fwd(a.in0, a.out, b, e, l, lanes);
}

// Sum / max over a 256-thread workgroup, result to every thread.
__device__ __forceinline__ double block_reduce(double v, bool take_max)
{
    __shared__ double part[4];
    v = take_max ? lanes_max(v, 64) : group_sum<double>(v, 64);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = v;
    __syncthreads();
    return take_max ? fmax(fmax(part[0], part[1]), fmax(part[2], part[3])) : (part[0] + part[1]) + (part[2] + part[3]);
}

__global__ __launch_bounds__(256) void k_edge_softmax_long(const SoftmaxArgs a)
{
    const int n = *a.queue_len;
    for (int q = blockIdx.x; q < n; q += gridDim.x) {
        const int u = a.queue[q];
        const int b = a.indptr[u], e = a.indptr[u + 1], l = threadIdx.x;
        if (!a.backward) {
            double m = -INFINITY;
            for (int k = b + l; k < e; k += 256) m = fmax(m, (double)a.in0[k]);
            m = block_reduce(m, true);
            double z = 0.0;
            for (int k = b + l; k < e; k += 256) z += exp((double)a.in0[k] - m);
            z = block_reduce(z, false);
            for (int k = b + l; k < e; k += 256) a.out[k] = (float)(exp((double)a.in0[k] - m) / z);
        } else {
            double s = 0.0;
            for (int k = b + l; k < e; k += 256) s += (double)a.in0[k] * (double)a.in1[k];
            s = block_reduce(s, false);
            for (int k = b + l; k < e; k += 256) a.out[k] = (float)((double)a.in0[k] * ((double)a.in1[k] - s));
        }
    }
}

__global__ void k_zero_i32(int32_t *p) { *p = 0; }

struct EdgeLayout {
    size_t edge_row, queue, queue_len, total;
};

EdgeLayout edge_layout(int64_t num_dst, int64_t E)
{
    (void)num_dst;
    EdgeLayout L;
    size_t off = 0;
    L.edge_row = off; off += align_up((size_t)(E > 0 ? E : 1) * 4, 256);
    L.queue = off; off += align_up((size_t)(E / kLongRow + 1) * 4, 256);
    L.queue_len = off; off += 256;
    L.total = off;
    return L;
}

fastgl_status check_csr(const int32_t *indptr, int64_t num_dst, int64_t E)
{
    if (num_dst < 0 || E < 0) {
        set_error("negative size (num_dst=%lld num_edges=%lld)", (long long)num_dst, (long long)E);
        return FASTGL_ERR_INVALID_ARG;
    }
    if (num_dst > kMaxIndex || E > kMaxIndex) {
        set_error("sizes must not exceed 2^31-1-1024 (int32 indices with look-ahead)");
        return FASTGL_ERR_UNSUPPORTED;
    }
    if (!indptr || ((uintptr_t)indptr & 3)) {
        set_error("indptr is NULL or misaligned");
        return FASTGL_ERR_INVALID_ARG;
    }
    if (E > 0 && num_dst == 0) {
        set_error("edges need at least one destination node");
        return FASTGL_ERR_INVALID_ARG;
    }
    return FASTGL_OK;
}

fastgl_status check_workspace(void *workspace, size_t have, size_t need)
{
    if (!workspace || ((uintptr_t)workspace & 255)) {
        set_error("workspace must be a 256-byte aligned device buffer");
        return FASTGL_ERR_INVALID_ARG;
    }
    if (have < need) {
        set_error("workspace too small: %zu < %zu bytes", have, need);
        return FASTGL_ERR_WORKSPACE;
    }
    return FASTGL_OK;
}

template <bool BF16, int PIECE>
void launch_dot(const DotArgs &a, hipStream_t s)
{
    const int groups_per_block = 256 / a.lanes;
    const int64_t blocks = ceil_div(a.E, (int64_t)groups_per_block * kEdgeUnroll * kEdgeSteps);
    hipLaunchKernelGGL((k_edge_dot<BF16, PIECE>), dim3((unsigned)blocks), dim3(256), 0, s, a);
}

fastgl_status softmax(bool backward, const int32_t *indptr, int64_t num_dst, int64_t E, const float *in0,
                      const float *in1, float *out, void *workspace, size_t workspace_bytes, void *stream)
{
    fastgl_status st = check_csr(indptr, num_dst, E);
    if (st != FASTGL_OK) return st;
    if (E == 0) return FASTGL_OK;
    if (!in0 || !out || (backward && !in1) || (((uintptr_t)in0 | (uintptr_t)in1 | (uintptr_t)out) & 3)) {
        set_error("per-edge array is NULL or misaligned");
        return FASTGL_ERR_INVALID_ARG;
    }
    const EdgeLayout L = edge_layout(num_dst, E);
    st = check_workspace(workspace, workspace_bytes, L.total);
    if (st != FASTGL_OK) return st;
    SoftmaxArgs a = {};
    a.indptr = indptr; a.num_dst = num_dst; a.in0 = in0; a.in1 = in1; a.out = out;
    a.queue = (int32_t *)((char *)workspace + L.queue);
    a.queue_len = (int32_t *)((char *)workspace + L.queue_len);
    a.backward = backward;
    hipStream_t s = (hipStream_t)stream;
    hipLaunchKernelGGL(k_zero_i32, dim3(1), dim3(1), 0, s, a.queue_len);
    FASTGL_LAUNCH_CHECK("edge softmax (reset)");
    // lanes per destination row by the block's mean row length (rows of sampled blocks are short)
    const int64_t mean = E / (num_dst > 0 ? num_dst : 1);
    if (mean < 24)
        hipLaunchKernelGGL(k_edge_softmax_rows<8>, dim3((unsigned)ceil_div(num_dst * 8, 256)), dim3(256), 0, s, a);
    else if (mean < 96)
        hipLaunchKernelGGL(k_edge_softmax_rows<32>, dim3((unsigned)ceil_div(num_dst * 32, 256)), dim3(256), 0, s, a);
    else
        hipLaunchKernelGGL(k_edge_softmax_rows<64>, dim3((unsigned)ceil_div(num_dst * 64, 256)), dim3(256), 0, s, a);
    FASTGL_LAUNCH_CHECK("edge softmax (rows)");
    hipLaunchKernelGGL(k_edge_softmax_long, dim3(kLongGrid), dim3(256), 0, s, a);
    FASTGL_LAUNCH_CHECK("edge softmax (long rows)");
    return FASTGL_OK;
}


// ---------------------------------------------------------------- attention logits of a GAT head
// score_e = LeakyReLU(el[u] + er[v]) and the sums of its gradient over rows.  The same kernels run on
// the block's CSR (rows = destinations, col = neighbours) and on its transpose (rows = neighbours,
// col = destinations, eid = original edge ids): `row_val` belongs to the row index, `col_val` to col.
struct ScoreArgs {
    const int32_t *rowptr, *col, *eid;     // eid NULL: the edge id is the position
    int64_t num_rows;
    const float *row_val, *col_val;
    const float *grad_score;               // backward only
    float *out;                            // forward: [E] scores; backward: [num_rows] sums
    double slope;
};

template <int lanes, bool BACKWARD>
__global__ __launch_bounds__(256) void k_edge_score(const ScoreArgs a)
{
    const int64_t r = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) / lanes;
    const int l = threadIdx.x % lanes;
    int b = 0, e = 0;
    double mine = 0.0;
    if (r < a.num_rows) {
        b = a.rowptr[r];
        e = a.rowptr[r + 1];
        mine = (double)a.row_val[r];
    }
    double acc = 0.0;
    for (int k = b + l; k < e; k += lanes) {
        const double x = mine + (double)a.col_val[a.col[k]];      // exact: both are fp32
        if (!BACKWARD)
            a.out[k] = (float)(x > 0.0 ? x : a.slope * x);
        else
            acc += (double)a.grad_score[a.eid ? a.eid[k] : k] * (x > 0.0 ? 1.0 : a.slope);
    }
    if (BACKWARD) {
        acc = group_sum<double>(acc, lanes);       // every lane of the group takes part
        if (l == 0 && r < a.num_rows) a.out[r] = (float)acc;
    }
}

template <bool BACKWARD>
void launch_score(const ScoreArgs &a, int64_t nnz, hipStream_t s)
{
    const int64_t mean = nnz / (a.num_rows > 0 ? a.num_rows : 1);
    if (mean < 24)
        hipLaunchKernelGGL((k_edge_score<8, BACKWARD>), dim3((unsigned)ceil_div(a.num_rows * 8, 256)), dim3(256), 0, s, a);
    else if (mean < 96)
        hipLaunchKernelGGL((k_edge_score<32, BACKWARD>), dim3((unsigned)ceil_div(a.num_rows * 32, 256)), dim3(256), 0, s, a);
    else
        hipLaunchKernelGGL((k_edge_score<64, BACKWARD>), dim3((unsigned)ceil_div(a.num_rows * 64, 256)), dim3(256), 0, s, a);
}

fastgl_status check_score_args(const int32_t *indptr, const int32_t *indices, int64_t num_dst, int64_t num_src,
                               int64_t E, const float *el, const float *er, float slope)
{
    fastgl_status st = check_csr(indptr, num_dst, E);
    if (st != FASTGL_OK) return st;
    if (num_src < 0 || num_src >= INT32_MAX) {
        set_error("num_src out of range");
        return FASTGL_ERR_INVALID_ARG;
    }
    if (!(slope == slope) || slope - slope != 0.f) {
        set_error("slope must be finite");
        return FASTGL_ERR_INVALID_ARG;
    }
    if (E > 0 && (!indices || !el || !er || num_src == 0 || (((uintptr_t)indices | (uintptr_t)el | (uintptr_t)er) & 3))) {
        set_error("NULL or misaligned array (indices, el or er), or no source nodes");
        return FASTGL_ERR_INVALID_ARG;
    }
    return FASTGL_OK;
}

}  // namespace
}  // namespace fastgl

using namespace fastgl;

extern "C" {

size_t fastgl_edge_workspace_bytes(int64_t num_dst, int64_t num_edges)
{
    if (num_dst < 0 || num_edges < 0 || num_edges >= INT32_MAX) return 0;
    return edge_layout(num_dst, num_edges).total;
}

int32_t fastgl_edge_softmax_long_row(void) { return kLongRow; }

fastgl_status fastgl_edge_weight_grad(const int32_t *indptr, const int32_t *indices, int64_t num_dst,
                                      int64_t num_src, int64_t num_edges, int64_t feat, fastgl_agg_mode mode,
                                      fastgl_dtype dtype, const void *X, const void *grad_out,
                                      const fastgl_plan *plan, float *grad_w, void *workspace,
                                      size_t workspace_bytes, void *stream)
{
    fastgl_status st = check_csr(indptr, num_dst, num_edges);
    if (st != FASTGL_OK) return st;
    if (num_src < 0 || num_src >= INT32_MAX) {
        set_error("num_src out of range");
        return FASTGL_ERR_INVALID_ARG;
    }
    if (feat <= 0 || feat > ((int64_t)1 << 24)) {
        set_error("feat must be in [1, 2^24] (got %lld)", (long long)feat);
        return FASTGL_ERR_INVALID_ARG;
    }
    if ((int)mode < 0 || (int)mode > 2 || (int)dtype < 0 || (int)dtype > 1) {
        set_error("unknown aggregation mode %d or dtype %d", (int)mode, (int)dtype);
        return FASTGL_ERR_INVALID_ARG;
    }
    if (num_edges == 0) return FASTGL_OK;
    if (!indices || !X || !grad_out || !grad_w || num_src == 0) {
        set_error("NULL array (indices, X, grad_out or grad_w) or no source nodes");
        return FASTGL_ERR_INVALID_ARG;
    }
    const int64_t elem = dtype == FASTGL_F32 ? 4 : 2;
    if ((((uintptr_t)X | (uintptr_t)grad_out) & (uintptr_t)(elem - 1)) || (((uintptr_t)indices | (uintptr_t)grad_w) & 3)) {
        set_error("misaligned buffer");
        return FASTGL_ERR_INVALID_ARG;
    }
    const float *src_scale = nullptr;
    if (mode == FASTGL_AGG_GCN) {
        if (!plan || plan->indptr != indptr || plan->indices != indices || plan->num_dst != num_dst ||
            plan->num_src != num_src || plan->num_edges != num_edges ||
            !(plan->parts & (FASTGL_PLAN_BWD | FASTGL_PLAN_SRC_DEG))) {
            set_error("GCN mode needs a plan of this block that holds the source degrees");
            return FASTGL_ERR_INVALID_ARG;
        }
        src_scale = plan->src_rsqrt;
    }
    const EdgeLayout L = edge_layout(num_dst, num_edges);
    st = check_workspace(workspace, workspace_bytes, L.total);
    if (st != FASTGL_OK) return st;

    DotArgs a = {};
    a.indptr = indptr; a.indices = indices;
    a.edge_row = (int32_t *)((char *)workspace + L.edge_row);
    a.X = (const char *)X; a.G = (const char *)grad_out;
    a.src_scale = src_scale; a.grad_w = grad_w;
    a.E = num_edges; a.row_bytes = feat * elem;
    a.mode = mode == FASTGL_AGG_MEAN ? 1 : (mode == FASTGL_AGG_GCN ? 2 : 0);
    const uintptr_t both = (uintptr_t)X | (uintptr_t)grad_out;
    int piece = (int)elem;
    for (int cand = 16; cand > elem; cand >>= 1)
        if (a.row_bytes % cand == 0 && (both & (uintptr_t)(cand - 1)) == 0) {
            piece = cand;
            break;
        }
    a.pieces = (int)(a.row_bytes / piece);
    a.lanes = 1;
    while (a.lanes < 64 && a.lanes < a.pieces) a.lanes *= 2;
    hipStream_t s = (hipStream_t)stream;
    hipLaunchKernelGGL(k_edge_rows, dim3((unsigned)ceil_div(num_dst * 8, 256)), dim3(256), 0, s, indptr, num_dst,
                       num_edges, (int32_t *)a.edge_row);
    FASTGL_LAUNCH_CHECK("fastgl_edge_weight_grad (edge rows)");
    const bool bf = dtype == FASTGL_BF16;
    switch (piece) {
    case 16: bf ? launch_dot<true, 16>(a, s) : launch_dot<false, 16>(a, s); break;
    case 8: bf ? launch_dot<true, 8>(a, s) : launch_dot<false, 8>(a, s); break;
    case 4: bf ? launch_dot<true, 4>(a, s) : launch_dot<false, 4>(a, s); break;
    default: launch_dot<true, 2>(a, s); break;
    }
    FASTGL_LAUNCH_CHECK("fastgl_edge_weight_grad");
    return FASTGL_OK;
}

fastgl_status fastgl_edge_softmax_fwd(const int32_t *indptr, int64_t num_dst, int64_t num_edges,
                                      const float *score, float *alpha, void *workspace, size_t workspace_bytes,
                                      void *stream)
{
    return softmax(false, indptr, num_dst, num_edges, score, nullptr, alpha, workspace, workspace_bytes, stream);
}

fastgl_status fastgl_edge_softmax_bwd(const int32_t *indptr, int64_t num_dst, int64_t num_edges,
                                      const float *alpha, const float *grad_alpha, float *grad_score,
                                      void *workspace, size_t workspace_bytes, void *stream)
{
    return softmax(true, indptr, num_dst, num_edges, alpha, grad_alpha, grad_score, workspace, workspace_bytes,
                   stream);
}

fastgl_status fastgl_edge_score_fwd(const int32_t *indptr, const int32_t *indices, int64_t num_dst, int64_t num_src,
                                    int64_t num_edges, const float *el, const float *er, float slope, float *score,
                                    void *stream)
{
    fastgl_status st = check_score_args(indptr, indices, num_dst, num_src, num_edges, el, er, slope);
    if (st != FASTGL_OK) return st;
    if (num_edges == 0) return FASTGL_OK;
    if (!score || ((uintptr_t)score & 3)) {
        set_error("score is NULL or misaligned");
        return FASTGL_ERR_INVALID_ARG;
    }
    ScoreArgs a = {};
    a.rowptr = indptr; a.col = indices; a.num_rows = num_dst;
    a.row_val = el; a.col_val = er; a.out = score; a.slope = (double)slope;
    launch_score<false>(a, num_edges, (hipStream_t)stream);
    FASTGL_LAUNCH_CHECK("fastgl_edge_score_fwd");
    return FASTGL_OK;
}

fastgl_status fastgl_edge_score_bwd(const int32_t *indptr, const int32_t *indices, int64_t num_dst, int64_t num_src,
                                    int64_t num_edges, const float *el, const float *er, float slope,
                                    const float *grad_score, const fastgl_plan *plan, float *grad_el, float *grad_er,
                                    void *stream)
{
    fastgl_status st = check_score_args(indptr, indices, num_dst, num_src, num_edges, el, er, slope);
    if (st != FASTGL_OK) return st;
    if ((((uintptr_t)grad_score | (uintptr_t)grad_el | (uintptr_t)grad_er) & 3) || (num_edges > 0 && !grad_score)) {
        set_error("grad_score is NULL, or a gradient array is misaligned");
        return FASTGL_ERR_INVALID_ARG;
    }
    hipStream_t s = (hipStream_t)stream;
    if (grad_er && num_src > 0) {   // checked before the first launch: a refused call leaves nothing on the stream
        const int need = FASTGL_PLAN_BWD | FASTGL_PLAN_PERM;
        if (!plan || plan->indptr != indptr || plan->indices != indices || plan->num_dst != num_dst ||
            plan->num_src != num_src || plan->num_edges != num_edges || (plan->parts & need) != need) {
            set_error("grad_er needs a plan of this block built with FASTGL_PLAN_BWD | FASTGL_PLAN_PERM");
            return FASTGL_ERR_INVALID_ARG;
        }
    }
    if (grad_el && num_dst > 0) {
        if (!el && num_edges == 0) el = grad_el;       // rows without edges read nothing but their own value
        ScoreArgs a = {};
        a.rowptr = indptr; a.col = indices; a.num_rows = num_dst;
        a.row_val = el; a.col_val = er; a.grad_score = grad_score; a.out = grad_el; a.slope = (double)slope;
        launch_score<true>(a, num_edges, s);
        FASTGL_LAUNCH_CHECK("fastgl_edge_score_bwd (grad_el)");
    }
    if (grad_er && num_src > 0) {
        if (!er && num_edges == 0) er = grad_er;
        ScoreArgs a = {};
        a.rowptr = plan->indptr_T; a.col = plan->indices_T; a.eid = plan->perm; a.num_rows = num_src;
        a.row_val = er; a.col_val = el; a.grad_score = grad_score; a.out = grad_er; a.slope = (double)slope;
        launch_score<true>(a, num_edges, s);
        FASTGL_LAUNCH_CHECK("fastgl_edge_score_bwd (grad_er)");
    }
    return FASTGL_OK;
}

}  // extern "C"
