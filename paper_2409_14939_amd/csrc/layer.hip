// One sampled GNN layer in one call: aggregation (paper Section 2.1, Eq. 1) followed by the update
// Y = act(H W + b) (Eq. 2).  See include/fastgl_update.h for the contract of fastgl_layer_fwd.
//
// For a narrow layer on few target nodes - the class-score layer of a sampled GCN: a few thousand
// seeds, 256 features in, a few dozen classes out - both steps run in ONE kernel: the aggregated
// rows never travel to memory and back (they are written once, for the backward pass, only if the
// caller asks for them).  The product of such a layer is a fraction of a GFLOP, a microsecond of
// the vector ALUs, and the kernel is bound by its row gathers like the aggregation kernel is, so
// the product is done with plain fp32 multiply-adds rather than on the matrix cores.
//
//   workgroup = 4 wavefronts; a wavefront owns kRowsPerWave consecutive target rows
//   1. W (K x N, zero-padded to 64 columns) is copied to LDS once per workgroup
//   2. each wavefront walks the edges of its rows as one flat list (the aggregation kernel's
//      walk: 64 lanes x 16 bytes cover a row of up to 256 floats, 12 row gathers in flight, fp64
//      sums), scales and rounds each finished row to fp32 exactly as the aggregation kernel does,
//      and keeps it in LDS
//   3. lane n of the wavefront forms y[r][n] = b[n] + sum_k H[r][k] W[k][n] for its rows, k
//      ascending, one fp32 multiply-add per term: W[k][n] is read once for all rows of the
//      wavefront, H[r][k..k+3] as one broadcast 16-byte read
//
// Every other shape takes the two kernels of the separate calls, back to back on the stream.
#include "fastgl_update.h"
#include "pull_walk.h"

namespace fastgl {
namespace {

constexpr int kRowsPerWave = 4;
constexpr int kWavesPerBlock = kBlock / kWave;
constexpr int kRowsPerBlock = kRowsPerWave * kWavesPerBlock;
constexpr int kMaxFusedK = 256;     // 64 lanes x 4 floats
constexpr int kFusedCols = 64;      // one lane per output column
constexpr int kFusedUnroll = 12;    // row gathers in flight per lane: LDS limits a CU to 8 wavefronts of this kernel, registers are plentiful

struct LayerParams {
    PullParams pull;                // rowptr, col, eid, edge_w, col_scale, in, G = 64, row_mode, row_bytes, feat
    const float *W, *bias;          // [K][N], [N] or NULL
    float *H, *Y;                   // [rows][K] or NULL, [rows][N]
    int64_t rows;
    int32_t K, N, relu;
};

// A finished row: scaled and rounded to fp32 once (the value the aggregation kernel would store),
// kept in LDS for the product and, if asked for, streamed to H.
struct RowToLds {
    float *lds_rows;                // this wavefront's rows, [kRowsPerWave][K]
    float *H;
    int64_t row0;                   // first row of the wavefront
    int32_t K, sub;
    bool active;
    __device__ __forceinline__ void operator()(int64_t row, const double (&acc)[4], double scale) const
    {
        if (!active) return;
        const float4 v = make_float4((float)(acc[0] * scale), (float)(acc[1] * scale), (float)(acc[2] * scale),
                                     (float)(acc[3] * scale));
        *reinterpret_cast<float4 *>(lds_rows + (row - row0) * K + 4 * sub) = v;
        if (H) {
            typedef float f32x4 __attribute__((ext_vector_type(4)));
            const f32x4 w = {v.x, v.y, v.z, v.w};
            __builtin_nontemporal_store(w, reinterpret_cast<f32x4 *>(H + row * K + 4 * sub));
        }
    }
};

template <bool HASW>
__global__ __launch_bounds__(kBlock) void k_layer_rows(const LayerParams L)
{
    extern __shared__ __attribute__((aligned(16))) float lds[];
    const PullParams &P = L.pull;
    const int K = L.K, N = L.N;
    float *w_lds = lds;                                   // [K][kFusedCols]
    float *h_lds = lds + (size_t)K * kFusedCols;          // [kRowsPerBlock][K]
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;

    // 1. W -> LDS, columns beyond N read as zero.  W is walked as the contiguous array it is, 16
    //    independent loads per lane at a time (a load that waits for the previous one's LDS write
    //    would make this loop the longest phase of the kernel).
    for (int i = tid; i < K * (kFusedCols - N); i += kBlock)
        w_lds[(i / (kFusedCols - N)) * kFusedCols + N + i % (kFusedCols - N)] = 0.f;
    const int total_w = K * N;
    for (int base = 0; base < total_w; base += 16 * kBlock) {
        float t[16];
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const int i = base + j * kBlock + tid;
            t[j] = i < total_w ? L.W[i] : 0.f;
        }
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const int i = base + j * kBlock + tid;
            if (i < total_w) w_lds[(i / N) * kFusedCols + i % N] = t[j];
        }
    }

    // 2. aggregate this wavefront's rows into LDS
    const int64_t row0 = (int64_t)blockIdx.x * kRowsPerBlock + wave * kRowsPerWave;
    const int nrows = L.rows - row0 < kRowsPerWave ? (int)(L.rows - row0) : kRowsPerWave;   // may be <= 0
    float *my_rows = h_lds + wave * kRowsPerWave * K;
    if (nrows > 0) {
        int pb = 0, pe = 0;
        if (lane < nrows) {
            pb = P.rowptr[row0 + lane];
            pe = P.rowptr[row0 + lane + 1];
        }
        const bool active = 4 * lane < K;
        const RowToLds sink = {my_rows, L.H, row0, K, lane, active};
        walk_run<FASTGL_F32, 16, HASW, false, kFusedUnroll>(P, row0, 0, nrows, pb, pe, lane, 0, (int64_t)lane * 16, active, sink);
    }
    __syncthreads();      // W is complete; every wavefront's rows are in LDS

    // 3. the product: lane = output column
    if (nrows <= 0) return;
    float acc[kRowsPerWave];
    const float b = (L.bias && lane < N) ? L.bias[lane] : 0.f;
#pragma unroll
    for (int r = 0; r < kRowsPerWave; ++r) acc[r] = b;
    for (int k = 0; k < K; k += 4) {
        float w[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) w[i] = w_lds[(k + i) * kFusedCols + lane];
#pragma unroll
        for (int r = 0; r < kRowsPerWave; ++r) {
            // rows beyond nrows hold whatever LDS held: computed, never stored
            const float4 h = *reinterpret_cast<const float4 *>(my_rows + r * K + k);
            acc[r] = __builtin_fmaf(h.x, w[0], acc[r]);
            acc[r] = __builtin_fmaf(h.y, w[1], acc[r]);
            acc[r] = __builtin_fmaf(h.z, w[2], acc[r]);
            acc[r] = __builtin_fmaf(h.w, w[3], acc[r]);
        }
    }
    if (lane < N) {
#pragma unroll
        for (int r = 0; r < kRowsPerWave; ++r) {
            if (r >= nrows) break;
            float v = acc[r];
            if (L.relu) v = v > 0.f ? v : 0.f;
            L.Y[(row0 + r) * N + lane] = v;
        }
    }
}

// X rows are read and H rows written 16 bytes per lane.
bool fuses(int64_t K, int64_t N, fastgl_dtype dtype, const void *X, const void *H)
{
    return dtype == FASTGL_F32 && K > 0 && K % 4 == 0 && K <= kMaxFusedK && N > 0 && N <= kFusedCols &&
           (((uintptr_t)X | (uintptr_t)H) & 15) == 0;
}

// The fused kernel's LDS (W and 16 rows of H: up to 80 KB) is beyond the default limit of a launch;
// the limit of each variant is raised once, to what the largest fused shape needs.
template <bool HASW>
fastgl_status raise_lds_limit()
{
    static bool done = false;       // benign if two threads both do it
    if (!done) {
        const int most = (kMaxFusedK * kFusedCols + kRowsPerBlock * kMaxFusedK) * (int)sizeof(float);
        FASTGL_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_layer_rows<HASW>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, most));
        done = true;
    }
    return FASTGL_OK;
}

}  // namespace
}  // namespace fastgl

using namespace fastgl;

extern "C" {

int fastgl_layer_fwd_fuses(int64_t K, int64_t N, fastgl_dtype dtype)
{
    return fuses(K, N, dtype, nullptr, nullptr) ? 1 : 0;
}

fastgl_status fastgl_layer_fwd(const int32_t *indptr, const int32_t *indices, const float *edge_w, int64_t num_dst,
                               int64_t num_src, int64_t num_edges, int64_t K, fastgl_agg_mode mode,
                               fastgl_dtype dtype, const void *X, const void *W, const float *bias, int64_t N,
                               int relu, void *H, void *Y, const fastgl_plan *plan, void *workspace,
                               size_t workspace_bytes, void *stream)
{
    if (N < 0 || N >= ((int64_t)1 << 24)) {
        set_error("N must be in [0, 2^24) (got %lld)", (long long)N);
        return FASTGL_ERR_INVALID_ARG;
    }
    const bool fused = fuses(K, N, dtype, X, H);
    if (!H && !fused && num_dst > 0 && N > 0) {
        set_error("H is NULL but this shape (K=%lld N=%lld) runs as two kernels, which hand H over in memory",
                  (long long)K, (long long)N);
        return FASTGL_ERR_INVALID_ARG;
    }
    // the aggregation's own checks; with H == NULL they are given Y's address only to pass the
    // "output pointer is not NULL" test - nothing is stored there by the aggregation
    size_t need = 0;
    fastgl_status st = aggregate_check(false, indptr, indices, edge_w, num_dst, num_src, num_edges, K, mode, dtype, X,
                                       H ? H : Y, plan, &need);
    if (st != FASTGL_OK) return st;
    const uintptr_t el = dtype == FASTGL_F32 ? 4 : 2;
    if (num_dst > 0 && N > 0 && (!W || !Y)) {
        set_error("W or Y is NULL");
        return FASTGL_ERR_INVALID_ARG;
    }
    if ((((uintptr_t)W | (uintptr_t)Y | (uintptr_t)H) & (el - 1)) || ((uintptr_t)bias & 3)) {
        set_error("matrices must be aligned to their element size");
        return FASTGL_ERR_INVALID_ARG;
    }
    if (!workspace || ((uintptr_t)workspace & 255)) {
        set_error("workspace must be a 256-byte aligned device buffer");
        return FASTGL_ERR_INVALID_ARG;
    }
    if (workspace_bytes < need) {
        set_error("workspace too small: %zu < %zu bytes", workspace_bytes, need);
        return FASTGL_ERR_WORKSPACE;
    }
    if (num_dst == 0 || (N == 0 && !H)) return FASTGL_OK;

    if (!fused) {
        // two kernels back to back: aggregation into H, then the update phase's kernel
        st = aggregate_run(false, indptr, indices, edge_w, num_dst, num_src, num_edges, K, mode, dtype, X, H, plan,
                           workspace, stream);
        if (st != FASTGL_OK || N == 0) return st;
        return dtype == FASTGL_F32
                   ? fastgl_update_fwd((const float *)H, (const float *)W, bias, num_dst, K, N, relu, (float *)Y, stream)
                   : fastgl_update_fwd_bf16((const uint16_t *)H, (const uint16_t *)W, bias, num_dst, K, N, relu,
                                            (uint16_t *)Y, stream);
    }

    fastgl_plan local;
    PullDesc d;
    st = aggregate_prepare(false, indptr, indices, edge_w, num_dst, num_src, num_edges, K, mode, dtype, X, H, plan,
                           workspace, stream, &local, &d);
    if (st != FASTGL_OK) return st;
    LayerParams L = {};
    PullParams &P = L.pull;
    P.rowptr = d.rowptr; P.col = d.col; P.eid = d.eid;
    P.edge_w = d.edge_w; P.col_scale = d.col_scale;
    P.in = (const char *)d.in; P.out = nullptr;
    P.G = kWave; P.ntiles = 1;
    P.row_mode = d.row_mode;
    P.row_bytes = K * 4;
    P.feat = K;
    P.num_rows = num_dst;
    L.W = (const float *)W; L.bias = bias;
    L.H = (float *)H; L.Y = (float *)Y;
    L.rows = num_dst; L.K = (int32_t)K; L.N = (int32_t)N; L.relu = relu != 0;
    const size_t lds_bytes = ((size_t)K * kFusedCols + (size_t)kRowsPerBlock * K) * sizeof(float);
    const unsigned blocks = (unsigned)ceil_div(num_dst, kRowsPerBlock);
    const bool hasw = d.edge_w != nullptr || d.col_scale != nullptr;
    hipStream_t s = (hipStream_t)stream;
    st = hasw ? raise_lds_limit<true>() : raise_lds_limit<false>();
    if (st != FASTGL_OK) return st;
    if (hasw) hipLaunchKernelGGL(k_layer_rows<true>, dim3(blocks), dim3(kBlock), lds_bytes, s, L);
    else hipLaunchKernelGGL(k_layer_rows<false>, dim3(blocks), dim3(kBlock), lds_bytes, s, L);
    FASTGL_LAUNCH_CHECK("fastgl_layer_fwd");
    return FASTGL_OK;
}

}  // extern "C"
