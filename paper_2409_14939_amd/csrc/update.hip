// Update phase of a sampled GCN layer (paper Section 2.1, Eq. 2) on the fp32
// matrix cores of gfx950: Y = act(H W + b) and its three gradients.  See
// include/fastgl_update.h for the contract of every entry point.
//
// One tiled kernel serves all four products.  A workgroup of 4 wavefronts owns
// a 128 x 128 tile of the result (each wavefront a 64 x 64 quarter = 2 x 2
// accumulators of v_mfma_f32_32x32x2_f32) and walks the contracted dimension in
// steps of 32, staged through LDS.  Each operand is copied to LDS in the layout
// it has in memory, so both kinds of operand get coalesced global loads:
//   "row" operand   mem[out][contract]  -> lds[out][32 + 4]  (read back 16 B per lane)
//   "col" operand   mem[contract][out]  -> lds[contract][128 + 8]
// Inside a group of 8 contracted indices lane half h (lanes 32h..32h+31) takes
// indices 4h..4h+3, and MFMA number t multiplies index 4h+t of both operands;
// the sum over the contracted index does not care about this order.
#include "fastgl_update.h"
#include "internal.h"

namespace fastgl {
namespace {

constexpr int kTile = 128;              // rows and columns of a workgroup's result tile
constexpr int kStep = 32;               // contracted indices per LDS stage
constexpr int kRowStride = kStep + 4;   // floats between rows of a "row" operand in LDS
constexpr int kColStride = kTile + 8;   // floats between contracted indices of a "col" operand
constexpr int kOperandFloats = (kTile * kRowStride > kStep * kColStride) ? kTile * kRowStride : kStep * kColStride;
constexpr int kSlabRows = 1024;         // rows of H per dW / db partial

typedef float f32x16 __attribute__((ext_vector_type(16)));

struct Operand {
    const float *p;       // element (out o, contracted k) at p[o*ld + k] ("row") or p[k*ld + o] ("col")
    const float *gate;    // same layout, or NULL; where gate <= 0 the element reads as 0 (ReLU derivative)
    int64_t ld;
    int vec;              // 16-byte loads allowed: ld % 4 == 0 and p, gate 16-byte aligned
};

struct GemmArgs {
    Operand a, b;
    float *c;                   // [R][C] result (of slab s: c + s*c_slab)
    int64_t ldc, c_slab;
    int64_t R, C, Kc;           // result rows, result columns, contracted length
    int64_t slab;               // contracted indices per slab (>= Kc when not split)
    int64_t n_outer;            // slabs (split) or row tiles (not split)
    int tiles_r, tiles_c;
    int split;                  // 1: outer index = slab, inner = (row tile, column tile)
    const float *bias;          // [C] or NULL, added before the activation
    int relu;
    float *colsum;              // [slab][colsum_slab]: sums of operand b over the slab, or NULL
    int64_t colsum_slab;
};

__device__ __forceinline__ float4 load4(const Operand &op, int64_t off, int nvalid)
{
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    if (nvalid <= 0) return v;
    if (op.vec && nvalid >= 4) {
        v = *reinterpret_cast<const float4 *>(op.p + off);
        if (op.gate) {
            const float4 g = *reinterpret_cast<const float4 *>(op.gate + off);
            v.x = g.x > 0.f ? v.x : 0.f;
            v.y = g.y > 0.f ? v.y : 0.f;
            v.z = g.z > 0.f ? v.z : 0.f;
            v.w = g.w > 0.f ? v.w : 0.f;
        }
        return v;
    }
    float e[4] = {0.f, 0.f, 0.f, 0.f};
    for (int i = 0; i < 4; ++i)
        if (i < nvalid) {
            e[i] = op.p[off + i];
            if (op.gate && !(op.gate[off + i] > 0.f)) e[i] = 0.f;
        }
    return make_float4(e[0], e[1], e[2], e[3]);
}

__device__ __forceinline__ int clamp4(int64_t n) { return n >= 4 ? 4 : (n <= 0 ? 0 : (int)n); }

// Global -> registers for one 128 (out) x 32 (contracted) operand tile.
template <bool COL>
__device__ __forceinline__ void fetch_tile(const Operand &op, int64_t o0, int64_t omax, int64_t k0, int64_t kend,
                                           float4 (&r)[4])
{
    const int t = threadIdx.x;
    if (!COL) {
        const int kq = t & 7, rr = t >> 3;                 // 8 lanes cover the 32 contracted indices of a row
        const int64_t k = k0 + 4 * kq;
        const int nv = clamp4(kend - k);
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const int64_t o = o0 + rr + 32 * s;
            r[s] = load4(op, o * op.ld + k, o < omax ? nv : 0);
        }
    } else {
        const int oq = t & 31, kk = t >> 5;                // 32 lanes cover the 128 out indices of one k
        const int64_t o = o0 + 4 * oq;
        const int nv = clamp4(omax - o);
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const int64_t k = k0 + kk + 8 * s;
            r[s] = load4(op, k * op.ld + o, k < kend ? nv : 0);
        }
    }
}

template <bool COL>
__device__ __forceinline__ void stage_tile(float *lds, const float4 (&r)[4])
{
    const int t = threadIdx.x;
    if (!COL) {
        const int kq = t & 7, rr = t >> 3;
#pragma unroll
        for (int s = 0; s < 4; ++s)
            *reinterpret_cast<float4 *>(lds + (rr + 32 * s) * kRowStride + 4 * kq) = r[s];
    } else {
        const int oq = t & 31, kk = t >> 5;
#pragma unroll
        for (int s = 0; s < 4; ++s)
            *reinterpret_cast<float4 *>(lds + (kk + 8 * s) * kColStride + 4 * oq) = r[s];
    }
}

// The four values (contracted indices 8c+4h .. 8c+4h+3) of out index o.
template <bool COL>
__device__ __forceinline__ float4 read_frag(const float *lds, int o, int c, int h)
{
    if (!COL) return *reinterpret_cast<const float4 *>(lds + o * kRowStride + 8 * c + 4 * h);
    const float *q = lds + (8 * c + 4 * h) * kColStride + o;
    return make_float4(q[0], q[kColStride], q[2 * kColStride], q[3 * kColStride]);
}

template <bool A_COL, bool B_COL>
__global__ __launch_bounds__(256) void k_update_gemm(const GemmArgs g)
{
    __shared__ __attribute__((aligned(16))) float lds_a[kOperandFloats];
    __shared__ __attribute__((aligned(16))) float lds_b[kOperandFloats];

    // Workgroups are dealt round-robin to the 8 L2 domains; the ones that share an operand tile
    // (same outer index) are given consecutive slots of one domain.
    const int64_t bid = blockIdx.x;
    const int xcd = (int)(bid % kXcds);
    const int64_t q = bid / kXcds;
    const int n_inner = g.split ? g.tiles_r * g.tiles_c : g.tiles_c;
    const int inner = (int)(q % n_inner);
    const int64_t outer = (q / n_inner) * kXcds + xcd;
    if (outer >= g.n_outer) return;
    int64_t tile_r, kbeg, kend, slab_id;
    int tile_c;
    if (g.split) {
        slab_id = outer;
        tile_r = inner / g.tiles_c;
        tile_c = inner % g.tiles_c;
        kbeg = slab_id * g.slab;
        kend = kbeg + g.slab < g.Kc ? kbeg + g.slab : g.Kc;
    } else {
        slab_id = 0;
        tile_r = outer;
        tile_c = inner;
        kbeg = 0;
        kend = g.Kc;
    }
    const int64_t r0 = tile_r * kTile, c0 = (int64_t)tile_c * kTile;

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wr = wave >> 1, wc = wave & 1;       // 2 x 2 wavefronts, 64 x 64 each
    const int h = lane >> 5, l32 = lane & 31;

    f32x16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
    float bsum[2] = {0.f, 0.f};

    float4 ra[4], rb[4];
    if (kbeg < kend) {
        fetch_tile<A_COL>(g.a, r0, g.R, kbeg, kend, ra);
        fetch_tile<B_COL>(g.b, c0, g.C, kbeg, kend, rb);
    }
    for (int64_t k0 = kbeg; k0 < kend; k0 += kStep) {
        stage_tile<A_COL>(lds_a, ra);
        stage_tile<B_COL>(lds_b, rb);
        __syncthreads();
        if (k0 + kStep < kend) {                   // next stage's global loads fly during the MFMAs
            fetch_tile<A_COL>(g.a, r0, g.R, k0 + kStep, kend, ra);
            fetch_tile<B_COL>(g.b, c0, g.C, k0 + kStep, kend, rb);
        }
        const int64_t left = kend - k0;
        const int nchunk = left >= kStep ? kStep / 8 : (int)((left + 7) / 8);
        for (int c = 0; c < nchunk; ++c) {
            float4 fa[2], fb[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) fa[i] = read_frag<A_COL>(lds_a, wr * 64 + i * 32 + l32, c, h);
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                fb[j] = read_frag<B_COL>(lds_b, wc * 64 + j * 32 + l32, c, h);
                bsum[j] += (fb[j].x + fb[j].y) + (fb[j].z + fb[j].w);
            }
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[i].x, fb[j].x, acc[i][j], 0, 0, 0);
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[i].y, fb[j].y, acc[i][j], 0, 0, 0);
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[i].z, fb[j].z, acc[i][j], 0, 0, 0);
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[i].w, fb[j].w, acc[i][j], 0, 0, 0);
                }
        }
        __syncthreads();
    }

    // Accumulator element e of lane (h, l32) is row 8*(e/4) + 4*h + e%4, column l32 of its 32 x 32 tile.
    float *cbase = g.c + slab_id * g.c_slab;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int64_t col = c0 + wc * 64 + j * 32 + l32;
        if (col >= g.C) continue;
        const float bj = g.bias ? g.bias[col] : 0.f;
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int64_t row = r0 + wr * 64 + i * 32 + 8 * (e >> 2) + 4 * h + (e & 3);
                if (row >= g.R) continue;
                float v = acc[i][j][e] + bj;
                if (g.relu) v = v > 0.f ? v : 0.f;
                cbase[row * g.ldc + col] = v;
            }
    }
    if (g.colsum && tile_r == 0 && wr == 0) {
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const float s = bsum[j] + __shfl_xor(bsum[j], 32);
            const int64_t col = c0 + wc * 64 + j * 32 + l32;
            if (h == 0 && col < g.C) g.colsum[slab_id * g.colsum_slab + col] = s;
        }
    }
}

// out[e] = sum over slabs, in slab order, in fp64, of part[s*stride + e]; the first n_w elements go
// to dW, the remaining n_b to db (either may be NULL).
__global__ __launch_bounds__(256) void k_update_reduce(const float *part, int64_t nslab, int64_t stride,
                                                       int64_t n_w, int64_t n_b, float *dW, float *db)
{
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= n_w + n_b) return;
    float *dst = e < n_w ? (dW ? dW + e : nullptr) : (db ? db + (e - n_w) : nullptr);
    if (!dst) return;
    double s = 0.0;
    for (int64_t k = 0; k < nslab; ++k) s += (double)part[k * stride + e];
    *dst = (float)s;
}

bool vec_ok(const float *p, const float *gate, int64_t ld)
{
    return ld % 4 == 0 && (((uintptr_t)p | (uintptr_t)gate) & 15) == 0;
}

template <bool A_COL, bool B_COL>
fastgl_status launch_gemm(GemmArgs &g, hipStream_t s, const char *what)
{
    g.tiles_r = (int)ceil_div(g.R, kTile);
    g.tiles_c = (int)ceil_div(g.C, kTile);
    if (g.split && g.tiles_r == 0) g.tiles_r = 1;          // column sums are still owed when R == 0
    const int64_t n_inner = g.split ? (int64_t)g.tiles_r * g.tiles_c : g.tiles_c;
    if (!g.split) g.n_outer = g.tiles_r;
    const int64_t blocks = ceil_div(g.n_outer, kXcds) * kXcds * n_inner;
    if (blocks == 0) return FASTGL_OK;
    if (blocks >= INT32_MAX) {
        set_error("%s: too many tiles (%lld)", what, (long long)blocks);
        return FASTGL_ERR_UNSUPPORTED;
    }
    hipLaunchKernelGGL((k_update_gemm<A_COL, B_COL>), dim3((unsigned)blocks), dim3(256), 0, s, g);
    FASTGL_LAUNCH_CHECK(what);
    return FASTGL_OK;
}

fastgl_status check_dims(int64_t M, int64_t K, int64_t N)
{
    if (M < 0 || K < 0 || N < 0) {
        set_error("negative size (M=%lld K=%lld N=%lld)", (long long)M, (long long)K, (long long)N);
        return FASTGL_ERR_INVALID_ARG;
    }
    if (M >= INT32_MAX || K >= INT32_MAX || N >= INT32_MAX || K * N >= ((int64_t)1 << 38)) {
        set_error("sizes must stay below 2^31-1 and K*N below 2^38");
        return FASTGL_ERR_UNSUPPORTED;
    }
    return FASTGL_OK;
}

bool misaligned(const void *p) { return ((uintptr_t)p & 3) != 0; }

size_t bwd_workspace(int64_t M, int64_t K, int64_t N)
{
    const int64_t nslab = ceil_div(M, kSlabRows);
    return align_up((size_t)nslab * (size_t)(K * N + N) * sizeof(float), 256);
}

}  // namespace
}  // namespace fastgl

using namespace fastgl;

extern "C" {

fastgl_status fastgl_update_fwd(const float *H, const float *W, const float *bias, int64_t M, int64_t K,
                                int64_t N, int relu, float *Y, void *stream)
{
    fastgl_status st = check_dims(M, K, N);
    if (st != FASTGL_OK) return st;
    if (M == 0 || N == 0) return FASTGL_OK;
    if (!Y || (K > 0 && (!H || !W))) {
        set_error("H, W or Y is NULL");
        return FASTGL_ERR_INVALID_ARG;
    }
    if (misaligned(H) || misaligned(W) || misaligned(bias) || misaligned(Y)) {
        set_error("matrices must be 4-byte aligned");
        return FASTGL_ERR_INVALID_ARG;
    }
    GemmArgs g = {};
    g.a = Operand{H, nullptr, K, vec_ok(H, nullptr, K)};
    g.b = Operand{W, nullptr, N, vec_ok(W, nullptr, N)};
    g.c = Y; g.ldc = N;
    g.R = M; g.C = N; g.Kc = K; g.slab = K;
    g.bias = bias; g.relu = relu != 0;
    return launch_gemm<false, true>(g, (hipStream_t)stream, "fastgl_update_fwd");
}

size_t fastgl_update_bwd_workspace_bytes(int64_t M, int64_t K, int64_t N)
{
    if (M < 0 || K < 0 || N < 0) return 0;
    return bwd_workspace(M, K, N);
}

fastgl_status fastgl_update_bwd(const float *H, const float *W, const float *Y, const float *dY, int64_t M,
                                int64_t K, int64_t N, int relu, float *dH, float *dW, float *db,
                                void *workspace, size_t workspace_bytes, void *stream)
{
    fastgl_status st = check_dims(M, K, N);
    if (st != FASTGL_OK) return st;
    const bool want_w = (dW && K > 0 && N > 0) || (db && N > 0);
    if ((M > 0 && N > 0 && !dY) || (relu && M > 0 && N > 0 && !Y)) {
        set_error("dY is NULL, or relu is set and Y is NULL");
        return FASTGL_ERR_INVALID_ARG;
    }
    if (dH && M > 0 && K > 0 && N > 0 && !W) {
        set_error("dH needs W");
        return FASTGL_ERR_INVALID_ARG;
    }
    if (dW && M > 0 && K > 0 && N > 0 && !H) {
        set_error("dW needs H");
        return FASTGL_ERR_INVALID_ARG;
    }
    if (misaligned(H) || misaligned(W) || misaligned(Y) || misaligned(dY) || misaligned(dH) || misaligned(dW) ||
        misaligned(db)) {
        set_error("matrices must be 4-byte aligned");
        return FASTGL_ERR_INVALID_ARG;
    }
    const size_t need = want_w ? bwd_workspace(M, K, N) : 0;
    if (want_w && need > 0) {
        if (!workspace || ((uintptr_t)workspace & 255)) {
            set_error("workspace must be a 256-byte aligned device buffer");
            return FASTGL_ERR_INVALID_ARG;
        }
        if (workspace_bytes < need) {
            set_error("workspace too small: %zu < %zu bytes", workspace_bytes, need);
            return FASTGL_ERR_WORKSPACE;
        }
    }
    hipStream_t s = (hipStream_t)stream;
    const float *gate = relu ? Y : nullptr;

    if (dH && M > 0 && K > 0) {
        // dH[m][k] = sum_n dZ[m][n] W[k][n]: both operands have the contracted index contiguous.
        GemmArgs g = {};
        g.a = Operand{dY, gate, N, vec_ok(dY, gate, N)};
        g.b = Operand{W, nullptr, N, vec_ok(W, nullptr, N)};
        g.c = dH; g.ldc = K;
        g.R = M; g.C = K; g.Kc = N; g.slab = N;
        st = launch_gemm<false, false>(g, s, "fastgl_update_bwd (dH)");
        if (st != FASTGL_OK) return st;
    }
    if (want_w) {
        // dW[k][n] = sum_m H[m][k] dZ[m][n], db[n] = sum_m dZ[m][n]: slabs of rows m, partials per slab.
        const int64_t nslab = ceil_div(M, kSlabRows);
        const int64_t stride = K * N + N;
        float *part = (float *)workspace;
        if (nslab > 0) {
            GemmArgs g = {};
            g.a = Operand{H, nullptr, K, vec_ok(H, nullptr, K)};
            g.b = Operand{dY, gate, N, vec_ok(dY, gate, N)};
            g.c = part; g.ldc = N; g.c_slab = stride;
            g.R = K; g.C = N; g.Kc = M; g.slab = kSlabRows;
            g.split = 1; g.n_outer = nslab;
            g.colsum = part + K * N; g.colsum_slab = stride;
            st = launch_gemm<true, true>(g, s, "fastgl_update_bwd (dW)");
            if (st != FASTGL_OK) return st;
        }
        const int64_t n_w = K * N, total = n_w + N;
        hipLaunchKernelGGL(k_update_reduce, dim3((unsigned)ceil_div(total, 256)), dim3(256), 0, s, part, nslab,
                           stride, n_w, N, dW, db);
        FASTGL_LAUNCH_CHECK("fastgl_update_bwd (reduce)");
    }
    return FASTGL_OK;
}

int32_t fastgl_update_slab_rows(void) { return kSlabRows; }

}  // extern "C"
