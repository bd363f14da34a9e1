// Update phase of a sampled GCN layer (paper Section 2.1, Eq. 2) on the fp32
// matrix cores of gfx950: Y = act(H W + b) and its three gradients.  See
// include/fastgl_update.h for the contract of every entry point.
//
// One tiled kernel serves all four products.  A workgroup of 4 wavefronts owns
// a 128 x 128 tile of the result (each wavefront a 64 x 64 quarter = 2 x 2
// accumulators of v_mfma_f32_32x32x2_f32) and walks the contracted dimension in
// steps of 16, staged through two LDS buffers; at most 128 registers per lane, so
// four workgroups share a compute unit.  Each operand is copied to LDS in the layout
// it has in memory, so both kinds of operand get coalesced global loads:
//   "row" operand   mem[out][contract]  -> lds[out][16 + 4]  (read back 16 B per lane)
//   "col" operand   mem[contract][out]  -> lds[contract][128 + 8]
// Inside a group of 8 contracted indices lane half h (lanes 32h..32h+31) takes
// indices 4h..4h+3, and MFMA number t multiplies index 4h+t of both operands;
// the sum over the contracted index does not care about this order.
#include "fastgl_update.h"
#include "internal.h"

namespace fastgl {
namespace {

constexpr int kTile = 128;              // rows and columns of a workgroup's result tile
constexpr int kStep = 16;               // contracted indices per LDS stage
constexpr int kBuffers = 2;             // LDS stages (one barrier per stage with two)
constexpr int kLoads = kStep / 8;       // 16-byte loads per thread and operand tile
constexpr int kRowStride = kStep + 4;   // floats between rows of a "row" operand in LDS
constexpr int kColStride = kTile + 8;   // floats between contracted indices of a "col" operand
constexpr int kOperandFloats = (kTile * kRowStride > kStep * kColStride) ? kTile * kRowStride : kStep * kColStride;
constexpr int kMaxSlabRows = 1024;      // most rows of H per dW / db partial
constexpr int kMinSlabRows = 128;
constexpr int kSlabFill = 640;          // workgroups wanted before slabs stop shrinking

typedef float f32x16 __attribute__((ext_vector_type(16)));

struct Operand {
    const void *p;        // element (out o, contracted k) at p[o*ld + k] ("row") or p[k*ld + o] ("col")
    const void *gate;     // same layout, or NULL; where gate <= 0 the element reads as 0 (ReLU derivative)
    int64_t ld;           // fp32 or bf16 elements (the kernel's BF16 argument says which)
};

struct GemmArgs {
    Operand a, b;
    void *c;                    // [R][C] result (of slab s: c + s*c_slab): fp32, or bf16 for Y / dH of a bf16 call
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

// A quad = four consecutive elements p[off..off+3] of which the first `nvalid` exist; the rest must
// read as 0.  Loading and masking are split so that the loads of the next stage stay in flight
// during the MFMAs of the current one: load_quad only issues loads (no control flow around them - a
// load behind a branch is waited for at the join - and no arithmetic on the result); an element
// that does not exist is loaded from offset 0, which the host guarantees to be readable.
// mask_quad, called when the registers are written to LDS, zeroes what does not exist or is gated
// off.  VEC: one 16-byte load; the host selects it only when every extent is a multiple of 4, so
// nvalid is 0 or 4.
template <bool BF16>
struct QuadBits;
template <>
struct QuadBits<false> {
    typedef float4 type;
    typedef float elem;
};
template <>
struct QuadBits<true> {
    typedef uint2 type;           // four bf16
    typedef uint16_t elem;
};

template <bool GATE, bool BF16>
struct Quad {
    typename QuadBits<BF16>::type v;
    typename QuadBits<BF16>::type g[GATE ? 1 : 0];
};

__device__ __forceinline__ float4 quad_to_f32(float4 q) { return q; }
__device__ __forceinline__ float4 quad_to_f32(uint2 q)
{
    return make_float4(__uint_as_float(q.x << 16), __uint_as_float(q.x & 0xFFFF0000u), __uint_as_float(q.y << 16),
                       __uint_as_float(q.y & 0xFFFF0000u));
}

// `base` is uniform over the workgroup (the tile's origin), `off` a per-lane 32-bit element offset.
template <bool VEC, bool GATE, bool BF16>
__device__ __forceinline__ void load_quad(const void *__restrict__ base_, const void *__restrict__ gate_,
                                          uint32_t off, int nvalid, Quad<GATE, BF16> &q)
{
    typedef typename QuadBits<BF16>::type Q;
    typedef typename QuadBits<BF16>::elem E;
    const E *base = static_cast<const E *>(base_), *gate = static_cast<const E *>(gate_);
    if (VEC) {
        const uint32_t o = nvalid >= 4 ? off : 0u;
        q.v = *reinterpret_cast<const Q *>(base + o);
        if (GATE) q.g[0] = *reinterpret_cast<const Q *>(gate + o);
    } else {
        E e[4], f[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint32_t o = i < nvalid ? off + i : 0u;
            e[i] = base[o];
            if (GATE) f[i] = gate[o];
        }
        if constexpr (BF16) {
            q.v = make_uint2((uint32_t)e[0] | ((uint32_t)e[1] << 16), (uint32_t)e[2] | ((uint32_t)e[3] << 16));
            if (GATE) q.g[0] = make_uint2((uint32_t)f[0] | ((uint32_t)f[1] << 16), (uint32_t)f[2] | ((uint32_t)f[3] << 16));
        } else {
            q.v = make_float4(e[0], e[1], e[2], e[3]);
            if (GATE) q.g[0] = make_float4(f[0], f[1], f[2], f[3]);
        }
    }
}

template <bool GATE, bool BF16>
__device__ __forceinline__ float4 mask_quad(const Quad<GATE, BF16> &q, int nvalid)
{
    float4 v = quad_to_f32(q.v);
    if (GATE) {
        const float4 g = quad_to_f32(q.g[0]);
        v.x = g.x > 0.f ? v.x : 0.f;
        v.y = g.y > 0.f ? v.y : 0.f;
        v.z = g.z > 0.f ? v.z : 0.f;
        v.w = g.w > 0.f ? v.w : 0.f;
    }
    v.x = nvalid > 0 ? v.x : 0.f;
    v.y = nvalid > 1 ? v.y : 0.f;
    v.z = nvalid > 2 ? v.z : 0.f;
    v.w = nvalid > 3 ? v.w : 0.f;
    return v;
}

// fp32 -> bf16, round to nearest even (NaN stays NaN).
__device__ __forceinline__ uint16_t f32_to_bf16(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x0040u);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

__device__ __forceinline__ int clamp4(int64_t n) { return n >= 4 ? 4 : (n <= 0 ? 0 : (int)n); }

// One 128 (out) x kStep (contracted) operand tile: global -> registers (fetch), registers -> LDS
// (stage).  "row" operand: kStep/4 lanes cover the contracted indices of one out index and slot s
// is out index t/(kStep/4) + s*(1024/kStep); "col" operand: 32 lanes cover the 128 out indices of
// one contracted index and slot s is contracted index t/32 + 8s.  Lane offsets are relative to
// the tile's origin and stay the same from stage to stage (the host keeps 160*ld below 2^32).
template <bool COL, bool VEC, bool GATE, bool BF16>
struct TileMover {
    static constexpr int kq_n = kStep / 4, rows = 256 / kq_n;
    typedef typename QuadBits<BF16>::elem E;
    Quad<GATE, BF16> r[kLoads];
    uint32_t off[kLoads];   // element offset of slot s from the tile origin
    int nv_out;             // row: bit s set if slot s is an existing out index; col: quad elements in range
    int64_t ld, o0;
    const E *p, *gate;

    __device__ __forceinline__ void init(const Operand &op, int64_t o0_, int64_t omax)
    {
        const int t = threadIdx.x;
        ld = op.ld; o0 = o0_; p = static_cast<const E *>(op.p); gate = static_cast<const E *>(op.gate);
        nv_out = 0;
#pragma unroll
        for (int s = 0; s < kLoads; ++s) {
            if (!COL) {
                const int dr = t / kq_n + rows * s;
                off[s] = (uint32_t)dr * (uint32_t)ld + 4u * (t % kq_n);
                if (o0 + dr < omax) nv_out |= 1 << s;
            } else {
                off[s] = (uint32_t)((t >> 5) + 8 * s) * (uint32_t)ld + 4u * (t & 31);
            }
        }
        if (COL) nv_out = clamp4(omax - (o0 + 4 * (t & 31)));
    }

    __device__ __forceinline__ int nvalid(int s, int64_t k0, int64_t kend) const
    {
        const int t = threadIdx.x;
        if (!COL) return (nv_out >> s) & 1 ? clamp4(kend - (k0 + 4 * (t % kq_n))) : 0;
        return k0 + (t >> 5) + 8 * s < kend ? nv_out : 0;
    }

    __device__ __forceinline__ void fetch(int64_t k0, int64_t kend)
    {
        const int64_t origin = COL ? k0 * ld + o0 : o0 * ld + k0;      // uniform
#pragma unroll
        for (int s = 0; s < kLoads; ++s)
            load_quad<VEC, GATE, BF16>(p + origin, GATE ? gate + origin : nullptr, off[s], nvalid(s, k0, kend), r[s]);
    }

    // (k0, kend) must be those of the fetch that filled the registers.
    __device__ __forceinline__ void stage(float *lds, int64_t k0, int64_t kend) const
    {
        const int t = threadIdx.x;
#pragma unroll
        for (int s = 0; s < kLoads; ++s) {
            const float4 v = mask_quad<GATE, BF16>(r[s], nvalid(s, k0, kend));
            if (!COL)
                *reinterpret_cast<float4 *>(lds + (t / kq_n + rows * s) * kRowStride + 4 * (t % kq_n)) = v;
            else
                *reinterpret_cast<float4 *>(lds + ((t >> 5) + 8 * s) * kColStride + 4 * (t & 31)) = v;
        }
    }
};

// The four values (contracted indices 8c+4h .. 8c+4h+3) of out index o.
template <bool COL>
__device__ __forceinline__ float4 read_frag(const float *lds, int o, int c, int h)
{
    if (!COL) return *reinterpret_cast<const float4 *>(lds + o * kRowStride + 8 * c + 4 * h);
    const float *q = lds + (8 * c + 4 * h) * kColStride + o;
    return make_float4(q[0], q[kColStride], q[2 * kColStride], q[3 * kColStride]);
}

// The MFMAs of one group of 8 contracted indices; consecutive MFMAs go to different accumulators.
__device__ __forceinline__ void mma_group(const float4 (&fa)[2], const float4 (&fb)[2], f32x16 (&acc)[2][2])
{
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const float av = t == 0 ? fa[i].x : t == 1 ? fa[i].y : t == 2 ? fa[i].z : fa[i].w;
                const float bv = t == 0 ? fb[j].x : t == 1 ? fb[j].y : t == 2 ? fb[j].z : fb[j].w;
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv, acc[i][j], 0, 0, 0);
            }
}

// All MFMAs of `nchunk` groups of 8 contracted indices of the staged tiles.
template <bool A_COL, bool B_COL, bool COLSUM>
__device__ __forceinline__ void mma_stage(const float *la, const float *lb, int nchunk, int wr, int wc, int l32,
                                          int h, f32x16 (&acc)[2][2], float (&bsum)[2])
{
#pragma unroll 1
    for (int c = 0; c < nchunk; ++c) {
        float4 fa[2], fb[2];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            fa[i] = read_frag<A_COL>(la, wr * 64 + i * 32 + l32, c, h);
            fb[i] = read_frag<B_COL>(lb, wc * 64 + i * 32 + l32, c, h);
        }
        if (COLSUM) {
#pragma unroll
            for (int j = 0; j < 2; ++j) bsum[j] += (fb[j].x + fb[j].y) + (fb[j].z + fb[j].w);
        }
        mma_group(fa, fb, acc);
    }
}

template <bool A_COL, bool B_COL, bool COLSUM, bool VEC, bool GATE_A, bool GATE_B, bool BF16>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(4, 4))) void k_update_gemm(const GemmArgs g)
{
    __shared__ __attribute__((aligned(16))) float lds_a[kBuffers][kOperandFloats];
    __shared__ __attribute__((aligned(16))) float lds_b[kBuffers][kOperandFloats];

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

    TileMover<A_COL, VEC, GATE_A, BF16> ma;
    TileMover<B_COL, VEC, GATE_B, BF16> mb;
    ma.init(g.a, r0, g.R);
    mb.init(g.b, c0, g.C);
    if (kbeg < kend) {
        ma.fetch(kbeg, kend);
        mb.fetch(kbeg, kend);
        ma.stage(lds_a[0], kbeg, kend);
        mb.stage(lds_b[0], kbeg, kend);
        __syncthreads();
    }
    int buf = 0;
    for (int64_t k0 = kbeg; k0 < kend; k0 += kStep) {
        const bool more = k0 + kStep < kend;
        if (more) {                                // next stage's global loads fly during the MFMAs
            ma.fetch(k0 + kStep, kend);
            mb.fetch(k0 + kStep, kend);
        }
        const int64_t left = kend - k0;
        mma_stage<A_COL, B_COL, COLSUM>(lds_a[buf], lds_b[buf], left >= kStep ? kStep / 8 : (int)((left + 7) / 8), wr,
                                        wc, l32, h, acc, bsum);
        if (kBuffers == 1) __syncthreads();
        const int nb = kBuffers == 1 ? 0 : buf ^ 1;
        if (more) {
            ma.stage(lds_a[nb], k0 + kStep, kend);
            mb.stage(lds_b[nb], k0 + kStep, kend);
        }
        __syncthreads();
        buf = nb;
    }

    // Accumulator element e of lane (h, l32) is row 8*(e/4) + 4*h + e%4, column l32 of its 32 x 32 tile.
    const int64_t row0 = r0 + wr * 64 + 4 * h, col0 = c0 + wc * 64 + l32;
    // Y and dH of a bf16 call are bf16; slab partials are always fp32.  Y and dH leave with streaming
    // stores; slab partials are re-read at once.
    constexpr bool OUT_BF16 = BF16 && !COLSUM, STREAM = !COLSUM;
    typedef typename QuadBits<OUT_BF16>::elem OutT;
    OutT *cb = static_cast<OutT *>(g.c) + slab_id * g.c_slab + row0 * g.ldc + col0;
    const bool relu = g.relu != 0;
    auto put = [](OutT *dst, float v, bool stream) {
        if constexpr (OUT_BF16) {
            const uint16_t w = f32_to_bf16(v);
            if (stream) __builtin_nontemporal_store(w, dst); else *dst = w;
        } else {
            if (stream) __builtin_nontemporal_store(v, dst); else *dst = v;
        }
    };
    if (r0 + kTile <= g.R && c0 + kTile <= g.C) {
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const float bj = g.bias ? g.bias[col0 + 32 * j] : 0.f;
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    float v = acc[i][j][e] + bj;
                    if (relu) v = v > 0.f ? v : 0.f;
                    put(&cb[(int64_t)(32 * i + 8 * (e >> 2) + (e & 3)) * g.ldc + 32 * j], v, STREAM);
                }
        }
    } else {
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int64_t col = col0 + 32 * j;
            if (col >= g.C) continue;
            const float bj = g.bias ? g.bias[col] : 0.f;
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int dr = 32 * i + 8 * (e >> 2) + (e & 3);
                    if (row0 + dr >= g.R) continue;
                    float v = acc[i][j][e] + bj;
                    if (relu) v = v > 0.f ? v : 0.f;
                    put(&cb[(int64_t)dr * g.ldc + 32 * j], v, false);
                }
        }
    }
    if (COLSUM && tile_r == 0 && wr == 0) {
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const float s = bsum[j] + __shfl_xor(bsum[j], 32);
            const int64_t col = c0 + wc * 64 + j * 32 + l32;
            if (h == 0 && col < g.C) g.colsum[slab_id * g.colsum_slab + col] = s;
        }
    }
}

// out[e] = sum over slabs of part[s*stride + e], in fp64 and in a fixed order: the slabs are cut into
// kReduceParts consecutive ranges, each summed in slab order by one thread, and the range sums are
// added in range order.  The first n_w elements go to dW, the remaining n_b to db (either may be NULL).
constexpr int kReduceParts = 8, kReduceElems = 256 / kReduceParts;

__global__ __launch_bounds__(256) void k_update_reduce(const float *__restrict__ part, int64_t nslab, int64_t stride,
                                                       int64_t n_w, int64_t n_b, float *dW, float *db)
{
    __shared__ double partial[kReduceParts][kReduceElems];
    const int el = threadIdx.x % kReduceElems, pt = threadIdx.x / kReduceElems;
    const int64_t e = (int64_t)blockIdx.x * kReduceElems + el;
    const int64_t per = (nslab + kReduceParts - 1) / kReduceParts;
    const int64_t lo = pt * per, hi = lo + per < nslab ? lo + per : nslab;
    double s = 0.0;
    if (e < n_w + n_b) {
        const float *q = part + e;
        int64_t k = lo;
        for (; k + 4 <= hi; k += 4) {
            const float v0 = q[k * stride], v1 = q[(k + 1) * stride], v2 = q[(k + 2) * stride],
                        v3 = q[(k + 3) * stride];
            s += (double)v0;
            s += (double)v1;
            s += (double)v2;
            s += (double)v3;
        }
        for (; k < hi; ++k) s += (double)q[k * stride];
    }
    partial[pt][el] = s;
    __syncthreads();
    if (pt != 0 || e >= n_w + n_b) return;
    double t = partial[0][el];
#pragma unroll
    for (int i = 1; i < kReduceParts; ++i) t += partial[i][el];
    float *dst = e < n_w ? (dW ? dW + e : nullptr) : (db ? db + (e - n_w) : nullptr);
    if (dst) *dst = (float)t;
}

// Quad loads (16 bytes of fp32, 8 bytes of bf16) need every row of the operand to start aligned to a
// quad and to hold whole quads.
bool quad_ok(const Operand &op, bool bf16)
{
    const uintptr_t m = bf16 ? 7 : 15;
    return op.p && op.ld % 4 == 0 && (((uintptr_t)op.p | (uintptr_t)op.gate) & m) == 0;
}

// WHICH names the operand that may carry a gate: 0 none, 1 a, 2 b.
template <bool A_COL, bool B_COL, bool COLSUM, int WHICH, bool VEC, bool BF16>
void launch_gates(const GemmArgs &g, unsigned blocks, hipStream_t s)
{
    if (WHICH == 1 && g.a.gate)
        hipLaunchKernelGGL((k_update_gemm<A_COL, B_COL, COLSUM, VEC, WHICH == 1, false, BF16>), dim3(blocks), dim3(256),
                           0, s, g);
    else if (WHICH == 2 && g.b.gate)
        hipLaunchKernelGGL((k_update_gemm<A_COL, B_COL, COLSUM, VEC, false, WHICH == 2, BF16>), dim3(blocks), dim3(256),
                           0, s, g);
    else
        hipLaunchKernelGGL((k_update_gemm<A_COL, B_COL, COLSUM, VEC, false, false, BF16>), dim3(blocks), dim3(256), 0, s,
                           g);
}

template <bool A_COL, bool B_COL, bool COLSUM, int WHICH>
fastgl_status launch_gemm(GemmArgs &g, bool bf16, hipStream_t s, const char *what)
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
    bool vec = quad_ok(g.a, bf16) && quad_ok(g.b, bf16);
    if (g.R == 0) {            // operand a has no elements: give its (all masked) loads a readable address
        g.a.p = g.b.p;
        g.a.gate = nullptr;
        vec = false;
    }
    const unsigned nb = (unsigned)blocks;
    if (bf16) {
        if (vec) launch_gates<A_COL, B_COL, COLSUM, WHICH, true, true>(g, nb, s);
        else launch_gates<A_COL, B_COL, COLSUM, WHICH, false, true>(g, nb, s);
    } else {
        if (vec) launch_gates<A_COL, B_COL, COLSUM, WHICH, true, false>(g, nb, s);
        else launch_gates<A_COL, B_COL, COLSUM, WHICH, false, false>(g, nb, s);
    }
    FASTGL_LAUNCH_CHECK(what);
    return FASTGL_OK;
}

fastgl_status check_dims(int64_t M, int64_t K, int64_t N)
{
    if (M < 0 || K < 0 || N < 0) {
        set_error("negative size (M=%lld K=%lld N=%lld)", (long long)M, (long long)K, (long long)N);
        return FASTGL_ERR_INVALID_ARG;
    }
    if (M >= INT32_MAX || K >= ((int64_t)1 << 24) || N >= ((int64_t)1 << 24)) {
        set_error("M must stay below 2^31-1, K and N below 2^24");
        return FASTGL_ERR_UNSUPPORTED;
    }
    return FASTGL_OK;
}

// Rows per slab: a function of the shape alone, so results do not depend on the device or the run.
int64_t slab_rows(int64_t M, int64_t K, int64_t N)
{
    const int64_t tiles = (K > 0 ? ceil_div(K, kTile) : 1) * ceil_div(N, kTile);
    int64_t rows = kMaxSlabRows;
    while (rows > kMinSlabRows && ceil_div(M, rows) * tiles < kSlabFill) rows /= 2;
    return rows;
}

size_t bwd_workspace(int64_t M, int64_t K, int64_t N)
{
    const int64_t nslab = ceil_div(M, slab_rows(M, K, N));
    return align_up((size_t)nslab * (size_t)(K * N + N) * sizeof(float), 256);
}

}  // namespace
}  // namespace fastgl

using namespace fastgl;

namespace {

bool misaligned_to(const void *p, uintptr_t bytes) { return ((uintptr_t)p & (bytes - 1)) != 0; }

fastgl_status update_fwd(bool bf16, const void *H, const void *W, const float *bias, int64_t M, int64_t K, int64_t N,
                         int relu, void *Y, void *stream)
{
    fastgl_status st = check_dims(M, K, N);
    if (st != FASTGL_OK) return st;
    if (M == 0 || N == 0) return FASTGL_OK;
    if (!Y || (K > 0 && (!H || !W))) {
        set_error("H, W or Y is NULL");
        return FASTGL_ERR_INVALID_ARG;
    }
    const uintptr_t el = bf16 ? 2 : 4;
    if (misaligned_to(H, el) || misaligned_to(W, el) || misaligned_to(bias, 4) || misaligned_to(Y, el)) {
        set_error("matrices must be aligned to their element size");
        return FASTGL_ERR_INVALID_ARG;
    }
    GemmArgs g = {};
    g.a = Operand{H, nullptr, K};
    g.b = Operand{W, nullptr, N};
    g.c = Y; g.ldc = N;
    g.R = M; g.C = N; g.Kc = K; g.slab = K;
    g.bias = bias; g.relu = relu != 0;
    return launch_gemm<false, true, false, 0>(g, bf16, (hipStream_t)stream, "fastgl_update_fwd");
}

fastgl_status update_bwd(bool bf16, const void *H, const void *W, const void *Y, const void *dY, int64_t M, int64_t K,
                         int64_t N, int relu, void *dH, float *dW, float *db, void *workspace, size_t workspace_bytes,
                         void *stream)
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
    const uintptr_t el = bf16 ? 2 : 4;
    if (misaligned_to(H, el) || misaligned_to(W, el) || misaligned_to(Y, el) || misaligned_to(dY, el) ||
        misaligned_to(dH, el) || misaligned_to(dW, 4) || misaligned_to(db, 4)) {
        set_error("matrices must be aligned to their element size");
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
    const void *gate = relu ? Y : nullptr;

    if (dH && M > 0 && K > 0) {
        // dH[m][k] = sum_n dZ[m][n] W[k][n]: both operands have the contracted index contiguous.
        GemmArgs g = {};
        g.a = Operand{dY, gate, N};
        g.b = Operand{W, nullptr, N};
        g.c = dH; g.ldc = K;
        g.R = M; g.C = K; g.Kc = N; g.slab = N;
        st = launch_gemm<false, false, false, 1>(g, bf16, s, "fastgl_update_bwd (dH)");
        if (st != FASTGL_OK) return st;
    }
    if (want_w) {
        // dW[k][n] = sum_m H[m][k] dZ[m][n], db[n] = sum_m dZ[m][n]: slabs of rows m, partials per slab.
        const int64_t rows = slab_rows(M, K, N), nslab = ceil_div(M, rows);
        const int64_t stride = K * N + N;
        float *part = (float *)workspace;
        if (nslab > 0) {
            GemmArgs g = {};
            g.a = Operand{H, nullptr, K};
            g.b = Operand{dY, gate, N};
            g.c = part; g.ldc = N; g.c_slab = stride;
            g.R = K; g.C = N; g.Kc = M; g.slab = rows;
            g.split = 1; g.n_outer = nslab;
            g.colsum = part + K * N; g.colsum_slab = stride;
            st = launch_gemm<true, true, true, 2>(g, bf16, s, "fastgl_update_bwd (dW)");
            if (st != FASTGL_OK) return st;
        }
        const int64_t n_w = K * N, total = n_w + N;
        hipLaunchKernelGGL(k_update_reduce, dim3((unsigned)ceil_div(total, kReduceElems)), dim3(256), 0, s, part, nslab,
                           stride, n_w, N, dW, db);
        FASTGL_LAUNCH_CHECK("fastgl_update_bwd (reduce)");
    }
    return FASTGL_OK;
}

}  // namespace

extern "C" {

fastgl_status fastgl_update_fwd(const float *H, const float *W, const float *bias, int64_t M, int64_t K,
                                int64_t N, int relu, float *Y, void *stream)
{
    return update_fwd(false, H, W, bias, M, K, N, relu, Y, stream);
}

fastgl_status fastgl_update_fwd_bf16(const uint16_t *H, const uint16_t *W, const float *bias, int64_t M, int64_t K,
                                     int64_t N, int relu, uint16_t *Y, void *stream)
{
    return update_fwd(true, H, W, bias, M, K, N, relu, Y, stream);
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
    return update_bwd(false, H, W, Y, dY, M, K, N, relu, dH, dW, db, workspace, workspace_bytes, stream);
}

fastgl_status fastgl_update_bwd_bf16(const uint16_t *H, const uint16_t *W, const uint16_t *Y, const uint16_t *dY,
                                     int64_t M, int64_t K, int64_t N, int relu, uint16_t *dH, float *dW, float *db,
                                     void *workspace, size_t workspace_bytes, void *stream)
{
    return update_bwd(true, H, W, Y, dY, M, K, N, relu, dH, dW, db, workspace, workspace_bytes, stream);
}

int32_t fastgl_update_slab_rows(int64_t M, int64_t K, int64_t N)
{
    if (M < 0 || K < 0 || N < 0) return 0;
    return (int32_t)slab_rows(M, K, N);
}

}  // extern "C"
