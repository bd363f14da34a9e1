// Update phase of a sampled GCN layer (paper Section 2.1, Eq. 2) on the matrix cores of gfx950:
// Y = act(H W + b) and its three gradients.  See include/fastgl_update.h for the contract of every
// entry point.
//
// One tiled kernel serves all four products.  A workgroup of 4 wavefronts owns a 128 x 128 tile of
// the result (each wavefront a 64 x 64 quarter = 2 x 2 accumulators of v_mfma_f32_32x32x16_bf16)
// and walks the contracted dimension in steps of 16, staged through two LDS buffers; three
// workgroups share a compute unit.
//
// The bf16 instruction runs at 16 times the rate of the fp32 one, so fp32 operands are not
// multiplied as fp32: an element x is cut into three bf16 planes, x = x1 + x2 + x3 exactly
// (x1 = bf16(x), x2 = bf16(x - x1), x3 = x - x1 - x2: 8 + 8 + 8 significant bits, each rounding to
// nearest, so |x2| <= 2^-8 |x| and |x3| <= 2^-16 |x|), when a tile is written to LDS.  Of the nine
// plane products six are kept: a1 b3, a3 b1, a2 b2, a1 b2, a2 b1, a1 b1 (smallest first, all into
// the same fp32 accumulator); the three dropped ones are below 2^-23 |a||b| together, and below
// 2^-28 |a||b| on average.  bf16 storage needs one plane and one product.  An element that is not
// finite, or beyond the largest bf16 (3.39e38), turns the results it enters into NaN.
//
// Each operand is copied to LDS from the layout it has in memory, so both kinds of operand get
// coalesced global loads.  One plane of an operand tile (128 out x 16 contracted) in LDS:
//   "row" operand   mem[out][contract]: 32 bytes per out index; the two 16-byte halves (contracted
//                   0..7, 8..15) swap places where bit 2 ^ bit 3 of the out index is set
//                   (conflict-free 16-byte reads)
//   "col" operand   mem[contract][out]: [pair p = contracted 2p, 2p+1][out] dwords, 128 + 8 per pair
// Lane half h (lanes 32h..32h+31) multiplies contracted indices 8h .. 8h+7 of both operands.
#include "fastgl_update.h"
#include "internal.h"

namespace fastgl {
namespace {

constexpr int kTile = 128;              // rows and columns of a workgroup's result tile
constexpr int kStep = 16;               // contracted indices per LDS stage
constexpr int kMaxSlabRows = 2048;      // most rows of H per dW / db partial
constexpr int kMinSlabRows = 32;
constexpr int kSlabRowStep = 32;        // slab heights considered: 32, 64, ..., 2048
constexpr int kRoundSlots = 768;        // workgroups the device this is tuned for holds at once (256 CUs x 3)

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

// Writes a wavefront's 64 x 64 quarter of the result tile at (r0, c0): bias, activation, rounding.
// Accumulator element e of lane (h, l32) is row 8*(e/4) + 4*h + e%4, column l32 of its 32 x 32 tile.
// Y and dH of a bf16 call are bf16; slab partials are always fp32.  Y and dH leave with streaming
// stores (STREAM); slab partials are re-read at once.
template <bool OUT_BF16, bool STREAM>
__device__ __forceinline__ void write_tile(const GemmArgs &g, const f32x16 (&acc)[2][2], int64_t r0, int64_t c0,
                                           int64_t slab_id, int wr, int wc, int h, int l32)
{
    const int64_t row0 = r0 + wr * 64 + 4 * h, col0 = c0 + wc * 64 + l32;
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
}

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

constexpr int kPairStride = kTile + 8;                        // dwords between pairs of a "col" plane
constexpr int kPlaneBytes = (kStep / 2) * kPairStride * 4;    // >= kTile * 32, the "row" plane
static_assert(kPlaneBytes >= kTile * 32 && kStep == 16, "plane size");

__device__ __forceinline__ int row_swizzle(int o) { return ((o >> 2) ^ (o >> 3)) & 1; }

// Planes of the pair (x0, x1), packed as two bf16 per dword (x0 in the low half).
template <int PLANES>
__device__ __forceinline__ void split_pair(float x0, float x1, uint32_t (&w)[PLANES])
{
#pragma unroll
    for (int p = 0; p < PLANES; ++p) {
        const bf16x2 b = {(__bf16)x0, (__bf16)x1};
        w[p] = __builtin_bit_cast(uint32_t, b);
        if (p + 1 < PLANES) {
            x0 -= __uint_as_float(w[p] << 16);
            x1 -= __uint_as_float(w[p] & 0xFFFF0000u);
        }
    }
}

// One 128 (out) x 16 (contracted) operand tile: global -> registers (fetch), registers -> bf16
// planes in LDS (stage).  "row": lane t holds contracted 4(t%4)..+3 of out indices t/4 and t/4 + 64;
// "col": lane t holds out indices 4(t%32)..+3 of contracted 2(t/32) and 2(t/32) + 1.  SUM keeps a
// running sum per held out index of everything staged ("col" only).  MASK = false is for whole steps
// of tiles that lie inside the matrices: no lane masks at all.
template <bool COL, bool VEC, bool GATE, bool BF16, int PLANES, bool SUM>
struct PlaneMover {
    typedef typename QuadBits<BF16>::elem E;
    Quad<GATE, BF16> r[2];      // [slot]
    uint32_t off[2];
    int nv_out;             // row: bit s set if slot s is an existing out index; col: quad elements in range
    int64_t ld, o0;
    const E *p, *gate;
    float sum[SUM ? 4 : 1];

    __device__ __forceinline__ void init(const Operand &op, int64_t o0_, int64_t omax)
    {
        static_assert(!SUM || COL, "running sums are kept for col operands");
        const int t = threadIdx.x;
        ld = op.ld; o0 = o0_; p = static_cast<const E *>(op.p); gate = static_cast<const E *>(op.gate);
        nv_out = 0;
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            if (!COL) {
                const int dr = t / 4 + 64 * s;
                off[s] = (uint32_t)dr * (uint32_t)ld + 4u * (t % 4);
                if (o0 + dr < omax) nv_out |= 1 << s;
            } else {
                off[s] = (uint32_t)(2 * (t >> 5) + s) * (uint32_t)ld + 4u * (t & 31);
            }
        }
        if (COL) nv_out = clamp4(omax - (o0 + 4 * (t & 31)));
#pragma unroll
        for (int j = 0; j < (SUM ? 4 : 1); ++j) sum[j] = 0.f;
    }

    template <bool MASK>
    __device__ __forceinline__ int nvalid(int s, int64_t k0, int64_t kend) const
    {
        if (!MASK) return 4;
        const int t = threadIdx.x;
        if (!COL) return (nv_out >> s) & 1 ? clamp4(kend - (k0 + 4 * (t % 4))) : 0;
        return k0 + 2 * (t >> 5) + s < kend ? nv_out : 0;
    }

    template <bool MASK>
    __device__ __forceinline__ void fetch(int64_t k0, int64_t kend)
    {
        // A step beyond kend has no element; its (all masked) loads go to contracted index 0 of the
        // tile's first out index, an element that exists whenever the operand has any (the host
        // substitutes a readable pointer when it has none).
        const int64_t kf = k0 < kend ? k0 : 0;                         // uniform
        const int64_t origin = COL ? kf * ld + o0 : o0 * ld + kf;      // uniform
#pragma unroll
        for (int s = 0; s < 2; ++s)
            load_quad<VEC, GATE, BF16>(p + origin, GATE ? gate + origin : nullptr, off[s],
                                       nvalid<MASK>(s, k0, kend), r[s]);
    }

    // (k0, kend) must be those of the fetch that filled the register set.
    template <bool MASK>
    __device__ __forceinline__ void stage(char *lds, int64_t k0, int64_t kend)
    {
        const int t = threadIdx.x;
        const float4 v0 = mask_quad<GATE, BF16>(r[0], nvalid<MASK>(0, k0, kend));
        const float4 v1 = mask_quad<GATE, BF16>(r[1], nvalid<MASK>(1, k0, kend));
        if (!COL) {
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                const float4 v = s == 0 ? v0 : v1;
                const int o = t / 4 + 64 * s, kq = t % 4;
                uint32_t lo[PLANES], hi[PLANES];
                split_pair<PLANES>(v.x, v.y, lo);
                split_pair<PLANES>(v.z, v.w, hi);
                char *dst = lds + o * 32 + 16 * ((kq >> 1) ^ row_swizzle(o)) + 8 * (kq & 1);
#pragma unroll
                for (int pl = 0; pl < PLANES; ++pl)
                    *reinterpret_cast<uint2 *>(dst + pl * kPlaneBytes) = make_uint2(lo[pl], hi[pl]);
            }
        } else {
            uint32_t w[4][PLANES];
            split_pair<PLANES>(v0.x, v1.x, w[0]);
            split_pair<PLANES>(v0.y, v1.y, w[1]);
            split_pair<PLANES>(v0.z, v1.z, w[2]);
            split_pair<PLANES>(v0.w, v1.w, w[3]);
            char *dst = lds + ((t >> 5) * kPairStride + 4 * (t & 31)) * 4;
#pragma unroll
            for (int pl = 0; pl < PLANES; ++pl)
                *reinterpret_cast<uint4 *>(dst + pl * kPlaneBytes) = make_uint4(w[0][pl], w[1][pl], w[2][pl], w[3][pl]);
            if (SUM) {
                sum[0] += v0.x + v1.x;
                sum[1] += v0.y + v1.y;
                sum[2] += v0.z + v1.z;
                sum[3] += v0.w + v1.w;
            }
        }
    }
};

// The eight values (contracted indices 8h .. 8h+7) of out index o in one plane.
template <bool COL>
__device__ __forceinline__ uint4 read_plane(const char *plane, int o, int h)
{
    if (!COL) return *reinterpret_cast<const uint4 *>(plane + o * 32 + 16 * (h ^ row_swizzle(o)));
    const uint32_t *q = reinterpret_cast<const uint32_t *>(plane) + 4 * h * kPairStride + o;
    return make_uint4(q[0], q[kPairStride], q[2 * kPairStride], q[3 * kPairStride]);
}

// A wavefront's fragments of one step: [operand a / b][32-wide fragment][plane].
template <int PLANES>
struct Frags {
    uint4 a[2][PLANES], b[2][PLANES];
};

template <bool A_COL, bool B_COL, int PLANES>
__device__ __forceinline__ void read_frags(const char *la, const char *lb, int wr, int wc, int l32, int h,
                                           Frags<PLANES> &f)
{
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int pl = 0; pl < PLANES; ++pl) {
            f.a[i][pl] = read_plane<A_COL>(la + pl * kPlaneBytes, wr * 64 + i * 32 + l32, h);
            f.b[i][pl] = read_plane<B_COL>(lb + pl * kPlaneBytes, wc * 64 + i * 32 + l32, h);
        }
}

// All MFMAs of one step; consecutive MFMAs go to different accumulators.
template <int PLANES>
__device__ __forceinline__ void mma_frags(const Frags<PLANES> &f, f32x16 (&acc)[2][2])
{
    constexpr int kTerms = PLANES == 3 ? 6 : 1;
    constexpr int pa[6] = {0, 2, 1, 0, 1, 0}, pb[6] = {2, 0, 1, 1, 0, 0};
#pragma unroll
    for (int t = 0; t < kTerms; ++t)
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int x = PLANES == 3 ? pa[t] : 0, y = PLANES == 3 ? pb[t] : 0;
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, f.a[i][x]),
                                                                   __builtin_bit_cast(bf16x8, f.b[j][y]), acc[i][j], 0, 0, 0);
            }
}

// One step of the contracted range: the loads of the next step are issued, this step is multiplied
// out of LDS buffer `cur`, and the next one is split into the other buffer.  No branch inside.
template <bool MASK, bool A_COL, bool B_COL, int PLANES, class MoverA, class MoverB>
__device__ __forceinline__ void one_step(MoverA &ma, MoverB &mb, char *la, char *lb, int cur, int operand_bytes,
                                         int64_t k0, int64_t kend, int wr, int wc, int l32, int h,
                                         f32x16 (&acc)[2][2])
{
    ma.template fetch<MASK>(k0 + kStep, kend);
    mb.template fetch<MASK>(k0 + kStep, kend);
    __builtin_amdgcn_sched_barrier(0);       // the loads stay ahead of the step's other work
    Frags<PLANES> f;
    read_frags<A_COL, B_COL, PLANES>(la + cur * operand_bytes, lb + cur * operand_bytes, wr, wc, l32, h, f);
    mma_frags<PLANES>(f, acc);
    ma.template stage<MASK>(la + (cur ^ 1) * operand_bytes, k0 + kStep, kend);
    mb.template stage<MASK>(lb + (cur ^ 1) * operand_bytes, k0 + kStep, kend);
    __syncthreads();
}

// The contracted range [kbeg, kend) of one result tile.  The first n_plain steps touch nothing but
// whole steps of a tile that lies inside both operands (a step also loads and converts the one after
// it) and run without lane masks; the others, at least one, mask what does not exist - a step beyond
// kend is a step of zeros.  The MFMAs are not behind any condition other than the two loop counts:
// accumulators that can reach the end by a path without MFMAs are given a second set of registers
// by the compiler.
template <bool A_COL, bool B_COL, int PLANES, class MoverA, class MoverB>
__device__ __forceinline__ void run_steps(MoverA &ma, MoverB &mb, char *la, char *lb, int operand_bytes, int64_t kbeg,
                                          int64_t kend, bool inside, int wr, int wc, int l32, int h,
                                          f32x16 (&acc)[2][2])
{
    const int64_t len = kend > kbeg ? kend - kbeg : 0;
    const int64_t nstep = len > 0 ? (len + kStep - 1) / kStep : 1;
    int64_t n_plain = inside ? len / kStep - 1 : 0;
    n_plain = n_plain < 0 ? 0 : (n_plain > nstep - 1 ? nstep - 1 : n_plain);
    ma.template fetch<true>(kbeg, kend);
    mb.template fetch<true>(kbeg, kend);
    ma.template stage<true>(la, kbeg, kend);
    mb.template stage<true>(lb, kbeg, kend);
    __syncthreads();
    int64_t k0 = kbeg;
    int cur = 0;
    for (int64_t i = 0; i < n_plain; ++i, k0 += kStep, cur ^= 1)
        one_step<false, A_COL, B_COL, PLANES>(ma, mb, la, lb, cur, operand_bytes, k0, kend, wr, wc, l32, h, acc);
    int64_t i = n_plain;
    do {
        one_step<true, A_COL, B_COL, PLANES>(ma, mb, la, lb, cur, operand_bytes, k0, kend, wr, wc, l32, h, acc);
        k0 += kStep;
        cur ^= 1;
    } while (++i < nstep);
}

template <bool A_COL, bool B_COL, bool COLSUM, bool VEC, bool GATE_A, bool GATE_B, bool BF16>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(3, 3))) void k_update_gemm(const GemmArgs g)
{
    constexpr int PLANES = BF16 ? 1 : 3;
    constexpr int kOperandBytes = PLANES * kPlaneBytes;
    __shared__ __attribute__((aligned(16))) char lds_a[2][kOperandBytes];
    __shared__ __attribute__((aligned(16))) char lds_b[2][kOperandBytes];

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

    const bool inside = VEC && r0 + kTile <= g.R && c0 + kTile <= g.C;   // uniform
    f32x16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
    PlaneMover<A_COL, VEC, GATE_A, BF16, PLANES, false> ma;
    PlaneMover<B_COL, VEC, GATE_B, BF16, PLANES, COLSUM> mb;
    ma.init(g.a, r0, g.R);
    mb.init(g.b, c0, g.C);
    run_steps<A_COL, B_COL, PLANES>(ma, mb, lds_a[0], lds_b[0], kOperandBytes, kbeg, kend, inside, wr, wc, l32, h, acc);
    write_tile<BF16 && !COLSUM, !COLSUM>(g, acc, r0, c0, slab_id, wr, wc, h, l32);
    if (COLSUM && tile_r == 0) {
        // Every barrier above has been passed by all lanes, so the LDS is free: add up the eight
        // running sums of each column in a fixed order.
        float *red = reinterpret_cast<float *>(lds_b[0]);
        const int t = threadIdx.x;
        *reinterpret_cast<float4 *>(red + (t >> 5) * kTile + 4 * (t & 31)) =
            make_float4(mb.sum[0], mb.sum[1], mb.sum[2], mb.sum[3]);
        __syncthreads();
        if (t < kTile) {
            float s = red[t];
#pragma unroll
            for (int i = 1; i < 8; ++i) s += red[i * kTile + t];
            if (c0 + t < g.C) g.colsum[slab_id * g.colsum_slab + c0 + t] = s;
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
    if (g.Kc == 0) {           // nothing to contract: the same for both operands (the result exists)
        g.a.p = g.b.p = g.c;
        g.a.gate = g.b.gate = nullptr;
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
// The height that minimises a model of the launch: the (slab, tile) workgroups run in rounds of
// kRoundSlots, a workgroup costs its steps plus a fixed part, and every slab adds a partial result
// that is written once and read once by the reduction.  Integer arithmetic (picoseconds).
int64_t slab_rows(int64_t M, int64_t K, int64_t N)
{
    const int64_t tiles = (K > 0 ? ceil_div(K, kTile) : 1) * ceil_div(N, kTile);
    const int64_t partial = K * N + N;                 // floats per slab
    int64_t best = kMinSlabRows, best_cost = INT64_MAX;
    for (int64_t rows = kMinSlabRows; rows <= kMaxSlabRows; rows += kSlabRowStep) {
        const int64_t nslab = ceil_div(M > 0 ? M : 1, rows);
        const int64_t rounds = ceil_div(nslab * tiles, kRoundSlots);
        // 2.5 us per step of 16 rows with three workgroups on a CU, 8 steps' worth of prologue and
        // epilogue; 8 bytes of traffic per float of a partial at 4 TB/s
        const int64_t cost = rounds * (rows * 156250 + 20000000) + nslab * partial * 2;
        if (cost < best_cost) {
            best_cost = cost;
            best = rows;
        }
    }
    return best;
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
