// Device code shared by the aggregation kernels: how a lane holds a slice of a
// feature row (load, multiply-add, round, store) and how a group of lanes walks
// the edges of consecutive rows as one flat list.  Included by aggregate.hip (the
// pull kernel of paper Section 2.1 Eq. 1 / Section 4.2 Eq. 5) and layer.hip (the
// aggregation fused with the update of Eq. 2).
#pragma once
#include "internal.h"

namespace fastgl {

constexpr int kUnroll = 6;        // row gathers in flight per lane (wide groups)
constexpr int kUnrollNarrow = 4;  // groups of <= 16 lanes fetch <= 16 column ids at a time: 4 divides that

template <int DT> struct AccT { using type = double; };
template <> struct AccT<FASTGL_BF16> { using type = float; };

template <int DT, int VB> struct Slice {
    static constexpr int NW = VB >= 4 ? VB / 4 : 1;                           // 32-bit words held per lane
    static constexpr int NE = DT == FASTGL_F32 ? VB / 4 : VB / 2;             // elements per lane
    using acc_t = typename AccT<DT>::type;

    __device__ static __forceinline__ void load(const char *p, uint32_t (&r)[NW])
    {
        if constexpr (VB == 16) {
            uint4 v = *reinterpret_cast<const uint4 *>(p);
            r[0] = v.x; r[1] = v.y; r[2] = v.z; r[3] = v.w;
        } else if constexpr (VB == 8) {
            uint2 v = *reinterpret_cast<const uint2 *>(p);
            r[0] = v.x; r[1] = v.y;
        } else if constexpr (VB == 4) {
            r[0] = *reinterpret_cast<const uint32_t *>(p);
        } else {
            r[0] = *reinterpret_cast<const uint16_t *>(p);
        }
    }

    template <bool HASW>
    __device__ static __forceinline__ void fma(acc_t (&acc)[NE], const uint32_t (&r)[NW], acc_t w)
    {
        if constexpr (DT == FASTGL_F32) {
#pragma unroll
            for (int i = 0; i < NW; ++i) {
                double x = (double)__uint_as_float(r[i]);
                acc[i] = HASW ? __builtin_fma(x, w, acc[i]) : acc[i] + x;
            }
        } else if constexpr (VB >= 4) {
#pragma unroll
            for (int i = 0; i < NW; ++i) {
                float lo = __uint_as_float(r[i] << 16), hi = __uint_as_float(r[i] & 0xFFFF0000u);
                acc[2 * i] = HASW ? __builtin_fmaf(lo, w, acc[2 * i]) : acc[2 * i] + lo;
                acc[2 * i + 1] = HASW ? __builtin_fmaf(hi, w, acc[2 * i + 1]) : acc[2 * i + 1] + hi;
            }
        } else {
            float lo = __uint_as_float(r[0] << 16);
            acc[0] = HASW ? __builtin_fmaf(lo, w, acc[0]) : acc[0] + lo;
        }
    }

    __device__ static __forceinline__ uint32_t to_bf16(float f)
    {
        uint32_t u = __float_as_uint(f);
        if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (u >> 16) | 0x40u;   // keep NaN quiet
        return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;                    // nearest even
    }

    __device__ static __forceinline__ void store(char *p, const acc_t (&acc)[NE], acc_t scale)
    {
        uint32_t r[NW];
        if constexpr (DT == FASTGL_F32) {
#pragma unroll
            for (int i = 0; i < NW; ++i) r[i] = __float_as_uint((float)(acc[i] * scale));
        } else if constexpr (VB >= 4) {
#pragma unroll
            for (int i = 0; i < NW; ++i)
                r[i] = to_bf16(acc[2 * i] * scale) | (to_bf16(acc[2 * i + 1] * scale) << 16);
        } else {
            r[0] = to_bf16(acc[0] * scale);
        }
        // output rows are written once and never read back by this kernel: streaming
        // stores keep them from displacing gathered rows in L2 / Infinity Cache
        typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
        typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
        if constexpr (VB == 16) {
            u32x4 v = {r[0], r[1], r[2], r[3]};
            __builtin_nontemporal_store(v, reinterpret_cast<u32x4 *>(p));
        } else if constexpr (VB == 8) {
            u32x2 v = {r[0], r[1]};
            __builtin_nontemporal_store(v, reinterpret_cast<u32x2 *>(p));
        } else if constexpr (VB == 4) {
            __builtin_nontemporal_store(r[0], reinterpret_cast<uint32_t *>(p));
        } else {
            __builtin_nontemporal_store((uint16_t)r[0], reinterpret_cast<uint16_t *>(p));
        }
    }
};

struct PullParams {
    const int32_t *rowptr, *col, *eid;
    const float *edge_w, *col_scale;
    const char *in;
    char *out;
    const int32_t *split;     // [nsets+1] first row of every fine row set (equal work each)
    int64_t nsets;            // fine row sets
    int64_t ngroups;          // groups per column tile = ceil(nsets / sets_per_group)
    int32_t ntiles;           // column tiles per row
    int32_t G;                // lanes per group (power of two)
    int32_t sets_per_group;   // consecutive fine row sets one group takes (1, 2, 4 or 8)
    int64_t num_rows;
    int32_t row_mode;
    int32_t long_thr;         // rows longer than this are left to the chunk kernels
    int64_t row_bytes;        // bytes of one feature row
    int64_t feat;
    int32_t xcd_run;          // consecutive logical blocks handed to one L2 domain
    int64_t num_blocks;       // launched blocks (multiple of kXcds)
    const int32_t *long_rows, *chunk_ptr, *n_long, *n_chunks;
    char *partials;
};

template <typename acc_t>
__device__ __forceinline__ acc_t row_scale(int mode, int len)
{
    acc_t d = (acc_t)(len < 1 ? 1 : len);
    if (mode == 1) return (acc_t)1 / d;
    if (mode == 2) return (acc_t)1 / (acc_t)sqrt((double)d);
    return (acc_t)1;
}

template <typename T> __device__ __forceinline__ T shfl_t(T v, int src);
template <> __device__ __forceinline__ float shfl_t<float>(float v, int src) { return __shfl(v, src, kWave); }
template <> __device__ __forceinline__ double shfl_t<double>(double v, int src) { return __shfl(v, src, kWave); }

// Column ids and weights of up to G consecutive edges, one per lane of a group.
template <bool HASW, typename acc_t>
__device__ __forceinline__ int load_cols(const PullParams &P, int k, int kend)
{
    return k < kend ? P.col[k] : 0;
}

template <bool HASW, typename acc_t>
__device__ __forceinline__ acc_t load_weight(const PullParams &P, int k, int kend, int c)
{
    acc_t w = (acc_t)1;
    if (HASW && k < kend) {
        if (P.edge_w) w = (acc_t)P.edge_w[P.eid ? P.eid[k] : k];
        if (P.col_scale) w *= (acc_t)P.col_scale[c];
    }
    return w;
}

// What happens to a finished row of walk_run is its SINK's business:
// sink(row index, sums of this lane's slice, the row's scale factor).  RowStore
// writes the scaled, rounded row to the output matrix.
template <int DT, int VB>
struct RowStore {
    char *out;
    int64_t row_bytes, lane_off;
    bool active;
    __device__ __forceinline__ void operator()(int64_t row, const typename Slice<DT, VB>::acc_t (&acc)[Slice<DT, VB>::NE],
                                               typename Slice<DT, VB>::acc_t scale) const
    {
        if (active) Slice<DT, VB>::store(out + row * row_bytes + lane_off, acc, scale);
    }
};

// A group walks the edges of a run of consecutive rows [ia, ib) of its row set as
// ONE flat edge list, so that U row gathers are in flight whatever the row
// lengths are (sampled blocks have rows of 1-15 edges, transposed ones of 0-3),
// and closes a row (hand its sum and scale factor to the sink, clear the sum)
// whenever the edge index passes the row's end.  pb / pe: lane i of the group holds
// rowptr of its i-th row.  Column ids are fetched two chunks ahead and weights one
// chunk ahead of use.
// PARTIAL: the "row" is a chunk of a long row; its unscaled sum goes to slot r0 of
// the partial-sum buffer and the sink is not called.
template <int DT, int VB, bool HASW, bool PARTIAL, int U, class Sink>
__device__ __forceinline__ void walk_run(const PullParams &P, int64_t r0, int ia, int ib, int pb, int pe,
                                         int sub, int gbase, int64_t lane_off, bool active, const Sink &sink)
{
    using S = Slice<DT, VB>;
    using acc_t = typename S::acc_t;
    const int G = P.G;
    const int ebeg = __shfl(pb, gbase + ia, kWave), eend = __shfl(pe, gbase + ib - 1, kWave);
    int row = ia;
    int rend = __shfl(pe, gbase + row, kWave);
    acc_t acc[S::NE];
#pragma unroll
    for (int i = 0; i < S::NE; ++i) acc[i] = (acc_t)0;

    auto close_row = [&]() {
        if constexpr (PARTIAL) {
            if (active) {
                acc_t *dst = reinterpret_cast<acc_t *>(P.partials) + r0 * P.feat + lane_off / VB * S::NE;
#pragma unroll
                for (int i = 0; i < S::NE; ++i) dst[i] = acc[i];
            }
        } else {
            const int len = rend - __shfl(pb, gbase + row, kWave);
            sink(r0 + row, acc, row_scale<acc_t>(P.row_mode, len));
        }
#pragma unroll
        for (int i = 0; i < S::NE; ++i) acc[i] = (acc_t)0;
        ++row;
        rend = __shfl(pe, gbase + (row < ib ? row : ib - 1), kWave);
    };

    int cur_c = load_cols<HASW, acc_t>(P, ebeg + sub, eend);
    int nxt_c = load_cols<HASW, acc_t>(P, ebeg + G + sub, eend);
    acc_t cur_w = load_weight<HASW, acc_t>(P, ebeg + sub, eend, cur_c);
    for (int k0 = ebeg; k0 < eend; k0 += G) {
        const int n = eend - k0 < G ? eend - k0 : G;
        const int nn_c = load_cols<HASW, acc_t>(P, k0 + 2 * G + sub, eend);
        const acc_t nxt_w = load_weight<HASW, acc_t>(P, k0 + G + sub, eend, nxt_c);
        for (int j0 = 0; j0 < n; j0 += U) {
            uint32_t raw[U][S::NW];
#pragma unroll
            for (int t = 0; t < U; ++t) {
                const int j = j0 + t;
                const int c = __shfl(cur_c, gbase + (j & (G - 1)), kWave);
                if (j < n && active) S::load(P.in + (int64_t)c * P.row_bytes + lane_off, raw[t]);
            }
#pragma unroll
            for (int t = 0; t < U; ++t) {
                const int j = j0 + t;
                acc_t w = (acc_t)1;
                if (HASW) w = shfl_t<acc_t>(cur_w, gbase + (j & (G - 1)));
                if (j < n) {
                    const int e = k0 + j;
                    while (e >= rend) close_row();
                    if (active) S::template fma<HASW>(acc, raw[t], w);
                }
            }
        }
        cur_c = nxt_c;
        cur_w = nxt_w;
        nxt_c = nn_c;
    }
    while (row < ib) close_row();
}

}  // namespace fastgl
