// Pull-mode block aggregation for gfx950 (paper Section 2.1 Eq. 1 forward;
// Section 4.2 Eq. 5 backward, run as the same pull over the transposed CSR).
//
//   out[r,:] = rowscale(len_r) * sum_{k in row r} a_k * colscale[col_k] * in[col_k,:]
//
// Mapping to the machine.  A feature row is cut into slices of VB bytes (16 when
// the row size allows, so one lane moves one dwordx4) and a "group" of G lanes
// (a power of two, <= 64) covers G consecutive slices.  One group owns a set of
// consecutive rows (x one column tile) from start to end, so each output element
// has a single writer and the summation order is fixed: results do not depend on
// scheduling.  The row sets come from the plan and carry equal work (edges +
// rows), so skewed degree distributions do not overload a group.
// The partial sum lives in registers (the paper keeps it in shared memory on its
// GPU; with one lane per slice registers serve the same purpose at no traffic).
// The lanes of a group fetch column ids and weights with one coalesced load and
// hand them round with cross-lane reads, then issue up to 6 independent row
// gathers before the first use.  Output rows leave with streaming stores.
//
// f32 rows accumulate in fp64, bf16 rows in fp32; one rounding at the store.
//
// Rows longer than kLongThreshold edges are not walked by one group: they are
// cut into chunks of kLongChunk edges that any group can take (in the same
// launch); the partial sums go to the workspace and are added in chunk order by
// a second, small kernel, so the result is still deterministic.
#include "pull_walk.h"

namespace fastgl {

constexpr int kXcdRun = 16;

// Which (row set, column tile) a lane group works on.
//
// Workgroup ids are dealt round-robin to the 8 XCDs, each with its own L2.
// Consecutive logical workgroups are handed to an XCD in runs of P.xcd_run, so
// that neighbouring rows (which share output cache lines and first-touch source
// rows) share an L2, while every XCD still samples the whole row range: blocks
// whose hubs all sit at low ids stay balanced.  The column tiles of a row set
// (rows wider than 64 slices) sit in neighbouring groups.
struct GroupId {
    int64_t g;        // index of the group's first fine row set / P.sets_per_group
    int tile;         // column tile
    int64_t count;    // launched groups per tile (chunk stride)
};

__device__ __forceinline__ GroupId map_group(const PullParams &P)
{
    const int gpb = kBlock / P.G;
    const int64_t x = blockIdx.x % kXcds, q = blockIdx.x / kXcds;
    const int64_t lb = ((q / P.xcd_run) * kXcds + x) * P.xcd_run + q % P.xcd_run;
    const int64_t vg = lb * gpb + threadIdx.x / P.G;
    const int64_t launched = P.num_blocks * gpb;
    GroupId r;
    r.tile = (int)(vg % P.ntiles);
    r.g = vg / P.ntiles;
    r.count = (launched - r.tile + P.ntiles - 1) / P.ntiles;
    return r;
}

// Chunks of long rows.  The number of chunks lives in device memory, so the host
// never needs to know the degrees; the groups of a column tile stride over the
// chunks and write fp64 / fp32 partial sums of their tile to the workspace.
template <int DT, int VB, bool HASW, int U>
__device__ __forceinline__ void pull_chunks(const PullParams &P, const GroupId &id, int sub, int gbase)
{
    const int n_long = *P.n_long;
    const int64_t total = *P.n_chunks;
    const int64_t lane_off = ((int64_t)id.tile * P.G + sub) * VB;
    for (int64_t chunk = id.g; chunk < total; chunk += id.count) {
        int lo = 0, hi = n_long;   // chunk_ptr[lo] <= chunk < chunk_ptr[hi]
        while (hi - lo > 1) {
            int mid = lo + ((hi - lo) >> 1);
            if (P.chunk_ptr[mid] <= chunk) lo = mid; else hi = mid;
        }
        const int row = P.long_rows[lo];
        const int rbeg = P.rowptr[row], rend = P.rowptr[row + 1];
        const int beg = rbeg + ((int)chunk - P.chunk_ptr[lo]) * kLongChunk;
        const int end = beg + kLongChunk < rend ? beg + kLongChunk : rend;
        const bool active = lane_off < P.row_bytes;
        const RowStore<DT, VB> unused = {nullptr, 0, 0, false};     // a chunk's sum goes to the partial-sum buffer
        walk_run<DT, VB, HASW, true, U>(P, chunk, 0, 1, beg, end, sub, gbase, lane_off, active, unused);
    }
}

// One launch covers every row.  Each group first takes its share of the long-row
// chunks (usually none), then its own row set: the consecutive rows
// of a few fine row sets, which the plan cut so that every set carries the same
// work (edges + rows), whatever the degree distribution is.  Rows that are long
// are skipped here; k_reduce_chunks finishes them.
template <int DT, int VB, bool HASW, int U>
__global__ __launch_bounds__(kBlock) void k_pull_rows(PullParams P)
{
    const int tid = threadIdx.x, lane = tid & (kWave - 1);
    const int sub = tid & (P.G - 1), gbase = lane & ~(P.G - 1);
    const GroupId id = map_group(P);
    if (P.long_rows) pull_chunks<DT, VB, HASW, U>(P, id, sub, gbase);
    if (id.g >= P.ngroups) return;
    const int64_t lane_off = ((int64_t)id.tile * P.G + sub) * VB;
    const bool active = lane_off < P.row_bytes;
    const int64_t s0 = id.g * P.sets_per_group;
    const int64_t s1 = s0 + P.sets_per_group < P.nsets ? s0 + P.sets_per_group : P.nsets;
    const int64_t rbeg = P.split[s0], rend = P.split[s1];
    const unsigned long long gmask = P.G == kWave ? ~0ull : ((1ull << P.G) - 1ull);
    const RowStore<DT, VB> sink = {P.out, P.row_bytes, lane_off, active};
    for (int64_t r0 = rbeg; r0 < rend; r0 += P.G) {
        const int nrows = rend - r0 < P.G ? (int)(rend - r0) : P.G;
        int pb = 0, pe = 0;
        if (sub < nrows) {
            pb = P.rowptr[r0 + sub];
            pe = P.rowptr[r0 + sub + 1];
        }
        unsigned long long lm = (__ballot(sub < nrows && pe - pb > P.long_thr) >> gbase) & gmask;
        int i = 0;
        while (i < nrows) {
            if ((lm >> i) & 1ull) {   // a long row: its chunks were handled above
                ++i;
                continue;
            }
            const unsigned long long rest = lm >> i;
            const int j = rest ? i + (__ffsll((long long)rest) - 1) : nrows;
            walk_run<DT, VB, HASW, false, U>(P, r0, i, j, pb, pe, sub, gbase, lane_off, active, sink);
            i = j;
        }
    }
}

template <int DT, int VB>
__global__ __launch_bounds__(kBlock) void k_reduce_chunks(PullParams P)
{
    using S = Slice<DT, VB>;
    using acc_t = typename S::acc_t;
    const int tid = threadIdx.x;
    const int sub = tid & (P.G - 1);
    const int64_t total = (int64_t)(*P.n_long) * P.ntiles;
    const int64_t stride = (int64_t)gridDim.x * kBlock / P.G;
    for (int64_t unit = ((int64_t)blockIdx.x * kBlock + tid) / P.G; unit < total; unit += stride) {
        const int li = (int)(unit / P.ntiles);
        const int tile = (int)(unit - (int64_t)li * P.ntiles);
        const int64_t lane_off = ((int64_t)tile * P.G + sub) * VB;
        if (lane_off >= P.row_bytes) continue;
        const int row = P.long_rows[li];
        acc_t acc[S::NE];
#pragma unroll
        for (int i = 0; i < S::NE; ++i) acc[i] = (acc_t)0;
        const acc_t *src = reinterpret_cast<const acc_t *>(P.partials) + ((int64_t)tile * P.G + sub) * S::NE;
        // partial sums are added in chunk order (fixed result); 8 are fetched at a time
        const int c1 = P.chunk_ptr[li + 1];
        for (int c0 = P.chunk_ptr[li]; c0 < c1; c0 += 8) {
            acc_t part[8][S::NE];
#pragma unroll
            for (int k = 0; k < 8; ++k)
#pragma unroll
                for (int i = 0; i < S::NE; ++i)
                    part[k][i] = c0 + k < c1 ? src[(int64_t)(c0 + k) * P.feat + i] : (acc_t)0;
#pragma unroll
            for (int k = 0; k < 8; ++k)
#pragma unroll
                for (int i = 0; i < S::NE; ++i) acc[i] += part[k][i];
        }
        const int len = P.rowptr[row + 1] - P.rowptr[row];
        S::store(P.out + (int64_t)row * P.row_bytes + lane_off, acc, row_scale<acc_t>(P.row_mode, len));
    }
}

template <int VB>
__global__ __launch_bounds__(kBlock) void k_gather_rows(const char *__restrict__ table,
                                                        const int64_t *__restrict__ ids, int64_t num_units,
                                                        int32_t ntiles, int32_t G, int64_t row_bytes,
                                                        char *__restrict__ out)
{
    const int tid = threadIdx.x;
    const int sub = tid & (G - 1);
    const int64_t unit = ((int64_t)blockIdx.x * kBlock + tid) / G;
    if (unit >= num_units) return;
    const int64_t row = unit / ntiles;
    const int tile = (int)(unit - row * ntiles);
    const int64_t lane_off = ((int64_t)tile * G + sub) * VB;
    if (lane_off >= row_bytes) return;
    uint32_t r[Slice<FASTGL_BF16, VB>::NW];
    Slice<FASTGL_BF16, VB>::load(table + ids[row] * row_bytes + lane_off, r);
    char *p = out + row * row_bytes + lane_off;
    if constexpr (VB == 16) *reinterpret_cast<uint4 *>(p) = make_uint4(r[0], r[1], r[2], r[3]);
    else if constexpr (VB == 8) *reinterpret_cast<uint2 *>(p) = make_uint2(r[0], r[1]);
    else if constexpr (VB == 4) *reinterpret_cast<uint32_t *>(p) = r[0];
    else *reinterpret_cast<uint16_t *>(p) = (uint16_t)r[0];
}

// ------------------------------------------------------------- host side ----
// Largest slice width (bytes) that divides the row size and the buffer alignment.
static int pick_slice_bytes(int64_t row_bytes, const void *a, const void *b, int elem)
{
    uintptr_t bits = (uintptr_t)a | (uintptr_t)b | (uintptr_t)row_bytes;
    for (int vb = 16; vb > elem; vb >>= 1)
        if ((bits & (uintptr_t)(vb - 1)) == 0) return vb;
    return elem;
}

static void group_shape(int64_t row_bytes, int vb, int *G, int *ntiles)
{
    int64_t slices = row_bytes / vb;
    int g = 1;
    while (g < kWave && g < slices) g <<= 1;
    *G = g;
    *ntiles = (int)ceil_div(slices, g);
}

template <int DT, int VB>
static fastgl_status launch_typed(const PullParams &P, bool hasw, bool with_long, int64_t nblocks, hipStream_t s)
{
    if (nblocks > 0) {
        dim3 grid((unsigned)P.num_blocks);
        const bool narrow = P.G <= 16;
        if (hasw && narrow) hipLaunchKernelGGL((k_pull_rows<DT, VB, true, kUnrollNarrow>), grid, dim3(kBlock), 0, s, P);
        else if (hasw) hipLaunchKernelGGL((k_pull_rows<DT, VB, true, kUnroll>), grid, dim3(kBlock), 0, s, P);
        else if (narrow) hipLaunchKernelGGL((k_pull_rows<DT, VB, false, kUnrollNarrow>), grid, dim3(kBlock), 0, s, P);
        else hipLaunchKernelGGL((k_pull_rows<DT, VB, false, kUnroll>), grid, dim3(kBlock), 0, s, P);
        FASTGL_LAUNCH_CHECK("k_pull_rows");
    }
    if (with_long) {
        hipLaunchKernelGGL((k_reduce_chunks<DT, VB>), dim3(512), dim3(kBlock), 0, s, P);
        FASTGL_LAUNCH_CHECK("k_reduce_chunks");
    }
    return FASTGL_OK;
}

fastgl_status launch_pull(const PullDesc &d, hipStream_t s)
{
    if (d.num_rows == 0) return FASTGL_OK;
    const int elem = d.dtype == FASTGL_F32 ? 4 : 2;
    PullParams P;
    P.rowptr = d.rowptr; P.col = d.col; P.eid = d.eid;
    P.edge_w = d.edge_w; P.col_scale = d.col_scale;
    P.in = (const char *)d.in; P.out = (char *)d.out;
    P.row_bytes = d.feat * elem;
    P.feat = d.feat;
    P.row_mode = d.row_mode;
    const int vb = pick_slice_bytes(P.row_bytes, d.in, d.out, elem);
    int G, ntiles;
    group_shape(P.row_bytes, vb, &G, &ntiles);
    P.G = G; P.ntiles = ntiles;
    P.num_rows = d.num_rows;
    P.split = d.split;
    P.nsets = d.nsets;
    // several fine sets per group when there are plenty: amortises the row-pointer /
    // column-id latency over more gathers while keeping >= ~16K groups in flight
    int spg = 1;
    while (spg < 8 && (d.nsets / (spg * 2)) * G * ntiles / kWave >= 16384) spg *= 2;
    P.sets_per_group = spg;
    P.ngroups = ceil_div(d.nsets, P.sets_per_group);
    const bool with_long = d.long_rows != nullptr;
    P.long_thr = with_long ? kLongThreshold : INT32_MAX;
    P.long_rows = d.long_rows; P.chunk_ptr = d.chunk_ptr; P.n_long = d.n_long; P.n_chunks = d.n_chunks;
    P.partials = (char *)d.partials;
    const int gpb = kBlock / G;
    P.xcd_run = kXcdRun;
    P.num_blocks = ceil_div(ceil_div(P.ngroups * ntiles, gpb), (int64_t)kXcds * P.xcd_run) * P.xcd_run * kXcds;
    const int64_t nblocks = P.num_blocks;
    if (P.num_blocks > 0x7FFFFFFFLL) {
        set_error("block too large for one launch (%lld workgroups)", (long long)nblocks);
        return FASTGL_ERR_UNSUPPORTED;
    }
    const bool hasw = d.edge_w != nullptr || d.col_scale != nullptr;
#define FASTGL_CASE(DT, VB) return launch_typed<DT, VB>(P, hasw, with_long, nblocks, s)
    if (d.dtype == FASTGL_F32) {
        switch (vb) {
            case 16: FASTGL_CASE(FASTGL_F32, 16);
            case 8: FASTGL_CASE(FASTGL_F32, 8);
            default: FASTGL_CASE(FASTGL_F32, 4);
        }
    } else {
        switch (vb) {
            case 16: FASTGL_CASE(FASTGL_BF16, 16);
            case 8: FASTGL_CASE(FASTGL_BF16, 8);
            case 4: FASTGL_CASE(FASTGL_BF16, 4);
            default: FASTGL_CASE(FASTGL_BF16, 2);
        }
    }
#undef FASTGL_CASE
}

fastgl_status launch_gather_rows(const void *table, const int64_t *ids, int64_t n, int64_t feat,
                                 fastgl_dtype dtype, void *out, hipStream_t s)
{
    if (n == 0) return FASTGL_OK;
    const int elem = dtype == FASTGL_F32 ? 4 : 2;
    const int64_t row_bytes = feat * elem;
    const int vb = pick_slice_bytes(row_bytes, table, out, elem);
    int G, ntiles;
    group_shape(row_bytes, vb, &G, &ntiles);
    const int64_t units = n * ntiles;
    const int64_t nblocks = ceil_div(units * G, kBlock);
    if (nblocks > 0x7FFFFFFFLL) {
        set_error("gather too large for one launch");
        return FASTGL_ERR_UNSUPPORTED;
    }
    dim3 grid((unsigned)nblocks);
    const char *t = (const char *)table;
    char *o = (char *)out;
    switch (vb) {
        case 16: hipLaunchKernelGGL(k_gather_rows<16>, grid, dim3(kBlock), 0, s, t, ids, units, ntiles, G, row_bytes, o); break;
        case 8: hipLaunchKernelGGL(k_gather_rows<8>, grid, dim3(kBlock), 0, s, t, ids, units, ntiles, G, row_bytes, o); break;
        case 4: hipLaunchKernelGGL(k_gather_rows<4>, grid, dim3(kBlock), 0, s, t, ids, units, ntiles, G, row_bytes, o); break;
        default: hipLaunchKernelGGL(k_gather_rows<2>, grid, dim3(kBlock), 0, s, t, ids, units, ntiles, G, row_bytes, o); break;
    }
    FASTGL_LAUNCH_CHECK("k_gather_rows");
    return FASTGL_OK;
}

}  // namespace fastgl
