// ID map of the sample phase (paper Section 2.2; Section 4.3, Algorithm 2): global IDs of one
// sampled hop -> consecutive local IDs.  See include/fastgl_idmap.h for the contract.
//
// Table: open addressing with linear probing, 64-bit keys claimed by compare-and-swap from the
// empty marker -1, capacity 1.5 x the number of input IDs (most of which repeat).  A thread reads the
// slot with a plain load first and only issues the compare-and-swap when it saw the empty marker:
// a key changes exactly once (from -1 to an ID), so anything else it reads is final; repeats of a
// hub node therefore cost loads, not atomics.
//
// FUSED mode is Algorithm 2: the claimant of a slot takes the next local ID from a counter (one
// atomic add per workgroup, the threads that claimed a slot share it), a second kernel translates.
// Its insertion only touches keys and its translation only local IDs, so it keeps them in two bare
// arrays (8 + 4 bytes per slot): the array the translation reads at random is a quarter of the size
// of a table of 16-byte entries and largely stays in L2.
// ORDERED mode replaces the counter by "smallest position seen at this slot" (atomic min), then a
// prefix count over the positions that are first occurrences gives every distinct ID its rank in
// order of first appearance.  Both remember the slot of every input ID, so translation does not
// probe again.
#include "fastgl_idmap.h"
#include "hash_table.h"
#include "internal.h"

namespace fastgl {
namespace {

constexpr int32_t kFirstBit = (int32_t)0x80000000u;

struct IdmapArgs {
    const int64_t *dst_gid, *nbr_gid;
    int64_t n_dst, n_nbr, n;
    Slot *table;              // [cap] ORDERED: 16-byte entries
    int64_t *keys;            // [cap] FUSED: keys ...
    int32_t *vals;            // [cap]        ... and local IDs
    int32_t *slot_of;         // [n] slot of every input position (kNoSlot: rejected ID); the ordered mode
                              // sets bit 31 on positions that are first occurrences
    int32_t *block_cnt;       // [blocks + 1]
    int32_t *local_nbr;
    int64_t *unique_gid;
    int32_t *result;          // [0] U, [1] violations
    int64_t cap;              // slots of the table
    int nblocks;
    int fused;
};

__device__ __forceinline__ int64_t id_at(const IdmapArgs &a, int64_t p)
{
    return p < a.n_dst ? a.dst_gid[p] : a.nbr_gid[p - a.n_dst];
}

__global__ __launch_bounds__(256) void k_idmap_fill(IdmapArgs a)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i == 0) {
        a.result[0] = a.fused ? (int32_t)a.n_dst : 0;
        a.result[1] = 0;
    }
    if (i >= a.cap) return;
    if (a.fused) {
        a.keys[i] = -1;       // a local ID is only read at a slot somebody claimed, after its claimant wrote it
        return;
    }
    Slot e;
    e.key = -1;
    e.val = INT32_MAX;
    e.lid = 0;
    a.table[i] = e;
}

// ORDERED pass 1: claim slots, keep the smallest position per slot.
__global__ __launch_bounds__(256) void k_idmap_insert_min(IdmapArgs a)
{
    const int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= a.n) return;
    const int64_t gid = id_at(a, p);
    if (gid < 0) {
        a.slot_of[p] = kNoSlot;
        atomicAdd(&a.result[1], 1);
        return;
    }
    bool fresh;
    const uint32_t slot = insert_id(a.table, (uint32_t)a.cap, gid, fresh);
    a.slot_of[p] = (int32_t)slot;
    // the value only ever decreases, so a (possibly stale) reading that is already smaller settles it
    if (__hip_atomic_load(&a.table[slot].val, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) > (int32_t)p)
        atomicMin(&a.table[slot].val, (int32_t)p);
}

// ORDERED pass 2: mark the positions that are first occurrences (bit 31 of slot_of) and count them
// per block of kScanBlock positions.
__global__ __launch_bounds__(kScanBlock) void k_idmap_count(IdmapArgs a)
{
    const int64_t p = (int64_t)blockIdx.x * kScanBlock + threadIdx.x;
    bool first = false;
    if (p < a.n) {
        const int32_t slot = a.slot_of[p];
        first = slot != kNoSlot && a.table[slot].val == (int32_t)p;
        if (first) a.slot_of[p] = slot | kFirstBit;
    }
    const int c = __syncthreads_count(first);
    if (threadIdx.x == 0) a.block_cnt[blockIdx.x] = c;
}

// ORDERED pass 3: block counts -> block offsets, total -> result[0].  One workgroup.
__global__ __launch_bounds__(kScanBlock) void k_idmap_scan(IdmapArgs a)
{
    const int total = scan_block_counts(a.block_cnt, a.nblocks);
    if (threadIdx.x == 0) a.result[0] = total;
}

// ORDERED pass 4: rank of every first occurrence = its local ID.
__global__ __launch_bounds__(kScanBlock) void k_idmap_rank(IdmapArgs a)
{
    const int64_t p = (int64_t)blockIdx.x * kScanBlock + threadIdx.x;
    const int32_t so = p < a.n ? a.slot_of[p] : kNoSlot;
    const bool first = so < 0;                     // bit 31
    int rank;
    block_exclusive_scan(first ? 1 : 0, a.block_cnt[blockIdx.x], rank);
    if (first) {
        a.table[so & kNoSlot].lid = rank;
        a.unique_gid[rank] = id_at(a, p);
    }
    if (p < a.n_dst && (!first || rank != (int)p)) atomicAdd(&a.result[1], 1);   // repeated destination
}

// Translation (both modes): the slot of every neighbour entry is known.
__global__ __launch_bounds__(256) void k_idmap_translate(IdmapArgs a)
{
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= a.n_nbr) return;
    const int32_t slot = a.slot_of[a.n_dst + e] & kNoSlot;
    a.local_nbr[e] = slot == kNoSlot ? -1 : (a.fused ? a.vals[slot] : a.table[slot].lid);
}

// FUSED pass 1a: destination i takes local ID i.
__global__ __launch_bounds__(256) void k_idmap_fused_dst(IdmapArgs a)
{
    const int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= a.n_dst) return;
    const int64_t gid = a.dst_gid[p];
    bool fresh = false;
    if (gid >= 0) {
        const uint32_t slot = insert_key<8>(a.keys, (uint32_t)a.cap, gid, fresh);
        if (fresh) {
            a.vals[slot] = (int32_t)p;
            a.unique_gid[p] = gid;
        }
    }
    if (!fresh) atomicAdd(&a.result[1], 1);       // negative or repeated destination
}

// FUSED pass 1b (Algorithm 2): whoever claims a slot takes the next local ID.  The claimants of a
// workgroup share one atomic add on the counter (a prefix count inside the workgroup hands out the
// IDs of the range it returns).
__global__ __launch_bounds__(kScanBlock) void k_idmap_fused_nbr(IdmapArgs a)
{
    __shared__ int range_base;
    const int64_t e = (int64_t)blockIdx.x * kScanBlock + threadIdx.x;
    const bool active = e < a.n_nbr;
    const int64_t gid = active ? a.nbr_gid[e] : -1;
    bool fresh = false;
    uint32_t slot = 0;
    if (gid >= 0) slot = insert_key<8>(a.keys, (uint32_t)a.cap, gid, fresh);
    if (active) {
        a.slot_of[a.n_dst + e] = gid >= 0 ? (int32_t)slot : kNoSlot;
        if (gid < 0) atomicAdd(&a.result[1], 1);
    }
    int mine;
    const int claimed = block_exclusive_scan(fresh ? 1 : 0, 0, mine);
    if (claimed == 0) return;
    if (threadIdx.x == 0) range_base = atomicAdd(&a.result[0], claimed);
    __syncthreads();
    if (fresh) {
        const int l = range_base + mine;
        a.vals[slot] = l;
        a.unique_gid[l] = gid;
    }
}

struct Layout {
    size_t table, slot_of, block_cnt, total;
};

Layout layout(int64_t n)
{
    const int64_t cap = idmap_slots(n);
    Layout L;
    size_t off = 0;
    L.table = off; off += align_up((size_t)cap * sizeof(Slot), 256);
    L.slot_of = off; off += align_up((size_t)(n > 0 ? n : 1) * 4, 256);
    L.block_cnt = off; off += align_up((size_t)(ceil_div(n, kScanBlock) + 1) * 4, 256);
    L.total = off;
    return L;
}

}  // namespace
}  // namespace fastgl

using namespace fastgl;

extern "C" {

int64_t fastgl_idmap_table_slots(int64_t n_ids)
{
    if (n_ids < 0 || n_ids >= kMaxIds) return 0;
    return idmap_slots(n_ids);
}

size_t fastgl_idmap_workspace_bytes(int64_t n_dst, int64_t n_nbr)
{
    if (n_dst < 0 || n_nbr < 0 || n_dst + n_nbr >= kMaxIds) return 0;
    return layout(n_dst + n_nbr).total;
}

fastgl_status fastgl_idmap(const int64_t *dst_gid, int64_t n_dst, const int64_t *nbr_gid, int64_t n_nbr,
                           fastgl_idmap_mode mode, int32_t *local_nbr, int64_t *unique_gid, int32_t *result,
                           void *workspace, size_t workspace_bytes, void *stream)
{
    if (n_dst < 0 || n_nbr < 0) {
        set_error("negative size (n_dst=%lld n_nbr=%lld)", (long long)n_dst, (long long)n_nbr);
        return FASTGL_ERR_INVALID_ARG;
    }
    if (n_dst + n_nbr >= kMaxIds) {
        set_error("n_dst + n_nbr must stay below 2^30");
        return FASTGL_ERR_UNSUPPORTED;
    }
    if ((int)mode != FASTGL_IDMAP_ORDERED && (int)mode != FASTGL_IDMAP_FUSED) {
        set_error("unknown ID-map mode %d", (int)mode);
        return FASTGL_ERR_INVALID_ARG;
    }
    const int64_t n = n_dst + n_nbr;
    if ((n_dst > 0 && !dst_gid) || (n_nbr > 0 && (!nbr_gid || !local_nbr)) || (n > 0 && !unique_gid) || !result) {
        set_error("NULL array (dst_gid, nbr_gid, local_nbr, unique_gid or result)");
        return FASTGL_ERR_INVALID_ARG;
    }
    if ((((uintptr_t)dst_gid | (uintptr_t)nbr_gid | (uintptr_t)unique_gid) & 7) ||
        (((uintptr_t)local_nbr | (uintptr_t)result) & 3)) {
        set_error("ID arrays must be 8-byte aligned, local_nbr and result 4-byte aligned");
        return FASTGL_ERR_INVALID_ARG;
    }
    if (!workspace || ((uintptr_t)workspace & 255)) {
        set_error("workspace must be a 256-byte aligned device buffer");
        return FASTGL_ERR_INVALID_ARG;
    }
    const Layout L = layout(n);
    if (workspace_bytes < L.total) {
        set_error("workspace too small: %zu < %zu bytes", workspace_bytes, L.total);
        return FASTGL_ERR_WORKSPACE;
    }
    char *ws = (char *)workspace;
    IdmapArgs a = {};
    a.dst_gid = dst_gid; a.nbr_gid = nbr_gid;
    a.n_dst = n_dst; a.n_nbr = n_nbr; a.n = n;
    a.table = (Slot *)(ws + L.table);
    a.keys = (int64_t *)(ws + L.table);                       // the fused mode's two arrays share the table's room
    a.slot_of = (int32_t *)(ws + L.slot_of);
    a.block_cnt = (int32_t *)(ws + L.block_cnt);
    a.local_nbr = local_nbr; a.unique_gid = unique_gid; a.result = result;
    a.cap = idmap_slots(n);
    a.vals = (int32_t *)(a.keys + a.cap);
    a.nblocks = (int)ceil_div(n, kScanBlock);
    a.fused = mode == FASTGL_IDMAP_FUSED;
    hipStream_t s = (hipStream_t)stream;
    auto grid = [](int64_t items, int per) { return dim3((unsigned)(items > 0 ? ceil_div(items, per) : 1)); };

    hipLaunchKernelGGL(k_idmap_fill, grid(a.cap, 256), dim3(256), 0, s, a);
    FASTGL_LAUNCH_CHECK("fastgl_idmap (fill)");
    if (a.fused) {
        if (n_dst > 0) {
            hipLaunchKernelGGL(k_idmap_fused_dst, grid(n_dst, 256), dim3(256), 0, s, a);
            FASTGL_LAUNCH_CHECK("fastgl_idmap (destinations)");
        }
        if (n_nbr > 0) {
            hipLaunchKernelGGL(k_idmap_fused_nbr, grid(n_nbr, kScanBlock), dim3(kScanBlock), 0, s, a);
            FASTGL_LAUNCH_CHECK("fastgl_idmap (fused map)");
        }
    } else if (n > 0) {
        hipLaunchKernelGGL(k_idmap_insert_min, grid(n, 256), dim3(256), 0, s, a);
        FASTGL_LAUNCH_CHECK("fastgl_idmap (insert)");
        hipLaunchKernelGGL(k_idmap_count, dim3((unsigned)a.nblocks), dim3(kScanBlock), 0, s, a);
        FASTGL_LAUNCH_CHECK("fastgl_idmap (count)");
        hipLaunchKernelGGL(k_idmap_scan, dim3(1), dim3(kScanBlock), 0, s, a);
        FASTGL_LAUNCH_CHECK("fastgl_idmap (scan)");
        hipLaunchKernelGGL(k_idmap_rank, dim3((unsigned)a.nblocks), dim3(kScanBlock), 0, s, a);
        FASTGL_LAUNCH_CHECK("fastgl_idmap (rank)");
    }
    if (n_nbr > 0) {
        hipLaunchKernelGGL(k_idmap_translate, grid(n_nbr, 256), dim3(256), 0, s, a);
        FASTGL_LAUNCH_CHECK("fastgl_idmap (translate)");
    }
    return FASTGL_OK;
}

}  // extern "C"
