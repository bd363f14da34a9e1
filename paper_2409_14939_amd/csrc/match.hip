// Match process and Greedy Reorder Strategy (paper Section 4.1, Algorithm 1).  See
// include/fastgl_match.h for the contract.
//
// Match = set intersection through the same hash table as the ID map: the last mini-batch's IDs are
// inserted with their row as value, the new mini-batch's IDs probe it; the misses are compacted in
// position order (count per block, one-workgroup scan, rank) into the load lists.  The pairwise
// overlaps of n mini-batches come from ONE table over all their IDs whose entries carry a 64-bit
// mask of the mini-batches that hold the ID; every ID then adds its mask to its mini-batch's row of
// the count matrix (LDS histogram per workgroup, one atomic per workgroup and column).
#include <vector>

#include "fastgl_match.h"
#include "hash_table.h"
#include "internal.h"

namespace fastgl {
namespace {

struct MatchArgs {
    const int64_t *prev_gid, *new_gid;
    int64_t n_prev, n_new;
    Slot *table;
    int64_t cap;
    int32_t *block_cnt;
    int nblocks;
    int32_t *src_row, *load_pos;
    int64_t *load_gid;
    int32_t *result;
};

__global__ __launch_bounds__(256) void k_table_fill(Slot *table, int64_t cap, int32_t *zero, int nzero)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < nzero) zero[i] = 0;
    if (i >= cap) return;
    Slot e;
    e.key = -1;
    e.val = 0;
    e.lid = 0;
    table[i] = e;
}

__global__ __launch_bounds__(256) void k_match_insert_prev(MatchArgs a)
{
    const int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= a.n_prev) return;
    const int64_t gid = a.prev_gid[j];
    bool fresh = false;
    if (gid >= 0) {
        const uint32_t slot = insert_id(a.table, (uint32_t)a.cap, gid, fresh);
        if (fresh) a.table[slot].val = (int32_t)j;
    }
    if (!fresh) atomicAdd(&a.result[1], 1);          // negative or repeated ID
}

// Probe; hits get their row, misses -1 for now; misses are counted per block.
__global__ __launch_bounds__(kScanBlock) void k_match_probe(MatchArgs a)
{
    const int64_t i = (int64_t)blockIdx.x * kScanBlock + threadIdx.x;
    bool miss = false;
    if (i < a.n_new) {
        const int64_t gid = a.new_gid[i];
        int32_t row = -1;
        if (gid >= 0) {
            const int32_t slot = find_id(a.table, (uint32_t)a.cap, gid);
            if (slot != kNoSlot) row = a.table[slot].val;
        } else {
            atomicAdd(&a.result[1], 1);
        }
        a.src_row[i] = row;
        miss = row < 0;
    }
    const int c = __syncthreads_count(miss);
    if (threadIdx.x == 0) a.block_cnt[blockIdx.x] = c;
}

__global__ __launch_bounds__(kScanBlock) void k_match_scan(MatchArgs a)
{
    const int total = scan_block_counts(a.block_cnt, a.nblocks);
    if (threadIdx.x == 0) a.result[0] = total;
}

__global__ __launch_bounds__(kScanBlock) void k_match_rank(MatchArgs a)
{
    const int64_t i = (int64_t)blockIdx.x * kScanBlock + threadIdx.x;
    const bool miss = i < a.n_new && a.src_row[i] < 0;
    int k;
    block_exclusive_scan(miss ? 1 : 0, a.block_cnt[blockIdx.x], k);
    if (miss) {
        a.src_row[i] = -1 - k;
        a.load_pos[k] = (int32_t)i;
        a.load_gid[k] = a.new_gid[i];
    }
}

// Row copy: one thread moves one VEC-byte piece; consecutive threads take consecutive pieces of a row.
template <int VEC>
__global__ __launch_bounds__(256) void k_assemble_rows(const char *__restrict__ X_prev, const char *__restrict__ X_load,
                                                       const int32_t *__restrict__ src_row, int64_t n_new,
                                                       int64_t row_bytes, int pieces, char *__restrict__ X_new)
{
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t i = t / pieces;
    if (i >= n_new) return;
    const int64_t off = (t - i * pieces) * VEC;
    const int32_t r = src_row[i];
    const char *src = r >= 0 ? X_prev + (int64_t)r * row_bytes : X_load + (int64_t)(-1 - r) * row_bytes;
    char *dst = X_new + i * row_bytes + off;
    typedef float f32x4 __attribute__((ext_vector_type(4)));
    if (VEC == 16)
        __builtin_nontemporal_store(*reinterpret_cast<const f32x4 *>(src + off), reinterpret_cast<f32x4 *>(dst));
    else if (VEC == 4)
        *reinterpret_cast<uint32_t *>(dst) = *reinterpret_cast<const uint32_t *>(src + off);
    else
        *reinterpret_cast<uint16_t *>(dst) = *reinterpret_cast<const uint16_t *>(src + off);
}

struct OverlapArgs {
    const int64_t *gid;
    int64_t offsets[FASTGL_MAX_REORDER_BATCHES + 1];
    int n;
    int64_t total;
    Slot *table;
    int64_t cap;
    int32_t *slot_of;
    unsigned long long *counts;
    int32_t *violations;
};

__device__ __forceinline__ unsigned long long *mask_of(Slot *s)
{
    return reinterpret_cast<unsigned long long *>(&s->val);      // (val, lid) = 8 aligned bytes
}

// blockIdx.y = mini-batch, blockIdx.x walks its IDs.
__global__ __launch_bounds__(256) void k_overlap_insert(OverlapArgs a)
{
    const int b = blockIdx.y;
    const int64_t p = a.offsets[b] + (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= a.offsets[b + 1]) return;
    const int64_t gid = a.gid[p];
    if (gid < 0) {
        a.slot_of[p] = kNoSlot;
        atomicAdd(a.violations, 1);
        return;
    }
    bool fresh;
    const uint32_t slot = insert_id(a.table, (uint32_t)a.cap, gid, fresh);
    a.slot_of[p] = (int32_t)slot;
    const unsigned long long old = atomicOr(mask_of(&a.table[slot]), 1ull << b);
    if (old & (1ull << b)) atomicAdd(a.violations, 1);           // the mini-batch repeats this ID
}

__global__ __launch_bounds__(256) void k_overlap_count(OverlapArgs a)
{
    __shared__ int hist[FASTGL_MAX_REORDER_BATCHES];
    const int b = blockIdx.y;
    if (threadIdx.x < FASTGL_MAX_REORDER_BATCHES) hist[threadIdx.x] = 0;
    __syncthreads();
    const int64_t p = a.offsets[b] + (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (p < a.offsets[b + 1]) {
        const int32_t slot = a.slot_of[p];
        unsigned long long m = slot != kNoSlot ? *mask_of(&a.table[slot]) : 0ull;
        while (m) {
            const int j = __ffsll((long long)m) - 1;
            m &= m - 1;
            atomicAdd(&hist[j], 1);
        }
    }
    __syncthreads();
    if ((int)threadIdx.x < a.n && hist[threadIdx.x])
        atomicAdd(&a.counts[(int64_t)b * a.n + threadIdx.x], (unsigned long long)hist[threadIdx.x]);
}

__global__ __launch_bounds__(256) void k_zero_u64(unsigned long long *p, int64_t n)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0;
}

struct MatchLayout {
    size_t table, block_cnt, total;
};

MatchLayout match_layout(int64_t n_prev, int64_t n_new)
{
    MatchLayout L;
    size_t off = 0;
    L.table = off; off += align_up((size_t)table_slots(n_prev) * sizeof(Slot), 256);
    L.block_cnt = off; off += align_up((size_t)(ceil_div(n_new, kScanBlock) + 1) * 4, 256);
    L.total = off;
    return L;
}

struct OverlapLayout {
    size_t table, slot_of, total;
};

OverlapLayout overlap_layout(int64_t total_ids)
{
    OverlapLayout L;
    size_t off = 0;
    L.table = off; off += align_up((size_t)table_slots(total_ids) * sizeof(Slot), 256);
    L.slot_of = off; off += align_up((size_t)(total_ids > 0 ? total_ids : 1) * 4, 256);
    L.total = off;
    return L;
}

dim3 grid_for(int64_t items, int per) { return dim3((unsigned)(items > 0 ? ceil_div(items, per) : 1)); }

fastgl_status check_ws(void *workspace, size_t have, size_t need)
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

}  // namespace
}  // namespace fastgl

using namespace fastgl;

extern "C" {

size_t fastgl_match_workspace_bytes(int64_t n_prev, int64_t n_new)
{
    if (n_prev < 0 || n_new < 0 || n_prev >= kMaxIds || n_new >= kMaxIds) return 0;
    return match_layout(n_prev, n_new).total;
}

fastgl_status fastgl_match(const int64_t *prev_gid, int64_t n_prev, const int64_t *new_gid, int64_t n_new,
                           int32_t *src_row, int32_t *load_pos, int64_t *load_gid, int32_t *result,
                           void *workspace, size_t workspace_bytes, void *stream)
{
    if (n_prev < 0 || n_new < 0) {
        set_error("negative size (n_prev=%lld n_new=%lld)", (long long)n_prev, (long long)n_new);
        return FASTGL_ERR_INVALID_ARG;
    }
    if (n_prev >= kMaxIds || n_new >= kMaxIds) {
        set_error("n_prev and n_new must stay below 2^30");
        return FASTGL_ERR_UNSUPPORTED;
    }
    if ((n_prev > 0 && !prev_gid) || (n_new > 0 && (!new_gid || !src_row || !load_pos || !load_gid)) || !result) {
        set_error("NULL array (prev_gid, new_gid, src_row, load_pos, load_gid or result)");
        return FASTGL_ERR_INVALID_ARG;
    }
    if ((((uintptr_t)prev_gid | (uintptr_t)new_gid | (uintptr_t)load_gid) & 7) ||
        (((uintptr_t)src_row | (uintptr_t)load_pos | (uintptr_t)result) & 3)) {
        set_error("ID arrays must be 8-byte aligned, src_row, load_pos and result 4-byte aligned");
        return FASTGL_ERR_INVALID_ARG;
    }
    const MatchLayout L = match_layout(n_prev, n_new);
    fastgl_status st = check_ws(workspace, workspace_bytes, L.total);
    if (st != FASTGL_OK) return st;
    MatchArgs a = {};
    a.prev_gid = prev_gid; a.new_gid = new_gid; a.n_prev = n_prev; a.n_new = n_new;
    a.table = (Slot *)((char *)workspace + L.table);
    a.cap = table_slots(n_prev);
    a.block_cnt = (int32_t *)((char *)workspace + L.block_cnt);
    a.nblocks = (int)ceil_div(n_new, kScanBlock);
    a.src_row = src_row; a.load_pos = load_pos; a.load_gid = load_gid; a.result = result;
    hipStream_t s = (hipStream_t)stream;
    hipLaunchKernelGGL(k_table_fill, grid_for(a.cap, 256), dim3(256), 0, s, a.table, a.cap, result, 2);
    FASTGL_LAUNCH_CHECK("fastgl_match (fill)");
    if (n_prev > 0) {
        hipLaunchKernelGGL(k_match_insert_prev, grid_for(n_prev, 256), dim3(256), 0, s, a);
        FASTGL_LAUNCH_CHECK("fastgl_match (insert)");
    }
    if (n_new > 0) {
        hipLaunchKernelGGL(k_match_probe, dim3((unsigned)a.nblocks), dim3(kScanBlock), 0, s, a);
        FASTGL_LAUNCH_CHECK("fastgl_match (probe)");
        hipLaunchKernelGGL(k_match_scan, dim3(1), dim3(kScanBlock), 0, s, a);
        FASTGL_LAUNCH_CHECK("fastgl_match (scan)");
        hipLaunchKernelGGL(k_match_rank, dim3((unsigned)a.nblocks), dim3(kScanBlock), 0, s, a);
        FASTGL_LAUNCH_CHECK("fastgl_match (rank)");
    }
    return FASTGL_OK;
}

fastgl_status fastgl_assemble_rows(const void *X_prev, int64_t n_prev, const void *X_load, int64_t n_load,
                                   const int32_t *src_row, int64_t n_new, int64_t feat, fastgl_dtype dtype,
                                   void *X_new, void *stream)
{
    if (n_prev < 0 || n_load < 0 || n_new < 0 || feat <= 0) {
        set_error("bad size (n_prev=%lld n_load=%lld n_new=%lld feat=%lld)", (long long)n_prev, (long long)n_load,
                  (long long)n_new, (long long)feat);
        return FASTGL_ERR_INVALID_ARG;
    }
    if ((int)dtype < 0 || (int)dtype > 1) {
        set_error("unknown dtype %d", (int)dtype);
        return FASTGL_ERR_INVALID_ARG;
    }
    if (n_new == 0) return FASTGL_OK;
    if (!src_row || !X_new || (n_prev > 0 && !X_prev) || (n_load > 0 && !X_load)) {
        set_error("NULL array (src_row, X_new, X_prev or X_load)");
        return FASTGL_ERR_INVALID_ARG;
    }
    const int64_t elem = dtype == FASTGL_F32 ? 4 : 2;
    if ((((uintptr_t)X_prev | (uintptr_t)X_load | (uintptr_t)X_new) & (uintptr_t)(elem - 1)) || ((uintptr_t)src_row & 3)) {
        set_error("misaligned buffer");
        return FASTGL_ERR_INVALID_ARG;
    }
    if (n_new >= kMaxIds || feat > ((int64_t)1 << 24)) {
        set_error("assemble too large");
        return FASTGL_ERR_UNSUPPORTED;
    }
    const int64_t row_bytes = feat * elem;
    const bool v16 = row_bytes % 16 == 0 && ((((uintptr_t)X_prev | (uintptr_t)X_load | (uintptr_t)X_new) & 15) == 0);
    const int vec = v16 ? 16 : (int)elem;
    const int64_t pieces = row_bytes / vec;
    const int64_t threads = n_new * pieces;
    if (ceil_div(threads, 256) >= INT32_MAX) {
        set_error("assemble too large");
        return FASTGL_ERR_UNSUPPORTED;
    }
    const dim3 g = grid_for(threads, 256);
    hipStream_t s = (hipStream_t)stream;
    const char *xp = (const char *)X_prev, *xl = (const char *)X_load;
    if (vec == 16)
        hipLaunchKernelGGL(k_assemble_rows<16>, g, dim3(256), 0, s, xp, xl, src_row, n_new, row_bytes, (int)pieces,
                           (char *)X_new);
    else if (vec == 4)
        hipLaunchKernelGGL(k_assemble_rows<4>, g, dim3(256), 0, s, xp, xl, src_row, n_new, row_bytes, (int)pieces,
                           (char *)X_new);
    else
        hipLaunchKernelGGL(k_assemble_rows<2>, g, dim3(256), 0, s, xp, xl, src_row, n_new, row_bytes, (int)pieces,
                           (char *)X_new);
    FASTGL_LAUNCH_CHECK("fastgl_assemble_rows");
    return FASTGL_OK;
}

size_t fastgl_overlap_workspace_bytes(int64_t total_ids)
{
    if (total_ids < 0 || total_ids >= kMaxIds) return 0;
    return overlap_layout(total_ids).total;
}

fastgl_status fastgl_overlap_counts(const int64_t *gid, const int64_t *offsets_host, int n, int64_t *counts,
                                    int32_t *violations, void *workspace, size_t workspace_bytes, void *stream)
{
    if (n < 0 || n > FASTGL_MAX_REORDER_BATCHES) {
        set_error("n must be in [0, %d]", FASTGL_MAX_REORDER_BATCHES);
        return FASTGL_ERR_INVALID_ARG;
    }
    if (!offsets_host || !violations || (n > 0 && !counts)) {
        set_error("NULL array (offsets_host, counts or violations)");
        return FASTGL_ERR_INVALID_ARG;
    }
    int64_t longest = 0;
    for (int b = 0; b < n; ++b) {
        if (offsets_host[b] < 0 || offsets_host[b + 1] < offsets_host[b]) {
            set_error("offsets_host must start at >= 0 and not decrease");
            return FASTGL_ERR_INVALID_ARG;
        }
        if (offsets_host[b + 1] - offsets_host[b] > longest) longest = offsets_host[b + 1] - offsets_host[b];
    }
    if (n > 0 && offsets_host[0] != 0) {
        set_error("offsets_host[0] must be 0");
        return FASTGL_ERR_INVALID_ARG;
    }
    const int64_t total = n > 0 ? offsets_host[n] : 0;
    if (total >= kMaxIds) {
        set_error("total number of IDs must stay below 2^30");
        return FASTGL_ERR_UNSUPPORTED;
    }
    if ((total > 0 && !gid) || ((uintptr_t)gid & 7) || ((uintptr_t)counts & 7) || ((uintptr_t)violations & 3)) {
        set_error("gid is NULL or an array is misaligned");
        return FASTGL_ERR_INVALID_ARG;
    }
    const OverlapLayout L = overlap_layout(total);
    fastgl_status st = check_ws(workspace, workspace_bytes, L.total);
    if (st != FASTGL_OK) return st;
    OverlapArgs a = {};
    a.gid = gid; a.n = n; a.total = total;
    for (int b = 0; b <= n; ++b) a.offsets[b] = offsets_host[b];
    a.table = (Slot *)((char *)workspace + L.table);
    const int64_t cap = table_slots(total);
    a.cap = cap;
    a.slot_of = (int32_t *)((char *)workspace + L.slot_of);
    a.counts = (unsigned long long *)counts;
    a.violations = violations;
    hipStream_t s = (hipStream_t)stream;
    hipLaunchKernelGGL(k_table_fill, grid_for(cap, 256), dim3(256), 0, s, a.table, cap, violations, 1);
    FASTGL_LAUNCH_CHECK("fastgl_overlap_counts (fill)");
    if (n == 0) return FASTGL_OK;
    hipLaunchKernelGGL(k_zero_u64, grid_for((int64_t)n * n, 256), dim3(256), 0, s, a.counts, (int64_t)n * n);
    FASTGL_LAUNCH_CHECK("fastgl_overlap_counts (zero)");
    if (longest == 0) return FASTGL_OK;
    const dim3 g((unsigned)ceil_div(longest, 256), (unsigned)n);
    hipLaunchKernelGGL(k_overlap_insert, g, dim3(256), 0, s, a);
    FASTGL_LAUNCH_CHECK("fastgl_overlap_counts (insert)");
    hipLaunchKernelGGL(k_overlap_count, g, dim3(256), 0, s, a);
    FASTGL_LAUNCH_CHECK("fastgl_overlap_counts (count)");
    return FASTGL_OK;
}

fastgl_status fastgl_greedy_reorder(const int64_t *overlap_host, const int64_t *size_host, int64_t n,
                                    int32_t *order_host)
{
    if (n < 0 || n > ((int64_t)1 << 15)) {
        set_error("n must be in [0, 32768]");
        return FASTGL_ERR_INVALID_ARG;
    }
    if (n > 0 && (!overlap_host || !size_host || !order_host)) {
        set_error("NULL host array");
        return FASTGL_ERR_INVALID_ARG;
    }
    if (n == 0) return FASTGL_OK;
    // Walk the list: `last` is the mini-batch appended last, `todo` the ones still to place.
    std::vector<int32_t> todo;
    for (int64_t k = 1; k < n; ++k) todo.push_back((int32_t)k);
    int32_t last = 0;
    int64_t filled = 0;
    order_host[filled++] = 0;
    while (!todo.empty()) {
        size_t best = 0;
        double best_deg = -1.0;
        for (size_t t = 0; t < todo.size(); ++t) {        // ascending index, strict improvement: ties stay low
            const int32_t k = todo[t];
            const int64_t small = size_host[last] < size_host[k] ? size_host[last] : size_host[k];
            const double deg = small > 0 ? (double)overlap_host[(int64_t)last * n + k] / (double)small : 0.0;
            if (deg > best_deg) {
                best_deg = deg;
                best = t;
            }
        }
        last = todo[best];
        todo.erase(todo.begin() + (long)best);
        order_host[filled++] = last;
    }
    return FASTGL_OK;
}

}  // extern "C"
