// Device-side pieces shared by the ID map and the Match process: an open-addressing table of
// 64-bit global IDs (linear probing, keys claimed by compare-and-swap from the empty marker -1) and
// a workgroup-wide exclusive prefix sum.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace fastgl {

constexpr int kScanBlock = 1024;             // threads (= positions) per block of the counting / ranking passes
constexpr int64_t kMaxIds = (int64_t)1 << 30;
constexpr int32_t kNoSlot = 0x7FFFFFFF;      // no table has this many slots

// One table entry: the key and what is looked up through it share a 16-byte line piece.
struct __attribute__((aligned(16))) Slot {
    int64_t key;              // global ID, -1 while empty
    int32_t val;              // ID map, ordered: smallest position seen; fused: local ID; Match: row
    int32_t lid;              // ID map, ordered: local ID.  (val, lid) together: 64-bit batch mask
};

// Capacity for n DISTINCT keys (Match, overlap counts): 2n slots (at least 1024), so the table is
// never more than half full and a probe sequence always ends at an empty slot.
inline int64_t table_slots(int64_t n)
{
    const int64_t cap = 2 * n;
    return cap < 1024 ? 1024 : cap;
}

// Capacity for the n input IDs of the ID map, most of which repeat (a sampled hop holds every hub
// many times): 1.5 n slots.  The table can never fill up (there are at most n keys), a hop whose IDs
// are all distinct loads it to two thirds, a typical one (a third to a half distinct) to a quarter.
// Sized by the distinct IDs it would be smaller still, but their number is only known afterwards.
inline int64_t idmap_slots(int64_t n)
{
    const int64_t cap = n + n / 2;
    return cap < 1024 ? 1024 : cap;
}

// Slot of an ID in a table of `cap` slots (any size below 2^31, not only powers of two): the upper
// half of a multiplicative hash scaled to [0, cap).
__device__ __forceinline__ uint32_t hash_slot(int64_t gid, uint32_t cap)
{
    const uint32_t h = (uint32_t)(((uint64_t)gid * 0x9E3779B97F4A7C15ull) >> 32);
    return (uint32_t)(((uint64_t)h * cap) >> 32);
}

__device__ __forceinline__ uint32_t next_slot(uint32_t slot, uint32_t cap) { return slot + 1 == cap ? 0u : slot + 1; }

// Slot that holds gid after the call; fresh = this thread put it there.  Keys sit STRIDE bytes apart
// from `keys` on (16: the key of a Slot; 8: a bare array of keys).  The slot is read with a plain load
// first and the compare-and-swap is only issued when that showed the empty marker: a key changes
// exactly once (from -1 to an ID), so anything else that is read is final.  Ends because the table
// always keeps empty slots.
template <int STRIDE>
__device__ __forceinline__ uint32_t insert_key(void *keys, uint32_t cap, int64_t gid, bool &fresh)
{
    uint32_t slot = hash_slot(gid, cap);
    fresh = false;
    for (;;) {
        int64_t *kp = reinterpret_cast<int64_t *>(static_cast<char *>(keys) + (size_t)slot * STRIDE);
        int64_t k = __hip_atomic_load(kp, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (k == -1) {
            k = (int64_t)atomicCAS((unsigned long long *)kp, (unsigned long long)-1ll, (unsigned long long)gid);
            if (k == -1) {
                fresh = true;
                return slot;
            }
        }
        if (k == gid) return slot;
        slot = next_slot(slot, cap);
    }
}

__device__ __forceinline__ uint32_t insert_id(Slot *table, uint32_t cap, int64_t gid, bool &fresh)
{
    return insert_key<(int)sizeof(Slot)>(table, cap, gid, fresh);
}

// Slot that holds gid in a table that is no longer written, or kNoSlot.  Ends at the first empty slot.
__device__ __forceinline__ int32_t find_id(const Slot *table, uint32_t cap, int64_t gid)
{
    uint32_t slot = hash_slot(gid, cap);
    for (;;) {
        const int64_t k = table[slot].key;
        if (k == gid) return (int32_t)slot;
        if (k == -1) return kNoSlot;
        slot = next_slot(slot, cap);
    }
}

// Exclusive prefix sum of v over the workgroup (blockDim.x a multiple of 64, at most kScanBlock),
// `base` added to every result; returns the workgroup's total to every thread.
__device__ __forceinline__ int block_exclusive_scan(int v, int base, int &out_excl)
{
    __shared__ int wave_sum[kScanBlock / 64];
    __shared__ int total_s;
    const int lane = threadIdx.x & 63, wv = threadIdx.x / 64;
    int incl = v;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const int t = __shfl_up(incl, d);
        if (lane >= d) incl += t;
    }
    if (lane == 63) wave_sum[wv] = incl;
    __syncthreads();
    if (wv == 0) {
        const int nw = blockDim.x / 64;
        const int w = lane < nw ? wave_sum[lane] : 0;
        int wi = w;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const int t = __shfl_up(wi, d);
            if (lane >= d) wi += t;
        }
        if (lane < nw) wave_sum[lane] = wi - w;
        if (lane == nw - 1) total_s = wi;
    }
    __syncthreads();
    out_excl = base + wave_sum[wv] + incl - v;
    const int total = total_s;
    __syncthreads();
    return total;
}

// Block counts -> exclusive block offsets in place, by ONE workgroup of kScanBlock threads; returns
// the grand total to every thread.
__device__ __forceinline__ int scan_block_counts(int32_t *block_cnt, int nblocks)
{
    int running = 0;
    for (int b0 = 0; b0 < nblocks; b0 += kScanBlock) {
        const int b = b0 + threadIdx.x;
        const int v = b < nblocks ? block_cnt[b] : 0;
        int excl;
        const int total = block_exclusive_scan(v, running, excl);
        if (b < nblocks) block_cnt[b] = excl;
        running += total;
    }
    return running;
}

}  // namespace fastgl
