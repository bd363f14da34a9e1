// Internal declarations shared by the translation units of libfastgl_agg.so.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "fastgl_agg.h"

namespace fastgl {

constexpr int kWave = 64;
constexpr int kBlock = 256;            // threads per workgroup (4 wavefronts)
constexpr int kLongThreshold = 256;    // rows longer than this go through the chunked path
constexpr int kLongChunk = 128;        // edges per partial-sum chunk
constexpr int kWorkPerGroup = 16;      // edges + rows per fine row set (a lane group takes 1-8 sets)
constexpr int kMaxScanBlocks = 1024;   // blocks of a two-kernel scan / compaction
constexpr int kRadixBits = 8;
constexpr int kRadixBins = 1 << kRadixBits;
constexpr int64_t kMaxIndex = INT32_MAX - 1024;   // largest num_dst / num_src / num_edges accepted
constexpr int kXcds = 8;               // workgroups are dealt round-robin to 8 L2 domains

void set_error(const char *fmt, ...);
fastgl_status hip_fail(hipError_t e, const char *what);

#define FASTGL_HIP(call)                                                    \
    do {                                                                    \
        hipError_t e__ = (call);                                            \
        if (e__ != hipSuccess) return ::fastgl::hip_fail(e__, #call);       \
    } while (0)

#define FASTGL_LAUNCH_CHECK(name)                                           \
    do {                                                                    \
        hipError_t e__ = hipGetLastError();                                 \
        if (e__ != hipSuccess) return ::fastgl::hip_fail(e__, name);        \
    } while (0)

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// Upper bounds used to size the bucket arrays without knowing the degrees.
inline int64_t cap_long_rows(int64_t num_edges) { return num_edges / (kLongThreshold + 1) + 1; }
inline int64_t num_row_sets(int64_t rows, int64_t nnz) { return ceil_div(rows + nnz, kWorkPerGroup); }
inline int64_t cap_chunks(int64_t num_edges) { return num_edges / kLongChunk + cap_long_rows(num_edges) + 1; }

}  // namespace fastgl

// Host handle of a plan: device pointers carved out of the caller's buffer.
struct fastgl_plan {
    int64_t num_dst, num_src, num_edges;
    const int32_t *indptr, *indices;
    int parts;
    int32_t *din, *dout, *indptr_T, *indices_T, *perm;
    float *dst_inv, *dst_rsqrt, *src_rsqrt;
    int32_t *long_dst, *chunk_ptr_dst, *long_src, *chunk_ptr_src;
    int32_t *split_dst, *split_src;   // [row sets + 1] first row of each equal-work row set
    int32_t *counters;      // [4] n_long_dst, n_chunks_dst, n_long_src, n_chunks_src
    // scratch
    int32_t *sort_buf[6];   // ping-pong keys / destination rows / edge ids, num_edges each
    int32_t *edge_dst;      // [num_edges] destination row of every edge
    int32_t *radix_cnt;     // [sort blocks][digits]: digit counts of a sort pass / of the split into buckets
    int32_t *bucket_tot;    // [buckets] edges per bucket of the bucketed transpose
    void *bucket_map;       // which bucket (and part of it) each workgroup of the bucket stage finishes
    void *bucket_subcnt;    // edges per source of the parts of buckets that are finished in several parts
    int32_t *block_sums;    // 2 * kMaxScanBlocks (destination-side bucket counts)
    int32_t *block_sums2;   // same for the source side
};

namespace fastgl {

// Carves a plan's arrays out of `base` (NULL: only the size is wanted).  fwd_only: room for what a
// forward pass without a caller's plan needs (degrees, scale factors, destination-side buckets and
// row sets); every transpose-side pointer is NULL then.
size_t plan_layout(fastgl_plan *p, void *base, int64_t num_dst, int64_t num_src, int64_t num_edges,
                   bool fwd_only = false);
fastgl_status plan_build(fastgl_plan *p, int parts, bool need_src_degrees, hipStream_t s);
fastgl_status plans_build(fastgl_plan *const *plans, const int *parts, const bool *src_deg, int n, hipStream_t s);

struct PullDesc {
    const int32_t *rowptr;     // [num_rows+1]
    const int32_t *col;        // [nnz] gathered row of `in` per edge
    const int32_t *eid;        // [nnz] index into edge_w, or NULL for identity
    const float *edge_w;       // or NULL
    const float *col_scale;    // [rows of in] or NULL
    int row_mode;              // 0: none, 1: 1/len, 2: 1/sqrt(len)  (len clamped to >= 1)
    int64_t num_rows;          // rows of out
    int64_t num_cols;          // rows of in
    int64_t nnz;
    int64_t feat;
    fastgl_dtype dtype;
    const void *in;
    void *out;
    // long-row bucket (device-resident counts)
    const int32_t *long_rows, *chunk_ptr, *n_long, *n_chunks;
    void *partials;            // cap_chunks * feat accumulators
    // equal-work row sets
    const int32_t *split;      // [nsets+1]
    int64_t nsets;
};

fastgl_status launch_pull(const PullDesc &d, hipStream_t s);

// The parts of fastgl_block_aggregate_fwd / _bwd.  aggregate_check: every host-side check, no HIP
// call; *need = workspace bytes the call takes.  aggregate_prepare: bookkeeping (when plan is NULL)
// and the descriptor of the pull; aggregate_run: that plus the aggregation launches - both for a call
// that passed the check, on a workspace of >= *need bytes.
fastgl_status aggregate_check(bool backward, const int32_t *indptr, const int32_t *indices, const float *edge_w,
                              int64_t num_dst, int64_t num_src, int64_t num_edges, int64_t feat,
                              fastgl_agg_mode mode, fastgl_dtype dtype, const void *in, void *out,
                              const fastgl_plan *plan, size_t *need);
fastgl_status aggregate_prepare(bool backward, const int32_t *indptr, const int32_t *indices, const float *edge_w,
                                int64_t num_dst, int64_t num_src, int64_t num_edges, int64_t feat,
                                fastgl_agg_mode mode, fastgl_dtype dtype, const void *in, void *out,
                                const fastgl_plan *plan, void *workspace, void *stream, fastgl_plan *local,
                                PullDesc *desc);
fastgl_status aggregate_run(bool backward, const int32_t *indptr, const int32_t *indices, const float *edge_w,
                            int64_t num_dst, int64_t num_src, int64_t num_edges, int64_t feat,
                            fastgl_agg_mode mode, fastgl_dtype dtype, const void *in, void *out,
                            const fastgl_plan *plan, void *workspace, void *stream);
fastgl_status launch_gather_rows(const void *table, const int64_t *ids, int64_t n, int64_t feat,
                                 fastgl_dtype dtype, void *out, hipStream_t s);
fastgl_status validate_block(const int32_t *indptr, const int32_t *indices, int64_t num_dst,
                             int64_t num_src, int64_t num_edges, void *scratch, int64_t *n_violations,
                             hipStream_t s);

}  // namespace fastgl
