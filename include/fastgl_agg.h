/*
 * fastgl_agg.h - C ABI of the MI355X (gfx950) block-aggregation library.
 *
 * The library implements the aggregation phase of a sampled GNN layer
 * (paper Section 2.1, Eq. 1) and its backward pass (Section 4.2, Eq. 5) over
 * one mini-batch "block": a bipartite graph from num_src source nodes to
 * num_dst destination (target) nodes, stored as CSR by destination row with
 * local node ids that are consecutive and start from 0 (Section 2.2).
 *
 *   forward :  out[u,:]  = sum_{e in row u}        w_e^{mode} * X[indices[e],:]
 *   backward:  dX[v,:]   = sum_{e : indices[e]=v}  w_e^{mode} * dOut[dst(e),:]
 *
 * with the per-edge weight of edge e = (u,v)
 *   SUM :  a_e
 *   MEAN:  a_e / max(din[u],1)
 *   GCN :  a_e / sqrt(max(din[u],1) * max(dout[v],1))
 * where a_e = edge_w[e] (or 1 if edge_w is NULL), din[u] is the length of row
 * u and dout[v] the number of edges whose source is v, both counted inside
 * the block.  The backward pass is the exact transpose of the forward pass
 * (Eq. 5 read as the chain rule of Eq. 1).  edge_w receives no gradient.
 *
 * Conventions common to every entry point
 *  - Every array argument is DEVICE memory owned by the caller unless the
 *    comment says "host".  The library never allocates or frees device memory;
 *    all scratch comes from the caller's plan / workspace buffers.
 *  - Work is enqueued on `stream` (a hipStream_t passed as void*; NULL is the
 *    default stream) and the call returns without synchronising the host,
 *    except fastgl_block_validate which says so.
 *  - indptr/indices are int32.  num_src, num_edges < 2^31.
 *  - Feature matrices are dense row-major with leading dimension `feat`;
 *    FASTGL_F32 rows are float, FASTGL_BF16 rows are bfloat16 bit patterns.
 *    f32 data is accumulated in fp64, bf16 data in fp32; the result is rounded
 *    once (nearest even) to the storage type.
 *  - Outputs are overwritten in full, including all-zero rows for nodes
 *    without edges.  Input and output buffers must not overlap.
 *  - Index contents are trusted on the fast path (use fastgl_block_validate).
 *    Everything checkable on the host is checked before any launch and
 *    reported through the return code; fastgl_last_error() holds the text.
 *  - Zero-sized blocks (num_dst == 0, num_src == 0 or num_edges == 0) are valid.
 */
#ifndef FASTGL_AGG_H
#define FASTGL_AGG_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    FASTGL_OK = 0,
    FASTGL_ERR_INVALID_ARG = 1, /* null pointer, negative size, bad enum, misaligned buffer */
    FASTGL_ERR_UNSUPPORTED = 2, /* sizes beyond the int32 index range */
    FASTGL_ERR_WORKSPACE = 3,   /* plan / workspace buffer too small */
    FASTGL_ERR_HIP = 4          /* a HIP call failed; see fastgl_last_error() */
} fastgl_status;

typedef enum { FASTGL_AGG_SUM = 0, FASTGL_AGG_MEAN = 1, FASTGL_AGG_GCN = 2 } fastgl_agg_mode;
typedef enum { FASTGL_F32 = 0, FASTGL_BF16 = 1 } fastgl_dtype;

/* Which parts of the per-block bookkeeping a plan holds. */
enum {
    FASTGL_PLAN_FWD = 1, /* in-degrees, scale factors, destination-side degree buckets */
    FASTGL_PLAN_BWD = 2, /* out-degrees, stable transpose CSR, source-side degree buckets;
                            implies FASTGL_PLAN_FWD */
    FASTGL_PLAN_ALL = 3,
    FASTGL_PLAN_PERM = 8,   /* with FASTGL_PLAN_BWD: also keep `perm`, the original edge id of every
                               transposed edge.  Only a backward pass WITH edge_w reads it. */
    FASTGL_PLAN_SRC_DEG = 4, /* with FASTGL_PLAN_FWD only: out-degrees and their scale factors by a
                               histogram, which is all a GCN-normalised FORWARD pass needs beyond
                               FASTGL_PLAN_FWD.  Lets the forward pass start before the transpose
                               (built in another plan, possibly on another stream) is ready. */
    FASTGL_PLAN_SHORT_DST_ROWS = 16 /* a hint that may be or-ed to any of the above: the caller states that
                               no destination row has more than fastgl_long_row_threshold() edges,
                               which a sampler with a fan-out below that knows for free (Section 2.2:
                               every target samples a fixed number of neighbours).  The degrees live in
                               device memory, so without the hint every forward pass has to launch the
                               long-row reduction kernel just to find that it has nothing to do; with
                               it that launch is skipped.  Only speed depends on the hint: a row that
                               is longer after all is still aggregated correctly, by one lane group
                               alone.  The backward pass (rows = sources) is not affected. */
};

/* Opaque host-side handle; points into the caller's device buffer. */
typedef struct fastgl_plan fastgl_plan;

/* Device views of what a plan built (all int32 unless noted).  Arrays a plan
 * was not asked to build are NULL.  Used by tests to compare the bookkeeping
 * bit for bit with the oracle. */
typedef struct {
    const int32_t *din;          /* [num_dst]   row lengths                                  */
    const int32_t *dout;         /* [num_src]   edges per source                              */
    const int32_t *indptr_T;     /* [num_src+1] transpose row pointers                        */
    const int32_t *indices_T;    /* [E] destination of the k-th edge in (source, edge id) order */
    const int32_t *perm;         /* [E] original edge id of that edge (FASTGL_PLAN_PERM only) */
    const float *dst_inv;        /* [num_dst]   1/max(din,1)                                  */
    const float *dst_rsqrt;      /* [num_dst]   1/sqrt(max(din,1))                            */
    const float *src_rsqrt;      /* [num_src]   1/sqrt(max(dout,1))                           */
    const int32_t *long_dst;     /* destination rows longer than fastgl_long_row_threshold(), ascending */
    const int32_t *chunk_ptr_dst;/* [n_long_dst+1] first partial-sum chunk of each such row   */
    const int32_t *long_src;     /* same for transpose rows                                   */
    const int32_t *chunk_ptr_src;
    const int32_t *counters;     /* [4] n_long_dst, n_chunks_dst, n_long_src, n_chunks_src    */
    const int32_t *split_dst;    /* [S+1], S = ceil((num_dst+E)/fastgl_work_per_group()): first row of
                                    every equal-work row set: min r with indptr[r] + r >= g * work  */
    const int32_t *split_src;    /* same over the transpose rows                              */
} fastgl_plan_view;

/* Forward aggregation of one block (Eq. 1).
 *  indptr[num_dst+1], indices[num_edges]: CSR by destination row.
 *  edge_w[num_edges] float or NULL.  X[num_src,feat] in, out[num_dst,feat] out.
 *  plan: NULL, or a plan built for exactly these indptr/indices with
 *        FASTGL_PLAN_FWD (mode GCN also needs FASTGL_PLAN_SRC_DEG or
 *        FASTGL_PLAN_BWD).  With NULL the bookkeeping is rebuilt inside
 *        `workspace` on every call.
 *  workspace: at least fastgl_block_workspace_bytes(...) bytes, 256-byte
 *        aligned; contents are scratch.  Calls that share a workspace or a
 *        plan must be ordered on one stream.
 * Errors: INVALID_ARG (nothing launched), WORKSPACE, UNSUPPORTED, HIP. */
fastgl_status fastgl_block_aggregate_fwd(
    const int32_t *indptr, const int32_t *indices, const float *edge_w,
    int64_t num_dst, int64_t num_src, int64_t num_edges, int64_t feat,
    fastgl_agg_mode mode, fastgl_dtype dtype,
    const void *X, void *out,
    const fastgl_plan *plan, void *workspace, size_t workspace_bytes, void *stream);

/* Backward aggregation of one block (Eq. 5): grad_X = A^T * grad_out with the
 * same edge weights as the forward pass.  grad_out[num_dst,feat] in,
 * grad_X[num_src,feat] out (every row written).  The pass pulls along a
 * stable transpose of the CSR, so results are deterministic (no atomics on
 * floating point).  plan needs FASTGL_PLAN_ALL, and FASTGL_PLAN_PERM as well when
 * edge_w is given; otherwise as forward. */
fastgl_status fastgl_block_aggregate_bwd(
    const int32_t *indptr, const int32_t *indices, const float *edge_w,
    int64_t num_dst, int64_t num_src, int64_t num_edges, int64_t feat,
    fastgl_agg_mode mode, fastgl_dtype dtype,
    const void *grad_out, void *grad_X,
    const fastgl_plan *plan, void *workspace, size_t workspace_bytes, void *stream);

/* Forward aggregation for callers that cannot allocate device memory and have no workspace to
 * hand over: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same arguments, checks, kernels and results as fastgl_block_aggregate_fwd with plan == NULL; the
 * scratch (forward bookkeeping of the block + partial sums of long rows) sits in a static device
 * array of FASTGL_STATIC_SCRATCH_BYTES that every GPU the library runs on holds until the process
 * ends.  The call allocates and frees nothing (no hipMalloc, no hipFree, no allocating library
 * routine).  Work is enqueued on `stream`, which must belong to the CURRENT device (the array of
 * that device is used); the first call on a device looks up the array's address (a symbol lookup,
 * no allocation) - make that call once before capturing a graph.
 * Limit: a block whose scratch need - roughly 12 num_dst + 8 num_src + (num_dst + num_edges) / 4 +
 * (num_edges / 85) * feat * (8 for f32, 4 for bf16) bytes - exceeds the array is refused with
 * FASTGL_ERR_WORKSPACE before anything is launched; fastgl_last_error() states both numbers.
 * All calls on one GPU share that GPU's array and it keeps the last call's contents: calls must
 * be ordered (one stream, or events); calls that overlap on one GPU race.  Nothing in the array
 * needs clearing between calls: every value is written by the call before the call reads it. */
#define FASTGL_STATIC_SCRATCH_BYTES (64u << 20)
fastgl_status fastgl_block_aggregate_fwd_static(
    const int32_t *indptr, const int32_t *indices, const float *edge_w,
    int64_t num_dst, int64_t num_src, int64_t num_edges, int64_t feat,
    fastgl_agg_mode mode, fastgl_dtype dtype,
    const void *X, void *out, void *stream);

/* Bytes of device memory a plan needs (includes sort scratch). */
size_t fastgl_block_plan_bytes(int64_t num_dst, int64_t num_src, int64_t num_edges);

/* Build the per-block bookkeeping on `stream` inside plan_mem (device,
 * 256-byte aligned, >= fastgl_block_plan_bytes): degrees, scale factors, the
 * stable transpose CSR (transposed rows keep ascending original edge id) and
 * the degree buckets.  `parts` is FASTGL_PLAN_FWD, FASTGL_PLAN_FWD | FASTGL_PLAN_SRC_DEG,
 * FASTGL_PLAN_BWD or FASTGL_PLAN_ALL, the last two optionally | FASTGL_PLAN_PERM.  The plan keeps
 * pointers to indptr/indices and plan_mem: they must outlive it and stay
 * unchanged.  *out receives a host handle to free with
 * fastgl_block_plan_destroy.  No host synchronisation. */
fastgl_status fastgl_block_plan_create(
    const int32_t *indptr, const int32_t *indices,
    int64_t num_dst, int64_t num_src, int64_t num_edges, int parts,
    void *plan_mem, size_t plan_bytes, void *stream, fastgl_plan **out);

/* One block of a mini-batch, for fastgl_block_plan_create_many (host struct;
 * the pointers inside are device pointers, as in fastgl_block_plan_create). */
typedef struct {
    const int32_t *indptr, *indices;
    int64_t num_dst, num_src, num_edges;
    int parts;
    void *plan_mem;
    size_t plan_bytes;
} fastgl_block_desc;

#define FASTGL_MAX_PLAN_BATCH 16

/* Build the plans of all blocks of a mini-batch (the layers of a sampled GNN,
 * paper Section 2.2) together: the same work as n calls of
 * fastgl_block_plan_create, but each stage of the bookkeeping is one launch for
 * all blocks, which matters because the stages are latency-bound.
 * blocks: host array of n <= FASTGL_MAX_PLAN_BATCH descriptors; out: host array
 * of n handles.  On any error no plan is created and every out[i] is NULL. */
fastgl_status fastgl_block_plan_create_many(int n, const fastgl_block_desc *blocks, void *stream,
                                            fastgl_plan **out);

/* Fill *view (host struct) with the plan's device pointers. */
fastgl_status fastgl_block_plan_export(const fastgl_plan *plan, fastgl_plan_view *view);

/* Free the host handle (device memory stays the caller's). NULL is allowed. */
void fastgl_block_plan_destroy(fastgl_plan *plan);

/* Workspace bytes for fwd/bwd on a block of this size: room for the partial
 * sums of long rows, plus a whole plan so that plan == NULL works. */
size_t fastgl_block_workspace_bytes(int64_t num_dst, int64_t num_src, int64_t num_edges,
                                    int64_t feat, fastgl_dtype dtype);

/* Rows longer than this many edges are split into chunks of
 * fastgl_long_row_chunk() edges whose partial sums are reduced in a fixed order. */
int32_t fastgl_long_row_threshold(void);
int32_t fastgl_long_row_chunk(void);

/* The plan cuts the rows into consecutive sets of this much work (edges + rows)
 * each; a lane group of the aggregation kernels takes 1-8 consecutive sets, so no
 * group is overloaded however skewed the degrees are. */
int32_t fastgl_work_per_group(void);

/* Row gather from a device-resident feature table, the device-side tail of the
 * memory-IO phase (Section 2.2): out[i,:] = table[ids[i],:], ids int64[n] in
 * [0, table_rows).  table_rows is used for 64-bit offset arithmetic only. */
fastgl_status fastgl_gather_rows(const void *table, int64_t table_rows, const int64_t *ids,
                                 int64_t n, int64_t feat, fastgl_dtype dtype, void *out,
                                 void *stream);

/* Debug check of a block's index arrays.  Counts violations (indptr[0] != 0,
 * decreasing indptr, indptr[num_dst] != num_edges, source id outside
 * [0,num_src)).  scratch: device, >= 8 bytes.  SYNCHRONISES the stream and
 * writes the count to *n_violations (host). */
fastgl_status fastgl_block_validate(const int32_t *indptr, const int32_t *indices,
                                    int64_t num_dst, int64_t num_src, int64_t num_edges,
                                    void *scratch, int64_t *n_violations, void *stream);

/* Text of the last error on the calling thread ("" if none). Host string. */
const char *fastgl_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* FASTGL_AGG_H */
