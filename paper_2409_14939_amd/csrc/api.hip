// C ABI of libfastgl_agg.so: argument checks, plan / workspace carving and the
// launch sequence of one forward or backward aggregation.  See
// include/fastgl_agg.h for the contract of every entry point.
#include <stdarg.h>
#include <stdio.h>
#include <new>

#include "internal.h"

namespace fastgl {

static thread_local char g_err[512] = "";

void set_error(const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

fastgl_status hip_fail(hipError_t e, const char *what)
{
    set_error("%s: %s", what, hipGetErrorString(e));
    return FASTGL_ERR_HIP;
}

static fastgl_status check_block(const int32_t *indptr, const int32_t *indices, int64_t num_dst,
                                 int64_t num_src, int64_t num_edges)
{
    if (num_dst < 0 || num_src < 0 || num_edges < 0) {
        set_error("negative size (num_dst=%lld num_src=%lld num_edges=%lld)", (long long)num_dst,
                  (long long)num_src, (long long)num_edges);
        return FASTGL_ERR_INVALID_ARG;
    }
    // the kernels look a few hundred positions ahead of the last edge / row in 32-bit arithmetic
    // (column ids two chunks ahead, the end of a long-row chunk), so the sizes keep that distance
    // from the top of the int32 range
    if (num_dst > kMaxIndex || num_src > kMaxIndex || num_edges > kMaxIndex) {
        set_error("sizes must not exceed 2^31-1-%d (int32 indices with look-ahead)", INT32_MAX - kMaxIndex);
        return FASTGL_ERR_UNSUPPORTED;
    }
    if (!indptr) {
        set_error("indptr is NULL");
        return FASTGL_ERR_INVALID_ARG;
    }
    if (!indices && num_edges > 0) {
        set_error("indices is NULL but num_edges > 0");
        return FASTGL_ERR_INVALID_ARG;
    }
    if (num_edges > 0 && (num_dst == 0 || num_src == 0)) {
        set_error("edges need at least one destination and one source node");
        return FASTGL_ERR_INVALID_ARG;
    }
    if (((uintptr_t)indptr | (uintptr_t)indices) & 3) {
        set_error("indptr / indices must be 4-byte aligned");
        return FASTGL_ERR_INVALID_ARG;
    }
    return FASTGL_OK;
}

static size_t partial_bytes(int64_t num_edges, int64_t feat, fastgl_dtype dtype)
{
    return align_up((size_t)cap_chunks(num_edges) * (size_t)feat * (dtype == FASTGL_F32 ? 8 : 4), 256);
}

// Host-side checks of a forward / backward call; nothing is launched.  *need = bytes of workspace the
// call takes (partial sums of long rows, plus the bookkeeping when no plan is passed).
fastgl_status aggregate_check(bool backward, const int32_t *indptr, const int32_t *indices, const float *edge_w,
                              int64_t num_dst, int64_t num_src, int64_t num_edges, int64_t feat,
                              fastgl_agg_mode mode, fastgl_dtype dtype, const void *in, void *out,
                              const fastgl_plan *plan, size_t *need)
{
    fastgl_status st = check_block(indptr, indices, num_dst, num_src, num_edges);
    if (st != FASTGL_OK) return st;
    if (feat <= 0) {
        set_error("feat must be positive (got %lld)", (long long)feat);
        return FASTGL_ERR_INVALID_ARG;
    }
    if ((int)mode < 0 || (int)mode > 2) {
        set_error("unknown aggregation mode %d", (int)mode);
        return FASTGL_ERR_INVALID_ARG;
    }
    if ((int)dtype < 0 || (int)dtype > 1) {
        set_error("unknown dtype %d", (int)dtype);
        return FASTGL_ERR_INVALID_ARG;
    }
    const int64_t in_rows = backward ? num_dst : num_src, out_rows = backward ? num_src : num_dst;
    if ((!in && in_rows > 0) || (!out && out_rows > 0)) {
        set_error("feature matrix pointer is NULL");
        return FASTGL_ERR_INVALID_ARG;
    }
    const uintptr_t emask = dtype == FASTGL_F32 ? 3 : 1;
    if ((((uintptr_t)in | (uintptr_t)out) & emask) || ((uintptr_t)edge_w & 3)) {
        set_error("feature / weight buffers must be aligned to their element size");
        return FASTGL_ERR_INVALID_ARG;
    }
    if (feat > (int64_t)1 << 24) {
        set_error("feat too large (%lld)", (long long)feat);
        return FASTGL_ERR_UNSUPPORTED;
    }
    *need = partial_bytes(num_edges, feat, dtype);
    if (plan) {
        const int need_parts = backward ? (FASTGL_PLAN_ALL | (edge_w ? FASTGL_PLAN_PERM : 0)) : FASTGL_PLAN_FWD;
        if (plan->indptr != indptr || plan->indices != indices || plan->num_dst != num_dst ||
            plan->num_src != num_src || plan->num_edges != num_edges) {
            set_error("plan was built for a different block");
            return FASTGL_ERR_INVALID_ARG;
        }
        if ((plan->parts & need_parts) != need_parts) {
            set_error("plan lacks the parts this pass needs (has %d, needs %d)", plan->parts, need_parts);
            return FASTGL_ERR_INVALID_ARG;
        }
        if (mode == FASTGL_AGG_GCN && !backward && !(plan->parts & (FASTGL_PLAN_BWD | FASTGL_PLAN_SRC_DEG))) {
            set_error("GCN forward needs a plan with source degrees (FASTGL_PLAN_SRC_DEG or FASTGL_PLAN_BWD)");
            return FASTGL_ERR_INVALID_ARG;
        }
    } else {
        // a forward pass needs no transpose: its bookkeeping takes a fraction of a whole plan's room
        *need += plan_layout(nullptr, nullptr, num_dst, num_src, num_edges, !backward);
    }
    return FASTGL_OK;
}

// What a call that passed aggregate_check launches, short of the aggregation kernel itself: the
// bookkeeping when no plan is passed (enqueued here, inside `workspace`), and the descriptor of the
// pull.  *local is storage for the plan built here; it must live until the launches are enqueued.
fastgl_status aggregate_prepare(bool backward, const int32_t *indptr, const int32_t *indices, const float *edge_w,
                                int64_t num_dst, int64_t num_src, int64_t num_edges, int64_t feat,
                                fastgl_agg_mode mode, fastgl_dtype dtype, const void *in, void *out,
                                const fastgl_plan *plan, void *workspace, void *stream, fastgl_plan *local,
                                PullDesc *desc)
{
    hipStream_t s = (hipStream_t)stream;
    const fastgl_plan *pl = plan;
    if (!plan) {
        const int need_parts = backward ? (FASTGL_PLAN_ALL | (edge_w ? FASTGL_PLAN_PERM : 0)) : FASTGL_PLAN_FWD;
        local->num_dst = num_dst; local->num_src = num_src; local->num_edges = num_edges;
        local->indptr = indptr; local->indices = indices;
        plan_layout(local, (char *)workspace + partial_bytes(num_edges, feat, dtype), num_dst, num_src, num_edges,
                    !backward);
        fastgl_status st = plan_build(local, need_parts, mode == FASTGL_AGG_GCN, s);
        if (st != FASTGL_OK) return st;
        pl = local;
    }

    PullDesc &d = *desc;
    d.edge_w = edge_w;
    d.feat = feat;
    d.dtype = dtype;
    d.in = in;
    d.out = out;
    d.nnz = num_edges;
    d.partials = workspace;
    if (!backward) {
        d.rowptr = indptr; d.col = indices; d.eid = nullptr;
        d.col_scale = mode == FASTGL_AGG_GCN ? pl->src_rsqrt : nullptr;
        d.row_mode = mode == FASTGL_AGG_MEAN ? 1 : mode == FASTGL_AGG_GCN ? 2 : 0;
        d.num_rows = num_dst; d.num_cols = num_src;
        // a plan with the short-rows hint: no chunk phase, no reduction launch (rows that are long
        // after all are walked like any other row)
        const bool chunked = !(pl->parts & FASTGL_PLAN_SHORT_DST_ROWS);
        d.long_rows = chunked ? pl->long_dst : nullptr; d.chunk_ptr = pl->chunk_ptr_dst;
        d.n_long = pl->counters; d.n_chunks = pl->counters + 1;
        d.split = pl->split_dst; d.nsets = num_row_sets(num_dst, num_edges);
    } else {
        d.rowptr = pl->indptr_T; d.col = pl->indices_T; d.eid = pl->perm;
        d.col_scale = mode == FASTGL_AGG_MEAN ? pl->dst_inv : mode == FASTGL_AGG_GCN ? pl->dst_rsqrt : nullptr;
        d.row_mode = mode == FASTGL_AGG_GCN ? 2 : 0;
        d.num_rows = num_src; d.num_cols = num_dst;
        d.long_rows = pl->long_src; d.chunk_ptr = pl->chunk_ptr_src;
        d.n_long = pl->counters + 2; d.n_chunks = pl->counters + 3;
        d.split = pl->split_src; d.nsets = num_row_sets(num_src, num_edges);
    }
    return FASTGL_OK;
}

// The launches of a call that passed aggregate_check; workspace holds at least the bytes it asked for.
fastgl_status aggregate_run(bool backward, const int32_t *indptr, const int32_t *indices, const float *edge_w,
                            int64_t num_dst, int64_t num_src, int64_t num_edges, int64_t feat,
                            fastgl_agg_mode mode, fastgl_dtype dtype, const void *in, void *out,
                            const fastgl_plan *plan, void *workspace, void *stream)
{
    fastgl_plan local;
    PullDesc d;
    fastgl_status st = aggregate_prepare(backward, indptr, indices, edge_w, num_dst, num_src, num_edges, feat, mode,
                                         dtype, in, out, plan, workspace, stream, &local, &d);
    if (st != FASTGL_OK) return st;
    return launch_pull(d, (hipStream_t)stream);
}

static fastgl_status aggregate(bool backward, const int32_t *indptr, const int32_t *indices, const float *edge_w,
                               int64_t num_dst, int64_t num_src, int64_t num_edges, int64_t feat,
                               fastgl_agg_mode mode, fastgl_dtype dtype, const void *in, void *out,
                               const fastgl_plan *plan, void *workspace, size_t workspace_bytes, void *stream)
{
    size_t need = 0;
    fastgl_status st = aggregate_check(backward, indptr, indices, edge_w, num_dst, num_src, num_edges, feat, mode,
                                       dtype, in, out, plan, &need);
    if (st != FASTGL_OK) return st;
    if (!workspace || ((uintptr_t)workspace & 255)) {
        set_error("workspace must be a 256-byte aligned device buffer");
        return FASTGL_ERR_INVALID_ARG;
    }
    if (workspace_bytes < need) {
        set_error("workspace too small: %zu < %zu bytes", workspace_bytes, need);
        return FASTGL_ERR_WORKSPACE;
    }
    return aggregate_run(backward, indptr, indices, edge_w, num_dst, num_src, num_edges, feat, mode, dtype, in, out,
                         plan, workspace, stream);
}

}  // namespace fastgl

using namespace fastgl;

extern "C" {

fastgl_status fastgl_block_aggregate_fwd(const int32_t *indptr, const int32_t *indices, const float *edge_w,
                                         int64_t num_dst, int64_t num_src, int64_t num_edges, int64_t feat,
                                         fastgl_agg_mode mode, fastgl_dtype dtype, const void *X, void *out,
                                         const fastgl_plan *plan, void *workspace, size_t workspace_bytes,
                                         void *stream)
{
    return aggregate(false, indptr, indices, edge_w, num_dst, num_src, num_edges, feat, mode, dtype, X, out,
                     plan, workspace, workspace_bytes, stream);
}

fastgl_status fastgl_block_aggregate_bwd(const int32_t *indptr, const int32_t *indices, const float *edge_w,
                                         int64_t num_dst, int64_t num_src, int64_t num_edges, int64_t feat,
                                         fastgl_agg_mode mode, fastgl_dtype dtype, const void *grad_out,
                                         void *grad_X, const fastgl_plan *plan, void *workspace,
                                         size_t workspace_bytes, void *stream)
{
    return aggregate(true, indptr, indices, edge_w, num_dst, num_src, num_edges, feat, mode, dtype, grad_out,
                     grad_X, plan, workspace, workspace_bytes, stream);
}

size_t fastgl_block_plan_bytes(int64_t num_dst, int64_t num_src, int64_t num_edges)
{
    if (num_dst < 0 || num_src < 0 || num_edges < 0) return 0;
    return plan_layout(nullptr, nullptr, num_dst, num_src, num_edges);
}

fastgl_status fastgl_block_plan_create_many(int n, const fastgl_block_desc *blocks, void *stream,
                                            fastgl_plan **out)
{
    if (n < 0 || n > FASTGL_MAX_PLAN_BATCH || (n > 0 && (!blocks || !out))) {
        set_error("n must be in [0, %d] and blocks / out must not be NULL", FASTGL_MAX_PLAN_BATCH);
        return FASTGL_ERR_INVALID_ARG;
    }
    for (int i = 0; i < n; ++i) out[i] = nullptr;
    for (int i = 0; i < n; ++i) {
        const fastgl_block_desc &d = blocks[i];
        fastgl_status st = check_block(d.indptr, d.indices, d.num_dst, d.num_src, d.num_edges);
        if (st != FASTGL_OK) return st;
        const int what = d.parts & ~FASTGL_PLAN_SHORT_DST_ROWS;      // the hint goes with any combination
        const int base = what & ~FASTGL_PLAN_PERM;
        const bool ok = what == FASTGL_PLAN_FWD || what == (FASTGL_PLAN_FWD | FASTGL_PLAN_SRC_DEG) ||
                        base == FASTGL_PLAN_BWD || base == FASTGL_PLAN_ALL;
        if (!ok || d.parts < 0 || d.parts > 31) {
            set_error("block %d: parts must be FWD, FWD|SRC_DEG, BWD[|PERM] or ALL[|PERM], each optionally "
                      "|SHORT_DST_ROWS (got %d)", i, d.parts);
            return FASTGL_ERR_INVALID_ARG;
        }
        if (!d.plan_mem || ((uintptr_t)d.plan_mem & 255)) {
            set_error("block %d: plan_mem must be a 256-byte aligned device buffer", i);
            return FASTGL_ERR_INVALID_ARG;
        }
        const size_t need = plan_layout(nullptr, nullptr, d.num_dst, d.num_src, d.num_edges);
        if (d.plan_bytes < need) {
            set_error("block %d: plan buffer too small: %zu < %zu bytes", i, d.plan_bytes, need);
            return FASTGL_ERR_WORKSPACE;
        }
    }
    fastgl_plan *plans[FASTGL_MAX_PLAN_BATCH];
    int parts[FASTGL_MAX_PLAN_BATCH];
    bool src_deg[FASTGL_MAX_PLAN_BATCH], short_dst[FASTGL_MAX_PLAN_BATCH];
    fastgl_status st = FASTGL_OK;
    int made = 0;
    for (; made < n; ++made) {
        const fastgl_block_desc &d = blocks[made];
        fastgl_plan *p = new (std::nothrow) fastgl_plan;
        if (!p) {
            set_error("out of host memory");
            st = FASTGL_ERR_INVALID_ARG;
            break;
        }
        p->num_dst = d.num_dst; p->num_src = d.num_src; p->num_edges = d.num_edges;
        p->indptr = d.indptr; p->indices = d.indices;
        plan_layout(p, d.plan_mem, d.num_dst, d.num_src, d.num_edges);
        plans[made] = p;
        // a backward plan also carries what the forward pass of the same block needs
        parts[made] = (d.parts & FASTGL_PLAN_BWD) ? (FASTGL_PLAN_ALL | (d.parts & FASTGL_PLAN_PERM)) : FASTGL_PLAN_FWD;
        src_deg[made] = (d.parts & FASTGL_PLAN_SRC_DEG) != 0;
        short_dst[made] = (d.parts & FASTGL_PLAN_SHORT_DST_ROWS) != 0;
    }
    if (st == FASTGL_OK) st = plans_build(plans, parts, src_deg, n, (hipStream_t)stream);
    if (st != FASTGL_OK) {
        for (int i = 0; i < made; ++i) delete plans[i];
        return st;
    }
    for (int i = 0; i < n; ++i) {
        if (short_dst[i]) plans[i]->parts |= FASTGL_PLAN_SHORT_DST_ROWS;
        out[i] = plans[i];
    }
    return FASTGL_OK;
}

fastgl_status fastgl_block_plan_create(const int32_t *indptr, const int32_t *indices, int64_t num_dst,
                                       int64_t num_src, int64_t num_edges, int parts, void *plan_mem,
                                       size_t plan_bytes, void *stream, fastgl_plan **out)
{
    if (!out) {
        set_error("out is NULL");
        return FASTGL_ERR_INVALID_ARG;
    }
    fastgl_block_desc d;
    d.indptr = indptr; d.indices = indices;
    d.num_dst = num_dst; d.num_src = num_src; d.num_edges = num_edges;
    d.parts = parts; d.plan_mem = plan_mem; d.plan_bytes = plan_bytes;
    return fastgl_block_plan_create_many(1, &d, stream, out);
}

fastgl_status fastgl_block_plan_export(const fastgl_plan *p, fastgl_plan_view *v)
{
    if (!p || !v) {
        set_error("plan or view is NULL");
        return FASTGL_ERR_INVALID_ARG;
    }
    const bool f = p->parts & FASTGL_PLAN_FWD, b = p->parts & FASTGL_PLAN_BWD;
    const bool sd = b || (p->parts & FASTGL_PLAN_SRC_DEG);
    v->din = f ? p->din : nullptr;
    v->dst_inv = f ? p->dst_inv : nullptr;
    v->dst_rsqrt = f ? p->dst_rsqrt : nullptr;
    v->long_dst = f ? p->long_dst : nullptr;
    v->chunk_ptr_dst = f ? p->chunk_ptr_dst : nullptr;
    v->split_dst = f ? p->split_dst : nullptr;
    v->split_src = b ? p->split_src : nullptr;
    v->dout = sd ? p->dout : nullptr;
    v->indptr_T = b ? p->indptr_T : nullptr;
    v->indices_T = b ? p->indices_T : nullptr;
    v->perm = (b && (p->parts & FASTGL_PLAN_PERM)) ? p->perm : nullptr;
    v->src_rsqrt = sd ? p->src_rsqrt : nullptr;
    v->long_src = b ? p->long_src : nullptr;
    v->chunk_ptr_src = b ? p->chunk_ptr_src : nullptr;
    v->counters = p->counters;
    return FASTGL_OK;
}

void fastgl_block_plan_destroy(fastgl_plan *p) { delete p; }

size_t fastgl_block_workspace_bytes(int64_t num_dst, int64_t num_src, int64_t num_edges, int64_t feat,
                                    fastgl_dtype dtype)
{
    if (num_dst < 0 || num_src < 0 || num_edges < 0 || feat <= 0) return 0;
    return partial_bytes(num_edges, feat, dtype) + plan_layout(nullptr, nullptr, num_dst, num_src, num_edges);
}

int32_t fastgl_long_row_threshold(void) { return kLongThreshold; }
int32_t fastgl_long_row_chunk(void) { return kLongChunk; }
int32_t fastgl_work_per_group(void) { return kWorkPerGroup; }

fastgl_status fastgl_gather_rows(const void *table, int64_t table_rows, const int64_t *ids, int64_t n,
                                 int64_t feat, fastgl_dtype dtype, void *out, void *stream)
{
    if (n < 0 || feat <= 0 || table_rows < 0) {
        set_error("bad size (n=%lld feat=%lld table_rows=%lld)", (long long)n, (long long)feat,
                  (long long)table_rows);
        return FASTGL_ERR_INVALID_ARG;
    }
    if ((int)dtype < 0 || (int)dtype > 1) {
        set_error("unknown dtype %d", (int)dtype);
        return FASTGL_ERR_INVALID_ARG;
    }
    if (n > 0 && (!table || !ids || !out || table_rows == 0)) {
        set_error("NULL pointer or empty table");
        return FASTGL_ERR_INVALID_ARG;
    }
    const uintptr_t emask = dtype == FASTGL_F32 ? 3 : 1;
    if ((((uintptr_t)table | (uintptr_t)out) & emask) || ((uintptr_t)ids & 7)) {
        set_error("misaligned buffer");
        return FASTGL_ERR_INVALID_ARG;
    }
    if (feat > (int64_t)1 << 24 || n * feat >= (int64_t)1 << 40) {
        set_error("gather too large");
        return FASTGL_ERR_UNSUPPORTED;
    }
    return launch_gather_rows(table, ids, n, feat, dtype, out, (hipStream_t)stream);
}

fastgl_status fastgl_block_validate(const int32_t *indptr, const int32_t *indices, int64_t num_dst,
                                    int64_t num_src, int64_t num_edges, void *scratch, int64_t *n_violations,
                                    void *stream)
{
    fastgl_status st = check_block(indptr, indices, num_dst, num_src, num_edges);
    if (st != FASTGL_OK) return st;
    if (!scratch || !n_violations || ((uintptr_t)scratch & 7)) {
        set_error("scratch (device, 8 bytes, aligned) and n_violations (host) are required");
        return FASTGL_ERR_INVALID_ARG;
    }
    return validate_block(indptr, indices, num_dst, num_src, num_edges, scratch, n_violations,
                          (hipStream_t)stream);
}

const char *fastgl_last_error(void) { return g_err; }

}  // extern "C"
