/*
 * fastgl_edge.h - C ABI for learned edge weights on MI355X (gfx950): the
 * gradient of the aggregation with respect to its edge weights, and the
 * softmax over a target node's incoming edges.
 *
 * Paper Section 2.1, Eq. 1: h_u = sum over v in N(u) of w_uv x_v.  GCN fixes
 * w_uv from the degrees; an attention layer (GAT, one of the three models of
 * the paper's evaluation, Section 6.1) learns it: w_uv = softmax over the
 * incoming edges of u of a per-edge score.  Training such a layer needs, next
 * to fastgl_block_aggregate_fwd / _bwd with edge_w:
 *   dL/dw_e     = c_u * s_v * <G[u,:], X[v,:]>      (G = dL/dh; c_u, s_v the
 *                 scale factors of the aggregation mode, 1 for SUM)
 *   alpha_e     = exp(score_e - m_u) / sum_row exp(score - m_u)
 *   dscore_e    = alpha_e * (dalpha_e - sum_row alpha * dalpha)
 * Blocks are the CSR-by-destination blocks of fastgl_agg.h (indptr int32
 * [num_dst+1], indices int32 [E]); per-edge arrays are fp32 [E] in edge order.
 * Conventions are those of fastgl_agg.h: caller-owned DEVICE memory, caller
 * workspace (256-byte aligned), work enqueued on `stream` (hipStream_t as
 * void*) without synchronising the host, return codes + fastgl_last_error().
 * Rows without edges produce nothing.  Results do not depend on scheduling.
 */
#ifndef FASTGL_EDGE_H
#define FASTGL_EDGE_H

#include "fastgl_agg.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Bytes of workspace for fastgl_edge_weight_grad and the two softmax calls. */
size_t fastgl_edge_workspace_bytes(int64_t num_dst, int64_t num_edges);

/* grad_w[e] = c_u * s_v * <grad_out[u,:], X[v,:]>, u = destination of edge e,
 * v = indices[e].  X [num_src, feat] and grad_out [num_dst, feat] of `dtype`
 * (f32: products summed in fp64; bf16: in fp32); grad_w fp32.  FASTGL_AGG_GCN
 * needs a plan of this block that holds the source degrees
 * (FASTGL_PLAN_SRC_DEG or FASTGL_PLAN_BWD); SUM and MEAN take plan = NULL. */
fastgl_status fastgl_edge_weight_grad(const int32_t *indptr, const int32_t *indices, int64_t num_dst,
                                      int64_t num_src, int64_t num_edges, int64_t feat, fastgl_agg_mode mode,
                                      fastgl_dtype dtype, const void *X, const void *grad_out,
                                      const fastgl_plan *plan, float *grad_w, void *workspace,
                                      size_t workspace_bytes, void *stream);

/* alpha = softmax of score over every destination's incoming edges. */
fastgl_status fastgl_edge_softmax_fwd(const int32_t *indptr, int64_t num_dst, int64_t num_edges,
                                      const float *score, float *alpha, void *workspace, size_t workspace_bytes,
                                      void *stream);

/* grad_score from alpha (the forward result) and grad_alpha. */
fastgl_status fastgl_edge_softmax_bwd(const int32_t *indptr, int64_t num_dst, int64_t num_edges,
                                      const float *alpha, const float *grad_alpha, float *grad_score,
                                      void *workspace, size_t workspace_bytes, void *stream);

/* Rows with more edges than this are handed to whole workgroups by the softmax calls. */
int32_t fastgl_edge_softmax_long_row(void);

#ifdef __cplusplus
}
#endif
#endif /* FASTGL_EDGE_H */
