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
 * and, for the score itself, what the GAT model defines (the paper evaluates
 * GAT without printing its formula):
 *   score_e     = LeakyReLU(el_u + er_v)            (el_u, er_v: projections of
 *                 the transformed features of target and neighbour on the two
 *                 halves of the head's attention vector)
 *   del_u       = sum over row u of g_e,  der_v = sum over the edges with
 *                 neighbour v of g_e,  g_e = dscore_e * (1 or the slope)
 * Several heads are several calls on head-major arrays ([head][node][...],
 * [head][edge]): every array of one head is then contiguous.
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

/* score[e] = LeakyReLU(el[u] + er[indices[e]]) for every edge e of every row u;
 * LeakyReLU(x) = x for x > 0 and slope * x otherwise (slope finite; 0.2 in the
 * GAT model).  el fp32 [num_dst], er fp32 [num_src], score fp32 [num_edges].
 * The sum is formed exactly (fp64) and the result rounded once. */
fastgl_status fastgl_edge_score_fwd(const int32_t *indptr, const int32_t *indices, int64_t num_dst,
                                    int64_t num_src, int64_t num_edges, const float *el, const float *er,
                                    float slope, float *score, void *stream);

/* grad_el[u] = sum over row u of g_e and grad_er[v] = sum over the edges with
 * indices[e] == v of g_e, g_e = grad_score[e] * (el[u] + er[v] > 0 ? 1 : slope);
 * fp64 sums, one rounding, every entry written (0 for nodes without edges).
 * Either result may be NULL.  grad_er walks the transposed block and needs a
 * plan of this block built with FASTGL_PLAN_BWD | FASTGL_PLAN_PERM; grad_el
 * alone takes plan = NULL. */
fastgl_status fastgl_edge_score_bwd(const int32_t *indptr, const int32_t *indices, int64_t num_dst,
                                    int64_t num_src, int64_t num_edges, const float *el, const float *er,
                                    float slope, const float *grad_score, const fastgl_plan *plan,
                                    float *grad_el, float *grad_er, void *stream);

/* Rows with more edges than this are handed to whole workgroups by the softmax calls. */
int32_t fastgl_edge_softmax_long_row(void);

#ifdef __cplusplus
}
#endif
#endif /* FASTGL_EDGE_H */
