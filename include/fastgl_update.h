/*
 * fastgl_update.h - C ABI of the update phase of a sampled GCN layer on MI355X
 * (gfx950), the dense step that follows neighbour aggregation.
 *
 * Paper Section 2.1, Eq. 2: the aggregated features h_u of every target node
 * are transformed into the layer output x_u^{k+1} = Update(h_u).  For the GCN
 * of the evaluation (Section 6.1) Update is the dense transform
 *
 *   forward   Y = act(H W + b)            act = identity or ReLU
 *   backward  dZ = dY (.) [Y > 0]         (all of dY for the identity)
 *             dH = dZ W^T,  dW = H^T dZ,  db = column sums of dZ
 *
 * H [M,K], W [K,N], Y/dY [M,N], dH [M,K], dW [K,N], b/db [N]: dense row-major
 * fp32 with no padding between rows.  Products run on the bf16 matrix cores
 * (v_mfma_f32_32x32x16_bf16) with fp32 accumulation: every fp32 element is cut
 * into three bf16 pieces whose sum is the element exactly, and six of the nine
 * piece products are added up, which leaves a relative error of at most 2^-23
 * (2^-28 on average) in a product of two elements - the accuracy of an fp32
 * multiply-add chain, at several times its speed.  An input element that is
 * not finite, or larger in magnitude than the largest bf16 (3.39e38), turns
 * every result it enters into NaN.  dW and db are reduced over fixed slabs of
 * rows whose partial results are summed in fp64 in a fixed order, so results
 * do not depend on scheduling.
 *
 * Conventions are those of fastgl_agg.h: every array is DEVICE memory owned by
 * the caller, the library allocates nothing, work is enqueued on `stream`
 * (hipStream_t as void*, NULL = default stream) without synchronising the host,
 * outputs are overwritten in full and must not overlap inputs, and everything
 * checkable on the host is checked before any launch (fastgl_last_error() has
 * the text).  0 <= M < 2^31-1, 0 <= K, N < 2^24; M == 0 or N == 0 writes
 * nothing in the forward pass; K == 0 gives Y = act(b).
 */
#ifndef FASTGL_UPDATE_H
#define FASTGL_UPDATE_H

#include "fastgl_agg.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Eq. 2 forward: Y = act(H W + bias).  bias may be NULL (no bias term);
 * relu != 0 selects ReLU, 0 the identity. */
fastgl_status fastgl_update_fwd(const float *H, const float *W, const float *bias,
                                int64_t M, int64_t K, int64_t N, int relu,
                                float *Y, void *stream);

/* Bytes of device workspace fastgl_update_bwd needs for the slab partials of
 * dW and db (0 when neither is requested is not assumed: this is the bound for
 * the full call). */
size_t fastgl_update_bwd_workspace_bytes(int64_t M, int64_t K, int64_t N);

/* Eq. 2 backward.  Y is the forward OUTPUT and is read only when relu != 0
 * (it may be NULL otherwise).  Any of dH, dW, db may be NULL to skip that
 * result; dW and db need `workspace` (256-byte aligned, at least
 * fastgl_update_bwd_workspace_bytes(M,K,N) bytes), dH alone does not. */
fastgl_status fastgl_update_bwd(const float *H, const float *W, const float *Y, const float *dY,
                                int64_t M, int64_t K, int64_t N, int relu,
                                float *dH, float *dW, float *db,
                                void *workspace, size_t workspace_bytes, void *stream);

/* The same two passes with bf16 storage (bit patterns in uint16_t): H, W, Y, dY
 * and dH are bf16; the bias and the weight gradients dW, db stay fp32.
 * One bf16 piece per element and one exact product per pair, summed in fp32 as
 * in the calls above; Y and dH are rounded to bf16 (nearest even) at the store.  Arrays must be aligned
 * to their element size; everything else is as above. */
fastgl_status fastgl_update_fwd_bf16(const uint16_t *H, const uint16_t *W, const float *bias,
                                     int64_t M, int64_t K, int64_t N, int relu,
                                     uint16_t *Y, void *stream);
fastgl_status fastgl_update_bwd_bf16(const uint16_t *H, const uint16_t *W, const uint16_t *Y,
                                     const uint16_t *dY, int64_t M, int64_t K, int64_t N, int relu,
                                     uint16_t *dH, float *dW, float *db,
                                     void *workspace, size_t workspace_bytes, void *stream);

/* One layer in one call: aggregation (Eq. 1) followed by the update (Eq. 2),
 *   H = aggregate(X)        [num_dst, K]   exactly what fastgl_block_aggregate_fwd writes
 *   Y = act(H W + bias)     [num_dst, N]
 * The graph arguments, edge_w, mode, plan and workspace are those of
 * fastgl_block_aggregate_fwd with feat = K (workspace >= fastgl_block_workspace_bytes);
 * W, bias, relu and Y are those of fastgl_update_fwd; X, W, H, Y are fp32 or, with
 * dtype FASTGL_BF16, bf16 bit patterns (bias fp32 either way).
 * For a narrow layer - fastgl_layer_fwd_fuses(K, N, dtype) != 0: fp32, K a multiple of 4 and at
 * most 256, N at most 64, X and H 16-byte aligned; the class-score layer of a sampled GCN - both
 * steps run in ONE kernel and the aggregated rows do not travel through memory: each is rounded to
 * fp32 once, as the separate call would store it, and multiplied out of on-chip memory with fp32
 * multiply-adds in ascending k (a chain of K + 1 roundings per element of Y).  H may then be NULL
 * (inference); when given it is written as a by-product for the backward pass.  Every row is
 * walked by one wavefront whatever its length: meant for sampled layers, whose rows are short.
 * Any other shape runs the two kernels of the separate calls back to back and needs H. */
fastgl_status fastgl_layer_fwd(const int32_t *indptr, const int32_t *indices, const float *edge_w,
                               int64_t num_dst, int64_t num_src, int64_t num_edges, int64_t K,
                               fastgl_agg_mode mode, fastgl_dtype dtype, const void *X,
                               const void *W, const float *bias, int64_t N, int relu,
                               void *H, void *Y,
                               const fastgl_plan *plan, void *workspace, size_t workspace_bytes,
                               void *stream);
int fastgl_layer_fwd_fuses(int64_t K, int64_t N, fastgl_dtype dtype);

/* Rows of H per dW/db slab for this shape (the length of the longest fp32
 * accumulation chain of the backward pass): a function of M, K, N alone,
 * a multiple of 32 between 32 and 2048; 0 for negative sizes. */
int32_t fastgl_update_slab_rows(int64_t M, int64_t K, int64_t N);

#ifdef __cplusplus
}
#endif
#endif /* FASTGL_UPDATE_H */
