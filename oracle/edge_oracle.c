/*
 * CPU oracle for learned edge weights: the gradient of Eq. 1 with respect to
 * the weights, and the softmax over a target node's incoming edges that an
 * attention layer (GAT, one of the paper's three evaluated models, Section 6.1)
 * uses to produce them.  TEST INFRASTRUCTURE ONLY: nothing in the product path
 * may call this.  It shares no code with the GPU library.
 *
 * Paper Section 2.1, Eq. 1: h_u = sum over v in N(u) of w_uv x_v.  With the
 * block's aggregation mode the edge's full coefficient is c_u * s_v * w_e
 * (c_u, s_v as in the aggregation oracle: 1 for SUM; c_u = 1/max(din,1) for
 * MEAN; 1/sqrt of the clamped degrees for GCN), so by the chain rule
 *   dL/dw_e = c_u * s_v * <G[u,:], X[v,:]>          G = dL/dh
 * Edge softmax over the incoming edges of each target node u:
 *   alpha_e = exp(score_e - m_u) / sum over e' in row u of exp(score_e' - m_u),
 *   m_u = the row's largest score (the shift changes nothing mathematically)
 * and its backward pass
 *   dscore_e = alpha_e * (dalpha_e - sum over e' in row u of alpha_e' dalpha_e').
 * The per-edge score of a GAT head (the paper evaluates GAT but does not print
 * its formula; this is the definition of the model itself): with el_u, er_v the
 * projections of the transformed features of target and neighbour on the two
 * halves of the attention vector,
 *   score_e = LeakyReLU(el_u + er_v),  LeakyReLU(x) = x for x > 0, slope * x otherwise
 * and by the chain rule, with g_e = dscore_e * (1 if el_u + er_v > 0 else slope),
 *   del_u = sum over the incoming edges of u of g_e
 *   der_v = sum over the edges whose neighbour is v of g_e.
 * All sums in fp64 in edge order, one rounding to fp32.  Rows without edges
 * produce nothing.
 *
 * Pins (tests/test_edge_oracle_pins.py): finite differences of <h, G> through
 * the pinned aggregation oracle (the loss is linear in w, so a central
 * difference is exact up to rounding), the dense form G X^T read at the edges,
 * hand-worked softmax values, rows that sum to 1, shift invariance, the
 * softmax Jacobian written out densely, finite differences of the softmax;
 * for the scores: hand-worked values, slope 1 (the identity, whose gradients
 * are the degree-weighted sums), the dense form of el 1^T + 1 er^T read at the
 * edges, finite differences.
 */
#include <math.h>
#include <stdint.h>

static double bf16_bits_to_double(uint16_t b)
{
    union { uint32_t u; float f; } c;
    c.u = (uint32_t)b << 16;
    return (double)c.f;
}

static double elem(const void *p, int dtype, int64_t i)
{
    return dtype == 0 ? (double)((const float *)p)[i] : bf16_bits_to_double(((const uint16_t *)p)[i]);
}

static double clamp1_inv(int mode, int64_t deg)      /* the scale a node contributes under `mode` */
{
    const double d = deg < 1 ? 1.0 : (double)deg;
    return mode == 1 ? 1.0 / d : (mode == 2 ? 1.0 / sqrt(d) : 1.0);
}

/* mode: 0 SUM, 1 MEAN, 2 GCN.  dtype: 0 f32, 1 bf16 (bit patterns).  grad_w is fp32[E]. */
int fastgl_oracle_edge_weight_grad(const int32_t *indptr, const int32_t *indices, int64_t num_dst,
                                   int64_t num_src, int64_t feat, int mode, int dtype, const void *X,
                                   const void *G, int32_t *dout_scratch, float *grad_w)
{
    if (num_dst < 0 || num_src < 0 || feat < 0 || mode < 0 || mode > 2) return 1;
    const int64_t E = indptr[num_dst];
    for (int64_t v = 0; v < num_src; ++v) dout_scratch[v] = 0;
    for (int64_t e = 0; e < E; ++e) {
        if (indices[e] < 0 || indices[e] >= num_src) return 2;
        dout_scratch[indices[e]] += 1;
    }
    for (int64_t u = 0; u < num_dst; ++u) {
        const double c_u = clamp1_inv(mode, indptr[u + 1] - indptr[u]);
        for (int64_t e = indptr[u]; e < indptr[u + 1]; ++e) {
            const int64_t v = indices[e];
            const double s_v = mode == 2 ? clamp1_inv(2, dout_scratch[v]) : 1.0;   /* only GCN scales by the source */
            double dot = 0.0;
            for (int64_t j = 0; j < feat; ++j) dot += elem(G, dtype, u * feat + j) * elem(X, dtype, v * feat + j);
            grad_w[e] = (float)(c_u * s_v * dot);
        }
    }
    return 0;
}

int fastgl_oracle_edge_softmax_fwd(const int32_t *indptr, int64_t num_dst, const float *score, float *alpha)
{
    if (num_dst < 0) return 1;
    for (int64_t u = 0; u < num_dst; ++u) {
        const int64_t b = indptr[u], e = indptr[u + 1];
        if (b == e) continue;
        double m = (double)score[b];
        for (int64_t k = b + 1; k < e; ++k) if ((double)score[k] > m) m = (double)score[k];
        double z = 0.0;
        for (int64_t k = b; k < e; ++k) z += exp((double)score[k] - m);
        for (int64_t k = b; k < e; ++k) alpha[k] = (float)(exp((double)score[k] - m) / z);
    }
    return 0;
}

int fastgl_oracle_edge_softmax_bwd(const int32_t *indptr, int64_t num_dst, const float *alpha,
                                   const float *grad_alpha, float *grad_score)
{
    if (num_dst < 0) return 1;
    for (int64_t u = 0; u < num_dst; ++u) {
        double s = 0.0;
        for (int64_t k = indptr[u]; k < indptr[u + 1]; ++k) s += (double)alpha[k] * (double)grad_alpha[k];
        for (int64_t k = indptr[u]; k < indptr[u + 1]; ++k)
            grad_score[k] = (float)((double)alpha[k] * ((double)grad_alpha[k] - s));
    }
    return 0;
}

/* score[e] = LeakyReLU(el[u] + er[indices[e]]) for every edge e of row u. */
int fastgl_oracle_edge_score_fwd(const int32_t *indptr, const int32_t *indices, int64_t num_dst, int64_t num_src,
                                 const float *el, const float *er, double slope, float *score)
{
    if (num_dst < 0 || num_src < 0) return 1;
    for (int64_t u = 0; u < num_dst; ++u)
        for (int64_t e = indptr[u]; e < indptr[u + 1]; ++e) {
            const int64_t v = indices[e];
            if (v < 0 || v >= num_src) return 2;
            const double x = (double)el[u] + (double)er[v];
            score[e] = (float)(x > 0.0 ? x : slope * x);
        }
    return 0;
}

/* grad_el [num_dst], grad_er [num_src] from grad_score [E]; either may be NULL. */
int fastgl_oracle_edge_score_bwd(const int32_t *indptr, const int32_t *indices, int64_t num_dst, int64_t num_src,
                                 const float *el, const float *er, double slope, const float *grad_score,
                                 double *acc_src, float *grad_el, float *grad_er)
{
    if (num_dst < 0 || num_src < 0) return 1;
    for (int64_t v = 0; v < num_src; ++v) acc_src[v] = 0.0;
    for (int64_t u = 0; u < num_dst; ++u) {
        double acc = 0.0;
        for (int64_t e = indptr[u]; e < indptr[u + 1]; ++e) {
            const int64_t v = indices[e];
            if (v < 0 || v >= num_src) return 2;
            const double x = (double)el[u] + (double)er[v];
            const double g = (double)grad_score[e] * (x > 0.0 ? 1.0 : slope);
            acc += g;
            acc_src[v] += g;
        }
        if (grad_el) grad_el[u] = (float)acc;
    }
    if (grad_er)
        for (int64_t v = 0; v < num_src; ++v) grad_er[v] = (float)acc_src[v];
    return 0;
}
