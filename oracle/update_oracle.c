/*
 * CPU oracle for the update phase of a sampled GCN layer.  TEST
 * INFRASTRUCTURE ONLY: nothing in the product path may call this; tests, the
 * smoke check and the benchmark's cpu_baseline leg do.  It shares no code with
 * the GPU library.
 *
 * What it computes (paper, Section 2.1, Eq. 2): the aggregated features h_u of
 * every target node are transformed into the layer's output x_u^{k+1} =
 * Update(h_u).  The paper leaves Update abstract; for the GCN it evaluates
 * (Section 6.1) this is the dense transform of Kipf & Welling's layer, read
 * here as
 *
 *   forward   Y = act(H W + b)          H [M,K], W [K,N], b [N] or absent,
 *                                       act = identity or ReLU
 *   backward  dZ = dY (.) act'(.)       act' = 1 where Y > 0, else 0 (ReLU);
 *                                       all ones for the identity
 *             dH = dZ W^T   [M,K]
 *             dW = H^T dZ   [K,N]
 *             db = column sums of dZ  [N]
 *
 * All matrices are row-major, fp32 or bf16 (see below).  Every output element is
 * one fp64 sum taken in index order and rounded to its storage type once.  Written as the definition: three
 * nested loops per product, no blocking.
 *
 * Pins (tests/test_update_oracle_pins.py): a hand-worked 2x3x2 example, numpy's fp64
 * matmul on non-square asymmetric operands, the identity / zero-weight special
 * cases, the adjoint identity <dY, J v> = <J^T dY, v>, and central finite
 * differences of a scalar loss through the ReLU.  Nothing here is "parity
 * unpinned".
 */
#include <stddef.h>
#include <stdint.h>
#include <string.h>

/* Storage types: 0 = fp32, 1 = bf16 (bit patterns in uint16).  With bf16 storage H, W, Y, dY and dH
 * are bf16 while the bias and the weight gradients dW, db stay fp32 (what an optimizer keeps in
 * full precision); every output element is still one fp64 sum rounded once to its storage type. */
uint16_t fastgl_oracle_double_to_bf16(double x);      /* one-step round to nearest even (aggregation oracle) */

static double ld(const void *p, int dtype, int64_t i)
{
    if (dtype == 0) return (double)((const float *)p)[i];
    uint32_t u = (uint32_t)((const uint16_t *)p)[i] << 16;
    float f;
    memcpy(&f, &u, 4);
    return (double)f;
}

static void st(void *p, int dtype, int64_t i, double v)
{
    if (dtype == 0) ((float *)p)[i] = (float)v;
    else ((uint16_t *)p)[i] = fastgl_oracle_double_to_bf16(v);
}

int fastgl_oracle_update_fwd_dt(const void *H, const void *W, const float *b, int64_t M, int64_t K, int64_t N,
                                int relu, int dtype, void *Y)
{
    if (M < 0 || K < 0 || N < 0 || dtype < 0 || dtype > 1) return 1;
    for (int64_t i = 0; i < M; ++i) {
        for (int64_t j = 0; j < N; ++j) {
            double z = 0.0;
            for (int64_t k = 0; k < K; ++k) z += ld(H, dtype, i * K + k) * ld(W, dtype, k * N + j);
            if (b) z += (double)b[j];
            if (relu && !(z > 0.0)) z = 0.0;
            st(Y, dtype, i * N + j, z);
        }
    }
    return 0;
}

/* Y is the forward OUTPUT (post-activation); it is read only when relu != 0.
 * Any of dH, dW, db may be NULL to skip that result. */
int fastgl_oracle_update_bwd_dt(const void *H, const void *W, const void *Y, const void *dY, int64_t M,
                                int64_t K, int64_t N, int relu, int dtype, void *dH, float *dW, float *db)
{
    if (M < 0 || K < 0 || N < 0 || dtype < 0 || dtype > 1) return 1;
    if (dH) {
        for (int64_t i = 0; i < M; ++i)
            for (int64_t k = 0; k < K; ++k) {
                double s = 0.0;
                for (int64_t j = 0; j < N; ++j) {
                    if (relu && !(ld(Y, dtype, i * N + j) > 0.0)) continue;
                    s += ld(dY, dtype, i * N + j) * ld(W, dtype, k * N + j);
                }
                st(dH, dtype, i * K + k, s);
            }
    }
    if (dW) {
        for (int64_t k = 0; k < K; ++k)
            for (int64_t j = 0; j < N; ++j) {
                double s = 0.0;
                for (int64_t i = 0; i < M; ++i) {
                    if (relu && !(ld(Y, dtype, i * N + j) > 0.0)) continue;
                    s += ld(H, dtype, i * K + k) * ld(dY, dtype, i * N + j);
                }
                dW[k * N + j] = (float)s;
            }
    }
    if (db) {
        for (int64_t j = 0; j < N; ++j) {
            double s = 0.0;
            for (int64_t i = 0; i < M; ++i) {
                if (relu && !(ld(Y, dtype, i * N + j) > 0.0)) continue;
                s += ld(dY, dtype, i * N + j);
            }
            db[j] = (float)s;
        }
    }
    return 0;
}

int fastgl_oracle_update_fwd(const float *H, const float *W, const float *b,
                             int64_t M, int64_t K, int64_t N, int relu, float *Y)
{
    return fastgl_oracle_update_fwd_dt(H, W, b, M, K, N, relu, 0, Y);
}

int fastgl_oracle_update_bwd(const float *H, const float *W, const float *Y, const float *dY,
                             int64_t M, int64_t K, int64_t N, int relu,
                             float *dH, float *dW, float *db)
{
    return fastgl_oracle_update_bwd_dt(H, W, Y, dY, M, K, N, relu, 0, dH, dW, db);
}
