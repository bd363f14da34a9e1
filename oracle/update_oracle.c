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
 * All matrices are row-major fp32.  Every output element is one fp64 sum taken
 * in index order and rounded to fp32 once.  Written as the definition: three
 * nested loops per product, no blocking.
 *
 * Pins (tests/test_oracle_pins.py): a hand-worked 2x3x2 example, numpy's fp64
 * matmul on non-square asymmetric operands, the identity / zero-weight special
 * cases, the adjoint identity <dY, J v> = <J^T dY, v>, and central finite
 * differences of a scalar loss through the ReLU.  Nothing here is "parity
 * unpinned".
 */
#include <stddef.h>
#include <stdint.h>

int fastgl_oracle_update_fwd(const float *H, const float *W, const float *b,
                             int64_t M, int64_t K, int64_t N, int relu, float *Y)
{
    if (M < 0 || K < 0 || N < 0) return 1;
    for (int64_t i = 0; i < M; ++i) {
        for (int64_t j = 0; j < N; ++j) {
            double z = 0.0;
            for (int64_t k = 0; k < K; ++k)
                z += (double)H[i * K + k] * (double)W[k * N + j];
            if (b) z += (double)b[j];
            if (relu && !(z > 0.0)) z = 0.0;
            Y[i * N + j] = (float)z;
        }
    }
    return 0;
}

/* Y is the forward OUTPUT (post-activation); it is read only when relu != 0.
 * Any of dH, dW, db may be NULL to skip that result. */
int fastgl_oracle_update_bwd(const float *H, const float *W, const float *Y, const float *dY,
                             int64_t M, int64_t K, int64_t N, int relu,
                             float *dH, float *dW, float *db)
{
    if (M < 0 || K < 0 || N < 0) return 1;
    if (dH) {
        for (int64_t i = 0; i < M; ++i)
            for (int64_t k = 0; k < K; ++k) {
                double s = 0.0;
                for (int64_t j = 0; j < N; ++j) {
                    if (relu && !(Y[i * N + j] > 0.0f)) continue;
                    s += (double)dY[i * N + j] * (double)W[k * N + j];
                }
                dH[i * K + k] = (float)s;
            }
    }
    if (dW) {
        for (int64_t k = 0; k < K; ++k)
            for (int64_t j = 0; j < N; ++j) {
                double s = 0.0;
                for (int64_t i = 0; i < M; ++i) {
                    if (relu && !(Y[i * N + j] > 0.0f)) continue;
                    s += (double)H[i * K + k] * (double)dY[i * N + j];
                }
                dW[k * N + j] = (float)s;
            }
    }
    if (db) {
        for (int64_t j = 0; j < N; ++j) {
            double s = 0.0;
            for (int64_t i = 0; i < M; ++i) {
                if (relu && !(Y[i * N + j] > 0.0f)) continue;
                s += (double)dY[i * N + j];
            }
            db[j] = (float)s;
        }
    }
    return 0;
}
