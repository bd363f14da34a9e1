/*
 * CPU oracle for block aggregation.  TEST INFRASTRUCTURE ONLY: nothing in the
 * product path may call this; tests, the smoke check and the benchmark's
 * cpu_baseline leg do.  It shares no code with the GPU library.
 *
 * What it computes (paper, Section 2.1, Eq. 1; Section 4.2 "Memory-Aware
 * Computation", Eq. 5):
 *
 *   forward   h_u = sum_{v in N(u)} w_uv * x_v            (Eq. 1)
 *   backward  dL/dx_v = sum_{u : v in N(u)} w_uv * dL/dh_u
 *             (Eq. 5 read as the chain rule of Eq. 1, i.e. the transpose of
 *              the forward operator applied to the upstream gradient)
 *
 * A block is a CSR by destination row u: the neighbours N(u) of u are
 * indices[indptr[u] .. indptr[u+1]).  The weight w_uv of edge e=(u,v) is
 *
 *   SUM : w_e                      (w_e = edge_w[e], or 1 when edge_w is NULL)
 *   MEAN: w_e / max(din[u],1)
 *   GCN : w_e / sqrt(max(din[u],1) * max(dout[v],1))
 *
 * with din[u] = row length and dout[v] = number of edges whose source is v,
 * both counted inside the block.  Rows without edges give zero rows; every
 * output row is written.
 *
 * The definitional functions below are single-threaded loops in the paper's
 * order (for each target node, for each neighbour) with fp64 accumulation and
 * ONE rounding to the storage type at the end.  The "par" variants (fp32
 * accumulation, OpenMP over rows, backward through this file's own stable
 * transpose) exist to be timed as the host baseline and are cross-checked
 * against the definitional ones by the tests.
 *
 * Pins (tests/test_oracle_pins.py): dense A*X and A^T*G in numpy fp64,
 * all-ones -> degree counts, constant preservation under MEAN, the GCN
 * sqrt-degree closed form, finite differences, the adjoint identity,
 * brute-force Python loops, transpose/bucket structural invariants.
 * Nothing here is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { MODE_SUM = 0, MODE_MEAN = 1, MODE_GCN = 2 };
enum { DT_F32 = 0, DT_BF16 = 1 };

/* ---- bf16 <-> double ---------------------------------------------------- */
static double bf16_to_double(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, 4);
    return (double)f;
}

/* Round a double to the nearest bfloat16 (ties to even) in one step.
 * bf16 has 8 significand bits (7 stored); work on the fp64 bit pattern so no
 * intermediate fp32 rounding happens. */
static uint16_t double_to_bf16(double x)
{
    if (isnan(x)) return 0x7FC0;
    uint16_t sign = signbit(x) ? 0x8000 : 0;
    double a = fabs(x);
    if (a == 0.0) return sign;
    if (isinf(a)) return sign | 0x7F80;
    int e;
    double m = frexp(a, &e);           /* a = m * 2^e, m in [0.5,1) */
    int E = e - 1;                     /* a = (2m) * 2^E, 2m in [1,2) */
    if (E < -126) {                    /* subnormal bf16: quantum 2^-133 */
        double q = ldexp(a, 133);
        double r = nearbyint(q);       /* default rounding mode: ties to even */
        uint32_t bits = (uint32_t)r;   /* may reach 0x80 = smallest normal */
        return sign | (uint16_t)bits;
    }
    double q = ldexp(m, 8);            /* in [128,256): 8 significant bits */
    double r = nearbyint(q);
    if (r >= 256.0) { r = 128.0; E += 1; }
    if (E > 127) return sign | 0x7F80;
    uint32_t frac = (uint32_t)r - 128u;
    return sign | (uint16_t)(((uint32_t)(E + 127) << 7) | frac);
}

static double load_elem(const void *p, int dtype, int64_t i)
{
    if (dtype == DT_F32) return (double)((const float *)p)[i];
    return bf16_to_double(((const uint16_t *)p)[i]);
}

static void store_elem(void *p, int dtype, int64_t i, double v)
{
    if (dtype == DT_F32) ((float *)p)[i] = (float)v;
    else ((uint16_t *)p)[i] = double_to_bf16(v);
}

/* exported for the rounding pins */
uint16_t fastgl_oracle_double_to_bf16(double x) { return double_to_bf16(x); }

/* ---- bookkeeping ---------------------------------------------------------- */
int fastgl_oracle_degrees(const int32_t *indptr, const int32_t *indices,
                          int64_t num_dst, int64_t num_src, int64_t num_edges,
                          int32_t *din, int32_t *dout)
{
    for (int64_t u = 0; u < num_dst; ++u) din[u] = indptr[u + 1] - indptr[u];
    for (int64_t v = 0; v < num_src; ++v) dout[v] = 0;
    for (int64_t e = 0; e < num_edges; ++e) {
        int32_t v = indices[e];
        if (v < 0 || v >= num_src) return 1;
        dout[v] += 1;
    }
    return 0;
}

/* Stable transpose: edges sorted by source id, ties keep ascending edge id.
 * indptr_T[num_src+1], indices_T[E] = destination of the k-th sorted edge,
 * perm[E] = original edge id of the k-th sorted edge. */
int fastgl_oracle_transpose(const int32_t *indptr, const int32_t *indices,
                            int64_t num_dst, int64_t num_src, int64_t num_edges,
                            int32_t *indptr_T, int32_t *indices_T, int32_t *perm)
{
    int32_t *cursor = (int32_t *)calloc((size_t)num_src + 1, sizeof(int32_t));
    if (!cursor) return 2;
    for (int64_t v = 0; v <= num_src; ++v) indptr_T[v] = 0;
    for (int64_t e = 0; e < num_edges; ++e) indptr_T[indices[e] + 1] += 1;
    for (int64_t v = 0; v < num_src; ++v) indptr_T[v + 1] += indptr_T[v];
    for (int64_t v = 0; v < num_src; ++v) cursor[v] = indptr_T[v];
    for (int64_t u = 0; u < num_dst; ++u)
        for (int32_t e = indptr[u]; e < indptr[u + 1]; ++e) {
            int32_t k = cursor[indices[e]]++;
            indices_T[k] = (int32_t)u;
            perm[k] = e;
        }
    free(cursor);
    return 0;
}

/* Degree buckets: rows whose length exceeds `threshold` are "long"; they are
 * listed in ascending row order, and long row i owns the partial-sum chunks
 * chunk_ptr[i] .. chunk_ptr[i+1), one chunk per `chunk` edges (last one short).
 * Returns the number of long rows. */
int64_t fastgl_oracle_long_rows(const int32_t *indptr, int64_t num_rows,
                                int32_t threshold, int32_t chunk,
                                int32_t *long_rows, int32_t *chunk_ptr)
{
    int64_t n = 0;
    int32_t c = 0;
    for (int64_t r = 0; r < num_rows; ++r) {
        int32_t len = indptr[r + 1] - indptr[r];
        if (len > threshold) {
            long_rows[n] = (int32_t)r;
            chunk_ptr[n] = c;
            c += (len + chunk - 1) / chunk;
            ++n;
        }
    }
    chunk_ptr[n] = c;
    return n;
}

/* Equal-work row sets: set g starts at the first row r with rowptr[r] + r >= g*work
 * (a row's work = its edges + 1).  split has ngroups+1 entries, ngroups =
 * ceil((num_rows + nnz) / work).  Returns ngroups. */
int64_t fastgl_oracle_work_split(const int32_t *rowptr, int64_t num_rows, int32_t work, int32_t *split)
{
    int64_t total = (int64_t)rowptr[num_rows] + num_rows;
    int64_t ngroups = (total + work - 1) / work;
    int64_t r = 0;
    for (int64_t g = 0; g <= ngroups; ++g) {
        while (r < num_rows && (int64_t)rowptr[r] + r < g * (int64_t)work) ++r;
        split[g] = (int32_t)r;
    }
    return ngroups;
}

/* ---- definitional aggregation (fp64, single thread) ------------------------ */
static double dst_scale(int mode, int32_t din)
{
    double d = din < 1 ? 1.0 : (double)din;
    if (mode == MODE_MEAN) return 1.0 / d;
    if (mode == MODE_GCN) return 1.0 / sqrt(d);
    return 1.0;
}

static double src_scale(int mode, int32_t dout)
{
    double d = dout < 1 ? 1.0 : (double)dout;
    if (mode == MODE_GCN) return 1.0 / sqrt(d);
    return 1.0;
}

int fastgl_oracle_aggregate_fwd(const int32_t *indptr, const int32_t *indices,
                                const float *edge_w, int64_t num_dst, int64_t num_src,
                                int64_t num_edges, int64_t feat, int mode, int dtype,
                                const void *X, void *out)
{
    if (mode < 0 || mode > 2 || dtype < 0 || dtype > 1) return 1;
    int32_t *dout = (int32_t *)calloc((size_t)num_src + 1, sizeof(int32_t));
    double *acc = (double *)malloc(sizeof(double) * (size_t)(feat > 0 ? feat : 1));
    if (!dout || !acc) { free(dout); free(acc); return 2; }
    for (int64_t e = 0; e < num_edges; ++e) dout[indices[e]] += 1;
    for (int64_t u = 0; u < num_dst; ++u) {
        for (int64_t j = 0; j < feat; ++j) acc[j] = 0.0;
        for (int32_t e = indptr[u]; e < indptr[u + 1]; ++e) {
            int32_t v = indices[e];
            double a = (edge_w ? (double)edge_w[e] : 1.0) * src_scale(mode, dout[v]);
            for (int64_t j = 0; j < feat; ++j)
                acc[j] += a * load_elem(X, dtype, (int64_t)v * feat + j);
        }
        double c = dst_scale(mode, indptr[u + 1] - indptr[u]);
        for (int64_t j = 0; j < feat; ++j)
            store_elem(out, dtype, u * feat + j, c * acc[j]);
    }
    free(dout);
    free(acc);
    return 0;
}

int fastgl_oracle_aggregate_bwd(const int32_t *indptr, const int32_t *indices,
                                const float *edge_w, int64_t num_dst, int64_t num_src,
                                int64_t num_edges, int64_t feat, int mode, int dtype,
                                const void *G, void *dX)
{
    if (mode < 0 || mode > 2 || dtype < 0 || dtype > 1) return 1;
    int32_t *dout = (int32_t *)calloc((size_t)num_src + 1, sizeof(int32_t));
    double *acc = (double *)calloc((size_t)(num_src * feat) + 1, sizeof(double));
    if (!dout || !acc) { free(dout); free(acc); return 2; }
    for (int64_t e = 0; e < num_edges; ++e) dout[indices[e]] += 1;
    for (int64_t u = 0; u < num_dst; ++u) {
        double c = dst_scale(mode, indptr[u + 1] - indptr[u]);
        for (int32_t e = indptr[u]; e < indptr[u + 1]; ++e) {
            int32_t v = indices[e];
            double a = (edge_w ? (double)edge_w[e] : 1.0) * src_scale(mode, dout[v]);
            double *row = acc + (int64_t)v * feat;
            for (int64_t j = 0; j < feat; ++j)
                row[j] += a * c * load_elem(G, dtype, u * feat + j);
        }
    }
    for (int64_t i = 0; i < num_src * feat; ++i) store_elem(dX, dtype, i, acc[i]);
    free(dout);
    free(acc);
    return 0;
}

/* Row gather from a device-resident feature table (the tail of the paper's
 * memory-IO phase, Section 2.2: the features of the sampled nodes are what the
 * computation reads): out[i,:] = table[ids[i],:].  Pure copy. */
int fastgl_oracle_gather_rows(const void *table, const int64_t *ids, int64_t n,
                              int64_t feat, int dtype, void *out)
{
    size_t s = dtype == DT_F32 ? 4 : 2;
    for (int64_t i = 0; i < n; ++i)
        memcpy((char *)out + (size_t)i * feat * s,
               (const char *)table + (size_t)ids[i] * feat * s, (size_t)feat * s);
    return 0;
}

/* ---- timed host baseline: rows in parallel, fp32 accumulation -------------- */
int fastgl_oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

static void par_pull(const int32_t *rowptr, const int32_t *col, const int32_t *eid,
                     const float *edge_w, const float *col_scale, int row_mode,
                     int64_t num_rows, int64_t feat, int dtype, const void *In, void *Out)
{
#pragma omp parallel
    {
        float *acc = (float *)malloc(sizeof(float) * (size_t)(feat > 0 ? feat : 1));
#pragma omp for schedule(dynamic, 64)
        for (int64_t r = 0; r < num_rows; ++r) {
            for (int64_t j = 0; j < feat; ++j) acc[j] = 0.f;
            for (int32_t k = rowptr[r]; k < rowptr[r + 1]; ++k) {
                int32_t c = col[k];
                float a = edge_w ? edge_w[eid ? eid[k] : k] : 1.f;
                if (col_scale) a *= col_scale[c];
                if (dtype == DT_F32) {
                    const float *x = (const float *)In + (int64_t)c * feat;
                    for (int64_t j = 0; j < feat; ++j) acc[j] += a * x[j];
                } else {
                    const uint16_t *x = (const uint16_t *)In + (int64_t)c * feat;
                    for (int64_t j = 0; j < feat; ++j) {
                        uint32_t b = (uint32_t)x[j] << 16;
                        float f;
                        memcpy(&f, &b, 4);
                        acc[j] += a * f;
                    }
                }
            }
            int32_t len = rowptr[r + 1] - rowptr[r];
            float d = len < 1 ? 1.f : (float)len;
            float s = row_mode == 1 ? 1.f / d : row_mode == 2 ? 1.f / sqrtf(d) : 1.f;
            for (int64_t j = 0; j < feat; ++j) store_elem(Out, dtype, r * feat + j, (double)(s * acc[j]));
        }
        free(acc);
    }
}

int fastgl_oracle_par_aggregate_fwd(const int32_t *indptr, const int32_t *indices,
                                    const float *edge_w, int64_t num_dst, int64_t num_src,
                                    int64_t num_edges, int64_t feat, int mode, int dtype,
                                    const void *X, void *out)
{
    float *cs = NULL;
    if (mode == MODE_GCN) {
        int32_t *dout = (int32_t *)calloc((size_t)num_src + 1, sizeof(int32_t));
        cs = (float *)malloc(sizeof(float) * ((size_t)num_src + 1));
        if (!dout || !cs) { free(dout); free(cs); return 2; }
        for (int64_t e = 0; e < num_edges; ++e) dout[indices[e]] += 1;
        for (int64_t v = 0; v < num_src; ++v) cs[v] = 1.f / sqrtf(dout[v] < 1 ? 1.f : (float)dout[v]);
        free(dout);
    }
    par_pull(indptr, indices, NULL, edge_w, cs, mode == MODE_MEAN ? 1 : mode == MODE_GCN ? 2 : 0,
             num_dst, feat, dtype, X, out);
    free(cs);
    return 0;
}

int fastgl_oracle_par_aggregate_bwd(const int32_t *indptr, const int32_t *indices,
                                    const float *edge_w, int64_t num_dst, int64_t num_src,
                                    int64_t num_edges, int64_t feat, int mode, int dtype,
                                    const void *G, void *dX)
{
    int32_t *pT = (int32_t *)malloc(sizeof(int32_t) * ((size_t)num_src + 1));
    int32_t *iT = (int32_t *)malloc(sizeof(int32_t) * ((size_t)num_edges + 1));
    int32_t *pm = (int32_t *)malloc(sizeof(int32_t) * ((size_t)num_edges + 1));
    float *cs = NULL;
    if (!pT || !iT || !pm) { free(pT); free(iT); free(pm); return 2; }
    fastgl_oracle_transpose(indptr, indices, num_dst, num_src, num_edges, pT, iT, pm);
    if (mode != MODE_SUM) {
        cs = (float *)malloc(sizeof(float) * ((size_t)num_dst + 1));
        for (int64_t u = 0; u < num_dst; ++u) {
            int32_t len = indptr[u + 1] - indptr[u];
            float d = len < 1 ? 1.f : (float)len;
            cs[u] = mode == MODE_MEAN ? 1.f / d : 1.f / sqrtf(d);
        }
    }
    par_pull(pT, iT, pm, edge_w, cs, mode == MODE_GCN ? 2 : 0, num_src, feat, dtype, G, dX);
    free(pT); free(iT); free(pm); free(cs);
    return 0;
}
