/* Memory-safety driver for the CPU oracle.  TEST INFRASTRUCTURE ONLY.
 *
 * Built together with the oracle's sources under -fsanitize=address,undefined
 * (tests/test_sanitizers.py) and run on the CPU: it calls every entry point of
 * the aggregation, bookkeeping, update, ID-map, Match and edge-weight oracles on
 * small seeded blocks, degenerate sizes included (no rows, no edges, one row of
 * many edges), with every buffer allocated at exactly the size the entry point's
 * contract states, so that an access one element outside any of them stops the
 * run.  It checks no values - the pins in tests/ do that - only a few structural
 * facts that make sure the calls did real work.  Exit code 0 = clean. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int fastgl_oracle_degrees(const int32_t *, const int32_t *, int64_t, int64_t, int64_t, int32_t *, int32_t *);
int fastgl_oracle_transpose(const int32_t *, const int32_t *, int64_t, int64_t, int64_t, int32_t *, int32_t *, int32_t *);
int64_t fastgl_oracle_long_rows(const int32_t *, int64_t, int32_t, int32_t, int32_t *, int32_t *);
int64_t fastgl_oracle_work_split(const int32_t *, int64_t, int32_t, int32_t *);
int fastgl_oracle_aggregate_fwd(const int32_t *, const int32_t *, const float *, int64_t, int64_t, int64_t, int64_t, int, int, const void *, void *);
int fastgl_oracle_aggregate_bwd(const int32_t *, const int32_t *, const float *, int64_t, int64_t, int64_t, int64_t, int, int, const void *, void *);
int fastgl_oracle_par_aggregate_fwd(const int32_t *, const int32_t *, const float *, int64_t, int64_t, int64_t, int64_t, int, int, const void *, void *);
int fastgl_oracle_par_aggregate_bwd(const int32_t *, const int32_t *, const float *, int64_t, int64_t, int64_t, int64_t, int, int, const void *, void *);
int fastgl_oracle_gather_rows(const void *, const int64_t *, int64_t, int64_t, int, void *);
uint16_t fastgl_oracle_double_to_bf16(double);
int fastgl_oracle_update_fwd_dt(const void *, const void *, const float *, int64_t, int64_t, int64_t, int, int, void *);
int fastgl_oracle_update_bwd_dt(const void *, const void *, const void *, const void *, int64_t, int64_t, int64_t, int, int, void *, float *, float *);
int64_t fastgl_oracle_idmap(const int64_t *, int64_t, const int64_t *, int64_t, int32_t *, int64_t *);
int64_t fastgl_oracle_fused_map_seq(const int64_t *, int64_t, int64_t, int64_t *, int64_t *, int64_t *);
int64_t fastgl_oracle_match(const int64_t *, int64_t, const int64_t *, int64_t, int32_t *, int32_t *, int64_t *);
int64_t fastgl_oracle_overlap(const int64_t *, int64_t, const int64_t *, int64_t);
int fastgl_oracle_greedy_reorder(const int64_t *, const int64_t *, int64_t, int32_t *);
int fastgl_oracle_assemble(const void *, const void *, const int32_t *, int64_t, int64_t, int64_t, void *);
int fastgl_oracle_edge_weight_grad(const int32_t *, const int32_t *, int64_t, int64_t, int64_t, int, int, const void *, const void *, int32_t *, float *);
int fastgl_oracle_edge_softmax_fwd(const int32_t *, int64_t, const float *, float *);
int fastgl_oracle_edge_softmax_bwd(const int32_t *, int64_t, const float *, const float *, float *);
int fastgl_oracle_edge_score_fwd(const int32_t *, const int32_t *, int64_t, int64_t, const float *, const float *, double, float *);
int fastgl_oracle_edge_score_bwd(const int32_t *, const int32_t *, int64_t, int64_t, const float *, const float *, double, const float *, double *, float *, float *);

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static uint32_t rnd(void)
{
    rng_state = rng_state * 6364136223846793005ull + 1442695040888963407ull;
    return (uint32_t)(rng_state >> 33);
}
static float rndf(void) { return (float)((int)(rnd() % 2001) - 1000) / 500.0f; }

/* exactly n elements (a 1-byte allocation stands in for "nothing": no element of it may be read) */
static void *exact(size_t n, size_t elem)
{
    const size_t bytes = n * elem;
    void *p = malloc(bytes > 0 ? bytes : 1);
    if (!p) { fprintf(stderr, "out of memory\n"); exit(3); }
    return p;
}
static float *floats(size_t n)
{
    float *p = (float *)exact(n, 4);
    for (size_t i = 0; i < n; ++i) p[i] = rndf();
    return p;
}
static uint16_t *halves(size_t n)
{
    uint16_t *p = (uint16_t *)exact(n, 2);
    for (size_t i = 0; i < n; ++i) p[i] = fastgl_oracle_double_to_bf16((double)rndf());
    return p;
}
#define MUST(cond) do { if (!(cond)) { fprintf(stderr, "check failed at line %d: %s\n", __LINE__, #cond); exit(2); } } while (0)

static void one_block(int64_t nd, int64_t ns, int max_deg, int hub_deg, int64_t feat)
{
    int32_t *indptr = (int32_t *)exact((size_t)nd + 1, 4);
    indptr[0] = 0;
    for (int64_t u = 0; u < nd; ++u) {
        int d = ns > 0 ? (int)(rnd() % (uint32_t)(max_deg + 1)) : 0;
        if (u == nd / 2 && ns > 0) d = hub_deg;
        indptr[u + 1] = indptr[u] + d;
    }
    const int64_t E = indptr[nd];
    int32_t *indices = (int32_t *)exact((size_t)E, 4);
    for (int64_t e = 0; e < E; ++e) indices[e] = (int32_t)(rnd() % (uint32_t)ns);
    float *w = floats((size_t)E);

    int32_t *din = (int32_t *)exact((size_t)nd, 4), *dout = (int32_t *)exact((size_t)ns, 4);
    MUST(fastgl_oracle_degrees(indptr, indices, nd, ns, E, din, dout) == 0);
    int64_t s = 0;
    for (int64_t v = 0; v < ns; ++v) s += dout[v];
    MUST(s == E);
    int32_t *pT = (int32_t *)exact((size_t)ns + 1, 4), *iT = (int32_t *)exact((size_t)E, 4), *pm = (int32_t *)exact((size_t)E, 4);
    MUST(fastgl_oracle_transpose(indptr, indices, nd, ns, E, pT, iT, pm) == 0);
    MUST(pT[ns] == E);
    int32_t *lr = (int32_t *)exact((size_t)nd + 1, 4), *cp = (int32_t *)exact((size_t)nd + 2, 4);
    const int64_t nl = fastgl_oracle_long_rows(indptr, nd, 256, 128, lr, cp);
    MUST(nl >= 0 && nl <= nd);
    int32_t *split = (int32_t *)exact((size_t)((E + nd) / 16 + 3), 4);
    MUST(fastgl_oracle_work_split(indptr, nd, 16, split) >= 0);

    for (int dtype = 0; dtype < 2; ++dtype) {
        const size_t el = dtype == 0 ? 4 : 2;
        void *X = dtype == 0 ? (void *)floats((size_t)(ns * feat)) : (void *)halves((size_t)(ns * feat));
        void *G = dtype == 0 ? (void *)floats((size_t)(nd * feat)) : (void *)halves((size_t)(nd * feat));
        void *out = exact((size_t)(nd * feat), el), *dX = exact((size_t)(ns * feat), el);
        for (int mode = 0; mode < 3; ++mode)
            for (int weighted = 0; weighted < 2; ++weighted) {
                const float *ew = weighted ? w : NULL;
                MUST(fastgl_oracle_aggregate_fwd(indptr, indices, ew, nd, ns, E, feat, mode, dtype, X, out) == 0);
                MUST(fastgl_oracle_aggregate_bwd(indptr, indices, ew, nd, ns, E, feat, mode, dtype, G, dX) == 0);
                MUST(fastgl_oracle_par_aggregate_fwd(indptr, indices, ew, nd, ns, E, feat, mode, dtype, X, out) == 0);
                MUST(fastgl_oracle_par_aggregate_bwd(indptr, indices, ew, nd, ns, E, feat, mode, dtype, G, dX) == 0);
            }
        if (ns > 0) {
            int64_t ids[5] = {0, ns - 1, ns / 2, 0, ns - 1};
            void *rows = exact((size_t)(5 * feat), el);
            MUST(fastgl_oracle_gather_rows(X, ids, 5, feat, dtype, rows) == 0);
            free(rows);
        }
        float *gw = (float *)exact((size_t)E, 4);
        int32_t *scratch = (int32_t *)exact((size_t)ns, 4);
        for (int mode = 0; mode < 3; ++mode)
            MUST(fastgl_oracle_edge_weight_grad(indptr, indices, nd, ns, feat, mode, dtype, X, G, scratch, gw) == 0);
        free(gw); free(scratch); free(X); free(G); free(out); free(dX);
    }
    /* edge softmax and attention logits */
    float *alpha = (float *)exact((size_t)E, 4), *gs = (float *)exact((size_t)E, 4), *score = (float *)exact((size_t)E, 4);
    float *el = floats((size_t)nd), *er = floats((size_t)ns), *gel = (float *)exact((size_t)nd, 4), *ger = (float *)exact((size_t)ns, 4);
    double *acc = (double *)exact((size_t)ns, 8);
    MUST(fastgl_oracle_edge_score_fwd(indptr, indices, nd, ns, el, er, 0.2, score) == 0);
    MUST(fastgl_oracle_edge_softmax_fwd(indptr, nd, score, alpha) == 0);
    MUST(fastgl_oracle_edge_softmax_bwd(indptr, nd, alpha, w, gs) == 0);
    MUST(fastgl_oracle_edge_score_bwd(indptr, indices, nd, ns, el, er, 0.2, gs, acc, gel, ger) == 0);
    free(alpha); free(gs); free(score); free(el); free(er); free(gel); free(ger); free(acc);
    free(indptr); free(indices); free(w); free(din); free(dout); free(pT); free(iT); free(pm); free(lr); free(cp); free(split);
}

static void update_phase(int64_t M, int64_t K, int64_t N)
{
    for (int dtype = 0; dtype < 2; ++dtype) {
        const size_t el = dtype == 0 ? 4 : 2;
        void *H = dtype == 0 ? (void *)floats((size_t)(M * K)) : (void *)halves((size_t)(M * K));
        void *W = dtype == 0 ? (void *)floats((size_t)(K * N)) : (void *)halves((size_t)(K * N));
        void *dY = dtype == 0 ? (void *)floats((size_t)(M * N)) : (void *)halves((size_t)(M * N));
        float *b = floats((size_t)N);
        void *Y = exact((size_t)(M * N), el), *dH = exact((size_t)(M * K), el);
        float *dW = (float *)exact((size_t)(K * N), 4), *db = (float *)exact((size_t)N, 4);
        for (int relu = 0; relu < 2; ++relu) {
            MUST(fastgl_oracle_update_fwd_dt(H, W, relu ? b : NULL, M, K, N, relu, dtype, Y) == 0);
            MUST(fastgl_oracle_update_bwd_dt(H, W, Y, dY, M, K, N, relu, dtype, dH, dW, db) == 0);
        }
        free(H); free(W); free(dY); free(b); free(Y); free(dH); free(dW); free(db);
    }
}

static void id_sets(int64_t n_dst, int64_t n_nbr, int64_t span)
{
    int64_t *dst = (int64_t *)exact((size_t)n_dst, 8), *nbr = (int64_t *)exact((size_t)n_nbr, 8);
    for (int64_t i = 0; i < n_dst; ++i) dst[i] = 1000000 + i * 7;          /* distinct */
    for (int64_t i = 0; i < n_nbr; ++i) nbr[i] = (rnd() % 3 == 0 && n_dst > 0) ? dst[rnd() % (uint32_t)n_dst] : (int64_t)(rnd() % (uint32_t)span);
    int32_t *local = (int32_t *)exact((size_t)n_nbr, 4);
    int64_t *uniq = (int64_t *)exact((size_t)(n_dst + n_nbr), 8);
    const int64_t U = fastgl_oracle_idmap(dst, n_dst, nbr, n_nbr, local, uniq);
    MUST(U >= n_dst && U <= n_dst + n_nbr);
    const int64_t n = n_dst + n_nbr, slots = n + 3;
    int64_t *ids = (int64_t *)exact((size_t)n, 8), *key = (int64_t *)exact((size_t)slots, 8), *val = (int64_t *)exact((size_t)slots, 8);
    int64_t *loc = (int64_t *)exact((size_t)n, 8);
    if (n_dst) memcpy(ids, dst, (size_t)n_dst * 8);
    if (n_nbr) memcpy(ids + n_dst, nbr, (size_t)n_nbr * 8);
    MUST(fastgl_oracle_fused_map_seq(ids, n, slots, key, val, loc) == U);
    /* Match of the hop's source list against itself shifted: some rows reused, some loaded */
    int64_t *prev = (int64_t *)exact((size_t)U, 8);
    for (int64_t i = 0; i < U; ++i) prev[i] = uniq[i] + (i % 3 == 0 ? 1 : 0) * 100000007;
    int32_t *mrow = (int32_t *)exact((size_t)U, 4), *lpos = (int32_t *)exact((size_t)U, 4);
    int64_t *lgid = (int64_t *)exact((size_t)U, 8);
    const int64_t nload = fastgl_oracle_match(prev, U, uniq, U, mrow, lpos, lgid);
    MUST(nload >= 0 && nload <= U);
    MUST(fastgl_oracle_overlap(prev, U, uniq, U) == U - nload);
    const int64_t feat = 5;
    float *Xp = floats((size_t)(U * feat)), *Xl = floats((size_t)(nload * feat)), *Xn = (float *)exact((size_t)(U * feat), 4);
    MUST(fastgl_oracle_assemble(Xp, Xl, mrow, U, feat, 4, Xn) == 0);
    free(dst); free(nbr); free(local); free(uniq); free(ids); free(key); free(val); free(loc); free(prev); free(mrow);
    free(lpos); free(lgid); free(Xp); free(Xl); free(Xn);
}

int main(void)
{
    one_block(0, 0, 0, 0, 8);            /* nothing at all */
    one_block(7, 0, 0, 0, 3);            /* rows but no source nodes, hence no edges */
    one_block(1, 1, 0, 1, 1);            /* one edge */
    one_block(40, 90, 6, 11, 5);         /* ordinary */
    one_block(9, 30, 0, 700, 4);         /* one row far above the long-row threshold, the rest empty */
    one_block(300, 17, 9, 300, 33);      /* heavy reuse of few sources */
    update_phase(0, 3, 2); update_phase(5, 0, 2); update_phase(5, 3, 0); update_phase(13, 7, 9); update_phase(1, 1, 1);
    id_sets(0, 0, 10); id_sets(5, 0, 10); id_sets(0, 9, 4); id_sets(20, 200, 50); id_sets(64, 64, 1 << 30);
    for (int64_t n = 0; n <= 6; ++n) {
        int64_t *O = (int64_t *)exact((size_t)(n * n), 8), *size = (int64_t *)exact((size_t)n, 8);
        int32_t *order = (int32_t *)exact((size_t)n, 4);
        for (int64_t i = 0; i < n; ++i) size[i] = 10 + i;
        for (int64_t i = 0; i < n; ++i)
            for (int64_t j = 0; j <= i; ++j) O[i * n + j] = O[j * n + i] = i == j ? size[i] : (int64_t)(rnd() % 9);
        MUST(fastgl_oracle_greedy_reorder(O, size, n, order) == 0);
        free(O); free(size); free(order);
    }
    printf("oracle sanitize check: clean\n");
    return 0;
}
