/*
 * CPU oracle for the Match process and the Greedy Reorder Strategy.  TEST
 * INFRASTRUCTURE ONLY: nothing in the product path may call this; tests, the
 * smoke check and the benchmark's cpu_baseline leg do.  It shares no code with
 * the GPU library.
 *
 * What it computes (paper Section 4.1, "Match-Reorder Strategy"):
 *   Match: before the features of a new mini-batch are loaded, the node set of
 *     the mini-batch is intersected with the node set of the last one
 *     (OverlapNodeID); only the rest (LoadNodeID) is loaded, the features of the
 *     overlapping nodes are reused.  Here: for every node i of the new batch
 *     (global IDs, distinct, in local-ID order) match_row[i] = its row in the
 *     last batch, or -1; load_pos = the positions with -1, ascending; and the
 *     new feature matrix is assembled from the last one and the loaded rows.
 *   Match degree: M_ij = N_o / min(N_i, N_j), N_o = number of common nodes.
 *   Greedy Reorder (Algorithm 1): start with the first sampled mini-batch; then
 *     always append the mini-batch with the largest match degree to the one
 *     appended last, and strike out (zero the row and column of) the one just
 *     left.  Readings: a mini-batch is never compared with itself; candidates
 *     are the mini-batches not yet in the list (the listing zeroes the rows of
 *     the inserted ones, which leaves ties at 0 between inserted and disjoint
 *     ones undecided); among equal match degrees the smallest index wins.
 *
 * Written as the definitions: sort + binary search for membership, a linear
 * merge for the intersection size, the listing's loop for the reorder.
 * Pins: tests/test_match_oracle_pins.py.  Nothing here is "parity unpinned".
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct { int64_t gid; int64_t row; } ent_t;

static int cmp_ent(const void *a, const void *b)
{
    const ent_t *x = (const ent_t *)a, *y = (const ent_t *)b;
    return x->gid < y->gid ? -1 : (x->gid > y->gid ? 1 : (x->row < y->row ? -1 : (x->row > y->row)));
}

static int cmp_i64(const void *a, const void *b)
{
    const int64_t x = *(const int64_t *)a, y = *(const int64_t *)b;
    return x < y ? -1 : (x > y);
}

/* Returns the number of positions to load (n_load), or -1 on bad arguments /
 * out of memory, or -2 if prev_gid repeats an ID.  load_pos / load_gid hold
 * n_new entries of room. */
int64_t fastgl_oracle_match(const int64_t *prev_gid, int64_t n_prev, const int64_t *new_gid, int64_t n_new,
                            int32_t *match_row, int32_t *load_pos, int64_t *load_gid)
{
    if (n_prev < 0 || n_new < 0) return -1;
    ent_t *p = (ent_t *)malloc((size_t)(n_prev > 0 ? n_prev : 1) * sizeof(ent_t));
    if (!p) return -1;
    for (int64_t j = 0; j < n_prev; ++j) { p[j].gid = prev_gid[j]; p[j].row = j; }
    qsort(p, (size_t)n_prev, sizeof(ent_t), cmp_ent);
    for (int64_t j = 1; j < n_prev; ++j)
        if (p[j].gid == p[j - 1].gid) { free(p); return -2; }
    int64_t n_load = 0;
    for (int64_t i = 0; i < n_new; ++i) {
        int64_t lo = 0, hi = n_prev;            /* first entry with gid >= new_gid[i] */
        while (lo < hi) {
            const int64_t mid = lo + (hi - lo) / 2;
            if (p[mid].gid < new_gid[i]) lo = mid + 1; else hi = mid;
        }
        if (lo < n_prev && p[lo].gid == new_gid[i]) {
            match_row[i] = (int32_t)p[lo].row;
        } else {
            match_row[i] = -1;
            load_pos[n_load] = (int32_t)i;
            load_gid[n_load] = new_gid[i];
            ++n_load;
        }
    }
    free(p);
    return n_load;
}

/* Number of common IDs of two lists of distinct IDs (N_o). */
int64_t fastgl_oracle_overlap(const int64_t *a, int64_t na, const int64_t *b, int64_t nb)
{
    if (na < 0 || nb < 0) return -1;
    int64_t *x = (int64_t *)malloc((size_t)(na > 0 ? na : 1) * 8), *y = (int64_t *)malloc((size_t)(nb > 0 ? nb : 1) * 8);
    if (!x || !y) { free(x); free(y); return -1; }
    memcpy(x, a, (size_t)na * 8);
    memcpy(y, b, (size_t)nb * 8);
    qsort(x, (size_t)na, 8, cmp_i64);
    qsort(y, (size_t)nb, 8, cmp_i64);
    int64_t i = 0, j = 0, n_o = 0;
    while (i < na && j < nb) {
        if (x[i] < y[j]) ++i;
        else if (x[i] > y[j]) ++j;
        else { ++n_o; ++i; ++j; }
    }
    free(x); free(y);
    return n_o;
}

/* Algorithm 1.  overlap[i*n + j] = N_o of mini-batches i and j, size[i] = N_i.
 * order[0..n-1] receives the ReorderedList as 0-based mini-batch indices. */
int fastgl_oracle_greedy_reorder(const int64_t *overlap, const int64_t *size, int64_t n, int32_t *order)
{
    if (n < 0) return 1;
    if (n == 0) return 0;
    double *M = (double *)malloc((size_t)n * (size_t)n * sizeof(double));
    char *inserted = (char *)calloc((size_t)n, 1);
    if (!M || !inserted) { free(M); free(inserted); return 1; }
    for (int64_t i = 0; i < n; ++i)
        for (int64_t j = 0; j < n; ++j) {
            const int64_t mn = size[i] < size[j] ? size[i] : size[j];
            M[i * n + j] = (i == j || mn <= 0) ? 0.0 : (double)overlap[i * n + j] / (double)mn;
        }
    order[0] = 0;                              /* ReorderedList.insert(SubG_1, 1) */
    inserted[0] = 1;
    int64_t z = 0;
    for (int64_t i = 1; i < n; ++i) {
        int64_t h = -1;
        for (int64_t k = 0; k < n; ++k) {      /* h = argmax_k m_zk over the mini-batches not yet inserted */
            if (inserted[k]) continue;
            if (h < 0 || M[z * n + k] > M[z * n + h]) h = k;
        }
        order[i] = (int32_t)h;
        inserted[h] = 1;
        for (int64_t k = 0; k < n; ++k) { M[z * n + k] = 0.0; M[k * n + z] = 0.0; }
        z = h;
    }
    free(M); free(inserted);
    return 0;
}

/* X_new[i,:] = X_prev[match_row[i],:] where match_row[i] >= 0, else the next row of X_load
 * (rows of X_load are in load_pos order).  elem = bytes per element. */
int fastgl_oracle_assemble(const void *X_prev, const void *X_load, const int32_t *match_row, int64_t n_new,
                           int64_t feat, int64_t elem, void *X_new)
{
    if (n_new < 0 || feat < 0 || elem <= 0) return 1;
    const size_t rb = (size_t)feat * (size_t)elem;
    int64_t k = 0;
    for (int64_t i = 0; i < n_new; ++i) {
        const char *src = match_row[i] >= 0 ? (const char *)X_prev + (size_t)match_row[i] * rb
                                            : (const char *)X_load + (size_t)(k++) * rb;
        memcpy((char *)X_new + (size_t)i * rb, src, rb);
    }
    return 0;
}
