/*
 * CPU oracle for the ID map of the sample phase.  TEST INFRASTRUCTURE ONLY:
 * nothing in the product path may call this; tests, the smoke check and the
 * benchmark's cpu_baseline leg do.  It shares no code with the GPU library.
 *
 * What the ID map computes (paper Section 2.2, "ID map"; Section 3.3, the three
 * steps; Section 4.3, Algorithm 2 "Fused-Map"): the global IDs of the nodes of
 * a sampled subgraph are replaced by local IDs that are consecutive and start
 * from 0.  For one sampled hop the input is the list of destination nodes
 * (distinct global IDs) followed by the sampled neighbour list (global IDs with
 * repeats); the output is
 *   unique_gid[l]   the global ID that got local ID l          (l = 0..U-1)
 *   local_nbr[e]    the local ID of neighbour entry e
 * Any bijection is a correct ID map; the one fixed here (and compared bit for
 * bit with the GPU's ordered mode) numbers the nodes in order of FIRST
 * APPEARANCE in the concatenated list, so destination i keeps local ID i.
 *
 * Two functions:
 *   fastgl_oracle_idmap         the definition, through a sort: the first
 *                               position of every distinct ID, ranked.
 *   fastgl_oracle_fused_map_seq Algorithm 2 run by ONE thread in list order,
 *                               in the paper's notation (HashTable keys -1 /
 *                               values 0 at start, HashFunction = id mod table
 *                               size as in the paper's example, linear probing,
 *                               LocalID counter).  Run sequentially the
 *                               algorithm must reproduce the definition; that
 *                               is one of the pins.  Reading: the probe index
 *                               wraps to 0 past the end of the table (the
 *                               listing only says HashIndex + 1).
 *
 * Pins (tests/test_idmap_oracle_pins.py): the paper's worked example (table of
 * 5 slots, id mod 5, global ID 3 gets local ID 0, a second insert of 3 changes
 * nothing), brute force with a Python dict, Algorithm 2 against the definition,
 * numpy's unique, colliding and wrapping probe chains worked by hand, and the
 * bijection invariants.  Nothing here is "parity unpinned".
 */
#include <stdint.h>
#include <stdlib.h>

typedef struct { int64_t gid; int64_t pos; } pair_t;

static int cmp_pair(const void *a, const void *b)
{
    const pair_t *x = (const pair_t *)a, *y = (const pair_t *)b;
    if (x->gid != y->gid) return x->gid < y->gid ? -1 : 1;
    return x->pos < y->pos ? -1 : (x->pos > y->pos ? 1 : 0);
}

/* Returns U >= 0, or -1 on bad arguments / out of memory, or -2 when the
 * destination list repeats an ID (destination i could not keep local ID i). */
int64_t fastgl_oracle_idmap(const int64_t *dst_gid, int64_t n_dst, const int64_t *nbr_gid, int64_t n_nbr,
                            int32_t *local_nbr, int64_t *unique_gid)
{
    if (n_dst < 0 || n_nbr < 0) return -1;
    const int64_t n = n_dst + n_nbr;
    if (n == 0) return 0;
    pair_t *p = (pair_t *)malloc((size_t)n * sizeof(pair_t));
    int64_t *first_of = (int64_t *)malloc((size_t)n * sizeof(int64_t));   /* first position of the ID at position i */
    int64_t *rank_at = (int64_t *)malloc((size_t)n * sizeof(int64_t));    /* local ID given at a first position */
    if (!p || !first_of || !rank_at) { free(p); free(first_of); free(rank_at); return -1; }
    for (int64_t i = 0; i < n; ++i) {
        p[i].gid = i < n_dst ? dst_gid[i] : nbr_gid[i - n_dst];
        p[i].pos = i;
    }
    qsort(p, (size_t)n, sizeof(pair_t), cmp_pair);
    for (int64_t i = 0; i < n;) {              /* a run of equal IDs: its first entry has the smallest position */
        int64_t j = i;
        while (j < n && p[j].gid == p[i].gid) { first_of[p[j].pos] = p[i].pos; ++j; }
        i = j;
    }
    int64_t U = 0;
    for (int64_t i = 0; i < n; ++i)
        if (first_of[i] == i) {
            rank_at[i] = U;
            unique_gid[U] = i < n_dst ? dst_gid[i] : nbr_gid[i - n_dst];
            ++U;
        }
    int64_t status = U;
    for (int64_t i = 0; i < n_dst; ++i)
        if (first_of[i] != i) status = -2;
    for (int64_t e = 0; e < n_nbr; ++e) local_nbr[e] = (int32_t)rank_at[first_of[n_dst + e]];
    free(p); free(first_of); free(rank_at);
    return status;
}

/* Algorithm 2, one thread.  key[] / value[] have table_size entries and are
 * initialised here (-1 / 0).  local[i] receives the local ID of ids[i], read
 * back from the table after all insertions (the paper's second kernel).
 * Returns LocalID (the number of distinct IDs), or -1 if the table is full. */
int64_t fastgl_oracle_fused_map_seq(const int64_t *ids, int64_t n, int64_t table_size, int64_t *key,
                                    int64_t *value, int64_t *local)
{
    if (n < 0 || table_size <= 0) return -1;
    for (int64_t s = 0; s < table_size; ++s) { key[s] = -1; value[s] = 0; }
    int64_t LocalID = 0;
    for (int64_t i = 0; i < n; ++i) {
        const int64_t GlobalID = ids[i];
        int64_t HashIndex = GlobalID % table_size;          /* HashFunction of the paper's example */
        if (HashIndex < 0) HashIndex += table_size;
        int Flag = 0;
        int64_t probes = 0;
        for (;;) {                                          /* InsertID */
            const int64_t Val = key[HashIndex];             /* atomicCAS(HashIndex, -1, GlobalID) ... */
            if (Val == -1) key[HashIndex] = GlobalID;       /* ... in one thread */
            if (Val == GlobalID || Val == -1) { Flag = (Val != -1); break; }
            HashIndex = HashIndex + 1 == table_size ? 0 : HashIndex + 1;    /* linear probing, wrapping */
            if (++probes >= table_size) return -1;
        }
        if (!Flag) {                                        /* a new node: it takes the current LocalID */
            value[HashIndex] = LocalID;
            LocalID += 1;
        }
    }
    for (int64_t i = 0; i < n; ++i) {                       /* transform global IDs to local IDs */
        int64_t HashIndex = ids[i] % table_size;
        if (HashIndex < 0) HashIndex += table_size;
        while (key[HashIndex] != ids[i]) HashIndex = HashIndex + 1 == table_size ? 0 : HashIndex + 1;
        local[i] = value[HashIndex];
    }
    return LocalID;
}
