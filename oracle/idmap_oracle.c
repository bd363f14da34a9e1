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

/* Where `id` sits in an open-addressing table with linear probing that wraps
 * past the last slot (Section 4.3): the first slot, starting at id mod
 * table_size (the hash of the paper's worked example), that holds `id` or is
 * still empty (-1).  Returns -1 when every slot holds another ID. */
static int64_t find_slot(const int64_t *key, int64_t table_size, int64_t id)
{
    int64_t s = id % table_size;
    if (s < 0) s += table_size;
    for (int64_t tried = 0; tried < table_size; ++tried) {
        if (key[s] == id || key[s] == -1) return s;
        s = (s + 1) % table_size;
    }
    return -1;
}

/* The Fused-Map of Section 4.3 (Algorithm 2) as ONE thread runs it: IDs are
 * inserted in input order; an ID that was not in the table yet claims its slot
 * and is numbered with the running count of distinct IDs; afterwards every ID
 * is looked up again to read its number.  With one thread the compare-and-swap
 * of the parallel version is just "write the ID if the slot is empty".
 * key[] / value[] have table_size entries and are initialised here (-1 / 0).
 * Returns the number of distinct IDs, or -1 if the table is full. */
int64_t fastgl_oracle_fused_map_seq(const int64_t *ids, int64_t n, int64_t table_size, int64_t *key,
                                    int64_t *value, int64_t *local)
{
    if (n < 0 || table_size <= 0) return -1;
    for (int64_t s = 0; s < table_size; ++s) { key[s] = -1; value[s] = 0; }
    int64_t distinct = 0;
    for (int64_t i = 0; i < n; ++i) {
        const int64_t s = find_slot(key, table_size, ids[i]);
        if (s < 0) return -1;
        if (key[s] == -1) {                 /* first time this ID is seen */
            key[s] = ids[i];
            value[s] = distinct++;
        }
    }
    for (int64_t i = 0; i < n; ++i) local[i] = value[find_slot(key, table_size, ids[i])];
    return distinct;
}
