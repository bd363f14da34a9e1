/*
 * fastgl_match.h - C ABI of the Match process and the Greedy Reorder Strategy
 * on MI355X (gfx950).
 *
 * Paper Section 4.1 ("Match-Reorder Strategy"): before the node features of a
 * new mini-batch are loaded, its node set is intersected with the node set of
 * the last mini-batch; the features of the overlapping nodes are reused and
 * only the rest (LoadNodeID) is loaded.  The match degree of two mini-batches
 * is M_ij = N_o / min(N_i, N_j) (N_o common nodes); Algorithm 1 reorders the n
 * sampled mini-batches greedily so that each one follows the mini-batch it
 * shares most with.
 *
 * Conventions are those of fastgl_agg.h (caller-owned DEVICE memory, caller
 * workspace, work enqueued on `stream` without synchronising the host, return
 * codes + fastgl_last_error()) with the exceptions stated at the functions
 * that take HOST arrays.  Global IDs are 64-bit and >= 0; the IDs of one
 * mini-batch are distinct.  A negative or repeated ID is counted as a
 * violation; with violations the other outputs are unspecified (all accesses
 * stay in bounds).  Sizes stay below 2^30.
 */
#ifndef FASTGL_MATCH_H
#define FASTGL_MATCH_H

#include "fastgl_agg.h"

#ifdef __cplusplus
extern "C" {
#endif

size_t fastgl_match_workspace_bytes(int64_t n_prev, int64_t n_new);

/* Match: prev_gid[n_prev] = nodes of the last mini-batch in the row order of
 * its feature matrix; new_gid[n_new] = nodes of the mini-batch to be computed,
 * in local-ID order.  Outputs (n_new entries of room each):
 *   src_row[i]   >= 0: node i is row src_row[i] of the last feature matrix;
 *                < 0 : node i must be loaded; it is entry k = -1 - src_row[i]
 *                      of the load lists
 *   load_pos[k]  position i of the k-th node to load (ascending)
 *   load_gid[k]  its global ID (what fastgl_gather_rows or a host loader takes)
 *   result[0] = n_load, result[1] = violations      (device int32[2])       */
fastgl_status fastgl_match(const int64_t *prev_gid, int64_t n_prev, const int64_t *new_gid, int64_t n_new,
                           int32_t *src_row, int32_t *load_pos, int64_t *load_gid, int32_t *result,
                           void *workspace, size_t workspace_bytes, void *stream);

/* The new feature matrix: X_new[i,:] = X_prev[src_row[i],:] if src_row[i] >= 0,
 * else X_load[-1 - src_row[i],:] (X_load = the loaded rows in load-list order).
 * Row-major [rows, feat], leading dimension feat; X_new must not overlap the
 * inputs (the two feature buffers of consecutive mini-batches alternate).
 * src_row is trusted like the indices of a block: entries must lie in
 * [-n_load, n_prev). */
fastgl_status fastgl_assemble_rows(const void *X_prev, int64_t n_prev, const void *X_load, int64_t n_load,
                                   const int32_t *src_row, int64_t n_new, int64_t feat, fastgl_dtype dtype,
                                   void *X_new, void *stream);

#define FASTGL_MAX_REORDER_BATCHES 64

size_t fastgl_overlap_workspace_bytes(int64_t total_ids);

/* N_o for every pair of n mini-batches at once.  gid = the node lists of the
 * mini-batches one after the other (device); offsets_host[n+1] (HOST) = where
 * each starts.  counts[i*n + j] (device int64) = number of common nodes of
 * mini-batches i and j (counts[i*n+i] = N_i); violations (device int32[1]).
 * n <= FASTGL_MAX_REORDER_BATCHES. */
fastgl_status fastgl_overlap_counts(const int64_t *gid, const int64_t *offsets_host, int n, int64_t *counts,
                                    int32_t *violations, void *workspace, size_t workspace_bytes, void *stream);

/* Algorithm 1 on the HOST (all three arrays are host memory): overlap[i*n+j] as
 * above, size[i] = N_i; order[0..n-1] = the reordered list as 0-based indices.
 * It starts with mini-batch 0; candidates are the mini-batches not yet listed;
 * equal match degrees go to the smaller index. */
fastgl_status fastgl_greedy_reorder(const int64_t *overlap_host, const int64_t *size_host, int64_t n,
                                    int32_t *order_host);

#ifdef __cplusplus
}
#endif
#endif /* FASTGL_MATCH_H */
