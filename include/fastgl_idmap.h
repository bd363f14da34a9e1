/*
 * fastgl_idmap.h - C ABI of the ID map of the sample phase on MI355X (gfx950).
 *
 * Paper Section 2.2 ("ID map"): the global IDs of the nodes of a sampled
 * subgraph are converted to local IDs that are consecutive and start from 0.
 * Section 3.3 splits this into building a hash table of the global IDs,
 * numbering the distinct ones, and translating every global ID; Section 4.3,
 * Algorithm 2 ("Fused-Map") fuses the numbering into the table build: the
 * thread whose compare-and-swap claims an empty slot takes the next local ID
 * from an atomic counter, and a second kernel translates.
 *
 * One call maps one sampled hop.  Input: the destination nodes of the hop
 * (n_dst DISTINCT global IDs) and the sampled neighbour list (n_nbr global IDs,
 * repeats allowed, in the edge order of the hop's CSR).  Output:
 *   local_nbr[e]   local ID of neighbour entry e  (the `indices` array of the block)
 *   unique_gid[l]  global ID of local ID l, l = 0 .. U-1  (the source nodes of
 *                  the block; what fastgl_gather_rows takes as ids)
 *   result[0] = U, result[1] = number of violations (see below)
 * Destination i always keeps local ID i (the block's destinations are a prefix
 * of its sources).  The other nodes are numbered
 *   FASTGL_IDMAP_ORDERED  by first appearance in the neighbour list: one valid
 *                         answer, the same on every run (compare-and-swap
 *                         insertion, then the smallest position per slot and a
 *                         prefix count instead of a counter);
 *   FASTGL_IDMAP_FUSED    as Algorithm 2 does, by the order in which threads
 *                         claim slots: any run gives a valid bijection, the
 *                         numbering may differ from run to run.
 *
 * Global IDs are 64-bit and must be >= 0 (-1 marks an empty slot).  A negative
 * ID or a repeated destination ID is counted in result[1]; with result[1] != 0
 * the other outputs are unspecified (but every access stays in bounds).
 *
 * Conventions are those of fastgl_agg.h: all arrays are DEVICE memory owned by
 * the caller (result too: int32[2]), nothing is allocated, work is enqueued on
 * `stream` (hipStream_t as void*) without synchronising the host; read
 * result[] after synchronising.  unique_gid must hold n_dst + n_nbr entries.
 * n_dst + n_nbr < 2^30.  Host-checkable mistakes are refused before any launch.
 */
#ifndef FASTGL_IDMAP_H
#define FASTGL_IDMAP_H

#include "fastgl_agg.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { FASTGL_IDMAP_ORDERED = 0, FASTGL_IDMAP_FUSED = 1 } fastgl_idmap_mode;

/* Slots of the hash table used for n_ids = n_dst + n_nbr global IDs: 1.5 per
 * input ID (at least 1024).  At most n_ids keys ever enter it, so it keeps empty
 * slots and linear probing always ends; a sampled hop, whose IDs mostly repeat,
 * fills a quarter of it. 0 if n_ids is negative or too large. */
int64_t fastgl_idmap_table_slots(int64_t n_ids);

/* Bytes of device workspace (256-byte aligned) one call needs: the table
 * (64-bit keys, two 32-bit words per slot), the slot of every input ID and
 * the block counts of the ordered mode. 0 for bad sizes. */
size_t fastgl_idmap_workspace_bytes(int64_t n_dst, int64_t n_nbr);

fastgl_status fastgl_idmap(const int64_t *dst_gid, int64_t n_dst, const int64_t *nbr_gid, int64_t n_nbr,
                           fastgl_idmap_mode mode, int32_t *local_nbr, int64_t *unique_gid, int32_t *result,
                           void *workspace, size_t workspace_bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* FASTGL_IDMAP_H */
