/*
 * hps_hostmap.h - a host-memory key -> row store with the call shape of the lower tiers that
 * Algorithm 1 of the paper falls back to (Sec. 3.1, Sec. 5: the volatile database is a hash map in
 * CPU memory, partitioned for parallel access).  It is a stand-in: one process, no network, no
 * eviction, no persistence; what it keeps of the real tier is the interface (batched lookup of the
 * missing keys into host memory) and the partitioning (keys are spread over 2^p independent hash
 * maps by their hash, and a batch is served partition by partition on a few threads).
 *
 * All pointers are HOST pointers.  put and fetch may be called from different threads; calls that
 * touch the same partition serialise on its lock.  Status codes are those of hps_cache.h.
 */
#ifndef HPS_HOSTMAP_H
#define HPS_HOSTMAP_H

#include <stddef.h>
#include <stdint.h>

#include "hps_cache.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct hps_hostmap hps_hostmap_t;

/* dim: 32-bit words per row (non-zero); partitions: a power of two in 1 .. 256; reserve: expected
 * number of keys (a hint).  Errors: HPS_ERR_INVALID_ARG, HPS_ERR_OOM. */
hps_status_t hps_hostmap_create(uint32_t dim, uint32_t partitions, size_t reserve, hps_hostmap_t **out);
hps_status_t hps_hostmap_destroy(hps_hostmap_t *map);

/* Insert or overwrite: rows[i*dim .. i*dim+dim) becomes the row of keys[i].  A key given twice
 * keeps its last row. */
hps_status_t hps_hostmap_put(hps_hostmap_t *map, const int64_t *keys, const float *rows, size_t n);

/* rows[i] = the row of keys[i]; a key that is not stored gets an all-zero row and is counted.
 * *n_absent (may be NULL) receives how many keys of this call were not stored. */
hps_status_t hps_hostmap_get(hps_hostmap_t *map, const int64_t *keys, size_t n, float *rows, size_t *n_absent);

/* The same lookup with the signature of hps_fetch_fn (hps_lookup.h): pass the map as `user`. */
void hps_hostmap_fetch(void *user, const int64_t *keys, size_t n, float *rows);

/* Number of keys stored; total number of absent keys served by fetch/get so far. */
hps_status_t hps_hostmap_stats(hps_hostmap_t *map, size_t *n_keys, size_t *n_absent_total);

#ifdef __cplusplus
}
#endif
#endif
