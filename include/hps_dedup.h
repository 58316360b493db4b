/*
 * hps_dedup.h - C ABI of the deduplication operator of the Hierarchical Parameter Server
 * (paper Sec. 2.2 "Deduplication and skewness": Q* = dedup(Q) is applied to every query batch
 * before any further step), and of the row expansion that hands every position of Q the row of
 * its key after Q* has been looked up.
 *
 *   dedup:   unique_keys[0 .. u) = the distinct values of keys[0 .. n), each once;
 *            inverse[i] = the place of keys[i] in unique_keys, so unique_keys[inverse[i]] == keys[i];
 *            *n_unique = u.
 *   expand:  out[i] = rows[inverse[i]]  (rows of `dim` 32-bit words, opaque bit patterns).
 *
 * The paper fixes no order of Q*; the order in which this operator lists the distinct keys is
 * unspecified and may differ from call to call (any order, with its matching inverse map, is a
 * correct result).  All 2^64 key values are ordinary to dedup, INT64_MIN included.
 *
 * Pointers named "device" are GPU addresses on the session's device; keys 8-byte, rows 16-byte,
 * index arrays 4-byte aligned.  Every call is asynchronous on `stream` (a hipStream_t passed as
 * void*, NULL = the null stream).  A session owns its scratch table: calls on one session must
 * not overlap (order them on one stream or with events); different sessions are independent.
 * Status codes and hps_status_t are those of hps_cache.h; the message of the last failing call
 * of this header on the calling thread is returned by hps_dedup_last_error().
 */
#ifndef HPS_DEDUP_H
#define HPS_DEDUP_H

#include <stddef.h>
#include <stdint.h>

#include "hps_cache.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct hps_dedup_session hps_dedup_t;

/* Create a session for batches of up to max_n keys (0 < max_n <= 2^30) on the current device.
 * Allocates three hash tables of the next power of two >= 2 * max_n slots each (12 bytes per
 * slot): two that alternate between calls, one for calls captured into a HIP graph.
 * Errors: HPS_ERR_INVALID_ARG, HPS_ERR_OOM, HPS_ERR_DEVICE; *out is NULL on failure. */
hps_status_t hps_dedup_create(size_t max_n, hps_dedup_t **out);

/* Waits for the device, then frees the session.  NULL is accepted. */
hps_status_t hps_dedup_destroy(hps_dedup_t *s);

/* Q* = dedup(Q), Sec. 2.2.
 *   keys        device, int64 [n], read only
 *   unique_keys device, int64 [n]  (first *n_unique entries written)
 *   inverse     device, uint32 [n]
 *   n_unique    device, one uint32
 * n == 0 writes *n_unique = 0 and nothing else.  n > max_n is HPS_ERR_INVALID_ARG. */
hps_status_t hps_dedup(hps_dedup_t *s, const int64_t *keys, size_t n, int64_t *unique_keys,
                       uint32_t *inverse, uint32_t *n_unique, void *stream);

/* hps_dedup for callers that cannot allocate device memory: code under HIP graph capture, tight
 * serving loops, harnesses that forbid allocation.  Same arguments and results as hps_dedup, but
 * no session: the hash table lives in a static device array of the library (3 MiB per GPU, held
 * until the process ends), so the call allocates and frees nothing (no hipMalloc, no hipFree, no
 * allocating library routine); it only launches three kernels on `stream`.  At most
 * HPS_DEDUP_NOALLOC_MAX keys per call: a larger n returns HPS_ERR_INVALID_ARG and launches
 * nothing.  Every call on a GPU uses that GPU's one array: calls that overlap on one GPU (on
 * different streams, or from different threads without ordering) race and must be ordered by the
 * caller; calls on one stream are ordered.  The current device is the one the call works on. */
#define HPS_DEDUP_NOALLOC_MAX 131072u
hps_status_t hps_dedup_noalloc(const int64_t *keys, size_t n, int64_t *unique_keys, uint32_t *inverse,
                               uint32_t *n_unique, void *stream);

/* out[i] = rows[inverse[i]] for i < n: the step after the lookup of Q* (Sec. 2.2).
 *   rows    device, [u][dim] 32-bit words, read only; every inverse[i] must be < u (not checked)
 *   inverse device, uint32 [n]
 *   out     device, [n][dim], must not overlap rows
 * dim a non-zero multiple of 4; n < 2^32.  Needs no session. */
hps_status_t hps_expand_rows(const float *rows, const uint32_t *inverse, size_t n, uint32_t dim,
                             float *out, void *stream);

const char *hps_dedup_last_error(void);

#ifdef __cplusplus
}
#endif
#endif
