/*
 * hps_lookup.h — Algorithm 1 of the paper ("Embedding cache insertion", Sec. 3.1 / Sec. 4.3) on top
 * of the GPU embedding cache of hps_cache.h: look the batch up in the cache, compute the hit rate,
 * and either fetch and insert the missing rows at once (synchronous insertion, hit rate below the
 * threshold) or hand out the default vector for them now and fetch and insert them in the
 * background (asynchronous insertion).
 *
 * The lower storage tiers (Sec. 5) are the caller's: a fetch callback that receives the missing
 * keys in host memory and fills their rows in host memory.  Everything else runs on the device,
 * including the deduplication of the missing keys (Sec. 2.2, hps_dedup.h): only distinct keys
 * travel to the host.  In asynchronous mode that, too, happens on the background thread's
 * stream: the call itself only copies the miss list aside, into one of the object's slots (device
 * buffers of max_batch keys allocated at create: at most 66 of them and at most 256 MiB, never
 * fewer than 2; a lookup call allocates nothing).  When no slot is free the oldest waiting batch
 * is dropped (its keys stay missing until a later batch asks for them again).
 * One lookup object serves one stream of batches (it owns one workspace, the paper's `ws`); use
 * one object per concurrent inference worker, all on the same cache.
 */
#ifndef HPS_LOOKUP_H
#define HPS_LOOKUP_H

#include "hps_cache.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct hps_lookup_session hps_lookup_t;

/*
 * Lower-tier fetch: write the row of keys[i] to rows[i*dim .. i*dim+dim) for i < n.  keys and rows
 * are host pointers (pinned, owned by the lookup object); keys are distinct, in no particular
 * order.  Called on the thread
 * that calls hps_lookup (synchronous insertion) or on the object's background thread.
 */
typedef void (*hps_fetch_fn)(void *user, const int64_t *keys, size_t n, float *rows);

/*
 * cache           the cache to serve from; it must allow concurrent writers
 *                 (hps_cache_set_concurrent_writers(cache, 1), the default) because background
 *                 inserts overlap later queries.
 * max_batch       largest n a lookup call may pass (1 .. 2^30).
 * hit_threshold   t of Alg. 1: hit rate < t selects synchronous insertion.  0 = always
 *                 asynchronous, anything above 1 = always synchronous.
 * default_row     [host, dim fp32] vector handed out for missing keys in asynchronous mode.
 * Errors: INVALID_ARG, OOM, DEVICE.
 */
hps_status_t hps_lookup_create(hps_cache_t *cache, size_t max_batch, float hit_threshold,
                               const float *default_row, hps_fetch_fn fetch, void *user,
                               hps_lookup_t **out_lookup);

/*
 * One pass of Alg. 1.  keys [device, n int64], out [device, n*dim fp32], stream as in hps_cache.h.
 * Hit rate = 1 - misses / n per position, computed and compared with the threshold in single
 * precision (a deliberate reading of the hit-rate step of Alg. 1, whose divisor is declared as the
 * capacity of the cache).  On return every row of out is either its key's cached row, its fetched
 * row (synchronous mode) or the default row (asynchronous mode), in stream order: the call
 * synchronises the host with `stream` once, to read the miss count, as Alg. 1 needs it.
 * *hit_rate [host] and *was_synchronous [host] may be NULL.
 */
hps_status_t hps_lookup(hps_lookup_t *lookup, const int64_t *keys, size_t n, float *out,
                        float *hit_rate, int *was_synchronous, void *stream);

/*
 * The cache refresh cycle of the paper (Sec. 6, Fig. 3 steps 1-5): dump the cached keys in batches
 * of `batch_slots` slots, look each batch up in the lower tiers through `fetch`, copy the rows to
 * the device and Update the cache with them.  The dump and the copy of the keys to the host run on
 * a stream of their own, so the host-side lookup of one batch overlaps the upload and Update of
 * the previous one.
 *
 * A session owns everything the cycle needs (two device and two pinned host buffers of
 * batch_slots keys and rows, its stream, its events), allocated by hps_refresh_create on the
 * current device; hps_refresh_run allocates nothing and may be called any number of times, one
 * call at a time per session.  batch_slots in 1 .. 2^31 - 1 (clamped to the size of the cache).
 *
 * hps_refresh_run returns when the whole cache has been refreshed; *n_refreshed [host] (may be
 * NULL) receives the number of keys that were dumped and updated.  Queries may run meanwhile (on
 * other streams, with the cache in its concurrent-writer mode).  Keys that an overlapping insert
 * evicts between dump and Update are skipped by the Update (Alg. 4).  The lower tier must hold
 * every cached key: `fetch` has no way to say "not found".  Errors: INVALID_ARG, OOM (create),
 * DEVICE.
 */
typedef struct hps_refresh_session hps_refresh_t;
hps_status_t hps_refresh_create(hps_cache_t *cache, size_t batch_slots, hps_refresh_t **out_session);
hps_status_t hps_refresh_run(hps_refresh_t *session, hps_fetch_fn fetch, void *user, size_t *n_refreshed,
                             void *stream);
hps_status_t hps_refresh_destroy(hps_refresh_t *session);

/* One refresh with a session made for this call only (create + run + destroy: it allocates). */
hps_status_t hps_cache_refresh(hps_cache_t *cache, size_t batch_slots, hps_fetch_fn fetch, void *user,
                               size_t *n_refreshed, void *stream);

/* Block until every queued asynchronous insertion has been applied to the cache. */
hps_status_t hps_lookup_drain(hps_lookup_t *lookup);

/* Drains, then frees the object (not the cache). */
hps_status_t hps_lookup_destroy(hps_lookup_t *lookup);

/* Message for the last error of the hps_lookup_* calls on this thread. */
const char *hps_lookup_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* HPS_LOOKUP_H */
