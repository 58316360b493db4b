/*
 * hps_cache.h — C ABI of the MI355X (gfx950) GPU embedding cache.
 *
 * The cache is the level-1 store of the Hierarchical Parameter Server (paper Sec. 3.1,
 * Sec. 4): a set-associative, hash-indexed table of fixed-width fp32 embedding rows in GPU
 * memory that answers batched key -> row lookups (problem statement: Sec. 2.1, Q -> R_Q).
 *
 * Conventions for every call
 *   - Pointers marked [device] are device pointers on the GPU that was current when the
 *     cache was created (which must also be current at every call).  Row buffers (out, vals,
 *     rows) must be 16-byte aligned, key buffers 8-byte, index and counter words 4-byte.
 *     They must stay valid until the stream has finished the call's work; the caller owns
 *     them.  Pointers marked [host] are ordinary host pointers.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Every call
 *     only enqueues kernels and returns at once (Sec. 4.2, last paragraph); nothing
 *     synchronises the host.  Device-side faults surface on the caller's next sync.
 *   - Calls on one stream take effect in order.  Calls on different streams may overlap;
 *     see hps_cache_set_concurrent_writers.
 *   - Return value: HPS_OK or a negative hps_status_t.  Nothing is thrown.  After an error
 *     hps_last_error() gives a message (thread-local).
 *   - Keys are int64.  INT64_MIN marks an empty slot ("Null" in Alg. 2-4) and, together with
 *     INT64_MIN+1, is reserved: query reports such keys as misses, insert/update skip them.
 *   - Rows are `dim` 32-bit words moved as opaque bit patterns; no floating-point arithmetic
 *     is performed anywhere, so results are byte-exact.
 */
#ifndef HPS_CACHE_H
#define HPS_CACHE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct hps_cache hps_cache_t;   /* opaque; owned by the library */

typedef enum {
    HPS_OK              =  0,
    HPS_ERR_INVALID_ARG = -1,
    HPS_ERR_OOM         = -2,
    HPS_ERR_DEVICE      = -3
} hps_status_t;

#define HPS_MAX_TABLES 32               /* most tables one hps_cache_query_multi call takes */

/* Replacement policies (which slot a new key takes when its set is full). */
#define HPS_POLICY_VICTIM_COUNTER 0     /* per-set counter, insertion order (hps_cache_create) */
#define HPS_POLICY_LRU            1     /* least recently used by access stamp (Sec. 4.2, Alg. 2-3) */

/*
 * Create a cache of `capacity` slots organised as capacity/ways sets of `ways` slots
 * (Sec. 4.1: a key hashes to one set and may occupy any slot of it), rows of `dim` fp32.
 * Set of a key: upper 32 bits of the splitmix64 finaliser of the key, modulo the set count
 * (Alg. 2 "slabsetHasher(q) mod |S|"; the paper names no hash).
 * Requirements: ways a power of two in [1, 64]; capacity a non-zero multiple of ways with
 * capacity/ways < 2^31; dim a non-zero multiple of 4.  Allocates on the current device:
 * keys (8 B/slot), rows (4*dim B/slot), one victim counter and one sequence word per set.
 * All slots start empty.  *out_handle [host] receives the handle.
 * Errors: INVALID_ARG, OOM (allocation failed), DEVICE.
 */
hps_status_t hps_cache_create(size_t capacity, uint32_t ways, uint32_t dim,
                              hps_cache_t **out_handle);

/*
 * As hps_cache_create, with the replacement policy chosen.  HPS_POLICY_LRU is the paper's rule
 * (Sec. 4.2 "Replace", Alg. 2-3): every slot carries an access stamp; each query call advances a
 * global iteration count g and stamps the slots it hits with it; insert stamps an already cached
 * key, puts a new key into the lowest-numbered empty slot of its set or else over the least
 * recently used one (largest g - stamp modulo 2^32, lowest way on ties) and stamps it.  Update
 * leaves stamps alone (Alg. 4).  Costs 4 bytes per slot and one scattered 4-byte store per hit.
 */
hps_status_t hps_cache_create_policy(size_t capacity, uint32_t ways, uint32_t dim, int policy,
                                     hps_cache_t **out_handle);

/* Free everything the cache owns.  The caller must have synchronised all streams that used it. */
hps_status_t hps_cache_destroy(hps_cache_t *cache);

/*
 * Query (Sec. 4.2 "Query", Alg. 2).  For every position i < n:
 *   - keys[i] is cached  -> out[i*dim .. i*dim+dim) receives its row;
 *   - otherwise          -> <i, keys[i]> is appended to the miss list and out's row i is
 *                           left untouched (the caller fills defaults or fetched rows, Alg. 1).
 * Duplicated keys are answered per position (a missing key occurring 5 times gives 5 entries).
 * keys [device, n int64]; out [device, n*dim fp32]; miss_idx [device, n uint32];
 * miss_keys [device, n int64]; n_miss [device, 1 uint32] receives the number of entries.
 * Entries appear in no particular order; entries past *n_miss are unspecified.
 * n may be 0 (then *n_miss = 0); n must be < 2^32.
 * Errors: INVALID_ARG (null handle, null/misaligned pointer with n > 0, n too large), DEVICE.
 */
hps_status_t hps_cache_query(hps_cache_t *cache, const int64_t *keys, size_t n,
                             float *out, uint32_t *miss_idx, int64_t *miss_keys,
                             uint32_t *n_miss, void *stream);

/*
 * Insert / replace (Sec. 4.2 "Replace", Alg. 3).  For every i < n: a key that is already
 * cached is ignored; a new key takes the slot `victim_counter[set] mod ways` of its set and
 * advances that counter, which fills empty slots first and afterwards overwrites in
 * insertion order (this build's replacement rule; the paper's is LRU by access counter).
 * Among duplicates of one new key exactly one is stored.  The order in which the keys of a
 * batch take effect is unspecified; it matters only when new keys overwrite slots whose keys
 * occur in the same batch, or when more than `ways` new keys of a batch share a set.
 * keys [device, n int64]; vals [device, n*dim fp32].
 */
hps_status_t hps_cache_insert(hps_cache_t *cache, const int64_t *keys, const float *vals,
                              size_t n, void *stream);

/*
 * Update (Sec. 4.2 "Update", Alg. 4; the last hop of the refresh cycle of Sec. 6): for every
 * i < n whose key is cached, overwrite its row with vals[i]; other keys are ignored.
 * Residency and victim counters never change.  When a key occurs several times in a batch,
 * one of its rows ends up stored, intact.
 */
hps_status_t hps_cache_update(hps_cache_t *cache, const int64_t *keys, const float *vals,
                              size_t n, void *stream);

/* Message for the last error on this thread ("" if none). */
const char *hps_last_error(void);

/* ---- Additions beyond the five calls of the problem statement ------------------------- */

/*
 * Declare whether insert/update calls on OTHER streams may overlap queries (Sec. 4.2 allows
 * concurrent invocation of all APIs).  enabled = 1 (the default): queries validate each row
 * they return against the set's sequence word and re-read rows that a writer touched
 * meanwhile, so a reader sees the old or the new row and never a mixture.  enabled = 0: the
 * caller promises that no writer overlaps a query; queries then use plain cached loads.
 * Takes effect for calls enqueued afterwards.  Rows longer than 4 KiB (dim > 1024) cannot be
 * validated in one piece: such a cache is created with enabled = 0 and enabling returns
 * HPS_ERR_INVALID_ARG.  With enabled = 1 a query that overlaps an insert never writes any part
 * of the `out` row of a position it reports as missing.
 */
hps_status_t hps_cache_set_concurrent_writers(hps_cache_t *cache, int enabled);

/*
 * Deduplicate the keys of each query tile before the lookup (the paper applies a dedup operator
 * to every batch before any lookup, Sec. 2.2).  enabled = 1: plain-mode queries
 * (set_concurrent_writers(0)) elect one representative per distinct key of a 256- or 512-key
 * tile in LDS, probe and read each distinct row once and fan it out to the duplicate positions.
 * Results are identical.  Default 0: on MI355X the duplicate reads of a Zipf batch already hit
 * in L2, and the extra LDS rounds cost more than they save (measured 29 us vs 18 us per batch).
 */
hps_status_t hps_cache_set_query_dedup(hps_cache_t *cache, int enabled);

/*
 * Flag word of a cache, raised by kernels (not a paper call; for callers that cannot tolerate a
 * silent skip).  HPS_FLAG_STUCK_SET: a kernel waited about a second for a set that a writer never
 * released (the writer's kernel must have died) and gave up: the query reported the affected keys
 * as misses, insert/update skipped them.  *flags [host] receives the bits; clear != 0 resets them.
 * Synchronous on the host; call it after synchronising the streams whose work is to be covered.
 */
#define HPS_FLAG_STUCK_SET 1u
hps_status_t hps_cache_flags(hps_cache_t *cache, uint32_t *flags, int clear);

/*
 * Test hook: overwrite the sequence word of one set (host-synchronous).  An odd value imitates
 * a writer that died while holding the set, which is how the bounded waits are tested.
 */
hps_status_t hps_cache_debug_set_seq(hps_cache_t *cache, uint64_t set, uint32_t value);

/* Geometry of a cache.  Any output pointer [host] may be NULL. */
hps_status_t hps_cache_info(const hps_cache_t *cache, uint64_t *num_sets, uint32_t *ways,
                            uint32_t *dim);

/*
 * State export / import for tests and checkpoints (the paper's Dump API, Sec. 4.2, is the
 * precedent).  keys [device, sets*ways int64] in [set][way] order, ctr [device, sets uint32],
 * vals [device, sets*ways*dim fp32] or NULL to skip the rows.  Export copies out; import
 * overwrites the whole state (sequence words are reset).  Enqueued on `stream`.
 */
hps_status_t hps_cache_export(hps_cache_t *cache, int64_t *keys, uint32_t *ctr, float *vals,
                              void *stream);
hps_status_t hps_cache_import(hps_cache_t *cache, const int64_t *keys, const uint32_t *ctr,
                              const float *vals, void *stream);

/*
 * LRU caches only: the access stamps (stamps [device, sets*ways uint32], [set][way] order) and
 * the global iteration count g of Alg. 2, which lives in a device word of the cache: the query
 * kernel advances it (so a query captured into a HIP graph advances it on every replay) and the
 * insert kernel reads it.  Export copies it to *g [host] and, for that, waits for `stream`;
 * import sets it in stream order.  Complements hps_cache_export/import.
 */
hps_status_t hps_cache_export_lru(hps_cache_t *cache, uint32_t *stamps, uint32_t *g, void *stream);
hps_status_t hps_cache_import_lru(hps_cache_t *cache, const uint32_t *stamps, uint32_t g, void *stream);

/*
 * Dump (Sec. 4.2 "Dump"; step 2 of the refresh cycle, Sec. 6): write the cached keys of the
 * slot range [first_slot, first_slot + n_slots) compactly to keys_out [device, n_slots int64]
 * and their number to n_out [device, 1 uint32].  Order is unspecified.
 */
hps_status_t hps_cache_dump(hps_cache_t *cache, size_t first_slot, size_t n_slots,
                            int64_t *keys_out, uint32_t *n_out, void *stream);

/*
 * Query several caches in one launch (one table per categorical feature, Sec. 7.1).
 * caches [host, n_tables handles], all with the same dim, n_tables <= HPS_MAX_TABLES.
 * keys [device, n_tables*batch int64] table-major: keys[t*batch + b] goes to caches[t].
 * out [device, n_tables*batch*dim fp32] in the same order.  The miss list holds
 * <t*batch + b, key> pairs; n_tables*batch must be < 2^32.  Otherwise as hps_cache_query.
 */
hps_status_t hps_cache_query_multi(hps_cache_t *const *caches, uint32_t n_tables,
                                   const int64_t *keys, size_t batch, float *out,
                                   uint32_t *miss_idx, int64_t *miss_keys, uint32_t *n_miss,
                                   void *stream);

/*
 * Stand-in for the lower storage tiers (Sec. 5) used by tests and benchmarks: writes the row
 * a backing store would return for each key, element j of key k being
 *   z = mix(k XOR mix(((version << 32) | j) + 0x9E3779B97F4A7C15)),
 *   value = (int(z >> 40) - 2^23) * 2^-23            (mix = splitmix64 finaliser),
 * to rows[i*dim + j] for i < n and, when scatter_idx is not NULL, also to
 * scatter_out[scatter_idx[i]*dim + j] (filling the missing rows of a query result).
 * n_dev [device, 1 uint32] or NULL: when given, only min(n, *n_dev) keys are processed, so a
 * miss list can be consumed without reading its length back to the host.
 * keys [device], rows [device, n*dim fp32] or NULL, scatter_idx [device, n uint32].
 */
hps_status_t hps_backing_fetch(const int64_t *keys, size_t n, const uint32_t *n_dev,
                               uint32_t dim, uint32_t version, float *rows,
                               const uint32_t *scatter_idx, float *scatter_out, void *stream);

/*
 * Variants of insert / update whose batch length is read on the device:
 * min(n_max, *n_dev) keys are processed.  Lets Alg. 1's "insert the missing keys" run without
 * a host round trip for the miss count.
 */
hps_status_t hps_cache_insert_dn(hps_cache_t *cache, const int64_t *keys, const float *vals,
                                 size_t n_max, const uint32_t *n_dev, void *stream);
hps_status_t hps_cache_update_dn(hps_cache_t *cache, const int64_t *keys, const float *vals,
                                 size_t n_max, const uint32_t *n_dev, void *stream);

/*
 * Query (Sec. 4.2, Alg. 2) whose batch length is read on the device: positions
 * 0 .. min(n_max, *n_dev) - 1 are looked up exactly as by hps_cache_query, the others are neither
 * read as keys nor written in `out` nor reported as misses.  keys must be readable up to n_max
 * entries; out / miss_idx / miss_keys are sized for n_max.  Lets a query follow a device-side
 * producer of its keys (the distinct keys of hps_dedup.h, Sec. 2.2) without a host round trip.
 * n_dev [device, one uint32, 4-byte aligned] must not be NULL.
 */
hps_status_t hps_cache_query_dn(hps_cache_t *cache, const int64_t *keys, size_t n_max,
                                const uint32_t *n_dev, float *out, uint32_t *miss_idx,
                                int64_t *miss_keys, uint32_t *n_miss, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* HPS_CACHE_H */
