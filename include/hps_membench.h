/*
 * hps_membench.h - measurement kernels, not part of the cache: what the memory system of the GPU
 * delivers for the byte movement of a query with everything else taken away.  The benchmark sets
 * their times beside the query kernel's (the query of Alg. 2 must hash, probe and compact misses
 * before and while it moves the same rows).
 *
 * All pointers are device pointers on the current device, 16-byte aligned; `stream` is a
 * hipStream_t passed as void* (NULL = the null stream); calls only enqueue one kernel.  Status
 * codes are those of hps_cache.h; the message of a failing call is returned by hps_last_error().
 */
#ifndef HPS_MEMBENCH_H
#define HPS_MEMBENCH_H

#include <stddef.h>
#include <stdint.h>

#include "hps_cache.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * The row movement of a query batch alone (Alg. 2 without hashing, probing and the miss list):
 * out[i] = rows[slot_of[i]] for every i < n whose slot_of[i] is not 0xFFFFFFFF.  Same work
 * distribution and copy loop as the query kernel (16 bytes per lane, non-temporal stores).
 *   rows    [n_rows][dim] fp32, read only     slot_of  uint32 [n], each < n_rows or 0xFFFFFFFF
 *   out     [n][dim] fp32
 * dim a non-zero multiple of 4; n < 2^32.
 */
hps_status_t hps_membench_gather(const float *rows, const uint32_t *slot_of, size_t n, uint32_t dim,
                                 float *out, void *stream);

/*
 * One half of that row movement at dim = 128 (512-byte rows), same work distribution and group
 * size: reads != 0 loads the rows rows[slot_of[i]] and stores nothing; reads == 0 loads nothing and
 * stores a register pattern to the rows out[i] of the same positions.  Their two times beside the
 * time of both together show how far reads and writes share the memory system's time.
 */
hps_status_t hps_membench_gather_half(const float *rows, const uint32_t *slot_of, size_t n, float *out,
                                      int reads, void *stream);

/*
 * Streaming copy of `bytes` (a multiple of 16) from src to dst, 16 bytes per lane, several loads
 * in flight per lane; nontemporal != 0 marks loads and stores as streaming.
 */
hps_status_t hps_membench_copy(const void *src, void *dst, size_t bytes, int nontemporal, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* HPS_MEMBENCH_H */
