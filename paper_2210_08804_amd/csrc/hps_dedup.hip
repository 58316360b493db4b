// Deduplication operator Q* = dedup(Q) of the paper's Sec. 2.2 and the row expansion that
// follows the lookup of Q*, for gfx950.
//
// dedup is a hash join of the batch with itself in two launches over an open-addressing table
// (one 8-byte key word per slot, 2n..4n slots).  A session has two tables: a call works on the
// clean one, and its second launch wipes the part of the other one that the previous call used,
// so no call waits for a clear.
//   insert   a work-group takes 1024 keys, elects one lane per distinct key of the tile in an
//            LDS table (so a hot key reaches the global table once per tile, not once per
//            occurrence), the elected lanes claim a slot of the global table with a 64-bit
//            compare-and-swap, the lanes whose swap succeeded are numbered (one global counter
//            atomic per tile) and write their key to unique_keys and their number beside the slot;
//   inverse  every position finds its key's slot again and reads the number; the same launch
//            clears the other table for the next call.
// The order of unique_keys is the order in which tiles reach the counter: unspecified.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <mutex>
#include <new>
#include <string>

#include "hps_dedup.h"
#include "hps_mix.h"

namespace {

constexpr int64_t  kEmpty = INT64_MIN;            // free slot of both hash tables
constexpr int      kBlock = 256;
constexpr int      kTile  = 1024;                 // keys (= threads) per work-group of the insert kernel
constexpr int      kLds   = 2 * kTile;            // LDS table slots (load <= 0.5)
constexpr uint64_t kMagic = 0x4850534445445550ull;
constexpr uint32_t kNone  = 0xFFFFFFFFu;

typedef float f32x4 __attribute__((ext_vector_type(4)));

// Scratch of hps_dedup_noalloc, the entry point for callers that cannot allocate: one hash table
// for batches of up to kNaMaxKeys keys (2 slots per key, 8-byte key word + 4-byte number per
// slot, one extra slot for the key that equals the free marker) and its counter words, in a
// static device array (3 MiB that every GPU the library runs on holds until the process ends).
constexpr uint32_t kNaMaxKeys  = HPS_DEDUP_NOALLOC_MAX;
constexpr uint32_t kNaSlots    = 2 * kNaMaxKeys;                        // a power of two
constexpr size_t   kNaKeyBytes = (((size_t)kNaSlots + 1) * 8 + 255) / 256 * 256;
constexpr size_t   kNaUidBytes = (((size_t)kNaSlots + 1) * 4 + 255) / 256 * 256;
constexpr size_t   kNaBytes    = kNaKeyBytes + kNaUidBytes + 256;       // + two counter words
static_assert((kNaSlots & (kNaSlots - 1)) == 0, "slot count must be a power of two");
static __device__ __align__(256) unsigned char scratch[kNaBytes];

constexpr int kNaMaxDevices = 64;
std::mutex g_na_mu;
unsigned char *g_na_ptr[kNaMaxDevices];          // device address of `scratch` on each device, once known

thread_local std::string g_err;

hps_status_t fail(hps_status_t code, const std::string &msg) {
    g_err = msg;
    return code;
}

#define HIP_TRY(expr)                                                                   \
    do {                                                                                \
        hipError_t e_ = (expr);                                                         \
        if (e_ != hipSuccess)                                                           \
            return fail(e_ == hipErrorOutOfMemory ? HPS_ERR_OOM : HPS_ERR_DEVICE,        \
                        std::string(#expr) + ": " + hipGetErrorString(e_));              \
    } while (0)

bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

// The table has slots 0..mask for ordinary keys and slot mask + 1 for the key whose value is the
// free-slot marker itself.
// (used once per table, when the session is created)
__global__ void dedup_clear_kernel(int64_t *tkey, uint64_t n_slots, uint32_t *counter) {
    const uint64_t t = blockIdx.x * (uint64_t)blockDim.x + threadIdx.x;
    for (uint64_t i = t; i < n_slots; i += (uint64_t)gridDim.x * blockDim.x) tkey[i] = kEmpty;
    if (t == 0) *counter = 0u;
}

__global__ void set_u32_kernel(uint32_t *p, uint32_t v) { *p = v; }

__global__ void __launch_bounds__(kTile) dedup_insert_kernel(const int64_t *__restrict__ keys, uint32_t n,
                                                             int64_t *tkey, uint32_t *tuid, uint32_t mask,
                                                             uint32_t *counter, int64_t *unique_keys) {
    __shared__ unsigned long long l_key[kLds];
    __shared__ uint32_t l_marker_seen, l_cnt, l_base;

    const uint32_t n_tiles = (n + kTile - 1) / kTile;
    for (uint32_t tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        for (uint32_t i = threadIdx.x; i < (uint32_t)kLds; i += kTile) l_key[i] = (unsigned long long)kEmpty;
        if (threadIdx.x == 0) {
            l_marker_seen = 0u;
            l_cnt = 0u;
        }
        __syncthreads();

        const uint32_t i = tile * kTile + threadIdx.x;
        const bool live = i < n;
        const int64_t key = live ? keys[i] : 0;
        // one lane per distinct key of the tile goes on
        bool elected = false;
        if (live) {
            if (key == kEmpty) {
                elected = atomicCAS(&l_marker_seen, 0u, 1u) == 0u;
            } else {
                uint32_t ls = (uint32_t)(mix64((uint64_t)key) >> 40) & (kLds - 1);
                for (;;) {
                    const unsigned long long old =
                        atomicCAS(&l_key[ls], (unsigned long long)kEmpty, (unsigned long long)key);
                    if (old == (unsigned long long)kEmpty) { elected = true; break; }
                    if (old == (unsigned long long)key) break;
                    ls = (ls + 1) & (kLds - 1);                // at most 1024 of 2048 slots are ever taken
                }
            }
        }
        // the elected lane claims the key's slot of the global table
        bool won = false;
        uint32_t slot = 0u;
        if (elected) {
            if (key == kEmpty) {
                slot = mask + 1u;
                won = atomicCAS(reinterpret_cast<unsigned long long *>(tkey + slot),
                                (unsigned long long)kEmpty, 0ull) == (unsigned long long)kEmpty;
            } else {
                uint32_t gs = (uint32_t)mix64((uint64_t)key) & mask;
                for (uint32_t probe = 0; probe <= mask; ++probe) {      // the table is at most half full
                    const int64_t cur = __hip_atomic_load(tkey + gs, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    if (cur == key) break;                               // another tile listed it
                    if (cur == kEmpty) {
                        const unsigned long long old =
                            atomicCAS(reinterpret_cast<unsigned long long *>(tkey + gs),
                                      (unsigned long long)kEmpty, (unsigned long long)key);
                        if (old == (unsigned long long)kEmpty) { won = true; break; }
                        if (old == (unsigned long long)key) break;
                    }
                    gs = (gs + 1) & mask;
                }
                slot = gs;
            }
        }
        const uint32_t rank = won ? atomicAdd(&l_cnt, 1u) : kNone;
        __syncthreads();
        if (threadIdx.x == 0) l_base = l_cnt ? atomicAdd(counter, l_cnt) : 0u;
        __syncthreads();
        if (won) {
            const uint32_t uid = l_base + rank;
            unique_keys[uid] = key;
            tuid[slot] = uid;
        }
        __syncthreads();                                              // LDS is reused by the next tile
    }
}

__global__ void __launch_bounds__(kBlock) dedup_inverse_kernel(const int64_t *__restrict__ keys, uint32_t n,
                                                               const int64_t *__restrict__ tkey,
                                                               const uint32_t *__restrict__ tuid, uint32_t mask,
                                                               const uint32_t *__restrict__ counter,
                                                               uint32_t *inverse, uint32_t *n_unique,
                                                               int64_t *other_tkey, uint64_t other_dirty,
                                                               uint32_t *other_counter) {
    const uint64_t t = blockIdx.x * (uint64_t)blockDim.x + threadIdx.x;
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    if (t == 0) {
        *n_unique = *counter;
        *other_counter = 0u;
    }
    for (uint64_t i = t; i < n; i += stride) {
        const int64_t key = keys[i];
        uint32_t gs = mask + 1u;
        if (key != kEmpty) {
            gs = (uint32_t)mix64((uint64_t)key) & mask;
            for (uint32_t probe = 0; probe <= mask && tkey[gs] != key; ++probe) gs = (gs + 1) & mask;
        }
        inverse[i] = tuid[gs];
    }
    // the slots the previous call used in the other table
    for (uint64_t i = t; i < other_dirty; i += stride) other_tkey[i] = kEmpty;
}

// out[i] = rows[inverse[i]].  LPR lanes move one row, 16 bytes per lane; four rows per lane group
// are in flight before the first store.  Lanes past the end repeat the last row (same bytes to
// the same place), lanes past the row's last chunk repeat chunk 0.
__global__ void __launch_bounds__(kBlock) expand_rows_kernel(const float *__restrict__ rows,
                                                             const uint32_t *__restrict__ inverse, uint32_t n,
                                                             uint32_t d, uint32_t C, uint32_t LPR, uint32_t lprShift,
                                                             uint32_t passes, float *__restrict__ out) {
    constexpr int U = 4;
    const uint32_t rpb = (uint32_t)kBlock >> lprShift;                // rows per block and step
    const uint32_t sub = threadIdx.x >> lprShift;
    const uint32_t cl  = threadIdx.x & (LPR - 1);
    for (uint64_t r0 = (uint64_t)blockIdx.x * rpb * U; r0 < n; r0 += (uint64_t)gridDim.x * rpb * U) {
        uint32_t src[U], dst[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint64_t r = r0 + (uint64_t)u * rpb + sub;
            dst[u] = r < n ? (uint32_t)r : n - 1u;
            src[u] = inverse[dst[u]];
        }
        for (uint32_t pass = 0; pass < passes; ++pass) {
            uint32_t chunk = cl + pass * LPR;
            chunk = chunk < C ? chunk : 0u;
            f32x4 buf[U];
#pragma unroll
            for (int u = 0; u < U; ++u)
                buf[u] = *reinterpret_cast<const f32x4 *>(rows + (uint64_t)src[u] * d + chunk * 4);
#pragma unroll
            for (int u = 0; u < U; ++u)
                __builtin_nontemporal_store(buf[u], reinterpret_cast<f32x4 *>(out + (uint64_t)dst[u] * d + chunk * 4));
        }
    }
}

}  // namespace

struct hps_dedup_session {
    uint64_t  magic;
    int       device;
    size_t    max_n;
    uint64_t  slots;        // power of two >= 2 * max_n (>= 1024); one more slot follows them
    int64_t  *tkey[3];      // [slots + 1] each; a call works on tkey[cur] (0 or 1), which is all free;
                            // table 2 serves calls that are being captured into a graph (see hps_dedup)
    uint32_t *tuid[3];      // [slots + 1] each
    uint32_t *counter;      // one word per table (zero for the table in turn) and a spare one
    uint64_t  dirty[2];     // leading slots of each table that a call has written and nobody cleared yet
    int       cur;
    int       n_cus;
};

namespace {

hps_status_t check_session(hps_dedup_session *s) {
    if (!s || s->magic != kMagic) return fail(HPS_ERR_INVALID_ARG, "not a live dedup session");
    int dev = -1;
    HIP_TRY(hipGetDevice(&dev));
    if (dev != s->device) return fail(HPS_ERR_INVALID_ARG, "session belongs to another device than the current one");
    return HPS_OK;
}

uint64_t pow2_at_least(uint64_t x) {
    uint64_t p = 1024;
    while (p < x) p <<= 1;
    return p;
}

}  // namespace

extern "C" {

const char *hps_dedup_last_error(void) { return g_err.c_str(); }

hps_status_t hps_dedup_create(size_t max_n, hps_dedup_t **out) {
    if (!out) return fail(HPS_ERR_INVALID_ARG, "out must not be NULL");
    *out = nullptr;
    // 2 * max_n slots must stay below 2^32: slot numbers, the mask and the extra slot behind the table are 32-bit
    if (max_n == 0 || max_n > (1ull << 30)) return fail(HPS_ERR_INVALID_ARG, "max_n must be in 1 .. 2^30");
    hps_dedup_session *s = new (std::nothrow) hps_dedup_session();
    if (!s) return fail(HPS_ERR_OOM, "host allocation failed");
    s->magic = 0;
    s->max_n = max_n;
    s->slots = pow2_at_least(2 * (uint64_t)max_n);
    s->tkey[0] = s->tkey[1] = s->tkey[2] = nullptr;
    s->tuid[0] = s->tuid[1] = s->tuid[2] = nullptr;
    s->counter = nullptr;
    s->dirty[0] = s->dirty[1] = 0;
    s->cur = 0;
    s->n_cus = 256;
    hipError_t e = hipGetDevice(&s->device);
    if (e == hipSuccess) e = hipDeviceGetAttribute(&s->n_cus, hipDeviceAttributeMultiprocessorCount, s->device);
    if (e == hipSuccess && s->n_cus <= 0) s->n_cus = 256;
    for (int t = 0; t < 3; ++t) {
        if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void **>(&s->tkey[t]), (s->slots + 1) * sizeof(int64_t));
        if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void **>(&s->tuid[t]), (s->slots + 1) * sizeof(uint32_t));
    }
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void **>(&s->counter), 256);
    for (int t = 0; t < 3 && e == hipSuccess; ++t) {
        hipLaunchKernelGGL(dedup_clear_kernel, dim3(4096), dim3(kBlock), 0, 0, s->tkey[t], s->slots + 1, s->counter + t);
        e = hipGetLastError();
    }
    if (e == hipSuccess) e = hipStreamSynchronize(0);
    if (e != hipSuccess) {
        for (int t = 0; t < 3; ++t) {
            (void)hipFree(s->tkey[t]);
            (void)hipFree(s->tuid[t]);
        }
        (void)hipFree(s->counter);
        delete s;
        (void)hipGetLastError();
        return fail(e == hipErrorOutOfMemory ? HPS_ERR_OOM : HPS_ERR_DEVICE,
                    std::string("hps_dedup_create: ") + hipGetErrorString(e));
    }
    s->magic = kMagic;
    *out = s;
    return HPS_OK;
}

hps_status_t hps_dedup_destroy(hps_dedup_t *s) {
    if (!s) return HPS_OK;
    if (s->magic != kMagic) return fail(HPS_ERR_INVALID_ARG, "not a live dedup session");
    int prev = -1;
    HIP_TRY(hipGetDevice(&prev));
    HIP_TRY(hipSetDevice(s->device));
    hipError_t e = hipDeviceSynchronize();
    for (int t = 0; t < 3; ++t) {
        (void)hipFree(s->tkey[t]);
        (void)hipFree(s->tuid[t]);
    }
    (void)hipFree(s->counter);
    s->magic = 0;
    delete s;
    (void)hipSetDevice(prev);
    if (e != hipSuccess) return fail(HPS_ERR_DEVICE, std::string("hipDeviceSynchronize: ") + hipGetErrorString(e));
    return HPS_OK;
}

hps_status_t hps_dedup(hps_dedup_t *s, const int64_t *keys, size_t n, int64_t *unique_keys,
                       uint32_t *inverse, uint32_t *n_unique, void *stream) {
    if (hps_status_t st = check_session(s)) return st;
    if (!n_unique || !aligned(n_unique, 4)) return fail(HPS_ERR_INVALID_ARG, "n_unique must be a 4-byte aligned device pointer");
    if (n > s->max_n) return fail(HPS_ERR_INVALID_ARG, "n exceeds the session's max_n");
    hipStream_t q = static_cast<hipStream_t>(stream);
    if (n == 0) {
        hipLaunchKernelGGL(set_u32_kernel, dim3(1), dim3(1), 0, q, n_unique, 0u);
        HIP_TRY(hipGetLastError());
        return HPS_OK;
    }
    if (!keys || !unique_keys || !inverse) return fail(HPS_ERR_INVALID_ARG, "keys, unique_keys and inverse must not be NULL when n > 0");
    if (!aligned(keys, 8) || !aligned(unique_keys, 8) || !aligned(inverse, 4))
        return fail(HPS_ERR_INVALID_ARG, "keys and unique_keys must be 8-byte, inverse 4-byte aligned");
    const uint64_t slots = pow2_at_least(2 * (uint64_t)n);            // <= s->slots because n <= max_n
    const uint32_t mask = (uint32_t)(slots - 1);
    const uint32_t cap = (uint32_t)s->n_cus * 8u;
    const uint64_t tiles = (n + kTile - 1) / kTile;
    // A call that is being captured into a graph must be complete in itself, because the graph may
    // be replayed any number of times between other calls: it clears its own table (the third
    // one, which no other call touches) first and leaves the two alternating tables alone.
    hipStreamCaptureStatus cap_status = hipStreamCaptureStatusNone;
    HIP_TRY(hipStreamIsCapturing(q, &cap_status));
    if (cap_status != hipStreamCaptureStatusNone) {
        const uint64_t cb = (slots + 1 + kBlock - 1) / kBlock;
        hipLaunchKernelGGL(dedup_clear_kernel, dim3((uint32_t)(cb < cap ? cb : cap)), dim3(kBlock), 0, q,
                           s->tkey[2], slots + 1, s->counter + 2);
        hipLaunchKernelGGL(dedup_insert_kernel, dim3((uint32_t)(tiles < cap ? tiles : cap)), dim3(kTile), 0, q,
                           keys, (uint32_t)n, s->tkey[2], s->tuid[2], mask, s->counter + 2, unique_keys);
        const uint64_t ib2 = (n + kBlock - 1) / kBlock;
        hipLaunchKernelGGL(dedup_inverse_kernel, dim3((uint32_t)(ib2 < 4 * cap ? ib2 : 4 * cap)), dim3(kBlock), 0, q,
                           keys, (uint32_t)n, s->tkey[2], s->tuid[2], mask, s->counter + 2, inverse, n_unique,
                           s->tkey[2], (uint64_t)0, s->counter + 3);
        HIP_TRY(hipGetLastError());
        return HPS_OK;
    }
    const int t = s->cur, o = 1 - t;
    hipLaunchKernelGGL(dedup_insert_kernel, dim3((uint32_t)(tiles < cap ? tiles : cap)), dim3(kTile), 0, q,
                       keys, (uint32_t)n, s->tkey[t], s->tuid[t], mask, s->counter + t, unique_keys);
    const uint64_t work = n > s->dirty[o] ? n : s->dirty[o];
    const uint64_t ib = (work + kBlock - 1) / kBlock;
    hipLaunchKernelGGL(dedup_inverse_kernel, dim3((uint32_t)(ib < 4 * cap ? ib : 4 * cap)), dim3(kBlock), 0, q,
                       keys, (uint32_t)n, s->tkey[t], s->tuid[t], mask, s->counter + t, inverse, n_unique,
                       s->tkey[o], s->dirty[o], s->counter + o);
    HIP_TRY(hipGetLastError());
    s->dirty[t] = slots + 1;          // this call's slots, the extra one included
    s->dirty[o] = 0;
    s->cur = o;
    return HPS_OK;
}

hps_status_t hps_dedup_noalloc(const int64_t *keys, size_t n, int64_t *unique_keys, uint32_t *inverse,
                               uint32_t *n_unique, void *stream) {
    if (!n_unique || !aligned(n_unique, 4)) return fail(HPS_ERR_INVALID_ARG, "n_unique must be a 4-byte aligned device pointer");
    if (n > kNaMaxKeys)
        return fail(HPS_ERR_INVALID_ARG, "hps_dedup_noalloc takes at most " + std::to_string(kNaMaxKeys) +
                                             " keys per call (its table is a fixed static array); use a session of hps_dedup for more");
    hipStream_t q = static_cast<hipStream_t>(stream);
    if (n == 0) {
        hipLaunchKernelGGL(set_u32_kernel, dim3(1), dim3(1), 0, q, n_unique, 0u);
        HIP_TRY(hipGetLastError());
        return HPS_OK;
    }
    if (!keys || !unique_keys || !inverse) return fail(HPS_ERR_INVALID_ARG, "keys, unique_keys and inverse must not be NULL when n > 0");
    if (!aligned(keys, 8) || !aligned(unique_keys, 8) || !aligned(inverse, 4))
        return fail(HPS_ERR_INVALID_ARG, "keys and unique_keys must be 8-byte, inverse 4-byte aligned");
    // The array's name is only a host-side stand-in: its device address is asked for once per
    // device (each GPU holds its own copy at its own address) and used from then on.
    int dev = -1;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kNaMaxDevices) return fail(HPS_ERR_INVALID_ARG, "device number beyond what hps_dedup_noalloc keeps track of");
    unsigned char *base = nullptr;
    {
        std::lock_guard<std::mutex> lk(g_na_mu);
        if (!g_na_ptr[dev]) {
            void *p = nullptr;
            HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
            if (!p) return fail(HPS_ERR_DEVICE, "hipGetSymbolAddress returned no address for the scratch array");
            g_na_ptr[dev] = static_cast<unsigned char *>(p);
        }
        base = g_na_ptr[dev];
    }
    int64_t  *tkey    = reinterpret_cast<int64_t *>(base);
    uint32_t *tuid    = reinterpret_cast<uint32_t *>(base + kNaKeyBytes);
    uint32_t *counter = reinterpret_cast<uint32_t *>(base + kNaKeyBytes + kNaUidBytes);
    int n_cus = 0;
    HIP_TRY(hipDeviceGetAttribute(&n_cus, hipDeviceAttributeMultiprocessorCount, dev));
    if (n_cus <= 0) n_cus = 256;
    const uint64_t slots = pow2_at_least(2 * (uint64_t)n);            // <= kNaSlots because n <= kNaMaxKeys
    const uint32_t mask = (uint32_t)(slots - 1);
    const uint32_t cap = (uint32_t)n_cus * 8u;
    const uint64_t tiles = (n + kTile - 1) / kTile;
    // The array keeps what the last call left in it: the slots this call may touch and its counter
    // are cleared first (by a kernel, so that the call can be captured into a graph), then the
    // same two launches as hps_dedup.
    const uint64_t cb = (slots + 1 + kBlock - 1) / kBlock;
    hipLaunchKernelGGL(dedup_clear_kernel, dim3((uint32_t)(cb < cap ? cb : cap)), dim3(kBlock), 0, q, tkey, slots + 1, counter);
    hipLaunchKernelGGL(dedup_insert_kernel, dim3((uint32_t)(tiles < cap ? tiles : cap)), dim3(kTile), 0, q,
                       keys, (uint32_t)n, tkey, tuid, mask, counter, unique_keys);
    const uint64_t ib = (n + kBlock - 1) / kBlock;
    hipLaunchKernelGGL(dedup_inverse_kernel, dim3((uint32_t)(ib < 4 * cap ? ib : 4 * cap)), dim3(kBlock), 0, q,
                       keys, (uint32_t)n, tkey, tuid, mask, counter, inverse, n_unique, tkey, (uint64_t)0, counter + 1);
    HIP_TRY(hipGetLastError());
    return HPS_OK;
}

hps_status_t hps_expand_rows(const float *rows, const uint32_t *inverse, size_t n, uint32_t dim,
                             float *out, void *stream) {
    if (dim == 0 || dim % 4 != 0) return fail(HPS_ERR_INVALID_ARG, "dim must be a non-zero multiple of 4");
    if (n == 0) return HPS_OK;
    if (n >= (1ull << 32)) return fail(HPS_ERR_INVALID_ARG, "n must be < 2^32");
    if (!rows || !inverse || !out) return fail(HPS_ERR_INVALID_ARG, "rows, inverse and out must not be NULL when n > 0");
    if (!aligned(rows, 16) || !aligned(out, 16) || !aligned(inverse, 4))
        return fail(HPS_ERR_INVALID_ARG, "rows and out must be 16-byte, inverse 4-byte aligned");
    const uint32_t C = dim / 4;
    uint32_t LPR = 1, shift = 0;
    while (LPR < C && LPR < 64) {
        LPR <<= 1;
        ++shift;
    }
    const uint32_t passes = (C + LPR - 1) / LPR;
    const uint64_t rows_per_block = ((uint64_t)kBlock >> shift) * 4;
    uint64_t blocks = (n + rows_per_block - 1) / rows_per_block;
    if (blocks > (1u << 16)) blocks = 1u << 16;
    hipLaunchKernelGGL(expand_rows_kernel, dim3((uint32_t)blocks), dim3(kBlock), 0, static_cast<hipStream_t>(stream),
                       rows, inverse, (uint32_t)n, dim, C, LPR, shift, passes, out);
    HIP_TRY(hipGetLastError());
    return HPS_OK;
}

}  // extern "C"
