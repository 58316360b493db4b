// Algorithm 1 of the paper (embedding cache insertion: hit-rate test, synchronous or asynchronous
// fill) and the cache refresh cycle of its Sec. 6, on top of the C ABI of the cache and of the
// dedup operator.  Host orchestration plus one small kernel; the lower tiers are a caller-supplied
// fetch callback working on pinned host buffers.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <condition_variable>
#include <cstdint>
#include <cstring>
#include <deque>
#include <mutex>
#include <new>
#include <string>
#include <thread>
#include <vector>

#include "hps_dedup.h"
#include "hps_lookup.h"

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));

// out[idx[j]] = rows[src[j]] for j < m (src == nullptr: rows[0], the default vector).
__global__ void place_rows_kernel(float *out, const uint32_t *__restrict__ idx,
                                  const uint32_t *__restrict__ src, const float *__restrict__ rows,
                                  uint32_t m, uint32_t d) {
    const uint32_t C = d / 4;
    const uint64_t total = (uint64_t)m * C;
    for (uint64_t t = blockIdx.x * (uint64_t)blockDim.x + threadIdx.x; t < total;
         t += (uint64_t)gridDim.x * blockDim.x) {
        const uint32_t j = (uint32_t)(t / C);
        const uint32_t c = (uint32_t)(t - (uint64_t)j * C);
        const uint64_t r = src ? src[j] : 0u;
        const f32x4 v = *reinterpret_cast<const f32x4 *>(rows + r * d + c * 4);
        *reinterpret_cast<f32x4 *>(out + (uint64_t)idx[j] * d + c * 4) = v;
    }
}

// Asynchronous insertions that may wait for the background thread: each waits in one of the
// object's slots (a device key buffer of max_batch keys and an event, all allocated at create, so
// that a lookup call allocates nothing).  There are at most 66 slots (64 waiting batches plus what
// the background thread is working on) and at most 256 MiB of them (never fewer than 2).  When every slot is taken the oldest waiting batch is dropped: cache
// insertion is best effort, its keys stay missing until a later batch asks again.
constexpr size_t kMaxQueued = 64;
constexpr size_t kMaxSlotBytes = 256ull << 20;

struct Slot {
    int64_t   *d_keys;        // device copy of a batch's miss list (every occurrence)
    hipEvent_t ready;         // that copy has finished
};

struct Task {                 // one queued asynchronous insertion
    Slot     *slot;
    uint32_t  m;              // how many keys
};

}  // namespace

struct hps_lookup_session {
    hps_cache_t *cache;
    int          device;
    size_t       max_batch;
    uint32_t     dim;
    float        threshold;
    hps_fetch_fn fetch;
    void        *user;
    hps_dedup_t *dd;          // dedup of the miss list before it leaves the device (Sec. 2.2)
    hps_dedup_t *dd_bg;       // the same for the background thread (its calls run on the side stream)
    // workspace (the paper's ws): device side
    uint32_t *d_miss_idx, *d_n_miss, *d_inv, *d_n_unique;
    int64_t  *d_miss_keys, *d_ukeys;
    float    *d_rows, *d_default;
    // pinned host side
    uint32_t *h_n_miss, *h_n_unique;
    int64_t  *h_ukeys;
    float    *h_rows;
    // background insertion
    hipStream_t side;
    int64_t  *bg_d_ukeys, *bg_d_keys, *bg_h_keys;
    uint32_t *bg_d_inv, *bg_d_n_unique, *bg_h_n_unique;
    float    *bg_d_rows, *bg_h_rows;
    std::thread worker;
    std::mutex mu;
    std::condition_variable cv, cv_idle;
    std::deque<Task> queue;
    std::vector<Slot> slots;              // all of them, for destruction
    std::vector<Slot *> free_slots;
    bool stop = false, busy = false;
    std::string worker_error;
};

struct hps_refresh_session {              // buffers, stream and events of the refresh cycle (Sec. 6)
    hps_cache_t *cache = nullptr;
    int          device = 0;
    uint64_t     slots = 0;               // slots of the cache
    size_t       B = 0;                   // slots per batch
    size_t       rowb = 0;                // bytes per row
    int64_t     *d_keys[2] = {nullptr, nullptr}, *h_keys[2] = {nullptr, nullptr};
    float       *d_rows[2] = {nullptr, nullptr}, *h_rows[2] = {nullptr, nullptr};
    uint32_t    *d_cnt = nullptr, *h_cnt = nullptr;
    hipStream_t  s2 = nullptr;            // dump and key download run here
    hipEvent_t   applied[2] = {nullptr, nullptr};
};

namespace {

thread_local std::string g_lookup_err;

hps_status_t lfail(hps_status_t code, const std::string &msg) {
    g_lookup_err = msg;
    return code;
}

#define LK_TRY(expr)                                                                         \
    do {                                                                                     \
        hipError_t e_ = (expr);                                                              \
        if (e_ != hipSuccess)                                                                \
            return lfail(e_ == hipErrorOutOfMemory ? HPS_ERR_OOM : HPS_ERR_DEVICE,            \
                         std::string(#expr) + ": " + hipGetErrorString(e_));                 \
    } while (0)

void launch_place(float *out, const uint32_t *idx, const uint32_t *src, const float *rows, uint32_t m,
                  uint32_t d, hipStream_t st) {
    const uint64_t total = (uint64_t)m * (d / 4);
    uint64_t blocks = (total + 255) / 256;
    if (blocks > (1u << 16)) blocks = 1u << 16;
    hipLaunchKernelGGL(place_rows_kernel, dim3((uint32_t)blocks), dim3(256), 0, st, out, idx, src, rows, m, d);
}

// Background thread: the asyncInsert procedure of Alg. 1 (lower-tier lookup, then insert).
void worker_main(hps_lookup_session *L) {
    (void)hipSetDevice(L->device);
    std::vector<Task> batch;
    for (;;) {
        batch.clear();
        {
            std::unique_lock<std::mutex> lk(L->mu);
            L->cv.wait(lk, [&] { return L->stop || !L->queue.empty(); });
            if (L->queue.empty()) return;                      // stop requested and nothing left
            // Everything that has queued up goes in one round (as long as it fits the buffers):
            // when the lower tier is slower than the callers, the backlog stays bounded and keys
            // that several queued batches ask for are fetched once.
            size_t total = 0;
            while (!L->queue.empty() && (batch.empty() || total + L->queue.front().m <= L->max_batch)) {
                total += L->queue.front().m;
                batch.push_back(L->queue.front());
                L->queue.pop_front();
            }
            L->busy = true;
        }
        std::string err;
        hipError_t e = hipSuccess;
        // the queued miss lists, one after the other in one device buffer, then made distinct
        uint32_t total = 0;
        for (const Task &t : batch) {
            if (e == hipSuccess) e = hipStreamWaitEvent(L->side, t.slot->ready, 0);
            if (e == hipSuccess)
                e = hipMemcpyAsync(L->bg_d_keys + total, t.slot->d_keys, (size_t)t.m * sizeof(int64_t),
                                   hipMemcpyDeviceToDevice, L->side);
            total += t.m;
        }
        if (e == hipSuccess &&
            hps_dedup(L->dd_bg, L->bg_d_keys, total, L->bg_d_ukeys, L->bg_d_inv, L->bg_d_n_unique, L->side) != HPS_OK)
            err = std::string("background dedup: ") + hps_dedup_last_error();
        if (e == hipSuccess) e = hipMemcpyAsync(L->bg_h_n_unique, L->bg_d_n_unique, 4, hipMemcpyDeviceToHost, L->side);
        if (e == hipSuccess)
            e = hipMemcpyAsync(L->bg_h_keys, L->bg_d_ukeys, (size_t)total * sizeof(int64_t), hipMemcpyDeviceToHost, L->side);
        if (e == hipSuccess) e = hipStreamSynchronize(L->side);
        if (e == hipSuccess && err.empty()) {
            const uint32_t u = *L->bg_h_n_unique;
            L->fetch(L->user, L->bg_h_keys, u, L->bg_h_rows);
            e = hipMemcpyAsync(L->bg_d_rows, L->bg_h_rows, (size_t)u * L->dim * sizeof(float),
                               hipMemcpyHostToDevice, L->side);
            if (e == hipSuccess && hps_cache_insert(L->cache, L->bg_d_ukeys, L->bg_d_rows, u, L->side) != HPS_OK)
                err = std::string("background insert: ") + hps_last_error();
            if (e == hipSuccess) e = hipStreamSynchronize(L->side);
        }
        if (e != hipSuccess) err = std::string("background insertion: ") + hipGetErrorString(e);
        if (e != hipSuccess || !err.empty()) (void)hipStreamSynchronize(L->side);   // the slots are idle before they go back
        {
            std::lock_guard<std::mutex> lk(L->mu);
            for (const Task &t : batch) L->free_slots.push_back(t.slot);
            if (!err.empty()) L->worker_error = err;
            L->busy = false;
        }
        L->cv_idle.notify_all();
    }
}

void free_all(hps_lookup_session *L) {
    (void)hps_dedup_destroy(L->dd);
    (void)hps_dedup_destroy(L->dd_bg);
    (void)hipFree(L->d_miss_idx); (void)hipFree(L->d_n_miss); (void)hipFree(L->d_inv); (void)hipFree(L->d_n_unique);
    (void)hipFree(L->d_miss_keys); (void)hipFree(L->d_ukeys); (void)hipFree(L->d_rows); (void)hipFree(L->d_default);
    (void)hipFree(L->bg_d_ukeys); (void)hipFree(L->bg_d_rows); (void)hipFree(L->bg_d_keys);
    (void)hipFree(L->bg_d_inv); (void)hipFree(L->bg_d_n_unique); (void)hipHostFree(L->bg_h_n_unique);
    (void)hipHostFree(L->h_n_miss); (void)hipHostFree(L->h_n_unique);
    (void)hipHostFree(L->h_ukeys); (void)hipHostFree(L->h_rows); (void)hipHostFree(L->bg_h_rows);
    (void)hipHostFree(L->bg_h_keys);
    for (Slot &sl : L->slots) {
        if (sl.d_keys) (void)hipFree(sl.d_keys);
        if (sl.ready) (void)hipEventDestroy(sl.ready);
    }
    if (L->side) (void)hipStreamDestroy(L->side);
}

}  // namespace

extern "C" {

hps_status_t hps_lookup_create(hps_cache_t *cache, size_t max_batch, float hit_threshold,
                               const float *default_row, hps_fetch_fn fetch, void *user,
                               hps_lookup_t **out_lookup) {
    if (!out_lookup) return lfail(HPS_ERR_INVALID_ARG, "out_lookup is NULL");
    *out_lookup = nullptr;
    uint32_t dim = 0;
    if (hps_cache_info(cache, nullptr, nullptr, &dim) != HPS_OK) return lfail(HPS_ERR_INVALID_ARG, "invalid cache handle");
    if (!fetch || !default_row) return lfail(HPS_ERR_INVALID_ARG, "fetch and default_row are required");
    if (max_batch == 0 || max_batch > (1ull << 30)) return lfail(HPS_ERR_INVALID_ARG, "max_batch must be in [1, 2^30]");
    hps_lookup_session *L = new (std::nothrow) hps_lookup_session();
    if (!L) return lfail(HPS_ERR_OOM, "host allocation failed");
    L->cache = cache; L->max_batch = max_batch; L->dim = dim; L->threshold = hit_threshold;
    L->fetch = fetch; L->user = user;
    L->dd = nullptr; L->dd_bg = nullptr;
    L->d_miss_idx = L->d_n_miss = L->d_inv = L->d_n_unique = nullptr; L->d_miss_keys = L->d_ukeys = nullptr;
    L->d_rows = L->d_default = nullptr; L->h_n_miss = L->h_n_unique = nullptr; L->h_ukeys = nullptr;
    L->h_rows = nullptr; L->side = nullptr; L->bg_d_ukeys = nullptr; L->bg_d_rows = L->bg_h_rows = nullptr;
    L->bg_h_keys = nullptr; L->bg_d_keys = nullptr; L->bg_d_inv = L->bg_d_n_unique = L->bg_h_n_unique = nullptr;
    const size_t nb = max_batch, rowb = (size_t)dim * sizeof(float);
    hipError_t e = hipGetDevice(&L->device);
    auto dev = [&](void **p, size_t bytes) { if (e == hipSuccess) e = hipMalloc(p, bytes); };
    auto pin = [&](void **p, size_t bytes) { if (e == hipSuccess) e = hipHostMalloc(p, bytes, hipHostMallocDefault); };
    dev((void **)&L->d_miss_idx, nb * 4); dev((void **)&L->d_n_miss, 4); dev((void **)&L->d_inv, nb * 4);
    dev((void **)&L->d_n_unique, 4);
    dev((void **)&L->d_miss_keys, nb * 8); dev((void **)&L->d_ukeys, nb * 8); dev((void **)&L->d_rows, nb * rowb);
    dev((void **)&L->d_default, rowb); dev((void **)&L->bg_d_ukeys, nb * 8); dev((void **)&L->bg_d_rows, nb * rowb);
    pin((void **)&L->h_n_miss, 4); pin((void **)&L->h_n_unique, 4);
    pin((void **)&L->h_ukeys, nb * 8); pin((void **)&L->h_rows, nb * rowb); pin((void **)&L->bg_h_rows, nb * rowb);
    pin((void **)&L->bg_h_keys, nb * 8); pin((void **)&L->bg_h_n_unique, 4);
    dev((void **)&L->bg_d_keys, nb * 8); dev((void **)&L->bg_d_inv, nb * 4); dev((void **)&L->bg_d_n_unique, 4);
    if (e == hipSuccess) e = hipStreamCreateWithFlags(&L->side, hipStreamNonBlocking);
    if (e == hipSuccess) e = hipMemcpy(L->d_default, default_row, rowb, hipMemcpyHostToDevice);
    {
        size_t n_slots = kMaxSlotBytes / (nb * 8);
        n_slots = n_slots > kMaxQueued + 2 ? kMaxQueued + 2 : (n_slots < 2 ? 2 : n_slots);
        L->slots.assign(n_slots, Slot{nullptr, nullptr});
        for (Slot &sl : L->slots) {
            dev((void **)&sl.d_keys, nb * 8);
            if (e == hipSuccess) e = hipEventCreateWithFlags(&sl.ready, hipEventDisableTiming);
        }
        if (e == hipSuccess) for (Slot &sl : L->slots) L->free_slots.push_back(&sl);
    }
    if (e != hipSuccess) {
        const std::string msg = std::string("hps_lookup_create: ") + hipGetErrorString(e);
        const hps_status_t code = e == hipErrorOutOfMemory ? HPS_ERR_OOM : HPS_ERR_DEVICE;
        (void)hipGetLastError();
        free_all(L);
        delete L;
        return lfail(code, msg);
    }
    hps_status_t ds = hps_dedup_create(max_batch, &L->dd);
    if (ds == HPS_OK) ds = hps_dedup_create(max_batch, &L->dd_bg);
    if (ds != HPS_OK) {
        const std::string msg = std::string("hps_lookup_create: ") + hps_dedup_last_error();
        free_all(L);
        delete L;
        return lfail(ds, msg);
    }
    L->worker = std::thread(worker_main, L);
    *out_lookup = L;
    return HPS_OK;
}

hps_status_t hps_lookup(hps_lookup_t *L, const int64_t *keys, size_t n, float *out, float *hit_rate,
                        int *was_synchronous, void *stream) {
    if (!L) return lfail(HPS_ERR_INVALID_ARG, "lookup is NULL");
    if (n > L->max_batch) return lfail(HPS_ERR_INVALID_ARG, "n exceeds max_batch");
    {
        std::lock_guard<std::mutex> lk(L->mu);
        if (!L->worker_error.empty()) {
            const std::string msg = L->worker_error;
            L->worker_error.clear();
            return lfail(HPS_ERR_DEVICE, msg);
        }
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (hit_rate) *hit_rate = 1.0f;
    if (was_synchronous) *was_synchronous = 0;
    if (n == 0) return HPS_OK;
    // EmbCacheLookup(Q): hits land in out, misses in the workspace
    if (hps_cache_query(L->cache, keys, n, out, L->d_miss_idx, L->d_miss_keys, L->d_n_miss, st) != HPS_OK)
        return lfail(HPS_ERR_INVALID_ARG, std::string("query: ") + hps_last_error());
    LK_TRY(hipMemcpyAsync(L->h_n_miss, L->d_n_miss, 4, hipMemcpyDeviceToHost, st));
    LK_TRY(hipStreamSynchronize(st));
    const uint32_t m = *L->h_n_miss;
    const float rate = 1.0f - (float)m / (float)n;
    if (hit_rate) *hit_rate = rate;
    if (m == 0) return HPS_OK;

    if (rate < L->threshold) {
        // synchronous insertion: ParServerLookup(missing keys), EmbCacheInsert, E_Q <- fetched vectors
        if (was_synchronous) *was_synchronous = 1;
        // the lower tiers see each missing key once (Sec. 2.2): dedup on the device, only the
        // distinct keys travel to the host; the map from miss-list entries to them stays here
        if (hps_dedup(L->dd, L->d_miss_keys, m, L->d_ukeys, L->d_inv, L->d_n_unique, st) != HPS_OK)
            return lfail(HPS_ERR_DEVICE, std::string("dedup: ") + hps_dedup_last_error());
        LK_TRY(hipMemcpyAsync(L->h_n_unique, L->d_n_unique, 4, hipMemcpyDeviceToHost, st));
        LK_TRY(hipMemcpyAsync(L->h_ukeys, L->d_ukeys, (size_t)m * 8, hipMemcpyDeviceToHost, st));
        LK_TRY(hipStreamSynchronize(st));
        const uint32_t u = *L->h_n_unique;
        L->fetch(L->user, L->h_ukeys, u, L->h_rows);
        LK_TRY(hipMemcpyAsync(L->d_rows, L->h_rows, (size_t)u * L->dim * sizeof(float), hipMemcpyHostToDevice, st));
        launch_place(out, L->d_miss_idx, L->d_inv, L->d_rows, m, L->dim, st);
        LK_TRY(hipGetLastError());
        if (hps_cache_insert(L->cache, L->d_ukeys, L->d_rows, u, st) != HPS_OK)
            return lfail(HPS_ERR_DEVICE, std::string("insert: ") + hps_last_error());
        // the workspace is reused by the next call: make sure this one is done with it
        LK_TRY(hipStreamSynchronize(st));
        return HPS_OK;
    }

    // asynchronous insertion: default vectors now, the real rows reach the cache later
    launch_place(out, L->d_miss_idx, nullptr, L->d_default, m, L->dim, st);
    LK_TRY(hipGetLastError());
    // The miss list (every occurrence) is copied aside on the device and handed to the background
    // thread, which deduplicates it on its own stream: this call does not wait for any of that.
    // A slot for it: a free one, else the one of the oldest waiting batch (the lower tier cannot
    // keep up: that batch is dropped).  If the background thread holds every slot right now (only
    // possible with two slots), this batch is the one that is not queued.
    Task t;
    t.slot = nullptr;
    t.m = m;
    bool taken_over = false;
    {
        std::lock_guard<std::mutex> lk(L->mu);
        if (!L->free_slots.empty()) {
            t.slot = L->free_slots.back();
            L->free_slots.pop_back();
        } else if (!L->queue.empty()) {
            t.slot = L->queue.front().slot;
            L->queue.pop_front();
            taken_over = true;
        }
    }
    if (!t.slot) return HPS_OK;
    // a dropped batch's copy into this buffer may still be in flight (on another stream, if the caller changes streams)
    hipError_t ce = taken_over ? hipStreamWaitEvent(st, t.slot->ready, 0) : hipSuccess;
    if (ce == hipSuccess) ce = hipMemcpyAsync(t.slot->d_keys, L->d_miss_keys, (size_t)m * 8, hipMemcpyDeviceToDevice, st);
    if (ce == hipSuccess) ce = hipEventRecord(t.slot->ready, st);
    {
        std::lock_guard<std::mutex> lk(L->mu);
        if (ce == hipSuccess) L->queue.push_back(t);
        else L->free_slots.push_back(t.slot);
    }
    if (ce != hipSuccess)
        return lfail(HPS_ERR_DEVICE, std::string("queueing the asynchronous insertion: ") + hipGetErrorString(ce));
    L->cv.notify_one();
    return HPS_OK;
}

hps_status_t hps_refresh_create(hps_cache_t *cache, size_t batch_slots, hps_refresh_t **out) {
    if (!out) return lfail(HPS_ERR_INVALID_ARG, "out is NULL");
    *out = nullptr;
    uint64_t sets = 0;
    uint32_t ways = 0, dim = 0;
    if (hps_cache_info(cache, &sets, &ways, &dim) != HPS_OK) return lfail(HPS_ERR_INVALID_ARG, "invalid cache handle");
    if (batch_slots == 0 || batch_slots >= (1ull << 31)) return lfail(HPS_ERR_INVALID_ARG, "batch_slots must be in [1, 2^31)");
    hps_refresh_session *R = new (std::nothrow) hps_refresh_session();
    if (!R) return lfail(HPS_ERR_OOM, "host allocation failed");
    R->cache = cache;
    R->slots = sets * ways;
    R->B = batch_slots < R->slots ? batch_slots : (size_t)R->slots;
    R->rowb = (size_t)dim * sizeof(float);
    hipError_t e = hipGetDevice(&R->device);
    for (int b = 0; b < 2; ++b) {
        if (e == hipSuccess) e = hipMalloc((void **)&R->d_keys[b], R->B * 8);
        if (e == hipSuccess) e = hipMalloc((void **)&R->d_rows[b], R->B * R->rowb);
        if (e == hipSuccess) e = hipHostMalloc((void **)&R->h_keys[b], R->B * 8, hipHostMallocDefault);
        if (e == hipSuccess) e = hipHostMalloc((void **)&R->h_rows[b], R->B * R->rowb, hipHostMallocDefault);
        if (e == hipSuccess) e = hipEventCreateWithFlags(&R->applied[b], hipEventDisableTiming);
    }
    if (e == hipSuccess) e = hipMalloc((void **)&R->d_cnt, 8);
    if (e == hipSuccess) e = hipHostMalloc((void **)&R->h_cnt, 8, hipHostMallocDefault);
    if (e == hipSuccess) e = hipStreamCreateWithFlags(&R->s2, hipStreamNonBlocking);
    if (e != hipSuccess) {
        const std::string msg = std::string("hps_refresh_create: ") + hipGetErrorString(e);
        (void)hipGetLastError();
        (void)hps_refresh_destroy(R);
        return lfail(e == hipErrorOutOfMemory ? HPS_ERR_OOM : HPS_ERR_DEVICE, msg);
    }
    *out = R;
    return HPS_OK;
}

hps_status_t hps_refresh_destroy(hps_refresh_t *R) {
    if (!R) return lfail(HPS_ERR_INVALID_ARG, "session is NULL");
    if (R->s2) (void)hipStreamSynchronize(R->s2);
    for (int b = 0; b < 2; ++b) {
        (void)hipFree(R->d_keys[b]); (void)hipFree(R->d_rows[b]);
        (void)hipHostFree(R->h_keys[b]); (void)hipHostFree(R->h_rows[b]);
        if (R->applied[b]) (void)hipEventDestroy(R->applied[b]);
    }
    (void)hipFree(R->d_cnt); (void)hipHostFree(R->h_cnt);
    if (R->s2) (void)hipStreamDestroy(R->s2);
    delete R;
    return HPS_OK;
}

hps_status_t hps_refresh_run(hps_refresh_t *R, hps_fetch_fn fetch, void *user, size_t *n_refreshed, void *stream) {
    if (n_refreshed) *n_refreshed = 0;
    if (!R) return lfail(HPS_ERR_INVALID_ARG, "session is NULL");
    if (!fetch) return lfail(HPS_ERR_INVALID_ARG, "fetch is required");
    hipStream_t st = static_cast<hipStream_t>(stream);
    const uint64_t slots = R->slots;
    const size_t B = R->B, rowb = R->rowb;
    // two sets of buffers: the host looks batch i + 1 up while batch i is uploaded and applied
    size_t total = 0;
    std::string err;
    hipError_t e = hipSuccess;
    bool used[2] = {false, false};
    for (uint64_t first = 0, i = 0; e == hipSuccess && err.empty() && first < slots; first += B, ++i) {
        const int b = (int)(i & 1);
        const size_t cnt_slots = (size_t)(slots - first < B ? slots - first : B);
        if (used[b]) e = hipEventSynchronize(R->applied[b]);       // this pair of buffers is free again
        if (e != hipSuccess) break;
        if (hps_cache_dump(R->cache, (size_t)first, cnt_slots, R->d_keys[b], R->d_cnt + b, R->s2) != HPS_OK) {
            err = std::string("dump: ") + hps_last_error();
            break;
        }
        e = hipMemcpyAsync(R->h_cnt + b, R->d_cnt + b, 4, hipMemcpyDeviceToHost, R->s2);
        if (e == hipSuccess) e = hipStreamSynchronize(R->s2);
        if (e != hipSuccess) break;
        const uint32_t m = R->h_cnt[b];
        if (m == 0) continue;
        e = hipMemcpyAsync(R->h_keys[b], R->d_keys[b], (size_t)m * 8, hipMemcpyDeviceToHost, R->s2);
        if (e == hipSuccess) e = hipStreamSynchronize(R->s2);
        if (e != hipSuccess) break;
        fetch(user, R->h_keys[b], m, R->h_rows[b]);                 // steps 2-3: lower tiers, key-vector buffer
        e = hipMemcpyAsync(R->d_rows[b], R->h_rows[b], (size_t)m * rowb, hipMemcpyHostToDevice, st);   // step 4
        if (e != hipSuccess) break;
        if (hps_cache_update(R->cache, R->d_keys[b], R->d_rows[b], m, st) != HPS_OK) {                 // step 5
            err = std::string("update: ") + hps_last_error();
            break;
        }
        e = hipEventRecord(R->applied[b], st);
        used[b] = true;
        total += m;
    }
    // the buffers are idle again when the call returns, also after an error
    hipError_t e2 = hipStreamSynchronize(st);
    if (e == hipSuccess) e = e2;
    (void)hipStreamSynchronize(R->s2);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        return lfail(e == hipErrorOutOfMemory ? HPS_ERR_OOM : HPS_ERR_DEVICE, std::string("hps_refresh_run: ") + hipGetErrorString(e));
    }
    if (!err.empty()) return lfail(HPS_ERR_DEVICE, err);
    if (n_refreshed) *n_refreshed = total;
    return HPS_OK;
}

hps_status_t hps_cache_refresh(hps_cache_t *cache, size_t batch_slots, hps_fetch_fn fetch, void *user,
                               size_t *n_refreshed, void *stream) {
    if (n_refreshed) *n_refreshed = 0;
    if (!fetch) return lfail(HPS_ERR_INVALID_ARG, "fetch is required");
    hps_refresh_t *R = nullptr;
    if (hps_status_t s = hps_refresh_create(cache, batch_slots, &R)) return s;
    const hps_status_t s = hps_refresh_run(R, fetch, user, n_refreshed, stream);
    const std::string msg = g_lookup_err;
    (void)hps_refresh_destroy(R);
    if (s != HPS_OK) g_lookup_err = msg;
    return s;
}

hps_status_t hps_lookup_drain(hps_lookup_t *L) {
    if (!L) return lfail(HPS_ERR_INVALID_ARG, "lookup is NULL");
    std::unique_lock<std::mutex> lk(L->mu);
    L->cv_idle.wait(lk, [&] { return L->queue.empty() && !L->busy; });
    if (!L->worker_error.empty()) {
        const std::string msg = L->worker_error;
        L->worker_error.clear();
        return lfail(HPS_ERR_DEVICE, msg);
    }
    return HPS_OK;
}

hps_status_t hps_lookup_destroy(hps_lookup_t *L) {
    if (!L) return lfail(HPS_ERR_INVALID_ARG, "lookup is NULL");
    (void)hps_lookup_drain(L);
    {
        std::lock_guard<std::mutex> lk(L->mu);
        L->stop = true;
    }
    L->cv.notify_all();
    if (L->worker.joinable()) L->worker.join();
    free_all(L);
    delete L;
    return HPS_OK;
}

const char *hps_lookup_last_error(void) { return g_lookup_err.c_str(); }

}  // extern "C"
