// Host-memory key -> row store: the stand-in for the lower tiers behind Algorithm 1 (Sec. 3.1,
// Sec. 5 of the paper).  Plain C++: partitioned hash maps, rows in per-partition slabs.
#include <atomic>
#include <condition_variable>
#include <cstdint>
#include <cstring>
#include <mutex>
#include <new>
#include <thread>
#include <vector>

#include "hps_hostmap.h"
#include "hps_mix.h"

namespace {

constexpr uint64_t kMagic = 0x4850534D41503031ull;
constexpr size_t kSlabRows = 1 << 14;           // rows per allocation unit of a partition
constexpr size_t kParallelFrom = 1024;          // batches at least this long are served by the helper threads too

constexpr uint64_t kFree = ~0ull;                 // row number of an unused slot

// Open-addressing index of one partition: key -> row number, linear probing, at most half full.
// (One cache line per lookup in the common case; a node-based map costs two.)
struct Slot {
    int64_t  key;
    uint64_t row;
};

struct Partition {
    std::mutex mu;
    std::vector<Slot> table;                          // size is a power of two
    std::vector<float *> slabs;                       // kSlabRows rows each
    uint64_t n_rows = 0;

    static uint64_t home(int64_t key, uint64_t mask) { return (mix64((uint64_t)key) >> 8) & mask; }

    // slot of `key`, or the free slot where it would go
    uint64_t find(int64_t key) const {
        const uint64_t mask = table.size() - 1;
        uint64_t i = home(key, mask);
        while (table[i].row != kFree && table[i].key != key) i = (i + 1) & mask;
        return i;
    }

    void reserve_slots(uint64_t n_keys) {             // table of at least 2 * n_keys slots
        uint64_t want = 1024;
        while (want < 2 * n_keys) want <<= 1;
        if (want <= table.size()) return;
        std::vector<Slot> old;
        old.swap(table);
        table.assign(want, Slot{0, kFree});
        for (const Slot &sl : old)
            if (sl.row != kFree) table[find(sl.key)] = sl;
    }
};

}  // namespace

// One batch lookup handed to the map's helper threads: thread t serves partitions
// [n_part * t / n_thr, n_part * (t + 1) / n_thr).
struct Job {
    const int64_t *keys = nullptr;
    float *rows = nullptr;
    const std::vector<uint32_t> *order = nullptr;      // positions sorted by partition
    const std::vector<size_t> *start = nullptr;        // [n_part + 1] first entry of each partition in `order`
    std::vector<size_t> absent;
};

struct hps_hostmap {
    uint64_t magic;
    uint32_t dim;
    uint32_t n_part;
    std::vector<Partition> parts;
    std::atomic<size_t> n_absent_total;
    // helper threads (n_thr - 1 of them; the caller is thread 0), woken once per parallel lookup
    uint32_t n_thr = 1;
    std::vector<std::thread> helpers;
    std::mutex job_mu;            // one parallel lookup at a time; a second caller serves itself alone
    std::mutex pool_mu;
    std::condition_variable pool_cv, done_cv;
    uint64_t generation = 0;
    uint32_t running = 0;
    bool stop = false;
    Job job;
};

namespace {

inline uint32_t part_of(const hps_hostmap *m, int64_t key) {
    return (uint32_t)(mix64((uint64_t)key) >> 40) & (m->n_part - 1);
}

float *row_ptr(const hps_hostmap *m, const Partition &p, uint64_t r) {
    return p.slabs[r / kSlabRows] + (r % kSlabRows) * m->dim;
}

// Serve positions whose key lives in partitions [p0, p1).  The positions have been bucketed by
// partition once per batch (order / start), so every partition's lock is taken once and no
// position is looked at by more than one thread.
size_t get_range(hps_hostmap *m, const int64_t *keys, float *rows, const std::vector<uint32_t> &order,
                 const std::vector<size_t> &start, uint32_t p0, uint32_t p1) {
    size_t absent = 0;
    for (uint32_t p = p0; p < p1; ++p) {
        const size_t b = start[p], e = start[p + 1];
        if (b == e) continue;
        Partition &P = m->parts[p];
        std::lock_guard<std::mutex> lk(P.mu);
        const uint64_t mask = P.table.size() - 1;
        for (size_t j = b; j < e; ++j) {
            if (j + 4 < e) __builtin_prefetch(&P.table[Partition::home(keys[order[j + 4]], mask)]);
            const size_t i = order[j];
            const Slot &sl = P.table[P.find(keys[i])];
            if (sl.row == kFree) {
                std::memset(rows + i * m->dim, 0, sizeof(float) * m->dim);
                ++absent;
            } else {
                std::memcpy(rows + i * m->dim, row_ptr(m, P, sl.row), sizeof(float) * m->dim);
            }
        }
    }
    return absent;
}

void helper_main(hps_hostmap *m, uint32_t t) {
    uint64_t seen = 0;
    for (;;) {
        {
            std::unique_lock<std::mutex> lk(m->pool_mu);
            m->pool_cv.wait(lk, [&] { return m->stop || m->generation != seen; });
            if (m->stop) return;
            seen = m->generation;
        }
        const uint32_t p0 = (uint32_t)((uint64_t)m->n_part * t / m->n_thr);
        const uint32_t p1 = (uint32_t)((uint64_t)m->n_part * (t + 1) / m->n_thr);
        m->job.absent[t] = get_range(m, m->job.keys, m->job.rows, *m->job.order, *m->job.start, p0, p1);
        {
            std::lock_guard<std::mutex> lk(m->pool_mu);
            if (--m->running == 0) m->done_cv.notify_one();
        }
    }
}

}  // namespace

extern "C" {

hps_status_t hps_hostmap_create(uint32_t dim, uint32_t partitions, size_t reserve, hps_hostmap_t **out) {
    if (!out) return HPS_ERR_INVALID_ARG;
    *out = nullptr;
    if (dim == 0 || partitions == 0 || partitions > 256 || (partitions & (partitions - 1)) != 0)
        return HPS_ERR_INVALID_ARG;
    hps_hostmap *m = new (std::nothrow) hps_hostmap();
    if (!m) return HPS_ERR_OOM;
    try {
        m->dim = dim;
        m->n_part = partitions;
        m->parts = std::vector<Partition>(partitions);
        for (auto &p : m->parts) p.reserve_slots(reserve / partitions + 16);
    } catch (const std::bad_alloc &) {
        delete m;
        return HPS_ERR_OOM;
    }
    m->n_absent_total.store(0);
    uint32_t n_thr = std::thread::hardware_concurrency();
    if (n_thr > 8) n_thr = 8;
    if (n_thr > partitions) n_thr = partitions;
    if (n_thr == 0) n_thr = 1;
    m->n_thr = n_thr;
    m->job.absent.assign(n_thr, 0);
    try {
        for (uint32_t t = 1; t < n_thr; ++t) m->helpers.emplace_back(helper_main, m, t);
    } catch (const std::exception &) {                     // fewer helpers than planned: run with those
        m->n_thr = (uint32_t)m->helpers.size() + 1;
    }
    m->magic = kMagic;
    *out = m;
    return HPS_OK;
}

hps_status_t hps_hostmap_destroy(hps_hostmap_t *m) {
    if (!m || m->magic != kMagic) return HPS_ERR_INVALID_ARG;
    m->magic = 0;
    {
        std::lock_guard<std::mutex> lk(m->pool_mu);
        m->stop = true;
    }
    m->pool_cv.notify_all();
    for (auto &th : m->helpers) th.join();
    for (auto &p : m->parts)
        for (float *s : p.slabs) delete[] s;
    delete m;
    return HPS_OK;
}

hps_status_t hps_hostmap_put(hps_hostmap_t *m, const int64_t *keys, const float *rows, size_t n) {
    if (!m || m->magic != kMagic) return HPS_ERR_INVALID_ARG;
    if (n == 0) return HPS_OK;
    if (!keys || !rows) return HPS_ERR_INVALID_ARG;
    try {
        for (size_t i = 0; i < n; ++i) {
            Partition &P = m->parts[part_of(m, keys[i])];
            std::lock_guard<std::mutex> lk(P.mu);
            uint64_t at = P.find(keys[i]);
            uint64_t r;
            if (P.table[at].row == kFree) {
                if (2 * (P.n_rows + 1) > P.table.size()) {       // keep the table at most half full
                    P.reserve_slots(P.n_rows + 1);
                    at = P.find(keys[i]);
                }
                r = P.n_rows;
                if (r / kSlabRows >= P.slabs.size()) P.slabs.push_back(new float[kSlabRows * (size_t)m->dim]);
                P.table[at] = Slot{keys[i], r};
                ++P.n_rows;
            } else {
                r = P.table[at].row;
            }
            std::memcpy(row_ptr(m, P, r), rows + i * m->dim, sizeof(float) * m->dim);
        }
    } catch (const std::bad_alloc &) {
        return HPS_ERR_OOM;
    }
    return HPS_OK;
}

hps_status_t hps_hostmap_get(hps_hostmap_t *m, const int64_t *keys, size_t n, float *rows, size_t *n_absent) {
    if (!m || m->magic != kMagic) return HPS_ERR_INVALID_ARG;
    if (n_absent) *n_absent = 0;
    if (n == 0) return HPS_OK;
    if (!keys || !rows) return HPS_ERR_INVALID_ARG;
    size_t absent = 0;
    try {
        if (n >= (1ull << 32)) return HPS_ERR_INVALID_ARG;
        // counting sort of the positions by partition: one pass to count, one to place
        std::vector<uint8_t> part(n);                      // n_part <= 256
        std::vector<size_t> start(m->n_part + 1, 0);
        for (size_t i = 0; i < n; ++i) {
            part[i] = (uint8_t)part_of(m, keys[i]);
            ++start[part[i] + 1];
        }
        for (uint32_t p = 0; p < m->n_part; ++p) start[p + 1] += start[p];
        std::vector<uint32_t> order(n);
        {
            std::vector<size_t> at(start.begin(), start.end() - 1);
            for (size_t i = 0; i < n; ++i) order[at[part[i]]++] = (uint32_t)i;
        }
        std::unique_lock<std::mutex> pool(m->job_mu, std::defer_lock);
        if (n >= kParallelFrom && m->n_thr > 1 && pool.try_lock()) {
            m->job.keys = keys;
            m->job.rows = rows;
            m->job.order = &order;
            m->job.start = &start;
            {
                std::lock_guard<std::mutex> lk(m->pool_mu);
                m->running = m->n_thr - 1;
                ++m->generation;
            }
            m->pool_cv.notify_all();
            const uint32_t p1 = (uint32_t)((uint64_t)m->n_part * 1 / m->n_thr);
            absent = get_range(m, keys, rows, order, start, 0, p1);           // the caller is thread 0
            {
                std::unique_lock<std::mutex> lk(m->pool_mu);
                m->done_cv.wait(lk, [&] { return m->running == 0; });
            }
            for (uint32_t t = 1; t < m->n_thr; ++t) absent += m->job.absent[t];
        } else {
            absent = get_range(m, keys, rows, order, start, 0, m->n_part);
        }
    } catch (const std::exception &) {
        return HPS_ERR_OOM;
    }
    m->n_absent_total.fetch_add(absent);
    if (n_absent) *n_absent = absent;
    return HPS_OK;
}

void hps_hostmap_fetch(void *user, const int64_t *keys, size_t n, float *rows) {
    (void)hps_hostmap_get(static_cast<hps_hostmap_t *>(user), keys, n, rows, nullptr);
}

hps_status_t hps_hostmap_stats(hps_hostmap_t *m, size_t *n_keys, size_t *n_absent_total) {
    if (!m || m->magic != kMagic) return HPS_ERR_INVALID_ARG;
    if (n_keys) {
        size_t k = 0;
        for (auto &p : m->parts) {
            std::lock_guard<std::mutex> lk(p.mu);
            k += p.n_rows;
        }
        *n_keys = k;
    }
    if (n_absent_total) *n_absent_total = m->n_absent_total.load();
    return HPS_OK;
}

}  // extern "C"
