// GPU embedding cache for MI355X (gfx950, wave64): kernels and the C ABI of include/hps_cache.h.
//
// Memory layout (all in HBM, owned by the cache):
//   K   int64  [S][W]      keys, one 64-byte line per set at W = 8; EMPTY = INT64_MIN
//   V   fp32   [S][W][d]   rows, 16-byte aligned, moved as opaque 128-bit chunks
//   sc  uint32 [S][2]      one 8-byte word per set: {seq, ctr}
//                            seq  sequence word: odd while a writer owns the set (lock + seqlock)
//                            ctr  victim counter: next way of the set = ctr mod W
//                          (together so that an insert gets both with its one 64-bit atomic and
//                          lets go of both with one store; every read is a 128-byte request)
//   T   uint32 [S][W]      access stamps, only for caches created with the LRU policy
//
// Paper passages: data model Sec. 4.1; Query Alg. 2; Replace Alg. 3; Update Alg. 4; Dump and
// the asynchronous, batch-in calling convention Sec. 4.2.  The paper's per-slabset warp lock
// (Sec. 4.1) survives as the per-set sequence word, but only writers take it: query is
// read-only because the victim rule keeps no access stamps.
#include <hip/hip_runtime.h>

#include <atomic>
#include <climits>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <unordered_map>

#include "hps_cache.h"
#include "hps_membench.h"
#include "hps_mix.h"

namespace {

constexpr int64_t  kEmpty      = INT64_MIN;
constexpr int      kBlock      = 256;          // threads per work-group: 4 waves of 64
constexpr int      kWave       = 64;
constexpr int      kWavesPerWg = kBlock / kWave;
constexpr int      kInsertKpw  = 16;           // keys per wave of the insert kernel
constexpr uint32_t kRing       = 1024;         // counter words per half of the pool (see counter_word)
constexpr uint64_t kMagic      = 0x4850534341434845ull;
// Every loop that waits for another kernel's writer to let go of a set gives up after this many
// rounds (a held set is released within microseconds; this many rounds take about a second) and
// raises HPS_FLAG_STUCK_SET in the cache's flag word, so that no wave can spin forever.
constexpr uint32_t kMaxRounds  = 1u << 16;
// Longest row (in fp32) that a query may read while writers run: a row is read whole (8 wave loads
// of 8 bytes per lane at this length) before it is validated and stored.
constexpr uint32_t kMaxCheckedDim = 1024;

typedef float f32x4 __attribute__((ext_vector_type(4)));   // one 16-byte chunk of a row

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

// ------------------------------------------------------------------ device helpers

// Alg. 2 "slabsetHasher(q) mod |S|": upper hash half modulo the set count (mask when S is 2^k).
__device__ __forceinline__ uint32_t set_of(int64_t key, uint32_t S, uint32_t smask) {
    uint32_t h = (uint32_t)(mix64((uint64_t)key) >> 32);
    return smask ? (h & smask) : (h % S);
}

__device__ __forceinline__ bool is_reserved(int64_t key) { return key < kEmpty + 2; }

__device__ __forceinline__ int lane_id() { return (int)(threadIdx.x & (kWave - 1)); }

__device__ __forceinline__ int64_t shfl64(int64_t v, int src) {
    int lo = __shfl((int)(uint32_t)(uint64_t)v, src, kWave);
    int hi = __shfl((int)(uint32_t)((uint64_t)v >> 32), src, kWave);
    return (int64_t)(((uint64_t)(uint32_t)hi << 32) | (uint32_t)lo);
}

// Number of set bits of m below this lane.
__device__ __forceinline__ int rank_in(uint64_t m) {
    return (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32),
                                          __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
}

// Orders this wave's LDS traffic against itself (no instructions, compiler-only).
__device__ __forceinline__ void wave_lds_fence() {
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

template <typename T> __device__ __forceinline__ T ld_agent(const T *p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
template <typename T> __device__ __forceinline__ void st_agent(T *p, T v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Data that kernels overlapping on different streams share (keys, rows, counters of the cache):
// every such load/store is itself an agent-scope relaxed atomic of 4 or 8 bytes (global_load /
// global_store with sc1: the access is performed at the memory side of the non-coherent per-XCD
// L2s, so it sees and is seen by every other agent-scope access of the device), and the order
// "sequence word, then data, then sequence word" is kept by waiting until the wave's outstanding
// vector memory operations have completed (s_waitcnt vmcnt(0)) between the steps: a wave's vector
// memory instruction counter reaches zero only when every earlier load has returned its data and
// every earlier store has been acknowledged by the level it was addressed to.
// The wait is the compiler's own s_waitcnt instruction (vmcnt(0), the other counters left alone:
// 0x0F70 in the gfx9 encoding), not inline assembly: the pass that places the waits in front of
// every use of a loaded register reads it and knows from there on that nothing is outstanding.
// Behind an assembly string it assumed that every row load might still be in flight and put a
// vmcnt(0) in front of each row store, so a wave had one store in flight at a time.
__device__ __forceinline__ void wait_vm0() {
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt(0x0F70);
    asm volatile("" ::: "memory");
}
__device__ __forceinline__ void shared_acquire() { wait_vm0(); }
__device__ __forceinline__ void shared_release() { wait_vm0(); }
__device__ __forceinline__ uint64_t shared_ld64(const uint64_t *p) { return ld_agent(p); }
__device__ __forceinline__ void shared_st64(uint64_t *p, uint64_t v) { st_agent(p, v); }

struct alignas(64) Table {     // one cache as the kernels see it (one 64-byte line of the kernel arguments)
    int64_t  *K;
    float    *V;
    uint32_t *sc;              // [S][2]: {sequence word, victim counter} of a set
    uint32_t  S;
    uint32_t  smask;           // S - 1 when S is a power of two, else 0
    uint32_t *T;               // [S][W] access stamps, LRU policy only (else nullptr)
    uint32_t *gdev;            // the cache's global iteration count g of Alg. 2 (LRU policy): one device word
    uint32_t *flags;           // one word of HPS_FLAG_* bits raised by kernels
};

__device__ __forceinline__ uint32_t *seq_of(const Table &tb, uint32_t set) { return tb.sc + 2ull * set; }

// Row geometry shared by all copy loops: a row is C = d/4 chunks of 16 bytes; LPR lanes
// cooperate on one row (16 B per lane, contiguous, so a wave load covers 64/LPR whole rows).
struct RowGeom {
    uint32_t d;                // fp32 per row
    uint32_t C;                // 16-byte chunks per row
    uint32_t LPR;              // lanes per row: min(64, next power of two >= C)
    uint32_t lprShift;         // log2(LPR)
    uint32_t passes;           // ceil(C / LPR): > 1 only for rows longer than 1 KiB
    // the same for 8-byte chunks (paths that move rows with 8-byte scoped accesses)
    uint32_t C8, LPR8, lpr8Shift, passes8;
};

// Copy `cnt` (> 0) rows listed in LDS: row srcRow[e] of `src` to row dstRow[e] of `dst`, for
// e < cnt.  LPR lanes move one row, 16 B per lane, so a wave load/store covers 64/LPR whole
// rows.  The rows go in groups of U wave loads: a group's loads are ALL issued, one wait for
// them follows, then the group's stores go out back to back.  With U = 26 the 52 rows of a wave
// of the 106,496-key batch (two 512-byte rows per wave load) are one group, every worker wave has
// its whole share of the batch in flight at once, and the launch takes 18.4 us in the stand-alone
// test bed against 21.5 us with two alternating buffers of 2 wave loads and 22.9 us with one
// buffer of 4 (two groups of 15: 20.3 us).  Non-temporal loads here cost 6 us (repeated keys live
// on L2 hits), non-temporal stores save 2 us (rows of `out` are written once and not read again
// here).  Lanes beyond the list load entry 0 and store nothing; lanes beyond the row (d/4 not a
// power of two) repeat chunk 0.
// kD = 128 fixes the row geometry at compile time (32 lanes per row, one pass, shifts instead
// of multiplications); kD = 0 takes it from g.
template <int U, int kD = 0, typename SrcIdx, typename DstIdx>
__device__ __forceinline__ void copy_rows(const RowGeom g, const float *__restrict__ src,
                                          float *__restrict__ dst, const SrcIdx *srcRow,
                                          const DstIdx *dstRow, uint32_t cnt) {
    static_assert(kD == 0 || kD == 128, "only the 128-word row is specialised");
    const uint32_t lane = (uint32_t)lane_id();
    const uint32_t lprShift = kD ? 5u : g.lprShift;
    const uint32_t LPR = kD ? 32u : g.LPR;
    const uint32_t C = kD ? 32u : g.C;
    const uint64_t d = kD ? (uint64_t)kD : (uint64_t)g.d;
    const uint32_t passes = kD ? 1u : g.passes;
    const uint32_t rpi = (uint32_t)kWave >> lprShift;        // rows per wave load
    const uint32_t sub = lane >> lprShift;                   // which of those rows this lane serves
    const uint32_t cl  = lane & (LPR - 1);                   // chunk of the row this lane moves
    for (uint32_t pass = 0; pass < passes; ++pass) {
        uint32_t chunk = cl + pass * LPR;
        chunk = chunk < C ? chunk : 0u;
        const uint32_t off = chunk * 4;
        for (uint32_t e0 = 0; e0 < cnt; e0 += rpi * U) {
            f32x4 buf[U];
            uint32_t ent[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const uint32_t e = e0 + u * rpi + sub;
                ent[u] = e < cnt ? e : 0xFFFFFFFFu;
                buf[u] = *reinterpret_cast<const f32x4 *>(src + (uint64_t)srcRow[e < cnt ? e : 0u] * d + off);
            }
            // One wait for the whole group, stated where the compiler can see it.  The stores are
            // predicated, so the compiler cannot count them among the outstanding operations and
            // would make store k wait until at most U-1-k operations are in flight: the later
            // stores of a group would wait for the earlier ones to be acknowledged.
            __builtin_amdgcn_s_waitcnt(0x0F70);                      // vmcnt(0), other counters untouched
#pragma unroll
            for (int u = 0; u < U; ++u)
                if (ent[u] != 0xFFFFFFFFu)
                    __builtin_nontemporal_store(buf[u], reinterpret_cast<f32x4 *>(dst + (uint64_t)dstRow[ent[u]] * d + off));
        }
    }
}

// copy_rows for a reader that may overlap writers (seqlock read side).  Entry e also carries
// the set it came from and the value v1 of that set's sequence word read before the probe.
// Rows are loaded into registers (8 bytes per lane, shared_ld64), then the sequence words are
// read again once those loads have completed; a row is stored only if its word is unchanged,
// i.e. no writer touched the set while the row was being read.  Entries to redo are flagged in
// the LDS word pair `retry`.
// The wave's rows go in groups of U wave loads, all of a group's loads in flight together; then
// ONE more wave load reads the sequence words again, lane l that of the group's row l, and a
// ballot of "changed" gives the rows to redo.  That is two dependent round trips per group, so
// the fewer groups the better (27.5 us per 106,496-key batch with groups of 16 rows, 21.6 us with
// one group per wave in the stand-alone test bed).  A row is always read whole inside one group
// (rows longer than 512 bytes take several of the group's wave loads; the longest row, 4 KiB, takes
// 8, which is why U >= 8 and why kMaxCheckedDim is 1024) and stored only after its validation:
// a position whose key turns out to be gone on the retry (evicted by an overlapping insert) has
// had nothing written to its `out` row.
template <int U, int kD = 0, bool kLong = false>
__device__ __forceinline__ void copy_rows_checked(const RowGeom g, const float *__restrict__ src,
                                                  float *__restrict__ dst, const uint64_t *srcRow,
                                                  const uint32_t *dstRow, const uint32_t *setOf,
                                                  const uint32_t *v1Of, const uint32_t *sc,
                                                  uint32_t cnt, uint32_t *retry) {
    static_assert(!(kD && kLong), "the compile-time geometry is a short row");
    const uint32_t lane = (uint32_t)lane_id();
    // Geometry of one wave load of 8 bytes per lane.  Short rows (kLong false, up to 512 bytes):
    // LPR8 lanes per row, rpi rows per wave load.  Long rows (kLong, up to kMaxCheckedDim fp32):
    // passes8 wave loads per row.  kD = 128: a 512-byte row is exactly one wave load.
    // A long row takes 2^pShift >= passes8 of a group's wave loads (those past the row's end are idle).
    const uint32_t pShift = kLong ? 32u - (uint32_t)__builtin_clz(g.passes8 - 1u) : 0u;
    const uint32_t rpiShift = (kD || kLong) ? 0u : 6u - g.lpr8Shift;
    const uint32_t sub = (kD || kLong) ? 0u : lane >> g.lpr8Shift;
    const uint32_t cl  = (kD || kLong) ? lane : lane & (g.LPR8 - 1);
    const uint64_t d = kD ? (uint64_t)kD : (uint64_t)g.d;
    // rows per group: every row of a group is read whole (all its wave loads are among the group's
    // U), and one lane per row re-reads its sequence word, so a group has at most 64 rows
    uint32_t span = kLong ? (uint32_t)U >> pShift : (uint32_t)U << rpiShift;
    span = span < (uint32_t)kWave ? span : (uint32_t)kWave;
    for (uint32_t e0 = 0; e0 < cnt; e0 += span) {
        const uint32_t rows = cnt - e0 < span ? cnt - e0 : span;
        uint64_t buf[U];
        // wave load u of the group: rows u*rpi .. (short rows), or part u mod 2^pShift of row
        // u >> pShift (long rows)
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint32_t r0 = kLong ? (uint32_t)u >> pShift : (uint32_t)u << rpiShift;
            if (r0 < rows) {                                         // uniform: this wave load has rows to fetch
                uint32_t r = r0 + sub;
                r = r < rows ? r : 0u;
                uint32_t chunk = kLong ? (((uint32_t)u & ((1u << pShift) - 1u)) << 6) + lane : cl;
                chunk = chunk < g.C8 || kD ? chunk : 0u;
                buf[u] = shared_ld64(reinterpret_cast<const uint64_t *>(src + srcRow[e0 + r] * d) + chunk);
            }
        }
        shared_acquire();                                            // row loads complete before the re-read
        const bool mine = lane < rows;
        const uint32_t v2 = mine ? ld_agent(sc + 2ull * setOf[e0 + lane]) : 0u;
        const uint64_t bad = __ballot(mine && v2 != v1Of[e0 + lane]);   // bit r: row e0 + r was touched by a writer
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint32_t r0 = kLong ? (uint32_t)u >> pShift : (uint32_t)u << rpiShift;
            if (r0 < rows) {
                const uint32_t r = r0 + sub;
                const uint32_t chunk = kLong ? (((uint32_t)u & ((1u << pShift) - 1u)) << 6) + lane : cl;
                if (r < rows && (chunk < g.C8 || kD) && !((bad >> r) & 1ull))
                    __builtin_nontemporal_store(
                        buf[u], reinterpret_cast<uint64_t *>(dst + (uint64_t)dstRow[e0 + r] * d) + chunk);
            }
        }
        if (bad && lane == 0) {                                      // e0 + rows <= cnt <= 64
            const uint64_t m = bad << e0;
            __hip_atomic_fetch_or(retry + 0, (uint32_t)m, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            __hip_atomic_fetch_or(retry + 1, (uint32_t)(m >> 32), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        }
    }
}

// Writer side: copy `cnt` (> 0) rows listed in LDS from the caller's batch into the cache with
// shared_st64 (8 bytes per lane), so that overlapping readers observe them without cache flushes.
// Two register buffers alternate: the loads of the next U wave loads are issued before the
// stores of the current ones, so a write-through store's long acknowledgement never sits between
// a wave and its next loads.  Lanes past the list repeat entry 0 (same bytes to the same place),
// and the loads issued past the last group re-read entry 0 and are dropped.  (Groups of 16 or 32
// wave loads all in flight before the first store, which is what the query's copy does, cost the
// writers occupancy and time: insert 102 us against 83 us per 2^18 rows, update 118 against 81 us.)
template <int U>
__device__ __forceinline__ void copy_rows_shared(const RowGeom g, const float *__restrict__ src,
                                                 float *dst, const uint32_t *srcRow,
                                                 const uint64_t *dstRow, uint32_t cnt) {
    const uint32_t lane = (uint32_t)lane_id();
    const uint32_t rpi = (uint32_t)kWave >> g.lpr8Shift;
    const uint32_t sub = lane >> g.lpr8Shift;
    const uint32_t cl  = lane & (g.LPR8 - 1);
    const uint32_t step = rpi * U;
    for (uint32_t pass = 0; pass < g.passes8; ++pass) {
        uint32_t chunk = cl + pass * g.LPR8;
        chunk = chunk < g.C8 ? chunk : 0u;
        uint64_t bufA[U], bufB[U];
        uint32_t entA[U], entB[U];
        auto load = [&](uint32_t e0, uint64_t (&buf)[U], uint32_t (&ent)[U]) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const uint32_t e = e0 + u * rpi + sub;
                ent[u] = e < cnt ? e : 0u;
                buf[u] = __builtin_nontemporal_load(reinterpret_cast<const uint64_t *>(src + (uint64_t)srcRow[ent[u]] * g.d) + chunk);
            }
        };
        auto store = [&](const uint64_t (&buf)[U], const uint32_t (&ent)[U]) {
#pragma unroll
            for (int u = 0; u < U; ++u)
                shared_st64(reinterpret_cast<uint64_t *>(dst + dstRow[ent[u]] * g.d) + chunk, buf[u]);
        };
        load(0, bufA, entA);
        for (uint32_t e0 = 0;; e0 += 2 * step) {
            load(e0 + step, bufB, entB);
            store(bufA, entA);
            if (e0 + step >= cnt) break;
            load(e0 + 2 * step, bufA, entA);
            store(bufB, entB);
            if (e0 + 2 * step >= cnt) break;
        }
    }
}

// Set probe for the first KPW lanes' keys of a wave (Alg. 2 "warpReadOutSlab" + match): W lanes
// read the W slot keys of one set (contiguous 8*W bytes), so one wave load covers 64/W sets; a
// ballot over the equality test gives every key its way.  Returns the way or -1.
template <int W, int KPW, bool kShared = false>
__device__ __forceinline__ int probe_wave(const int64_t *__restrict__ K, int64_t key,
                                          uint32_t set, bool want) {
    constexpr int G = kWave / W;                       // keys per wave load
    constexpr int R = (KPW + G - 1) / G;               // wave loads needed for KPW keys
    constexpr int RC = R > 32 ? 32 : R;                // wave loads in flight together (64 for W = 64 would not fit the registers)
    const int lane = lane_id();
    const int slot = lane & (W - 1);
    const int sub  = lane / W;
    int way = -1;
#pragma unroll
    for (int r0 = 0; r0 < R; r0 += RC) {
        int64_t sk[RC];
#pragma unroll
        for (int r = 0; r < RC; ++r) {
            const int j = (r0 + r) * G + sub;
            const uint32_t sj = (uint32_t)__shfl((int)set, j, kWave);   // 0 for lanes without a key: a valid set
            const int64_t *p = K + (uint64_t)sj * W + slot;
            sk[r] = kShared ? (int64_t)shared_ld64(reinterpret_cast<const uint64_t *>(p)) : *p;
        }
#pragma unroll
        for (int r = 0; r < RC; ++r) {
            const int j = (r0 + r) * G + sub;
            const int64_t kj = shfl64(key, j);
            const int wj = __shfl((int)want, j, kWave);
            const uint64_t m = __ballot(wj && sk[r] == kj);
            if (lane / G == r0 + r) {
                const uint64_t field = (W == 64) ? m : ((m >> ((lane % G) * W)) & ((1ull << (W & 63)) - 1));
                if (field) way = __builtin_ctzll(field);
            }
        }
    }
    return way;
}

// ------------------------------------------------------------------ query

// The scalars come first, in two 64-byte lines, then one line per table: a kernel's first reads of
// its arguments miss in the scalar cache line by line.
struct QueryArgs {
    const int64_t *keys;        // [T][B]
    float         *out;         // [T][B][d]
    uint32_t      *miss_idx;
    int64_t       *miss_keys;
    uint32_t      *n_miss;
    uint64_t      *slot;        // the stream's counter word: low 32 bits = misses so far, high 32 = tiles done
    const uint32_t *n_dev;      // optional: the real batch length (<= B) is read on the device (one table only)
    uint32_t       B;           // keys per table
    uint32_t       kpw;         // keys per worker wave (<= 64): lanes kpw..63 of a worker wave stay idle
    uint32_t       tiles_per_table;
    uint32_t       n_tiles;     // T * tiles_per_table (>= 1 even when B == 0)
    uint32_t       n_tables;    // T (<= HPS_MAX_TABLES <= 64: one helper lane per table finishes the call)
    RowGeom        g;
    Table          tab[HPS_MAX_TABLES];
};

// Kernel arguments are read with scalar loads where they are first used, each followed by its own
// wait; spread over several cache lines and basic blocks that put three to five dependent
// scalar-cache misses in front of a wave's first key load (0.7 us of a 19 us query launch).  The
// kernels therefore name everything a tile needs in ONE empty asm statement: all the loads are
// issued together ahead of it and waited for once.
#define HPS_ARGS_NOW(...) asm volatile("" ::__VA_ARGS__)

// What the tile that finds every other tile of its call finished does (helper wave, all lanes):
// publish the miss count, clear the call's counter word for the next call on the stream, and
// advance the iteration count g of every LRU table of the call (Alg. 2 has thread 0 do the
// atomic add; every tile has read g by then, because a tile reads it before it adds its count).
__device__ __forceinline__ void finish_call(const QueryArgs &a, uint32_t n_miss, int lane) {
    if (lane == 0) {
        *a.n_miss = n_miss;
        __hip_atomic_store(a.slot, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    if ((uint32_t)lane < a.n_tables && a.tab[lane].T)
        __hip_atomic_fetch_add(a.tab[lane].gdev, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Query (Alg. 2).  A work-group is WPB worker waves plus one helper wave and handles tiles of
// WPB*KPW positions; the first KPW lanes of each worker wave own one key each.
//   workers  load key, hash, probe the set (probe_wave); misses are compacted per wave into LDS
//            (ballot + mbcnt prefix), hits into the wave's <source slot, destination position>
//            list; the wave then copies its rows (copy_rows) without waiting for the others.
//   helper   once every worker wave has listed its misses (an LDS counter in the plain variant,
//            a barrier in the checked one) it adds the tile's miss count to the call's counter
//            word with one 64-bit atomic (low half: misses so far, high half: tiles done), then
//            writes the tile's miss entries from LDS to the global list.  The tile that finds
//            every other tile done publishes *n_miss and clears the word for the next call.
// The helper exists so that no worker has the atomic's round trip in front of its row loads
// (vector memory results return in issue order).
//
// kCoherent = true is the variant for queries that may overlap insert/update kernels on other
// streams: each worker reads its sets' sequence words before probing, skips sets a writer holds
// (odd word), copies rows with copy_rows_checked and repeats for the keys whose set changed under
// it.  A miss needs no check (an 8-byte key is read whole, and a key that stays cached is never
// absent from its slot), so only hits are validated.
// kFull = true is launched for calls that name an LRU table or take their length from the device
// (n_dev): only those kernels read g, stamp their hits and read *n_dev.  (As never-taken branches
// in every kernel the three cost 0.4 us of a 19 us launch.)
template <int W, int KPW, int U, int WPB, bool kCoherent, int kD = 0, bool kFull = false>
__global__ void __launch_bounds__((WPB + 1) * kWave) query_kernel(const QueryArgs a) {
    __shared__ uint64_t s_src[WPB][KPW];
    __shared__ uint32_t s_dst[WPB][KPW];
    __shared__ int64_t  s_mkey[WPB][KPW];
    __shared__ uint32_t s_mpos[WPB][KPW];
    __shared__ uint32_t s_wcnt[WPB];
    __shared__ uint32_t s_ready;                   // worker waves that have listed their misses (plain variant)
    __shared__ uint32_t s_set[kCoherent ? WPB : 1][kCoherent ? KPW : 1];
    __shared__ uint32_t s_v1[kCoherent ? WPB : 1][kCoherent ? KPW : 1];
    __shared__ uint32_t s_retry[kCoherent ? WPB : 1][2];

    const int lane = lane_id();
    const int wave = (int)(threadIdx.x / kWave);
    HPS_ARGS_NOW("s"(a.keys), "s"(a.out), "s"(a.n_dev), "s"(a.B), "s"(a.kpw), "s"(a.tiles_per_table), "s"(a.n_tiles),
                 "s"(a.tab[0].K), "s"(a.tab[0].V), "s"(a.tab[0].T), "s"(a.tab[0].S), "s"(a.tab[0].smask));
    const RowGeom g = a.g;
    const bool many_tiles = a.n_tiles > gridDim.x;     // this work-group may take several tiles

    if (!kCoherent) {
        // The plain variant has no work-group barrier between probe and row copy: each worker
        // wave goes on to its rows as soon as its own probe is done and only tells the helper,
        // through s_ready, that its misses are listed.  (The barrier made every wave wait for the
        // slowest probe of the work-group: 22.9 -> 22.1 us per 106,496-key batch without it.)
        if (threadIdx.x == 0) s_ready = 0u;
        __syncthreads();
    }
    for (uint32_t tile = blockIdx.x; tile < a.n_tiles; tile += gridDim.x) {
        const uint32_t t  = tile / a.tiles_per_table;
        const uint32_t lt = tile - t * a.tiles_per_table;
        if (wave < WPB) {
            const Table   &tb   = a.tab[t];
            HPS_ARGS_NOW("s"(tb.K), "s"(tb.V), "s"(tb.T), "s"(tb.gdev), "s"(tb.S), "s"(tb.smask), "s"(tb.sc));
            // Alg. 2 "g <- g + 1": every tile of the call stamps with the count the call will leave
            // behind; the tile that finishes the call stores it (see the helper wave below).
            const uint32_t g_call = kFull && tb.T ? *tb.gdev + 1u : 0u;
            const uint32_t b    = (lt * WPB + wave) * a.kpw + lane;
            const bool     inb  = lane < (int)a.kpw && b < a.B;
            const uint32_t pos  = t * a.B + b;         // position in keys/out (< 2^32 checked on host)

            const int64_t key  = inb ? a.keys[pos] : kEmpty;      // keys[0 .. B) is readable also when n_dev says less
            const bool    live = inb && (!kFull || !a.n_dev || b < *a.n_dev);
            const bool    want = live && !is_reserved(key);
            const uint32_t set = want ? set_of(key, tb.S, tb.smask) : 0u;
            bool hit;
            int  way;
            if (kCoherent) {
                hit = false;
                way = -1;
                bool pending = want;
                uint32_t rounds = 0;
                while (__ballot(pending)) {
                    if (++rounds > kMaxRounds) {                     // a set never came free: report a miss
                        if (pending) __hip_atomic_fetch_or(tb.flags, (uint32_t)HPS_FLAG_STUCK_SET, __ATOMIC_RELAXED,
                                                           __HIP_MEMORY_SCOPE_AGENT);
                        break;
                    }
                    const uint32_t v1 = pending ? ld_agent(seq_of(tb, set)) : 0u;
                    const bool busy = pending && (v1 & 1u);          // a writer holds the set: look again later
                    shared_acquire();                                // the word is read before any key or row
                    const int w = probe_wave<W, KPW, true>(tb.K, key, set, pending && !busy);
                    const bool found = w >= 0;
                    const uint64_t fmask = __ballot(found);
                    if (lane < 2) s_retry[wave][lane] = 0u;
                    if (found) {
                        const int r = rank_in(fmask);
                        s_src[wave][r] = (uint64_t)set * W + (uint32_t)w;
                        s_dst[wave][r] = pos;
                        s_set[wave][r] = set;
                        s_v1[wave][r]  = v1;
                    }
                    wave_lds_fence();
                    if (fmask) {
                        const uint32_t nf = (uint32_t)__popcll(fmask);
                        if (kD != 0 || g.passes8 == 1)
                            copy_rows_checked<U, kD, false>(g, tb.V, a.out, &s_src[wave][0], &s_dst[wave][0], &s_set[wave][0],
                                                            &s_v1[wave][0], tb.sc, nf, &s_retry[wave][0]);
                        else
                            copy_rows_checked<(U > 16 ? 16 : U), 0, true>(g, tb.V, a.out, &s_src[wave][0], &s_dst[wave][0], &s_set[wave][0],
                                                          &s_v1[wave][0], tb.sc, nf, &s_retry[wave][0]);
                    }
                    wave_lds_fence();
                    bool again = false;
                    if (found) {
                        const int r = rank_in(fmask);
                        again = (s_retry[wave][r >> 5] >> (r & 31)) & 1u;
                        if (!again) { hit = true; way = w; }
                    }
                    pending = busy || again;                         // a clean miss is final
                    wave_lds_fence();
                    if (__ballot(pending)) __builtin_amdgcn_s_sleep(2);
                }
            } else {
                way = probe_wave<W, KPW>(tb.K, key, set, want);
                hit = way >= 0;
            }

            const uint64_t missmask = __ballot(live && !hit);
            if (live && !hit) {
                const int r = rank_in(missmask);
                s_mpos[wave][r] = pos;
                s_mkey[wave][r] = key;
            }
            if (lane == 0) s_wcnt[wave] = (uint32_t)__popcll(missmask);
            // Alg. 2: refresh the counter.  A plain store: the XCD's write-back L2 merges the many stores
            // a hot key draws (an agent-scope store per hit serialises them at the memory side and
            // triples the kernel time); they reach memory at the latest when the kernel ends.
            if (kFull && tb.T && hit) tb.T[(uint64_t)set * W + (uint32_t)way] = g_call;

            if (kCoherent) {
                __syncthreads();                           // rows were copied inside the retry loop
            } else {
                const uint64_t hitmask = __ballot(hit);
                const uint32_t nh      = (uint32_t)__popcll(hitmask);
                if (hit) {
                    const int r = rank_in(hitmask);
                    s_src[wave][r] = (uint64_t)set * W + (uint32_t)way;
                    s_dst[wave][r] = pos;
                }
                wave_lds_fence();
                if (lane == 0) __hip_atomic_fetch_add(&s_ready, 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
                if (nh) copy_rows<U, kD>(g, tb.V, a.out, &s_src[wave][0], &s_dst[wave][0], nh);
            }
        } else {
            if (kCoherent) {
                __syncthreads();
            } else {
                // every worker wave of the work-group reaches its increment (none leaves early), so this ends
                while (__hip_atomic_load(&s_ready, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP) < (uint32_t)WPB)
                    __builtin_amdgcn_s_sleep(2);
            }
            uint32_t total = 0;
#pragma unroll
            for (int w = 0; w < WPB; ++w) total += s_wcnt[w];
            uint64_t old = 0;
            if (lane == 0)
                old = __hip_atomic_fetch_add(a.slot, (1ull << 32) | (uint64_t)total, __ATOMIC_RELAXED,
                                             __HIP_MEMORY_SCOPE_AGENT);
            old = (uint64_t)shfl64((int64_t)old, 0);
            uint32_t o = (uint32_t)old;
#pragma unroll
            for (int w = 0; w < WPB; ++w) {
                const uint32_t c = s_wcnt[w];
                for (uint32_t j = (uint32_t)lane; j < c; j += kWave) {
                    a.miss_idx[o + j]  = s_mpos[w][j];
                    a.miss_keys[o + j] = s_mkey[w][j];
                }
                o += c;
            }
            if ((uint32_t)(old >> 32) + 1u == a.n_tiles) {   // every tile has added its count (and read g)
                finish_call(a, (uint32_t)old + total, lane);
            }
            if (!kCoherent && many_tiles && lane == 0) s_ready = 0u;
        }
        if (kCoherent || many_tiles) __syncthreads();   // LDS lists are reused by the next tile
    }
}

// Query with in-tile deduplication (the paper deduplicates a batch before the lookup, Sec. 2.2;
// here each tile of WPB*64 positions does it in LDS).  An LDS hash table (2 slots per position,
// 64-bit compare-and-swap, linear probing) elects one representative position per distinct key of
// the tile.  Only representatives probe the cache and only their rows are read from memory; a
// row is then stored to the representative's position and to every duplicate position, which
// hang off the representative in an LDS linked list (atomic exchange on the list head).  Misses
// are reported per position as in query_kernel, and the helper wave does the same counter work.
template <int W, int U, int WPB>
__global__ void __launch_bounds__((WPB + 1) * kWave) query_dedup_kernel(const QueryArgs a) {
    constexpr int kTile = kWave * WPB;
    constexpr int kHash = 2 * kTile;
    static_assert((kHash & (kHash - 1)) == 0, "the LDS table is probed with a mask: its size must be a power of two");
    constexpr uint32_t kNil = 0xFFFFFFFFu;
    constexpr uint64_t kMissed = ~0ull;
    __shared__ unsigned long long h_key[kHash];
    __shared__ uint32_t h_own[kHash];
    __shared__ uint64_t r_slot[kTile];
    __shared__ uint32_t head[kTile];
    __shared__ uint32_t nxt[kTile];
    __shared__ uint64_t s_src[WPB][kWave];
    __shared__ uint32_t s_rep[WPB][kWave];
    __shared__ int64_t  s_mkey[WPB][kWave];
    __shared__ uint32_t s_mpos[WPB][kWave];
    __shared__ uint32_t s_wcnt[WPB];

    const int lane = lane_id();
    const int wave = (int)(threadIdx.x / kWave);
    const RowGeom g = a.g;
    const uint32_t rpi = (uint32_t)kWave >> g.lprShift;
    const uint32_t sub = (uint32_t)lane >> g.lprShift;
    const uint32_t cl  = (uint32_t)lane & (g.LPR - 1);

    for (uint32_t tile = blockIdx.x; tile < a.n_tiles; tile += gridDim.x) {
        const uint32_t t  = tile / a.tiles_per_table;
        const uint32_t lt = tile - t * a.tiles_per_table;
        const uint32_t pos0 = t * a.B + lt * WPB * a.kpw;      // position of this tile's first key
        if (wave < WPB) {
            const Table   &tb   = a.tab[t];
            const uint32_t g_call = tb.T ? *tb.gdev + 1u : 0u;               // as in query_kernel
            const uint32_t tid  = (uint32_t)wave * a.kpw + (uint32_t)lane;   // index in the tile (idle lanes alias, unused)
            const uint32_t b    = lt * WPB * a.kpw + tid;
            const bool     inb  = lane < (int)a.kpw && b < a.B;
            const uint32_t pos  = pos0 + tid;
            const int64_t  key  = inb ? a.keys[pos] : kEmpty;
            const bool     live = inb && (!a.n_dev || b < *a.n_dev);
            const bool     want = live && !is_reserved(key);
            const uint64_t h    = mix64((uint64_t)key);
            const uint32_t hs   = (uint32_t)(h >> 32);
            const uint32_t set  = want ? (tb.smask ? (hs & tb.smask) : (hs % tb.S)) : 0u;

            for (uint32_t i = threadIdx.x; i < (uint32_t)kHash; i += kTile) h_key[i] = (unsigned long long)kEmpty;
            head[threadIdx.x] = kNil;
            __syncthreads();                                    // #1 table cleared

            bool is_rep = false;
            uint32_t my = 0;
            if (want) {
                uint32_t slot = (uint32_t)h & (kHash - 1);
                for (;;) {
                    const unsigned long long old =
                        atomicCAS(&h_key[slot], (unsigned long long)kEmpty, (unsigned long long)key);
                    if (old == (unsigned long long)kEmpty) { is_rep = true; h_own[slot] = tid; break; }
                    if (old == (unsigned long long)key) break;
                    slot = (slot + 1) & (kHash - 1);
                }
                my = slot;
            }
            __syncthreads();                                    // #2 representatives elected
            const uint32_t rep = is_rep ? tid : (want ? h_own[my] : tid);
            const int way = probe_wave<W, kWave>(tb.K, key, set, is_rep);
            if (is_rep) r_slot[tid] = way >= 0 ? (uint64_t)set * W + (uint32_t)way : kMissed;
            if (tb.T && is_rep && way >= 0) tb.T[(uint64_t)set * W + (uint32_t)way] = g_call;
            __syncthreads();                                    // #3 probe results visible
            const uint64_t res = want ? r_slot[rep] : kMissed;
            const bool hit = res != kMissed;

            const uint64_t missmask = __ballot(live && !hit);
            if (live && !hit) {
                const int r = rank_in(missmask);
                s_mpos[wave][r] = pos;
                s_mkey[wave][r] = key;
            }
            if (lane == 0) s_wcnt[wave] = (uint32_t)__popcll(missmask);

            if (hit && !is_rep) nxt[tid] = atomicExch(&head[rep], tid);     // join the representative's list
            const uint64_t repmask = __ballot(hit && is_rep);
            const uint32_t nh = (uint32_t)__popcll(repmask);
            if (hit && is_rep) {
                const int r = rank_in(repmask);
                s_src[wave][r] = res;
                s_rep[wave][r] = tid;
            }
            __syncthreads();                                    // #4 lists complete; helper starts

            const float *__restrict__ V = tb.V;
            for (uint32_t pass = 0; pass < g.passes; ++pass) {
                uint32_t chunk = cl + pass * g.LPR;
                chunk = chunk < g.C ? chunk : 0u;
                const uint32_t off = chunk * 4;
                for (uint32_t e0 = 0; e0 < nh; e0 += rpi * U) {
                    f32x4 buf[U];
                    uint32_t rp[U];
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        uint32_t e = e0 + u * rpi + sub;
                        e = e < nh ? e : 0u;
                        rp[u] = s_rep[wave][e];
                        buf[u] = *reinterpret_cast<const f32x4 *>(V + s_src[wave][e] * g.d + off);
                    }
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        __builtin_nontemporal_store(
                            buf[u], reinterpret_cast<f32x4 *>(a.out + (uint64_t)(pos0 + rp[u]) * g.d + off));
                        uint32_t p = head[rp[u]];
                        while (p != kNil) {                     // duplicate positions of this key
                            __builtin_nontemporal_store(
                                buf[u], reinterpret_cast<f32x4 *>(a.out + (uint64_t)(pos0 + p) * g.d + off));
                            p = nxt[p];
                        }
                    }
                }
            }
        } else {
            __syncthreads();
            __syncthreads();
            __syncthreads();
            __syncthreads();
            uint32_t total = 0;
#pragma unroll
            for (int w = 0; w < WPB; ++w) total += s_wcnt[w];
            uint64_t old = 0;
            if (lane == 0)
                old = __hip_atomic_fetch_add(a.slot, (1ull << 32) | (uint64_t)total, __ATOMIC_RELAXED,
                                             __HIP_MEMORY_SCOPE_AGENT);
            old = (uint64_t)shfl64((int64_t)old, 0);
            uint32_t o = (uint32_t)old;
#pragma unroll
            for (int w = 0; w < WPB; ++w) {
                const uint32_t c = s_wcnt[w];
                for (uint32_t j = (uint32_t)lane; j < c; j += kWave) {
                    a.miss_idx[o + j]  = s_mpos[w][j];
                    a.miss_keys[o + j] = s_mkey[w][j];
                }
                o += c;
            }
            if ((uint32_t)(old >> 32) + 1u == a.n_tiles) finish_call(a, (uint32_t)old + total, lane);
        }
        __syncthreads();                                        // #5 LDS is reused by the next tile
    }
}

// ------------------------------------------------------------------ insert / update

struct WriteArgs {
    Table           tab;
    const int64_t  *keys;
    const float    *vals;
    const uint32_t *n_dev;      // optional device-side batch length
    uint32_t        n;
    RowGeom         g;
};

// Replace (Alg. 3).  The first KPW lanes of a wave own one key each; all 64 lanes copy rows.  A
// pending lane takes its set's sequence word (the paper's slabset lock, Sec. 4.1) with one
// fetch-or of bit 0: it owns the set if the bit was clear.  The owners' sets are then searched with the wave-wide probe and their
// counters read in the same round trip, new keys get their slot (key, counter, stamp) and row,
// and every owner lets go again: word + 2 if it changed the set, the old word if the key was
// already there.  Lanes that did not get their set search it without owning it before every
// further attempt.  No lane ever waits while the wave owns a set: each round every pending lane
// tries once, the owners' rows are copied by the whole wave, the sets are released, and the
// others try again.  KPW = 16: four times as many waves as keys / 64 share the row copies, and a
// wave's chain of dependent memory round trips is two copy groups long instead of eight.
template <int W, int KPW>
__global__ void __launch_bounds__(kBlock) insert_kernel(const WriteArgs a) {
    __shared__ uint64_t s_dst[kWavesPerWg][kWave];
    __shared__ uint32_t s_srcrow[kWavesPerWg][kWave];
    __shared__ uint32_t s_owner[kWavesPerWg][kWave * 2];

    const int lane = lane_id();
    const int wave = (int)(threadIdx.x / kWave);
    const RowGeom g = a.g;
    const Table tb = a.tab;
    uint32_t n = a.n;
    if (a.n_dev) {
        const uint32_t nd = *a.n_dev;
        n = nd < n ? nd : n;
    }
    const uint32_t n_tiles = (n + KPW - 1) / KPW;
    const uint32_t wave_global = blockIdx.x * kWavesPerWg + wave;
    const uint32_t n_waves = gridDim.x * kWavesPerWg;
    const uint32_t g_now = tb.T ? *tb.gdev : 0u;            // Alg. 3 stamps with the current iteration count

    for (uint32_t tile = wave_global; tile < n_tiles; tile += n_waves) {
        const uint32_t i = tile * KPW + lane;
        const bool mine = lane < KPW && i < n;
        const int64_t key = mine ? a.keys[i] : kEmpty;
        bool pending = mine && !is_reserved(key);
        const uint64_t h = mix64((uint64_t)key);
        const uint32_t hs = (uint32_t)(h >> 32);
        const uint32_t set = pending ? (tb.smask ? (hs & tb.smask) : (hs % tb.S)) : 0u;

        // Copies of a key inside this wave: all of them write their lane number into the key's
        // hash slot, the one whose number stays carries the key, the others drop out (Alg. 3
        // ignores a key that is already there, so only one copy can ever take effect).  A slot
        // shared by different keys thins nothing.
        if (pending) s_owner[wave][h & (kWave * 2 - 1)] = (uint32_t)lane;
        wave_lds_fence();
        const int o = pending ? (int)s_owner[wave][h & (kWave * 2 - 1)] : lane;
        const int64_t ko = shfl64(key, o);
        if (pending && o != lane && ko == key) pending = false;
        wave_lds_fence();

        uint32_t rounds = 0;
        while (__ballot(pending)) {
            if (++rounds > kMaxRounds) {                             // a set never came free: skip these keys
                if (pending) __hip_atomic_fetch_or(tb.flags, (uint32_t)HPS_FLAG_STUCK_SET, __ATOMIC_RELAXED,
                                                   __HIP_MEMORY_SCOPE_AGENT);
                break;
            }
            if (rounds > 1) {
                // A lane that lost its first attempt looks before it tries again: a key given many
                // times (a miss list carries every occurrence) is found by all but the first
                // without taking the word, instead of each occurrence owning the set in turn.
                const int seen = probe_wave<W, KPW, true>(tb.K, key, set, pending);
                if (pending && seen >= 0) {
                    if (tb.T) st_agent(tb.T + (uint64_t)set * W + (uint32_t)seen, g_now);    // Alg. 3: refresh
                    pending = false;
                }
            }
            // one 64-bit atomic on the set's {seq, ctr} word: takes the set and reads its counter
            uint64_t word = 1ull;
            if (pending)
                word = __hip_atomic_fetch_or(reinterpret_cast<uint64_t *>(seq_of(tb, set)), 1ull, __ATOMIC_RELAXED,
                                             __HIP_MEMORY_SCOPE_AGENT);
            const uint32_t old = (uint32_t)word;
            const uint32_t c = (uint32_t)(word >> 32);
            const bool own = pending && !(old & 1u);
            if (!__ballot(own)) {
                __builtin_amdgcn_s_sleep(8);
                continue;
            }
            shared_acquire();                                        // the word is owned before the set is read
            int way = probe_wave<W, KPW, true>(tb.K, key, set, own);
            bool fresh = own && way < 0;
            if (tb.T) {                                              // LRU policy (Alg. 3)
                if (fresh) {
                    int empty_way = -1;
                    uint32_t best = 0;
                    int oldest = 0;
#pragma unroll
                    for (int w = W - 1; w >= 0; --w) {
                        const int64_t kw = ld_agent(tb.K + (uint64_t)set * W + w);
                        const uint32_t age = g_now - ld_agent(tb.T + (uint64_t)set * W + w);
                        if (kw == kEmpty) empty_way = w;             // ends as the lowest empty way
                        if (w == W - 1 || age >= best) { best = age; oldest = w; }   // largest age, lowest way on ties
                    }
                    way = empty_way >= 0 ? empty_way : oldest;
                }
                if (own) st_agent(tb.T + (uint64_t)set * W + (uint32_t)way, g_now);
            } else if (fresh) {
                way = (int)(c & (W - 1));                            // victim counter
            }
            const uint64_t freshmask = __ballot(fresh);
            if (fresh) {
                st_agent(tb.K + (uint64_t)set * W + (uint32_t)way, key);
                const int r = rank_in(freshmask);
                s_dst[wave][r] = (uint64_t)set * W + (uint32_t)way;
                s_srcrow[wave][r] = i;
            }
            if (freshmask) {
                wave_lds_fence();
                copy_rows_shared<8>(g, a.vals, tb.V, &s_srcrow[wave][0], &s_dst[wave][0],
                                    (uint32_t)__popcll(freshmask));
                wave_lds_fence();
            }
            shared_release();                                        // rows and keys land before the words move on
            if (own) {
                // let go: a changed set gets seq + 2 and ctr + 1 in one store, an unchanged one its old word
                st_agent(reinterpret_cast<uint64_t *>(seq_of(tb, set)),
                         fresh ? (((uint64_t)(c + 1u) << 32) | (uint64_t)(old + 2u)) : word);
                pending = false;
            }
        }
    }
}

// Update (Alg. 4) with one lock acquisition per run of lanes that share a set.  Key batches that
// come from a dump are in slot order: eight neighbouring keys belong to one set, and taking the
// set's word once per key would serialise them over eight rounds.  Here adjacent pending lanes
// with the same set form a group; the group's first lane reads the word and, if any lane of the
// group found its key, takes it once; all those lanes' rows are then written under that one hold.
// Two lanes of a group that found the same slot (a key given twice) are thinned to one per round.
// Lanes of different groups that meet on a set compete by compare-and-swap on its word; no lane
// waits while its wave owns a set.
template <int W, int KPW>
__global__ void __launch_bounds__(kBlock) update_kernel(const WriteArgs a) {
    __shared__ uint64_t s_dst[kWavesPerWg][kWave];
    __shared__ uint32_t s_srcrow[kWavesPerWg][kWave];

    const int lane = lane_id();
    const int wave = (int)(threadIdx.x / kWave);
    const RowGeom g = a.g;
    const Table tb = a.tab;
    uint32_t n = a.n;
    if (a.n_dev) {
        const uint32_t nd = *a.n_dev;
        n = nd < n ? nd : n;
    }
    const uint32_t n_tiles = (n + KPW - 1) / KPW;
    const uint32_t wave_global = blockIdx.x * kWavesPerWg + wave;
    const uint32_t n_waves = gridDim.x * kWavesPerWg;
    const uint64_t le_lane = lane == 63 ? ~0ull : ((2ull << lane) - 1);     // bits 0..lane

    for (uint32_t tile = wave_global; tile < n_tiles; tile += n_waves) {
        const uint32_t i = tile * KPW + lane;
        const bool mine = lane < KPW && i < n;
        const int64_t key = mine ? a.keys[i] : kEmpty;
        bool pending = mine && !is_reserved(key);
        const uint32_t set = pending ? set_of(key, tb.S, tb.smask) : 0u;

        uint32_t rounds = 0;
        while (const uint64_t pendmask = __ballot(pending)) {
            if (++rounds > kMaxRounds) {                             // a set never came free: skip these keys
                if (pending) __hip_atomic_fetch_or(tb.flags, (uint32_t)HPS_FLAG_STUCK_SET, __ATOMIC_RELAXED,
                                                   __HIP_MEMORY_SCOPE_AGENT);
                break;
            }
            // groups: maximal runs of adjacent pending lanes with equal set
            const uint32_t prev_set = (uint32_t)__shfl_up((int)set, 1, kWave);
            const int prev_pend = __shfl_up((int)pending, 1, kWave);
            const bool start = pending && (lane == 0 || !prev_pend || prev_set != set);
            const uint64_t startmask = __ballot(start);
            const int leader = pending ? 63 - __builtin_clzll(startmask & le_lane) : lane;
            const uint64_t le_leader = leader == 63 ? ~0ull : ((2ull << leader) - 1);
            const uint64_t above = startmask & ~le_leader;
            const uint64_t lt_end = above ? ((1ull << __builtin_ctzll(above)) - 1) : ~0ull;
            const uint64_t gmask = pendmask & lt_end & ~(le_leader >> 1);    // lanes leader .. end-1 that are pending
            const bool is_leader = pending && lane == leader;

            uint32_t v = is_leader ? ld_agent(seq_of(tb, set)) : 0u;
            v = (uint32_t)__shfl((int)v, leader, kWave);
            const bool busy = pending && (v & 1u);
            shared_acquire();                                        // the word is read before the keys
            int way = -1;
            if (pending && !busy) {
#pragma unroll
                for (int w = 0; w < W; ++w)
                    if (ld_agent(tb.K + (uint64_t)set * W + w) == key) way = w;
                if (way < 0) pending = false;                        // not cached: ignored
            }
            bool winner = pending && !busy && way >= 0;
#pragma unroll
            for (int w = 0; w < W; ++w) {                            // one lane per slot and round
                const uint64_t m = __ballot(winner && way == w) & gmask;
                if (winner && way == w && lane != __builtin_ctzll(m)) winner = false;
            }
            const bool group_needs = (__ballot(winner) & gmask) != 0;
            bool won = false;
            if (is_leader && !busy && group_needs) {
                uint32_t expect = v;
                won = __hip_atomic_compare_exchange_strong(seq_of(tb, set), &expect, v + 1u, __ATOMIC_RELAXED,
                                                           __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            const bool gwon = __shfl((int)won, leader, kWave) != 0;
            const bool act = winner && gwon;
            const uint64_t actmask = __ballot(act);
            if (actmask) {
                shared_acquire();
                if (act) {
                    const int r = rank_in(actmask);
                    s_dst[wave][r] = (uint64_t)set * W + (uint32_t)way;
                    s_srcrow[wave][r] = i;
                }
                wave_lds_fence();
                copy_rows_shared<8>(g, a.vals, tb.V, &s_srcrow[wave][0], &s_dst[wave][0],
                                    (uint32_t)__popcll(actmask));
                wave_lds_fence();
                shared_release();                                    // rows land before the word moves on
                if (won) st_agent(seq_of(tb, set), v + 2u);
                if (act) pending = false;
            }
        }
    }
}

// ------------------------------------------------------------------ small kernels

__global__ void set_u32_kernel(uint32_t *p, uint32_t v) { *p = v; }

__global__ void fill_keys_kernel(int64_t *K, uint64_t n, int64_t v) {
    for (uint64_t i = blockIdx.x * (uint64_t)blockDim.x + threadIdx.x; i < n;
         i += (uint64_t)gridDim.x * blockDim.x)
        K[i] = v;
}

// Export / import of the victim counters: ctr[s] <-> the upper half of the set's {seq, ctr} word.
// An import leaves every sequence word at zero (no writer, nothing in flight).
__global__ void counters_out_kernel(const uint32_t *sc, uint64_t S, uint32_t *ctr) {
    for (uint64_t i = blockIdx.x * (uint64_t)blockDim.x + threadIdx.x; i < S;
         i += (uint64_t)gridDim.x * blockDim.x)
        ctr[i] = sc[2 * i + 1];
}
__global__ void counters_in_kernel(uint32_t *sc, uint64_t S, const uint32_t *ctr) {
    for (uint64_t i = blockIdx.x * (uint64_t)blockDim.x + threadIdx.x; i < S;
         i += (uint64_t)gridDim.x * blockDim.x) {
        sc[2 * i] = 0u;
        sc[2 * i + 1] = ctr[i];
    }
}

// Dump (Sec. 4.2): compact the non-empty keys of a slot range.  A work-group takes a tile of
// 256*KPT consecutive slots, keeps KPT keys per lane in registers, and needs one counter atomic
// per tile (same counter-word scheme as query).  The output keeps slot order inside a tile, so the
// keys of one set stay next to each other: an Update over the dumped keys then takes each set once
// for all its keys (update_kernel groups such runs) and writes the rows of a set, which are
// contiguous in memory, together.
template <int KPT>
__global__ void __launch_bounds__(kBlock) dump_kernel(const int64_t *__restrict__ K, uint64_t first,
                                                      uint64_t n_slots, int64_t *keys_out,
                                                      uint32_t *n_out, uint64_t *slot,
                                                      uint32_t n_tiles) {
    constexpr uint32_t kTileSlots = kBlock * KPT;
    constexpr int kCnt = KPT * kWavesPerWg;                // one count per (j, wave)
    static_assert(kCnt <= kBlock, "the count scan gives every count its own thread");
    __shared__ uint32_t s_cnt[kCnt];                       // [j][wave] counts, then exclusive prefixes
    __shared__ uint32_t s_wtot[kWavesPerWg];
    __shared__ uint32_t s_base;
    const int lane = lane_id();
    const int wave = (int)(threadIdx.x / kWave);
    for (uint32_t tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        int64_t key[KPT];
#pragma unroll
        for (int j = 0; j < KPT; ++j) {
            const uint32_t q = (uint32_t)j * kBlock + threadIdx.x;
            const uint64_t i = (uint64_t)tile * kTileSlots + q;
            key[j] = i < n_slots ? __builtin_nontemporal_load(K + first + i) : kEmpty;     // read once
        }
#pragma unroll
        for (int j = 0; j < KPT; ++j) {
            const uint64_t m = __ballot(key[j] != kEmpty);
            if (lane == 0) s_cnt[j * kWavesPerWg + wave] = (uint32_t)__popcll(m);
        }
        __syncthreads();
        // exclusive scan of the kCnt counts over the work-group: inside each wave, then across waves
        const uint32_t c = threadIdx.x < (uint32_t)kCnt ? s_cnt[threadIdx.x] : 0u;
        uint32_t incl = c;
#pragma unroll
        for (int o = 1; o < kWave; o <<= 1) {
            const uint32_t up = (uint32_t)__shfl_up((int)incl, o, kWave);
            if (lane >= o) incl += up;
        }
        if (lane == kWave - 1) s_wtot[wave] = incl;
        __syncthreads();
        uint32_t woff = 0, total = 0;
#pragma unroll
        for (int w = 0; w < kWavesPerWg; ++w) {
            const uint32_t t = s_wtot[w];
            if (w < wave) woff += t;
            total += t;
        }
        if (threadIdx.x < (uint32_t)kCnt) s_cnt[threadIdx.x] = woff + incl - c;
        if (threadIdx.x == 0) {
            const uint64_t old = __hip_atomic_fetch_add(slot, (1ull << 32) | (uint64_t)total,
                                                        __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            s_base = (uint32_t)old;
            if ((uint32_t)(old >> 32) + 1u == n_tiles) {
                *n_out = (uint32_t)old + total;
                __hip_atomic_store(slot, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
        __syncthreads();
        const uint32_t base = s_base;
#pragma unroll
        for (int j = 0; j < KPT; ++j) {
            const uint64_t m = __ballot(key[j] != kEmpty);
            if (key[j] != kEmpty)
                __builtin_nontemporal_store(key[j], keys_out + base + s_cnt[j * kWavesPerWg + wave] + (uint32_t)rank_in(m));
        }
        __syncthreads();
    }
}

// Lower-tier stand-in: four consecutive elements of one row per thread.
__global__ void backing_kernel(const int64_t *__restrict__ keys, uint32_t n,
                               const uint32_t *__restrict__ n_dev, uint32_t d, uint32_t version,
                               float *rows, const uint32_t *__restrict__ scatter_idx,
                               float *scatter_out) {
    if (n_dev) {
        const uint32_t nd = *n_dev;
        n = nd < n ? nd : n;
    }
    const uint32_t C = d / 4;
    const uint64_t total = (uint64_t)n * C;
    for (uint64_t t = blockIdx.x * (uint64_t)blockDim.x + threadIdx.x; t < total;
         t += (uint64_t)gridDim.x * blockDim.x) {
        const uint32_t i = (uint32_t)(t / C);
        const uint32_t c = (uint32_t)(t - (uint64_t)i * C);
        const uint64_t k = (uint64_t)keys[i];
        float x[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const uint64_t j = c * 4 + e;
            const uint64_t z = mix64(k ^ mix64((((uint64_t)version << 32) | j) + 0x9E3779B97F4A7C15ull));
            x[e] = (float)((int32_t)(z >> 40) - (1 << 23)) * 0x1.0p-23f;   // exact: 24-bit integer * 2^-23
        }
        const f32x4 v4 = {x[0], x[1], x[2], x[3]};
        if (rows) *reinterpret_cast<f32x4 *>(rows + (uint64_t)i * d + c * 4) = v4;
        if (scatter_idx)
            *reinterpret_cast<f32x4 *>(scatter_out + (uint64_t)scatter_idx[i] * d + c * 4) = v4;
    }
}

// ------------------------------------------------------------------ measurement kernels (hps_membench.h)

// The row movement of query_kernel's plain variant alone: same tile shape, same copy loop, but the
// source slot of every position is given, so nothing is hashed, probed or compacted.
template <int U, int WPB, int kD>
__global__ void __launch_bounds__(WPB * kWave) membench_gather_kernel(const float *__restrict__ rows,
                                                                      const uint32_t *__restrict__ slot_of, uint32_t n,
                                                                      uint32_t kpw, const RowGeom g, float *__restrict__ out) {
    __shared__ uint32_t s_src[WPB][kWave];
    __shared__ uint32_t s_dst[WPB][kWave];
    const int lane = lane_id();
    const int wave = (int)(threadIdx.x / kWave);
    const uint32_t pos = (blockIdx.x * WPB + wave) * kpw + lane;
    const bool inb = lane < (int)kpw && pos < n;
    const uint32_t sl = inb ? slot_of[pos] : 0xFFFFFFFFu;
    const bool hit = sl != 0xFFFFFFFFu;
    const uint64_t hitmask = __ballot(hit);
    const uint32_t nh = (uint32_t)__popcll(hitmask);
    if (hit) {
        const int r = rank_in(hitmask);
        s_src[wave][r] = sl;
        s_dst[wave][r] = pos;
    }
    wave_lds_fence();
    if (nh) copy_rows<U, kD>(g, rows, out, &s_src[wave][0], &s_dst[wave][0], nh);
}

// Half of that row movement: kReads = true issues the group's row loads and stores nothing (the
// loaded words are folded into one value that is stored only if it equals a constant the data never
// produces, so the loads stay); kReads = false stores a register pattern to the same destination
// rows and loads nothing.  Work distribution, group size and access width are copy_rows'.
template <int U, int WPB, bool kReads>
__global__ void __launch_bounds__(WPB * kWave) membench_half_kernel(const float *__restrict__ rows,
                                                                    const uint32_t *__restrict__ slot_of, uint32_t n,
                                                                    uint32_t kpw, float *__restrict__ out) {
    __shared__ uint32_t s_src[WPB][kWave];
    __shared__ uint32_t s_dst[WPB][kWave];
    const uint32_t lane = (uint32_t)lane_id();
    const int wave = (int)(threadIdx.x / kWave);
    const uint32_t pos = (blockIdx.x * WPB + wave) * kpw + lane;
    const bool inb = lane < kpw && pos < n;
    const uint32_t sl = inb ? slot_of[pos] : 0xFFFFFFFFu;
    const bool hit = sl != 0xFFFFFFFFu;
    const uint64_t hitmask = __ballot(hit);
    const uint32_t cnt = (uint32_t)__popcll(hitmask);
    if (hit) {
        const int r = rank_in(hitmask);
        s_src[wave][r] = sl;
        s_dst[wave][r] = pos;
    }
    wave_lds_fence();
    const uint32_t sub = lane >> 5, off = (lane & 31u) * 4u;            // 512-byte rows: 32 lanes per row, 2 rows per wave load
    for (uint32_t e0 = 0; e0 < cnt; e0 += 2 * U) {
        f32x4 buf[U];
        uint32_t ent[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint32_t e = e0 + 2 * u + sub;
            ent[u] = e < cnt ? e : 0xFFFFFFFFu;
            if (kReads) buf[u] = *reinterpret_cast<const f32x4 *>(rows + (uint64_t)s_src[wave][e < cnt ? e : 0u] * 128 + off);
            else        buf[u] = f32x4{(float)lane, (float)u, (float)e, 1.0f};
        }
        if (kReads) {
            __builtin_amdgcn_s_waitcnt(0x0F70);
            f32x4 acc = buf[0];
#pragma unroll
            for (int u = 1; u < U; ++u) acc += buf[u];
            if (acc.x == 1.2345678e-30f && acc.y == acc.x) out[0] = acc.z;     // never true for the backing rows
        } else {
#pragma unroll
            for (int u = 0; u < U; ++u)
                if (ent[u] != 0xFFFFFFFFu)
                    __builtin_nontemporal_store(buf[u], reinterpret_cast<f32x4 *>(out + (uint64_t)s_dst[wave][ent[u]] * 128 + off));
        }
    }
}

template <int U, bool kNT>
__global__ void __launch_bounds__(kBlock) membench_copy_kernel(const f32x4 *__restrict__ src, f32x4 *__restrict__ dst, uint64_t n16) {
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    uint64_t i = blockIdx.x * (uint64_t)blockDim.x + threadIdx.x;
    for (; i + (U - 1) * stride < n16; i += U * stride) {
        f32x4 x[U];
#pragma unroll
        for (int u = 0; u < U; ++u) x[u] = kNT ? __builtin_nontemporal_load(src + i + u * stride) : src[i + u * stride];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (kNT) __builtin_nontemporal_store(x[u], dst + i + u * stride);
            else dst[i + u * stride] = x[u];
        }
    }
    for (; i < n16; i += stride) dst[i] = src[i];
}

// ------------------------------------------------------------------ host side

RowGeom make_geom(uint32_t d) {
    RowGeom g;
    g.d = d;
    g.C = d / 4;
    uint32_t lpr = 1, sh = 0;
    while (lpr < g.C && lpr < (uint32_t)kWave) { lpr <<= 1; ++sh; }
    g.LPR = lpr;
    g.lprShift = sh;
    g.passes = (g.C + lpr - 1) / lpr;
    g.C8 = d / 2;
    lpr = 1; sh = 0;
    while (lpr < g.C8 && lpr < (uint32_t)kWave) { lpr <<= 1; ++sh; }
    g.LPR8 = lpr;
    g.lpr8Shift = sh;
    g.passes8 = (g.C8 + lpr - 1) / lpr;
    return g;
}

bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

}  // namespace

struct hps_cache {
    uint64_t magic;
    int      device;
    uint64_t S;
    uint32_t W, d;
    int64_t  *K;
    float    *V;
    uint32_t *sc;                         // [S][2]: {sequence word, victim counter}
    uint64_t *ring;                       // 2 * kRing counter words, all zero between calls
    std::mutex word_mu;
    std::unordered_map<void *, uint32_t> word_of_stream;
    uint32_t word_half;                   // which half of `ring` is being handed out
    std::atomic<int> concurrent_writers;
    std::atomic<int> query_dedup;
    int      policy;                      // HPS_POLICY_*
    uint32_t *T;                          // access stamps (LRU policy), else nullptr
    uint32_t *flags;                      // device words: [0] HPS_FLAG_* bits, [1] g, the global iteration
                                          // count of Alg. 2 (one step per query call, LRU policy)
    int      n_cus;                       // compute units of the device
};

namespace {

hps_status_t check_handle(const hps_cache *c) {
    if (!c || c->magic != kMagic) return fail(HPS_ERR_INVALID_ARG, "invalid cache handle");
    int dev = -1;
    HIP_TRY(hipGetDevice(&dev));
    if (dev != c->device)
        return fail(HPS_ERR_INVALID_ARG, "cache was created on device " + std::to_string(c->device) +
                                             " but device " + std::to_string(dev) + " is current");
    return HPS_OK;
}

Table table_of(const hps_cache *c) {
    Table t;
    t.K = c->K;
    t.V = c->V;
    t.sc = c->sc;
    t.S = (uint32_t)c->S;
    t.smask = (c->S & (c->S - 1)) == 0 ? (uint32_t)(c->S - 1) : 0u;
    if (c->S == 1) t.smask = 0;           // S = 1: "h % 1" = 0 (a zero mask means "use modulo")
    t.T = c->T;
    t.gdev = c->flags + 1;
    t.flags = c->flags;
    return t;
}

// Counter word of query/dump calls on `stream`.  Calls on one stream run one after the other and
// each leaves its word at zero, so they can share one; calls on different streams may overlap and
// get different words.  The pool is two halves of kRing words: streams are given words of the
// current half in order of first sight; when a half is used up (kRing different stream handles,
// e.g. a caller that keeps creating streams) the table is forgotten and the other half is
// handed out, so a kernel still running with a word of the old half is never disturbed.
// A kernel captured into a graph keeps the word of the stream it was captured on.
uint64_t *counter_word(hps_cache *c, void *stream) {
    std::lock_guard<std::mutex> lk(c->word_mu);
    auto it = c->word_of_stream.find(stream);
    if (it == c->word_of_stream.end()) {
        if (c->word_of_stream.size() >= kRing) {
            c->word_of_stream.clear();
            c->word_half ^= 1u;
        }
        it = c->word_of_stream.emplace(stream, c->word_half * kRing + (uint32_t)c->word_of_stream.size()).first;
    }
    return c->ring + it->second;
}

// Launch shape of the query kernel: KPW keys per worker wave, row copy in groups of U wave loads,
// WPB worker waves per work-group.  Chosen from the batch size (measured on 256 CUs with 512-byte
// rows): small batches want many small work-groups, ~10^5 keys want 512-key tiles (half as many
// same-address counter atomics, which cost ~11 ns each and serialise).  U is large enough for a
// wave's whole share of 512-byte rows to be one group (26 wave loads for the 52 keys per wave of
// the 106,496-key batch, 32 for 64 keys per wave).
struct QueryShape { int kpw, u, wpb; };

QueryShape query_shape(uint64_t n, bool coherent, bool dedup) {
    if (coherent) {
        // The checked variant reads rows 8 bytes per lane (one 512-byte row per wave load) and pays two
        // dependent round trips per group (rows, then the sequence words again), so a wave's rows
        // should be ONE group: 64 keys per wave need 128 data registers, which 8 waves per
        // work-group (2 per SIMD, 256 registers each) leave room for and 9 do not.  Measured in the
        // stand-alone test bed on the 106,496-key batch: groups of 16 rows, 9 waves 27.5 us; groups
        // of 32, 8 waves 23.1 us; one group, 8 waves 21.6 us.
        // (1.7 M keys against a 64 GiB cache: 0.375 ms with this shape, 0.38-0.39 ms with groups of 16 or
        // 32 rows and 5 waves, 0.49 ms with one group and 5 waves)
        if (n < (1u << 16)) return QueryShape{64, 64, 4};
        return QueryShape{64, 64, 7};
    }
    // Large batches run several work-groups per CU one after the other; measured (us per launch) for
    // 425,984 / 851,968 / 1,703,936 keys of the hot cache, the 425,984-key streaming step and the
    // 26-table launch:
    //   4 waves, one group of 32   76.6 / 141.2 / 275.4 / 77.6 / 439
    //   8 waves, one group of 26   65.5 / 143.0 / 278.9 / 67.2 / 400
    //   7 waves, one group of 32   65.3 / 125.7 / 244.0 / 65.4 / 378
    //   8 waves, groups of 16      73.8 / 140.4 / 263.0 / 72.8 / 392
    // (a second group waits, with its own loads, for the first group's stores: one group per wave)
    // (4 against 8 workers, us per launch: 1,664 keys 5.6 / 6.1; 6,656 keys 6.9 / 7.3; 13,312 keys 8.3 / 8.3;
    //  39,936 keys 12.5 / 11.6; 53,248 keys 14.3 / 12.8; 62,400 keys 16.8 / 13.5)
    if (n < (1u << 14)) return QueryShape{64, 26, 4};
    if (n < (1u << 18)) return QueryShape{64, 26, 8};
    if (!dedup) return QueryShape{64, 32, 7};
    return QueryShape{64, 16, 8};                  // (the in-tile dedup needs a power-of-two tile)
}

template <int W, int KPW, int U, int WPB>
void launch_query_plain(const QueryArgs &a, bool dedup, bool full, hipStream_t st) {
    const uint32_t grid = a.n_tiles < (1u << 20) ? a.n_tiles : (1u << 20);
    const dim3 block((WPB + 1) * kWave);
    if constexpr ((WPB & (WPB - 1)) == 0) {      // (the shapes chosen for dedup mode have 4 or 8 worker waves)
        if (dedup && KPW == kWave) {
            hipLaunchKernelGGL((query_dedup_kernel<W, (WPB == 8 ? 4 : 8), WPB>), dim3(grid), block, 0, st, a);
            return;
        }
    }
    // any row width but 128: run-time row geometry needs more registers, so smaller groups under the 9-wave limit
    constexpr int UG = WPB == 8 ? 16 : U;
    if (a.g.d == 128) {
        if (full) hipLaunchKernelGGL((query_kernel<W, KPW, U, WPB, false, 128, true>), dim3(grid), block, 0, st, a);
        else     hipLaunchKernelGGL((query_kernel<W, KPW, U, WPB, false, 128, false>), dim3(grid), block, 0, st, a);
    } else {
        if (full) hipLaunchKernelGGL((query_kernel<W, KPW, UG, WPB, false, 0, true>), dim3(grid), block, 0, st, a);
        else     hipLaunchKernelGGL((query_kernel<W, KPW, UG, WPB, false, 0, false>), dim3(grid), block, 0, st, a);
    }
}

template <int W, int KPW, int U, int WPB>
void launch_query_checked(const QueryArgs &a, bool full, hipStream_t st) {
    const uint32_t grid = a.n_tiles < (1u << 20) ? a.n_tiles : (1u << 20);
    const dim3 block((WPB + 1) * kWave);
    // any row width but 128: run-time row geometry, groups of 16 wave loads keep the kernel inside its registers
    if (a.g.d == 128) {
        if (full) hipLaunchKernelGGL((query_kernel<W, KPW, U, WPB, true, 128, true>), dim3(grid), block, 0, st, a);
        else     hipLaunchKernelGGL((query_kernel<W, KPW, U, WPB, true, 128, false>), dim3(grid), block, 0, st, a);
    } else {
        if (full) hipLaunchKernelGGL((query_kernel<W, KPW, 16, WPB, true, 0, true>), dim3(grid), block, 0, st, a);
        else     hipLaunchKernelGGL((query_kernel<W, KPW, 16, WPB, true, 0, false>), dim3(grid), block, 0, st, a);
    }
}

template <int W>
hps_status_t launch_query_w(const QueryArgs &a, QueryShape q, bool coherent, bool dedup, bool full, hipStream_t st) {
    const int id = q.kpw * 10000 + q.u * 100 + q.wpb;
    if (coherent) {
        switch (id) {
            case 646404: launch_query_checked<W, 64, 64, 4>(a, full, st); break;
            case 646407: launch_query_checked<W, 64, 64, 7>(a, full, st); break;
            default: return fail(HPS_ERR_INVALID_ARG, "query shape not compiled in");
        }
    } else {
        switch (id) {
            case 642604: launch_query_plain<W, 64, 26, 4>(a, dedup, full, st); break;
            case 642608: launch_query_plain<W, 64, 26, 8>(a, dedup, full, st); break;
            case 641304: launch_query_plain<W, 64, 13, 4>(a, dedup, full, st); break;
            case 641308: launch_query_plain<W, 64, 13, 8>(a, dedup, full, st); break;
            case 643207: launch_query_plain<W, 64, 32, 7>(a, dedup, full, st); break;
            case 641608: launch_query_plain<W, 64, 16, 8>(a, dedup, full, st); break;
            default: return fail(HPS_ERR_INVALID_ARG, "query shape not compiled in");
        }
    }
    HIP_TRY(hipGetLastError());
    return HPS_OK;
}

hps_status_t launch_query(uint32_t W, const QueryArgs &a, QueryShape q, bool coherent, bool dedup,
                          bool full, hipStream_t st) {
    switch (W) {
        case 1:  return launch_query_w<1>(a, q, coherent, dedup, full, st);
        case 2:  return launch_query_w<2>(a, q, coherent, dedup, full, st);
        case 4:  return launch_query_w<4>(a, q, coherent, dedup, full, st);
        case 8:  return launch_query_w<8>(a, q, coherent, dedup, full, st);
        case 16: return launch_query_w<16>(a, q, coherent, dedup, full, st);
        case 32: return launch_query_w<32>(a, q, coherent, dedup, full, st);
        case 64: return launch_query_w<64>(a, q, coherent, dedup, full, st);
        default: return fail(HPS_ERR_INVALID_ARG, "unsupported ways");
    }
}

template <bool kInsert>
hps_status_t launch_write(hps_cache *c, const int64_t *keys, const float *vals, size_t n,
                          const uint32_t *n_dev, hipStream_t st) {
    WriteArgs a;
    a.tab = table_of(c);
    a.keys = keys;
    a.vals = vals;
    a.n_dev = n_dev;
    a.n = (uint32_t)n;
    a.g = make_geom(c->d);
    // insert: 16 keys per wave while 64 would leave fewer than 8 waves per CU
    // insert: 16 keys per wave (measured best from 1 K to 1 M keys: 8, 32 and 64 are 3-45 % slower)
    // update: 64 keys per wave, 16 for batches below 32,768 keys (measured: 8,192 rows 16 us instead
    // of 23 us, equal at 45,056, 8-18 % slower from 65,536 rows up and 9-55 % on a 40 GB refresh)
    const uint32_t kpw = kInsert ? (uint32_t)kInsertKpw : (n < 32768 ? 16u : (uint32_t)kWave);
    const uint64_t tiles = (n + kpw - 1) / kpw;
    uint64_t blocks = (tiles + kWavesPerWg - 1) / kWavesPerWg;
    if (blocks > (1u << 16)) blocks = 1u << 16;
    const dim3 grid((uint32_t)blocks), block(kBlock);
    switch (c->W) {
#define HPS_CASE(w)                                                                         \
    case w:                                                                                 \
        if (kInsert) hipLaunchKernelGGL((insert_kernel<w, kInsertKpw>), grid, block, 0, st, a); \
        else if (kpw == 16) hipLaunchKernelGGL((update_kernel<w, 16>), grid, block, 0, st, a);  \
        else hipLaunchKernelGGL((update_kernel<w, 64>), grid, block, 0, st, a);                 \
        break;
        HPS_CASE(1) HPS_CASE(2) HPS_CASE(4) HPS_CASE(8) HPS_CASE(16) HPS_CASE(32) HPS_CASE(64)
#undef HPS_CASE
        default: return fail(HPS_ERR_INVALID_ARG, "unsupported ways");
    }
    HIP_TRY(hipGetLastError());
    return HPS_OK;
}

hps_status_t write_call(hps_cache *c, const int64_t *keys, const float *vals, size_t n,
                        const uint32_t *n_dev, void *stream, bool insert) {
    if (hps_status_t s = check_handle(c)) return s;
    if (n == 0) return HPS_OK;
    if (n >= (1ull << 32)) return fail(HPS_ERR_INVALID_ARG, "n must be < 2^32");
    if (!keys || !vals) return fail(HPS_ERR_INVALID_ARG, "keys/vals must not be NULL when n > 0");
    if (!aligned(keys, 8) || !aligned(vals, 16) || !aligned(n_dev, 4))
        return fail(HPS_ERR_INVALID_ARG, "keys must be 8-byte and vals 16-byte aligned");
    hipStream_t st = static_cast<hipStream_t>(stream);
    return insert ? launch_write<true>(c, keys, vals, n, n_dev, st)
                  : launch_write<false>(c, keys, vals, n, n_dev, st);
}

}  // namespace

// ------------------------------------------------------------------ C ABI

extern "C" {

const char *hps_last_error(void) { return g_err.c_str(); }

hps_status_t hps_cache_create(size_t capacity, uint32_t ways, uint32_t dim, hps_cache_t **out_handle) {
    return hps_cache_create_policy(capacity, ways, dim, HPS_POLICY_VICTIM_COUNTER, out_handle);
}

hps_status_t hps_cache_create_policy(size_t capacity, uint32_t ways, uint32_t dim, int policy,
                                     hps_cache_t **out_handle) {
    if (!out_handle) return fail(HPS_ERR_INVALID_ARG, "out_handle is NULL");
    *out_handle = nullptr;
    if (policy != HPS_POLICY_VICTIM_COUNTER && policy != HPS_POLICY_LRU)
        return fail(HPS_ERR_INVALID_ARG, "unknown replacement policy");
    if (ways == 0 || ways > 64 || (ways & (ways - 1)) != 0)
        return fail(HPS_ERR_INVALID_ARG, "ways must be a power of two in [1, 64]");
    if (capacity == 0 || capacity % ways != 0)
        return fail(HPS_ERR_INVALID_ARG, "capacity must be a non-zero multiple of ways");
    if (capacity / ways >= (1ull << 31))
        return fail(HPS_ERR_INVALID_ARG, "capacity / ways must be < 2^31");
    if (dim == 0 || dim % 4 != 0) return fail(HPS_ERR_INVALID_ARG, "dim must be a non-zero multiple of 4");

    hps_cache *c = new (std::nothrow) hps_cache();
    if (!c) return fail(HPS_ERR_OOM, "host allocation failed");
    c->magic = kMagic;
    c->S = capacity / ways;
    c->W = ways;
    c->d = dim;
    c->K = nullptr; c->V = nullptr; c->sc = nullptr; c->ring = nullptr; c->T = nullptr; c->flags = nullptr; c->word_half = 0;
    c->policy = policy;
    c->concurrent_writers.store(dim <= kMaxCheckedDim ? 1 : 0);
    c->query_dedup.store(0);

    hipError_t e = hipGetDevice(&c->device);
    c->n_cus = 256;
    if (e == hipSuccess) e = hipDeviceGetAttribute(&c->n_cus, hipDeviceAttributeMultiprocessorCount, c->device);
    if (e == hipSuccess && c->n_cus <= 0) c->n_cus = 256;
    if (e == hipSuccess) e = hipMalloc(&c->K, capacity * sizeof(int64_t));
    if (e == hipSuccess) e = hipMalloc(&c->V, capacity * (size_t)dim * sizeof(float));
    if (e == hipSuccess) e = hipMalloc(&c->sc, c->S * 2 * sizeof(uint32_t));
    if (e == hipSuccess) e = hipMalloc(&c->ring, 2 * kRing * sizeof(uint64_t));
    if (e == hipSuccess) e = hipMalloc(&c->flags, 2 * sizeof(uint32_t));
    if (e == hipSuccess) e = hipMemsetAsync(c->flags, 0, 2 * sizeof(uint32_t), 0);
    if (e == hipSuccess && policy == HPS_POLICY_LRU) {
        e = hipMalloc(&c->T, capacity * sizeof(uint32_t));
        if (e == hipSuccess) e = hipMemsetAsync(c->T, 0, capacity * sizeof(uint32_t), 0);
    }
    if (e == hipSuccess) {
        hipLaunchKernelGGL(fill_keys_kernel, dim3(4096), dim3(256), 0, 0, c->K, (uint64_t)capacity, kEmpty);
        e = hipGetLastError();
    }
    if (e == hipSuccess) e = hipMemsetAsync(c->V, 0, capacity * (size_t)dim * sizeof(float), 0);
    if (e == hipSuccess) e = hipMemsetAsync(c->sc, 0, c->S * 2 * sizeof(uint32_t), 0);
    if (e == hipSuccess) e = hipMemsetAsync(c->ring, 0, 2 * kRing * sizeof(uint64_t), 0);
    if (e == hipSuccess) e = hipStreamSynchronize(0);
    if (e != hipSuccess) {
        const hps_status_t code = e == hipErrorOutOfMemory ? HPS_ERR_OOM : HPS_ERR_DEVICE;
        std::string msg = std::string("hps_cache_create: ") + hipGetErrorString(e);
        (void)hipGetLastError();
        if (c->K) (void)hipFree(c->K);
        if (c->V) (void)hipFree(c->V);
        if (c->sc) (void)hipFree(c->sc);
        if (c->ring) (void)hipFree(c->ring);
        if (c->T) (void)hipFree(c->T);
        if (c->flags) (void)hipFree(c->flags);
        delete c;
        return fail(code, msg);
    }
    *out_handle = c;
    return HPS_OK;
}

hps_status_t hps_cache_destroy(hps_cache_t *c) {
    if (!c || c->magic != kMagic) return fail(HPS_ERR_INVALID_ARG, "invalid cache handle");
    c->magic = 0;
    hipError_t e = hipSuccess, e2;
    if ((e2 = hipFree(c->K)) != hipSuccess) e = e2;
    if ((e2 = hipFree(c->V)) != hipSuccess) e = e2;
    if ((e2 = hipFree(c->sc)) != hipSuccess) e = e2;
    if ((e2 = hipFree(c->ring)) != hipSuccess) e = e2;
    if (c->T && (e2 = hipFree(c->T)) != hipSuccess) e = e2;
    if ((e2 = hipFree(c->flags)) != hipSuccess) e = e2;
    delete c;
    if (e != hipSuccess) return fail(HPS_ERR_DEVICE, std::string("hipFree: ") + hipGetErrorString(e));
    return HPS_OK;
}

hps_status_t hps_cache_info(const hps_cache_t *c, uint64_t *num_sets, uint32_t *ways, uint32_t *dim) {
    if (!c || c->magic != kMagic) return fail(HPS_ERR_INVALID_ARG, "invalid cache handle");
    if (num_sets) *num_sets = c->S;
    if (ways) *ways = c->W;
    if (dim) *dim = c->d;
    return HPS_OK;
}

hps_status_t hps_cache_set_concurrent_writers(hps_cache_t *c, int enabled) {
    if (!c || c->magic != kMagic) return fail(HPS_ERR_INVALID_ARG, "invalid cache handle");
    if (enabled && c->d > kMaxCheckedDim)
        return fail(HPS_ERR_INVALID_ARG, "queries overlapping writers are supported for dim <= " +
                                             std::to_string(kMaxCheckedDim) + " (4 KiB rows)");
    c->concurrent_writers.store(enabled ? 1 : 0);
    return HPS_OK;
}

hps_status_t hps_cache_flags(hps_cache_t *c, uint32_t *flags, int clear) {
    if (hps_status_t s = check_handle(c)) return s;
    if (!flags) return fail(HPS_ERR_INVALID_ARG, "flags is NULL");
    HIP_TRY(hipMemcpy(flags, c->flags, sizeof(uint32_t), hipMemcpyDeviceToHost));
    if (clear) HIP_TRY(hipMemset(c->flags, 0, sizeof(uint32_t)));
    return HPS_OK;
}

hps_status_t hps_cache_debug_set_seq(hps_cache_t *c, uint64_t set, uint32_t value) {
    if (hps_status_t s = check_handle(c)) return s;
    if (set >= c->S) return fail(HPS_ERR_INVALID_ARG, "set index out of range");
    HIP_TRY(hipMemcpy(c->sc + 2 * set, &value, sizeof(uint32_t), hipMemcpyHostToDevice));
    return HPS_OK;
}

hps_status_t hps_cache_set_query_dedup(hps_cache_t *c, int enabled) {
    if (!c || c->magic != kMagic) return fail(HPS_ERR_INVALID_ARG, "invalid cache handle");
    c->query_dedup.store(enabled ? 1 : 0);
    return HPS_OK;
}

static hps_status_t query_call(hps_cache_t *const *caches, uint32_t n_tables, const int64_t *keys,
                               size_t batch, const uint32_t *n_dev, float *out, uint32_t *miss_idx,
                               int64_t *miss_keys, uint32_t *n_miss, void *stream) {
    if (!caches || n_tables == 0 || n_tables > HPS_MAX_TABLES)
        return fail(HPS_ERR_INVALID_ARG, "n_tables must be in [1, HPS_MAX_TABLES]");
    for (uint32_t t = 0; t < n_tables; ++t) {
        if (hps_status_t s = check_handle(caches[t])) return s;
        if (caches[t]->d != caches[0]->d || caches[t]->W != caches[0]->W)
            return fail(HPS_ERR_INVALID_ARG, "all tables of one call must share dim and ways");
    }
    if (!n_miss || !aligned(n_miss, 4)) return fail(HPS_ERR_INVALID_ARG, "n_miss must be a 4-byte aligned device pointer");
    const uint64_t total = (uint64_t)n_tables * batch;
    if (total >= (1ull << 32)) return fail(HPS_ERR_INVALID_ARG, "n_tables * batch must be < 2^32");
    if (total > 0) {
        if (!keys || !out || !miss_idx || !miss_keys)
            return fail(HPS_ERR_INVALID_ARG, "keys/out/miss_idx/miss_keys must not be NULL when n > 0");
        if (!aligned(keys, 8) || !aligned(miss_keys, 8) || !aligned(out, 16) || !aligned(miss_idx, 4))
            return fail(HPS_ERR_INVALID_ARG, "misaligned buffer (keys 8, out 16, miss_idx 4 bytes)");
    }
    QueryArgs a;
    std::memset(&a, 0, sizeof(a));
    for (uint32_t t = 0; t < n_tables; ++t) a.tab[t] = table_of(caches[t]);
    a.n_tables = n_tables;
    a.keys = keys;
    a.out = out;
    a.miss_idx = miss_idx;
    a.miss_keys = miss_keys;
    a.n_miss = n_miss;
    a.slot = counter_word(caches[0], stream);
    a.B = (uint32_t)batch;
    a.n_dev = n_dev;
    bool coherent = false;                      // any table that may see concurrent writers makes the call careful
    for (uint32_t t = 0; t < n_tables; ++t) coherent = coherent || caches[t]->concurrent_writers.load() != 0;
    const bool dedup = !coherent && caches[0]->query_dedup.load() != 0;
    QueryShape shape = query_shape(total, coherent, dedup);
    // Keys per worker wave: at most 64, trimmed so that the work-groups come out as a whole number
    // of rounds over the CUs (106,496 keys in tiles of 8 x 52 are exactly 256 work-groups; tiles of
    // 8 x 64 would be 208, leaving 48 CUs idle).  Small batches go down to 16 keys per wave (8 below
    // 4,096 keys): more work-groups, each with a shorter chain of dependent row copies (1,664 keys:
    // 5.5 us instead of 8.3 us; 13,312 keys: 8.9 instead of 11.1 us).
    uint32_t kpw = (uint32_t)shape.kpw;
    {
        const uint64_t cus = (uint64_t)caches[0]->n_cus;
        const uint64_t full = (uint64_t)shape.wpb * shape.kpw * cus;       // keys per round at 64 keys per wave
        const uint64_t rounds = (total + full - 1) / full;
        const uint64_t floor_k = total < 4096 ? 8 : 16;
        if (rounds > 0 && rounds <= 8) {
            uint64_t k = (total + shape.wpb * cus * rounds - 1) / (shape.wpb * cus * rounds);
            if (k < floor_k) k = floor_k;
            if (k <= (uint64_t)shape.kpw) kpw = (uint32_t)k;
        }
    }
    // At most 26 keys per wave: a group of 13 wave loads holds them all (rows of up to 512 bytes), and the 13 loads
    // of a 26-load group that would only repeat entry 0 are not issued (26,624 keys: 10.6 -> 9.7 us).
    if (!coherent && shape.u == 26 && kpw <= 26 && caches[0]->d <= 128) shape.u = 13;
    a.kpw = kpw;
    const uint32_t tile = kpw * (uint32_t)shape.wpb;
    a.tiles_per_table = (uint32_t)((batch + tile - 1) / tile);
    if (a.tiles_per_table == 0) a.tiles_per_table = 1;          // an empty batch still publishes n_miss = 0
    a.n_tiles = a.tiles_per_table * n_tables;
    a.g = make_geom(caches[0]->d);
    bool full = n_dev != nullptr;               // a device-side length or any LRU table (Alg. 2 stamps) selects the full kernels
    for (uint32_t t = 0; t < n_tables; ++t) full = full || a.tab[t].T != nullptr;
    return launch_query(caches[0]->W, a, shape, coherent, dedup, full, static_cast<hipStream_t>(stream));
}

hps_status_t hps_cache_query_multi(hps_cache_t *const *caches, uint32_t n_tables, const int64_t *keys,
                                   size_t batch, float *out, uint32_t *miss_idx, int64_t *miss_keys,
                                   uint32_t *n_miss, void *stream) {
    return query_call(caches, n_tables, keys, batch, nullptr, out, miss_idx, miss_keys, n_miss, stream);
}

hps_status_t hps_cache_query(hps_cache_t *c, const int64_t *keys, size_t n, float *out,
                             uint32_t *miss_idx, int64_t *miss_keys, uint32_t *n_miss, void *stream) {
    if (n >= (1ull << 32)) return fail(HPS_ERR_INVALID_ARG, "n must be < 2^32");
    hps_cache_t *one[1] = {c};
    return query_call(one, 1, keys, n, nullptr, out, miss_idx, miss_keys, n_miss, stream);
}

hps_status_t hps_cache_query_dn(hps_cache_t *c, const int64_t *keys, size_t n_max, const uint32_t *n_dev,
                                float *out, uint32_t *miss_idx, int64_t *miss_keys, uint32_t *n_miss,
                                void *stream) {
    if (n_max >= (1ull << 32)) return fail(HPS_ERR_INVALID_ARG, "n_max must be < 2^32");
    if (!n_dev || !aligned(n_dev, 4)) return fail(HPS_ERR_INVALID_ARG, "n_dev must be a 4-byte aligned device pointer");
    hps_cache_t *one[1] = {c};
    return query_call(one, 1, keys, n_max, n_dev, out, miss_idx, miss_keys, n_miss, stream);
}

hps_status_t hps_cache_insert(hps_cache_t *c, const int64_t *keys, const float *vals, size_t n, void *stream) {
    return write_call(c, keys, vals, n, nullptr, stream, true);
}
hps_status_t hps_cache_update(hps_cache_t *c, const int64_t *keys, const float *vals, size_t n, void *stream) {
    return write_call(c, keys, vals, n, nullptr, stream, false);
}
hps_status_t hps_cache_insert_dn(hps_cache_t *c, const int64_t *keys, const float *vals, size_t n_max,
                                 const uint32_t *n_dev, void *stream) {
    if (!n_dev) return fail(HPS_ERR_INVALID_ARG, "n_dev is NULL");
    return write_call(c, keys, vals, n_max, n_dev, stream, true);
}
hps_status_t hps_cache_update_dn(hps_cache_t *c, const int64_t *keys, const float *vals, size_t n_max,
                                 const uint32_t *n_dev, void *stream) {
    if (!n_dev) return fail(HPS_ERR_INVALID_ARG, "n_dev is NULL");
    return write_call(c, keys, vals, n_max, n_dev, stream, false);
}

hps_status_t hps_cache_export(hps_cache_t *c, int64_t *keys, uint32_t *ctr, float *vals, void *stream) {
    if (hps_status_t s = check_handle(c)) return s;
    if (!keys || !ctr) return fail(HPS_ERR_INVALID_ARG, "keys and ctr must not be NULL");
    hipStream_t st = static_cast<hipStream_t>(stream);
    const size_t slots = c->S * c->W;
    HIP_TRY(hipMemcpyAsync(keys, c->K, slots * sizeof(int64_t), hipMemcpyDeviceToDevice, st));
    hipLaunchKernelGGL(counters_out_kernel, dim3(1024), dim3(256), 0, st, c->sc, (uint64_t)c->S, ctr);
    HIP_TRY(hipGetLastError());
    if (vals)
        HIP_TRY(hipMemcpyAsync(vals, c->V, slots * c->d * sizeof(float), hipMemcpyDeviceToDevice, st));
    return HPS_OK;
}

hps_status_t hps_cache_import(hps_cache_t *c, const int64_t *keys, const uint32_t *ctr, const float *vals,
                              void *stream) {
    if (hps_status_t s = check_handle(c)) return s;
    if (!keys || !ctr) return fail(HPS_ERR_INVALID_ARG, "keys and ctr must not be NULL");
    hipStream_t st = static_cast<hipStream_t>(stream);
    const size_t slots = c->S * c->W;
    HIP_TRY(hipMemcpyAsync(c->K, keys, slots * sizeof(int64_t), hipMemcpyDeviceToDevice, st));
    if (vals)
        HIP_TRY(hipMemcpyAsync(c->V, vals, slots * c->d * sizeof(float), hipMemcpyDeviceToDevice, st));
    hipLaunchKernelGGL(counters_in_kernel, dim3(1024), dim3(256), 0, st, c->sc, (uint64_t)c->S, ctr);
    HIP_TRY(hipGetLastError());
    return HPS_OK;
}

hps_status_t hps_cache_export_lru(hps_cache_t *c, uint32_t *stamps, uint32_t *g, void *stream) {
    if (hps_status_t s = check_handle(c)) return s;
    if (c->policy != HPS_POLICY_LRU) return fail(HPS_ERR_INVALID_ARG, "the cache was not created with the LRU policy");
    if (!stamps || !g) return fail(HPS_ERR_INVALID_ARG, "stamps and g must not be NULL");
    hipStream_t st = static_cast<hipStream_t>(stream);
    HIP_TRY(hipMemcpyAsync(stamps, c->T, c->S * c->W * sizeof(uint32_t), hipMemcpyDeviceToDevice, st));
    HIP_TRY(hipMemcpyAsync(g, c->flags + 1, sizeof(uint32_t), hipMemcpyDeviceToHost, st));
    HIP_TRY(hipStreamSynchronize(st));                   // *g is a host word: it is valid on return
    return HPS_OK;
}

hps_status_t hps_cache_import_lru(hps_cache_t *c, const uint32_t *stamps, uint32_t g, void *stream) {
    if (hps_status_t s = check_handle(c)) return s;
    if (c->policy != HPS_POLICY_LRU) return fail(HPS_ERR_INVALID_ARG, "the cache was not created with the LRU policy");
    if (!stamps) return fail(HPS_ERR_INVALID_ARG, "stamps must not be NULL");
    hipStream_t st = static_cast<hipStream_t>(stream);
    HIP_TRY(hipMemcpyAsync(c->T, stamps, c->S * c->W * sizeof(uint32_t), hipMemcpyDeviceToDevice, st));
    hipLaunchKernelGGL(set_u32_kernel, dim3(1), dim3(1), 0, st, c->flags + 1, g);
    HIP_TRY(hipGetLastError());
    return HPS_OK;
}

hps_status_t hps_cache_dump(hps_cache_t *c, size_t first_slot, size_t n_slots, int64_t *keys_out,
                            uint32_t *n_out, void *stream) {
    if (hps_status_t s = check_handle(c)) return s;
    const size_t slots = c->S * c->W;
    if (first_slot > slots || n_slots > slots - first_slot)
        return fail(HPS_ERR_INVALID_ARG, "slot range exceeds the cache");
    if (n_slots >= (1ull << 32)) return fail(HPS_ERR_INVALID_ARG, "n_slots must be < 2^32 per call");
    if (!n_out || (n_slots > 0 && !keys_out)) return fail(HPS_ERR_INVALID_ARG, "output pointer is NULL");
    if (!aligned(keys_out, 8) || !aligned(n_out, 4)) return fail(HPS_ERR_INVALID_ARG, "misaligned output buffer");
    constexpr int kDumpKpt = 32;                       // 8192 slots per tile (16 and 64 dump 15-20 % slower)
    uint32_t n_tiles = (uint32_t)((n_slots + kBlock * kDumpKpt - 1) / (kBlock * kDumpKpt));
    if (n_tiles == 0) n_tiles = 1;
    const uint32_t grid = n_tiles < (1u << 20) ? n_tiles : (1u << 20);
    hipLaunchKernelGGL((dump_kernel<kDumpKpt>), dim3(grid), dim3(kBlock), 0, static_cast<hipStream_t>(stream), c->K,
                       (uint64_t)first_slot, (uint64_t)n_slots, keys_out, n_out, counter_word(c, stream), n_tiles);
    HIP_TRY(hipGetLastError());
    return HPS_OK;
}

hps_status_t hps_membench_gather(const float *rows, const uint32_t *slot_of, size_t n, uint32_t dim, float *out,
                                 void *stream) {
    if (dim == 0 || dim % 4 != 0) return fail(HPS_ERR_INVALID_ARG, "dim must be a non-zero multiple of 4");
    if (n == 0) return HPS_OK;
    if (n >= (1ull << 32)) return fail(HPS_ERR_INVALID_ARG, "n must be < 2^32");
    if (!rows || !slot_of || !out) return fail(HPS_ERR_INVALID_ARG, "rows, slot_of and out must not be NULL");
    if (!aligned(rows, 16) || !aligned(out, 16) || !aligned(slot_of, 4)) return fail(HPS_ERR_INVALID_ARG, "misaligned buffer");
    int dev = 0, cus = 256;
    HIP_TRY(hipGetDevice(&dev));
    HIP_TRY(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
    if (cus <= 0) cus = 256;
    // the query kernel's shape for this batch size: 8 waves x up to 64 positions, trimmed to whole rounds over the CUs
    constexpr int kWpb = 8;
    const uint64_t full = (uint64_t)kWpb * kWave * (uint64_t)cus;
    const uint64_t rounds = (n + full - 1) / full;
    uint64_t kpw = (n + kWpb * (uint64_t)cus * rounds - 1) / (kWpb * (uint64_t)cus * rounds);
    if (kpw < 16) kpw = 16;
    if (kpw > (uint64_t)kWave) kpw = kWave;
    const uint64_t tile = kpw * kWpb;
    const uint64_t blocks = (n + tile - 1) / tile;
    if (blocks >= (1ull << 31)) return fail(HPS_ERR_INVALID_ARG, "n too large");
    if (dim == 128)
        hipLaunchKernelGGL((membench_gather_kernel<26, kWpb, 128>), dim3((uint32_t)blocks), dim3(kWpb * kWave), 0,
                           static_cast<hipStream_t>(stream), rows, slot_of, (uint32_t)n, (uint32_t)kpw, make_geom(dim), out);
    else
        hipLaunchKernelGGL((membench_gather_kernel<26, kWpb, 0>), dim3((uint32_t)blocks), dim3(kWpb * kWave), 0,
                           static_cast<hipStream_t>(stream), rows, slot_of, (uint32_t)n, (uint32_t)kpw, make_geom(dim), out);
    HIP_TRY(hipGetLastError());
    return HPS_OK;
}

hps_status_t hps_membench_gather_half(const float *rows, const uint32_t *slot_of, size_t n, float *out,
                                      int reads, void *stream) {
    if (n == 0) return HPS_OK;
    if (!rows || !slot_of || !out) return fail(HPS_ERR_INVALID_ARG, "null pointer");
    if (n >= (1ull << 32)) return fail(HPS_ERR_INVALID_ARG, "n must be < 2^32");
    if (!aligned(rows, 16) || !aligned(out, 16)) return fail(HPS_ERR_INVALID_ARG, "rows and out must be 16-byte aligned");
    int dev = 0, cus = 256;
    HIP_TRY(hipGetDevice(&dev));
    HIP_TRY(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
    if (cus <= 0) cus = 256;
    constexpr int kWpb = 8;                     // the shape hps_membench_gather uses
    const uint64_t full = (uint64_t)kWpb * kWave * (uint64_t)cus;
    const uint64_t rounds = (n + full - 1) / full;
    uint64_t kpw = (n + kWpb * (uint64_t)cus * rounds - 1) / (kWpb * (uint64_t)cus * rounds);
    if (kpw < 16) kpw = 16;
    if (kpw > (uint64_t)kWave) kpw = kWave;
    const uint64_t tile = kpw * kWpb;
    const uint64_t blocks = (n + tile - 1) / tile;
    if (blocks >= (1ull << 31)) return fail(HPS_ERR_INVALID_ARG, "n too large");
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (reads)
        hipLaunchKernelGGL((membench_half_kernel<26, kWpb, true>), dim3((uint32_t)blocks), dim3(kWpb * kWave), 0, st,
                           rows, slot_of, (uint32_t)n, (uint32_t)kpw, out);
    else
        hipLaunchKernelGGL((membench_half_kernel<26, kWpb, false>), dim3((uint32_t)blocks), dim3(kWpb * kWave), 0, st,
                           rows, slot_of, (uint32_t)n, (uint32_t)kpw, out);
    HIP_TRY(hipGetLastError());
    return HPS_OK;
}

hps_status_t hps_membench_copy(const void *src, void *dst, size_t bytes, int nontemporal, void *stream) {
    if (bytes == 0) return HPS_OK;
    if (!src || !dst || bytes % 16 != 0 || !aligned(src, 16) || !aligned(dst, 16))
        return fail(HPS_ERR_INVALID_ARG, "src and dst must be 16-byte aligned and bytes a multiple of 16");
    const uint64_t n16 = bytes / 16;
    uint64_t blocks = (n16 + (uint64_t)kBlock * 8 - 1) / ((uint64_t)kBlock * 8);
    if (blocks > 16384) blocks = 16384;
    if (blocks == 0) blocks = 1;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (nontemporal)
        hipLaunchKernelGGL((membench_copy_kernel<8, true>), dim3((uint32_t)blocks), dim3(kBlock), 0, st,
                           static_cast<const f32x4 *>(src), static_cast<f32x4 *>(dst), n16);
    else
        hipLaunchKernelGGL((membench_copy_kernel<8, false>), dim3((uint32_t)blocks), dim3(kBlock), 0, st,
                           static_cast<const f32x4 *>(src), static_cast<f32x4 *>(dst), n16);
    HIP_TRY(hipGetLastError());
    return HPS_OK;
}

hps_status_t hps_backing_fetch(const int64_t *keys, size_t n, const uint32_t *n_dev, uint32_t dim,
                               uint32_t version, float *rows, const uint32_t *scatter_idx,
                               float *scatter_out, void *stream) {
    if (dim == 0 || dim % 4 != 0) return fail(HPS_ERR_INVALID_ARG, "dim must be a non-zero multiple of 4");
    if (n == 0) return HPS_OK;
    if (n >= (1ull << 32)) return fail(HPS_ERR_INVALID_ARG, "n must be < 2^32");
    if (!keys || (!rows && !scatter_idx)) return fail(HPS_ERR_INVALID_ARG, "keys and one output are required");
    if (scatter_idx && !scatter_out) return fail(HPS_ERR_INVALID_ARG, "scatter_out is NULL");
    if (!aligned(keys, 8) || !aligned(rows, 16) || !aligned(scatter_out, 16) || !aligned(scatter_idx, 4))
        return fail(HPS_ERR_INVALID_ARG, "misaligned buffer");
    const uint64_t total = (uint64_t)n * (dim / 4);
    uint64_t blocks = (total + 255) / 256;
    if (blocks > (1u << 18)) blocks = 1u << 18;
    hipLaunchKernelGGL(backing_kernel, dim3((uint32_t)blocks), dim3(256), 0, static_cast<hipStream_t>(stream),
                       keys, (uint32_t)n, n_dev, dim, version, rows, scatter_idx, scatter_out);
    HIP_TRY(hipGetLastError());
    return HPS_OK;
}

}  // extern "C"
