/*
 * CPU oracle for the GPU embedding cache (level-1 store of the Hierarchical Parameter Server).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, single-threaded, obviously-correct
 * statement of what the cache computes.  Only tests, the smoke check and the benchmark's
 * cpu_baseline leg may load it; the product path never does.  It shares no code, header,
 * table or constant generator with the HIP implementation.
 *
 * What it follows (paper sections / algorithms):
 *   - Data model, Sec. 4.1: a slot holds a key and an embedding vector; a key is mapped by a
 *     hash to exactly one set (the paper's "slabset") and may sit in any slot of that set.
 *   - Query, Sec. 4.2 and Alg. 2: for each key, search its set; a hit copies the stored
 *     vector to the result row of that key's index; a miss appends <index, key> to M.
 *     The result row of a missing index is not written.
 *   - Replace, Sec. 4.2 and Alg. 3: a key that is already cached is ignored; otherwise empty
 *     slots are filled first and, when the set is full, a resident slot is overwritten.
 *   - Update, Sec. 4.2 and Alg. 4: a cached key gets its vector overwritten; any other key is
 *     ignored.
 *   - Dump, Sec. 4.2: the keys currently cached.
 *   - Deduplication, Sec. 2.2: Q* = dedup(Q), the distinct keys of a query batch, with the map
 *     from every position of Q to its key's place in Q* (what a caller needs to hand every
 *     position its row after looking up Q* only).
 *   - Embedding cache insertion, Sec. 4.3 and Alg. 1: look the batch up, compute the hit rate,
 *     and below the threshold fetch the missing vectors from the lower tiers, insert them and
 *     return them (synchronous insertion); otherwise return the default vector for the missing
 *     keys and insert the fetched vectors afterwards (asynchronous insertion).
 *
 * Readings where the paper is silent or differs from this build's contract:
 *   - Geometry: a set has W slots (W a power of two, 1..64); the paper's 32-slot slabs and
 *     the choice of the first slab to probe only permute the search order inside one set
 *     and cannot change any result, so they do not appear here.
 *   - Victim choice, policy 0 (this build's contract): one counter per set,
 *     way = C[s] mod W, then C[s] += 1.  Because nothing is ever deleted, that fills
 *     ways 0..W-1 first ("empty slots first") and afterwards evicts in insertion order.
 *     Query is then read-only.
 *   - Victim choice, policy 1 (the paper's, Sec. 4.2 Replace, Alg. 2-3): every slot has an
 *     access stamp T; a global iteration count g goes up by one per Query call; a Query hit and
 *     a Replace of an already cached key set T = g; a new key takes the lowest-numbered empty
 *     slot, else the least recently used slot (largest g - T mod 2^32, lowest way on ties),
 *     and gets T = g.  Update leaves stamps alone (Alg. 4).
 *   - Hash: the paper names none.  set = (upper 32 bits of mix64(key)) mod S where mix64 is
 *     the 64-bit finaliser of the splitmix64 generator.
 *   - Empty marker: INT64_MIN ("Null" in Alg. 2-4).  INT64_MIN and INT64_MIN+1 are reserved:
 *     query reports them as misses, insert and update skip them.
 *   - Duplicates in a batch are handled by plain index order: every missing position gets
 *     its own miss-list entry; the first occurrence of a new key inserts, later ones find it.
 *   - Rows are opaque 32-bit patterns (no floating-point arithmetic anywhere on the cache path).
 *   - Alg. 1: the hit rate is 1 - |missing| / |Q| per position (the listing divides by "N = total
 *     size of embedding cache", which cannot be meant); it is computed and compared with the
 *     threshold t in single precision, the precision the product's call takes the decision in;
 *     "hit rate < t" selects synchronous insertion, so a hit rate equal to t is asynchronous.
 *     The lookup is per position (the C ABI takes Q, not Q*); what is fetched and inserted is the
 *     distinct missing keys in order of first occurrence.  The lower tiers are an input: the
 *     caller passes the vector they hold for every position's key.  The asynchronous task is
 *     modelled as having run to completion when the call returns (the tests drain the product's
 *     queue before they compare), so both modes leave the same cache state and differ only in
 *     the rows handed out for the missing positions.
 *   - dedup: the paper fixes no order of Q*; here it is the order of first occurrence (any
 *     permutation of Q* with the matching map is an equally valid result).  All 2^64 key values
 *     are ordinary to dedup, the two reserved ones included.
 *
 * Every batch is processed sequentially in index order.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define HPSO_EMPTY    INT64_MIN
#define HPSO_RESERVED (INT64_MIN + 1)

typedef struct {
    uint64_t S;      /* number of sets                        */
    uint32_t W;      /* slots per set                         */
    uint32_t d;      /* 32-bit words per row                  */
    int64_t  *K;     /* [S][W]    keys, HPSO_EMPTY when free  */
    uint32_t *V;     /* [S][W][d] rows as bit patterns        */
    uint32_t *C;     /* [S]       per-set victim counter (policy 0); number of inserts (policy 1) */
    uint32_t policy; /* 0 = victim counter, 1 = LRU by access stamp */
    uint32_t *T;     /* [S][W]    access stamps (policy 1)    */
    uint32_t g;      /* global iteration count (policy 1)     */
} hpso_t;

/* Finaliser of splitmix64: three xor-shifts around two odd multipliers, all mod 2^64. */
uint64_t hpso_mix64(uint64_t x)
{
    x ^= x >> 30;
    x *= 0xBF58476D1CE4E5B9ULL;
    x ^= x >> 27;
    x *= 0x94D049BB133111EBULL;
    x ^= x >> 31;
    return x;
}

/* Alg. 2, "find slabset": hash of the key modulo the number of sets. */
uint64_t hpso_set_of(const hpso_t *c, int64_t key)
{
    uint32_t h = (uint32_t)(hpso_mix64((uint64_t)key) >> 32);
    return (uint64_t)h % c->S;
}

/* The same for a batch of keys (test plumbing: no per-key call from Python). */
void hpso_sets_of(const hpso_t *c, const int64_t *keys, uint64_t n, uint64_t *sets_out)
{
    for (uint64_t i = 0; i < n; ++i) sets_out[i] = hpso_set_of(c, keys[i]);
}

static int is_reserved(int64_t key)
{
    return key == HPSO_EMPTY || key == HPSO_RESERVED;
}

/* Search the key's set; returns the way holding it, or -1. */
static int find_way(const hpso_t *c, uint64_t s, int64_t key)
{
    for (uint32_t w = 0; w < c->W; ++w)
        if (c->K[s * c->W + w] == key)
            return (int)w;
    return -1;
}

hpso_t *hpso_create_policy(uint64_t capacity, uint32_t W, uint32_t d, uint32_t policy)
{
    if (W == 0 || W > 64 || (W & (W - 1)) != 0 || d == 0 || capacity == 0 ||
        capacity % W != 0 || capacity / W >= (1ULL << 31) || policy > 1)
        return NULL;
    hpso_t *c = (hpso_t *)calloc(1, sizeof(hpso_t));
    if (!c) return NULL;
    c->S = capacity / W;
    c->W = W;
    c->d = d;
    c->K = (int64_t *)malloc(sizeof(int64_t) * capacity);
    c->V = (uint32_t *)calloc(capacity * (uint64_t)d, sizeof(uint32_t));
    c->C = (uint32_t *)calloc(c->S, sizeof(uint32_t));
    c->T = (uint32_t *)calloc(capacity, sizeof(uint32_t));
    c->policy = policy;
    c->g = 0;
    if (!c->K || !c->V || !c->C || !c->T) {
        free(c->K); free(c->V); free(c->C); free(c->T); free(c);
        return NULL;
    }
    for (uint64_t i = 0; i < capacity; ++i) c->K[i] = HPSO_EMPTY;
    return c;
}

hpso_t *hpso_create(uint64_t capacity, uint32_t W, uint32_t d)
{
    return hpso_create_policy(capacity, W, d, 0);
}

void hpso_destroy(hpso_t *c)
{
    if (!c) return;
    free(c->K); free(c->V); free(c->C); free(c->T); free(c);
}

uint64_t  hpso_num_sets(const hpso_t *c) { return c->S; }
uint32_t  hpso_ways(const hpso_t *c)     { return c->W; }
uint32_t  hpso_dim(const hpso_t *c)      { return c->d; }
int64_t  *hpso_keys(hpso_t *c)           { return c->K; }
uint32_t *hpso_vals(hpso_t *c)           { return c->V; }
uint32_t *hpso_ctr(hpso_t *c)            { return c->C; }
uint32_t *hpso_stamps(hpso_t *c)         { return c->T; }
uint32_t  hpso_get_g(const hpso_t *c)    { return c->g; }
void      hpso_set_g(hpso_t *c, uint32_t g) { c->g = g; }

/*
 * Query (Alg. 2).  out is [n][d]; rows of missing positions are left untouched.
 * miss_idx / miss_keys receive <index, key> in ascending index order.  Returns |M|.
 */
uint64_t hpso_query(hpso_t *c, const int64_t *keys, uint64_t n,
                    uint32_t *out, uint32_t *miss_idx, int64_t *miss_keys)
{
    uint64_t n_miss = 0;
    if (c->policy == 1) c->g += 1;                     /* Alg. 2: g <- g + 1, Query only */
    for (uint64_t i = 0; i < n; ++i) {
        int64_t q = keys[i];
        int w = -1;
        uint64_t s = 0;
        if (!is_reserved(q)) {
            s = hpso_set_of(c, q);
            w = find_way(c, s, q);
        }
        if (w < 0) {
            miss_idx[n_miss] = (uint32_t)i;
            miss_keys[n_miss] = q;
            ++n_miss;
        } else {
            memcpy(out + i * c->d, c->V + (s * c->W + (uint64_t)w) * c->d,
                   sizeof(uint32_t) * c->d);
            if (c->policy == 1) c->T[s * c->W + (uint64_t)w] = c->g;   /* refresh the counter */
        }
    }
    return n_miss;
}

/* Replace (Alg. 3); the slot of a new key is chosen by the cache's policy (see the header). */
void hpso_insert(hpso_t *c, const int64_t *keys, const uint32_t *vals, uint64_t n)
{
    for (uint64_t i = 0; i < n; ++i) {
        int64_t q = keys[i];
        if (is_reserved(q)) continue;
        uint64_t s = hpso_set_of(c, q);
        int f = find_way(c, s, q);
        if (f >= 0) {                                   /* already cached: row ignored */
            if (c->policy == 1) c->T[s * c->W + (uint64_t)f] = c->g;
            continue;
        }
        uint32_t w;
        if (c->policy == 0) {
            w = c->C[s] % c->W;                         /* wraps mod 2^32; W divides 2^32 */
        } else {
            int e = find_way(c, s, HPSO_EMPTY);         /* empty slots first */
            if (e >= 0) {
                w = (uint32_t)e;
            } else {                                    /* least recently used: largest age */
                w = 0;
                for (uint32_t x = 1; x < c->W; ++x)
                    if ((uint32_t)(c->g - c->T[s * c->W + x]) > (uint32_t)(c->g - c->T[s * c->W + w]))
                        w = x;
            }
            c->T[s * c->W + w] = c->g;
        }
        c->C[s] += 1;
        c->K[s * c->W + w] = q;
        memcpy(c->V + (s * c->W + w) * c->d, vals + i * c->d, sizeof(uint32_t) * c->d);
    }
}

/* Update (Alg. 4): overwrite the vector of keys that are cached, ignore the rest. */
void hpso_update(hpso_t *c, const int64_t *keys, const uint32_t *vals, uint64_t n)
{
    for (uint64_t i = 0; i < n; ++i) {
        int64_t q = keys[i];
        if (is_reserved(q)) continue;
        uint64_t s = hpso_set_of(c, q);
        int w = find_way(c, s, q);
        if (w < 0) continue;
        memcpy(c->V + (s * c->W + (uint64_t)w) * c->d, vals + i * c->d,
               sizeof(uint32_t) * c->d);
    }
}

/* Dump (Sec. 4.2): the cached keys, in slot order.  Returns how many were written. */
uint64_t hpso_dump(const hpso_t *c, int64_t *keys_out)
{
    uint64_t m = 0;
    for (uint64_t i = 0; i < c->S * c->W; ++i)
        if (c->K[i] != HPSO_EMPTY)
            keys_out[m++] = c->K[i];
    return m;
}

/*
 * dedup (Sec. 2.2): unique_out receives the distinct keys in order of first occurrence,
 * inverse_out[i] the place of keys[i] among them.  Returns |Q*|.  Written as the definition: every
 * key is compared with the distinct keys found so far.
 */
uint64_t hpso_dedup(const int64_t *keys, uint64_t n, int64_t *unique_out, uint32_t *inverse_out)
{
    uint64_t u = 0;
    for (uint64_t i = 0; i < n; ++i) {
        uint64_t j = 0;
        while (j < u && unique_out[j] != keys[i]) ++j;
        if (j == u) unique_out[u++] = keys[i];
        inverse_out[i] = (uint32_t)j;
    }
    return u;
}

/* The step after looking up Q*: position i gets the row of its key, out[i] = rows[inverse[i]]. */
void hpso_expand(const uint32_t *rows, const uint32_t *inverse, uint64_t n, uint32_t d, uint32_t *out)
{
    for (uint64_t i = 0; i < n; ++i)
        memcpy(out + i * d, rows + (uint64_t)inverse[i] * d, sizeof(uint32_t) * d);
}

/*
 * One pass of Alg. 1 (embedding cache insertion) for the batch Q = keys[0..n).
 *   lower[i*d .. i*d+d)  the vector the lower tiers hold for keys[i] (ParServerLookup's answer)
 *   t                    hit rate threshold
 *   default_row[d]       vector handed out for missing keys in asynchronous mode
 *   out[n][d]            E_Q: cached vector on a hit; on a miss the fetched vector (synchronous)
 *                        or the default vector (asynchronous)
 *   ins_keys[<= n]       receives the distinct missing keys in order of first occurrence: what
 *                        ParServerLookup is asked for and what is inserted
 * Returns the number of distinct missing keys; *hit_rate and *synchronous describe the decision.
 * When do_insert is zero the cache is left as the lookup found it (the caller inserts ins_keys
 * itself, e.g. after classifying the batch); otherwise the insertion is done here.
 */
uint64_t hpso_lookup(hpso_t *c, const int64_t *keys, uint64_t n, const uint32_t *lower, float t,
                     const uint32_t *default_row, uint32_t *out, float *hit_rate, int *synchronous,
                     int64_t *ins_keys, int do_insert)
{
    *hit_rate = 1.0f;
    *synchronous = 0;
    if (n == 0) return 0;
    /* EmbCacheLookup(Q): hits land in E_Q, misses in the workspace */
    uint32_t *miss_idx  = (uint32_t *)malloc(sizeof(uint32_t) * n);
    int64_t  *miss_keys = (int64_t *)malloc(sizeof(int64_t) * n);
    uint32_t *ins_rows  = (uint32_t *)malloc(sizeof(uint32_t) * n * c->d);
    if (!miss_idx || !miss_keys || !ins_rows) abort();
    uint64_t m = hpso_query(c, keys, n, out, miss_idx, miss_keys);
    /* hitRate <- 1 - |missingKeys| / |Q| */
    float rate = 1.0f - (float)m / (float)n;
    *hit_rate = rate;
    uint64_t u = 0;
    if (m > 0) {
        /* ParServerLookup(missingKeys): each missing key once, with the vector of the lower tiers */
        for (uint64_t j = 0; j < m; ++j) {
            uint64_t e = 0;
            while (e < u && ins_keys[e] != miss_keys[j]) ++e;
            if (e == u) {
                ins_keys[u] = miss_keys[j];
                memcpy(ins_rows + u * c->d, lower + (uint64_t)miss_idx[j] * c->d, sizeof(uint32_t) * c->d);
                ++u;
            }
        }
        if (rate < t) {
            /* synchronous insertion: E_Q <- the fetched vectors */
            *synchronous = 1;
            for (uint64_t j = 0; j < m; ++j)
                memcpy(out + (uint64_t)miss_idx[j] * c->d, lower + (uint64_t)miss_idx[j] * c->d,
                       sizeof(uint32_t) * c->d);
        } else {
            /* asynchronous insertion: E_Q <- default values now, the insertion is queued */
            for (uint64_t j = 0; j < m; ++j)
                memcpy(out + (uint64_t)miss_idx[j] * c->d, default_row, sizeof(uint32_t) * c->d);
        }
        /* EmbCacheInsert(missingKeys, vectors): at once, or by the queued task */
        if (do_insert) hpso_insert(c, ins_keys, ins_rows, u);
    }
    free(miss_idx); free(miss_keys); free(ins_rows);
    return u;
}
