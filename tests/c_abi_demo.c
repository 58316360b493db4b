/*
 * A caller of the cache written in plain C99: proves that the boundary of include/hps_cache.h and
 * include/hps_dedup.h is usable without C++, Python or torch.  Built into a small shared library
 * whose one entry point runs a create / insert / query / update / dedup / expand round on the
 * current device and checks every result on the host.  Returns 0, or the source line of the
 * first check that failed (the message goes to `msg`).
 */
#define __HIP_PLATFORM_AMD__ 1
#include <hip/hip_runtime_api.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "hps_cache.h"
#include "hps_dedup.h"

#define FAIL(...) do { snprintf(msg, msg_len, __VA_ARGS__); rc = __LINE__; goto done; } while (0)
#define HIP_OK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) FAIL("%s: %s", #x, hipGetErrorString(e_)); } while (0)
#define HPS_OK_(x, err) do { if ((x) != HPS_OK) FAIL("%s: %s", #x, err()); } while (0)

static float row_word(int64_t key, uint32_t j, uint32_t version) {
    return (float)((key * 31 + (int64_t)j * 7 + (int64_t)version * 1009) % 65536) * 0.5f;   /* exact in fp32 */
}

int hps_c_demo_run(char *msg, size_t msg_len)
{
    enum { SETS = 512, WAYS = 8, DIM = 16, N_IN = 1000, N_Q = 3000 };
    int rc = 0;
    hps_cache_t *cache = NULL;
    hps_dedup_t *dd = NULL;
    int64_t *h_keys = NULL, *d_keys = NULL, *d_mkeys = NULL, *h_mkeys = NULL, *d_ukeys = NULL, *h_ukeys = NULL;
    float *h_rows = NULL, *d_rows = NULL, *d_out = NULL, *h_out = NULL, *d_exp = NULL;
    uint32_t *d_midx = NULL, *h_midx = NULL, *d_nmiss = NULL, *d_inv = NULL, *h_inv = NULL, *d_nu = NULL;
    uint32_t n_miss = 0, n_unique = 0, i, j;
    const size_t rowb = DIM * sizeof(float);

    if (msg_len) msg[0] = 0;
    h_keys = (int64_t *)malloc(N_Q * sizeof(int64_t));
    h_mkeys = (int64_t *)malloc(N_Q * sizeof(int64_t));
    h_ukeys = (int64_t *)malloc(N_Q * sizeof(int64_t));
    h_rows = (float *)malloc(N_Q * rowb);
    h_out = (float *)malloc(N_Q * rowb);
    h_midx = (uint32_t *)malloc(N_Q * sizeof(uint32_t));
    h_inv = (uint32_t *)malloc(N_Q * sizeof(uint32_t));
    if (!h_keys || !h_mkeys || !h_ukeys || !h_rows || !h_out || !h_midx || !h_inv) FAIL("host allocation failed");
    HIP_OK(hipMalloc((void **)&d_keys, N_Q * sizeof(int64_t)));
    HIP_OK(hipMalloc((void **)&d_mkeys, N_Q * sizeof(int64_t)));
    HIP_OK(hipMalloc((void **)&d_ukeys, N_Q * sizeof(int64_t)));
    HIP_OK(hipMalloc((void **)&d_rows, N_Q * rowb));
    HIP_OK(hipMalloc((void **)&d_out, N_Q * rowb));
    HIP_OK(hipMalloc((void **)&d_exp, N_Q * rowb));
    HIP_OK(hipMalloc((void **)&d_midx, N_Q * sizeof(uint32_t)));
    HIP_OK(hipMalloc((void **)&d_inv, N_Q * sizeof(uint32_t)));
    HIP_OK(hipMalloc((void **)&d_nmiss, sizeof(uint32_t)));
    HIP_OK(hipMalloc((void **)&d_nu, sizeof(uint32_t)));

    HPS_OK_(hps_cache_create((size_t)SETS * WAYS, WAYS, DIM, &cache), hps_last_error);

    /* insert keys 0, 3, 6, ... (N_IN of them: far fewer than slots, no set overflows with 8 ways
       and 512 sets unless the hash were degenerate, which the miss count below would show) */
    for (i = 0; i < N_IN; ++i) {
        h_keys[i] = 3 * (int64_t)i;
        for (j = 0; j < DIM; ++j) h_rows[i * DIM + j] = row_word(h_keys[i], j, 0);
    }
    HIP_OK(hipMemcpy(d_keys, h_keys, N_IN * sizeof(int64_t), hipMemcpyHostToDevice));
    HIP_OK(hipMemcpy(d_rows, h_rows, N_IN * rowb, hipMemcpyHostToDevice));
    HPS_OK_(hps_cache_insert(cache, d_keys, d_rows, N_IN, NULL), hps_last_error);

    /* query keys 0 .. N_Q-1: multiples of 3 hit, the others miss */
    for (i = 0; i < N_Q; ++i) h_keys[i] = (int64_t)i;
    HIP_OK(hipMemcpy(d_keys, h_keys, N_Q * sizeof(int64_t), hipMemcpyHostToDevice));
    HIP_OK(hipMemset(d_out, 0xFF, N_Q * rowb));
    HPS_OK_(hps_cache_query(cache, d_keys, N_Q, d_out, d_midx, d_mkeys, d_nmiss, NULL), hps_last_error);
    HIP_OK(hipDeviceSynchronize());
    HIP_OK(hipMemcpy(&n_miss, d_nmiss, sizeof(uint32_t), hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(h_out, d_out, N_Q * rowb, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(h_midx, d_midx, N_Q * sizeof(uint32_t), hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(h_mkeys, d_mkeys, N_Q * sizeof(int64_t), hipMemcpyDeviceToHost));
    if (n_miss != N_Q - N_IN) FAIL("n_miss = %u, expected %u", n_miss, (unsigned)(N_Q - N_IN));
    for (i = 0; i < n_miss; ++i)
        if (h_midx[i] >= N_Q || h_midx[i] % 3 == 0 || h_mkeys[i] != (int64_t)h_midx[i])
            FAIL("miss entry %u is <%u, %lld>", i, h_midx[i], (long long)h_mkeys[i]);
    for (i = 0; i < N_Q; ++i)
        for (j = 0; j < DIM; ++j) {
            uint32_t bits;
            memcpy(&bits, &h_out[i * DIM + j], 4);
            if (i % 3 == 0 ? h_out[i * DIM + j] != row_word(i, j, 0) : bits != 0xFFFFFFFFu)
                FAIL("out[%u][%u] wrong after query", i, j);
        }

    /* update every second cached key (and some absent ones, which must stay absent) */
    for (i = 0; i < N_IN; ++i) {
        h_keys[i] = 6 * (int64_t)i + (i >= N_IN / 2 ? 1 : 0);      /* first half cached (multiples of 6), second half absent */
        for (j = 0; j < DIM; ++j) h_rows[i * DIM + j] = row_word(h_keys[i], j, 1);
    }
    HIP_OK(hipMemcpy(d_keys, h_keys, N_IN * sizeof(int64_t), hipMemcpyHostToDevice));
    HIP_OK(hipMemcpy(d_rows, h_rows, N_IN * rowb, hipMemcpyHostToDevice));
    HPS_OK_(hps_cache_update(cache, d_keys, d_rows, N_IN, NULL), hps_last_error);

    /* dedup a batch with repeats, look the distinct keys up, expand to the positions */
    for (i = 0; i < N_Q; ++i) h_keys[i] = (int64_t)((i * 7) % 600);    /* 600 distinct values */
    HIP_OK(hipMemcpy(d_keys, h_keys, N_Q * sizeof(int64_t), hipMemcpyHostToDevice));
    HPS_OK_(hps_dedup_create(N_Q, &dd), hps_dedup_last_error);
    HPS_OK_(hps_dedup(dd, d_keys, N_Q, d_ukeys, d_inv, d_nu, NULL), hps_dedup_last_error);
    HIP_OK(hipMemset(d_out, 0xFF, N_Q * rowb));
    HPS_OK_(hps_cache_query_dn(cache, d_ukeys, N_Q, d_nu, d_out, d_midx, d_mkeys, d_nmiss, NULL), hps_last_error);
    HPS_OK_(hps_expand_rows(d_out, d_inv, N_Q, DIM, d_exp, NULL), hps_dedup_last_error);
    HIP_OK(hipDeviceSynchronize());
    HIP_OK(hipMemcpy(&n_unique, d_nu, sizeof(uint32_t), hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(&n_miss, d_nmiss, sizeof(uint32_t), hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(h_ukeys, d_ukeys, N_Q * sizeof(int64_t), hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(h_inv, d_inv, N_Q * sizeof(uint32_t), hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(h_out, d_exp, N_Q * rowb, hipMemcpyDeviceToHost));
    if (n_unique != 600) FAIL("n_unique = %u, expected 600", n_unique);
    if (n_miss != 400) FAIL("distinct misses = %u, expected 400", n_miss);
    for (i = 0; i < N_Q; ++i) {
        if (h_inv[i] >= n_unique || h_ukeys[h_inv[i]] != h_keys[i]) FAIL("inverse[%u] does not lead back to its key", i);
        for (j = 0; j < DIM; ++j) {
            const int64_t k = h_keys[i];
            uint32_t bits;
            memcpy(&bits, &h_out[i * DIM + j], 4);
            /* cached keys are multiples of 3; those that are multiples of 6 below 6 * N_IN / 2 were updated */
            if (k % 3 == 0 ? h_out[i * DIM + j] != row_word(k, j, (k % 6 == 0 && k < 6 * (N_IN / 2)) ? 1u : 0u)
                           : bits != 0xFFFFFFFFu)
                FAIL("expanded row %u word %u wrong (key %lld)", i, j, (long long)k);
        }
    }

done:
    if (dd) (void)hps_dedup_destroy(dd);
    if (cache) (void)hps_cache_destroy(cache);
    (void)hipFree(d_keys); (void)hipFree(d_mkeys); (void)hipFree(d_ukeys); (void)hipFree(d_rows);
    (void)hipFree(d_out); (void)hipFree(d_exp); (void)hipFree(d_midx); (void)hipFree(d_inv);
    (void)hipFree(d_nmiss); (void)hipFree(d_nu);
    free(h_keys); free(h_mkeys); free(h_ukeys); free(h_rows); free(h_out); free(h_midx); free(h_inv);
    return rc;
}
