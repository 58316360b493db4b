"""Algorithm 1 (cache lookup with hit-rate-controlled synchronous or asynchronous insertion)
through hps_lookup against the oracle's statement of the same procedure (hpso_lookup).

The lower tiers are a Python callback that returns the backing generator's rows.  After every
asynchronous lookup the test drains the background queue, which makes the cache state after each
step unique; rows of `out`, hit rate, chosen mode and the canonical cache state are compared."""
import ctypes as C

import numpy as np
import pytest
import torch

from oracle import OracleCache
from paper_2210_08804_amd import binding as B
from paper_2210_08804_amd import inputs
from harness import (DeviceCache, SENTINEL, assert_same_state, check_state_invariants,
                     insert_is_order_independent)

pytestmark = pytest.mark.gpu


def make_fetch(d, log):
    def fetch(user, keys_p, n, rows_p):
        keys = np.ctypeslib.as_array(keys_p, shape=(n,))
        assert len(np.unique(keys)) == n                      # the lower tiers see each key once
        log.append(int(n))
        np.ctypeslib.as_array(rows_p, shape=(n, d))[...] = inputs.backing_rows(keys, d, 0)
    return B.FETCH_FN(fetch)


def reference_step(oc, keys, d, threshold, default_row):
    """Alg. 1 on the oracle (oracle/hps_oracle.c: hpso_lookup, pinned by tests/test_oracle_lookup.py),
    stopping before the insertion so that the test can classify the batch first.  Returns
    (out, hit_rate, synchronous, distinct missing keys in first-occurrence order or None)."""
    out, rate, sync, to_insert = oc.lookup(keys, inputs.backing_rows(keys, d, 0), threshold, default_row,
                                           do_insert=False)
    return out, rate, sync, (to_insert if len(to_insert) else None)


@pytest.mark.parametrize("threshold", [0.0, 0.8, 2.0])
def test_lookup_follows_algorithm_1(threshold):
    S, W, d, n = 1 << 10, 8, 32, 6000
    default_row = np.linspace(-1, 1, d).astype(np.float32)
    log = []
    fetch = make_fetch(d, log)
    with DeviceCache(S * W, W, d, concurrent_writers=True) as gc:
        oc = OracleCache(S * W, W, d)
        lk = B.hps_lookup_create(gc.h, n, threshold, default_row, fetch)
        try:
            modes = []
            for step in range(14):
                keys = inputs.zipf_keys(n if step % 3 else n // 2, 12000, 1.1, step + 1)
                out = torch.zeros(len(keys), d, dtype=torch.float32, device="cuda")
                rate, sync = B.hps_lookup(lk, torch.from_numpy(keys).cuda(), len(keys), out)
                B.hps_lookup_drain(lk)
                torch.cuda.synchronize()
                exp_out, exp_rate, exp_sync, to_insert = reference_step(oc, keys, d, threshold, default_row)
                assert np.float32(rate) == exp_rate and sync == exp_sync
                assert (out.cpu().numpy().view(np.uint32) == exp_out).all()
                modes.append(sync)
                if to_insert is not None:
                    exact = insert_is_order_independent(oc, to_insert)
                    oc.insert(to_insert, inputs.backing_rows(to_insert, d, 0))
                    state = gc.export()
                    if exact:
                        assert_same_state(state, oc)
                    else:
                        check_state_invariants(*state, oc.set_of)
                    oc.load_state(*state)
            if threshold == 0.0:
                assert not any(modes)
            elif threshold == 2.0:
                assert all(modes)
            else:
                assert modes[0] and not modes[-1]             # warm-up synchronous, then asynchronous (Sec. 4.3)
            assert len(log) >= 10
        finally:
            B.hps_lookup_destroy(lk)


def test_lookup_argument_errors_and_empty_batch():
    d = 16
    fetch = make_fetch(d, [])
    with DeviceCache(64, 8, d) as gc:
        with pytest.raises(B.HpsError):
            B.hps_lookup_create(None, 10, 0.5, np.zeros(d, np.float32), fetch)
        with pytest.raises(B.HpsError):
            B.hps_lookup_create(gc.h, 0, 0.5, np.zeros(d, np.float32), fetch)
        lk = B.hps_lookup_create(gc.h, 100, 0.5, np.zeros(d, np.float32), fetch)
        try:
            keys = torch.zeros(200, dtype=torch.int64, device="cuda")
            out = torch.zeros(200, d, dtype=torch.float32, device="cuda")
            with pytest.raises(B.HpsError):
                B.hps_lookup(lk, keys, 200, out)              # beyond max_batch
            rate, sync = B.hps_lookup(lk, keys, 0, out)
            assert rate == 1.0 and not sync
        finally:
            B.hps_lookup_destroy(lk)


@pytest.mark.parametrize("threshold", [0.8, 2.0])
def test_lookup_with_the_native_host_map_as_lower_tier(threshold):
    """Alg. 1 end to end without Python in the loop: the lower tier is the library's host map
    (hps_hostmap.h), handed to the lookup object as its fetch function."""
    S, W, d, n, space = 1 << 10, 8, 32, 6000, 12000
    default_row = np.full(d, 0.25, dtype=np.float32)
    all_keys = np.arange(space, dtype=np.int64)
    hm = B.hps_hostmap_create(d, 16, space)
    B.hps_hostmap_put(hm, all_keys, inputs.backing_rows(all_keys, d, 0))
    fetch = B.hps_hostmap_fetch_fn()
    with DeviceCache(S * W, W, d, concurrent_writers=True) as gc:
        oc = OracleCache(S * W, W, d)
        lk = B.hps_lookup_create(gc.h, n, threshold, default_row, fetch, user=hm)
        try:
            modes = []
            for step in range(12):
                keys = inputs.zipf_keys(n, space, 1.1, step + 1)
                out = torch.zeros(n, d, dtype=torch.float32, device="cuda")
                rate, sync = B.hps_lookup(lk, torch.from_numpy(keys).cuda(), n, out)
                B.hps_lookup_drain(lk)
                torch.cuda.synchronize()
                exp_out, exp_rate, exp_sync, to_insert = reference_step(oc, keys, d, threshold, default_row)
                assert np.float32(rate) == exp_rate and sync == exp_sync
                assert (out.cpu().numpy().view(np.uint32) == exp_out).all()
                modes.append(sync)
                if to_insert is not None:
                    exact = insert_is_order_independent(oc, to_insert)
                    oc.insert(to_insert, inputs.backing_rows(to_insert, d, 0))
                    state = gc.export()
                    if exact:
                        assert_same_state(state, oc)
                    else:
                        check_state_invariants(*state, oc.set_of)
                    oc.load_state(*state)
            assert modes[0] and (threshold > 1 or not modes[-1])
            n_keys, n_absent = B.hps_hostmap_stats(hm)
            assert n_keys == space and n_absent == 0          # every key asked for was a stored one
        finally:
            B.hps_lookup_destroy(lk)
            B.hps_hostmap_destroy(hm)


def test_queued_background_batches_are_merged_and_stay_distinct():
    """Asynchronous calls issued faster than the lower tier answers queue up; the worker merges
    what has queued, the lower tier still sees distinct keys in every call, and once drained the
    cache holds every key that was asked for."""
    import time
    S, W, d, n = 1 << 16, 8, 16, 5000                      # 27 k keys over 65 k sets: no set overflows
    calls = []

    def slow_fetch(user, keys_p, m, rows_p):
        keys = np.ctypeslib.as_array(keys_p, shape=(m,)).copy()
        calls.append(keys)
        time.sleep(0.02)                                       # a slow tier: later batches pile up
        rows = np.ctypeslib.as_array(rows_p, shape=(m, d))
        rows[...] = inputs.backing_rows(keys, d, 0)

    fetch = B.FETCH_FN(slow_fetch)
    with DeviceCache(S * W, W, d, concurrent_writers=True) as gc:
        lk = B.hps_lookup_create(gc.h, 4 * n, 0.0, np.zeros(d, np.float32), fetch)
        try:
            asked = []
            for step in range(8):
                keys = inputs.uniform_keys(n, 40000, 80 + step)
                asked.append(keys)
                out = torch.zeros(n, d, dtype=torch.float32, device="cuda")
                rate, sync = B.hps_lookup(lk, torch.from_numpy(keys).cuda(), n, out)
                assert not sync
            B.hps_lookup_drain(lk)
            torch.cuda.synchronize()
            assert all(len(np.unique(c)) == len(c) for c in calls), "the lower tier was handed a key twice in one call"
            assert len(calls) < 8, "queued batches were not merged"
            everything = np.unique(np.concatenate(asked))
            got, mi, _ = gc.query(everything)
            assert len(mi) == 0
            assert (got == inputs.backing_rows(everything, d, 0).view(np.uint32)).all()
        finally:
            B.hps_lookup_destroy(lk)


def test_a_lower_tier_that_falls_far_behind_loses_the_oldest_batches_only():
    """More asynchronous batches than may wait (64): the oldest are dropped, nothing breaks, and
    what was not dropped arrives whole."""
    import time
    S, W, d, n, calls_n = 1 << 16, 8, 16, 500, 120
    fetched = []

    def slow_fetch(user, keys_p, m, rows_p):
        keys = np.ctypeslib.as_array(keys_p, shape=(m,)).copy()
        fetched.append(keys)
        time.sleep(0.01)
        np.ctypeslib.as_array(rows_p, shape=(m, d))[...] = inputs.backing_rows(keys, d, 0)

    fetch = B.FETCH_FN(slow_fetch)
    with DeviceCache(S * W, W, d, concurrent_writers=True) as gc:
        lk = B.hps_lookup_create(gc.h, n, 0.0, np.zeros(d, np.float32), fetch)      # one batch per background round
        try:
            asked = [np.arange(step * n, (step + 1) * n, dtype=np.int64) for step in range(calls_n)]
            out = torch.zeros(n, d, dtype=torch.float32, device="cuda")
            for keys in asked:
                B.hps_lookup(lk, torch.from_numpy(keys).cuda(), n, out)
            B.hps_lookup_drain(lk)
            torch.cuda.synchronize()
            got_keys = np.concatenate(fetched)
            assert len(np.unique(got_keys)) == len(got_keys)
            assert 64 * n <= len(got_keys) < calls_n * n, "either nothing was dropped or too much"
            everything = np.concatenate(asked)
            out_all, mi, mk = gc.query(everything)
            assert sorted(mk.tolist()) == sorted(set(everything.tolist()) - set(got_keys.tolist()))
            hit = np.ones(len(everything), dtype=bool)
            hit[mi] = False
            assert (out_all[hit] == inputs.backing_rows(everything[hit], d, 0).view(np.uint32)).all()
            # the object still works
            rate, sync = B.hps_lookup(lk, torch.from_numpy(asked[-1]).cuda(), n, out)
            assert rate == 1.0 and not sync
        finally:
            B.hps_lookup_destroy(lk)


@pytest.mark.parametrize("batch_slots", [1000, 4096, 1 << 20])
def test_refresh_cycle_from_the_host_map(batch_slots):
    """Sec. 6, Fig. 3 steps 1-5 through hps_cache_refresh: every cached key gets the row the lower
    tier holds now; nothing else changes (same keys, same counters)."""
    S, W, d = 1 << 10, 8, 32
    keys = np.unique(inputs.uniform_keys(6000, 1 << 30, 91))
    with DeviceCache(S * W, W, d, concurrent_writers=True) as gc:
        oc = OracleCache(S * W, W, d)
        for ck in np.array_split(keys, 4):
            gc.insert(ck, inputs.backing_rows(ck, d, 0))
        oc.load_state(*gc.export())
        cached = oc.dump()
        hm = B.hps_hostmap_create(d, 8, len(keys))
        try:
            B.hps_hostmap_put(hm, keys, inputs.backing_rows(keys, d, 1))          # the lower tier has moved on
            n = B.hps_cache_refresh(gc.h, batch_slots, B.hps_hostmap_fetch_fn(), user=hm)
            torch.cuda.synchronize()
            assert n == len(cached)
            oc.update(cached, inputs.backing_rows(cached, d, 1))
            assert_same_state(gc.export(), oc)
            assert B.hps_hostmap_stats(hm)[1] == 0                               # only stored keys were asked for
            # the same through a session that is created once and run twice (its runs allocate nothing)
            rs = B.hps_refresh_create(gc.h, batch_slots)
            try:
                for version in (2, 3):
                    B.hps_hostmap_put(hm, keys, inputs.backing_rows(keys, d, version))
                    assert B.hps_refresh_run(rs, B.hps_hostmap_fetch_fn(), user=hm) == len(cached)
                    torch.cuda.synchronize()
                    oc.update(cached, inputs.backing_rows(cached, d, version))
                    assert_same_state(gc.export(), oc)
            finally:
                B.hps_refresh_destroy(rs)
        finally:
            B.hps_hostmap_destroy(hm)


def test_refresh_cycle_overlapping_queries_returns_whole_rows():
    S, W, d, n_q = 1 << 12, 8, 64, 20000
    keys = np.unique(inputs.uniform_keys(30000, 1 << 30, 92))
    with DeviceCache(S * W, W, d, concurrent_writers=True) as gc:
        for ck in np.array_split(keys, 8):
            gc.insert(ck, inputs.backing_rows(ck, d, 0))
        hm = B.hps_hostmap_create(d, 8, len(keys))
        try:
            B.hps_hostmap_put(hm, keys, inputs.backing_rows(keys, d, 1))
            qs = torch.cuda.Stream()
            rs = torch.cuda.Stream()
            q = keys[np.random.Generator(np.random.PCG64(5)).integers(0, len(keys), n_q)]
            dq = torch.from_numpy(q).cuda()
            outs = [torch.full((n_q, d), SENTINEL, dtype=torch.int32, device="cuda").view(torch.float32) for _ in range(40)]
            mi = torch.empty(n_q, dtype=torch.int32, device="cuda")
            mk = torch.empty(n_q, dtype=torch.int64, device="cuda")
            nm = torch.zeros(40, dtype=torch.int32, device="cuda")
            torch.cuda.synchronize()
            import threading
            t = threading.Thread(target=lambda: B.hps_cache_refresh(gc.h, 2048, B.hps_hostmap_fetch_fn(), user=hm, stream=rs))
            t.start()
            for i in range(40):
                B.hps_cache_query(gc.h, dq, n_q, outs[i], mi, mk, nm[i:i + 1], qs)
            t.join()
            torch.cuda.synchronize()
            v0 = inputs.backing_rows(q, d, 0).view(np.uint32)
            v1 = inputs.backing_rows(q, d, 1).view(np.uint32)
            seen_new = 0
            for i in range(40):
                o = outs[i].view(torch.int32).cpu().numpy().view(np.uint32)
                hit = ~(o == SENTINEL).all(axis=1)
                is0 = (o == v0).all(axis=1)
                is1 = (o == v1).all(axis=1)
                assert (is0 | is1)[hit].all(), "a row is neither the old nor the new version"
                seen_new += int(is1[hit].sum())
            got, mi2, _ = gc.query(q)
            hit = np.ones(n_q, dtype=bool)
            hit[mi2] = False
            assert (got[hit] == v1[hit]).all()                                   # after the refresh everything is new
        finally:
            B.hps_hostmap_destroy(hm)


@pytest.mark.parametrize("threshold", [2.0, 0.7])
def test_three_lookup_objects_on_three_threads_share_one_cache(threshold):
    """Several inference workers share the GPU's embedding cache (Sec. 3.1, Sec. 7.2.2): three
    threads, each with its own lookup object and stream, look batches up at the same time.  In
    synchronous mode every row must be its key's row; in the mixed mode a row is its key's row or
    the default row; afterwards the cache state is a legal one."""
    import threading
    S, W, d, n, space, steps = 1 << 12, 8, 32, 4000, 60000, 12
    default_row = np.full(d, -3.0, dtype=np.float32)
    all_keys = np.arange(space, dtype=np.int64)
    hm = B.hps_hostmap_create(d, 16, space)
    B.hps_hostmap_put(hm, all_keys, inputs.backing_rows(all_keys, d, 0))
    fetch = B.hps_hostmap_fetch_fn()
    errors = []
    with DeviceCache(S * W, W, d, concurrent_writers=True) as gc:
        lks = [B.hps_lookup_create(gc.h, n, threshold, default_row, fetch, user=hm) for _ in range(3)]

        def worker(t):
            try:
                torch.cuda.set_device(0)
                st = torch.cuda.Stream()
                for step in range(steps):
                    keys = inputs.zipf_keys(n, space, 1.1, 1000 * t + step)
                    dk = torch.from_numpy(keys).cuda()
                    out = torch.zeros(n, d, dtype=torch.float32, device="cuda")
                    torch.cuda.synchronize()
                    rate, sync = B.hps_lookup(lks[t], dk, n, out, st)
                    st.synchronize()
                    got = out.cpu().numpy().view(np.uint32)
                    exp = inputs.backing_rows(keys, d, 0).view(np.uint32)
                    right = (got == exp).all(axis=1)
                    dflt = (got == default_row.view(np.uint32)).all(axis=1)
                    if threshold > 1.0 and not right.all():
                        errors.append(f"thread {t} step {step}: {int((~right).sum())} wrong rows in synchronous mode")
                    if not (right | dflt).all():
                        errors.append(f"thread {t} step {step}: a row is neither its key's row nor the default row")
                    if not 0.0 <= rate <= 1.0:
                        errors.append(f"thread {t}: hit rate {rate}")
            except Exception as exc:                         # noqa: BLE001 - reported by the main thread
                errors.append(f"thread {t}: {exc!r}")

        threads = [threading.Thread(target=worker, args=(t,)) for t in range(3)]
        try:
            for th in threads:
                th.start()
            for th in threads:
                th.join()
            for lk in lks:
                B.hps_lookup_drain(lk)
            torch.cuda.synchronize()
            assert not errors, errors[:5]
            oc = OracleCache(S * W, W, d)
            check_state_invariants(*gc.export(), oc.set_of,
                                   expect_row=lambda k: [inputs.backing_rows(np.array([k]), d, 0).view(np.uint32)[0]])
            assert B.hps_hostmap_stats(hm)[1] == 0
        finally:
            for lk in lks:
                B.hps_lookup_destroy(lk)
            B.hps_hostmap_destroy(hm)
