"""Update on one stream while queries run on another (the online-update path, Sec. 6): a reader
must see, for every hit, the complete row of ONE version of its key, never a mixture, and on one
stream later queries never see an older version than earlier ones.  After both streams are
synchronised a full re-query must equal the oracle (last version) bit for bit."""
import os

import numpy as np
import pytest
import torch

from oracle import OracleCache
from paper_2210_08804_amd import binding as B
from paper_2210_08804_amd import inputs
from harness import DeviceCache, SENTINEL

pytestmark = pytest.mark.gpu

# HPS_TEST_SEED_SHIFT=k in the environment runs the same tests on other random streams (a longer
# soak is then a shell loop over k); the default is the fixed stream the suite is tuned to.
SEED_SHIFT = int(os.environ.get("HPS_TEST_SEED_SHIFT", "0"))


def versions_seen(out_u32, keys, d, n_versions):
    """For every position: the version v whose generated row equals the output row exactly,
    -1 for untouched (sentinel) rows, -2 if the row matches no single version (torn)."""
    seen = np.full(len(keys), -2, dtype=np.int64)
    seen[(out_u32 == SENTINEL).all(axis=1)] = -1
    for v in range(n_versions):
        exp = inputs.backing_rows(keys, d, v).view(np.uint32)
        seen[(out_u32 == exp).all(axis=1)] = v
    return seen


@pytest.mark.parametrize("S,W,d,n_q,n_u", [(1 << 12, 8, 128, 20000, 16384), (1 << 10, 8, 320, 6000, 4096),
                                           (1 << 12, 8, 16, 30000, 24576)])
def test_update_overlapping_queries_never_tears_rows(S, W, d, n_q, n_u):
    n_versions, n_queries = 8, 24
    ids = np.arange(S * W // 2, dtype=np.int64)                         # about half full
    rng = np.random.Generator(np.random.PCG64(S + d + SEED_SHIFT))
    with DeviceCache(S * W, W, d, concurrent_writers=True) as gc:
        oc = OracleCache(S * W, W, d)
        for ck in np.array_split(ids, 16):
            gc.insert(ck, inputs.backing_rows(ck, d, 0))
        oc.load_state(*gc.export())         # a few sets overflow: take the GPU's (legal) choice of survivors
        resident = np.sort(oc.dump())
        assert len(resident) > 0.95 * len(ids)

        qs, us = torch.cuda.Stream(), torch.cuda.Stream()
        # update batches: 50 % resident keys, 50 % absent ones; version = batch number
        upd_keys = [np.concatenate([rng.choice(resident, n_u // 2, replace=False),
                                    rng.integers(S * W, 4 * S * W, n_u // 2)]).astype(np.int64)
                    for _ in range(1, n_versions)]
        d_upd = [(torch.from_numpy(k).cuda(),
                  torch.from_numpy(inputs.backing_rows(k, d, v + 1)).cuda()) for v, k in enumerate(upd_keys)]
        q_keys = [rng.choice(resident, n_q).astype(np.int64) for _ in range(n_queries)]
        d_q = [torch.from_numpy(k).cuda() for k in q_keys]
        outs = [torch.full((n_q, d), SENTINEL, dtype=torch.int32, device="cuda").view(torch.float32)
                for _ in range(n_queries)]
        mi = [torch.empty(n_q, dtype=torch.int32, device="cuda") for _ in range(n_queries)]
        mk = [torch.empty(n_q, dtype=torch.int64, device="cuda") for _ in range(n_queries)]
        nm = torch.full((n_queries,), -1, dtype=torch.int32, device="cuda")
        torch.cuda.synchronize()

        # interleave the launches so that the two streams overlap on the device
        ui = 0
        for qi in range(n_queries):
            B.hps_cache_query(gc.h, d_q[qi], n_q, outs[qi], mi[qi], mk[qi], nm[qi:qi + 1], qs)
            if qi % 3 == 1 and ui < len(d_upd):
                B.hps_cache_update(gc.h, d_upd[ui][0], d_upd[ui][1], n_u, us)
                ui += 1
        while ui < len(d_upd):
            B.hps_cache_update(gc.h, d_upd[ui][0], d_upd[ui][1], n_u, us)
            ui += 1
        torch.cuda.synchronize()

        assert (nm.cpu().numpy() == 0).all(), "update must not change residency"
        last = {}
        for qi in range(n_queries):
            out = outs[qi].view(torch.int32).cpu().numpy().view(np.uint32)
            seen = versions_seen(out, q_keys[qi], d, n_versions)
            assert (seen != -2).all(), f"query {qi}: {(seen == -2).sum()} rows match no single version (torn)"
            assert (seen >= 0).all()
            # positions of one query are not ordered in time, queries on one stream are:
            # nothing in this query may be older than the newest version an earlier query saw
            newest = {}
            for k, v in zip(q_keys[qi].tolist(), seen.tolist()):
                assert v >= last.get(k, 0), "a later query saw an older version"
                newest[k] = max(newest.get(k, 0), v)
            last.update(newest)
        # quiesced: equals the oracle with every update applied in order
        for v, k in enumerate(upd_keys):
            oc.update(k, inputs.backing_rows(k, d, v + 1))
        allk = np.arange(S * W, dtype=np.int64)
        out_g, mi_g, mk_g = gc.query(allk)
        out_o = np.full((len(allk), d), SENTINEL, dtype=np.uint32)
        _, mi_o, mk_o = oc.query(allk, out_o)
        assert (mi_g == mi_o).all() and (out_g == out_o).all()


@pytest.mark.parametrize("S,d,n_q,n_i", [(1 << 9, 128, 20000, 4096), (1 << 7, 320, 6000, 1024),
                                         (1 << 7, 512, 6000, 1024), (1 << 6, 1024, 3000, 512)])
def test_insert_overlapping_queries_keeps_rows_whole(S, d, n_q, n_i):
    """Queries racing with inserts (cache filling up and evicting): every row returned is the
    complete row of its key (rows are a function of the key here), misses leave `out` untouched.
    Rows longer than 1 KiB (d > 256) are read in several wave loads: a key that an insert evicts
    between them must come out as a miss whose `out` row still holds the sentinel in every word."""
    W = 8
    rng = np.random.Generator(np.random.PCG64(99 + SEED_SHIFT))
    with DeviceCache(S * W, W, d, concurrent_writers=True) as gc:
        qs, ws = torch.cuda.Stream(), torch.cuda.Stream()
        ins_keys = [rng.integers(0, 3 * S * W, n_i).astype(np.int64) for _ in range(12)]
        d_ins = [(torch.from_numpy(k).cuda(), torch.from_numpy(inputs.backing_rows(k, d, 0)).cuda()) for k in ins_keys]
        q_keys = [rng.integers(0, 3 * S * W, n_q).astype(np.int64) for _ in range(24)]
        d_q = [torch.from_numpy(k).cuda() for k in q_keys]
        outs = [torch.full((n_q, d), SENTINEL, dtype=torch.int32, device="cuda").view(torch.float32) for _ in q_keys]
        mi = [torch.full((n_q,), -1, dtype=torch.int32, device="cuda") for _ in q_keys]
        mk = [torch.empty(n_q, dtype=torch.int64, device="cuda") for _ in q_keys]
        nm = torch.full((len(q_keys),), -1, dtype=torch.int32, device="cuda")
        torch.cuda.synchronize()
        for qi in range(len(q_keys)):
            B.hps_cache_query(gc.h, d_q[qi], n_q, outs[qi], mi[qi], mk[qi], nm[qi:qi + 1], qs)
            if qi % 2 == 0:
                B.hps_cache_insert(gc.h, d_ins[qi // 2][0], d_ins[qi // 2][1], n_i, ws)
        torch.cuda.synchronize()
        n_late = 0
        for qi in range(len(q_keys)):
            out = outs[qi].view(torch.int32).cpu().numpy().view(np.uint32)
            m = int(nm[qi].item())
            midx = np.sort(mi[qi][:m].cpu().numpy().view(np.uint32))
            assert len(np.unique(midx)) == m
            missed = np.zeros(n_q, dtype=bool)
            missed[midx] = True
            exp = inputs.backing_rows(q_keys[qi], d, 0).view(np.uint32)
            assert (out[~missed] == exp[~missed]).all(), "a hit returned something else than its key's row"
            assert (out[missed] == SENTINEL).all(), "a miss row was written"
            got_mk = mk[qi][:m].cpu().numpy()[np.argsort(mi[qi][:m].cpu().numpy().view(np.uint32))]
            assert (got_mk == q_keys[qi][midx]).all()
        # final state is a legal cache state
        from harness import check_state_invariants
        gk, gctr, gv = gc.export()
        oc = OracleCache(S * W, W, d)
        check_state_invariants(gk, gctr, gv, oc.set_of,
                               expect_row=lambda k: [inputs.backing_rows(np.array([k]), d, 0).view(np.uint32)[0]])


def test_inserts_and_updates_on_three_streams_keep_the_invariants():
    """insert || insert || update across streams (batches that share keys, sets that fill up and
    evict): after every round the state must be a legal cache state - no key twice, every key in
    its own set, ways filled in order, counters equal to the number of keys each set took in, and
    every row whole: the inserted row of its key or one of the rows an update gave it."""
    from harness import check_state_invariants
    S, W, d, n_i, n_u = 1 << 9, 8, 64, 3000, 2048
    space = 3 * S * W
    rng = np.random.Generator(np.random.PCG64(123 + SEED_SHIFT))
    oc = OracleCache(S * W, W, d)                        # only for set_of
    with DeviceCache(S * W, W, d, concurrent_writers=True) as gc:
        sa, sb, su = torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream()
        versions = {}                                    # key -> versions an update carried for it
        prev_ctr = np.zeros(S, dtype=np.int64)
        for rnd in range(1, 9):
            ka = rng.integers(0, space, n_i).astype(np.int64)
            kb = np.concatenate([ka[: n_i // 2], rng.integers(0, space, n_i // 2).astype(np.int64)])   # half shared with ka
            rng.shuffle(kb)
            ku = rng.integers(0, space, n_u).astype(np.int64)
            for k in ku.tolist():
                versions.setdefault(k, set()).add(rnd)
            da, db, du = (torch.from_numpy(k).cuda() for k in (ka, kb, ku))
            ra = torch.from_numpy(inputs.backing_rows(ka, d, 0)).cuda()
            rb = torch.from_numpy(inputs.backing_rows(kb, d, 0)).cuda()
            ru = torch.from_numpy(inputs.backing_rows(ku, d, rnd)).cuda()
            torch.cuda.synchronize()
            B.hps_cache_insert(gc.h, da, ra, n_i, sa)
            B.hps_cache_insert(gc.h, db, rb, n_i, sb)
            B.hps_cache_update(gc.h, du, ru, n_u, su)
            torch.cuda.synchronize()
            gk, gctr, gv = gc.export()

            def allowed(k):
                vs = [0] + sorted(versions.get(k, ()))
                return [inputs.backing_rows(np.array([k]), d, v).view(np.uint32)[0] for v in vs]
            check_state_invariants(gk, gctr, gv, oc.set_of, expect_row=allowed)
            # a set's counter grows by the number of keys it took in: never backwards, and never by more
            # than the keys offered (a key of both batches can go in twice when its set overflowed
            # and evicted it in between)
            ctr = gctr.astype(np.int64)
            assert (ctr >= prev_ctr).all()
            assert 0 < (ctr - prev_ctr).sum() <= 2 * n_i
            prev_ctr = ctr
        assert B.hps_cache_flags(gc.h) == 0


def test_more_stream_handles_than_counter_words():
    """Every stream that queries gets a counter word of its own; a caller that goes through more
    stream handles than the pool has words must still get correct miss lists on all of them."""
    import ctypes as C
    hip = C.CDLL("libamdhip64.so")
    hip.hipStreamCreateWithFlags.argtypes = [C.POINTER(C.c_void_p), C.c_uint]
    hip.hipStreamDestroy.argtypes = [C.c_void_p]
    S, W, d, n = 64, 8, 16, 300
    keys = inputs.uniform_keys(n, 500, 9)
    with DeviceCache(S * W, W, d, concurrent_writers=False) as gc:
        oc = OracleCache(S * W, W, d)
        resident = np.unique(keys)[::2].copy()
        gc.insert(resident, inputs.backing_rows(resident, d))
        oc.insert(resident, inputs.backing_rows(resident, d).view(np.uint32))
        exp_out = np.full((n, d), SENTINEL, dtype=np.uint32)
        _, exp_mi, _ = oc.query(keys, exp_out)
        dk = torch.from_numpy(keys).cuda()
        streams, results = [], []
        try:
            for i in range(1100):
                h = C.c_void_p()
                assert hip.hipStreamCreateWithFlags(C.byref(h), 1) == 0          # non-blocking
                streams.append(h)
                st = torch.cuda.ExternalStream(h.value)
                out = torch.full((n, d), SENTINEL, dtype=torch.int32, device="cuda").view(torch.float32)
                mi = torch.empty(n, dtype=torch.int32, device="cuda")
                mk = torch.empty(n, dtype=torch.int64, device="cuda")
                nm = torch.zeros(1, dtype=torch.int32, device="cuda")
                torch.cuda.current_stream().synchronize()                        # the fills above are done
                B.hps_cache_query(gc.h, dk, n, out, mi, mk, nm, st)
                results.append((out, mi, nm))
                if i % 100 == 99 or i >= 1020:                                   # around the switch of pools, and samples
                    torch.cuda.synchronize()
                    for o, m_i, n_m in results:
                        m = int(n_m.item())
                        assert m == len(exp_mi)
                        assert (np.sort(m_i[:m].cpu().numpy().view(np.uint32)) == exp_mi).all()
                        assert (o.view(torch.int32).cpu().numpy().view(np.uint32) == exp_out).all()
                    results.clear()
        finally:
            torch.cuda.synchronize()
            for h in streams:
                hip.hipStreamDestroy(h)
