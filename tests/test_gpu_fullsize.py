"""Parity at the full sizes of the workloads, in the launch configuration the benchmark times.

The oracle runs with dim = 1: its one-word row is the version tag of the key's row, and the
expected fp32 row is the backing generator's row for (key, version), generated on the host by
paper_2210_08804_amd.inputs and compared with every row the GPU returned (the comparison itself,
an index and an equality test, runs as torch ops on the device; no expected value comes from a
HIP kernel of the library).

Cache states are built on the GPU through hps_cache_insert and followed by the oracle batch by
batch.  The canonical state of an insert batch is unique when no set receives more than W new
keys; which way each of several same-batch arrivals of one set takes is free and decides later
evictions, so after every batch the oracle adopts the GPU's way order in exactly those sets
(after checking that the sets hold the same keys).  Sets that overflow within one batch are
checked by the invariants and adopted whole.
"""
import time

import numpy as np
import pytest
import torch

from oracle import OracleCache
from paper_2210_08804_amd import binding as B
from paper_2210_08804_amd import inputs
from harness import DeviceCache, SENTINEL, EMPTY_KEY, canonical

pytestmark = pytest.mark.gpu

MISS_TAG = 0xFFFFFFFF


# ---------------------------------------------------------------- plumbing

class DeviceState:
    """Keys and counters of a GPU cache exported into device buffers (hps_cache_export); only
    the sets a test asks for travel to the host."""

    def __init__(self, gc):
        self.gc = gc
        self.k = torch.empty(gc.S * gc.W, dtype=torch.int64, device="cuda")
        self.c = torch.empty(gc.S, dtype=torch.int32, device="cuda")

    def refresh(self):
        B.hps_cache_export(self.gc.h, self.k, self.c, None)
        torch.cuda.synchronize()

    def sets(self, set_ids):
        idx = torch.from_numpy(np.ascontiguousarray(set_ids, dtype=np.int64)).cuda()
        keys = self.k.view(self.gc.S, self.gc.W)[idx].cpu().numpy()
        ctr = self.c[idx].cpu().numpy().view(np.uint32)
        return keys, ctr

    def full(self):
        return self.k.cpu().numpy().reshape(self.gc.S, self.gc.W), self.c.cpu().numpy().view(np.uint32)


def oracle_tags(oc, keys):
    """(hit mask, version tag) per position; also returns the oracle's miss list."""
    tags = np.full((len(keys), 1), MISS_TAG, dtype=np.uint32)
    _, omi, omk = oc.query(keys, tags)
    return tags[:, 0] != MISS_TAG, tags[:, 0], omi, omk


def follow_insert(oc, dstate, batch_keys):
    """The batch has been given to hps_cache_insert (enqueued or done) with rows of version 0;
    apply it to the oracle and bring the oracle's way order in line with the GPU's where the
    batch left it open.  Returns (#sets with several new keys, #sets that overflowed in the batch)."""
    W = oc.W
    uk = np.unique(batch_keys)
    uk = uk[uk > EMPTY_KEY + 1]
    resident, _, _, _ = oracle_tags(oc, uk)
    new = uk[~resident]
    sets = oc.sets_of(new)
    us, cnt = np.unique(sets, return_counts=True)
    multi = us[cnt >= 2]
    over = us[cnt > W]
    old_keys = {int(s): oc.keys[int(s)].copy() for s in over}
    ctr_before = oc.ctr[us].copy()
    oc.insert(batch_keys, np.zeros((len(batch_keys), 1), dtype=np.uint32))
    fits = cnt <= W
    assert (oc.ctr[us[fits]] - ctr_before[fits] == cnt[fits].astype(np.uint32)).all()   # one step per new key
    dstate.refresh()
    if len(multi):
        gk, gctr = dstate.sets(multi)
        exact = ~np.isin(multi, over)
        assert (gctr[exact] == oc.ctr[multi[exact]]).all(), "victim counters differ in sets that received several keys"
        assert (np.sort(gk[exact], axis=1) == np.sort(oc.keys[multi[exact]], axis=1)).all(), \
            "a set that received several new keys holds different keys on the GPU"
        for j in np.nonzero(~exact)[0]:                     # overflowed within the batch: any legal outcome
            s = int(multi[j])
            row = gk[j]
            allowed = set(old_keys[s].tolist()) | set(new[sets == s].tolist())
            assert len(set(row.tolist())) == W and set(row.tolist()) <= allowed and EMPTY_KEY not in row
        assert (oc.vals[multi] == 0).all()                  # one tag everywhere: permuting keys needs no row moves
        oc.keys[multi] = gk                                 # same keys per set, the GPU's way order
        oc.ctr[multi] = gctr                                # (only changes overflowed sets)
    return len(multi), len(over)


def assert_full_state(dstate, oc):
    gk, gctr = dstate.full()
    assert (gctr == oc.ctr).all(), "victim counters differ"
    assert (np.sort(gk, axis=1) == np.sort(oc.keys, axis=1)).all(), "resident key sets differ"


class RowChecker:
    """Expected rows from the host generator, compared with device rows on the device.  Rows of
    the ids below `hot_ids` (version 0) are generated once and kept on the device as a table;
    everything else is generated per call for the distinct keys it needs."""

    def __init__(self, d, hot_ids):
        self.d = d
        self.hot = hot_ids
        self.table = torch.empty(hot_ids, d, dtype=torch.int32, device="cuda")
        step = 1 << 16
        for lo in range(0, hot_ids, step):
            hi = min(hot_ids, lo + step)
            rows = inputs.backing_rows(np.arange(lo, hi, dtype=np.int64), d, 0)
            self.table[lo:hi] = torch.from_numpy(rows.view(np.int32)).cuda()

    def expected(self, keys, versions=None):
        """Device int32 [n, d]: row of (key, version) for every position."""
        n = len(keys)
        exp = torch.empty(n, self.d, dtype=torch.int32, device="cuda")
        v = np.zeros(n, dtype=np.int64) if versions is None else np.asarray(versions, dtype=np.int64)
        hot = (keys >= 0) & (keys < self.hot) & (v == 0)
        if hot.any():
            pos = torch.from_numpy(np.nonzero(hot)[0]).cuda()
            exp[pos] = self.table[torch.from_numpy(keys[hot]).cuda()]
        cold = np.nonzero(~hot)[0]
        if len(cold):
            pairs = np.stack([keys[cold], v[cold]], axis=1)
            up, inv = np.unique(pairs, axis=0, return_inverse=True)
            chunk = 1 << 16
            rows = torch.empty(len(up), self.d, dtype=torch.int32, device="cuda")
            for lo in range(0, len(up), chunk):
                r = inputs.backing_rows(up[lo:lo + chunk, 0], self.d, up[lo:lo + chunk, 1])
                rows[lo:lo + chunk] = torch.from_numpy(r.view(np.int32)).cuda()
            exp[torch.from_numpy(cold).cuda()] = rows[torch.from_numpy(inv.reshape(-1)).cuda()]
        return exp

    def mismatches(self, out, keys, hit, versions=None):
        """Positions whose row is not what it must be: the row of (key, version) on a hit, the
        untouched sentinel on a miss.  Every row of `out` is looked at."""
        got = out.view(torch.int32)
        exp = self.expected(keys, versions)
        miss = torch.from_numpy(~hit).cuda()
        exp[miss] = SENTINEL
        bad = (got != exp).any(dim=1)
        return torch.nonzero(bad).reshape(-1).cpu().numpy()


def gpu_query(gc, dkeys, n):
    out = torch.full((n, gc.d), SENTINEL, dtype=torch.int32, device="cuda").view(torch.float32)
    mi = torch.empty(n, dtype=torch.int32, device="cuda")
    mk = torch.empty(n, dtype=torch.int64, device="cuda")
    nm = torch.full((1,), -1, dtype=torch.int32, device="cuda")
    B.hps_cache_query(gc.h, dkeys, n, out, mi, mk, nm)
    torch.cuda.synchronize()
    m = int(nm.item())
    return out, *sorted_miss_list(mi, mk, m)


def sorted_miss_list(mi, mk, m):
    order = torch.argsort(mi[:m].to(torch.int64) & 0xFFFFFFFF)
    return mi[:m][order].cpu().numpy().view(np.uint32), mk[:m][order].cpu().numpy()


def refresh_cycle(gc, version, slots_per_batch):
    """Sec. 6 steps 2-5 on the device: dump a slot range, fetch the rows, update the cache."""
    total = gc.S * gc.W
    keys = torch.empty(slots_per_batch, dtype=torch.int64, device="cuda")
    rows = torch.empty(slots_per_batch, gc.d, dtype=torch.float32, device="cuda")
    cnt = torch.zeros(1, dtype=torch.int32, device="cuda")
    dumped = 0
    for first in range(0, total, slots_per_batch):
        m = min(slots_per_batch, total - first)
        B.hps_cache_dump(gc.h, first, m, keys, cnt)
        B.hps_backing_fetch(keys, m, gc.d, version=version, rows=rows, n_dev=cnt)
        B.hps_cache_update_dn(gc.h, keys, rows, m, cnt)
        dumped += int(cnt.item())
    torch.cuda.synchronize()
    return dumped


def gpu_prefill_descending(gc, oc, n_ids, chunk):
    """ids n_ids-1 .. 0 through hps_cache_insert in chunks (rows from the device-side lower-tier
    stand-in), the oracle following every chunk.  Returns the DeviceState used."""
    dstate = DeviceState(gc)
    ids = torch.empty(chunk, dtype=torch.int64, device="cuda")
    rows = torch.empty(chunk, gc.d, dtype=torch.float32, device="cuda")
    n_multi = n_over = 0
    for hi in range(n_ids, 0, -chunk):
        lo = max(0, hi - chunk)
        m = hi - lo
        batch = np.arange(hi - 1, lo - 1, -1, dtype=np.int64)
        ids[:m] = torch.from_numpy(batch).cuda()
        B.hps_backing_fetch(ids, m, gc.d, version=0, rows=rows)
        B.hps_cache_insert(gc.h, ids, rows, m)
        a, b = follow_insert(oc, dstate, batch)
        n_multi += a
        n_over += b
    return dstate, n_multi, n_over


def oracle_prefill_descending(oc, n_ids, chunk):
    tags = np.zeros((chunk, 1), dtype=np.uint32)
    for hi in range(n_ids, 0, -chunk):
        lo = max(0, hi - chunk)
        oc.insert(np.arange(hi - 1, lo - 1, -1, dtype=np.int64), tags[: hi - lo])


# ---------------------------------------------------------------- hot-cache query

@pytest.fixture(scope="module")
def c2_state():
    """The hot-cache state, built once: on the GPU through hps_cache_insert (chunks of 2^18 ids,
    descending), followed by the oracle chunk by chunk and compared in full at the end.  The
    other query variants import the same state."""
    S, W, d = 1 << 21, 8, 128
    oc = OracleCache(S * W, W, 1)
    with DeviceCache(S * W, W, d, concurrent_writers=False) as gc:
        dstate, n_multi, n_over = gpu_prefill_descending(gc, oc, S * W, 1 << 18)
        assert n_multi > 1000 and n_over == 0            # way order was open in many sets, none overflowed in a chunk
        assert_full_state(dstate, oc)
        occupied = int((oc.keys != EMPTY_KEY).sum())
        assert 0.84 < occupied / (S * W) < 0.88          # Poisson(8) loads truncated at 8 ways: about 0.86
        assert (oc.ctr > W).sum() > 0.3 * S              # many sets evicted (counter beyond the ways)
        checker = RowChecker(d, 1 << 20)
        # the rows the inserts stored, read back through queries: every 16th id, all rows compared
        sweep = np.arange(0, S * W, 16, dtype=np.int64)
        hit, _, omi, omk = oracle_tags(oc, sweep)
        out, gmi, gmk = gpu_query(gc, torch.from_numpy(sweep).cuda(), len(sweep))
        assert len(gmi) == len(omi) and (gmi == omi).all() and (gmk == omk).all()
        assert len(checker.mismatches(out, sweep, hit)) == 0
        yield oc, gc, checker
    oc.close()


@pytest.mark.parametrize("mode", ["plain", "checked", "dedup"])
def test_c2_hot_cache_query_full_size(c2_state, mode):
    oc, gc0, checker = c2_state
    S, W, d = 1 << 21, 8, 128
    n = 4096 * 26
    if mode == "plain":
        run_c2_batches(gc0, oc, checker, n)
        return
    with DeviceCache(S * W, W, d, concurrent_writers=(mode == "checked")) as gc:
        B.hps_cache_set_query_dedup(gc.h, mode == "dedup")
        gc.load(np.array(oc.keys), np.array(oc.ctr))
        assert refresh_cycle(gc, 0, 1 << 22) == int((oc.keys != EMPTY_KEY).sum())
        run_c2_batches(gc, oc, checker, n)


def run_c2_batches(gc, oc, checker, n):
    for seed in (1, 2, 500, 1000):
        keys = inputs.zipf_keys(n, 10 ** 8, 1.05, seed)
        hit, _, omi, omk = oracle_tags(oc, keys)
        out, gmi, gmk = gpu_query(gc, torch.from_numpy(keys).cuda(), n)
        assert len(gmi) == len(omi) and (gmi == omi).all() and (gmk == omk).all()
        assert 0.90 < hit.mean() < 0.96
        assert len(checker.mismatches(out, keys, hit)) == 0      # all n rows


# ---------------------------------------------------------------- streaming query + miss fill

def test_c3_streaming_query_and_miss_fill_full_size():
    """All 500 steps.  Per step: query -> fetch the missing rows from the lower-tier stand-in on
    the device -> insert them (Alg. 1, synchronous branch).  Every step: miss list exact, every
    row of the filled `out` equal to the host generator's row of its key, the oracle following
    the insert; every 25 steps and at the end the whole state.  On every 50th step the fill is
    held back until the raw query output (sentinel on every miss row) has been checked too."""
    S, W, d = 1 << 20, 8, 128
    n = 16384 * 26
    steps = 500
    t_begin = time.time()
    oc = OracleCache(S * W, W, 1)
    hit_rates, multi_total, over_total = [], 0, 0
    with DeviceCache(S * W, W, d, concurrent_writers=False) as gc:
        dstate = DeviceState(gc)
        checker = RowChecker(d, 1 << 20)
        rows = torch.empty(n, d, dtype=torch.float32, device="cuda")
        out = torch.empty(n, d, dtype=torch.float32, device="cuda")
        mi = torch.empty(n, dtype=torch.int32, device="cuda")
        mk = torch.empty(n, dtype=torch.int64, device="cuda")
        nm = torch.zeros(1, dtype=torch.int32, device="cuda")
        all_hit = np.ones(n, dtype=bool)
        for step in range(1, steps + 1):
            keys = inputs.zipf_keys(n, 10 ** 8, 1.1, step)
            dk = torch.from_numpy(keys).cuda()
            out.view(torch.int32).fill_(SENTINEL)
            B.hps_cache_query(gc.h, dk, n, out, mi, mk, nm)
            hit, _, omi, omk = oracle_tags(oc, keys)
            if step % 50 == 0 or step == 1:
                torch.cuda.synchronize()
                assert len(checker.mismatches(out, keys, hit)) == 0, f"step {step}: raw query output"
            B.hps_backing_fetch(mk, n, d, version=0, rows=rows, n_dev=nm, scatter_idx=mi, scatter_out=out)
            B.hps_cache_insert_dn(gc.h, mk, rows, n, nm)
            torch.cuda.synchronize()
            m = int(nm.item())
            gmi, gmk = sorted_miss_list(mi, mk, m)
            assert m == len(omi) and (gmi == omi).all() and (gmk == omk).all(), f"step {step}: miss list"
            hit_rates.append(1.0 - m / n)
            # after the fill every row of `out` is the row of its key (hits gathered, misses fetched)
            assert len(checker.mismatches(out, keys, all_hit)) == 0, f"step {step}: rows"
            a, b = follow_insert(oc, dstate, omk)
            multi_total += a
            over_total += b
            if step % 25 == 0 or step == steps:
                assert_full_state(dstate, oc)
                print(f"C3 step {step}: hit rate {hit_rates[-1]:.4f}, occupied "
                      f"{(oc.keys != EMPTY_KEY).mean():.3f}, sets past their ways {(oc.ctr > W).mean():.3f}, "
                      f"{time.time() - t_begin:.0f} s", flush=True)
    print("C3 hit rate per step (every 20th):", [round(x, 4) for x in hit_rates[::20]], flush=True)
    assert hit_rates[0] == 0.0
    assert all(b >= a - 0.02 for a, b in zip(hit_rates[:40], hit_rates[1:41])), hit_rates[:41]   # warm-up: rising
    assert hit_rates[-1] > 0.85 and abs(hit_rates[-1] - hit_rates[-50]) < 0.02                  # saturated
    assert (oc.ctr > W).mean() > 0.25, "replacement in full sets was not reached"
    assert multi_total > 10000
    oc.close()


# ---------------------------------------------------------------- 26 tables, one launch

def test_c4_multi_table_lookup_one_launch_full_size():
    W, d, Bn = 8, 128, 131072
    vocab = inputs.log_uniform_vocab(26, 1e3, 1e8, 7)
    slots = [int(min(0.2 * v, 1 << 22)) // 8 * 8 for v in vocab]
    caches, oracles = [], []
    try:
        keys = np.empty((26, Bn), dtype=np.int64)
        for t, (v, s) in enumerate(zip(vocab.tolist(), slots)):
            oc = OracleCache(s, W, 1)
            gc = DeviceCache(s, W, d, concurrent_writers=False)
            caches.append(gc)
            oracles.append(oc)
            if s <= (1 << 18):
                # small tables: the hottest `s` ids (hottest last) through hps_cache_insert in
                # chunks of at most a quarter of the sets, the oracle following
                dstate, _, _ = gpu_prefill_descending(gc, oc, s, max(8, (s // W) // 4))
                assert_full_state(dstate, oc)
            else:
                oracle_prefill_descending(oc, s, 1 << 18)
                gc.load(np.array(oc.keys), np.array(oc.ctr))
                refresh_cycle(gc, 0, min(s, 1 << 22))
            keys[t] = inputs.zipf_keys(Bn, v, 1.05, 7 + 1000 * t)
        n = 26 * Bn
        dk = torch.from_numpy(keys).cuda()
        out = torch.full((n, d), SENTINEL, dtype=torch.int32, device="cuda").view(torch.float32)
        mi = torch.empty(n, dtype=torch.int32, device="cuda")
        mk = torch.empty(n, dtype=torch.int64, device="cuda")
        nm = torch.zeros(1, dtype=torch.int32, device="cuda")
        B.hps_cache_query_multi([c.h for c in caches], dk, Bn, out, mi, mk, nm)
        torch.cuda.synchronize()
        m = int(nm.item())
        gmi, gmk = sorted_miss_list(mi, mk, m)
        emi, emk, hit = [], [], np.zeros(n, dtype=bool)
        for t, oc in enumerate(oracles):
            h, _, omi, omk = oracle_tags(oc, keys[t])
            emi.append(omi.astype(np.int64) + t * Bn)
            emk.append(omk)
            hit[t * Bn:(t + 1) * Bn] = h
        emi, emk = np.concatenate(emi), np.concatenate(emk)
        assert m == len(emi) and (gmi == emi).all() and (gmk == emk).all()
        checker = RowChecker(d, 1 << 20)
        flat = keys.reshape(-1)
        for t in range(26):                                  # all 3.4 M rows, one table at a time
            sl = slice(t * Bn, (t + 1) * Bn)
            assert len(checker.mismatches(out[sl], flat[sl], hit[sl])) == 0, f"table {t}"
    finally:
        for c in caches:
            c.close()
        for o in oracles:
            o.close()


# ---------------------------------------------------------------- update concurrent with query

def test_c5_online_update_concurrent_with_query_full_size():
    """64 GiB cache (2^24 sets x 8 ways x 128 fp32).  Query batches of 65,536 x 26 Zipf keys on
    one stream, update batches of 262,144 <key, row> pairs (half of the keys resident) on a
    second stream.  Every row of every query is looked at: a hit must carry the complete row of
    one version of its key (version 0 unless the key is in an update batch), a miss the sentinel;
    versions seen never go backwards from one query to the next; hit/miss sets equal the oracle's
    (update never changes residency); after both streams are drained a re-query equals the oracle."""
    S, W, d = 1 << 24, 8, 128
    n_q, n_u, rounds = 65536 * 26, 262144, 6
    oc = OracleCache(S * W, W, 1)
    oracle_prefill_descending(oc, S * W, 1 << 20)
    rng = np.random.Generator(np.random.PCG64(5))
    with DeviceCache(S * W, W, d, concurrent_writers=True) as gc:
        gc.load(np.array(oc.keys), np.array(oc.ctr))
        occupied = int((np.array(oc.keys) != EMPTY_KEY).sum())
        assert refresh_cycle(gc, 0, 1 << 24) == occupied
        checker = RowChecker(d, 1 << 20)

        q_keys = [inputs.zipf_keys(n_q, 10 ** 9, 1.05, 100 + r) for r in range(rounds)]
        upd_keys = []
        for r in range(rounds):
            cand = np.unique(np.concatenate([q_keys[r][: n_u], rng.integers(0, S * W, n_u)]))
            resident, _, _, _ = oracle_tags(oc, cand)
            res = rng.permutation(cand[resident])[: n_u // 2]
            absent = rng.integers(2 * 10 ** 9, 3 * 10 ** 9, n_u - len(res))
            upd_keys.append(rng.permutation(np.concatenate([res, absent])).astype(np.int64))
        qs, us = torch.cuda.Stream(), torch.cuda.Stream()
        d_q = [torch.from_numpy(k).cuda() for k in q_keys]
        d_u = [torch.from_numpy(k).cuda() for k in upd_keys]
        d_urows = [torch.empty(n_u, d, dtype=torch.float32, device="cuda") for _ in range(rounds)]
        for r in range(rounds):
            B.hps_backing_fetch(d_u[r], n_u, d, version=r + 1, rows=d_urows[r])
        outs = [torch.full((n_q, d), SENTINEL, dtype=torch.int32, device="cuda").view(torch.float32) for _ in range(rounds)]
        mi = [torch.empty(n_q, dtype=torch.int32, device="cuda") for _ in range(rounds)]
        mk = [torch.empty(n_q, dtype=torch.int64, device="cuda") for _ in range(rounds)]
        nm = torch.zeros(rounds, dtype=torch.int32, device="cuda")
        torch.cuda.synchronize()
        for r in range(rounds):
            B.hps_cache_query(gc.h, d_q[r], n_q, outs[r], mi[r], mk[r], nm[r:r + 1], qs)
            B.hps_cache_update(gc.h, d_u[r], d_urows[r], n_u, us)
        torch.cuda.synchronize()

        all_upd = np.unique(np.concatenate(upd_keys))
        last = {}
        n_new_seen = 0
        for r in range(rounds):
            m = int(nm[r].item())
            hit, _, omi, omk = oracle_tags(oc, q_keys[r])
            gmi, gmk = sorted_miss_list(mi[r], mk[r], m)
            assert m == len(omi) and (gmi == omi).all() and (gmk == omk).all()
            # every row against version 0; what differs must be a hit on an updated key that
            # carries, whole, one of the versions issued so far
            bad = checker.mismatches(outs[r], q_keys[r], hit)
            ks = q_keys[r][bad]
            assert hit[bad].all() and np.isin(ks, all_upd).all(), f"round {r}: a row differs that no update touched"
            got = outs[r][torch.from_numpy(bad).cuda()].view(torch.int32).cpu().numpy().view(np.uint32)
            seen = np.zeros(len(bad), dtype=np.int64)
            for v in range(1, rounds + 1):
                seen[(got == inputs.backing_rows(ks, d, v).view(np.uint32)).all(axis=1)] = v
            assert (seen > 0).all(), f"round {r}: {(seen == 0).sum()} rows match no single version"
            n_new_seen += len(bad)
            # versions never go backwards: positions of updated keys that still show version 0 count too
            upd_pos = np.nonzero(np.isin(q_keys[r], all_upd) & hit)[0]
            ver = np.zeros(n_q, dtype=np.int64)
            ver[bad] = seen
            newest = {}
            for k, v in zip(q_keys[r][upd_pos].tolist(), ver[upd_pos].tolist()):
                assert v >= last.get(k, 0), "a later query saw an older version"
                newest[k] = max(newest.get(k, 0), v)
            last.update(newest)
        print(f"C5: {n_new_seen} rows of updated versions seen by the overlapping queries", flush=True)
        # drained: the oracle applies the updates in order (tag = version); re-query and compare
        for r in range(rounds):
            oc.update(upd_keys[r], np.full((n_u, 1), r + 1, dtype=np.uint32))
        keys = np.concatenate([np.concatenate(upd_keys)[:: 4], q_keys[0][:200000]])
        n = len(keys)
        hit, tags, omi, omk = oracle_tags(oc, keys)
        out, gmi, gmk = gpu_query(gc, torch.from_numpy(keys).cuda(), n)
        assert len(gmi) == len(omi) and (gmi == omi).all() and (gmk == omk).all()
        assert (tags[hit] > 0).sum() > 50000              # plenty of updated rows among them
        versions = np.where(hit, tags, 0).astype(np.int64)
        assert len(checker.mismatches(out, keys, hit, versions)) == 0      # all rows
    oc.close()
