"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element.

Integer/byte work throughout, so the bar is bit-exact: `out` rows, hit/miss sets and miss lists
(compared after sorting by index: the order of the list is the one thing that is not unique),
and the canonical post-insert state (per set: sorted keys with their rows, plus the victim
counter) whenever the batch is order-independent.  Batches that are not (set overflow within a
batch, or new keys overwriting keys of the same batch) are checked by the invariants.  After
every insert the oracle adopts the GPU's way placement, because the order in which the new keys
of one batch take their ways is free and decides which of them is evicted first later on.
"""
import os

import numpy as np
import pytest
import torch

from oracle import OracleCache
from paper_2210_08804_amd import binding as B
from paper_2210_08804_amd import inputs
from harness import (DeviceCache, EMPTY_KEY, RESERVED_KEY, SENTINEL, assert_same_state,
                     check_state_invariants, insert_is_order_independent)

pytestmark = pytest.mark.gpu

# HPS_TEST_SEED_SHIFT=k runs the randomised sequence test on another random stream (for soak runs)
SEED_SHIFT = int(os.environ.get("HPS_TEST_SEED_SHIFT", "0"))


@pytest.fixture(autouse=True, params=["checked", "plain", "dedup"])
def query_variant(request):
    """Every test runs against the three query kernels: the one that validates rows against
    concurrent writers (the default), the plain one for query-only phases, and the plain one
    with in-tile key deduplication."""
    import harness
    harness.CONCURRENT_WRITERS = request.param == "checked"
    harness.QUERY_DEDUP = request.param == "dedup"
    yield request.param
    harness.CONCURRENT_WRITERS = True
    harness.QUERY_DEDUP = False


def rows_u32(keys, d, version=0):
    return inputs.backing_rows(keys, d, version).view(np.uint32)


def compare_query(gc, oc, keys):
    out_g, mi_g, mk_g = gc.query(keys)
    out_o = np.full((len(keys), oc.d), SENTINEL, dtype=np.uint32)
    _, mi_o, mk_o = oc.query(keys, out_o)
    assert len(mi_g) == len(mi_o), f"n_miss {len(mi_g)} != {len(mi_o)}"
    assert (mi_g == mi_o).all(), "miss positions differ"
    assert (mk_g == mk_o).all(), "miss keys differ"
    assert (out_g == out_o).all(), "rows differ (or a miss row was written)"
    return len(mi_o)


def insert_both(gc, oc, keys, rows, expect_rows=None):
    """Insert on both sides; compare canonically when the batch allows it, else check the
    invariants on the GPU state and re-seat the oracle from it.  Returns True if compared exactly."""
    exact = insert_is_order_independent(oc, keys)
    keys_before = np.array(oc.keys).copy()
    vals_before = np.array(oc.vals).copy()
    before = set(keys_before.reshape(-1).tolist())
    ctr_before = np.array(oc.ctr).copy()
    gc.insert(keys, rows)
    oc.insert(keys, rows)
    state = gc.export()
    if exact:
        assert_same_state(state, oc)
        # Which way each new key of one batch lands in is arrival order, which the contract
        # leaves open; it decides later evictions, so the oracle adopts the GPU's placement
        # (an equivalent state: same keys, rows and counters per set).
        oc.load_state(*state)
    else:
        gk, gctr, gv = state
        rows_of = {}
        for k, r in zip(np.asarray(keys).tolist(), np.asarray(rows).view(np.uint32)):
            rows_of.setdefault(k, []).append(r)
        old_row = {int(keys_before[s, w]): vals_before[s, w]
                   for s, w in zip(*np.nonzero(keys_before != EMPTY_KEY))}
        check_state_invariants(gk, gctr, gv, oc.set_of)
        # every resident key is an old resident with its old row, or a key of this batch with
        # one of the rows the batch carries for it
        ss, ww = np.nonzero(gk != EMPTY_KEY)
        for s, w in zip(ss.tolist(), ww.tolist()):
            k = int(gk[s, w])
            ok = k in old_row and (gv[s, w] == old_row[k]).all()
            ok = ok or (k in rows_of and any((gv[s, w] == r).all() for r in rows_of[k]))
            assert ok, f"slot ({s},{w}) holds key {k} with a row nobody wrote for it"
        # counters advanced by at least the number of distinct new keys of each set
        new = {k for k in rows_of if k not in before and k not in (EMPTY_KEY, RESERVED_KEY)}
        adv = (gctr.astype(np.int64) - ctr_before.astype(np.int64))
        per_set = np.zeros(oc.S, dtype=np.int64)
        for k in new:
            per_set[oc.set_of(k)] += 1
        assert (adv >= per_set).all()
        oc.load_state(gk, gctr, gv)
    return exact


# ------------------------------------------------------------------ config 1 (tiny, end to end)

def test_c1_tiny_query_insert_requery():
    S, W, d = 4096, 8, 16
    keys = inputs.uniform_keys(1024 * 26, 1 << 18, 0)
    rows = rows_u32(keys, d)
    # (a) one insert call: many sets receive more than 8 new keys -> invariants + re-seat
    with DeviceCache(S * W, W, d) as gc:
        oc = OracleCache(S * W, W, d)
        assert compare_query(gc, oc, keys) == len(keys)            # cold cache: all miss
        exact = insert_both(gc, oc, keys, rows)
        assert not exact
        compare_query(gc, oc, keys)
    # (b) chunked insert: each chunk is order-independent -> state compared bit-exactly
    with DeviceCache(S * W, W, d) as gc:
        oc = OracleCache(S * W, W, d)
        n_exact = 0
        for ck, cr in zip(np.array_split(keys, 32), np.array_split(rows, 32)):
            n_exact += insert_both(gc, oc, ck, cr)
        assert n_exact >= 16
        m = compare_query(gc, oc, keys)
        assert 0 < m < len(keys)
        # insert the misses again (the Alg. 1 loop), then everything resident that fits
        _, mi, mk = oc.query(keys)
        insert_both(gc, oc, mk, rows[mi])
        compare_query(gc, oc, keys)


# ------------------------------------------------------------------ geometry sweep

@pytest.mark.parametrize("W", [1, 2, 4, 8, 16, 32, 64])
def test_ways_sweep(W):
    S, d = 97, 8                                  # non-power-of-two set count
    rng = np.random.Generator(np.random.PCG64(100 + W))
    with DeviceCache(S * W, W, d) as gc:
        oc = OracleCache(S * W, W, d)
        for step in range(6):
            keys = rng.integers(0, 3 * S * W, size=int(rng.integers(1, 700)), dtype=np.int64)
            compare_query(gc, oc, keys)
            _, mi, mk = oc.query(keys)
            insert_both(gc, oc, mk, rows_u32(mk, d))
            compare_query(gc, oc, keys)
        gk, gctr, gv = gc.export()
        check_state_invariants(gk, gctr, gv, oc.set_of)


@pytest.mark.parametrize("d", [4, 16, 100, 128, 132, 256, 320])
def test_dim_sweep(d):
    S, W = 512, 8
    rng = np.random.Generator(np.random.PCG64(200 + d))
    with DeviceCache(S * W, W, d) as gc:
        oc = OracleCache(S * W, W, d)
        keys = rng.integers(0, 6000, size=3000, dtype=np.int64)
        for ck in np.array_split(keys, 6):
            insert_both(gc, oc, ck, rows_u32(ck, d))
        q = rng.integers(0, 9000, size=2001, dtype=np.int64)       # ragged tail: 2001 = 7*256 + 209
        m = compare_query(gc, oc, q)
        assert 0 < m < len(q)
        upd = rng.integers(0, 9000, size=777, dtype=np.int64)
        upd = np.unique(upd)                                        # distinct keys: deterministic result
        gc.update(upd, rows_u32(upd, d, version=3))
        oc.update(upd, rows_u32(upd, d, version=3))
        assert_same_state(gc.export(), oc)
        compare_query(gc, oc, q)


# ------------------------------------------------------------------ edge cases

def test_empty_reserved_duplicate_and_extreme_batches():
    S, W, d = 64, 8, 16
    with DeviceCache(S * W, W, d) as gc:
        oc = OracleCache(S * W, W, d)
        # n = 0 everywhere
        out, mi, mk = gc.query(np.zeros(0, dtype=np.int64))
        assert out.shape[0] == 0 and mi.size == 0
        gc.insert(np.zeros(0, dtype=np.int64), np.zeros((0, d), np.uint32))
        gc.update(np.zeros(0, dtype=np.int64), np.zeros((0, d), np.uint32))
        # reserved keys and extreme values
        ks = np.array([EMPTY_KEY, RESERVED_KEY, EMPTY_KEY + 2, -1, 0, (1 << 63) - 1, 5, 5, 5], dtype=np.int64)
        insert_both(gc, oc, ks, rows_u32(ks, d))
        assert compare_query(gc, oc, ks) == 2
        assert int(np.array(oc.ctr).sum()) == 5
        # all-hit, all-miss, heavy duplicates, single key
        hit = np.array([5, -1, 0, 5, 5, (1 << 63) - 1] * 100, dtype=np.int64)
        assert compare_query(gc, oc, hit) == 0
        miss = np.arange(1000, 1700, dtype=np.int64)
        assert compare_query(gc, oc, miss) == 700
        assert compare_query(gc, oc, np.array([5], dtype=np.int64)) == 0
        assert compare_query(gc, oc, np.array([6], dtype=np.int64)) == 1
        dup_new = np.array([77] * 300 + [78] * 300, dtype=np.int64)     # duplicates of new keys across waves
        insert_both(gc, oc, dup_new, rows_u32(dup_new, d))
        assert int(np.array(oc.ctr).sum()) == 7
        compare_query(gc, oc, dup_new)


def test_duplicates_with_different_rows_store_one_intact():
    S, W, d = 16, 4, 32
    with DeviceCache(S * W, W, d) as gc:
        keys = np.array([9] * 500, dtype=np.int64)
        rows = np.repeat(np.arange(500, dtype=np.uint32)[:, None], d, axis=1)   # row i = all words i
        gc.insert(keys, rows)
        out, mi, _ = gc.query(np.array([9], dtype=np.int64))
        assert mi.size == 0 and (out[0] == out[0, 0]).all() and out[0, 0] < 500
        gk, gctr, _ = gc.export()
        assert int(gctr.sum()) == 1 and int((gk == 9).sum()) == 1
        gc.update(keys, rows + 1000)
        out, _, _ = gc.query(np.array([9], dtype=np.int64))
        assert (out[0] == out[0, 0]).all() and 1000 <= out[0, 0] < 1500


def test_key_given_very_many_times_does_not_starve_its_set():
    """A miss list carries every occurrence of a missing key, so a hot key can come tens of
    thousands of times in one insert batch.  Keys that share its set, each given once, must
    still get in, and no wave may give up (the flag word is checked when the cache closes)."""
    from oracle import set_of
    S, W, d = 1 << 10, 8, 128
    hot = 1
    mates = [k for k in range(2, 200000) if set_of(k, S) == set_of(hot, S)][:W - 1]
    assert len(mates) == W - 1
    other = np.unique(inputs.uniform_keys(1500, 1 << 40, 21))
    other = other[[set_of(int(k), S) != set_of(hot, S) for k in other]]
    keys = np.concatenate([np.full(120000, hot, dtype=np.int64), np.array(mates, dtype=np.int64), other])
    keys = keys[np.random.Generator(np.random.PCG64(8)).permutation(len(keys))]
    with DeviceCache(S * W, W, d) as gc:
        oc = OracleCache(S * W, W, d)
        insert_both(gc, oc, keys, rows_u32(keys, d))
        resident = set(np.array(oc.keys).reshape(-1).tolist())
        assert hot in resident and set(mates) <= resident
        compare_query(gc, oc, np.concatenate([keys[:4096], np.array(mates, dtype=np.int64)]))
        # the same batch again: every key is cached now, nothing changes
        insert_both(gc, oc, keys, rows_u32(keys, d, version=1))
        compare_query(gc, oc, keys[:4096])


@pytest.mark.parametrize("dtype,dim", [(torch.bfloat16, 128), (torch.float16, 64), (torch.float16, 200)])
def test_half_precision_rows_travel_as_opaque_words(dtype, dim):
    """Rows are bit patterns to every kernel, so a table of 16-bit values is a cache of dim/2
    32-bit words: the caller reinterprets its tensors (a view, no conversion)."""
    S, W = 1024, 8
    words = dim // 2
    keys = np.unique(inputs.uniform_keys(1500, 1 << 32, 31))
    table = torch.randn(len(keys), dim, generator=torch.Generator().manual_seed(5)).to(dtype)
    as_words = table.view(torch.float32).numpy().view(np.uint32)
    assert as_words.shape == (len(keys), words)
    with DeviceCache(S * W, W, words) as gc:
        oc = OracleCache(S * W, W, words)
        insert_both(gc, oc, keys, as_words)
        q = np.concatenate([keys[::3], keys[:100] + (1 << 40)])
        dk = torch.from_numpy(q).cuda()
        out = torch.zeros(len(q), dim, dtype=dtype, device="cuda")
        mi = torch.empty(len(q), dtype=torch.int32, device="cuda")
        mk = torch.empty(len(q), dtype=torch.int64, device="cuda")
        nm = torch.zeros(1, dtype=torch.int32, device="cuda")
        B.hps_cache_query(gc.h, dk, len(q), out.view(torch.float32), mi, mk, nm)
        torch.cuda.synchronize()
        exp = np.zeros((len(q), words), dtype=np.uint32)
        _, omi, _ = oc.query(q, exp)
        assert int(nm.item()) == len(omi) >= 100
        assert (out.cpu().view(torch.float32).numpy().view(np.uint32) == exp).all()
        hit = np.ones(len(q), dtype=bool)
        hit[omi] = False
        pos = {int(k): i for i, k in enumerate(keys.tolist())}
        src = torch.tensor([pos[int(k)] for k in q[hit]])
        assert torch.equal(out.cpu()[torch.from_numpy(hit)], table[src])      # the very same 16-bit values


def test_one_set_overflow_keeps_invariants():
    # all keys of the batch fall into one set of a 4-way cache: far more than W new keys
    S, W, d = 8, 4, 8
    with DeviceCache(S * W, W, d) as gc:
        oc = OracleCache(S * W, W, d)
        pool = [k for k in range(4000) if oc.set_of(k) == 3][:200]
        ks = np.array(pool, dtype=np.int64)
        exact = insert_both(gc, oc, ks, rows_u32(ks, d))
        assert not exact
        gk, gctr, _ = gc.export()
        assert int(gctr[3]) == 200 and int((gk[3] != EMPTY_KEY).sum()) == W
        compare_query(gc, oc, ks)


# ------------------------------------------------------------------ other entry points

def test_backing_fetch_matches_numpy_generator():
    d = 128
    keys = inputs.zipf_keys(5000, 10 ** 8, 1.1, 3)
    dk = torch.from_numpy(keys).cuda()
    rows = torch.zeros(5000, d, dtype=torch.float32, device="cuda")
    B.hps_backing_fetch(dk, 5000, d, version=7, rows=rows)
    torch.cuda.synchronize()
    assert (rows.cpu().numpy().view(np.uint32) == rows_u32(keys, d, 7)).all()
    # device-side length and scatter
    idx = torch.randperm(8000, device="cuda")[:5000].to(torch.int32)
    target = torch.full((8000, d), -5.0, dtype=torch.float32, device="cuda")
    n_dev = torch.tensor([1234], dtype=torch.int32, device="cuda")
    B.hps_backing_fetch(dk, 5000, d, version=0, rows=None, n_dev=n_dev, scatter_idx=idx, scatter_out=target)
    torch.cuda.synchronize()
    t = target.cpu().numpy()
    idx_np = idx.cpu().numpy()
    exp = inputs.backing_rows(keys[:1234], d, 0)
    assert (t[idx_np[:1234]].view(np.uint32) == exp.view(np.uint32)).all()
    untouched = np.ones(8000, dtype=bool)
    untouched[idx_np[:1234]] = False
    assert (t[untouched] == -5.0).all()


def test_dump_returns_resident_keys():
    S, W, d = 1000, 8, 4
    with DeviceCache(S * W, W, d) as gc:
        oc = OracleCache(S * W, W, d)
        keys = np.unique(inputs.uniform_keys(5000, 1 << 30, 4))
        for ck in np.array_split(keys, 8):
            insert_both(gc, oc, ck, rows_u32(ck, d))
        buf = torch.empty(S * W, dtype=torch.int64, device="cuda")
        cnt = torch.full((1,), -1, dtype=torch.int32, device="cuda")
        B.hps_cache_dump(gc.h, 0, S * W, buf, cnt)
        torch.cuda.synchronize()
        m = int(cnt.item())
        assert sorted(buf[:m].cpu().tolist()) == sorted(oc.dump().tolist())
        # in two halves (batched dump, Sec. 6 step 2), and an empty range
        got = []
        for first in (0, S * W // 2):
            B.hps_cache_dump(gc.h, first, S * W // 2, buf, cnt)
            torch.cuda.synchronize()
            got += buf[: int(cnt.item())].cpu().tolist()
        assert sorted(got) == sorted(oc.dump().tolist())
        B.hps_cache_dump(gc.h, 10, 0, buf, cnt)
        torch.cuda.synchronize()
        assert int(cnt.item()) == 0


def test_device_side_batch_length_variants():
    S, W, d = 256, 8, 16
    with DeviceCache(S * W, W, d) as gc:
        oc = OracleCache(S * W, W, d)
        keys = np.arange(1, 601, dtype=np.int64)
        rows = rows_u32(keys, d)
        n_dev = torch.tensor([450], dtype=torch.int32, device="cuda")
        B.hps_cache_insert_dn(gc.h, torch.from_numpy(keys).cuda(),
                              torch.from_numpy(rows.view(np.float32)).cuda(), 600, n_dev)
        torch.cuda.synchronize()
        oc.insert(keys[:450], rows[:450])
        assert_same_state(gc.export(), oc)
        rows2 = rows_u32(keys, d, 2)
        n_dev.fill_(100)
        B.hps_cache_update_dn(gc.h, torch.from_numpy(keys).cuda(),
                              torch.from_numpy(rows2.view(np.float32)).cuda(), 600, n_dev)
        torch.cuda.synchronize()
        oc.update(keys[:100], rows2[:100])
        assert_same_state(gc.export(), oc)


def test_batch_sizes_around_the_launch_shape_boundaries():
    """The query's tiling follows the batch size (keys per wave, waves per work-group, rounds over
    the CUs); sizes just below, at and above every switch must all give the oracle's answer."""
    S, W, d = 1 << 12, 8, 4
    sizes = [255, 256, 257, 1023, 1024, 1025, 4095, 4096, 4097, 16383, 16384, 16385, 32767, 32769,
             65535, 65536, 65537, 106496, 131071, 131072, 131073, 262143, 262144, 262145, 300001]
    with DeviceCache(S * W, W, d) as gc:
        oc = OracleCache(S * W, W, d)
        resident = np.unique(inputs.uniform_keys(24000, 60000, 51))
        for ck in np.array_split(resident, 6):
            insert_both(gc, oc, ck, rows_u32(ck, d))
        keys = inputs.uniform_keys(max(sizes), 60000, 52)
        for n in sizes:
            m = compare_query(gc, oc, keys[:n])
            assert 0 < m < n


def test_write_batch_sizes_around_the_kernel_switches():
    """Insert and update pick their keys-per-wave from the batch size; sizes around a wave's key
    count and around the update kernel's switch must leave the oracle's state."""
    S, W, d = 1 << 14, 8, 4
    with DeviceCache(S * W, W, d) as gc:
        oc = OracleCache(S * W, W, d)
        pool = np.unique(inputs.uniform_keys(90000, 1 << 40, 61))
        rng = np.random.Generator(np.random.PCG64(62))
        version = 0
        for n in [1, 15, 16, 17, 63, 64, 65, 4095, 4097, 32767, 32768, 32769, 50000]:
            version += 1
            ins = rng.choice(pool, n, replace=False)
            insert_both(gc, oc, ins, rows_u32(ins, d, 0))
            upd = rng.choice(pool, n, replace=False)             # some cached, some not
            gc.update(upd, rows_u32(upd, d, version))
            oc.update(upd, rows_u32(upd, d, version))
            assert_same_state(gc.export(), oc)
        compare_query(gc, oc, pool[:50000])


def test_query_with_device_side_batch_length():
    """hps_cache_query_dn looks up min(n_max, *n_dev) positions; the rest of the buffers is
    neither read as keys, nor written, nor reported."""
    S, W, d, n_max = 512, 8, 32, 3000
    with DeviceCache(S * W, W, d) as gc:
        oc = OracleCache(S * W, W, d)
        resident = np.unique(inputs.uniform_keys(2500, 6000, 41))
        insert_both(gc, oc, resident, rows_u32(resident, d))
        keys = inputs.uniform_keys(n_max, 6000, 42)
        dk = torch.from_numpy(keys).cuda()
        for n_real in [0, 1, 63, 64, 65, 1000, 2999, 3000, 5000]:
            out = torch.full((n_max, d), SENTINEL, dtype=torch.int32, device="cuda").view(torch.float32)
            mi = torch.full((n_max,), -1, dtype=torch.int32, device="cuda")
            mk = torch.full((n_max,), 0x5A5A5A5A, dtype=torch.int64, device="cuda")
            nm = torch.full((1,), 777, dtype=torch.int32, device="cuda")
            nd = torch.tensor([n_real], dtype=torch.int32, device="cuda")
            B.hps_cache_query_dn(gc.h, dk, n_max, nd, out, mi, mk, nm)
            torch.cuda.synchronize()
            n = min(n_real, n_max)
            exp = np.full((n_max, d), SENTINEL, dtype=np.uint32)
            _, omi, omk = oc.query(keys[:n], exp[:n])
            m = int(nm.item())
            assert m == len(omi)
            order = np.argsort(mi[:m].cpu().numpy().view(np.uint32))
            assert (mi[:m].cpu().numpy().view(np.uint32)[order] == omi).all()
            assert (mk[:m].cpu().numpy()[order] == omk).all()
            assert (out.view(torch.int32).cpu().numpy().view(np.uint32) == exp).all()
            assert (mi[m:] == -1).all() and (mk[m:] == 0x5A5A5A5A).all()
        with pytest.raises(B.HpsError):
            B.hps_cache_query_dn(gc.h, dk, n_max, None, out, mi, mk, nm)


def test_query_multi_matches_per_table_oracles():
    d, W = 32, 8
    vocab = [50, 1000, 30000, 200]
    slots = [16, 200, 4096, 40]
    Bn = 700
    rng = np.random.Generator(np.random.PCG64(7))
    caches, oracles = [], []
    try:
        for v, s in zip(vocab, slots):
            gc, oc = DeviceCache(s, W, d), OracleCache(s, W, d)
            ids = np.arange(min(v, s), dtype=np.int64)[::-1].copy()
            for ck in np.array_split(ids, max(1, len(ids) // 64)):
                insert_both(gc, oc, ck, rows_u32(ck, d))
            caches.append(gc)
            oracles.append(oc)
        keys = np.stack([rng.integers(0, v, size=Bn, dtype=np.int64) for v in vocab])     # [T, B]
        T = len(vocab)
        out = torch.full((T * Bn, d), SENTINEL, dtype=torch.int32, device="cuda").view(torch.float32)
        mi = torch.empty(T * Bn, dtype=torch.int32, device="cuda")
        mk = torch.empty(T * Bn, dtype=torch.int64, device="cuda")
        nm = torch.empty(1, dtype=torch.int32, device="cuda")
        B.hps_cache_query_multi([c.h for c in caches], torch.from_numpy(keys).cuda(), Bn, out, mi, mk, nm)
        torch.cuda.synchronize()
        m = int(nm.item())
        out_np = out.view(torch.int32).cpu().numpy().view(np.uint32).reshape(T, Bn, d)
        order = np.argsort(mi[:m].cpu().numpy().view(np.uint32))
        mi_np = mi[:m].cpu().numpy().view(np.uint32)[order]
        mk_np = mk[:m].cpu().numpy()[order]
        exp_mi, exp_mk = [], []
        for t, oc in enumerate(oracles):
            o = np.full((Bn, d), SENTINEL, dtype=np.uint32)
            _, omi, omk = oc.query(keys[t], o)
            assert (out_np[t] == o).all()
            exp_mi += (omi.astype(np.int64) + t * Bn).tolist()
            exp_mk += omk.tolist()
        assert mi_np.tolist() == exp_mi and mk_np.tolist() == exp_mk
    finally:
        for c in caches:
            c.close()


def test_random_op_sequences_against_oracle():
    S, W, d = 300, 8, 16
    rng = np.random.Generator(np.random.PCG64(77 + SEED_SHIFT))
    with DeviceCache(S * W, W, d) as gc:
        oc = OracleCache(S * W, W, d)
        ver = 0
        for step in range(40):
            n = int(rng.integers(1, 1500))
            keys = rng.integers(0, 5000, size=n, dtype=np.int64)
            op = step % 3
            if op == 0:
                compare_query(gc, oc, keys)
            elif op == 1:
                _, mi, mk = oc.query(keys)
                insert_both(gc, oc, mk, rows_u32(mk, d, ver))
            else:
                ver += 1
                uk = np.unique(keys)
                gc.update(uk, rows_u32(uk, d, ver))
                oc.update(uk, rows_u32(uk, d, ver))
                assert_same_state(gc.export(), oc)
        compare_query(gc, oc, np.arange(5000, dtype=np.int64))
