"""Pins for the oracle's Alg. 1 step (hpso_lookup): no GPU, no HIP library.

The paper prints no worked run of Alg. 1, so what pins the function is
  * a batch worked out by hand (positions, miss list, hit rate, mode, rows, keys to insert),
    at the threshold itself and one float above it;
  * the degenerate batches (all hits, all misses, empty, one key repeated);
  * the decision taken in single precision (a batch where double precision decides otherwise);
  * an independent model: as long as no set overflows the cache is a dict, and Alg. 1 over a
    dict is a dozen lines of Python.
"""
import numpy as np
import pytest

from oracle import OracleCache


def rows_of(keys, d, salt=0):
    """Arbitrary row content per (key, salt); the lower tiers hold salt 7 in these tests."""
    keys = np.asarray(keys, dtype=np.int64).astype(np.uint64)
    return ((keys[:, None] * np.uint64(2654435761) + np.uint64(salt) * np.uint64(97)
             + np.arange(d, dtype=np.uint64)[None, :] * np.uint64(40503)) & np.uint64(0xFFFFFFFF)).astype(np.uint32)


def make_cache(d=4):
    oc = OracleCache(64 * 8, 8, d)              # 512 slots for a handful of keys: no set overflows
    cached = np.array([10, 11, 12], dtype=np.int64)
    oc.insert(cached, rows_of(cached, d, 1))
    return oc


def test_worked_batch_at_and_above_the_threshold():
    d = 4
    Q = np.array([10, 99, 11, 99, 50, 10, 12, 50], dtype=np.int64)
    lower = rows_of(Q, d, 7)
    default = np.array([1, 2, 3, 4], dtype=np.uint32)
    hit_pos, miss_pos = [0, 2, 5, 6], [1, 3, 4, 7]

    # hit rate = 1 - 4/8 = 0.5; t = 0.5 is not "below the threshold": asynchronous
    oc = make_cache(d)
    out, rate, sync, ins = oc.lookup(Q, lower, 0.5, default)
    assert rate == np.float32(0.5) and sync is False
    assert ins.tolist() == [99, 50]                              # each missing key once, first occurrence first
    assert (out[hit_pos] == rows_of(Q[hit_pos], d, 1)).all()     # cached rows, not the lower tiers' rows
    assert (out[miss_pos] == default).all()
    # the queued insertion has run: both keys are cached now, with the lower tiers' rows
    out2, rate2, sync2, ins2 = oc.lookup(Q, lower, 0.5, default)
    assert rate2 == np.float32(1.0) and sync2 is False and len(ins2) == 0
    assert (out2[miss_pos] == lower[miss_pos]).all() and (out2[hit_pos] == rows_of(Q[hit_pos], d, 1)).all()
    oc.close()

    # one float above 0.5 the same batch is below the threshold: synchronous, fetched rows handed out
    oc = make_cache(d)
    out, rate, sync, ins = oc.lookup(Q, lower, float(np.nextafter(np.float32(0.5), np.float32(1))), default)
    assert rate == np.float32(0.5) and sync is True and ins.tolist() == [99, 50]
    assert (out[miss_pos] == lower[miss_pos]).all()
    assert (out[hit_pos] == rows_of(Q[hit_pos], d, 1)).all()
    _, mi, _ = oc.query(Q)
    assert len(mi) == 0                                          # inserted before the call returned
    oc.close()


def test_do_insert_zero_leaves_the_cache_alone():
    d = 4
    Q = np.array([10, 99, 50, 99], dtype=np.int64)
    oc = make_cache(d)
    before = (np.array(oc.keys).copy(), np.array(oc.ctr).copy(), np.array(oc.vals).copy())
    out, rate, sync, ins = oc.lookup(Q, rows_of(Q, d, 7), 2.0, np.zeros(d, np.uint32), do_insert=False)
    assert sync and rate == np.float32(0.25) and ins.tolist() == [99, 50]
    assert (np.array(oc.keys) == before[0]).all() and (np.array(oc.ctr) == before[1]).all()
    assert (np.array(oc.vals) == before[2]).all()
    oc.close()


def test_degenerate_batches():
    d = 4
    default = np.full(d, 0xABCD, dtype=np.uint32)
    oc = make_cache(d)
    # all hits: nothing fetched, nothing inserted, never synchronous (even with t above 1)
    Q = np.array([12, 10, 10, 11], dtype=np.int64)
    ctr0 = np.array(oc.ctr).copy()
    out, rate, sync, ins = oc.lookup(Q, rows_of(Q, d, 7), 2.0, default)
    assert rate == np.float32(1.0) and sync is False and len(ins) == 0
    assert (out == rows_of(Q, d, 1)).all() and (np.array(oc.ctr) == ctr0).all()
    # all misses: hit rate 0; t = 0 is asynchronous (0 < 0 is false), any t > 0 synchronous
    Q = np.array([70, 71, 70, 72], dtype=np.int64)
    out, rate, sync, ins = oc.lookup(Q, rows_of(Q, d, 7), 0.0, default, do_insert=False)
    assert rate == np.float32(0.0) and sync is False and ins.tolist() == [70, 71, 72] and (out == default).all()
    out, rate, sync, ins = oc.lookup(Q, rows_of(Q, d, 7), 1e-6, default, do_insert=False)
    assert sync is True and (out == rows_of(Q, d, 7)).all()
    # empty batch
    out, rate, sync, ins = oc.lookup(np.empty(0, np.int64), np.empty((0, d), np.uint32), 0.5, default)
    assert out.shape == (0, d) and rate == np.float32(1.0) and sync is False and len(ins) == 0
    # one missing key given many times: one insertion (the counter of its set moves by one)
    Q = np.full(9, 555, dtype=np.int64)
    s = oc.set_of(555)
    c0 = int(oc.ctr[s])
    out, rate, sync, ins = oc.lookup(Q, rows_of(Q, d, 7), 0.5, default)
    assert ins.tolist() == [555] and sync is True and int(oc.ctr[s]) == c0 + 1
    oc.close()


def test_decision_is_taken_in_single_precision():
    # n = 10, seven misses: 7/10 rounds down in float32, so the float32 hit rate 1 - 7/10 is
    # 0.30000001..., above the double-precision 0.3.  With t = that float32 value the hit rate
    # equals t (asynchronous); computed in double precision it would be below t (synchronous).
    d = 4
    oc = make_cache(d)
    Q = np.array([10, 11, 12, 90, 91, 92, 93, 94, 95, 96], dtype=np.int64)
    t32 = np.float32(1.0) - np.float32(7.0) / np.float32(10.0)
    assert 1.0 - 7.0 / 10.0 < float(t32)
    out, rate, sync, ins = oc.lookup(Q, rows_of(Q, d, 7), float(t32), np.zeros(d, np.uint32), do_insert=False)
    assert rate == t32 and sync is False
    oc.close()


def alg1_over_a_dict(table, Q, lower, t, default):
    """Alg. 1 with a dict as the cache (valid while no set of the real cache overflows)."""
    n = len(Q)
    out = np.zeros((n, lower.shape[1]), dtype=np.uint32)
    missing = [i for i in range(n) if int(Q[i]) not in table]
    for i in range(n):
        if int(Q[i]) in table:
            out[i] = table[int(Q[i])]
    rate = np.float32(1.0) - np.float32(len(missing)) / np.float32(n)
    sync = bool(missing) and bool(rate < np.float32(t))
    fetched = {}
    for i in missing:
        fetched.setdefault(int(Q[i]), lower[i].copy())
        out[i] = lower[i] if sync else default
    for k, r in fetched.items():
        table[k] = r
    return out, rate, sync, list(fetched)


@pytest.mark.parametrize("seed,t", [(1, 0.0), (2, 0.3), (3, 0.6), (4, 0.85), (5, 2.0)])
def test_against_alg1_over_a_dict(seed, t):
    d = 6
    rng = np.random.Generator(np.random.PCG64(seed))
    oc = OracleCache(4096 * 8, 8, d)            # 32768 slots, < 400 distinct keys: Poisson(0.01) per set
    table = {}
    default = rng.integers(0, 1 << 32, d, dtype=np.uint32)
    modes = set()
    for step in range(40):
        n = int(rng.integers(1, 60))
        Q = rng.integers(0, 10 * (step + 1), n).astype(np.int64)
        lower = rows_of(Q, d, 7)
        out, rate, sync, ins = oc.lookup(Q, lower, t, default)
        eout, erate, esync, eins = alg1_over_a_dict(table, Q, lower, t, default)
        assert rate == erate and sync == esync and ins.tolist() == eins
        assert (out == eout).all()
        modes.add(sync)
        assert int((np.array(oc.keys) != -(1 << 63)).sum()) == len(table)
    if t == 0.0:
        assert modes == {False}
    if 0.0 < t <= 1.0:
        assert modes == {False, True}           # both branches were taken
    oc.close()
