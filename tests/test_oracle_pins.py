"""Pins for the CPU oracle: everything here runs without a GPU and without the HIP library.

The paper prints no worked example of the cache (no key -> slot trace), so parity with the
paper's own numbers is unpinned.  What pins the oracle instead:
  * the published outputs of splitmix64 (tests/golden/splitmix64_seed0.txt) for the hash,
    plus an independent big-integer implementation on many keys;
  * special cases that reduce to library structures: dict (no set ever overflows),
    collections.deque(maxlen=W) (one set in isolation), direct-mapped (W = 1),
    fully associative FIFO (S = 1);
  * brute force on tiny caches: residency found by scanning every slot, and the invariant list
    (last written row returned, miss set = non-resident positions, no key twice, every key in
    its own set, occupancy = min(counter, W), empty slots after the occupied ones);
  * closed forms: occupancy after m distinct inserts = sum_s min(load_s, W); counter = load;
    set loads of sequential keys follow Poisson(mean load).
"""
import collections
import os

import numpy as np
import pytest

from oracle import OracleCache, mix64, EMPTY_KEY, RESERVED_KEY

M64 = (1 << 64) - 1
GOLDEN_DIR = os.path.join(os.path.dirname(__file__), "golden")


def py_mix64(x: int) -> int:
    x &= M64
    x ^= x >> 30
    x = (x * 0xBF58476D1CE4E5B9) & M64
    x ^= x >> 27
    x = (x * 0x94D049BB133111EB) & M64
    x ^= x >> 31
    return x


def py_set_of(key: int, S: int) -> int:
    return (py_mix64(key) >> 32) % S


def rows_for(keys, d, salt=0):
    """Arbitrary distinct row content per (key, salt): plain bit patterns, not the backing generator."""
    keys = np.asarray(keys, dtype=np.int64)
    base = (keys.astype(np.uint64) * np.uint64(2654435761) + np.uint64(salt * 977)) & np.uint64(0xFFFFFFFF)
    return (base[:, None] + np.arange(d, dtype=np.uint64)[None, :] * np.uint64(40503)).astype(np.uint32)


# ---------------------------------------------------------------- hash

def test_mix64_published_vectors():
    with open(os.path.join(GOLDEN_DIR, "splitmix64_seed0.txt")) as f:
        rows = [ln.split() for ln in f if ln.strip() and not ln.startswith("#")]
    assert len(rows) == 3
    for arg, val in rows:
        assert mix64(int(arg, 16)) == int(val, 16)


def test_mix64_against_bigint_many_keys():
    rng = np.random.Generator(np.random.PCG64(11))
    xs = [0, 1, 2, M64, 1 << 63, (1 << 63) - 1, 0xFFFFFFFF, 1 << 32]
    xs += [int(v) for v in rng.integers(0, 1 << 63, size=12000, dtype=np.int64)]
    xs += [(-int(v)) & M64 for v in rng.integers(1, 1 << 62, size=2000, dtype=np.int64)]
    for x in xs:
        assert mix64(x) == py_mix64(x)


def test_mix64_is_a_bijection_on_samples():
    # each step of the finaliser is invertible, so distinct inputs give distinct outputs
    xs = list(range(50000))
    assert len({mix64(x) for x in xs}) == len(xs)


@pytest.mark.parametrize("S", [1, 2, 25, 4096, 1000003, (1 << 31) - 1])
def test_set_of_uses_upper_32_bits_mod_S(S):
    c = None
    rng = np.random.Generator(np.random.PCG64(S))
    keys = [0, 1, -1, (1 << 63) - 1, -(1 << 63) + 2] + [int(v) for v in rng.integers(-(1 << 62), 1 << 62, size=500)]
    if S * 1 < (1 << 22):
        c = OracleCache(S, 1, 1)
        for k in keys:
            assert c.set_of(k) == py_set_of(k, S)
    else:
        # large S: allocate nothing, use the module helper built on the C mix64
        from oracle import set_of
        for k in keys:
            assert set_of(k, S) == py_set_of(k, S)


def test_set_loads_of_sequential_keys_are_poisson():
    # 2^21 sequential ids into 2^18 sets: loads must look like Poisson(8) (chi-square, 20 bins)
    S, W, n = 1 << 18, 8, 1 << 21
    c = OracleCache(S * W, W, 1)
    keys = np.arange(n, dtype=np.int64)
    c.insert(keys, np.zeros((n, 1), dtype=np.uint32))
    loads = c.ctr.astype(np.int64)            # distinct keys: counter = load of the set
    assert loads.sum() == n
    lam = n / S
    from scipy import stats
    kmax = 20
    obs = np.bincount(np.minimum(loads, kmax), minlength=kmax + 1).astype(float)
    p = stats.poisson.pmf(np.arange(kmax + 1), lam)
    p[kmax] = 1.0 - p[:kmax].sum()
    chi2 = ((obs - S * p) ** 2 / (S * p)).sum()
    # 20 degrees of freedom: 99.99th percentile is about 52
    assert chi2 < 60.0, chi2
    # closed form for occupancy and for the occupied fraction
    occ = int((c.keys != EMPTY_KEY).sum())
    assert occ == int(np.minimum(loads, W).sum())
    expect = S * sum(min(k, W) * stats.poisson.pmf(k, lam) for k in range(200))
    assert abs(occ - expect) < 0.005 * expect


# ---------------------------------------------------------------- special cases

def test_no_overflow_behaves_like_dict():
    # 2^16 slots, 3000 distinct keys: practically no set gets more than 8 keys; verify, then compare with a dict
    S, W, d = 1 << 13, 8, 4
    c = OracleCache(S * W, W, d)
    rng = np.random.Generator(np.random.PCG64(5))
    ref = {}
    for step in range(30):
        keys = rng.integers(0, 3000, size=400, dtype=np.int64)
        rows = rows_for(keys, d, salt=step)
        op = step % 3
        if op == 0:
            c.insert(keys, rows)
            for k, r in zip(keys.tolist(), rows):
                ref.setdefault(k, r.copy())           # existing keys are ignored
        elif op == 1:
            c.update(keys, rows)
            for k, r in zip(keys.tolist(), rows):
                if k in ref:
                    ref[k] = r.copy()                 # last writer in index order wins
        else:
            out = np.full((400, d), 0xDEADBEEF, dtype=np.uint32)
            _, mi, mk = c.query(keys, out)
            exp_miss = [i for i, k in enumerate(keys.tolist()) if k not in ref]
            assert mi.tolist() == exp_miss
            assert mk.tolist() == [int(keys[i]) for i in exp_miss]
            for i, k in enumerate(keys.tolist()):
                if k in ref:
                    assert (out[i] == ref[k]).all()
                else:
                    assert (out[i] == 0xDEADBEEF).all()
    assert c.ctr.max() <= W                            # premise of the special case
    assert sorted(c.dump().tolist()) == sorted(ref.keys())


def keys_in_set(target, S, count, start=0):
    out, k = [], start
    while len(out) < count:
        if py_set_of(k, S) == target:
            out.append(k)
        k += 1
    return out


@pytest.mark.parametrize("W", [1, 2, 8, 64])
def test_one_set_is_a_fifo_deque(W):
    S, d = 37, 2
    c = OracleCache(S * W, W, d)
    pool = keys_in_set(5, S, 4 * W + 3)
    rng = np.random.Generator(np.random.PCG64(W))
    dq = collections.deque(maxlen=W)
    for step in range(60):
        ks = rng.choice(pool, size=rng.integers(1, 6)).astype(np.int64)
        c.insert(ks, rows_for(ks, d))
        for k in ks.tolist():
            if k not in dq:
                dq.append(k)                           # maxlen drops the oldest
        resident = sorted(c.dump().tolist())
        assert resident == sorted(dq)
        _, mi, _ = c.query(np.array(pool, dtype=np.int64))
        assert sorted(set(pool) - {pool[i] for i in mi.tolist()}) == sorted(dq)
    # only set 5 was ever touched
    assert (np.delete(c.ctr, 5) == 0).all()


def test_direct_mapped_last_writer_of_set_wins():
    S, d = 64, 3
    c = OracleCache(S, 1, d)
    rng = np.random.Generator(np.random.PCG64(3))
    table = {}
    for step in range(20):
        ks = rng.integers(0, 5000, size=50, dtype=np.int64)
        c.insert(ks, rows_for(ks, d, step))
        for k, r in zip(ks.tolist(), rows_for(ks, d, step)):
            s = py_set_of(k, S)
            if s in table and table[s][0] == k:
                continue
            table[s] = (k, r.copy())
        for s, (k, r) in table.items():
            assert c.keys[s, 0] == k and (c.vals[s, 0] == r).all()
    assert int((c.keys != EMPTY_KEY).sum()) == len(table)


def test_single_set_fully_associative_fifo():
    W, d = 16, 2
    c = OracleCache(W, W, d)
    dq = collections.deque(maxlen=W)
    rng = np.random.Generator(np.random.PCG64(9))
    for step in range(40):
        ks = rng.integers(-1000, 1000, size=7, dtype=np.int64)
        c.insert(ks, rows_for(ks, d))
        for k in ks.tolist():
            if k not in dq:
                dq.append(k)
        assert sorted(c.dump().tolist()) == sorted(dq)
        assert int(c.ctr[0]) >= len(dq)


# ---------------------------------------------------------------- brute force + invariants

def check_invariants(c, last_row):
    S, W = c.S, c.W
    flat = c.keys.reshape(-1)
    res = flat[flat != EMPTY_KEY]
    assert len(set(res.tolist())) == len(res), "a key is resident twice"
    assert len(res) <= S * W
    for s in range(S):
        occ = min(int(c.ctr[s]), W)
        assert (c.keys[s, :occ] != EMPTY_KEY).all()
        assert (c.keys[s, occ:] == EMPTY_KEY).all()
        for w in range(occ):
            k = int(c.keys[s, w])
            assert py_set_of(k, S) == s, "key lives outside its set"
            assert (c.vals[s, w] == last_row[k]).all(), "row is not the last one written"


@pytest.mark.parametrize("S,W", [(1, 1), (1, 4), (3, 2), (7, 8), (16, 4), (16, 8)])
def test_brute_force_random_op_sequences(S, W):
    """Two caches get the same operations: `c` as whole batches, `c1` one element at a time.
    On `c1` residency is decided by scanning every slot before each single operation, which
    gives the bookkeeping of "last row written" without knowing anything about sets; the two
    states must then agree exactly, because a batch is defined as its elements in index order.
    """
    d = 3
    rng = np.random.Generator(np.random.PCG64(1000 * S + W))
    for trial in range(25):
        c = OracleCache(S * W, W, d)
        c1 = OracleCache(S * W, W, d)
        last_row = {}
        salt = 0
        for step in range(40):
            n = int(rng.integers(0, 12))
            ks = rng.integers(0, 96, size=n, dtype=np.int64)
            if rng.random() < 0.1 and n:
                ks[rng.integers(0, n)] = EMPTY_KEY if rng.random() < 0.5 else RESERVED_KEY
            op = rng.integers(0, 3)
            salt += 1
            rows = rows_for(ks, d, salt) if n else np.zeros((0, d), np.uint32)
            if op == 0:
                before = set(c.keys.reshape(-1).tolist())
                new_per_set = collections.Counter(
                    py_set_of(k, S) for k in set(ks.tolist()) - before - {EMPTY_KEY, RESERVED_KEY})
                ctr_before = c.ctr.copy()
                keys_before_ins = c.keys.copy()
                c.insert(ks, rows)
                for i in range(n):
                    k = int(ks[i])
                    resident = k in set(c1.keys.reshape(-1).tolist())
                    ctr1 = int(c1.ctr.sum())
                    c1.insert(ks[i:i + 1], rows[i:i + 1])
                    if k in (EMPTY_KEY, RESERVED_KEY) or resident:
                        assert int(c1.ctr.sum()) == ctr1          # ignored
                    else:
                        assert int(c1.ctr.sum()) == ctr1 + 1
                        assert k in c1.keys                       # a single insert always lands
                        last_row[k] = rows[i].copy()
                after = set(c.keys.reshape(-1).tolist())
                # The batch is order-independent when, in every set, the new keys number at
                # most W and the slots they overwrite hold no key of this same batch.
                batch = set(ks.tolist())
                calm = True
                for s_, cnt in new_per_set.items():
                    victims = {(int(ctr_before[s_]) + t) % W for t in range(cnt)}
                    if cnt > W or any(int(keys_before_ins[s_, w]) in batch for w in victims):
                        calm = False
                if calm:
                    # one counter step per distinct new key, and every new key is resident
                    for s in range(S):
                        assert int(c.ctr[s]) == int(ctr_before[s]) + new_per_set.get(s, 0)
                    assert (batch - before - {EMPTY_KEY, RESERVED_KEY}) <= after
            elif op == 1:
                resident = set(c.keys.reshape(-1).tolist())
                keys_before = c.keys.copy()
                ctr_before = c.ctr.copy()
                c.update(ks, rows)
                assert (c.keys == keys_before).all() and (c.ctr == ctr_before).all()
                for i in range(n):
                    c1.update(ks[i:i + 1], rows[i:i + 1])
                    k = int(ks[i])
                    if k in resident and k not in (EMPTY_KEY, RESERVED_KEY):
                        last_row[k] = rows[i].copy()
            else:
                resident = set(c.keys.reshape(-1).tolist()) - {EMPTY_KEY}
                out = np.full((n, d), 0xABCD1234, dtype=np.uint32)
                keys_before = c.keys.copy()
                _, mi, mk = c.query(ks, out)
                assert (c.keys == keys_before).all()          # query is read-only
                exp = [i for i, k in enumerate(ks.tolist()) if k not in resident]
                assert mi.tolist() == exp
                assert mk.tolist() == [int(ks[i]) for i in exp]
                for i, k in enumerate(ks.tolist()):
                    if k in resident:
                        assert (out[i] == last_row[k]).all()
                    else:
                        assert (out[i] == 0xABCD1234).all()
            assert (c.keys == c1.keys).all() and (c.ctr == c1.ctr).all() and (c.vals == c1.vals).all()
            check_invariants(c, last_row)


def test_hypothesis_sequences_keep_invariants():
    hyp = pytest.importorskip("hypothesis")
    st = hyp.strategies

    op = st.tuples(st.sampled_from(["ins", "upd"]),
                   st.lists(st.integers(min_value=0, max_value=40), min_size=0, max_size=10))

    @hyp.settings(max_examples=150, deadline=None)
    @hyp.given(st.lists(op, min_size=1, max_size=25), st.sampled_from([(2, 2), (4, 4), (5, 1), (1, 8)]))
    def run(ops, geom):
        S, W = geom
        c = OracleCache(S * W, W, 2)
        last_row = {}
        for salt, (kind, ks) in enumerate(ops):
            ks = np.array(ks, dtype=np.int64)
            rows = rows_for(ks, 2, salt) if len(ks) else np.zeros((0, 2), np.uint32)
            for i in range(len(ks)):                      # one element at a time
                k = int(ks[i])
                resident = k in set(c.keys.reshape(-1).tolist())
                if kind == "ins":
                    c.insert(ks[i:i + 1], rows[i:i + 1])
                    if not resident:
                        last_row[k] = rows[i].copy()
                else:
                    c.update(ks[i:i + 1], rows[i:i + 1])
                    if resident:
                        last_row[k] = rows[i].copy()
            check_invariants(c, last_row)

    run()


# ---------------------------------------------------------------- contract details

def test_duplicates_and_reserved_keys_in_query():
    c = OracleCache(64, 8, 2)
    c.insert(np.array([10, 11], dtype=np.int64), rows_for([10, 11], 2))
    q = np.array([10, 99, 10, EMPTY_KEY, 99, RESERVED_KEY, 11], dtype=np.int64)
    out = np.full((7, 2), 7, dtype=np.uint32)
    _, mi, mk = c.query(q, out)
    assert mi.tolist() == [1, 3, 4, 5]                       # one entry per missing position
    assert mk.tolist() == [99, EMPTY_KEY, 99, RESERVED_KEY]
    assert (out[0] == out[2]).all() and (out[0] == rows_for([10], 2)[0]).all()
    assert (out[[1, 3, 4, 5]] == 7).all()


def test_insert_ignores_existing_and_duplicates_take_first():
    c = OracleCache(64, 8, 2)
    ks = np.array([5, 5, 6], dtype=np.int64)
    rows = np.array([[1, 1], [2, 2], [3, 3]], dtype=np.uint32)
    c.insert(ks, rows)
    out, mi, _ = c.query(np.array([5, 6], dtype=np.int64))
    assert mi.size == 0 and out.tolist() == [[1, 1], [3, 3]]
    c.insert(np.array([5], dtype=np.int64), np.array([[9, 9]], dtype=np.uint32))
    out, _, _ = c.query(np.array([5], dtype=np.int64))
    assert out.tolist() == [[1, 1]]                          # already cached: ignored
    assert int(c.ctr.sum()) == 2
    c.update(np.array([5, 7], dtype=np.int64), np.array([[4, 4], [8, 8]], dtype=np.uint32))
    out, mi, _ = c.query(np.array([5, 7], dtype=np.int64))
    assert out[0].tolist() == [4, 4] and mi.tolist() == [1]  # update never inserts
    # reserved keys are never stored
    c.insert(np.array([EMPTY_KEY, RESERVED_KEY], dtype=np.int64), np.zeros((2, 2), np.uint32))
    assert int(c.ctr.sum()) == 2 and RESERVED_KEY not in c.keys


def test_empty_batches_and_bad_geometry():
    c = OracleCache(16, 4, 2)
    out, mi, mk = c.query(np.zeros(0, dtype=np.int64))
    assert out.shape == (0, 2) and mi.size == 0 and mk.size == 0
    c.insert(np.zeros(0, dtype=np.int64), np.zeros((0, 2), np.uint32))
    c.update(np.zeros(0, dtype=np.int64), np.zeros((0, 2), np.uint32))
    assert (c.keys == EMPTY_KEY).all()
    for cap, W, d in [(10, 4, 2), (16, 3, 2), (16, 128, 2), (16, 4, 0), (0, 4, 2)]:
        with pytest.raises(ValueError):
            OracleCache(cap, W, d)
