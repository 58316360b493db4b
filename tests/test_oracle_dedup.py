"""Pins for the oracle's dedup operator (Sec. 2.2, Q* = dedup(Q)) and the row expansion that
follows a lookup of Q*.

The distinct keys of a batch are a set, which Python's own set and numpy.unique state
independently; the order (first occurrence) and the inverse map are pinned by a worked example,
by dict.fromkeys (insertion-ordered) and by the defining property unique[inverse[i]] == keys[i].
"""
import numpy as np
import pytest

import oracle
from oracle import EMPTY_KEY, RESERVED_KEY
from paper_2210_08804_amd import inputs


def test_worked_example():
    uniq, inv = oracle.dedup([5, 3, 5, 7, 3, 3, -1])
    assert uniq.tolist() == [5, 3, 7, -1]
    assert inv.tolist() == [0, 1, 0, 2, 1, 1, 3]


def test_degenerate_batches():
    uniq, inv = oracle.dedup([])
    assert uniq.size == 0 and inv.size == 0
    uniq, inv = oracle.dedup([9] * 1000)
    assert uniq.tolist() == [9] and (inv == 0).all() and inv.size == 1000
    keys = np.arange(500, dtype=np.int64)[::-1].copy()
    uniq, inv = oracle.dedup(keys)
    assert (uniq == keys).all() and (inv == np.arange(500)).all()
    # the cache's two reserved values and the extremes are ordinary keys to dedup
    keys = [EMPTY_KEY, RESERVED_KEY, (1 << 63) - 1, EMPTY_KEY, 0, RESERVED_KEY]
    uniq, inv = oracle.dedup(keys)
    assert uniq.tolist() == [EMPTY_KEY, RESERVED_KEY, (1 << 63) - 1, 0] and inv.tolist() == [0, 1, 2, 0, 3, 1]


@pytest.mark.parametrize("seed,alpha", [(1, 1.05), (2, 1.5), (3, 0.0)])
def test_against_set_dict_and_numpy_unique(seed, alpha):
    n = 20000
    keys = (inputs.zipf_keys(n, 10 ** 6, alpha, seed) if alpha else inputs.uniform_keys(n, 5000, seed))
    uniq, inv = oracle.dedup(keys)
    assert set(uniq.tolist()) == set(keys.tolist()) and len(uniq) == len(set(keys.tolist()))
    assert uniq.tolist() == list(dict.fromkeys(keys.tolist()))          # first-occurrence order
    nu, ninv = np.unique(keys, return_inverse=True)
    assert len(nu) == len(uniq) and (np.sort(uniq) == nu).all()
    assert (uniq[inv] == keys).all() and (nu[ninv] == uniq[inv]).all()
    assert inv.dtype == np.uint32 and int(inv.max()) == len(uniq) - 1
    # the place of a key is the number of distinct keys before its first occurrence
    first = {}
    for i, k in enumerate(keys.tolist()):
        first.setdefault(k, len(first))
    assert inv.tolist() == [first[k] for k in keys.tolist()]


def test_brute_force_small_alphabets():
    rng = np.random.Generator(np.random.PCG64(4))
    for _ in range(300):
        n = int(rng.integers(0, 40))
        keys = rng.integers(-3, 4, size=n).astype(np.int64)
        uniq, inv = oracle.dedup(keys)
        exp_u, exp_inv = [], []
        for k in keys.tolist():
            if k not in exp_u:
                exp_u.append(k)
            exp_inv.append(exp_u.index(k))
        assert uniq.tolist() == exp_u and inv.tolist() == exp_inv


def test_expand_is_a_row_gather():
    rng = np.random.Generator(np.random.PCG64(5))
    rows = rng.integers(0, 1 << 32, size=(37, 12), dtype=np.uint64).astype(np.uint32)
    inv = rng.integers(0, 37, size=500).astype(np.uint32)
    out = oracle.expand(rows, inv)
    assert out.shape == (500, 12) and (out == rows[inv]).all()          # numpy's own gather
    assert oracle.expand(rows, np.zeros(0, dtype=np.uint32)).shape == (0, 12)
    # float32 rows are reinterpreted, never converted
    f = rows.view(np.float32)
    assert (oracle.expand(f, inv) == out).all()


def test_lookup_of_unique_keys_then_expand_equals_direct_lookup():
    """The reason the operator exists: querying Q* and expanding gives every position what a
    direct query of Q gives it (rows of hits; the positions of missing keys are those whose
    unique key is missing)."""
    d = 8
    c = oracle.OracleCache(64 * 4, 4, d)
    resident = np.unique(inputs.uniform_keys(150, 400, 6))
    c.insert(resident, inputs.backing_rows(resident, d).view(np.uint32))
    keys = inputs.zipf_keys(3000, 400, 1.2, 7)
    direct = np.full((len(keys), d), 0xAAAAAAAA, dtype=np.uint32)
    _, mi, mk = c.query(keys, direct)
    uniq, inv = oracle.dedup(keys)
    urows = np.full((len(uniq), d), 0xAAAAAAAA, dtype=np.uint32)
    _, umi, umk = c.query(uniq, urows)
    assert (oracle.expand(urows, inv) == direct).all()
    missing_u = np.zeros(len(uniq), dtype=bool)
    missing_u[umi] = True
    assert (np.nonzero(missing_u[inv])[0] == mi).all() and (uniq[inv][mi] == mk).all()
    assert sorted(set(mk.tolist())) == sorted(umk.tolist())
