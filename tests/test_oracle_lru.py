"""Pins for the oracle's LRU policy (the paper's replacement rule, Sec. 4.2 Replace, Alg. 2-3).

With one key per call the rule is textbook LRU, which collections.OrderedDict states in four
lines; with batches, everything touched by one call shares one stamp, which a small independent
Python model spells out.  Stamps are compared as ages modulo 2^32, pinned by a wrap-around case.
"""
import collections

import numpy as np
import pytest

from oracle import OracleCache, EMPTY_KEY
from test_oracle_pins import py_set_of, rows_for


def lookup_then_fill(c, k, d):
    """Alg. 1 with one key: query; on a miss fetch and insert."""
    key = np.array([k], dtype=np.int64)
    _, mi, _ = c.query(key)
    if mi.size:
        c.insert(key, rows_for(key, d))
    return mi.size == 0


@pytest.mark.parametrize("W", [1, 2, 4, 8, 64])
def test_single_key_calls_are_textbook_lru(W):
    d = 2
    c = OracleCache(W, W, d, policy=1)                   # one set: fully associative
    lru = collections.OrderedDict()
    rng = np.random.Generator(np.random.PCG64(W))
    for _ in range(600):
        k = int(rng.integers(0, 3 * W + 2))
        hit = lookup_then_fill(c, k, d)
        assert hit == (k in lru)
        if k in lru:
            lru.move_to_end(k)
        else:
            if len(lru) == W:
                lru.popitem(last=False)                  # least recently used goes
            lru[k] = True
        assert sorted(c.dump().tolist()) == sorted(lru)


def test_each_set_is_its_own_lru():
    S, W, d = 5, 4, 2
    c = OracleCache(S * W, W, d, policy=1)
    per_set = collections.defaultdict(collections.OrderedDict)
    rng = np.random.Generator(np.random.PCG64(2))
    for _ in range(1500):
        k = int(rng.integers(0, 90))
        lru = per_set[py_set_of(k, S)]
        hit = lookup_then_fill(c, k, d)
        assert hit == (k in lru)
        if k in lru:
            lru.move_to_end(k)
        else:
            if len(lru) == W:
                lru.popitem(last=False)
            lru[k] = True
    resident = sorted(c.dump().tolist())
    assert resident == sorted(k for lru in per_set.values() for k in lru)


class PyLru:
    """Independent model of the batched rule: dict slot state, explicit scans."""

    def __init__(self, S, W):
        self.S, self.W, self.g = S, W, 0
        self.slots = [[None] * W for _ in range(S)]      # (key, stamp) or None

    def _find(self, s, k):
        for w, e in enumerate(self.slots[s]):
            if e is not None and e[0] == k:
                return w
        return None

    def query(self, keys):
        self.g = (self.g + 1) % (1 << 32)
        miss = []
        for i, k in enumerate(keys):
            s = py_set_of(k, self.S)
            w = self._find(s, k)
            if w is None:
                miss.append(i)
            else:
                self.slots[s][w] = (k, self.g)
        return miss

    def insert(self, keys):
        for k in keys:
            s = py_set_of(k, self.S)
            w = self._find(s, k)
            if w is not None:
                self.slots[s][w] = (k, self.g)
                continue
            empties = [w for w, e in enumerate(self.slots[s]) if e is None]
            if empties:
                w = empties[0]
            else:
                ages = [(self.g - e[1]) % (1 << 32) for e in self.slots[s]]
                w = ages.index(max(ages))                # first way among the oldest
            self.slots[s][w] = (k, self.g)


@pytest.mark.parametrize("S,W", [(1, 4), (3, 2), (7, 8), (16, 4)])
def test_batched_calls_match_independent_model(S, W):
    d = 2
    rng = np.random.Generator(np.random.PCG64(S * 100 + W))
    for trial in range(10):
        c = OracleCache(S * W, W, d, policy=1)
        m = PyLru(S, W)
        if trial % 2:                                    # start close to the 32-bit wrap
            c.g = (1 << 32) - 5
            m.g = (1 << 32) - 5
        for step in range(60):
            ks = rng.integers(0, 12 * S, size=int(rng.integers(1, 10)), dtype=np.int64)
            if rng.random() < 0.6:
                _, mi, _ = c.query(ks)
                assert mi.tolist() == m.query(ks.tolist())
            else:
                c.insert(ks, rows_for(ks, d))
                m.insert(ks.tolist())
            for s in range(S):
                for w in range(W):
                    e = m.slots[s][w]
                    if e is None:
                        assert c.keys[s, w] == EMPTY_KEY
                    else:
                        assert (int(c.keys[s, w]), int(c.stamps[s, w])) == e
            assert c.g == m.g


def test_keys_touched_by_a_call_outlive_untouched_ones():
    # one set of 8: fill, touch three keys by a query, insert five new keys: the three survive
    W, d = 8, 2
    c = OracleCache(W, W, d, policy=1)
    base = np.arange(100, 108, dtype=np.int64)
    c.insert(base, rows_for(base, d))
    touched = np.array([101, 104, 106], dtype=np.int64)
    _, mi, _ = c.query(touched)
    assert mi.size == 0
    new = np.arange(200, 205, dtype=np.int64)
    c.insert(new, rows_for(new, d))
    resident = set(c.dump().tolist())
    assert set(touched.tolist()) <= resident and set(new.tolist()) <= resident
    assert len(resident) == W
    # update does not refresh a stamp (Alg. 4), a found key in a Replace call does (Alg. 3)
    stamps_before = c.stamps.copy()
    c.update(touched, rows_for(touched, d, 9))
    assert (c.stamps == stamps_before).all()
    c.query(np.array([999], dtype=np.int64))             # g moves on
    c.insert(np.array([200], dtype=np.int64), rows_for([200], d))
    w = int(np.nonzero(c.keys[0] == 200)[0][0])
    assert int(c.stamps[0, w]) == c.g and (c.vals[0, w] == rows_for([200], d)[0]).all()   # row ignored, stamp refreshed


def test_policy0_is_unaffected_by_stamps():
    c0 = OracleCache(32, 4, 2, policy=0)
    ks = np.arange(50, dtype=np.int64)
    c0.insert(ks, rows_for(ks, 2))
    c0.query(ks)
    assert (c0.stamps == 0).all() and c0.g == 0
    with pytest.raises(ValueError):
        OracleCache(32, 4, 2, policy=2)
