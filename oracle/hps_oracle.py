"""ctypes front end of oracle/hps_oracle.c (test infrastructure only).

All arithmetic of the method lives in the C file; this module only marshals numpy arrays.
Rows are carried as uint32 bit patterns ([n, d] arrays); float32 arrays are reinterpreted,
never converted.
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

EMPTY_KEY = -(1 << 63)          # "Null" key of Alg. 2-4
RESERVED_KEY = -(1 << 63) + 1   # second reserved value of the build's contract

_lib = None


def load_library(path=None):
    """Load the oracle library.  `path` names another build of it (the mutation tests compile
    deliberately broken copies); the default is the library built from oracle/hps_oracle.c."""
    global _lib
    if path is None and _lib is not None:
        return _lib
    lib = C.CDLL(path if path is not None else _build.build())
    vp, u64, u32 = C.c_void_p, C.c_uint64, C.c_uint32
    lib.hpso_mix64.restype = u64
    lib.hpso_mix64.argtypes = [u64]
    lib.hpso_create.restype = vp
    lib.hpso_create.argtypes = [u64, u32, u32]
    lib.hpso_create_policy.restype = vp
    lib.hpso_create_policy.argtypes = [u64, u32, u32, u32]
    lib.hpso_get_g.restype = u32
    lib.hpso_get_g.argtypes = [vp]
    lib.hpso_set_g.restype = None
    lib.hpso_set_g.argtypes = [vp, u32]
    lib.hpso_destroy.restype = None
    lib.hpso_destroy.argtypes = [vp]
    lib.hpso_set_of.restype = u64
    lib.hpso_set_of.argtypes = [vp, C.c_int64]
    lib.hpso_sets_of.restype = None
    lib.hpso_sets_of.argtypes = [vp, vp, u64, vp]
    lib.hpso_num_sets.restype = u64
    lib.hpso_num_sets.argtypes = [vp]
    for name in ("hpso_keys", "hpso_vals", "hpso_ctr", "hpso_stamps"):
        getattr(lib, name).restype = vp
        getattr(lib, name).argtypes = [vp]
    lib.hpso_query.restype = u64
    lib.hpso_query.argtypes = [vp, vp, u64, vp, vp, vp]
    lib.hpso_insert.restype = None
    lib.hpso_insert.argtypes = [vp, vp, vp, u64]
    lib.hpso_update.restype = None
    lib.hpso_update.argtypes = [vp, vp, vp, u64]
    lib.hpso_dump.restype = u64
    lib.hpso_dump.argtypes = [vp, vp]
    lib.hpso_dedup.restype = u64
    lib.hpso_dedup.argtypes = [vp, u64, vp, vp]
    lib.hpso_expand.restype = None
    lib.hpso_expand.argtypes = [vp, vp, u64, u32, vp]
    lib.hpso_lookup.restype = u64
    lib.hpso_lookup.argtypes = [vp, vp, u64, vp, C.c_float, vp, vp, C.POINTER(C.c_float),
                                C.POINTER(C.c_int), vp, C.c_int]
    if path is None:
        _lib = lib
    return lib


def _load():
    return load_library()


def mix64(x: int, lib=None) -> int:
    return int((lib or _load()).hpso_mix64(C.c_uint64(x & 0xFFFFFFFFFFFFFFFF)))


def _keys(a):
    a = np.ascontiguousarray(a, dtype=np.int64)
    return a


def _rows(a, n, d):
    a = np.ascontiguousarray(a)
    if a.dtype == np.float32:
        a = a.view(np.uint32)
    if a.dtype != np.uint32:
        raise TypeError("rows must be float32 or uint32 bit patterns")
    if a.shape != (n, d):
        raise ValueError(f"rows must have shape {(n, d)}, got {a.shape}")
    return a


class OracleCache:
    """One set-associative cache of `capacity` slots, `ways` slots per set, `dim` words per row."""

    def __init__(self, capacity: int, ways: int, dim: int, policy: int = 0, lib=None):
        """policy 0: per-set victim counter; policy 1: LRU by access stamp (the paper's rule)."""
        lib = lib or _load()
        self._lib = lib
        self.policy = policy
        self._h = lib.hpso_create_policy(capacity, ways, dim, policy)
        if not self._h:
            raise ValueError("invalid cache geometry")
        self.S = int(lib.hpso_num_sets(self._h))
        self.W = ways
        self.d = dim
        n = self.S * self.W
        self.keys = np.ctypeslib.as_array(
            C.cast(lib.hpso_keys(self._h), C.POINTER(C.c_int64)), shape=(self.S, self.W))
        self.vals = np.ctypeslib.as_array(
            C.cast(lib.hpso_vals(self._h), C.POINTER(C.c_uint32)), shape=(self.S, self.W, dim))
        self.ctr = np.ctypeslib.as_array(
            C.cast(lib.hpso_ctr(self._h), C.POINTER(C.c_uint32)), shape=(self.S,))
        self.stamps = np.ctypeslib.as_array(
            C.cast(lib.hpso_stamps(self._h), C.POINTER(C.c_uint32)), shape=(self.S, self.W))
        assert self.keys.size == n

    def close(self):
        if self._h:
            self.keys = self.vals = self.ctr = self.stamps = None
            self._lib.hpso_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @property
    def g(self) -> int:
        return int(self._lib.hpso_get_g(self._h))

    @g.setter
    def g(self, value: int):
        self._lib.hpso_set_g(self._h, value & 0xFFFFFFFF)

    def set_of(self, key: int) -> int:
        return int(self._lib.hpso_set_of(self._h, C.c_int64(key)))

    def sets_of(self, keys) -> np.ndarray:
        """Set index of every key of a batch (int64 array)."""
        keys = _keys(keys)
        out = np.empty(keys.shape[0], dtype=np.uint64)
        self._lib.hpso_sets_of(self._h, keys.ctypes.data, keys.shape[0], out.ctypes.data)
        return out.astype(np.int64)

    def query(self, keys, out=None):
        """Returns (out, miss_idx, miss_keys).  `out` ([n, d] uint32) keeps its miss rows."""
        keys = _keys(keys)
        n = keys.shape[0]
        if out is None:
            out = np.zeros((n, self.d), dtype=np.uint32)
        else:
            assert out.dtype == np.uint32 and out.shape == (n, self.d) and out.flags.c_contiguous
        mi = np.empty(max(n, 1), dtype=np.uint32)
        mk = np.empty(max(n, 1), dtype=np.int64)
        m = self._lib.hpso_query(self._h, keys.ctypes.data, n, out.ctypes.data,
                                 mi.ctypes.data, mk.ctypes.data)
        return out, mi[:m].copy(), mk[:m].copy()

    def insert(self, keys, rows):
        keys = _keys(keys)
        rows = _rows(rows, keys.shape[0], self.d)
        self._lib.hpso_insert(self._h, keys.ctypes.data, rows.ctypes.data, keys.shape[0])

    def update(self, keys, rows):
        keys = _keys(keys)
        rows = _rows(rows, keys.shape[0], self.d)
        self._lib.hpso_update(self._h, keys.ctypes.data, rows.ctypes.data, keys.shape[0])

    def lookup(self, keys, lower_rows, threshold, default_row, do_insert=True):
        """One pass of Alg. 1.  lower_rows[i] is the vector the lower tiers hold for keys[i].
        Returns (out, hit_rate as float32, synchronous, distinct missing keys in first-occurrence order)."""
        keys = _keys(keys)
        n = keys.shape[0]
        lower = _rows(lower_rows, n, self.d)
        dflt = _rows(np.asarray(default_row).reshape(1, -1), 1, self.d)
        out = np.zeros((n, self.d), dtype=np.uint32)
        ins = np.empty(max(n, 1), dtype=np.int64)
        rate, sync = C.c_float(), C.c_int()
        u = self._lib.hpso_lookup(self._h, keys.ctypes.data, n, lower.ctypes.data, C.c_float(threshold),
                                  dflt.ctypes.data, out.ctypes.data, C.byref(rate), C.byref(sync),
                                  ins.ctypes.data, 1 if do_insert else 0)
        return out, np.float32(rate.value), bool(sync.value), ins[:u].copy()

    def dump(self):
        buf = np.empty(self.S * self.W, dtype=np.int64)
        m = self._lib.hpso_dump(self._h, buf.ctypes.data)
        return buf[:m].copy()

    def load_state(self, keys, ctr, vals=None, stamps=None):
        """Overwrite the whole state (used to re-seat the oracle after an overflowing batch)."""
        if stamps is not None:
            self.stamps[...] = np.asarray(stamps, dtype=np.uint32).reshape(self.S, self.W)
        self.keys[...] = np.asarray(keys, dtype=np.int64).reshape(self.S, self.W)
        self.ctr[...] = np.asarray(ctr, dtype=np.uint32).reshape(self.S)
        if vals is not None:
            v = np.asarray(vals)
            if v.dtype == np.float32:
                v = v.view(np.uint32)
            self.vals[...] = v.reshape(self.S, self.W, self.d)


def set_of(key: int, num_sets: int, lib=None) -> int:
    """Set index of a key for a cache with `num_sets` sets (same rule as the C file, via its mix64)."""
    return (mix64(key, lib) >> 32) % num_sets


def dedup(keys, lib=None):
    """Q* = dedup(Q) (Sec. 2.2): (distinct keys in order of first occurrence, inverse map)."""
    keys = _keys(keys)
    n = keys.shape[0]
    uniq = np.empty(max(n, 1), dtype=np.int64)
    inv = np.empty(max(n, 1), dtype=np.uint32)
    u = (lib or _load()).hpso_dedup(keys.ctypes.data, n, uniq.ctypes.data, inv.ctypes.data)
    return uniq[:u].copy(), inv[:n].copy()


def expand(rows, inverse, lib=None):
    """out[i] = rows[inverse[i]] for rows given as [u, d] uint32/float32 bit patterns."""
    rows = np.ascontiguousarray(rows)
    if rows.dtype == np.float32:
        rows = rows.view(np.uint32)
    inverse = np.ascontiguousarray(inverse, dtype=np.uint32)
    n, d = inverse.shape[0], rows.shape[1]
    assert n == 0 or int(inverse.max()) < rows.shape[0]
    out = np.empty((n, d), dtype=np.uint32)
    (lib or _load()).hpso_expand(rows.ctypes.data, inverse.ctypes.data, n, d, out.ctypes.data)
    return out
