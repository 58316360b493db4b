"""Thin ctypes binding of include/hps_cache.h, hps_lookup.h and hps_dedup.h: argument marshalling only.

Every function has the name of the C entry point it calls.  Tensors are torch CUDA (ROCm)
tensors used purely as device buffers; `stream` is a torch.cuda.Stream or None (= the current
stream).  Nothing here computes anything and there is no CPU fallback: if the HIP library
has not been built, loading raises.
"""
import ctypes as C
import os

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libhps_cache.so")

HPS_OK = 0
HPS_ERR_INVALID_ARG = -1
HPS_ERR_OOM = -2
HPS_ERR_DEVICE = -3
HPS_MAX_TABLES = 32
HPS_POLICY_VICTIM_COUNTER = 0
HPS_POLICY_LRU = 1
HPS_FLAG_STUCK_SET = 1

EXPORTS = (
    "hps_cache_create", "hps_cache_destroy", "hps_cache_query", "hps_cache_insert",
    "hps_cache_update", "hps_last_error", "hps_cache_set_concurrent_writers", "hps_cache_info",
    "hps_cache_export", "hps_cache_import", "hps_cache_dump", "hps_cache_query_multi",
    "hps_backing_fetch", "hps_cache_insert_dn", "hps_cache_update_dn", "hps_cache_set_query_dedup",
    "hps_cache_create_policy", "hps_cache_export_lru", "hps_cache_import_lru",
    "hps_cache_flags", "hps_cache_debug_set_seq", "hps_cache_query_dn",
    "hps_lookup_create", "hps_lookup", "hps_lookup_drain", "hps_lookup_destroy", "hps_lookup_last_error",
    "hps_cache_refresh", "hps_refresh_create", "hps_refresh_run", "hps_refresh_destroy",
    "hps_dedup_create", "hps_dedup_destroy", "hps_dedup", "hps_expand_rows", "hps_dedup_last_error",
    "hps_dedup_noalloc",
    "hps_hostmap_create", "hps_hostmap_destroy", "hps_hostmap_put", "hps_hostmap_get", "hps_hostmap_fetch",
    "hps_hostmap_stats",
    "hps_membench_gather", "hps_membench_gather_half", "hps_membench_copy",
)

# lower-tier fetch callback of hps_lookup.h: (user, keys*, n, rows*)
FETCH_FN = C.CFUNCTYPE(None, C.c_void_p, C.POINTER(C.c_int64), C.c_size_t, C.POINTER(C.c_float))

_lib = None


class HpsError(RuntimeError):
    def __init__(self, status, message):
        super().__init__(f"hps status {status}: {message}")
        self.status = status


def load_library():
    """Load the built HIP library; raise if it is missing (build it with __graft_entry__.build())."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            f"{LIB_PATH} is missing: build the HIP extension first "
            "(python -c 'import __graft_entry__ as g; g.build()'); there is no CPU fallback")
    lib = C.CDLL(LIB_PATH)
    vp, sz, u32 = C.c_void_p, C.c_size_t, C.c_uint32
    lib.hps_last_error.restype = C.c_char_p
    lib.hps_last_error.argtypes = []
    lib.hps_lookup_last_error.restype = C.c_char_p
    lib.hps_lookup_last_error.argtypes = []
    lib.hps_dedup_last_error.restype = C.c_char_p
    lib.hps_dedup_last_error.argtypes = []
    sigs = {
        "hps_cache_create": [sz, u32, u32, C.POINTER(vp)],
        "hps_cache_create_policy": [sz, u32, u32, C.c_int, C.POINTER(vp)],
        "hps_cache_export_lru": [vp, vp, C.POINTER(u32), vp],
        "hps_cache_import_lru": [vp, vp, u32, vp],
        "hps_cache_flags": [vp, C.POINTER(u32), C.c_int],
        "hps_cache_debug_set_seq": [vp, C.c_uint64, u32],
        "hps_lookup_create": [vp, sz, C.c_float, vp, FETCH_FN, vp, C.POINTER(vp)],
        "hps_lookup": [vp, vp, sz, vp, C.POINTER(C.c_float), C.POINTER(C.c_int), vp],
        "hps_lookup_drain": [vp],
        "hps_lookup_destroy": [vp],
        "hps_cache_refresh": [vp, sz, FETCH_FN, vp, C.POINTER(sz), vp],
        "hps_refresh_create": [vp, sz, C.POINTER(vp)],
        "hps_refresh_run": [vp, FETCH_FN, vp, C.POINTER(sz), vp],
        "hps_refresh_destroy": [vp],
        "hps_dedup_create": [sz, C.POINTER(vp)],
        "hps_dedup_destroy": [vp],
        "hps_dedup": [vp, vp, sz, vp, vp, vp, vp],
        "hps_dedup_noalloc": [vp, sz, vp, vp, vp, vp],
        "hps_expand_rows": [vp, vp, sz, u32, vp, vp],
        "hps_hostmap_create": [u32, u32, sz, C.POINTER(vp)],
        "hps_hostmap_destroy": [vp],
        "hps_hostmap_put": [vp, vp, vp, sz],
        "hps_hostmap_get": [vp, vp, sz, vp, C.POINTER(sz)],
        "hps_hostmap_stats": [vp, C.POINTER(sz), C.POINTER(sz)],
        "hps_membench_gather": [vp, vp, sz, u32, vp, vp],
        "hps_membench_gather_half": [vp, vp, sz, vp, C.c_int, vp],
        "hps_membench_copy": [vp, vp, sz, C.c_int, vp],
        "hps_cache_destroy": [vp],
        "hps_cache_query": [vp, vp, sz, vp, vp, vp, vp, vp],
        "hps_cache_insert": [vp, vp, vp, sz, vp],
        "hps_cache_update": [vp, vp, vp, sz, vp],
        "hps_cache_set_concurrent_writers": [vp, C.c_int],
        "hps_cache_set_query_dedup": [vp, C.c_int],
        "hps_cache_info": [vp, C.POINTER(C.c_uint64), C.POINTER(u32), C.POINTER(u32)],
        "hps_cache_export": [vp, vp, vp, vp, vp],
        "hps_cache_import": [vp, vp, vp, vp, vp],
        "hps_cache_dump": [vp, sz, sz, vp, vp, vp],
        "hps_cache_query_multi": [C.POINTER(vp), u32, vp, sz, vp, vp, vp, vp, vp],
        "hps_backing_fetch": [vp, sz, vp, u32, u32, vp, vp, vp, vp],
        "hps_cache_insert_dn": [vp, vp, vp, sz, vp, vp],
        "hps_cache_query_dn": [vp, vp, sz, vp, vp, vp, vp, vp, vp],
        "hps_cache_update_dn": [vp, vp, vp, sz, vp, vp],
    }
    for name, argtypes in sigs.items():
        fn = getattr(lib, name)
        fn.restype = C.c_int
        fn.argtypes = argtypes
    lib.hps_hostmap_fetch.restype = None
    lib.hps_hostmap_fetch.argtypes = [vp, vp, sz, vp]
    _lib = lib
    return lib


def _check(status):
    if status != HPS_OK:
        raise HpsError(status, load_library().hps_last_error().decode())


def _ptr(t, dtype=None):
    if t is None:
        return None
    if not t.is_cuda:
        raise TypeError("device tensor expected")
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"expected {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise ValueError("contiguous tensor expected")
    return t.data_ptr()


def _stream(stream):
    s = stream if stream is not None else torch.cuda.current_stream()
    return s.cuda_stream


def hps_cache_create(capacity: int, ways: int, dim: int) -> int:
    h = C.c_void_p()
    _check(load_library().hps_cache_create(capacity, ways, dim, C.byref(h)))
    return h.value


def hps_cache_create_policy(capacity: int, ways: int, dim: int, policy: int) -> int:
    h = C.c_void_p()
    _check(load_library().hps_cache_create_policy(capacity, ways, dim, policy, C.byref(h)))
    return h.value


def hps_cache_export_lru(handle, stamps, stream=None) -> int:
    g = C.c_uint32()
    _check(load_library().hps_cache_export_lru(handle, _ptr(stamps, torch.int32), C.byref(g), _stream(stream)))
    return g.value


def hps_cache_import_lru(handle, stamps, g: int, stream=None) -> None:
    _check(load_library().hps_cache_import_lru(handle, _ptr(stamps, torch.int32), g, _stream(stream)))


def hps_cache_flags(handle, clear: bool = False) -> int:
    f = C.c_uint32()
    _check(load_library().hps_cache_flags(handle, C.byref(f), 1 if clear else 0))
    return f.value


def hps_cache_debug_set_seq(handle, set_index: int, value: int) -> None:
    _check(load_library().hps_cache_debug_set_seq(handle, set_index, value))


def hps_cache_destroy(handle) -> None:
    _check(load_library().hps_cache_destroy(handle))


def hps_cache_query(handle, keys, n, out, miss_idx, miss_keys, n_miss, stream=None) -> None:
    _check(load_library().hps_cache_query(
        handle, _ptr(keys, torch.int64), n, _ptr(out, torch.float32), _ptr(miss_idx, torch.int32),
        _ptr(miss_keys, torch.int64), _ptr(n_miss, torch.int32), _stream(stream)))


def hps_cache_query_dn(handle, keys, n_max, n_dev, out, miss_idx, miss_keys, n_miss, stream=None) -> None:
    _check(load_library().hps_cache_query_dn(
        handle, _ptr(keys, torch.int64), n_max, _ptr(n_dev, torch.int32), _ptr(out, torch.float32),
        _ptr(miss_idx, torch.int32), _ptr(miss_keys, torch.int64), _ptr(n_miss, torch.int32), _stream(stream)))


def hps_cache_insert(handle, keys, vals, n, stream=None) -> None:
    _check(load_library().hps_cache_insert(
        handle, _ptr(keys, torch.int64), _ptr(vals, torch.float32), n, _stream(stream)))


def hps_cache_update(handle, keys, vals, n, stream=None) -> None:
    _check(load_library().hps_cache_update(
        handle, _ptr(keys, torch.int64), _ptr(vals, torch.float32), n, _stream(stream)))


def hps_cache_insert_dn(handle, keys, vals, n_max, n_dev, stream=None) -> None:
    _check(load_library().hps_cache_insert_dn(
        handle, _ptr(keys, torch.int64), _ptr(vals, torch.float32), n_max,
        _ptr(n_dev, torch.int32), _stream(stream)))


def hps_cache_update_dn(handle, keys, vals, n_max, n_dev, stream=None) -> None:
    _check(load_library().hps_cache_update_dn(
        handle, _ptr(keys, torch.int64), _ptr(vals, torch.float32), n_max,
        _ptr(n_dev, torch.int32), _stream(stream)))


def hps_cache_set_concurrent_writers(handle, enabled: bool) -> None:
    _check(load_library().hps_cache_set_concurrent_writers(handle, 1 if enabled else 0))


def hps_cache_set_query_dedup(handle, enabled: bool) -> None:
    _check(load_library().hps_cache_set_query_dedup(handle, 1 if enabled else 0))


def hps_cache_info(handle):
    s, w, d = C.c_uint64(), C.c_uint32(), C.c_uint32()
    _check(load_library().hps_cache_info(handle, C.byref(s), C.byref(w), C.byref(d)))
    return s.value, w.value, d.value


def hps_cache_export(handle, keys, ctr, vals=None, stream=None) -> None:
    _check(load_library().hps_cache_export(
        handle, _ptr(keys, torch.int64), _ptr(ctr, torch.int32), _ptr(vals, torch.float32),
        _stream(stream)))


def hps_cache_import(handle, keys, ctr, vals=None, stream=None) -> None:
    _check(load_library().hps_cache_import(
        handle, _ptr(keys, torch.int64), _ptr(ctr, torch.int32), _ptr(vals, torch.float32),
        _stream(stream)))


def hps_cache_dump(handle, first_slot, n_slots, keys_out, n_out, stream=None) -> None:
    _check(load_library().hps_cache_dump(
        handle, first_slot, n_slots, _ptr(keys_out, torch.int64), _ptr(n_out, torch.int32),
        _stream(stream)))


def hps_cache_query_multi(handles, keys, batch, out, miss_idx, miss_keys, n_miss, stream=None) -> None:
    arr = (C.c_void_p * len(handles))(*handles)
    _check(load_library().hps_cache_query_multi(
        arr, len(handles), _ptr(keys, torch.int64), batch, _ptr(out, torch.float32),
        _ptr(miss_idx, torch.int32), _ptr(miss_keys, torch.int64), _ptr(n_miss, torch.int32),
        _stream(stream)))


def hps_backing_fetch(keys, n, dim, version=0, rows=None, n_dev=None, scatter_idx=None,
                      scatter_out=None, stream=None) -> None:
    _check(load_library().hps_backing_fetch(
        _ptr(keys, torch.int64), n, _ptr(n_dev, torch.int32), dim, version,
        _ptr(rows, torch.float32), _ptr(scatter_idx, torch.int32),
        _ptr(scatter_out, torch.float32), _stream(stream)))


def hps_membench_gather(rows, slot_of, n, dim, out, stream=None) -> None:
    _check(load_library().hps_membench_gather(_ptr(rows, torch.float32), _ptr(slot_of, torch.int32), n, dim,
                                              _ptr(out, torch.float32), _stream(stream)))


def hps_membench_gather_half(rows, slot_of, n, out, reads, stream=None) -> None:
    _check(load_library().hps_membench_gather_half(_ptr(rows, torch.float32), _ptr(slot_of, torch.int32), n,
                                                   _ptr(out, torch.float32), 1 if reads else 0, _stream(stream)))


def hps_membench_copy(src, dst, nbytes, nontemporal=True, stream=None) -> None:
    _check(load_library().hps_membench_copy(_ptr(src), _ptr(dst), nbytes, 1 if nontemporal else 0, _stream(stream)))


def hps_last_error() -> str:
    return load_library().hps_last_error().decode()


def _check_lookup(status):
    if status != HPS_OK:
        raise HpsError(status, load_library().hps_lookup_last_error().decode())


def hps_lookup_last_error() -> str:
    return load_library().hps_lookup_last_error().decode()


def hps_lookup_create(cache, max_batch: int, hit_threshold: float, default_row, fetch, user=None) -> int:
    """default_row: host float32 array of dim values; fetch: a FETCH_FN object, which the caller
    must keep alive as long as the lookup object exists; user: the pointer handed to fetch
    (for hps_hostmap_fetch_fn(): the host map)."""
    import numpy as np
    row = np.ascontiguousarray(default_row, dtype=np.float32)
    h = C.c_void_p()
    _check_lookup(load_library().hps_lookup_create(cache, max_batch, hit_threshold, row.ctypes.data, fetch, user,
                                                   C.byref(h)))
    return h.value


def hps_lookup(lookup, keys, n, out, stream=None):
    """Returns (hit_rate, was_synchronous)."""
    rate, sync = C.c_float(), C.c_int()
    _check_lookup(load_library().hps_lookup(lookup, _ptr(keys, torch.int64), n, _ptr(out, torch.float32),
                                            C.byref(rate), C.byref(sync), _stream(stream)))
    return rate.value, bool(sync.value)


def hps_cache_refresh(cache, batch_slots: int, fetch, user=None, stream=None) -> int:
    """The refresh cycle of Sec. 6 (dump, lower-tier lookup, upload, Update); returns the number
    of keys refreshed."""
    n = C.c_size_t()
    _check_lookup(load_library().hps_cache_refresh(cache, batch_slots, fetch, user, C.byref(n), _stream(stream)))
    return n.value


def hps_refresh_create(cache, batch_slots: int) -> int:
    h = C.c_void_p()
    _check_lookup(load_library().hps_refresh_create(cache, batch_slots, C.byref(h)))
    return h.value


def hps_refresh_run(session, fetch, user=None, stream=None) -> int:
    """One refresh cycle with the session's buffers (nothing is allocated); returns the number of keys refreshed."""
    n = C.c_size_t()
    _check_lookup(load_library().hps_refresh_run(session, fetch, user, C.byref(n), _stream(stream)))
    return n.value


def hps_refresh_destroy(session) -> None:
    _check_lookup(load_library().hps_refresh_destroy(session))


def hps_lookup_drain(lookup) -> None:
    _check_lookup(load_library().hps_lookup_drain(lookup))


def hps_lookup_destroy(lookup) -> None:
    _check_lookup(load_library().hps_lookup_destroy(lookup))


# ---- hps_dedup.h: Q* = dedup(Q) (Sec. 2.2) and the row expansion after the lookup of Q*

def _check_dedup(status):
    if status != HPS_OK:
        raise HpsError(status, load_library().hps_dedup_last_error().decode())


def hps_dedup_last_error() -> str:
    return load_library().hps_dedup_last_error().decode()


def hps_dedup_create(max_n: int) -> int:
    h = C.c_void_p()
    _check_dedup(load_library().hps_dedup_create(max_n, C.byref(h)))
    return h.value


def hps_dedup_destroy(session) -> None:
    _check_dedup(load_library().hps_dedup_destroy(session))


def hps_dedup(session, keys, n, unique_keys, inverse, n_unique, stream=None) -> None:
    _check_dedup(load_library().hps_dedup(
        session, _ptr(keys, torch.int64), n, _ptr(unique_keys, torch.int64), _ptr(inverse, torch.int32),
        _ptr(n_unique, torch.int32), _stream(stream)))


HPS_DEDUP_NOALLOC_MAX = 131072


def hps_dedup_noalloc(keys, n, unique_keys, inverse, n_unique, stream=None) -> None:
    """hps_dedup without a session: the table is a static device array of the library."""
    _check_dedup(load_library().hps_dedup_noalloc(
        _ptr(keys, torch.int64), n, _ptr(unique_keys, torch.int64), _ptr(inverse, torch.int32),
        _ptr(n_unique, torch.int32), _stream(stream)))


def hps_expand_rows(rows, inverse, n, dim, out, stream=None) -> None:
    _check_dedup(load_library().hps_expand_rows(
        _ptr(rows, torch.float32), _ptr(inverse, torch.int32), n, dim, _ptr(out, torch.float32), _stream(stream)))


# ---- hps_hostmap.h: host-memory stand-in for the lower tiers behind Alg. 1 (host numpy arrays)

def _check_hostmap(status, what):
    if status != HPS_OK:
        raise HpsError(status, what)


def hps_hostmap_create(dim: int, partitions: int = 16, reserve: int = 0) -> int:
    h = C.c_void_p()
    _check_hostmap(load_library().hps_hostmap_create(dim, partitions, reserve, C.byref(h)), "hps_hostmap_create")
    return h.value


def hps_hostmap_destroy(m) -> None:
    _check_hostmap(load_library().hps_hostmap_destroy(m), "hps_hostmap_destroy")


def hps_hostmap_put(m, keys, rows) -> None:
    """keys: host int64 numpy array [n]; rows: host float32 numpy array [n, dim] (C-contiguous)."""
    import numpy as np
    keys = np.ascontiguousarray(keys, dtype=np.int64)
    rows = np.ascontiguousarray(rows, dtype=np.float32)
    _check_hostmap(load_library().hps_hostmap_put(m, keys.ctypes.data, rows.ctypes.data, keys.shape[0]), "hps_hostmap_put")


def hps_hostmap_get(m, keys, dim: int):
    """Returns (rows [n, dim] float32, number of keys that were not stored)."""
    import numpy as np
    keys = np.ascontiguousarray(keys, dtype=np.int64)
    rows = np.empty((keys.shape[0], dim), dtype=np.float32)
    absent = C.c_size_t()
    _check_hostmap(load_library().hps_hostmap_get(m, keys.ctypes.data, keys.shape[0], rows.ctypes.data, C.byref(absent)),
                   "hps_hostmap_get")
    return rows, absent.value


def hps_hostmap_stats(m):
    """Returns (keys stored, absent keys served so far)."""
    nk, na = C.c_size_t(), C.c_size_t()
    _check_hostmap(load_library().hps_hostmap_stats(m, C.byref(nk), C.byref(na)), "hps_hostmap_stats")
    return nk.value, na.value


def hps_hostmap_fetch_fn():
    """The library's own hps_hostmap_fetch as a FETCH_FN, to pass to hps_lookup_create together
    with user=<the host map>."""
    return C.cast(load_library().hps_hostmap_fetch, FETCH_FN)


def hps_hostmap_fetch(m, keys, dim: int):
    """Calls the C entry point of that name (the hps_fetch_fn-shaped lookup) on host arrays."""
    import numpy as np
    keys = np.ascontiguousarray(keys, dtype=np.int64)
    rows = np.empty((keys.shape[0], dim), dtype=np.float32)
    load_library().hps_hostmap_fetch(m, keys.ctypes.data, keys.shape[0], rows.ctypes.data)
    return rows
