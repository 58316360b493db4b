"""The host-memory stand-in for the lower tiers (include/hps_hostmap.h) against a Python dict:
pure host code, runs without a GPU."""
import ctypes as C
import threading

import numpy as np
import pytest

from paper_2210_08804_amd import binding as B
from paper_2210_08804_amd import inputs


@pytest.mark.parametrize("dim,partitions", [(1, 1), (16, 4), (128, 16), (33, 256)])
def test_put_get_overwrite_and_absent_keys(dim, partitions):
    m = B.hps_hostmap_create(dim, partitions, 1000)
    try:
        rng = np.random.Generator(np.random.PCG64(dim))
        ref = {}
        for rnd in range(6):
            keys = rng.integers(-50000, 50000, size=5000).astype(np.int64)
            rows = rng.standard_normal((5000, dim)).astype(np.float32)
            B.hps_hostmap_put(m, keys, rows)
            for k, r in zip(keys.tolist(), rows):
                ref[k] = r                                        # a key given twice keeps its last row
            q = rng.integers(-60000, 60000, size=7000).astype(np.int64)
            got, absent = B.hps_hostmap_get(m, q, dim)
            exp = np.stack([ref.get(k, np.zeros(dim, np.float32)) for k in q.tolist()])
            assert (got.view(np.uint32) == exp.view(np.uint32)).all()
            assert absent == sum(k not in ref for k in q.tolist())
        n_keys, n_absent = B.hps_hostmap_stats(m)
        assert n_keys == len(ref) and n_absent > 0
        got, absent = B.hps_hostmap_get(m, np.zeros(0, np.int64), dim)
        assert got.shape == (0, dim) and absent == 0
    finally:
        B.hps_hostmap_destroy(m)


def test_fetch_callback_has_the_lower_tier_signature():
    d = 8
    m = B.hps_hostmap_create(d, 8, 0)
    try:
        keys = np.arange(100, dtype=np.int64) * 7
        B.hps_hostmap_put(m, keys, inputs.backing_rows(keys, d))
        fn = B.hps_hostmap_fetch_fn()
        q = np.array([7, 700, 3, 0], dtype=np.int64)              # 700 and 3 are not stored
        out = np.full((4, d), 9.0, dtype=np.float32)
        fn(m, q.ctypes.data_as(C.POINTER(C.c_int64)), 4, out.ctypes.data_as(C.POINTER(C.c_float)))
        assert (out[0] == inputs.backing_rows(q[:1], d)[0]).all() and (out[3] == inputs.backing_rows(q[3:], d)[0]).all()
        assert (out[1] == 0).all() and (out[2] == 0).all()
        assert B.hps_hostmap_stats(m) == (100, 2)
    finally:
        B.hps_hostmap_destroy(m)


def test_concurrent_put_and_get_from_threads():
    d, n = 16, 20000
    m = B.hps_hostmap_create(d, 16, n)
    try:
        keys = np.arange(n, dtype=np.int64)
        rows = inputs.backing_rows(keys, d)
        errors = []

        def writer(lo, hi):
            for a in range(lo, hi, 1000):
                B.hps_hostmap_put(m, keys[a:a + 1000], rows[a:a + 1000])

        def reader():
            for _ in range(20):
                got, _ = B.hps_hostmap_get(m, keys, d)
                stored = (got != 0).any(axis=1)
                if not (got[stored] == rows[stored]).all():        # a stored row is whole, an absent one zero
                    errors.append("torn row")

        threads = [threading.Thread(target=writer, args=(0, n // 2)), threading.Thread(target=writer, args=(n // 2, n)),
                   threading.Thread(target=reader), threading.Thread(target=reader)]
        for t in threads:
            t.start()
        for t in threads:
            t.join()
        assert not errors
        got, absent = B.hps_hostmap_get(m, keys, d)
        assert absent == 0 and (got == rows).all()
    finally:
        B.hps_hostmap_destroy(m)


def test_bad_arguments():
    lib = B.load_library()
    h = C.c_void_p()
    assert lib.hps_hostmap_create(0, 4, 0, C.byref(h)) == -1
    assert lib.hps_hostmap_create(8, 3, 0, C.byref(h)) == -1
    assert lib.hps_hostmap_create(8, 512, 0, C.byref(h)) == -1
    assert lib.hps_hostmap_create(8, 4, 0, None) == -1
    assert lib.hps_hostmap_destroy(None) == -1 and lib.hps_hostmap_put(None, None, None, 1) == -1
    assert lib.hps_hostmap_get(None, None, 1, None, None) == -1
