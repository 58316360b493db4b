"""Error returns of the C ABI on a live device, and the bounded waits: a set whose sequence word is
left odd (as by a writer whose kernel died) must not hang anybody; kernels give up after a
bounded number of rounds, raise HPS_FLAG_STUCK_SET and exit normally.  The condition is forced
from the host through the test hook; no kernel is made to fault or spin without bound."""
import ctypes as C

import numpy as np
import pytest
import torch

from oracle import OracleCache
from paper_2210_08804_amd import binding as B
from paper_2210_08804_amd import inputs
from harness import DeviceCache, SENTINEL

pytestmark = pytest.mark.gpu


def test_argument_errors_on_a_live_cache():
    lib = B.load_library()
    with DeviceCache(64, 8, 16) as gc:
        n = 32
        keys = torch.zeros(n + 1, dtype=torch.int64, device="cuda")
        out = torch.zeros(n + 1, 16, dtype=torch.float32, device="cuda")
        mi = torch.zeros(n + 1, dtype=torch.int32, device="cuda")
        mk = torch.zeros(n + 1, dtype=torch.int64, device="cuda")
        nm = torch.zeros(2, dtype=torch.int32, device="cuda")
        st = torch.cuda.current_stream().cuda_stream
        ok = (gc.h, keys.data_ptr(), n, out.data_ptr(), mi.data_ptr(), mk.data_ptr(), nm.data_ptr(), st)
        assert lib.hps_cache_query(*ok) == 0
        bad = [
            (None,) + ok[1:],                                            # null handle
            ok[:1] + (None,) + ok[2:],                                   # null keys with n > 0
            ok[:3] + (out.data_ptr() + 4,) + ok[4:],                     # out not 16-byte aligned
            ok[:1] + (keys.data_ptr() + 4,) + ok[2:],                    # keys not 8-byte aligned
            ok[:6] + (None, st),                                         # n_miss null
            ok[:2] + (1 << 32,) + ok[3:],                                # n too large
        ]
        for args in bad:
            assert lib.hps_cache_query(*args) == B.HPS_ERR_INVALID_ARG
            assert len(B.hps_last_error()) > 0
        assert lib.hps_cache_insert(gc.h, keys.data_ptr(), out.data_ptr() + 8, n, st) == B.HPS_ERR_INVALID_ARG
        assert lib.hps_cache_update(gc.h, None, out.data_ptr(), n, st) == B.HPS_ERR_INVALID_ARG
        assert lib.hps_cache_dump(gc.h, 60, 8, mk.data_ptr(), nm.data_ptr(), st) == B.HPS_ERR_INVALID_ARG
        assert lib.hps_cache_debug_set_seq(gc.h, 8, 1) == B.HPS_ERR_INVALID_ARG       # only 8 sets
        # tables of one multi-table call must agree in dim and ways
        with DeviceCache(64, 4, 16) as other:
            arr = (C.c_void_p * 2)(gc.h, other.h)
            assert lib.hps_cache_query_multi(arr, 2, keys.data_ptr(), 8, out.data_ptr(), mi.data_ptr(),
                                             mk.data_ptr(), nm.data_ptr(), st) == B.HPS_ERR_INVALID_ARG
        torch.cuda.synchronize()
        assert B.hps_cache_flags(gc.h) == 0


def test_a_set_that_is_never_released_cannot_hang_a_kernel():
    S, W, d = 16, 8, 16
    with DeviceCache(S * W, W, d, concurrent_writers=True) as gc:
        oc = OracleCache(S * W, W, d)
        keys = np.arange(60, dtype=np.int64)
        rows = inputs.backing_rows(keys, d)
        gc.insert(keys, rows)
        oc.load_state(*gc.export())
        stuck = oc.set_of(int(keys[0]))
        in_stuck = np.array([oc.set_of(int(k)) == stuck for k in keys])
        assert in_stuck.any() and (~in_stuck).any()
        B.hps_cache_debug_set_seq(gc.h, stuck, 1)                        # "a writer died holding this set"

        out, mi, mk = gc.query(keys)                                      # checked variant: bounded wait, then misses
        resident = np.isin(keys, oc.dump())
        exp_miss = np.nonzero(in_stuck | ~resident)[0]
        assert mi.tolist() == exp_miss.tolist()
        assert (out[in_stuck] == SENTINEL).all()
        hit = ~in_stuck & resident
        assert (out[hit] == rows.view(np.uint32)[hit]).all()
        assert B.hps_cache_flags(gc.h, clear=True) == B.HPS_FLAG_STUCK_SET
        assert B.hps_cache_flags(gc.h) == 0

        new_rows = inputs.backing_rows(keys, d, 1)
        gc.update(keys, new_rows)                                         # keys of the stuck set are skipped
        assert B.hps_cache_flags(gc.h, clear=True) == B.HPS_FLAG_STUCK_SET
        more = np.arange(1000, 1040, dtype=np.int64)
        gc.insert(more, inputs.backing_rows(more, d))                     # likewise
        more_stuck = np.array([oc.set_of(int(k)) == stuck for k in more])
        assert (B.hps_cache_flags(gc.h, clear=True) == B.HPS_FLAG_STUCK_SET) == bool(more_stuck.any())

        B.hps_cache_debug_set_seq(gc.h, stuck, 2)                         # released: everything works again
        gk, _, _ = gc.export()
        assert not np.isin(more[more_stuck], gk).any()                    # inserts into the stuck set were skipped
        resident = np.isin(keys, gk)                                      # (the other inserts may have evicted a few keys)
        out, mi, _ = gc.query(keys)
        assert mi.tolist() == np.nonzero(~resident)[0].tolist()
        assert (out[resident & ~in_stuck] == new_rows.view(np.uint32)[resident & ~in_stuck]).all()
        assert (out[resident & in_stuck] == rows.view(np.uint32)[resident & in_stuck]).all()   # those updates were skipped
        assert B.hps_cache_flags(gc.h) == 0


def test_create_reports_out_of_memory_and_recovers():
    lib = B.load_library()
    h = C.c_void_p()
    # 2^33 slots of 512 bytes = 4 TiB of rows: more than the device has
    assert lib.hps_cache_create(1 << 33, 8, 128, C.byref(h)) == B.HPS_ERR_OOM
    assert h.value is None and "hps_cache_create" in B.hps_last_error()
    with DeviceCache(1 << 12, 8, 128) as gc:                 # the device is still usable afterwards
        keys = np.arange(100, dtype=np.int64)
        gc.insert(keys, inputs.backing_rows(keys, 128))
        out, mi, _ = gc.query(keys)
        assert mi.size == 0 and (out == inputs.backing_rows(keys, 128).view(np.uint32)).all()


def test_rows_too_long_to_validate_in_one_piece_cannot_overlap_writers():
    """A query that overlaps writers stages a long row whole before it stores it; that is built for
    rows of up to 4 KiB.  Longer rows: the cache starts in the no-overlap mode, switching the
    validation on is refused, and the Alg. 1 object (whose background inserts overlap queries)
    cannot be created on it.  Plain queries work."""
    import numpy as np
    from paper_2210_08804_amd import inputs
    d = 1028
    with DeviceCache(64, 8, d, concurrent_writers=False) as gc:
        with pytest.raises(B.HpsError) as e:
            B.hps_cache_set_concurrent_writers(gc.h, True)
        assert e.value.status == B.HPS_ERR_INVALID_ARG and "dim" in str(e.value)
        keys = np.arange(40, dtype=np.int64)
        gc.insert(keys, inputs.backing_rows(keys, d))
        out, mi, _ = gc.query(keys)
        hit = np.ones(40, dtype=bool)
        hit[mi] = False
        assert hit.sum() >= 30 and (out[hit] == inputs.backing_rows(keys, d).view(np.uint32)[hit]).all()
    with DeviceCache(64, 8, 1024, concurrent_writers=True):
        pass                                                 # 4 KiB rows are fine
