"""The C ABI called from plain C99 (tests/c_abi_demo.c, built by gcc into a small shared library):
create, insert, query, update, dedup, query with a device-side count and expand, every result
checked on the host by the C code itself."""
import ctypes as C
import os

import pytest

from paper_2210_08804_amd import build as hip_build

pytestmark = pytest.mark.gpu


def test_plain_c_caller_round_trip():
    assert os.path.exists(hip_build.C_DEMO_LIB), "tests/libhps_c_demo.so is not built (run __graft_entry__.build())"
    lib = C.CDLL(hip_build.C_DEMO_LIB)
    lib.hps_c_demo_run.restype = C.c_int
    lib.hps_c_demo_run.argtypes = [C.c_char_p, C.c_size_t]
    msg = C.create_string_buffer(512)
    rc = lib.hps_c_demo_run(msg, len(msg))
    assert rc == 0, f"c_abi_demo.c line {rc}: {msg.value.decode()}"
