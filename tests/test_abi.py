"""The C-ABI library loads, exports every function the header declares, and rejects bad
arguments before touching the GPU.  No kernel is launched here."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADERS = sorted(os.path.join(ROOT, "include", f) for f in os.listdir(os.path.join(ROOT, "include"))
                 if f.endswith(".h"))


def declared_functions():
    names = set()
    for header in HEADERS:
        text = open(header).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(hps_[a-z_]+)\s*\(", text))
    return sorted(names - {"hps_fetch_fn"})


@pytest.fixture(scope="module")
def lib():
    from paper_2210_08804_amd import binding
    return binding.load_library()


def test_header_and_binding_list_the_same_entry_points():
    from paper_2210_08804_amd import binding
    assert declared_functions() == sorted(binding.EXPORTS)
    for name in binding.EXPORTS:
        assert callable(getattr(binding, name))


def test_library_exports_every_declared_symbol(lib):
    names = declared_functions()
    assert {"hps_cache_create", "hps_cache_query", "hps_cache_insert", "hps_cache_update",
            "hps_cache_destroy"} <= set(names)
    for name in names:
        assert hasattr(lib, name), name


def test_bad_arguments_are_rejected_on_the_host(lib):
    h = C.c_void_p()
    bad = [(0, 8, 128), (64, 3, 128), (64, 128, 128), (60, 8, 128), (64, 8, 0), (64, 8, 6),
           ((1 << 31) * 8, 8, 4)]
    for cap, ways, dim in bad:
        assert lib.hps_cache_create(cap, ways, dim, C.byref(h)) == -1
        assert h.value is None
        assert len(lib.hps_last_error()) > 0
    assert lib.hps_cache_create(64, 8, 128, None) == -1
    assert lib.hps_cache_destroy(None) == -1
    assert lib.hps_cache_info(None, None, None, None) == -1
    assert lib.hps_cache_set_concurrent_writers(None, 1) == -1
    assert lib.hps_cache_set_query_dedup(None, 1) == -1
    assert lib.hps_cache_query_multi(None, 0, None, 0, None, None, None, None, None) == -1
    assert lib.hps_backing_fetch(None, 5, None, 6, 0, None, None, None, None) == -1
    assert lib.hps_backing_fetch(None, 5, None, 8, 0, None, None, None, None) == -1   # keys NULL
    assert lib.hps_cache_query_dn(None, None, 0, None, None, None, None, None, None) == -1
    assert lib.hps_lookup(None, None, 0, None, None, None, None) == -1
    from paper_2210_08804_amd import binding
    assert lib.hps_cache_refresh(None, 10, binding.FETCH_FN(), None, None, None) == -1
    assert lib.hps_lookup_drain(None) == -1 and lib.hps_lookup_destroy(None) == -1
    assert len(lib.hps_lookup_last_error()) > 0
    assert lib.hps_dedup_create(0, C.byref(h)) == -1 and lib.hps_dedup_create(1 << 31, C.byref(h)) == -1
    assert lib.hps_dedup_create(16, None) == -1 and lib.hps_dedup_destroy(None) == 0
    assert lib.hps_dedup(None, None, 0, None, None, None, None) == -1
    assert lib.hps_expand_rows(None, None, 5, 6, None, None) == -1       # dim not a multiple of 4
    assert lib.hps_expand_rows(None, None, 5, 8, None, None) == -1       # NULL pointers
    assert lib.hps_expand_rows(None, None, 0, 8, None, None) == 0        # nothing to do
    assert len(lib.hps_dedup_last_error()) > 0


def test_binding_fails_loudly_without_the_library(monkeypatch, tmp_path):
    from paper_2210_08804_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", str(tmp_path / "missing.so"))
    with pytest.raises(RuntimeError, match="no CPU fallback"):
        binding.hps_cache_create(64, 8, 128)


def test_headers_are_plain_c(tmp_path):
    """The boundary is a C ABI: both headers must compile as C99 with no HIP or C++ in sight."""
    import subprocess
    src = tmp_path / "use.c"
    src.write_text('#include "hps_lookup.h"\n#include "hps_dedup.h"\n#include "hps_hostmap.h"\n#include "hps_cache.h"\n'
                   "int main(void) { hps_cache_t *c = 0; hps_lookup_t *l = 0; (void)c; (void)l; return HPS_OK; }\n")
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-fsyntax-only",
                    "-I", os.path.join(ROOT, "include"), str(src)], check=True)
