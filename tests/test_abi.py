"""The C-ABI library loads and exports every entry point its header declares (no GPU needed)."""
import ctypes
import os
import re

from paper_2112_07221_amd import hetcache as hc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_entry_points():
    text = open(os.path.join(ROOT, "include", "het_cache.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(het_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_entry_points()
    assert "het_lookup" in names and "het_update" in names and "het_flush" in names
    assert sorted(hc.EXPORTS) == names
    lib = ctypes.CDLL(hc.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), n


def test_argument_errors_need_no_gpu():
    lib = hc.load()
    h = ctypes.c_void_p()
    assert lib.het_cache_create(None, 10, 4, 1, 0) == hc.HET_EINVAL
    assert lib.het_cache_create(ctypes.byref(h), 0, 4, 1, 0) == hc.HET_EINVAL
    assert lib.het_cache_create(ctypes.byref(h), 10, 0, 1, 0) == hc.HET_EINVAL
    assert lib.het_cache_create(ctypes.byref(h), 10, 4, -1, 0) == hc.HET_EINVAL
    assert lib.het_cache_create(ctypes.byref(h), 10, 4, 1, 7) == hc.HET_EINVAL
    assert lib.het_cache_create(ctypes.byref(h), 10, 4, hc.S_INFINITE, 1) == hc.HET_OK
    # not configured yet: every data call is refused
    assert lib.het_lookup(h, None, 4, None) == hc.HET_EINVAL
    assert lib.het_update(h, None, None, 4, 0.1) == hc.HET_EINVAL
    assert lib.het_flush(h) == hc.HET_EINVAL
    assert lib.het_cache_destroy(h) == hc.HET_OK
    assert lib.het_cache_destroy(None) == hc.HET_OK
    assert hc.strerror(hc.HET_ESTATE) and hc.strerror(-99) == "unknown status"
