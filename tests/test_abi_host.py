"""Host-side checks of the C ABI: the library loads and exports every symbol the header declares (no compute)."""
import ctypes
import os
import re

import paper_2307_12059_amd as kgc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "kgc.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(kgc_[a-z0-9_]+)\s*\(", text)))


def test_header_symbols_are_exported():
    lib = kgc.load_library()
    names = _declared()
    assert set(names) == set(kgc.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_version_and_struct_sizes():
    assert re.fullmatch(r"\d+\.\d+\.\d+", kgc.kgc_version())
    assert ctypes.sizeof(kgc.kgc_triple) == 16
    assert ctypes.sizeof(kgc.kgc_config) == 56
    assert ctypes.sizeof(kgc.kgc_stats) == 112


def test_null_arguments_are_rejected_without_a_device():
    lib = kgc.load_library()
    assert lib.kgc_create(None, None) == kgc.KGC_E_INVALID
    bad = kgc.kgc_config(); bad.dtype = 7
    out = ctypes.c_void_p()
    assert lib.kgc_create(ctypes.byref(bad), ctypes.byref(out)) == kgc.KGC_E_INVALID and not out.value
    cnt = ctypes.c_uint64(5)
    assert lib.kgc_join(None, None, 0, 1, None, 0, 2, 1.0, None, 0, ctypes.byref(cnt)) == kgc.KGC_E_INVALID
    lib.kgc_destroy(None)
    assert kgc.kgc_last_error(None) == "null handle"
