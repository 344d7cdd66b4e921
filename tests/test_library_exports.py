"""CPU-only: the C-ABI library loads and exports every symbol declared in include/inshr.h."""
import os
import re

from paper_2306_11800_amd import api

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "inshr.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(inshr_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    lib = api.load_library()
    names = declared_functions()
    assert set(names) == set(api.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_bounds_and_errors_without_gpu():
    import ctypes as C
    lib = api.load_library()
    words, cap = C.c_uint64(), C.c_uint64()
    cfg = api.CConfig(4, 0, 100000, 1000)
    assert lib.inshr_quantize_bound(1000003, C.byref(cfg), C.byref(words), C.byref(cap)) == 0
    assert words.value == (1000003 * 5 + 63) // 64 and cap.value == 1000
    bad = api.CConfig(9, 0, 0, 0)
    assert lib.inshr_quantize_bound(10, C.byref(bad), C.byref(words), C.byref(cap)) == -2
    bad = api.CConfig(4, 0, 600000, 400000)
    assert lib.inshr_quantize_bound(10, C.byref(bad), C.byref(words), C.byref(cap)) == -2
    p = api.CCodes(None, 5, 4, 0, 100)
    c = api.CCodes(None, 9, 8, 0, 100)
    assert lib.inshr_delta_bound(C.byref(p), C.byref(c), C.byref(words)) == 0
    assert words.value == (100 * 9 + 63) // 64
    c2 = api.CCodes(None, 9, 8, 0, 101)
    assert lib.inshr_delta_bound(C.byref(p), C.byref(c2), C.byref(words)) == -5
    assert lib.inshr_strerror(-3).decode().lower().startswith("nan")
