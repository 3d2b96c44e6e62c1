"""The C-ABI library loads without a GPU and exports every symbol include/layoutcopy.h declares."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "layoutcopy.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(lc_[a-z0-9_]+)\s*\(", text)))


def test_header_symbols_are_exported():
    from paper_2603_02298_amd import build
    assert os.path.exists(build.LIB_PATH), "build the library first (python -m paper_2603_02298_amd.build)"
    lib = ctypes.CDLL(build.LIB_PATH)
    names = _declared()
    assert len(names) >= 28, names
    for n in names:
        assert hasattr(lib, n), "missing export: " + n


def test_status_strings_and_dtypes():
    import paper_2603_02298_amd as lc
    L = lc.lib()
    seen = set()
    for code in range(20):
        s = L.lc_status_string(code).decode()
        assert s != "UNKNOWN" and s not in seen
        seen.add(s)
    assert L.lc_status_string(99).decode() == "UNKNOWN"
    assert [L.lc_dtype_bytes(i) for i in range(8)] == [4, 2, 2, 1, 2, 4, 8, 16] and L.lc_dtype_bytes(42) == 0


def test_null_arguments_are_errors_not_crashes():
    import paper_2603_02298_amd as lc
    L = lc.lib()
    h = ctypes.c_void_p()
    assert L.lc_layout_parse(None, ctypes.byref(h)) == 1
    assert L.lc_coalesce(None, ctypes.byref(h)) == 1
    assert L.lc_composition(None, None, ctypes.byref(h)) == 1
    assert L.lc_plan_create(None, None, 0, 256, 256, ctypes.byref(h)) == 1
    assert L.lc_plan_execute(None, None, None, None) == 1
    a = lc.Layout("8:1")
    assert L.lc_copy(None, a._h, None, a._h, 0, None) == 1
    assert L.lc_plan_create(a._h, a._h, 42, 256, 256, ctypes.byref(h)) == 13
    assert L.lc_plan_create(a._h, a._h, 0, 3, 256, ctypes.byref(h)) == 1      # alignment not a power of two
    k = ctypes.c_int64()
    assert L.lc_max_common_vector(a._h, lc.Layout("9:1")._h, ctypes.byref(k)) == 6
