"""The C-ABI library builds, loads and exports every symbol the header declares (no GPU, no compute calls)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2410_03348_amd", "libdolphin_hip.so")


def declared_functions():
    names = set()
    inc = os.path.join(ROOT, "include")
    for fn in os.listdir(inc):
        if fn.endswith(".h"):
            text = open(os.path.join(inc, fn)).read()
            text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
            names.update(re.findall(r"\b(dol_[a-z0-9_]+)\s*\(", text))
    return sorted(names)


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        import __graft_entry__ as g
        g.build()
    return ctypes.CDLL(LIB)


def test_header_declares_the_operator_calls():
    names = declared_functions()
    for need in ("dol_apply2", "dol_filter", "dol_union", "dol_backward", "dol_fn_table_create_dense",
                 "dol_fn_table_create_sparse", "dol_filter_plan", "dol_union_plan", "dol_dtkp_init", "dol_last_error"):
        assert need in names


def test_library_exports_every_declared_symbol(lib):
    for name in declared_functions():
        assert hasattr(lib, name), name


def test_version_and_error_string(lib):
    lib.dol_version.restype = ctypes.c_char_p
    lib.dol_last_error.restype = ctypes.c_char_p
    assert re.match(rb"\d+\.\d+\.\d+", lib.dol_version())
    assert isinstance(lib.dol_last_error(), bytes)


def test_host_side_plans_need_no_gpu(lib):
    """dol_filter_plan / dol_union_plan are pure host logic; check them against the paper's examples."""
    class Dist(ctypes.Structure):
        _fields_ = [("batch", ctypes.c_int32), ("n_sym", ctypes.c_int32), ("ld", ctypes.c_int64),
                    ("sym_ids", ctypes.POINTER(ctypes.c_int32)), ("prob", ctypes.c_void_p),
                    ("proof_mask", ctypes.c_void_p), ("proof_prob", ctypes.c_void_p)]

    def dist(ids):
        arr = (ctypes.c_int32 * len(ids))(*ids)
        return Dist(0, len(ids), len(ids), arr, None, None, None), arr

    d, keep_d = dist(list(range(10)))
    pred = (ctypes.c_uint8 * 10)(*[1 if i % 2 == 0 else 0 for i in range(10)])
    n = ctypes.c_int32()
    out = (ctypes.c_int32 * 10)()
    assert lib.dol_filter_plan(ctypes.byref(d), pred, ctypes.byref(n), out) == 0
    assert n.value == 5 and list(out[:5]) == [0, 2, 4, 6, 8]          # Ex. 3.3
    a, keep_a = dist([0, 1])
    b, keep_b = dist([0, 4])
    out2 = (ctypes.c_int32 * 4)()
    assert lib.dol_union_plan(ctypes.byref(a), ctypes.byref(b), ctypes.byref(n), out2) == 0
    assert n.value == 3 and list(out2[:3]) == [0, 1, 4]               # union example of Sec. 3.1.2
    bad, keep_bad = dist([3, 3])
    assert lib.dol_union_plan(ctypes.byref(bad), ctypes.byref(b), ctypes.byref(n), out2) == 1   # DOL_EINVAL
    lib.dol_last_error.restype = ctypes.c_char_p
    assert b"ascending" in lib.dol_last_error()


def test_binding_refuses_to_import_without_the_library(tmp_path, monkeypatch):
    """The product path has no CPU fallback: a missing shared library is an ImportError."""
    import importlib.util
    src = os.path.join(ROOT, "paper_2410_03348_amd", "binding.py")
    dst = tmp_path / "binding_copy.py"
    dst.write_text(open(src).read())
    spec = importlib.util.spec_from_file_location("binding_copy", str(dst))
    mod = importlib.util.module_from_spec(spec)
    with pytest.raises(ImportError):
        spec.loader.exec_module(mod)
