"""The C-ABI library loads without a GPU and exports every function the header declares."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "ivfadcr.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ivfr_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    import paper_1102_3828_amd as pkg
    names = _declared()
    assert "ivfr_search" in names and "ivfr_create" in names and len(names) >= 15
    lib = ctypes.CDLL(pkg.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(pkg.EXPORTED) == names


def test_synth_library_loads():
    lib = ctypes.CDLL(os.path.join(ROOT, "synthdata", "libsynthgen.so"))
    assert hasattr(lib, "synth_generate")


def test_argument_errors_need_no_gpu():
    import paper_1102_3828_amd as pkg
    h = ctypes.c_void_p()
    p = pkg.binding.Params(127, 16, 8, 8, 0)
    assert pkg.lib.ivfr_create(ctypes.byref(p), ctypes.byref(h)) == pkg.binding.ERR_INVALID_ARG
    assert b"multiple of 8" in pkg.lib.ivfr_last_error()
    p = pkg.binding.Params(128, 16, 7, 8, 0)
    assert pkg.lib.ivfr_create(ctypes.byref(p), ctypes.byref(h)) == pkg.binding.ERR_INVALID_ARG
    p = pkg.binding.Params(128, 16, 8, 24, 0)   # 128 % 24 != 0
    assert pkg.lib.ivfr_create(ctypes.byref(p), ctypes.byref(h)) == pkg.binding.ERR_INVALID_ARG
    assert pkg.lib.ivfr_create(None, ctypes.byref(h)) == pkg.binding.ERR_INVALID_ARG
    assert pkg.lib.ivfr_ntotal(None) == pkg.binding.ERR_INVALID_ARG
