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


def test_capacity_check_is_host_arithmetic():
    """What an index of 10^9 vectors holds on the device, and the refusal to plan beyond the memory that is
    available, without touching a GPU."""
    import pytest
    import paper_1102_3828_amd as pkg
    # resident bytes per vector: the m-byte code stream of the scan plus one 32- or 64-byte record
    # (id, list, code, refinement code: m + m' + 8 bytes rounded up to a power of two) for the re-rank
    ib, sb = pkg.memory_required(128, 8192, 8, 8, 10 ** 9)
    assert sb == 0 and 40 * 10 ** 9 < ib < 40.3 * 10 ** 9
    ib32, _ = pkg.memory_required(128, 8192, 8, 32, 10 ** 9)
    assert 72 * 10 ** 9 < ib32 < 72.3 * 10 ** 9
    ib, sb = pkg.memory_required(128, 8192, 8, 8, 10 ** 9, nq=1000, w=64, kprime=1000)
    assert 0.5e9 < sb < 2e9                                         # 512 MB of tables + keys + candidate pool
    pkg.memory_required(128, 8192, 8, 8, 10 ** 9, nq=1000, w=64, kprime=1000, available=288 * 10 ** 9)
    with pytest.raises(pkg.IvfrError) as e:
        pkg.memory_required(128, 8192, 8, 32, 10 ** 9, nq=1000, w=64, kprime=1000, available=64 * 10 ** 9)
    assert e.value.code == pkg.binding.ERR_OOM and "exceed" in str(e.value)
    with pytest.raises(pkg.IvfrError) as e:
        pkg.memory_required(128, 16, 8, 8, 1000, nq=10, w=17, kprime=5)     # w > c
    assert e.value.code == pkg.binding.ERR_INVALID_ARG
