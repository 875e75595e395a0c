"""The C-ABI library loads and exports every symbol include/rv.h declares (no compute)."""
import ctypes
import os
import re

from paper_2401_01728_amd import _lib

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared(header="rv.h"):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(rv_[a-z0-9_]+)\s*\(", text)))


def test_header_and_binding_agree():
    assert _declared() == sorted(_lib.SYMBOLS)
    assert _declared("rv_kernels.h") == sorted(_lib.KERNEL_SYMBOLS)


def test_library_exports_every_symbol():
    lib = _lib.lib()
    for name in _declared() + _declared("rv_kernels.h"):
        assert getattr(lib, name) is not None


def test_argument_validation_needs_no_device():
    lib = _lib.lib()
    INVAL = -1
    assert lib.rv_cluster_average(None, 2, 8, 1, None, 1, None, 0, 0.0, None) == INVAL
    arr = (ctypes.c_void_p * 2)(16, 32)
    assert lib.rv_cluster_average(arr, 0, 8, 1, None, 1, None, 0, 0.0, None) == INVAL     # C < 1
    assert lib.rv_cluster_average(arr, 2, 8, 0, None, 1, None, 0, 0.0, None) == INVAL     # R < 1
    assert lib.rv_cluster_average(arr, 2, 0, 1, None, 1, None, 0, 0.0, None) == INVAL     # n == 0
    assert lib.rv_cluster_average(arr, 2, 8, 1, None, 0, None, 0, 0.0, None) == INVAL     # no output
    assert lib.rv_cluster_average(arr, 2, 8, 1, None, 1, 64, 2, 0.0, None) == INVAL       # grad_replica
    same = (ctypes.c_void_p * 2)(16, 16)
    assert lib.rv_cluster_average(same, 2, 8, 1, None, 1, None, 0, 0.0, None) == INVAL    # aliasing
    assert lib.rv_block_update(None, 16, 4, 0.1, None, None) == INVAL
    assert lib.rv_stage_create(None, None) == INVAL
    dims = (ctypes.c_int64 * 3)(4, 0, 3)
    d = _lib.StageDesc(0, 0, 2, dims, 8, 1, 0.1, 1e-5, None)
    h = ctypes.c_void_p()
    assert lib.rv_stage_create(ctypes.byref(d), ctypes.byref(h)) == INVAL                 # zero width
    d = _lib.StageDesc(0, 1, 2, dims, 8, 1, 0.1, 1e-5, None)
    assert lib.rv_stage_create(ctypes.byref(d), ctypes.byref(h)) == INVAL                 # MLP must be fp32
    d = _lib.StageDesc(0, 0, 2, dims, 8, -1, 0.1, 1e-5, None)
    assert lib.rv_stage_create(ctypes.byref(d), ctypes.byref(h)) == INVAL                 # tau < 0
    assert lib.rv_stage_num_params(None) == 0
    assert lib.rv_strerror(-2).decode().startswith("tau+1")
