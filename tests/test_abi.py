"""CPU-only checks of the boundary: the shared library loads and exports every function that
include/llma.h declares, the binding lists the same names, and argument errors that are
detected before any device work come back as negative codes (no GPU needed for those)."""
import ctypes
import os
import re

import pytest

import paper_2304_04487_amd as llma

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "llma.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(llma_[a-z_]+)\s*\(", text)))


def test_header_declares_the_three_calls_of_the_method():
    names = _declared()
    for must in ("llma_find_trigger", "llma_verify_step", "llma_generate"):
        assert must in names


def test_library_exports_every_declared_symbol():
    if not os.path.exists(llma.LIB_PATH):
        pytest.fail("libllma.so not built: run __graft_entry__.build()")
    lib = ctypes.CDLL(llma.LIB_PATH)
    for name in _declared():
        assert hasattr(lib, name), f"{name} declared in llma.h but not exported"
    assert sorted(llma.EXPORTS) == _declared()


def test_argument_errors_without_device_work():
    lib = llma.load_library()
    doc, pos = ctypes.c_int32(), ctypes.c_int32()
    i32p = ctypes.POINTER(ctypes.c_int32)
    offs = (ctypes.c_int32 * 2)(0, 0)
    y = (ctypes.c_int32 * 2)(1, 2)
    null = ctypes.cast(None, i32p)
    assert lib.llma_find_trigger(y, 2, null, offs, 1, 0, ctypes.byref(doc), ctypes.byref(pos)) == llma.LLMA_E_INVAL   # n < 1
    assert b"n must be" in lib.llma_last_error(None)
    assert lib.llma_find_trigger(y, 2, null, null, 1, 1, ctypes.byref(doc), ctypes.byref(pos)) == llma.LLMA_E_INVAL  # null offsets
    bad = (ctypes.c_int32 * 3)(0, 5, 3)
    assert lib.llma_find_trigger(y, 2, y, bad, 2, 1, ctypes.byref(doc), ctypes.byref(pos)) == llma.LLMA_E_INVAL       # decreasing
    # empty reference / tail longer than y: no device work, plain "no match"
    assert lib.llma_find_trigger(y, 2, null, offs, 1, 1, ctypes.byref(doc), ctypes.byref(pos)) == 0
    assert (doc.value, pos.value) == (-1, -1)
    assert lib.llma_find_trigger(y, 2, y, (ctypes.c_int32 * 2)(0, 2), 1, 3, ctypes.byref(doc), ctypes.byref(pos)) == 0
    # context calls with a null context
    assert lib.llma_reset(None, 0) == llma.LLMA_E_INVAL
    assert lib.llma_verify_step(None, 0, null, 0, null, null, null) == llma.LLMA_E_INVAL
    assert lib.llma_destroy(None) == llma.LLMA_OK
    # llma_create rejects bad shapes before touching the device
    cfg = llma.ModelCfgC(2, 128, 4, 31, 512, 512, 128, 1, 4, llma.LLMA_DTYPE_F32, 0, 1e-6, 10000.0)
    w = llma.WeightsC()
    h = ctypes.c_void_p()
    assert lib.llma_create(ctypes.byref(cfg), ctypes.byref(w), None, ctypes.byref(h)) == llma.LLMA_E_INVAL
    cfg = llma.ModelCfgC(2, 128, 4, 32, 512, 512, 128, 1, 33, llma.LLMA_DTYPE_F32, 0, 1e-6, 10000.0)
    assert lib.llma_create(ctypes.byref(cfg), ctypes.byref(w), None, ctypes.byref(h)) == llma.LLMA_E_INVAL
    cfg = llma.ModelCfgC(2, 128, 4, 32, 512, 512, 128, 1, 4, llma.LLMA_DTYPE_F32, 0, 1e-6, 10000.0)
    assert lib.llma_create(ctypes.byref(cfg), ctypes.byref(w), None, ctypes.byref(h)) == llma.LLMA_E_INVAL  # null weights
    assert not h.value
