"""The C-ABI library on a machine without a GPU: it loads, exports every declared symbol, and
rejects bad arguments before touching HIP.  No compute call is made here."""
import ctypes
import os
import re

import pytest

from paper_1903_03640_amd import redux

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

pytestmark = pytest.mark.skipif(not os.path.exists(redux.LIB_PATH), reason="libredux.so not built (run __graft_entry__.build())")


def test_every_declared_symbol_is_exported():
    header = open(os.path.join(ROOT, "include", "redux.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(redux_[a-z0-9_]+)\s*\(", header))
    assert declared == set(redux.SYMBOLS)
    lib = ctypes.CDLL(redux.LIB_PATH)
    for name in declared:
        assert hasattr(lib, name), name


def test_argument_errors_come_before_any_hip_call():
    lib = redux.load()
    buf = (ctypes.c_char * 64)()
    p = ctypes.addressof(buf)
    p16 = (p + 15) & ~15
    assert redux.sum_raw(0, 8, redux.F16, p16, 0) == -1            # x NULL, n > 0
    assert redux.sum_raw(p16, 8, redux.F16, 0, 0) == -1            # out NULL
    assert redux.sum_raw(p16, 8, 7, p16 + 32, 0) == -2             # unknown dtype
    assert redux.sum_raw(p16 + 1, 8, redux.F16, p16 + 32, 0) == -4 # x not 2-byte aligned
    assert redux.sum_raw(p16, 4, redux.F16, p16 + 34, 0) == -4     # out not 4-byte aligned
    assert redux.sum_raw(p16, 4, redux.I8, p16 + 36, 0) == -4      # out not 8-byte aligned
    assert redux.sum_raw(p16, 8, redux.F16, p16 + 8, 0) == -7      # out inside the input
    assert redux.sum_raw(p16, 1 << 63, redux.I8, p16 + 32, 0) == -3
    assert redux.sum_segmented_raw(p16, 1 << 40, 1 << 40, redux.F16, p16 + 32, 0) == -3
    assert redux.sum_segmented_raw(0, 4, 4, redux.F16, p16, 0) == -1
    assert redux.sum_segmented_raw(p16, 4, 4, 9, p16 + 32, 0) == -2
    assert redux.sum_segmented_raw(0, 0, 0, redux.F16, 0, 0) == 0  # no segments: a no-op, nothing launched
    assert redux.sum_segmented_raw(0, 0, 5, redux.I8, 0, 0) == 0
    assert redux.sum_multipass_raw(p16, 8, redux.BF16, p16 + 32, 0)[0] == -2   # this form: binary16 / int8 only
    assert redux.sum_raw(p16 + 2, 4, redux.F32, p16 + 32, 0) == -4             # binary32 input not 4-byte aligned
    assert redux.mma_group_probe_raw(p16, 513, redux.F16, p16, p16, 0) == -3
    assert redux.mma_group_probe_raw(p16, 1025, redux.I8, p16, p16, 0) == -3
    assert redux.mma_group_probe_raw(0, 4, redux.F16, p16, p16, 0) == -1
    assert lib.redux_strerror(-4).decode().startswith("pointer not aligned")
    assert "unknown" in lib.redux_strerror(-99).decode()


def test_settings():
    old = redux.get_variant()
    try:
        redux.set_variant("classic")
        assert redux.get_variant() == 2
        redux.set_variant("mfma")
        assert redux.get_variant() == 1
        with pytest.raises(redux.ReduxError):
            redux.set_variant(9)
    finally:
        redux.set_variant(old)
    assert redux.get_param("max_chain") >= 1
    keep = redux.get_param("unroll")
    redux.set_param("unroll", 4)
    assert redux.get_param("unroll") == 4
    redux.set_param("unroll", keep)
    for bad in (("unroll", 3), ("unroll", 16), ("blocks_per_cu", 0), ("nontemporal", 2), ("no_such_param", 1), ("max_chain", 1 << 20)):
        with pytest.raises(redux.ReduxError):
            redux.set_param(*bad)
    assert redux.get_param("no_such_param") < -(1 << 40)
    assert "gfx950" in redux.version()


def test_resolved_variant_without_a_gpu():
    """What 'auto' resolves to: the MMA family, except the 8-bit floats (classic everywhere: their MFMAs drop bits) and
    binary32 (classic: measured faster); an explicit setting wins; unknown dtypes are an error."""
    redux.set_variant("auto")
    for dt in (redux.F16, redux.I8, redux.BF16):
        assert redux.resolved_variant(dt, segmented=False) == "mfma"
    for dt in (redux.F32, redux.F8E4M3, redux.F8E5M2):
        assert redux.resolved_variant(dt, segmented=False) == "classic"
    for dt in (redux.F16, redux.I8, redux.BF16):
        assert redux.resolved_variant(dt, segmented=True) == "mfma"
    for dt in (redux.F32, redux.F8E4M3, redux.F8E5M2):
        assert redux.resolved_variant(dt, segmented=True) == "classic"
    for v in ("mfma", "classic"):
        redux.set_variant(v)
        assert redux.resolved_variant(redux.F8E4M3, segmented=True) == v and redux.resolved_variant(redux.F16, segmented=False) == v
    redux.set_variant("auto")
    assert redux.load().redux_resolved_variant(9, 0) == -2
