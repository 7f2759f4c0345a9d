"""ctypes binding of libredux (see include/redux.h).  Argument marshalling only.

Every arithmetic step runs in the HIP kernels of ``libredux.so``; PyTorch is used
for device memory and the current stream, nothing else.  There is no CPU
fallback: if the library has not been built, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libredux.so")

F16, I8, BF16, F32, F8E4M3, F8E5M2 = 0, 1, 2, 3, 4, 5
VARIANTS = {"auto": 0, "mfma": 1, "classic": 2}

# every symbol include/redux.h declares
SYMBOLS = (
    "redux_sum", "redux_sum_static", "redux_sum_segmented", "redux_sum_multipass", "redux_mma_group_probe", "redux_calibration_copy",
    "redux_plan_sum", "redux_plan_sum_segmented", "redux_plan_block_slabs", "redux_plan_run_share",
    "redux_set_variant", "redux_get_variant", "redux_resolved_variant", "redux_set_param", "redux_get_param",
    "redux_strerror", "redux_last_hip_error", "redux_shutdown", "redux_version",
)

_lib = None


class Plan(ctypes.Structure):
    """Mirror of redux_plan."""
    _fields_ = [("kernel", ctypes.c_int), ("unroll", ctypes.c_int), ("grid", ctypes.c_uint), ("finish", ctypes.c_int),
                ("parts", ctypes.c_uint64), ("part_len", ctypes.c_uint64), ("head", ctypes.c_uint), ("tail", ctypes.c_uint),
                ("vectors", ctypes.c_uint64), ("chain", ctypes.c_uint)]


KERNEL_FLAT, KERNEL_ROWS, KERNEL_WAVE, KERNEL_PIECES, KERNEL_TILES, KERNEL_BLOCK, KERNEL_SHORT, KERNEL_RAGGED, KERNEL_RUNS = 0, 1, 2, 3, 4, 5, 6, 7, 8


class ReduxError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = _lib.redux_strerror(status).decode() if _lib is not None else "?"
        hip = _lib.redux_last_hip_error() if _lib is not None and status in (-5, -6) else 0
        super().__init__("%s failed: %s (status %d%s)" % (where, msg, status, ", hipError %d" % hip if hip else ""))


def load():
    """Load libredux.so (built by __graft_entry__.build()); raises if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError("libredux.so is not built: run `python __graft_entry__.py` (there is no CPU fallback)")
        lib = ctypes.CDLL(LIB_PATH)
        vp, sz, ci = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int
        lib.redux_sum.restype = ci
        lib.redux_sum.argtypes = [vp, sz, ci, vp, vp]
        lib.redux_sum_static.restype = ci
        lib.redux_sum_static.argtypes = [vp, sz, ci, vp, vp]
        lib.redux_sum_segmented.restype = ci
        lib.redux_sum_segmented.argtypes = [vp, sz, sz, ci, vp, vp]
        lib.redux_sum_multipass.restype = ci
        lib.redux_sum_multipass.argtypes = [vp, sz, ci, vp, ctypes.POINTER(ci), vp]
        lib.redux_mma_group_probe.restype = ci
        lib.redux_mma_group_probe.argtypes = [vp, sz, ci, vp, vp, vp]
        lib.redux_calibration_copy.restype = ci
        lib.redux_calibration_copy.argtypes = [vp, vp, sz, vp]
        u64p = ctypes.POINTER(ctypes.c_uint64)
        lib.redux_plan_sum.restype = ci
        lib.redux_plan_sum.argtypes = [sz, ci, ctypes.c_size_t, ci, ctypes.POINTER(Plan)]
        lib.redux_plan_sum_segmented.restype = ci
        lib.redux_plan_sum_segmented.argtypes = [sz, sz, ci, ctypes.c_size_t, ci, ctypes.POINTER(Plan)]
        lib.redux_plan_block_slabs.restype = ci
        lib.redux_plan_block_slabs.argtypes = [ci, ctypes.c_uint64, ctypes.c_uint64, ctypes.c_uint64, u64p, u64p, u64p]
        lib.redux_plan_run_share.restype = ci
        lib.redux_plan_run_share.argtypes = [ci, ctypes.c_uint64, ctypes.c_uint, ctypes.c_uint64, ctypes.c_uint64, ctypes.c_uint,
                                             u64p, u64p, u64p, u64p, ctypes.POINTER(ctypes.c_uint)]
        lib.redux_set_variant.restype = ci
        lib.redux_set_variant.argtypes = [ci]
        lib.redux_get_variant.restype = ci
        lib.redux_get_variant.argtypes = []
        lib.redux_resolved_variant.restype = ci
        lib.redux_resolved_variant.argtypes = [ci, ci]
        lib.redux_set_param.restype = ci
        lib.redux_set_param.argtypes = [ctypes.c_char_p, ctypes.c_long]
        lib.redux_get_param.restype = ctypes.c_long
        lib.redux_get_param.argtypes = [ctypes.c_char_p]
        lib.redux_strerror.restype = ctypes.c_char_p
        lib.redux_strerror.argtypes = [ci]
        lib.redux_last_hip_error.restype = ci
        lib.redux_last_hip_error.argtypes = []
        lib.redux_shutdown.restype = None
        lib.redux_shutdown.argtypes = []
        lib.redux_version.restype = ctypes.c_char_p
        lib.redux_version.argtypes = []
        _lib = lib
    return _lib


def _check(status: int, where: str) -> None:
    if status != 0:
        raise ReduxError(status, where)


def version() -> str:
    return load().redux_version().decode()


def strerror(status: int) -> str:
    return load().redux_strerror(status).decode()


def set_variant(variant) -> None:
    v = VARIANTS[variant] if isinstance(variant, str) else int(variant)
    _check(load().redux_set_variant(v), "redux_set_variant")


def get_variant() -> int:
    return load().redux_get_variant()


def resolved_variant(dtype: int, segmented: bool) -> str:
    """'mfma' or 'classic': the family a call on `dtype` runs with under the current setting."""
    v = load().redux_resolved_variant(dtype, 1 if segmented else 0)
    if v < 0:
        raise ReduxError(v, "redux_resolved_variant")
    return {1: "mfma", 2: "classic"}[v]


def set_param(name: str, value: int) -> None:
    _check(load().redux_set_param(name.encode(), int(value)), "redux_set_param(%s)" % name)


def get_param(name: str) -> int:
    return int(load().redux_get_param(name.encode()))


def shutdown() -> None:
    load().redux_shutdown()


# ---- raw calls: pointers and sizes, exactly the C signatures --------------------------------------

def sum_raw(x_ptr: int, n: int, dtype: int, out_ptr: int, stream: int = 0) -> int:
    return load().redux_sum(x_ptr, n, dtype, out_ptr, stream)


def sum_static_raw(x_ptr: int, n: int, dtype: int, out_ptr: int, stream: int = 0) -> int:
    return load().redux_sum_static(x_ptr, n, dtype, out_ptr, stream)


def sum_segmented_raw(x_ptr: int, nseg: int, seglen: int, dtype: int, out_ptr: int, stream: int = 0) -> int:
    return load().redux_sum_segmented(x_ptr, nseg, seglen, dtype, out_ptr, stream)


def sum_multipass_raw(x_ptr: int, n: int, dtype: int, out_ptr: int, stream: int = 0):
    """Returns (status, levels)."""
    levels = ctypes.c_int(0)
    rc = load().redux_sum_multipass(x_ptr, n, dtype, out_ptr, ctypes.byref(levels), stream)
    return rc, levels.value


def mma_group_probe_raw(x_ptr: int, count: int, dtype: int, d_ptr: int, dp_ptr: int, stream: int = 0) -> int:
    return load().redux_mma_group_probe(x_ptr, count, dtype, d_ptr, dp_ptr, stream)


def calibration_copy_raw(dst_ptr: int, src_ptr: int, nbytes: int, stream: int = 0) -> int:
    return load().redux_calibration_copy(dst_ptr, src_ptr, nbytes, stream)


def plan_sum(n: int, dtype: int, x_address: int = 0, compute_units: int = 256) -> Plan:
    p = Plan()
    _check(load().redux_plan_sum(n, dtype, x_address, compute_units, ctypes.byref(p)), "redux_plan_sum")
    return p


def plan_sum_segmented(nseg: int, seglen: int, dtype: int, x_address: int = 0, compute_units: int = 256) -> Plan:
    p = Plan()
    _check(load().redux_plan_sum_segmented(nseg, seglen, dtype, x_address, compute_units, ctypes.byref(p)),
           "redux_plan_sum_segmented")
    return p


def plan_block_slabs(layout: int, nslab: int, grid: int, block: int):
    """(start, stride, count) of the slabs one block reads."""
    a, b, c = ctypes.c_uint64(), ctypes.c_uint64(), ctypes.c_uint64()
    _check(load().redux_plan_block_slabs(layout, nslab, grid, block, ctypes.byref(a), ctypes.byref(b), ctypes.byref(c)),
           "redux_plan_block_slabs")
    return a.value, b.value, c.value


def plan_run_share(layout: int, nseg: int, per_run: int, grid: int, block: int, wave: int):
    """(first, stride, rounds, tail_first, tail_count) of the segments one wavefront of the RUNS kernel sums."""
    a, b, c, d, e = ctypes.c_uint64(), ctypes.c_uint64(), ctypes.c_uint64(), ctypes.c_uint64(), ctypes.c_uint()
    _check(load().redux_plan_run_share(layout, nseg, per_run, grid, block, wave, ctypes.byref(a), ctypes.byref(b),
                                       ctypes.byref(c), ctypes.byref(d), ctypes.byref(e)), "redux_plan_run_share")
    return a.value, b.value, c.value, d.value, e.value


# ---- torch conveniences: allocate the output, pass the current stream --------------------------------

_DTYPES = None


def _dtype_of(x) -> int:
    global _DTYPES
    if _DTYPES is None:
        import torch
        _DTYPES = {torch.float16: F16, torch.int8: I8, torch.bfloat16: BF16, torch.float32: F32,
                   torch.float8_e4m3fn: F8E4M3, torch.float8_e5m2: F8E5M2}
    dt = _DTYPES.get(x.dtype)
    if dt is None:
        raise TypeError("redux supports float16, int8, bfloat16, float32, float8_e4m3fn and float8_e5m2 tensors, got %s" % x.dtype)
    return dt


def _prep(x) -> int:
    """Checks x and returns the raw handle of the current stream of x's device."""
    import torch
    if not x.is_cuda:
        raise ValueError("redux needs a device tensor (there is no CPU path)")
    if not x.is_contiguous():
        raise ValueError("redux needs a contiguous tensor")
    return torch._C._cuda_getCurrentRawStream(x.device.index)


class _Device:
    """Make x's device current for the call; a no-op (no context-manager cost) when it already is."""
    __slots__ = ("ctx",)

    def __init__(self, x):
        import torch
        self.ctx = None if torch._C._cuda_getDevice() == x.device.index else torch.cuda.device(x.device)

    def __enter__(self):
        if self.ctx is not None:
            self.ctx.__enter__()

    def __exit__(self, *exc):
        if self.ctx is not None:
            self.ctx.__exit__(*exc)


def sum(x, out=None):
    """Sum of all elements of a float16 (-> float32) or int8 (-> int64) device tensor; returns a 1-element tensor."""
    import torch
    stream = _prep(x)
    dt = _dtype_of(x)
    if out is None:
        out = torch.empty(1, dtype=torch.int64 if dt == I8 else torch.float32, device=x.device)
    n = x.numel()
    lib = _lib if _lib is not None else load()
    if torch._C._cuda_getDevice() == x.device.index:      # the usual case: nothing to switch, no context manager
        rc = lib.redux_sum(x.data_ptr() if n else 0, n, dt, out.data_ptr(), stream)
    else:
        with torch.cuda.device(x.device):
            rc = lib.redux_sum(x.data_ptr() if n else 0, n, dt, out.data_ptr(), stream)
    if rc:
        raise ReduxError(rc, "redux_sum")
    return out


def sum_multipass(x, out=None):
    """The level-by-level form of the sum (one kernel launch per level); returns (1-element tensor, levels)."""
    import torch
    stream = _prep(x)
    dt = _dtype_of(x)
    if out is None:
        out = torch.empty(1, dtype=torch.float32 if dt == F16 else torch.int64, device=x.device)
    with _Device(x):
        rc, levels = sum_multipass_raw(x.data_ptr() if x.numel() else 0, x.numel(), dt, out.data_ptr(), stream)
    _check(rc, "redux_sum_multipass")
    return out, levels


def sum_segmented(x, nseg: Optional[int] = None, seglen: Optional[int] = None, out=None):
    """Per-segment sums of a row-major [nseg][seglen] device tensor; returns nseg results."""
    import torch
    stream = _prep(x)
    dt = _dtype_of(x)
    if nseg is None or seglen is None:
        if x.dim() != 2:
            raise ValueError("give nseg and seglen, or a 2-D tensor")
        nseg, seglen = x.shape
    if nseg * seglen != x.numel():
        raise ValueError("nseg*seglen != numel")
    if out is None:
        out = torch.empty(nseg, dtype=torch.int64 if dt == I8 else torch.float32, device=x.device)
    with _Device(x):
        _check(sum_segmented_raw(x.data_ptr() if x.numel() else 0, nseg, seglen, dt,
                                 out.data_ptr() if nseg else 0, stream), "redux_sum_segmented")
    return out


def mma_group_probe(x):
    """Both MMA result matrices (D, D') of one group, as 16x16 tensors."""
    import torch
    stream = _prep(x)
    dt = _dtype_of(x)
    D = torch.empty(16, 16, dtype=torch.float32 if dt == F16 else torch.int32, device=x.device)
    Dp = torch.empty(16, 16, dtype=torch.float32 if dt == F16 else torch.float64, device=x.device)
    with _Device(x):
        _check(mma_group_probe_raw(x.data_ptr() if x.numel() else 0, x.numel(), dt, D.data_ptr(), Dp.data_ptr(), stream),
               "redux_mma_group_probe")
    return D, Dp
