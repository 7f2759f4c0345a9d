"""CPU oracle for the arithmetic reduction (paper Section III, R(X) = sum x_i).

TEST INFRASTRUCTURE ONLY.  The product (the HIP library and its Python
binding) never imports this package; only the tests, the smoke check and the
``cpu_baseline`` leg of the benchmark do.  It shares no code with the GPU path.

Two parts:

* ``redux_oracle.c`` -- the definition of the sum written out in plain C
  (binary64 serial / pairwise / Neumaier / exact 128-bit fixed point for
  binary16 input, int64 for int8 input), loaded here through ctypes; plus a
  many-core form of the same sums (contiguous chunks, one OpenMP thread each,
  combined in chunk order) for timing the oracle on all host cores.
* ``mma_reduction.py`` -- a numpy replay of the paper's own algorithm
  (Section IV-A: MMA against all-ones, then all-ones against the result,
  applied level by level), used to pin the encoding.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "redux_oracle.c")
_LIB = os.path.join(_HERE, "libredux_oracle.so")

_lib = None


def build(force: bool = False) -> str:
    """Compile redux_oracle.c with gcc (no HIP, no flags that relax IEEE arithmetic)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fopenmp", "-Wall", "-Wextra", "-shared", "-fPIC", "-o", tmp, _SRC, "-lm"]
        )
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        # REDUX_ORACLE_LIB: load this build instead; the mutation test points it at deliberately broken
        # copies of redux_oracle.c to show that the pins catch them.
        lib = ctypes.CDLL(os.environ.get("REDUX_ORACLE_LIB") or build())
        c_sz, c_dp = ctypes.c_size_t, ctypes.POINTER(ctypes.c_double)
        c_ip = ctypes.POINTER(ctypes.c_int64)
        vp = ctypes.c_void_p
        lib.redux_oracle_f16_decode.restype = ctypes.c_double
        lib.redux_oracle_f16_decode.argtypes = [ctypes.c_uint16]
        for name in ("redux_oracle_sum_f16", "redux_oracle_sum_f16_serial", "redux_oracle_sum_f16_neumaier"):
            fn = getattr(lib, name)
            fn.restype = ctypes.c_int
            fn.argtypes = [vp, c_sz, c_dp, c_dp]
        lib.redux_oracle_sum_f16_exact.restype = ctypes.c_int
        lib.redux_oracle_sum_f16_exact.argtypes = [
            vp, c_sz, c_dp, c_dp, c_ip, ctypes.POINTER(ctypes.c_uint64), ctypes.POINTER(ctypes.c_int)]
        lib.redux_oracle_sum_i8.restype = ctypes.c_int
        lib.redux_oracle_sum_i8.argtypes = [vp, c_sz, c_ip, c_ip]
        lib.redux_oracle_sum_segmented_f16.restype = ctypes.c_int
        lib.redux_oracle_sum_segmented_f16.argtypes = [vp, c_sz, c_sz, vp, vp]
        lib.redux_oracle_sum_segmented_i8.restype = ctypes.c_int
        lib.redux_oracle_sum_segmented_i8.argtypes = [vp, c_sz, c_sz, vp, vp]
        for name in ("redux_oracle_sum_any", "redux_oracle_sum_any_neumaier"):
            fn = getattr(lib, name)
            fn.restype = ctypes.c_int
            fn.argtypes = [vp, c_sz, ctypes.c_int, c_dp, c_dp]
        lib.redux_oracle_sum_f8_exact.restype = ctypes.c_int
        lib.redux_oracle_sum_f8_exact.argtypes = [vp, c_sz, ctypes.c_int, c_ip, c_ip, ctypes.POINTER(ctypes.c_int)]
        lib.redux_oracle_sum_segmented_any.restype = ctypes.c_int
        lib.redux_oracle_sum_segmented_any.argtypes = [vp, c_sz, c_sz, ctypes.c_int, vp, vp]
        lib.redux_oracle_max_threads.restype = ctypes.c_int
        lib.redux_oracle_max_threads.argtypes = []
        lib.redux_oracle_sum_f16_chunks.restype = ctypes.c_int
        lib.redux_oracle_sum_f16_chunks.argtypes = [vp, c_sz, ctypes.c_int, c_dp, c_dp]
        lib.redux_oracle_sum_i8_chunks.restype = ctypes.c_int
        lib.redux_oracle_sum_i8_chunks.argtypes = [vp, c_sz, ctypes.c_int, c_ip, c_ip]
        lib.redux_oracle_sum_segmented_f16_chunks.restype = ctypes.c_int
        lib.redux_oracle_sum_segmented_f16_chunks.argtypes = [vp, c_sz, c_sz, ctypes.c_int, vp, vp]
        for name, argt in (("redux_oracle_bf16_decode", ctypes.c_uint16), ("redux_oracle_f32_decode", ctypes.c_uint32),
                           ("redux_oracle_f8e4m3_decode", ctypes.c_uint8), ("redux_oracle_f8e5m2_decode", ctypes.c_uint8)):
            fn = getattr(lib, name)
            fn.restype = ctypes.c_double
            fn.argtypes = [argt]
        _lib = lib
    return _lib


def _as_u16(x) -> np.ndarray:
    """Accept float16 or uint16 storage; return a contiguous 1-D uint16 view of the raw patterns."""
    a = np.asarray(x)
    if a.dtype == np.float16:
        a = a.view(np.uint16)
    if a.dtype != np.uint16:
        raise TypeError("binary16 oracle wants float16 or uint16 storage, got %s" % a.dtype)
    return np.ascontiguousarray(a).reshape(-1)


def _as_i8(x) -> np.ndarray:
    a = np.asarray(x)
    if a.dtype != np.int8:
        raise TypeError("int8 oracle wants int8 storage, got %s" % a.dtype)
    return np.ascontiguousarray(a).reshape(-1)


def _ptr(a: np.ndarray):
    return ctypes.c_void_p(a.ctypes.data) if a.size else ctypes.c_void_p(0)


def f16_decode(pattern: int) -> float:
    """Exact binary64 value of one binary16 bit pattern."""
    return float(_load().redux_oracle_f16_decode(int(pattern) & 0xFFFF))


def _f16_call(name: str, x) -> Tuple[float, float]:
    a = _as_u16(x)
    s, sa = ctypes.c_double(), ctypes.c_double()
    rc = getattr(_load(), name)(_ptr(a), a.size, ctypes.byref(s), ctypes.byref(sa))
    if rc:
        raise RuntimeError("%s failed: %d" % (name, rc))
    return s.value, sa.value


def sum_f16(x) -> Tuple[float, float]:
    """Primary oracle: (sum, sum of |x|) by binary64 pairwise summation."""
    return _f16_call("redux_oracle_sum_f16", x)


def sum_f16_serial(x) -> Tuple[float, float]:
    """Single-accumulator binary64 loop in index order (Section III's serial algorithm)."""
    return _f16_call("redux_oracle_sum_f16_serial", x)


def sum_f16_neumaier(x) -> Tuple[float, float]:
    """Compensated (Kahan-Babuska/Neumaier) binary64 sum."""
    return _f16_call("redux_oracle_sum_f16_neumaier", x)


def sum_f16_exact(x):
    """Exact sum in units of 2**-24.

    Returns (sum as float, sum|x| as float, exact integer number of 2**-24 units, nonfinite flag).
    """
    a = _as_u16(x)
    s, sa = ctypes.c_double(), ctypes.c_double()
    hi, lo, nf = ctypes.c_int64(), ctypes.c_uint64(), ctypes.c_int()
    rc = _load().redux_oracle_sum_f16_exact(
        _ptr(a), a.size, ctypes.byref(s), ctypes.byref(sa), ctypes.byref(hi), ctypes.byref(lo), ctypes.byref(nf))
    if rc:
        raise RuntimeError("redux_oracle_sum_f16_exact failed: %d" % rc)
    units = (hi.value << 64) + lo.value
    return s.value, sa.value, units, bool(nf.value)


def sum_i8(x) -> Tuple[int, int]:
    """(sum, sum of |x|) of int8 values as Python ints (int64 arithmetic)."""
    a = _as_i8(x)
    s, sa = ctypes.c_int64(), ctypes.c_int64()
    rc = _load().redux_oracle_sum_i8(_ptr(a), a.size, ctypes.byref(s), ctypes.byref(sa))
    if rc:
        raise RuntimeError("redux_oracle_sum_i8 failed: %d" % rc)
    return s.value, sa.value


def sum_segmented_f16(x, nseg: int, seglen: int) -> Tuple[np.ndarray, np.ndarray]:
    """Per-segment (sums, sums of |x|) as float64 arrays of length nseg; row-major [nseg][seglen]."""
    a = _as_u16(x)
    if a.size != nseg * seglen:
        raise ValueError("size %d != nseg*seglen %d" % (a.size, nseg * seglen))
    s = np.zeros(nseg, dtype=np.float64)
    sa = np.zeros(nseg, dtype=np.float64)
    rc = _load().redux_oracle_sum_segmented_f16(_ptr(a), nseg, seglen, _ptr(s), _ptr(sa))
    if rc:
        raise RuntimeError("redux_oracle_sum_segmented_f16 failed: %d" % rc)
    return s, sa


def sum_segmented_i8(x, nseg: int, seglen: int) -> Tuple[np.ndarray, np.ndarray]:
    """Per-segment (sums, sums of |x|) as int64 arrays of length nseg."""
    a = _as_i8(x)
    if a.size != nseg * seglen:
        raise ValueError("size %d != nseg*seglen %d" % (a.size, nseg * seglen))
    s = np.zeros(nseg, dtype=np.int64)
    sa = np.zeros(nseg, dtype=np.int64)
    rc = _load().redux_oracle_sum_segmented_i8(_ptr(a), nseg, seglen, _ptr(s), _ptr(sa))
    if rc:
        raise RuntimeError("redux_oracle_sum_segmented_i8 failed: %d" % rc)
    return s, sa


# ---- many-core form: contiguous chunks, one OpenMP thread each, combined in chunk order ----------------------

def max_threads() -> int:
    """Threads the many-core form gets by default on this host (OMP_NUM_THREADS or the core count)."""
    return int(_load().redux_oracle_max_threads())


def sum_f16_chunks(x, chunks: int = 0) -> Tuple[float, float]:
    """(sum, sum|x|): the array cut into `chunks` contiguous chunks (0 = max_threads()), each summed pairwise by
    its own thread, chunk sums added in chunk order."""
    a = _as_u16(x)
    s, sa = ctypes.c_double(), ctypes.c_double()
    rc = _load().redux_oracle_sum_f16_chunks(_ptr(a), a.size, chunks or max_threads(), ctypes.byref(s), ctypes.byref(sa))
    if rc:
        raise RuntimeError("redux_oracle_sum_f16_chunks failed: %d" % rc)
    return s.value, sa.value


def sum_i8_chunks(x, chunks: int = 0) -> Tuple[int, int]:
    a = _as_i8(x)
    s, sa = ctypes.c_int64(), ctypes.c_int64()
    rc = _load().redux_oracle_sum_i8_chunks(_ptr(a), a.size, chunks or max_threads(), ctypes.byref(s), ctypes.byref(sa))
    if rc:
        raise RuntimeError("redux_oracle_sum_i8_chunks failed: %d" % rc)
    return s.value, sa.value


def sum_segmented_f16_chunks(x, nseg: int, seglen: int, chunks: int = 0) -> Tuple[np.ndarray, np.ndarray]:
    a = _as_u16(x)
    if a.size != nseg * seglen:
        raise ValueError("size %d != nseg*seglen %d" % (a.size, nseg * seglen))
    s = np.zeros(nseg, dtype=np.float64)
    sa = np.zeros(nseg, dtype=np.float64)
    rc = _load().redux_oracle_sum_segmented_f16_chunks(_ptr(a), nseg, seglen, chunks or max_threads(), _ptr(s), _ptr(sa))
    if rc:
        raise RuntimeError("redux_oracle_sum_segmented_f16_chunks failed: %d" % rc)
    return s, sa


# ---- bfloat16, binary32 and the OCP 8-bit formats (raw storage patterns in, binary64 out) --------------------

BF16, F32, F8E4M3, F8E5M2 = 2, 3, 4, 5
_STORAGE = {BF16: np.uint16, F32: np.uint32, F8E4M3: np.uint8, F8E5M2: np.uint8}


def _as_storage(x, dtype: int) -> np.ndarray:
    a = np.asarray(x)
    want = _STORAGE[dtype]
    if dtype == F32 and a.dtype == np.float32:
        a = a.view(np.uint32)
    if a.dtype != want:
        raise TypeError("dtype %d wants %s storage (raw bit patterns), got %s" % (dtype, want.__name__, a.dtype))
    return np.ascontiguousarray(a).reshape(-1)


def decode(pattern: int, dtype: int) -> float:
    """Exact binary64 value of one storage pattern of dtype BF16 / F32 / F8E4M3 / F8E5M2."""
    fn = {BF16: "redux_oracle_bf16_decode", F32: "redux_oracle_f32_decode",
          F8E4M3: "redux_oracle_f8e4m3_decode", F8E5M2: "redux_oracle_f8e5m2_decode"}[dtype]
    return float(getattr(_load(), fn)(int(pattern)))


def sum_any(x, dtype: int, method: str = "pairwise") -> Tuple[float, float]:
    """(sum, sum|x|) of raw patterns of dtype BF16 / F32 / F8E4M3 / F8E5M2; method 'pairwise' or 'neumaier'."""
    a = _as_storage(x, dtype)
    s, sa = ctypes.c_double(), ctypes.c_double()
    fn = "redux_oracle_sum_any" if method == "pairwise" else "redux_oracle_sum_any_neumaier"
    rc = getattr(_load(), fn)(_ptr(a), a.size, dtype, ctypes.byref(s), ctypes.byref(sa))
    if rc:
        raise RuntimeError("%s failed: %d" % (fn, rc))
    return s.value, sa.value


def sum_f8_exact(x, dtype: int):
    """Exact sum of an 8-bit format: (units, units of sum|x|, scale, nonfinite) with value = units * scale."""
    a = _as_storage(x, dtype)
    u, ua, nf = ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int()
    rc = _load().redux_oracle_sum_f8_exact(_ptr(a), a.size, dtype, ctypes.byref(u), ctypes.byref(ua), ctypes.byref(nf))
    if rc:
        raise RuntimeError("redux_oracle_sum_f8_exact failed: %d" % rc)
    return u.value, ua.value, 2.0 ** (-9 if dtype == F8E4M3 else -16), bool(nf.value)


def sum_segmented_any(x, nseg: int, seglen: int, dtype: int) -> Tuple[np.ndarray, np.ndarray]:
    a = _as_storage(x, dtype)
    if a.size != nseg * seglen:
        raise ValueError("size %d != nseg*seglen %d" % (a.size, nseg * seglen))
    s = np.zeros(nseg, dtype=np.float64)
    sa = np.zeros(nseg, dtype=np.float64)
    rc = _load().redux_oracle_sum_segmented_any(_ptr(a), nseg, seglen, dtype, _ptr(s), _ptr(sa))
    if rc:
        raise RuntimeError("redux_oracle_sum_segmented_any failed: %d" % rc)
    return s, sa
