"""Seeded synthetic workloads: the five benchmark configurations and helpers.

This module only produces input bytes (host numpy arrays).  It contains none
of the reduction's arithmetic; it is the one module that both the GPU tests and
the CPU-oracle tests take inputs from.

Generator (counter based, chunkable):
    z(seed, i)   = mix64(seed * 0x9E3779B97F4A7C15 + i)   mod 2**64
    u24(seed, i) = (z >> 40) * 2**-24  in [0, 1)
with mix64 the SplitMix64 finaliser.  The fast path is ``csrc/workloads.c``
(gcc + OpenMP, built on first use); ``*_numpy`` are the same recipes written
with numpy and are what the tests check the C code against.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "csrc", "workloads.c")
_LIB = os.path.join(_HERE, "libredux_workloads.so")
_lib = None

GOLDEN = 0x9E3779B97F4A7C15
_M1 = 0xBF58476D1CE4E5B9
_M2 = 0x94D049BB133111EB


def build(force: bool = False) -> str:
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-Wall", "-Wextra", "-fopenmp", "-shared", "-fPIC", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        u64, vp = ctypes.c_uint64, ctypes.c_void_p
        lib.redux_gen_uniform_f16.restype = None
        lib.redux_gen_uniform_f16.argtypes = [vp, u64, u64, u64, ctypes.c_int]
        lib.redux_gen_normal_f16.restype = None
        lib.redux_gen_normal_f16.argtypes = [vp, u64, u64, u64]
        lib.redux_gen_uniform_i8.restype = None
        lib.redux_gen_uniform_i8.argtypes = [vp, u64, u64, u64]
        lib.redux_checksum_u16.restype = u64
        lib.redux_checksum_u16.argtypes = [vp, u64]
        lib.redux_checksum_u8.restype = u64
        lib.redux_checksum_u8.argtypes = [vp, u64]
        _lib = lib
    return _lib


# --------------------------------------------------------------------------
# generators (C fast path)
# --------------------------------------------------------------------------

def uniform_f16(seed: int, n: int, start: int = 0, symmetric: bool = False) -> np.ndarray:
    """n binary16 values, i.i.d. uniform on [0,1) (or [-1,1) if symmetric), as float16."""
    out = np.empty(n, dtype=np.float16)
    if n:
        _load().redux_gen_uniform_f16(out.ctypes.data, seed, start, n, int(symmetric))
    return out


def normal_f16(seed: int, n: int, start: int = 0) -> np.ndarray:
    """n binary16 values, i.i.d. N(0,1) by Box-Muller in binary64, rounded once."""
    out = np.empty(n, dtype=np.float16)
    if n:
        _load().redux_gen_normal_f16(out.ctypes.data, seed, start, n)
    return out


def uniform_i8(seed: int, n: int, start: int = 0) -> np.ndarray:
    """n int8 values, i.i.d. uniform on [-128, 127]."""
    out = np.empty(n, dtype=np.int8)
    if n:
        _load().redux_gen_uniform_i8(out.ctypes.data, seed, start, n)
    return out


def checksum(x: np.ndarray) -> int:
    """Sum of the raw 16-bit or 8-bit storage patterns mod 2**64."""
    a = np.ascontiguousarray(x).reshape(-1)
    if a.size == 0:
        return 0
    if a.dtype.itemsize == 2:
        return int(_load().redux_checksum_u16(a.ctypes.data, a.size))
    if a.dtype.itemsize == 1:
        return int(_load().redux_checksum_u8(a.ctypes.data, a.size))
    raise TypeError("checksum wants 1- or 2-byte elements")


# --------------------------------------------------------------------------
# the same recipes in numpy (slow; for cross-checking the C code)
# --------------------------------------------------------------------------

def _z_numpy(seed: int, idx: np.ndarray) -> np.ndarray:
    with np.errstate(over="ignore"):
        z = (np.uint64(seed) * np.uint64(GOLDEN)) + idx.astype(np.uint64)
        z ^= z >> np.uint64(30)
        z *= np.uint64(_M1)
        z ^= z >> np.uint64(27)
        z *= np.uint64(_M2)
        z ^= z >> np.uint64(31)
    return z


def _u24_numpy(seed: int, idx: np.ndarray) -> np.ndarray:
    return (_z_numpy(seed, idx) >> np.uint64(40)).astype(np.float64) * 2.0 ** -24


def uniform_f16_numpy(seed: int, n: int, start: int = 0, symmetric: bool = False) -> np.ndarray:
    idx = np.arange(start, start + n, dtype=np.uint64)
    u = _u24_numpy(seed, idx)
    v = (2.0 * u - 1.0) if symmetric else u
    h = v.astype(np.float16).view(np.uint16)
    h[h == 0x3C00] = 0x3BFF
    return h.view(np.float16)


def normal_f16_numpy(seed: int, n: int, start: int = 0) -> np.ndarray:
    idx = np.arange(start, start + n, dtype=np.uint64)
    u1 = _u24_numpy(seed, np.uint64(2) * idx)
    u2 = _u24_numpy(seed, np.uint64(2) * idx + np.uint64(1))
    x = np.sqrt(-2.0 * np.log(1.0 - u1)) * np.cos(2.0 * np.pi * u2)
    return x.astype(np.float16)


def uniform_i8_numpy(seed: int, n: int, start: int = 0) -> np.ndarray:
    idx = np.arange(start, start + n, dtype=np.uint64)
    return (_z_numpy(seed, idx) >> np.uint64(56)).astype(np.uint8).view(np.int8)


# --------------------------------------------------------------------------
# inputs for the other element types (numpy recipes; storage returned as raw bit patterns)
# --------------------------------------------------------------------------

def normal_f32(seed: int, n: int, start: int = 0) -> np.ndarray:
    """n binary32 values, N(0,1) by the same Box-Muller recipe, rounded once to binary32 (float32 array)."""
    idx = np.arange(start, start + n, dtype=np.uint64)
    u1 = _u24_numpy(seed, np.uint64(2) * idx)
    u2 = _u24_numpy(seed, np.uint64(2) * idx + np.uint64(1))
    return (np.sqrt(-2.0 * np.log(1.0 - u1)) * np.cos(2.0 * np.pi * u2)).astype(np.float32)


def normal_bf16(seed: int, n: int, start: int = 0) -> np.ndarray:
    """n bfloat16 patterns (uint16): N(0,1) in binary32, truncated to the upper 16 bits."""
    return (normal_f32(seed, n, start).view(np.uint32) >> np.uint32(16)).astype(np.uint16)


def finite_f8(seed: int, n: int, fmt: str, start: int = 0) -> np.ndarray:
    """n patterns (uint8) of an OCP 8-bit format, uniform over its finite values' patterns.

    fmt 'e4m3': the two NaN patterns (0x7F, 0xFF) are replaced by zero of the same sign;
    fmt 'e5m2': patterns with exponent 31 (Inf/NaN) get the top exponent bit cleared."""
    b = uniform_i8(seed, n, start).view(np.uint8).copy()
    if fmt == "e4m3":
        b[(b & 0x7F) == 0x7F] &= 0x80
    elif fmt == "e5m2":
        b[(b & 0x7C) == 0x7C] &= 0xBF
    else:
        raise ValueError(fmt)
    return b


# --------------------------------------------------------------------------
# the benchmark configurations
# --------------------------------------------------------------------------

@dataclass(frozen=True)
class Config:
    name: str
    dtype: str            # "f16" or "i8"
    n: int                # total elements
    seed: int
    dist: str             # "uniform01", "normal", "uniform_i8", "uniform11"
    nseg: Optional[int] = None
    seglen: Optional[int] = None

    @property
    def nbytes(self) -> int:
        return self.n * (2 if self.dtype == "f16" else 1)

    @property
    def segmented(self) -> bool:
        return self.nseg is not None


CONFIGS = {
    "C1": Config("C1", "f16", 1 << 20, 0, "uniform01"),
    "C2": Config("C2", "f16", 1 << 26, 1, "normal"),
    "C3": Config("C3", "f16", (1 << 30) + 12345, 2, "uniform01"),
    "C4": Config("C4", "i8", 1 << 30, 3, "uniform_i8"),
    "C5": Config("C5", "f16", 65536 * 4096, 4, "uniform11", nseg=65536, seglen=4096),
}


def make(cfg: Config, n: Optional[int] = None, start: int = 0) -> np.ndarray:
    """Host array for a configuration (optionally only elements [start, start+n))."""
    n = cfg.n if n is None else n
    if cfg.dist == "uniform01":
        return uniform_f16(cfg.seed, n, start, symmetric=False)
    if cfg.dist == "uniform11":
        return uniform_f16(cfg.seed, n, start, symmetric=True)
    if cfg.dist == "normal":
        return normal_f16(cfg.seed, n, start)
    if cfg.dist == "uniform_i8":
        return uniform_i8(cfg.seed, n, start)
    raise ValueError(cfg.dist)
