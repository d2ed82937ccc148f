"""ctypes loader for the plain-C oracle (brace_oracle.c) -- TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import
this.  It marshals numpy arrays into the C functions and does no arithmetic
of its own.
"""

from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "brace_oracle.c")
_LIB = os.path.join(_HERE, "liboracle_brace.so")

_lib = None


def build(force: bool = True) -> str:
    """Compile brace_oracle.c with gcc; returns the library path."""
    if force or not os.path.exists(_LIB):
        cmd = ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def load():
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB):
        build(force=True)
    lib = ctypes.CDLL(_LIB)
    f32p = ctypes.POINTER(ctypes.c_float)
    lib.oracle_threads.argtypes = [ctypes.c_int]
    lib.oracle_threads.restype = ctypes.c_int
    lib.oracle_brace_direct.argtypes = [
        f32p, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, ctypes.c_double,
        ctypes.c_int, f32p, ctypes.POINTER(ctypes.c_int32),
        ctypes.POINTER(ctypes.c_uint8), ctypes.c_int]
    lib.oracle_brace_direct.restype = ctypes.c_int
    lib.oracle_rar_sum.argtypes = [
        f32p, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, ctypes.c_double,
        ctypes.POINTER(ctypes.c_double), ctypes.c_int]
    lib.oracle_rar_sum.restype = ctypes.c_int
    lib.oracle_rar_sum_ring_f32.argtypes = [
        f32p, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64,
        ctypes.c_int, f32p, ctypes.c_int]
    lib.oracle_rar_sum_ring_f32.restype = ctypes.c_int
    _lib = lib
    return lib


def threads(requested: int = 0) -> int:
    return int(load().oracle_threads(int(requested)))


def _rows(updates: np.ndarray):
    if updates.dtype != np.float32 or updates.ndim != 2:
        raise ValueError("updates must be a 2-D float32 array")
    n, d = updates.shape
    # numpy leaves the strides of length-1 axes unspecified
    col_ok = d <= 1 or updates.strides[1] == 4
    row_ok = n <= 1 or (updates.strides[0] % 4 == 0 and updates.strides[0] >= 4 * d)
    if not (col_ok and row_ok):
        raise ValueError("updates must have unit column stride and row pitch >= d")
    ld = updates.strides[0] // 4 if n > 1 else max(d, 1)
    return n, d, ld


def brace_direct(updates: np.ndarray, lam: float, zero_sign: int = 0,
                 want_sums: bool = True, want_bits: bool = True, nthreads: int = 0):
    """Eq. (1) for every coordinate through the C oracle.

    Returns (out float32[d], sums int32[d] or None, bits uint8[ceil(d/8)] or None).
    """
    lib = load()
    n, d, ld = _rows(updates)
    out = np.empty(d, dtype=np.float32)
    sums = np.empty(d, dtype=np.int32) if want_sums else None
    bits = np.empty((d + 7) // 8, dtype=np.uint8) if want_bits else None
    rc = lib.oracle_brace_direct(
        updates.ctypes.data_as(ctypes.POINTER(ctypes.c_float)), n, d, ld,
        float(lam), int(zero_sign),
        out.ctypes.data_as(ctypes.POINTER(ctypes.c_float)),
        sums.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)) if want_sums else None,
        bits.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8)) if want_bits else None,
        int(nthreads))
    if rc != 0:
        raise ValueError("oracle_brace_direct rejected its arguments")
    return out, sums, bits


def rar_sum(updates: np.ndarray, scale: float = 1.0, nthreads: int = 0) -> np.ndarray:
    lib = load()
    n, d, ld = _rows(updates)
    out = np.empty(d, dtype=np.float64)
    rc = lib.oracle_rar_sum(
        updates.ctypes.data_as(ctypes.POINTER(ctypes.c_float)), n, d, ld,
        float(scale), out.ctypes.data_as(ctypes.POINTER(ctypes.c_double)), int(nthreads))
    if rc != 0:
        raise ValueError("oracle_rar_sum rejected its arguments")
    return out


def rar_sum_ring_f32(updates: np.ndarray, mean: bool = False, nthreads: int = 0,
                     d_total: int | None = None, k0: int = 0) -> np.ndarray:
    """Ring-order fp32 sum (or mean) of the client rows through the C oracle.  `updates` is
    the whole (n, d) matrix, or its columns [k0, k0 + width) of a vector of d_total."""
    lib = load()
    n, d, ld = _rows(updates)
    out = np.empty(d, dtype=np.float32)
    rc = lib.oracle_rar_sum_ring_f32(
        updates.ctypes.data_as(ctypes.POINTER(ctypes.c_float)), n, d, ld,
        d if d_total is None else int(d_total), int(k0), 1 if mean else 0,
        out.ctypes.data_as(ctypes.POINTER(ctypes.c_float)), int(nthreads))
    if rc != 0:
        raise ValueError("oracle_rar_sum_ring_f32 rejected its arguments")
    return out
