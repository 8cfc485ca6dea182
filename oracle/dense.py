"""ctypes front end of the C oracle: the product by its plain definition.

``out[b][c] = sum_r v[b][r] * A[r][c]`` (Section 2.2, Problems 1 and 2), one
accumulator per column, rows visited in order.  Float activations accumulate in
float64, int8 activations in int64.  Test infrastructure only.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import numpy as np

from . import build as _build

_lib: Optional[ctypes.CDLL] = None

_i8p = ctypes.POINTER(ctypes.c_int8)
_f32p = ctypes.POINTER(ctypes.c_float)
_f64p = ctypes.POINTER(ctypes.c_double)
_i64p = ctypes.POINTER(ctypes.c_int64)
_i64 = ctypes.c_int64


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        path = _build.build()
        L = ctypes.CDLL(path)
        L.rsr_oracle_matvec_f32.argtypes = [_i8p, _i64, _i64, _f32p, _i64, _f64p]
        L.rsr_oracle_matvec_f32.restype = None
        L.rsr_oracle_matvec_i8.argtypes = [_i8p, _i64, _i64, _i8p, _i64, _i64p]
        L.rsr_oracle_matvec_i8.restype = None
        L.rsr_oracle_matvec_f32_cols.argtypes = [_i8p, _i64, _i64, _f32p, _i64, _f64p, _i64, _i64]
        L.rsr_oracle_matvec_f32_cols.restype = None
        L.rsr_oracle_matvec_i8_cols.argtypes = [_i8p, _i64, _i64, _i8p, _i64, _i64p, _i64, _i64]
        L.rsr_oracle_matvec_i8_cols.restype = None
        L.rsr_oracle_matvec_f32_mt.argtypes = [_i8p, _i64, _i64, _f32p, _i64, _f64p, ctypes.c_int]
        L.rsr_oracle_matvec_f32_mt.restype = ctypes.c_int
        L.rsr_oracle_matvec_i8_mt.argtypes = [_i8p, _i64, _i64, _i8p, _i64, _i64p, ctypes.c_int]
        L.rsr_oracle_matvec_i8_mt.restype = ctypes.c_int
        L.rsr_oracle_check_entries.argtypes = [_i8p, _i64, _i64]
        L.rsr_oracle_check_entries.restype = _i64
        _lib = L
    return _lib


def _prep(A: np.ndarray, v: np.ndarray, vdtype, qbits: Optional[int] = None):
    A = np.ascontiguousarray(A, dtype=np.int8)
    if A.ndim != 2:
        raise ValueError("A must be 2-D (rows x cols)")
    v = np.ascontiguousarray(v, dtype=vdtype)
    squeeze = v.ndim == 1
    if squeeze:
        v = v[None, :]
    if v.ndim != 2 or v.shape[1] != A.shape[0]:
        raise ValueError(f"v must be [batch][rows={A.shape[0]}], got {v.shape}")
    if qbits is None:
        bad = lib().rsr_oracle_check_entries(A.ctypes.data_as(_i8p), A.shape[0], A.shape[1])
        if bad:
            raise ValueError(f"A has an entry outside {{-1,0,1}} at flat index {bad - 1}")
    else:
        # a matrix with q bits per entry (appendix "Generalization"): the same definition of the
        # product, entries in the two's complement range of q bits
        lo, hi = -(1 << (qbits - 1)), (1 << (qbits - 1)) - 1
        if not 2 <= qbits <= 8 or A.min() < lo or A.max() > hi:
            raise ValueError(f"A has an entry outside {lo}..{hi}, or q is not in 2..8")
    return A, v, squeeze


def matvec_f32(A: np.ndarray, v: np.ndarray, threads: int = 1, cols: Optional[tuple] = None,
               qbits: Optional[int] = None) -> np.ndarray:
    """float activations -> float64 result ``[batch][cols]`` (or ``[cols]`` for a 1-D ``v``).

    ``cols=(c0, c1)`` computes only that column range; the other outputs are NaN.
    ``qbits=q`` admits entries of q bits (two's complement) instead of {-1,0,1}.
    """
    A, v, squeeze = _prep(A, v, np.float32, qbits)
    rows, ncols = A.shape
    out = np.full((v.shape[0], ncols), np.nan, dtype=np.float64)
    a, vp, op = A.ctypes.data_as(_i8p), v.ctypes.data_as(_f32p), out.ctypes.data_as(_f64p)
    if cols is not None:
        lib().rsr_oracle_matvec_f32_cols(a, rows, ncols, vp, v.shape[0], op, int(cols[0]), int(cols[1]))
    elif threads > 1:
        if lib().rsr_oracle_matvec_f32_mt(a, rows, ncols, vp, v.shape[0], op, int(threads)) < 1:
            raise RuntimeError("oracle: could not start threads")
    else:
        lib().rsr_oracle_matvec_f32(a, rows, ncols, vp, v.shape[0], op)
    return out[0] if squeeze else out


def matvec_i8(A: np.ndarray, v: np.ndarray, threads: int = 1, cols: Optional[tuple] = None,
              qbits: Optional[int] = None) -> np.ndarray:
    """int8 activations -> int64 result ``[batch][cols]`` (or ``[cols]`` for a 1-D ``v``).

    ``cols=(c0, c1)`` computes only that column range; the other outputs are left at int64 min.
    ``qbits=q`` admits entries of q bits (two's complement) instead of {-1,0,1}.
    """
    A, v, squeeze = _prep(A, v, np.int8, qbits)
    rows, ncols = A.shape
    out = np.full((v.shape[0], ncols), np.iinfo(np.int64).min, dtype=np.int64)
    a, vp, op = A.ctypes.data_as(_i8p), v.ctypes.data_as(_i8p), out.ctypes.data_as(_i64p)
    if cols is not None:
        lib().rsr_oracle_matvec_i8_cols(a, rows, ncols, vp, v.shape[0], op, int(cols[0]), int(cols[1]))
    elif threads > 1:
        if lib().rsr_oracle_matvec_i8_mt(a, rows, ncols, vp, v.shape[0], op, int(threads)) < 1:
            raise RuntimeError("oracle: could not start threads")
    else:
        lib().rsr_oracle_matvec_i8(a, rows, ncols, vp, v.shape[0], op)
    return out[0] if squeeze else out


def host_threads() -> int:
    """Threads the timing harness may use: the CPUs this process is allowed to run on."""
    try:
        return max(1, len(os.sched_getaffinity(0)))
    except AttributeError:  # pragma: no cover
        return max(1, os.cpu_count() or 1)
