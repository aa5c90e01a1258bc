"""ctypes front end of the plain-C SpMM oracle (``spmm_oracle.c``).

TEST INFRASTRUCTURE ONLY.  Computes the definition of the sparse-dense product
(paper, Section 2.2) with binary16 operands (Section 4.1, Problem
Configuration) widened exactly to fp64 and summed in fp64.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "spmm_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain -O2, OpenMP for row parallelism)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11",
                               "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        lib.oracle_spmm.restype = ctypes.c_int
        lib.oracle_spmm.argtypes = [ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                    ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p, ctypes.c_int64,
                                    ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int]
        lib.oracle_half_to_double.restype = None
        lib.oracle_half_to_double.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p]
        _lib = lib
    return _lib


def half_bits_to_double(bits: np.ndarray) -> np.ndarray:
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    out = np.empty(bits.shape, dtype=np.float64)
    _load().oracle_half_to_double(bits.ctypes.data, bits.size, out.ctypes.data)
    return out


def spmm(row_ptr, col_idx, val_f16, B_f16, rows=None, want_scale=True, threads=0):
    """C = A @ B in fp64, plus S = |A| @ |B|.

    row_ptr int64 [n_rows+1]; col_idx int32 [nnz]; val_f16 float16 [nnz];
    B_f16 float16 [n_cols, N] row-major.  ``rows`` (optional int64 list)
    restricts the computation to those output rows.
    Returns (C, S, threads_used); S is None when ``want_scale`` is False.
    """
    row_ptr = np.ascontiguousarray(row_ptr, dtype=np.int64)
    col_idx = np.ascontiguousarray(col_idx, dtype=np.int32)
    val = np.ascontiguousarray(val_f16, dtype=np.float16)
    B = np.ascontiguousarray(B_f16, dtype=np.float16)
    assert B.ndim == 2
    n_rows = row_ptr.shape[0] - 1
    N = B.shape[1]
    if col_idx.size:
        assert 0 <= int(col_idx.min()) and int(col_idx.max()) < B.shape[0]
    if rows is not None:
        rows = np.ascontiguousarray(rows, dtype=np.int64)
        n_out = rows.shape[0]
        rows_p, n_sel = rows.ctypes.data, n_out
    else:
        n_out, rows_p, n_sel = n_rows, None, 0
    C = np.empty((n_out, N), dtype=np.float64)
    S = np.empty((n_out, N), dtype=np.float64) if want_scale else None
    used = _load().oracle_spmm(n_rows, row_ptr.ctypes.data, col_idx.ctypes.data, val.ctypes.data,
                               B.ctypes.data, N, rows_p, n_sel, C.ctypes.data,
                               S.ctypes.data if want_scale else None, int(threads))
    return C, S, used
