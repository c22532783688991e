"""fp64 CPU oracle of Y = W_bcr * X (thin ctypes front end of bcr_oracle.c).

TEST INFRASTRUCTURE ONLY -- see the header of bcr_oracle.c.  The arithmetic
lives in the C file (mask a dense matrix by the BCR rule of Section 3.2, then
a naive triple loop following the GEMM view of Section 3.1); this module only
marshals NumPy arrays.

Pins (tests/test_oracle_pins.py): brute force by an independent per-block loop
nest, dense / one-block / 1x1-block special cases against numpy.matmul and
scipy.sparse, a hand-worked fixture, integer-exactness, linearity and column
permutation invariants, and the survivor-count closed form of Section 3.2.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "bcr_oracle.c")
_LIB = os.path.join(_HERE, "libbcr_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile bcr_oracle.c with gcc (OpenMP) into libbcr_oracle.so."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        i64, i32, p = ctypes.c_int64, ctypes.c_int32, ctypes.c_void_p
        lib.bcr_oracle_mask.argtypes = [p, i64, i64, i32, i32, p, p, p, p, p]
        lib.bcr_oracle_mask.restype = ctypes.c_int
        lib.bcr_oracle_matmul.argtypes = [p, p, i64, i64, i64, p, p, i32]
        lib.bcr_oracle_matmul.restype = ctypes.c_int
        lib.bcr_oracle_threads.restype = i32
        _lib = lib
    return _lib


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def threads() -> int:
    return int(_load().bcr_oracle_threads())


def masked_dense(W64: np.ndarray, BR: int, BC: int, row_ptr, row_idx, col_ptr, col_idx) -> np.ndarray:
    """Dense fp64 W_bcr: survivors keep their value, everything else is +0.0."""
    W64 = np.ascontiguousarray(W64, dtype=np.float64)
    M, K = W64.shape
    row_ptr = np.ascontiguousarray(row_ptr, dtype=np.int32)
    col_ptr = np.ascontiguousarray(col_ptr, dtype=np.int32)
    row_idx = np.ascontiguousarray(row_idx, dtype=np.uint16)
    col_idx = np.ascontiguousarray(col_idx, dtype=np.uint16)
    nb = (M // BR) * (K // BC) if BR > 0 and BC > 0 else -1
    if M % BR or K % BC or row_ptr.shape[0] != nb + 1 or col_ptr.shape[0] != nb + 1:
        raise ValueError("block size must divide the matrix and ptr arrays must have nb+1 entries")
    out = np.empty_like(W64)
    rc = _load().bcr_oracle_mask(_ptr(W64), M, K, BR, BC, _ptr(row_ptr), _ptr(row_idx),
                                 _ptr(col_ptr), _ptr(col_idx), _ptr(out))
    if rc != 0:
        raise ValueError("bcr_oracle_mask rejected its arguments")
    return out


def matmul(Wm64: np.ndarray, X64: np.ndarray, want_scale: bool = True,
           skip_zero: bool = True) -> Tuple[np.ndarray, Optional[np.ndarray]]:
    """(Y, S) with Y = Wm @ X by the triple loop and S = |Wm| @ |X| termwise."""
    Wm64 = np.ascontiguousarray(Wm64, dtype=np.float64)
    X64 = np.ascontiguousarray(X64, dtype=np.float64)
    M, K = Wm64.shape
    K2, N = X64.shape
    if K != K2:
        raise ValueError("inner dimensions differ")
    Y = np.empty((M, N), dtype=np.float64)
    S = np.empty((M, N), dtype=np.float64) if want_scale else None
    rc = _load().bcr_oracle_matmul(_ptr(Wm64), _ptr(X64), M, K, N, _ptr(Y), _ptr(S), int(skip_zero))
    if rc != 0:
        raise ValueError("bcr_oracle_matmul rejected its arguments")
    return Y, S


def bcr_product(W64, X64, mask, want_scale: bool = True, skip_zero: bool = True,
                rows: Optional[np.ndarray] = None, cols: Optional[np.ndarray] = None):
    """Y = W_bcr * X for a mask object carrying M, K, BR, BC and the four index
    arrays.  ``rows`` / ``cols`` restrict the computed outputs to a sample
    (Y[rows][:, cols]); the definition of each sampled entry is unchanged."""
    Wm = masked_dense(W64, mask.BR, mask.BC, mask.row_ptr, mask.row_idx, mask.col_ptr, mask.col_idx)
    X64 = np.asarray(X64, dtype=np.float64)
    if X64.ndim == 1:
        X64 = X64[:, None]
    if rows is not None:
        Wm = Wm[np.asarray(rows)]
    if cols is not None:
        X64 = X64[:, np.asarray(cols)]
    return matmul(Wm, X64, want_scale, skip_zero)
