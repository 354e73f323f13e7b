"""FP64 reference and naive FP32 GEMM (C, via ctypes) plus the error metrics.

TEST INFRASTRUCTURE ONLY.  BLAS conventions: matrices are column-major numpy arrays of
shape (ld, cols) in Fortran order; C <- alpha * op(A) * op(B) + beta * C with op(A)
M x K and op(B) K x N.  This wrapper only slices, transposes and copies (no
arithmetic); the sums are formed in gemm_oracle.c.

Results are returned as logical M x N arrays (or len(rows) x N when a row subset is
asked for), float32 for the naive product and float64 for the reference.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

from . import build as _build

_lib = None


def _load():
    global _lib
    if _lib is None:
        path = _build.LIB if os.path.exists(_build.LIB) else _build.build()
        lib = ctypes.CDLL(path)
        i64, f32, f64, ptr = ctypes.c_int64, ctypes.c_float, ctypes.c_double, ctypes.c_void_p
        lib.oracle_gemm_fp32_naive.argtypes = [i64, i64, i64, f32, ptr, ptr, f32, ptr, ptr]
        lib.oracle_gemm_fp32_naive.restype = None
        lib.oracle_gemm_fp64_ref.argtypes = [i64, i64, i64, f64, ptr, ptr, f64, ptr, ptr]
        lib.oracle_gemm_fp64_ref.restype = None
        lib.oracle_num_threads.argtypes = []
        lib.oracle_num_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def num_threads() -> int:
    """OpenMP threads the C loops will use."""
    return int(_load().oracle_num_threads())


def logical(op: str, X: np.ndarray, rows: int, cols: int) -> np.ndarray:
    """op(X) as a rows x cols view of the column-major store X (shape (ld, stored_cols))."""
    if op == "N":
        return X[:rows, :cols]
    if op == "T":
        return X[:cols, :rows].T
    raise ValueError("op must be 'N' or 'T'")


def _operands(transA, transB, M, N, K, A, B, C, beta, rows):
    opA = logical(transA, A, M, K)
    opB = logical(transB, B, K, N)
    Cin = None
    if rows is not None:
        opA = opA[rows, :]
    if beta != 0:
        if C is None:
            raise ValueError("beta != 0 needs C")
        Cin = C[:M, :N]
        if rows is not None:
            Cin = Cin[rows, :]
        Cin = np.ascontiguousarray(Cin, dtype=np.float32)
    opA = np.ascontiguousarray(opA, dtype=np.float32)
    opB = np.ascontiguousarray(opB, dtype=np.float32)
    return opA, opB, Cin


def sgemm_fp32_naive(transA, transB, M, N, K, alpha, A, B, beta=0.0, C=None, rows=None):
    """Naive FP32 product: one FP32 running sum per element, k ascending, no FMA."""
    opA, opB, Cin = _operands(transA, transB, M, N, K, A, B, C, beta, rows)
    out = np.empty((opA.shape[0], N), dtype=np.float32)
    _load().oracle_gemm_fp32_naive(opA.shape[0], N, K, float(alpha), opA.ctypes.data, opB.ctypes.data,
                                   float(beta), None if Cin is None else Cin.ctypes.data, out.ctypes.data)
    return out


def sgemm_fp64_ref(transA, transB, M, N, K, alpha, A, B, beta=0.0, C=None, rows=None):
    """FP64 reference on the FP32 inputs (C_FP64 of Eq. eval-matmul, with alpha/beta in FP64)."""
    opA, opB, Cin = _operands(transA, transB, M, N, K, A, B, C, beta, rows)
    out = np.empty((opA.shape[0], N), dtype=np.float64)
    _load().oracle_gemm_fp64_ref(opA.shape[0], N, K, float(alpha), opA.ctypes.data, opB.ctypes.data,
                                 float(beta), None if Cin is None else Cin.ctypes.data, out.ctypes.data)
    return out


def relative_residual(c64: np.ndarray, target: np.ndarray) -> float:
    """||C_FP64 - C_target||_F / ||C_FP64||_F (Eq. eval-matmul), norms summed in FP64."""
    c64 = np.asarray(c64, dtype=np.float64)
    diff = c64 - np.asarray(target, dtype=np.float64)
    num = np.sqrt(np.sum(diff * diff))
    den = np.sqrt(np.sum(c64 * c64))
    return float(num / den)


def max_deviation(c64: np.ndarray, target: np.ndarray) -> float:
    """max_ij |C_FP64 - C_target|."""
    return float(np.max(np.abs(np.asarray(c64, dtype=np.float64) - np.asarray(target, dtype=np.float64))))
