"""Seeded synthetic input generators shared by the tests, the bench and the smoke run.

This module holds no arithmetic of the GEMM method: it only draws matrices.  Every
element is a pure function of (seed, matrix_id, linear index) through a SplitMix64
counter hash, so any element can be regenerated on its own and the CPU oracle and the
GPU path are always fed bit-identical inputs.

Matrices are handed out the way BLAS stores them: column-major with a leading dimension,
as a numpy array of shape (ld, cols) in Fortran order, float32.  Rows >= `rows` (the
padding between `rows` and `ld`) are filled with NaN on purpose: a routine that reads
the padding shows up at once.

Distributions (Accuracy evaluation section of the paper):
  urand(-1, 1)     uniform in (-1, 1), rounded to nearest float32 from a 53-bit draw,
                   so every binade carries a full 23-bit mantissa
  exp_rand(a, b)   (2s-1) * 2^e * m with e uniform integer in [a, b], m uniform in
                   [1, 2) over all 2^23 mantissas, s a fair sign bit (Eq. exp-rand)
"""
from __future__ import annotations

import numpy as np

_CHUNK = 1 << 24
_U64 = np.uint64


def _splitmix64(x: np.ndarray) -> np.ndarray:
    """SplitMix64 finaliser applied to a uint64 counter array (wraps modulo 2^64)."""
    with np.errstate(over="ignore"):
        z = x + _U64(0x9E3779B97F4A7C15)
        z = (z ^ (z >> _U64(30))) * _U64(0xBF58476D1CE4E5B9)
        z = (z ^ (z >> _U64(27))) * _U64(0x94D049BB133111EB)
        return z ^ (z >> _U64(31))


def _counter_base(seed: int, matrix_id: int) -> int:
    if not (0 <= seed < (1 << 20)) or not (0 <= matrix_id < 16):
        raise ValueError("seed must be in [0, 2^20) and matrix_id in [0, 16)")
    return (seed << 40) + (matrix_id << 36)


def _draw_flat(kind: str, n: int, seed: int, matrix_id: int, lo: int, hi: int) -> np.ndarray:
    out = np.empty(n, dtype=np.float32)
    base = _counter_base(seed, matrix_id)
    for start in range(0, n, _CHUNK):
        stop = min(n, start + _CHUNK)
        ctr = np.arange(start, stop, dtype=np.uint64) + _U64(base)
        z = _splitmix64(ctr)
        if kind == "urand":
            u = (z >> _U64(11)).astype(np.float64) * (2.0 ** -52) - 1.0
            out[start:stop] = u.astype(np.float32)
        elif kind == "exp_rand":
            span = hi - lo + 1
            mant = (z & _U64(0x7FFFFF)).astype(np.uint32)
            sign = ((z >> _U64(23)) & _U64(1)).astype(np.uint32)
            e = ((z >> _U64(32)) % _U64(span)).astype(np.int64) + lo
            bits = (sign << np.uint32(31)) | ((e + 127).astype(np.uint32) << np.uint32(23)) | mant
            out[start:stop] = bits.view(np.float32)
        elif kind == "randint":
            span = hi - lo + 1
            out[start:stop] = (((z >> _U64(32)) % _U64(span)).astype(np.int64) + lo).astype(np.float32)
        else:
            raise ValueError(kind)
    return out


def _as_colmajor(flat: np.ndarray, rows: int, cols: int, ld: int | None) -> np.ndarray:
    """Place a rows*cols column-major flat draw into an (ld, cols) Fortran array."""
    ld = rows if ld is None else ld
    if ld < max(rows, 1):
        raise ValueError("ld < rows")
    store = np.full((ld, cols), np.nan, dtype=np.float32, order="F")
    store[:rows, :] = flat.reshape((rows, cols), order="F")
    return store


def urand(rows: int, cols: int, seed: int, matrix_id: int, ld: int | None = None) -> np.ndarray:
    """rows x cols matrix of uniform(-1, 1) float32 values, column-major, leading dim ld."""
    return _as_colmajor(_draw_flat("urand", rows * cols, seed, matrix_id, 0, 0), rows, cols, ld)


def exp_rand(rows: int, cols: int, a: int, b: int, seed: int, matrix_id: int,
             ld: int | None = None) -> np.ndarray:
    """rows x cols matrix drawn from exp_rand(a, b); needs -126 <= a <= b <= 127."""
    if not (-126 <= a <= b <= 127):
        raise ValueError("exponent range must stay inside the normal float32 range")
    return _as_colmajor(_draw_flat("exp_rand", rows * cols, seed, matrix_id, a, b), rows, cols, ld)


def randint(rows: int, cols: int, lo: int, hi: int, seed: int, matrix_id: int,
            ld: int | None = None) -> np.ndarray:
    """rows x cols matrix of integers uniform in [lo, hi], stored as float32."""
    return _as_colmajor(_draw_flat("randint", rows * cols, seed, matrix_id, lo, hi), rows, cols, ld)


def sample_indices(n: int, count: int, seed: int) -> np.ndarray:
    """`count` distinct sorted indices out of range(n), reproducible from `seed`."""
    count = min(count, n)
    keys = _splitmix64(np.arange(n, dtype=np.uint64) + _U64(_counter_base(seed, 15)))
    return np.sort(np.argsort(keys, kind="stable")[:count]).astype(np.int64)


def stratified_indices(n: int, stride: int, seed: int) -> np.ndarray:
    """One index out of every block of `stride` consecutive ones in range(n) (the last block may be shorter),
    sorted, reproducible from `seed`: a sample of rows that leaves no tile row of C out."""
    starts = np.arange(0, n, stride, dtype=np.int64)
    sizes = np.minimum(stride, n - starts)
    keys = _splitmix64(starts.astype(np.uint64) + _U64(_counter_base(seed, 14)))
    return starts + (keys % sizes.astype(np.uint64)).astype(np.int64)


# Matrix ids used throughout: keep A, B and C draws of one problem independent.
ID_A, ID_B, ID_C = 0, 1, 2
