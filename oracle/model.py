"""The split-and-correct product written out step by step, with exact accumulation.

TEST INFRASTRUCTURE ONLY.  These are diagnostic models, not the pass/fail oracle: they
say what the method would return if the only error left were the split itself (and the
dropped terms), because every partial product of two 11-bit (or 8-bit) significands is
exact and the sums here run in FP64.  The GPU result differs from them only by its FP32
accumulation order, which gives an element-wise bound.

FP16 mode (Eq. corr-5-1024-reduce):
    C = A16 B16 + (dA16 B16 + A16 dB16) / 2^11            (dA16 dB16 / 2^22 dropped)
Markidis' four-product form (Eq. corr-5 / corr-5-1024) is available for the
dropped-term pin.
BF16 mode (a = a0 + a1 + a2, b likewise; terms grouped by order of magnitude):
    C = a0 b0 + (a0 b1 + a1 b0) + (a1 b1 + a0 b2 + a2 b0)  (a1 b2, a2 b1, a2 b2 dropped)
"""
from __future__ import annotations

import numpy as np

from . import split as _split


def fp16_terms(opA: np.ndarray, opB: np.ndarray):
    """(A16 B16, dA16 B16 + A16 dB16, dA16 dB16) as FP64 matrices, unscaled by 2^-11 / 2^-22."""
    a, da = (p.astype(np.float64) for p in _split.split_fp16(opA))
    b, db = (p.astype(np.float64) for p in _split.split_fp16(opB))
    return a @ b, da @ b + a @ db, da @ db


def gemm_fp16_mode(opA: np.ndarray, opB: np.ndarray, products: int = 3) -> np.ndarray:
    """op(A) op(B) through the halfhalf split with 3 (the method) or 4 (Markidis) products."""
    main, corr, corr2 = fp16_terms(opA, opB)
    out = main + corr * 2.0 ** -11
    if products == 4:
        out = out + corr2 * 2.0 ** -22
    elif products != 3:
        raise ValueError("products must be 3 or 4")
    return out


def gemm_bf16_mode(opA: np.ndarray, opB: np.ndarray, products: int = 6) -> np.ndarray:
    """op(A) op(B) through the three-term BF16 split with 6 (the method) or all 9 products."""
    a = [_split.bf16_bits_to_fp32(p).astype(np.float64) for p in _split.split_bf16x3(opA)]
    b = [_split.bf16_bits_to_fp32(p).astype(np.float64) for p in _split.split_bf16x3(opB)]
    out = a[0] @ b[0] + (a[0] @ b[1] + a[1] @ b[0]) + (a[1] @ b[1] + a[0] @ b[2] + a[2] @ b[0])
    if products == 9:
        out = out + (a[1] @ b[2] + a[2] @ b[1]) + a[2] @ b[2]
    elif products != 6:
        raise ValueError("products must be 6 or 9")
    return out
