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


def fp16_terms(opA: np.ndarray, opB: np.ndarray, scaled: bool = True):
    """(A16 B16, dA16 B16 + A16 dB16, dA16 dB16) as FP64 matrices, before any 2^-11 / 2^-22 factor."""
    a, da = (p.astype(np.float64) for p in _split.split_fp16(opA, scaled=scaled))
    b, db = (p.astype(np.float64) for p in _split.split_fp16(opB, scaled=scaled))
    return a @ b, da @ b + a @ db, da @ db


def gemm_fp16_mode(opA: np.ndarray, opB: np.ndarray, products: int = 3, scaled: bool = True) -> np.ndarray:
    """op(A) op(B) through the FP16 pair split with 3 (the method) or 4 (Markidis) products.

    scaled=True is the paper's halfhalf (Eq. corr-5-1024 / corr-5-1024-reduce); scaled=False is Markidis'
    halfhalf (Eq. corr-5), where the residual is not multiplied by 2^11 and nothing is divided out."""
    main, corr, corr2 = fp16_terms(opA, opB, scaled)
    s = 2.0 ** -11 if scaled else 1.0
    out = main + corr * s
    if products == 4:
        out = out + corr2 * s * s
    elif products != 3:
        raise ValueError("products must be 3 or 4")
    return out


def gemm_plain(opA: np.ndarray, opB: np.ndarray, fmt: str) -> np.ndarray:
    """toFP16(A) toFP16(B) or toBF16(A) toBF16(B): one low-precision product, no correction."""
    if fmt == "fp16":
        return _split.to_fp16_rn(opA).astype(np.float64) @ _split.to_fp16_rn(opB).astype(np.float64)
    if fmt == "bf16":
        return (_split.bf16_bits_to_fp32(_split.to_bf16_rn_bits(opA)).astype(np.float64)
                @ _split.bf16_bits_to_fp32(_split.to_bf16_rn_bits(opB)).astype(np.float64))
    raise ValueError("fmt must be 'fp16' or 'bf16'")


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
