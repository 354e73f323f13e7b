"""Software models of one mixed-precision matrix multiply-accumulate, D = A16 B16 + C32.

TEST INFRASTRUCTURE ONLY.  These are the two emulators of section "Avoiding RZ during Tensor Core accumulation":
every element product is formed in FP32 (exact for FP16 and BF16 inputs), the products are accumulated in FP64
with the accumulator's significand cut back to 25 bits after every addition, and the addition of C is rounded to
FP32 either to nearest (`mma_rn`) or toward zero (`mma_rz`, what the paper attributes to Tensor Cores).  They are
used to show which of the two the MI355X matrix unit resembles, and to re-run the paper's emulator experiment.
"""
from __future__ import annotations

import numpy as np


def _truncate_significand(x: np.ndarray, bits: int) -> np.ndarray:
    """Keeps the leading `bits` significand bits of FP64 values (truncation toward zero)."""
    m, e = np.frexp(x)                      # x = m * 2^e, 0.5 <= |m| < 1
    scaled = np.trunc(m * 2.0 ** bits)
    return np.ldexp(scaled, e - bits)


def _round_to_fp32(x: np.ndarray, mode: str) -> np.ndarray:
    near = x.astype(np.float32)
    if mode == "rn":
        return near
    if mode == "rz":
        too_big = np.abs(near.astype(np.float64)) > np.abs(x)
        return np.where(too_big, np.nextafter(near, np.float32(0.0)), near).astype(np.float32)
    raise ValueError("mode must be 'rn' or 'rz'")


def mma(A: np.ndarray, B: np.ndarray, C: np.ndarray, final: str = "rn") -> np.ndarray:
    """D = A B + C for A (m x k), B (k x n) holding FP16/BF16-representable values, C FP32 (m x n)."""
    A = np.asarray(A, dtype=np.float32)
    B = np.asarray(B, dtype=np.float32)
    acc = np.zeros((A.shape[0], B.shape[1]), dtype=np.float64)
    for k in range(A.shape[1]):
        prod = np.outer(A[:, k], B[k, :])                       # FP32 product, exact
        acc = _truncate_significand(acc + prod.astype(np.float64), 25)
    return _round_to_fp32(acc + np.asarray(C, dtype=np.float32).astype(np.float64), final)


def mma_rn(A, B, C):
    return mma(A, B, C, "rn")


def mma_rz(A, B, C):
    return mma(A, B, C, "rz")


def gemm_blocked(A, B, mma_fn, block_k: int = 8) -> np.ndarray:
    """A B computed as a chain of multiply-accumulates over k blocks of `block_k` (the last one may be shorter),
    k ascending, the FP32 accumulator fed back through C: what a kernel built on such an instruction does."""
    acc = np.zeros((A.shape[0], B.shape[1]), dtype=np.float32)
    for k0 in range(0, A.shape[1], block_k):
        acc = mma_fn(A[:, k0:k0 + block_k], B[k0:k0 + block_k, :], acc)
    return acc
