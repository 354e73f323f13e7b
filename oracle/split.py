"""Element splits of an FP32 value into low-precision parts, in numpy.

TEST INFRASTRUCTURE ONLY.  Written from the paper's equations; shares nothing with the
HIP split kernel, for which `split_fp16` and `split_bf16x3` are the bit-exact reference.

halfhalf (Eqs. corr-elm-1 and corr-elm-2-1024):
    v16  = toFP16(v32)
    dv16 = toFP16((v32 - toFP32(v16)) * 2^11)          v32 ~ v16 + dv16 * 2^-11
Markidis' halfhalf (Eqs. corr-elm-1 and corr-elm-2): the same without the 2^11.
toFP16 rounds to nearest, ties to even (the paper's choice for FP16); an RZ variant
exists only because the paper's worked bit example and its underflow analysis assume
truncation.

Three-term BF16 split (stands where the paper uses TF32 for the full exponent range):
    b0 = toBF16(v); b1 = toBF16(v - b0); b2 = toBF16(v - b0 - b1),    v = b0 + b1 + b2
with round to nearest even; 8 + 8 + 8 significand bits cover FP32's 24.

Readings where the paper is silent (the HIP kernel follows the same ones):
  * saturation: a finite input never produces an infinite part.  toFP16 / toBF16 results
    that would round to +-Inf are replaced by the largest finite value of the format
    (65504 for FP16); the residual then carries the remainder.  The scaled residual
    saturates too: a residual beyond +-32 (whose 2^11-fold is beyond FP16 anyway) is cut
    to +-32 before the multiplication, so that the multiplication itself cannot overflow
    FP32 for inputs of magnitude 2^117 and more.
  * Inf input: the high part is +-Inf and every lower part is 0.  NaN: all parts NaN.
"""
from __future__ import annotations

import numpy as np

FP16_MAX = np.float32(65504.0)
RESIDUAL_SCALE = np.float32(2048.0)  # 2^(l_F16 + 1) = 2^11


def to_fp16_rn(x: np.ndarray) -> np.ndarray:
    """FP32 -> FP16, round to nearest even, finite inputs saturate at +-65504."""
    x = np.asarray(x, dtype=np.float32)
    with np.errstate(over="ignore", invalid="ignore"):
        h = x.astype(np.float16)
    overflowed = np.isinf(h) & np.isfinite(x)
    if np.any(overflowed):
        h = np.where(overflowed, np.copysign(np.float16(65504.0), h), h)
    return h


def to_fp16_rz(x: np.ndarray) -> np.ndarray:
    """FP32 -> FP16, round toward zero (truncate), subnormals included.  Finite |x| only."""
    x = np.asarray(x, dtype=np.float32)
    with np.errstate(over="ignore"):
        near = x.astype(np.float16)
    # stepping one FP16 toward zero whenever rounding to nearest went away from zero
    too_big = np.abs(near.astype(np.float32)) > np.abs(x)
    toward_zero = np.nextafter(near, np.float16(0.0))
    out = np.where(too_big, toward_zero, near)
    return np.where(np.isinf(out), np.copysign(np.float16(65504.0), out), out).astype(np.float16)


def split_fp16(x: np.ndarray, scaled: bool = True, rounding: str = "rn"):
    """halfhalf split.  Returns (v16, dv16) as float16 arrays.

    scaled=True  : the paper's halfhalf, residual multiplied by 2^11 before conversion
    scaled=False : Markidis' halfhalf
    rounding     : "rn" (method) or "rz" (only for the paper's RZ analysis)
    """
    x = np.asarray(x, dtype=np.float32)
    conv = {"rn": to_fp16_rn, "rz": to_fp16_rz}[rounding]
    v16 = conv(x)
    with np.errstate(invalid="ignore", over="ignore"):
        residual = x - v16.astype(np.float32)
        if scaled:
            residual = np.clip(residual, np.float32(-32.0), np.float32(32.0)) * RESIDUAL_SCALE   # NaN stays NaN
        dv16 = conv(residual)
    dv16 = np.where(np.isinf(v16), np.float16(0.0), dv16).astype(np.float16)
    return v16, dv16


def fp16_pair_value(v16: np.ndarray, dv16: np.ndarray, scaled: bool = True) -> np.ndarray:
    """What the pair stands for, in FP64: v16 + dv16 * 2^-11 (or v16 + dv16)."""
    s = 2.0 ** -11 if scaled else 1.0
    return v16.astype(np.float64) + dv16.astype(np.float64) * s


def fp16_pair_lost_fraction(x: np.ndarray) -> float:
    """|x - (v16 + dv16 2^-11)|_F / |x|_F in FP64: how much of an operand the halfhalf pair fails to represent.

    The quantity behind the library's automatic choice between the FP16 pair and the full-range mode (the trade-off
    of section "Effect of the exponent range of input matrices", taken from the data instead of left to the user).
    0 for an all-zero operand; NaN if the operand holds a NaN."""
    x = np.asarray(x, dtype=np.float32)
    exact = x.astype(np.float64)
    with np.errstate(invalid="ignore", over="ignore"):
        lost = exact - fp16_pair_value(*split_fp16(x))
        err2, norm2 = float(np.sum(lost * lost)), float(np.sum(exact * exact))
    if norm2 == 0.0 and err2 == 0.0:
        return 0.0
    return float(np.sqrt(err2 / norm2)) if np.isfinite(err2) and np.isfinite(norm2) else float("nan")


def fp16_pair_represents(opA: np.ndarray, opB: np.ndarray, tolerance: float = 2.0 ** -24) -> bool:
    """The automatic choice: True (FP16 pair) iff both operands lose at most `tolerance`, relative, in the Frobenius norm.

    2^-24 is the unit roundoff of FP32: the pair must represent each operand as well as FP32 rounding would have.
    A NaN (comparison false) or a value beyond the FP16 range (lost fraction near 1) gives False."""
    return bool(fp16_pair_lost_fraction(opA) <= tolerance and fp16_pair_lost_fraction(opB) <= tolerance)


def row_scale_exponents(x: np.ndarray, target: int = 14) -> np.ndarray:
    """Per-row power-of-two scaling (the remedy named at the end of section "Effect of the exponent range of input
    matrices", applied row by row): for each row of x the exponent e that moves the row's largest non-zero finite
    element into the binade 2^target, i.e. target - floor(log2 max|x|), with FP32 subnormals counted as 2^-127, kept
    within [-126, 126]; 0 for a row without such an element."""
    x = np.atleast_2d(np.asarray(x, dtype=np.float32))
    field = ((x.view(np.uint32) >> np.uint32(23)) & np.uint32(0xFF)).astype(np.int64)      # biased exponent
    counts = (x != 0) & (field != 255)
    top = np.where(counts, field - 127, -(1 << 40)).max(axis=1)
    return np.where(top > -(1 << 40), np.clip(target - top, -126, 126), 0).astype(np.int64)


def scale_rows(x: np.ndarray, exponents: np.ndarray) -> np.ndarray:
    """x with row r multiplied by 2^exponents[r], in FP32 (exact unless the result leaves the normal range)."""
    x = np.atleast_2d(np.asarray(x, dtype=np.float32))
    with np.errstate(over="ignore", under="ignore", invalid="ignore"):
        return (x * np.ldexp(np.float32(1.0), np.asarray(exponents, dtype=np.int32))[:, None]).astype(np.float32)


def participation(x: np.ndarray) -> float:
    """(sum |x|)^2 / (rows sum x^2) in FP64: about how many elements of a row of x carry the row's weight (rows of
    equal elements give the row length, a row with one non-zero element gives 1).  Infinite for an all-zero x."""
    x = np.atleast_2d(np.asarray(x, dtype=np.float32)).astype(np.float64)
    with np.errstate(invalid="ignore", over="ignore", divide="ignore"):
        norm2 = float(np.sum(x * x))
        return float("inf") if norm2 == 0.0 else float(np.sum(np.abs(x)) ** 2 / (x.shape[0] * norm2))


def fp16_pair_suffices(rows_a: np.ndarray, rows_b: np.ndarray, tolerance: float = 2.0 ** -24, min_terms: float = 16.0) -> bool:
    """The test both candidates of the automatic mode have to pass, on op(A) (M x K) and op(B)^T (N x K) as they
    would be split: the pair represents both to within `tolerance` (fp16_pair_represents), and at least one of them
    spreads a row's weight over `min_terms` elements or more.  The pair holds 22.75 of FP32's 24 bits (the paper's
    mantissa-length table); that is as good as an FP32 product only where the product's own summation error
    outweighs the missing bit, i.e. not for dot products carried by a handful of terms (the small-k end of the
    paper's error-against-k figure)."""
    if not fp16_pair_represents(rows_a, rows_b, tolerance):
        return False
    return bool(participation(rows_a) >= min_terms or participation(rows_b) >= min_terms)


def automatic_choice(opA: np.ndarray, opB: np.ndarray, tolerance: float = 2.0 ** -24, target: int = 14,
                     min_terms: float = 16.0) -> str:
    """What the library's automatic mode runs for op(A) (M x K) and op(B) (K x N): "fp16" if the pair suffices for
    both operands as they are; else "fp16 scaled" if it suffices once every row of op(A) and every column of op(B)
    has its largest binade at 2^target; else "bf16"."""
    bt = np.asarray(opB, dtype=np.float32).T
    if fp16_pair_suffices(opA, bt, tolerance, min_terms):
        return "fp16"
    scaled_a = scale_rows(opA, row_scale_exponents(opA, target))
    scaled_b = scale_rows(bt, row_scale_exponents(bt, target))
    return "fp16 scaled" if fp16_pair_suffices(scaled_a, scaled_b, tolerance, min_terms) else "bf16"


BF16_MAX_BITS = np.uint32(0x7F7F)


def to_bf16_rn_bits(x: np.ndarray) -> np.ndarray:
    """FP32 -> BF16 bit pattern (uint16), round to nearest even, finite inputs saturate."""
    x = np.asarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    with np.errstate(over="ignore"):
        rounded = (u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    sign = (u >> np.uint32(16)) & np.uint32(0x8000)
    exp_all_ones = (rounded & np.uint32(0x7F80)) == np.uint32(0x7F80)
    finite_in = np.isfinite(x)
    rounded = np.where(exp_all_ones & finite_in, sign | BF16_MAX_BITS, rounded)
    rounded = np.where(np.isnan(x), sign | np.uint32(0x7FC0), rounded)
    rounded = np.where(np.isinf(x), sign | np.uint32(0x7F80), rounded)
    return rounded.astype(np.uint16)


def bf16_bits_to_fp32(b: np.ndarray) -> np.ndarray:
    return (np.asarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def split_bf16x3(x: np.ndarray):
    """Three-term BF16 split.  Returns (b0, b1, b2) as uint16 BF16 bit patterns."""
    x = np.asarray(x, dtype=np.float32)
    b0 = to_bf16_rn_bits(x)
    with np.errstate(invalid="ignore", over="ignore"):
        r1 = x - bf16_bits_to_fp32(b0)
        b1 = to_bf16_rn_bits(r1)
        r2 = r1 - bf16_bits_to_fp32(b1)
        b2 = to_bf16_rn_bits(r2)
    is_inf = np.isinf(x)
    if np.any(is_inf):
        b1 = np.where(is_inf, np.uint16(0), b1).astype(np.uint16)
        b2 = np.where(is_inf, np.uint16(0), b2).astype(np.uint16)
    return b0, b1, b2


def bf16_triple_value(b0, b1, b2) -> np.ndarray:
    """b0 + b1 + b2 in FP64."""
    return (bf16_bits_to_fp32(b0).astype(np.float64) + bf16_bits_to_fp32(b1).astype(np.float64)
            + bf16_bits_to_fp32(b2).astype(np.float64))
