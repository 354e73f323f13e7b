"""Pins for the CPU oracle: it is checked against what the paper prints and what the
mathematics fixes, never against itself and never against the GPU path.

Each test names the plausible oracle mistake it would catch.
"""
import json
import os
from fractions import Fraction

import numpy as np
import pytest

import seeded_inputs as si
from oracle import gemm, model, split

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _golden(name):
    with open(os.path.join(GOLDEN, name)) as f:
        return json.load(f)


def _binade(exponent: int, mantissas: np.ndarray) -> np.ndarray:
    """float32 values 1.m * 2^exponent for the given 23-bit mantissa integers."""
    bits = (np.uint32(exponent + 127) << np.uint32(23)) | mantissas.astype(np.uint32)
    return bits.view(np.float32)


ALL_MANTISSAS = np.arange(1 << 23, dtype=np.uint32)


# --------------------------------------------------------------------------- splits

def _kept_length(x: np.ndarray, reconstructed: np.ndarray) -> np.ndarray:
    """Mantissa bits kept (out of 23): 23 minus the bit length of the error in ulps of x."""
    ulp = np.spacing(np.abs(x)).astype(np.float64)
    err_ulps = np.rint(np.abs(x.astype(np.float64) - reconstructed) / ulp).astype(np.int64)
    lost = np.zeros_like(err_ulps)
    nz = err_ulps > 0
    lost[nz] = np.floor(np.log2(err_ulps[nz])).astype(np.int64) + 1
    return 23 - lost


@pytest.mark.parametrize("rounding", ["rn", "rz"])
def test_halfhalf_mantissa_length_table(rounding):
    """Exhaustive over one binade: the (len, prob) columns of the two mantissa tables and
    the expectations 22.75 / 22.25.  Catches a wrong rounding mode, a wrong scale and a
    residual taken against the wrong high part."""
    table = _golden("mantissa_length_tables.json")[rounding]
    x = _binade(0, ALL_MANTISSAS)
    v16, dv16 = split.split_fp16(x, scaled=True, rounding=rounding)
    kept = _kept_length(x, split.fp16_pair_value(v16, dv16))
    n = x.size
    for length in (21, 22, 23):
        expected = Fraction(table.get(str(length), 0.0))
        assert Fraction(int(np.sum(kept == length)), n) == expected, (rounding, length)
    assert kept.min() >= 21
    assert float(np.mean(kept)) == table["expectation"]


def test_lsb_truncation_length():
    """Dropping the last FP32 mantissa bit keeps 22.5 bits on average (the comparison the
    paper draws against the 22.75 of the split).  Pins _kept_length itself."""
    table = _golden("mantissa_length_tables.json")["lsb_truncation"]
    x = _binade(3, ALL_MANTISSAS)
    truncated = (x.view(np.uint32) & np.uint32(0xFFFFFFFE)).view(np.float32)
    kept = _kept_length(x, truncated.astype(np.float64))
    assert float(np.mean(kept)) == table["expectation"]
    assert Fraction(int(np.sum(kept == 23)), x.size) == Fraction(table["23"])


def test_halfhalf_worked_example():
    """The 24-bit significand 10000000000'10000000000'11 of Eq. mantissa-example."""
    g = _golden("mantissa_split_example.json")
    I = int(g["I_FP32_bits"], 2)
    x = np.array([I * 2.0 ** -23], dtype=np.float32)
    assert float(x[0]) * 2 ** 23 == I
    # RZ: hi = 10000000000, lo = +10000000000 two places up, trailing "11" lost
    v16, dv16 = split.split_fp16(x, rounding="rz")
    hi_units = float(v16[0]) * 2 ** 23
    lo_units = float(dv16[0]) * 2.0 ** -11 * 2 ** 23
    assert hi_units == int(g["rz"]["hi_bits"], 2) * 2 ** 13
    assert lo_units == g["rz"]["lo_sign"] * int(g["rz"]["lo_bits_at_2"], 2) * 2 ** 2
    assert I - hi_units - lo_units == g["rz"]["loss_units"] == 0b11
    # RN: hi rounds up to 10000000001, lo is negative, one bit lost
    v16, dv16 = split.split_fp16(x, rounding="rn")
    hi_units = float(v16[0]) * 2 ** 23
    lo_units = float(dv16[0]) * 2.0 ** -11 * 2 ** 23
    assert hi_units == int(g["rn"]["hi_bits"], 2) * 2 ** 13
    assert lo_units == g["rn"]["lo_sign"] * int(g["rn"]["lo_bits_at_1"], 2) * 2 ** 1
    assert abs(I - hi_units - lo_units) == g["rn"]["loss_units"]


def test_halfhalf_residual_is_exact_and_one_ulp():
    """v - toFP32(v16) and the 2^11 scaling are exact, so the pair is off by at most one
    FP32 ulp wherever the scaled residual stays a normal FP16 number (2^-13 <= |v| < 2^15);
    one binade lower the residual goes subnormal and the error may reach two ulps."""
    x = si.exp_rand(1 << 20, 1, -13, 14, seed=3, matrix_id=0)[:, 0]
    v16, dv16 = split.split_fp16(x)
    r64 = x.astype(np.float64) - v16.astype(np.float64)
    r32 = x - v16.astype(np.float32)
    assert np.array_equal(r32.astype(np.float64), r64)
    assert np.array_equal((r32 * np.float32(2048)).astype(np.float64), r64 * 2048)
    err = np.abs(split.fp16_pair_value(v16, dv16) - x)
    assert np.all(err <= np.spacing(np.abs(x)).astype(np.float64))
    wide = np.abs(x) >= 2.0 ** -12                   # residual never subnormal here: the table's 3/4 holds
    frac_exact = np.mean(err[wide] == 0)
    assert abs(frac_exact - 0.75) < 3 * np.sqrt(0.75 * 0.25 / wide.sum())
    low = si.exp_rand(1 << 18, 1, -14, -14, seed=3, matrix_id=1)[:, 0]
    err_low = np.abs(split.fp16_pair_value(*split.split_fp16(low)) - low)
    assert 1.0 < np.max(err_low / np.spacing(np.abs(low))) <= 2.0


def _p_l0(n, l32=23, l16=10):
    if n < 0:
        return Fraction(0)
    if n < l32 - l16:
        return Fraction(1, 2 ** (n + 1))
    if n == l32 - l16:
        return Fraction(1, 2 ** (l32 - l16))
    return Fraction(0)


@pytest.mark.parametrize("scaled", [False, True])
def test_underflow_probabilities(scaled):
    """Eqs. up, prob_g_u and prob_u: probability that the residual of the (RZ) split lands in
    FP16's subnormal range or vanishes, per exponent e_v.  The residual only depends on the
    low 13 mantissa bits, so enumerating those gives the probabilities exactly.  With the
    2^11 scaling both curves move by 11 exponents.  Catches a wrong scale constant and an
    unscaled/scaled mix-up."""
    g = _golden("underflow_model.json")
    b16, l16, l32 = g["b_F16"], g["l_F16"], g["l_F32"]
    shift = g["scale_log2"] if scaled else 0
    low = np.arange(1 << (l32 - l16), dtype=np.uint32)
    high = np.uint32(0b1011001110) << np.uint32(l32 - l16)
    min_normal = 2.0 ** (-b16 + 1)
    for e_v in range(-14, 16):
        x = _binade(e_v, high | low)
        _, dv16 = split.split_fp16(x, scaled=scaled, rounding="rz")
        mag = np.abs(dv16.astype(np.float64))
        e_eff = e_v + shift
        first_gu = (e_eff - l16 + b16 - 2) + 1
        first_u = (e_eff + b16 - 2) + 1
        p_gu = sum(_p_l0(l) for l in range(max(first_gu, 0), l32 - l16 + 1))
        p_u = sum(_p_l0(l) for l in range(max(first_u, 0), l32 - l16 + 1))
        zero_residual = low == 0                     # the l0 = 13 case of Eq. up
        counts_zero_gu = first_gu <= l32 - l16
        counts_zero_u = first_u <= l32 - l16
        ev_gu = (mag < min_normal) & (~zero_residual | counts_zero_gu)
        ev_u = (mag == 0) & (~zero_residual | counts_zero_u)
        assert Fraction(int(ev_gu.sum()), low.size) == p_gu, (e_v, scaled)
        assert Fraction(int(ev_u.sum()), low.size) == p_u, (e_v, scaled)
    if scaled:
        # with the scaling no residual of a normal-range FP16 value is lost to zero
        assert p_u == 0


def test_bf16_triple_is_exact():
    """8 + 8 + 8 significand bits: b0 + b1 + b2 == v for every mantissa, at the centre and
    near both ends of the exponent range the full-range mode has to cover."""
    for e in (0, -100, 100, 127 - 1, -126 + 24):
        x = _binade(e, ALL_MANTISSAS[:: 7] if e not in (0,) else ALL_MANTISSAS)
        for sign in (1.0, -1.0):
            xs = (x * np.float32(sign)).astype(np.float32)
            assert np.array_equal(split.bf16_triple_value(*split.split_bf16x3(xs)), xs.astype(np.float64))
    x = si.exp_rand(1 << 20, 1, -100, 100, seed=5, matrix_id=0)[:, 0]
    b0, b1, b2 = split.split_bf16x3(x)
    assert np.array_equal(split.bf16_triple_value(b0, b1, b2), x.astype(np.float64))
    # the parts are ordered by magnitude: each at most half an ulp (2^-8) of the previous one
    f = [np.abs(split.bf16_bits_to_fp32(b).astype(np.float64)) for b in (b0, b1, b2)]
    assert np.all(f[1] <= f[0] * 2.0 ** -8) and np.all(f[2] <= f[0] * 2.0 ** -16)


def test_bf16_rounding_is_nearest_even():
    """toBF16 against hand-worked patterns: below half, tie to even (down and up), above half."""
    cases = {0x3F800000: 0x3F80, 0x3F807FFF: 0x3F80, 0x3F808000: 0x3F80, 0x3F808001: 0x3F81,
             0x3F818000: 0x3F82, 0x3F81FFFF: 0x3F82, 0xBF808001: 0xBF81, 0x7F7FFFFF: 0x7F7F,
             0x00000000: 0x0000, 0x80000000: 0x8000, 0x7F800000: 0x7F80, 0x00010000: 0x0001}
    x = np.array(list(cases.keys()), dtype=np.uint32).view(np.float32)
    assert split.to_bf16_rn_bits(x).tolist() == list(cases.values())
    assert np.all(np.isnan(split.bf16_bits_to_fp32(split.to_bf16_rn_bits(np.array([np.nan], np.float32)))))


def test_split_edge_values():
    """Saturation reading: a finite input never yields an infinite part, and the pair still
    reconstructs values up to 2^16 to better than 2^-22; Inf keeps only its high part."""
    x = np.array([65504.0, 65519.996, 65520.0, 65535.996, -65535.996, 0.0, -0.0, 2.0 ** -24, 2.0 ** -35,
                  1e-45], dtype=np.float32)
    v16, dv16 = split.split_fp16(x)
    assert np.all(np.isfinite(v16)) and np.all(np.isfinite(dv16))
    assert v16[3] == np.float16(65504) and v16[4] == np.float16(-65504)
    rec = split.fp16_pair_value(v16, dv16)
    assert np.all(np.abs(rec[:5] - x[:5]) <= np.abs(x[:5]) * 2.0 ** -22)
    assert rec[7] == x[7] and rec[8] == x[8]          # down to 2^-35 through the scaled residual
    assert rec[9] == 0.0                              # below that the pair holds nothing
    inf = np.array([np.inf, -np.inf], dtype=np.float32)
    v16, dv16 = split.split_fp16(inf)
    assert np.all(np.isinf(v16)) and np.all(dv16 == 0)
    b0, b1, b2 = split.split_bf16x3(inf)
    assert b0.tolist() == [0x7F80, 0xFF80] and not b1.any() and not b2.any()
    big = np.array([np.finfo(np.float32).max, -np.finfo(np.float32).max], dtype=np.float32)
    parts = split.split_bf16x3(big)
    assert np.all(np.isfinite(split.bf16_triple_value(*parts)))
    assert np.all(np.abs(split.bf16_triple_value(*parts) - big) <= np.abs(big) * 2.0 ** -22)
    # far outside the FP16 window both parts saturate; in particular the 2^11-fold of the residual, which would
    # overflow FP32 from 2^117 upward, does not turn into an infinity (an infinite part times a zero of the other
    # operand would put a NaN where the FP32 product is finite)
    huge = np.array([2.0 ** 116, 2.0 ** 117, -2.0 ** 117, 1e36, -1e38, np.finfo(np.float32).max, 100000.0, -1e30],
                    dtype=np.float32)
    v16, dv16 = split.split_fp16(huge)
    assert np.array_equal(v16, np.copysign(np.float16(65504), huge).astype(np.float16))
    assert np.array_equal(dv16, np.copysign(np.float16(65504), huge).astype(np.float16))
    v16, dv16 = split.split_fp16(huge, scaled=False)
    assert np.all(np.isfinite(v16)) and np.all(np.isfinite(dv16))


def test_the_saturating_splits_reduce_to_the_plain_equations_where_nothing_saturates():
    """Eqs. corr-1-1024 .. corr-4-1024 as printed have no clamps; the oracle's splits add them for values the format
    cannot hold.  Wherever plain round-to-nearest conversion of the input gives a finite high part (|x| < 65520 for
    FP16, |x| below the midpoint between the largest BF16 number and 2^128 for BF16), the clamps and the infinity
    rule must be inactive: the parts equal those of the printed equations written out with numpy's own conversions,
    bit for bit.  (The one-launch kernel relies on exactly this to split ordinary values without the clamps.)  Also
    the scaled residual as one fused operation, hi * -2^11 + x * 2^11 rounded once, is the two-step (x - hi) * 2^11."""
    rng = np.random.default_rng(3)
    x = np.concatenate([
        (rng.standard_normal(200000) * np.exp2(rng.uniform(-40, 15.9, 200000))).astype(np.float32),
        np.array([65504.0, 65519.996, -65519.996, 65505.0, 2.0 ** -14, 2.0 ** -24, 2.0 ** -25, 6.1e-5, 5.96e-8, 1e-41, 0.0, -0.0,
                  2.0 ** -126, 1.0, -3.0], dtype=np.float32)])
    x = x[np.abs(x) < np.float32(65520.0)]
    with np.errstate(over="ignore"):
        hi = x.astype(np.float16)
    assert np.all(np.isfinite(hi))
    residual = (x - hi.astype(np.float32)) * np.float32(2048.0)
    lo = residual.astype(np.float16)
    v16, dv16 = split.split_fp16(x)
    assert np.array_equal(v16.view(np.uint16), hi.view(np.uint16)) and np.array_equal(dv16.view(np.uint16), lo.view(np.uint16))
    fused = (hi.astype(np.float64) * -2048.0 + x.astype(np.float64) * 2048.0).astype(np.float32)   # exact in FP64, one rounding
    assert np.array_equal(fused.view(np.uint32), residual.view(np.uint32))
    # beyond that bound the two differ: the plain conversion overflows, the oracle saturates
    over = np.array([65520.0, -70000.0, 1e10], dtype=np.float32)
    with np.errstate(over="ignore"):
        assert np.all(np.isinf(over.astype(np.float16))) and np.all(np.isfinite(split.split_fp16(over)[0]))
    # the BF16 triple: plain nearest-even conversions (add half an ulp of the kept part, truncate) and plain residuals
    def bf16_plain(v):
        u = v.view(np.uint32).astype(np.uint64)
        return (((u + 0x7FFF + ((u >> 16) & 1)) >> 16) & 0xFFFF).astype(np.uint16)
    with np.errstate(over="ignore"):
        y = np.concatenate([(rng.standard_normal(200000) * np.exp2(rng.uniform(-120, 127, 200000))).astype(np.float32),
                            np.array([3.38e38, -3.38e38, 1e-45, 2.0 ** -126, 0.0, 1.0], dtype=np.float32)])
    y = y[np.isfinite(y)]
    y = y[(bf16_plain(y) & 0x7F80) != 0x7F80]               # the plain conversion stays finite
    assert len(y) > 190000
    b0 = bf16_plain(y)
    r1 = y - split.bf16_bits_to_fp32(b0)
    b1 = bf16_plain(r1)
    r2 = r1 - split.bf16_bits_to_fp32(b1)
    b2 = bf16_plain(r2)
    o0, o1, o2 = split.split_bf16x3(y)
    assert np.array_equal(o0, b0) and np.array_equal(o1, b1) and np.array_equal(o2, b2)


def test_split_of_nan_is_nan_in_every_part():
    """Reading for non-numbers: a NaN input gives a NaN in every part of either split (so that whichever products are
    kept, the NaN reaches C); an infinity keeps only its high part (pinned in test_split_edge_values)."""
    x = np.array([np.nan, -np.nan, 1.0, np.float32(np.nan)], dtype=np.float32)
    x[3] = np.array([0x7F800001], dtype=np.uint32).view(np.float32)[0]      # a signalling pattern
    is_nan = np.array([True, True, False, True])
    for scaled in (True, False):
        v16, dv16 = split.split_fp16(x, scaled=scaled)
        assert np.array_equal(np.isnan(v16), is_nan) and np.array_equal(np.isnan(dv16), is_nan)
    for part in split.split_bf16x3(x):
        assert np.array_equal(np.isnan(split.bf16_bits_to_fp32(part)), is_nan)
    assert np.isnan(split.fp16_pair_value(*split.split_fp16(x)))[is_nan].all()
    assert np.isnan(split.bf16_triple_value(*split.split_bf16x3(x)))[is_nan].all()


# ----------------------------------------------------------------------------- GEMMs

def _python_gemm_exact(opA, opB, alpha, beta, Cin):
    """alpha * op(A) op(B) + beta * C in exact rational arithmetic (tiny sizes only)."""
    M, K = opA.shape
    N = opB.shape[1]
    out = [[Fraction(0)] * N for _ in range(M)]
    for i in range(M):
        for j in range(N):
            s = Fraction(0)
            for k in range(K):
                s += Fraction(float(opA[i, k])) * Fraction(float(opB[k, j]))
            out[i][j] = Fraction(float(alpha)) * s + (Fraction(float(beta)) * Fraction(float(Cin[i, j])) if beta else 0)
    return out


def _python_gemm_fp32(opA, opB, alpha, beta, Cin):
    """The naive FP32 product in pure Python, np.float32 scalars, i-j-k loop order."""
    M, K = opA.shape
    N = opB.shape[1]
    out = np.zeros((M, N), dtype=np.float32)
    f = np.float32
    for i in range(M):
        for j in range(N):
            acc = f(0)
            for k in range(K):
                acc = f(acc + f(opA[i, k] * opB[k, j]))
            val = f(f(alpha) * acc)
            if beta != 0:
                val = f(val + f(f(beta) * Cin[i, j]))
            out[i, j] = val
    return out


TINY = [(1, 1, 1), (2, 3, 5), (5, 2, 3), (3, 5, 2), (8, 8, 8), (17, 5, 8), (4, 17, 9)]


@pytest.mark.parametrize("transA", ["N", "T"])
@pytest.mark.parametrize("transB", ["N", "T"])
def test_gemm_brute_force_tiny(transA, transB):
    """All transposes, padded leading dimensions, several alpha/beta: the FP64 reference
    against exact rational arithmetic, the naive FP32 product bit-for-bit against a pure
    Python loop.  Catches transposed operands, swapped M/N/K, wrong ld handling, a reading
    of C when beta == 0, fused multiply-adds."""
    for idx, (M, N, K) in enumerate(TINY):
        for alpha, beta in [(1.0, 0.0), (1.5, 0.5), (-1.0, 1.0), (0.0, 2.0), (1.0, -1.0)]:
            ar, ac = (M, K) if transA == "N" else (K, M)
            br, bc = (K, N) if transB == "N" else (N, K)
            A = si.urand(ar, ac, seed=idx, matrix_id=si.ID_A, ld=ar + 3)
            B = si.exp_rand(br, bc, -4, 4, seed=idx, matrix_id=si.ID_B, ld=br + 1)
            C = si.urand(M, N, seed=idx, matrix_id=si.ID_C, ld=M + 2)
            if beta == 0.0:
                C[:] = np.nan                       # must not be read
            opA, opB = gemm.logical(transA, A, M, K), gemm.logical(transB, B, K, N)
            c64 = gemm.sgemm_fp64_ref(transA, transB, M, N, K, alpha, A, B, beta, C)
            c32 = gemm.sgemm_fp32_naive(transA, transB, M, N, K, alpha, A, B, beta, C)
            exact = _python_gemm_exact(opA, opB, alpha, beta, C[:M, :N])
            mag = np.abs(alpha) * (np.abs(opA).astype(np.float64) @ np.abs(opB).astype(np.float64))
            if beta != 0:
                mag = mag + np.abs(beta * C[:M, :N].astype(np.float64))
            for i in range(M):
                for j in range(N):
                    assert abs(Fraction(float(c64[i, j])) - exact[i][j]) <= (K + 3) * 2.0 ** -53 * mag[i, j] + 1e-300
                    assert abs(Fraction(float(c32[i, j])) - exact[i][j]) <= (K + 3) * 2.0 ** -24 * mag[i, j] + 1e-40
            ref32 = _python_gemm_fp32(opA, opB, alpha, beta, C[:M, :N])
            assert np.array_equal(c32.view(np.uint32), ref32.view(np.uint32)), (M, N, K, alpha, beta)


def test_gemm_row_subset_matches_full():
    M, N, K = 37, 29, 53
    A = si.urand(K, M, 1, si.ID_A)
    B = si.urand(K, N, 1, si.ID_B)
    C = si.urand(M, N, 1, si.ID_C)
    rows = si.sample_indices(M, 9, seed=4)
    assert len(set(rows.tolist())) == 9
    for fn in (gemm.sgemm_fp32_naive, gemm.sgemm_fp64_ref):
        full = fn("T", "N", M, N, K, 1.5, A, B, 0.5, C)
        part = fn("T", "N", M, N, K, 1.5, A, B, 0.5, C, rows=rows)
        assert np.array_equal(full[rows], part)


def test_small_integers_are_exact():
    """Integer entries small enough that every partial sum is below 2^24: FP32, FP64 and the
    method models must all equal the integer product, whatever the summation order."""
    M, N, K = 24, 40, 512
    A = si.randint(M, K, -15, 15, seed=0, matrix_id=si.ID_A)
    B = si.randint(K, N, -15, 15, seed=0, matrix_id=si.ID_B)
    exact = A.astype(np.int64) @ B.astype(np.int64)
    assert np.abs(exact).max() < 2 ** 24
    assert np.array_equal(gemm.sgemm_fp32_naive("N", "N", M, N, K, 1.0, A, B).astype(np.int64), exact)
    assert np.array_equal(gemm.sgemm_fp64_ref("N", "N", M, N, K, 1.0, A, B).astype(np.int64), exact)
    assert np.array_equal(model.gemm_fp16_mode(A, B), exact.astype(np.float64))
    assert np.array_equal(model.gemm_bf16_mode(A, B), exact.astype(np.float64))
    # integers that need the low parts: up to 2^20 in A (FP16 residual / second BF16 term)
    A2 = si.randint(8, 64, -(2 ** 20), 2 ** 20, seed=1, matrix_id=si.ID_A)
    B2 = si.randint(64, 8, -7, 7, seed=1, matrix_id=si.ID_B)
    exact2 = A2.astype(np.int64) @ B2.astype(np.int64)
    assert np.array_equal(gemm.sgemm_fp64_ref("N", "N", 8, 8, 64, 1.0, A2, B2).astype(np.int64), exact2)
    assert np.array_equal(model.gemm_bf16_mode(A2, B2), exact2.astype(np.float64))


def test_fp64_reference_against_library_dgemm():
    M, N, K = 96, 80, 700
    A = si.exp_rand(M, K, -15, 14, 2, si.ID_A)
    B = si.exp_rand(N, K, -15, 14, 2, si.ID_B)
    c64 = gemm.sgemm_fp64_ref("N", "T", M, N, K, 1.0, A, B)
    lib = A.astype(np.float64) @ B.astype(np.float64).T
    bound = (np.abs(A).astype(np.float64) @ np.abs(B).astype(np.float64).T) * K * 2.0 ** -52
    assert np.all(np.abs(c64 - lib) <= bound)


def test_metric_definitions():
    """Eq. eval-matmul on a case worked by hand: C64 = [[3, 4]], target = [[3, 4.5]]."""
    c64 = np.array([[3.0, 4.0]])
    tgt = np.array([[3.0, 4.5]], dtype=np.float32)
    assert gemm.relative_residual(c64, tgt) == 0.5 / 5.0
    assert gemm.max_deviation(c64, tgt) == 0.5
    assert gemm.relative_residual(c64, c64) == 0.0


def test_fp32_error_grows_like_sqrt_k():
    """The experiment of the paper's first figure (A 16 x k, B k x 16, uniform(-1, 1)):
    the naive FP32 product's relative residual grows about as sqrt(k) * 2^-24, far below
    the worst-case bound k * 2^-24; the exact-accumulation models of both modes stay flat
    and below it.  Catches an oracle that accumulates in higher precision (too small an
    error) or fuses/reorders (wrong growth)."""
    ks = [2 ** p for p in range(4, 17, 2)]
    errs, floor16, floor_bf = [], [], []
    for k in ks:
        e, f16, fbf = [], [], []
        for seed in range(4):
            A = si.urand(16, k, seed, si.ID_A)
            B = si.urand(k, 16, seed, si.ID_B)
            c64 = gemm.sgemm_fp64_ref("N", "N", 16, 16, k, 1.0, A, B)
            e.append(gemm.relative_residual(c64, gemm.sgemm_fp32_naive("N", "N", 16, 16, k, 1.0, A, B)))
            f16.append(gemm.relative_residual(c64, model.gemm_fp16_mode(A, B)))
            fbf.append(gemm.relative_residual(c64, model.gemm_bf16_mode(A, B)))
        errs.append(np.mean(e)); floor16.append(np.mean(f16)); floor_bf.append(np.mean(fbf))
    u = 2.0 ** -24
    for k, e in zip(ks, errs):
        assert 0.02 * np.sqrt(k) * u <= e <= 1.0 * np.sqrt(k) * u, (k, e)
    slope = np.polyfit(np.log2(ks), np.log2(errs), 1)[0]
    assert 0.35 <= slope <= 0.65, slope
    assert max(floor16) < 2.0 * u and max(floor_bf) < 0.2 * u
    assert all(f < e for f, e in zip(floor16, errs))


def test_dropped_terms_are_negligible():
    """dA16 dB16 / 2^22 is at least 2^22 times smaller than A16 B16 in norm, and leaving it
    out does not move the relative residual; likewise the three BF16 products left out."""
    n = 256
    A = si.urand(n, n, 0, si.ID_A)
    B = si.urand(n, n, 0, si.ID_B)
    main, _, corr2 = model.fp16_terms(A, B)
    assert np.linalg.norm(corr2 * 2.0 ** -22) <= np.linalg.norm(main) * 2.0 ** -22
    c64 = gemm.sgemm_fp64_ref("N", "N", n, n, n, 1.0, A, B)
    r3 = gemm.relative_residual(c64, model.gemm_fp16_mode(A, B, 3))
    r4 = gemm.relative_residual(c64, model.gemm_fp16_mode(A, B, 4))
    r32 = gemm.relative_residual(c64, gemm.sgemm_fp32_naive("N", "N", n, n, n, 1.0, A, B))
    # the fourth product moves the result by less than a quarter ulp: far inside FP32's own error
    assert abs(r3 - r4) <= 2.0 ** -26 and abs(r3 - r4) <= 0.05 * r32 and r3 < r32
    r6 = gemm.relative_residual(c64, model.gemm_bf16_mode(A, B, 6))
    r9 = gemm.relative_residual(c64, model.gemm_bf16_mode(A, B, 9))
    assert r9 < 1e-12 and r6 < 2.0 ** -26


def test_models_reach_fp32_accuracy_in_their_exponent_ranges():
    """The paper's accuracy claims, checked on the exact-accumulation models: halfhalf matches
    FP32 for exp_rand(-15, 14) inputs and degrades for exp_rand(-35, -15); the full-range
    split (TF32 in the paper, three BF16 terms here) holds for exp_rand(-100, -35) x
    exp_rand(-15, 14), where halfhalf cannot work at all."""
    n = 192

    def run(a_rng, b_rng):
        A = si.exp_rand(n, n, *a_rng, 0, si.ID_A)
        B = si.exp_rand(n, n, *b_rng, 0, si.ID_B)
        c64 = gemm.sgemm_fp64_ref("N", "N", n, n, n, 1.0, A, B)
        r32 = gemm.relative_residual(c64, gemm.sgemm_fp32_naive("N", "N", n, n, n, 1.0, A, B))
        return r32, gemm.relative_residual(c64, model.gemm_fp16_mode(A, B)), \
            gemm.relative_residual(c64, model.gemm_bf16_mode(A, B))

    r32, r16, rbf = run((-15, 14), (-15, 14))          # Type 1
    assert r16 <= r32 and rbf <= r32
    r32, r16, rbf = run((-35, -15), (-35, -15))        # Type 3
    assert r16 > 3 * r32 and rbf <= r32
    r32, r16, rbf = run((-100, -35), (-15, 14))        # Type 2 / 4
    assert r16 > 0.1 and rbf <= r32          # above the 0.1 "broken kernel" threshold of the tuning section


def test_comparison_method_models():
    """Models of the methods the paper compares against.  Plain conversion: the relative residual is the
    conversion error: rounding to p fraction bits (10 for FP16, 7 for BF16) is off by a uniform +-2^-(p+1) of the
    binade, so per operand the relative rms is 2^-(p+1) / sqrt(3) * sqrt(E[1/m^2]) with m uniform in [1, 2)
    (E[1/m^2] = 1/2), and two operands give sqrt(2) times that: 2.8e-4 and 2.3e-3, independent of k.  Markidis' unscaled
    residual equals the scaled one wherever nothing underflows (inputs of magnitude >= 1 here), and loses
    accuracy on small inputs (exp_rand(-14, -8): the residual sits in FP16's subnormal range), where the scaled
    split does not: this is what the 2^11 of Eq. corr-elm-2-1024 is for."""
    n = 256
    A = si.exp_rand(n, n, -3, 3, 0, si.ID_A)
    B = si.exp_rand(n, n, -3, 3, 0, si.ID_B)
    c64 = gemm.sgemm_fp64_ref("N", "N", n, n, n, 1.0, A, B)
    r16 = gemm.relative_residual(c64, model.gemm_plain(A, B, "fp16"))
    rbf = gemm.relative_residual(c64, model.gemm_plain(A, B, "bf16"))
    assert 2.3e-4 <= r16 <= 3.3e-4 and 1.8e-3 <= rbf <= 2.7e-3
    big_a = si.exp_rand(n, n, 0, 3, 1, si.ID_A)
    big_b = si.exp_rand(n, n, 0, 3, 1, si.ID_B)
    for products in (3, 4):
        assert np.array_equal(model.gemm_fp16_mode(big_a, big_b, products, scaled=True),
                              model.gemm_fp16_mode(big_a, big_b, products, scaled=False))
    A = si.exp_rand(n, n, -14, -8, 2, si.ID_A)
    B = si.exp_rand(n, n, -14, -8, 2, si.ID_B)
    c64 = gemm.sgemm_fp64_ref("N", "N", n, n, n, 1.0, A, B)
    r32 = gemm.relative_residual(c64, gemm.sgemm_fp32_naive("N", "N", n, n, n, 1.0, A, B))
    r_scaled = gemm.relative_residual(c64, model.gemm_fp16_mode(A, B, 3, scaled=True))
    r_unscaled = gemm.relative_residual(c64, model.gemm_fp16_mode(A, B, 4, scaled=False))
    assert r_scaled < r32 < 0.1 * r_unscaled


def test_mma_emulators():
    """The paper's mma_rn / mma_rz emulators.  Pinned by exact integer products, by hand-worked single additions
    (1 + 0.75 ulp: RN gives 1 + ulp, RZ gives 1; 1 - 0.25 ulp(1-): RN gives 1, RZ gives the next value below 1) and
    by the paper's emulator experiment: Markidis' method through mma_rn is as accurate as the naive FP32 product,
    through mma_rz it is clearly worse."""
    from oracle import mma_emulator as emu
    rng = np.random.default_rng(0)
    A = rng.integers(-7, 8, (8, 8)).astype(np.float32)
    B = rng.integers(-7, 8, (8, 8)).astype(np.float32)
    C = rng.integers(-100, 100, (8, 8)).astype(np.float32)
    exact = (A.astype(np.int64) @ B.astype(np.int64) + C.astype(np.int64)).astype(np.float32)
    assert np.array_equal(emu.mma_rn(A, B, C), exact) and np.array_equal(emu.mma_rz(A, B, C), exact)
    ulp = 2.0 ** -23
    one = np.ones((1, 1), dtype=np.float32)
    a = np.array([[0.75 * 2.0 ** -10]], dtype=np.float32)
    b = np.array([[2.0 ** -13]], dtype=np.float32)
    assert emu.mma_rn(a, b, one)[0, 0] == np.float32(1 + ulp) and emu.mma_rz(a, b, one)[0, 0] == np.float32(1.0)
    assert emu.mma_rn(-a / 6, b, one)[0, 0] == np.float32(1.0) and emu.mma_rz(-a / 6, b, one)[0, 0] == np.float32(1 - ulp / 2)
    # Markidis' method (four products, one accumulator, unscaled residual) through both emulators
    k = 1024
    err = {"rn": [], "rz": [], "fp32": []}
    for seed in range(3):
        A32 = si.urand(16, k, seed, si.ID_A)
        B32 = si.urand(k, 16, seed, si.ID_B)
        a16, da16 = (p.astype(np.float32) for p in split.split_fp16(A32, scaled=False))
        b16, db16 = (p.astype(np.float32) for p in split.split_fp16(B32, scaled=False))
        c64 = gemm.sgemm_fp64_ref("N", "N", 16, 16, k, 1.0, A32, B32)
        for name, fn in (("rn", emu.mma_rn), ("rz", emu.mma_rz)):
            acc = np.zeros((16, 16), dtype=np.float32)
            for k0 in range(0, k, 8):
                s = slice(k0, k0 + 8)
                for x, y in ((da16, db16), (da16, b16), (a16, db16), (a16, b16)):
                    acc = fn(x[:, s], y[s, :], acc)
            err[name].append(gemm.relative_residual(c64, acc))
        err["fp32"].append(gemm.relative_residual(c64, gemm.sgemm_fp32_naive("N", "N", 16, 16, k, 1.0, A32, B32)))
    rn, rz, fp32 = (float(np.mean(err[n])) for n in ("rn", "rz", "fp32"))
    assert rn <= 1.25 * fp32 and rz > 2 * rn


def test_gemm_blocked_chains_the_blocks_in_ascending_k():
    """gemm_blocked: exact on small integers whatever the block depth (ragged last block included); equal to the chain
    of single multiply-accumulates written out by hand; and on a case where the order of the blocks decides the result
    (2^24, then 1, then -2^24: ascending gives 0 because 2^24 + 1 ties to 2^24; descending gives 1) it gives the
    ascending answer, with both emulators."""
    from oracle import mma_emulator as emu
    rng = np.random.default_rng(1)
    A = rng.integers(-7, 8, (5, 20)).astype(np.float32)
    B = rng.integers(-7, 8, (20, 3)).astype(np.float32)
    exact = (A.astype(np.int64) @ B.astype(np.int64)).astype(np.float32)
    for block_k in (1, 3, 8, 16, 20, 64):
        for fn in (emu.mma_rn, emu.mma_rz):
            assert np.array_equal(emu.gemm_blocked(A, B, fn, block_k), exact), block_k
    # the hand-written chain on values whose FP32 sum depends on the order
    A32 = si.urand(4, 40, 3, si.ID_A)
    B32 = si.urand(40, 4, 3, si.ID_B)
    a16 = split.to_fp16_rn(A32).astype(np.float32)
    b16 = split.to_fp16_rn(B32).astype(np.float32)
    for fn in (emu.mma_rn, emu.mma_rz):
        acc = np.zeros((4, 4), dtype=np.float32)
        for k0 in (0, 8, 16, 24, 32):
            acc = fn(a16[:, k0:k0 + 8], b16[k0:k0 + 8, :], acc)
        assert np.array_equal(emu.gemm_blocked(a16, b16, fn, 8), acc)
    # block order: one product per block
    a = np.array([[2.0 ** 12, 1.0, -2.0 ** 12]], dtype=np.float32)
    b = np.array([[2.0 ** 12], [1.0], [2.0 ** 12]], dtype=np.float32)
    for fn in (emu.mma_rn, emu.mma_rz):
        assert emu.gemm_blocked(a, b, fn, 1)[0, 0] == 0.0
        assert emu.gemm_blocked(a[:, ::-1], b[::-1, :], fn, 1)[0, 0] == 1.0


def test_fp16_pair_lost_fraction_and_the_automatic_choice():
    """The criterion of the automatic mode, against values worked out by hand and against what it is for.

    By hand (halfhalf, round to nearest even): an 11 + 11 bit value is represented exactly; 1 + 2^-12 + 2^-23 has
    v16 = 1 and a scaled residual 2^-1 + 2^-12 that ties down to 2^-1, so exactly 2^-23 is lost; 2^-40 is below
    everything the pair can hold (all of it is lost); 70000 saturates at 65504, and the scaled residual (32 x 2^11 after the cut) at 65504 too.
    For what it is for: on the paper's input types the choice agrees with which of the two models reaches the accuracy
    of FP32 (section "Effect of the exponent range of input matrices")."""
    assert split.fp16_pair_lost_fraction(np.float32([1.0 + 2.0 ** -10 + 2.0 ** -21, -3.5, 0.0])) == 0.0
    x = np.float32([1.0 + 2.0 ** -12 + 2.0 ** -23])
    assert split.fp16_pair_lost_fraction(x) == pytest.approx(2.0 ** -23 / float(x[0]), rel=1e-12)
    assert split.fp16_pair_lost_fraction(np.float32([2.0 ** -40])) == 1.0
    assert split.fp16_pair_lost_fraction(np.float32([70000.0])) == pytest.approx((70000.0 - 65504.0 - 65504.0 / 2048.0) / 70000.0, rel=1e-12)
    assert split.fp16_pair_lost_fraction(np.zeros(5, np.float32)) == 0.0
    assert np.isnan(split.fp16_pair_lost_fraction(np.float32([1.0, np.nan])))
    # two elements: sqrt((e1^2 + e2^2) / (x1^2 + x2^2)), not a mean of ratios
    pair = np.float32([1.0 + 2.0 ** -12 + 2.0 ** -23, 4.0])
    assert split.fp16_pair_lost_fraction(pair) == pytest.approx(2.0 ** -23 / np.sqrt(float(pair[0]) ** 2 + 16.0), rel=1e-12)
    one = np.float32([[1.0]])
    assert split.fp16_pair_represents(one, one)
    assert not split.fp16_pair_represents(one, np.float32([[1.0, np.nan]]))
    assert not split.fp16_pair_represents(np.float32([[2.0 ** -40]]), one)      # either operand decides
    assert not split.fp16_pair_represents(one, np.float32([[70000.0]]))
    assert split.fp16_pair_represents(x, x, tolerance=2.0 ** -23) and not split.fp16_pair_represents(x, x)

    n = 192
    for a_rng, b_rng in (((-15, 14), (-15, 14)), ((-35, -15), (-35, -15)), ((-100, -35), (-15, 14)), (None, None)):
        A = si.urand(n, n, 0, si.ID_A) if a_rng is None else si.exp_rand(n, n, *a_rng, 0, si.ID_A)
        B = si.urand(n, n, 0, si.ID_B) if b_rng is None else si.exp_rand(n, n, *b_rng, 0, si.ID_B)
        c64 = gemm.sgemm_fp64_ref("N", "N", n, n, n, 1.0, A, B)
        r32 = gemm.relative_residual(c64, gemm.sgemm_fp32_naive("N", "N", n, n, n, 1.0, A, B))
        r16 = gemm.relative_residual(c64, model.gemm_fp16_mode(A, B))
        assert split.fp16_pair_represents(A, B) == (r16 <= r32), (a_rng, b_rng, r16, r32)


def test_row_scaling_and_the_three_way_automatic_choice():
    """Scaling exponents against hand-worked rows; the scaled FP16 candidate against what it is for: on the paper's
    input types that the unscaled pair cannot hold (Types 2 to 4), the pair applied to row / column scaled operands,
    with the factors divided out again, is as accurate as the FP32 product (modelled with exact accumulation)."""
    rows = np.float32([[3.0, -0.5, 0.0], [0.0, 0.0, 0.0], [np.inf, 0.25, -0.125], [2.0 ** 100, 1.0, -2.0 ** 99],
                       [1e-45, 0.0, 2e-45], [np.nan, 2.0 ** -126, 0.0]])
    # largest binades: 2^1, none, 2^-2 (the infinity does not count), 2^100, subnormal = 2^-127, 2^-126 (NaN does not count)
    assert list(split.row_scale_exponents(rows, 14)) == [13, 0, 16, -86, 126, 126]
    assert list(split.row_scale_exponents(rows, 0)) == [-1, 0, 2, -100, 126, 126]
    assert list(split.row_scale_exponents(np.float32([[2.0 ** -120]]), -126)) == [-6]
    assert list(split.row_scale_exponents(np.float32([[2.0 ** 120]]), -126)) == [-126]          # clipped from -246
    scaled = split.scale_rows(rows[[0, 3]], [13, -86])
    assert np.array_equal(scaled, np.float32([[3.0 * 8192, -4096.0, 0.0], [16384.0, 2.0 ** -86, -8192.0]]))

    # how many elements carry a row: equal elements give the row length, a single one gives 1
    assert split.participation(np.ones((3, 7), np.float32)) == pytest.approx(7.0)
    assert split.participation(np.float32([[0, -5, 0, 0]])) == pytest.approx(1.0)
    assert split.participation(np.float32([[1, 1, 1, 1], [2, 0, 0, 0]])) == pytest.approx(36.0 / 16.0)
    assert split.participation(np.zeros((2, 3), np.float32)) == float("inf")
    assert split.participation(si.urand(64, 4096, 0, si.ID_A)) == pytest.approx(0.75 * 4096, rel=0.02)   # (E|x|)^2 / E x^2 = 3/4

    def run(n, k, a_rng, b_rng):
        A = si.exp_rand(n, k, *a_rng, 0, si.ID_A)
        B = si.exp_rand(k, n, *b_rng, 0, si.ID_B)
        choice = split.automatic_choice(A, B)
        ea, eb = split.row_scale_exponents(A), split.row_scale_exponents(B.T)
        with np.errstate(over="ignore"):
            c64 = gemm.sgemm_fp64_ref("N", "N", n, n, k, 1.0, A, B)
            r32 = gemm.relative_residual(c64, gemm.sgemm_fp32_naive("N", "N", n, n, k, 1.0, A, B))
        product = model.gemm_fp16_mode(split.scale_rows(A, ea), split.scale_rows(B.T, eb).T.copy())
        unscaled = np.ldexp(np.ldexp(product, -ea[:, None].astype(np.int32)), -eb[None, :].astype(np.int32))
        return choice, gemm.relative_residual(c64, unscaled) / r32

    # Long enough rows: the scaled arrangement is chosen and is at least as accurate as the FP32 product.
    for k, a_rng, b_rng, want in ((192, (-15, 14), (-15, 14), "fp16"), (192, (-15, 14), (-100, -35), "fp16 scaled"),
                                  (192, (-35, -15), (-35, -15), "fp16 scaled"), (1024, (-100, -35), (-100, -35), "fp16 scaled"),
                                  (192, (-100, 100), (-15, 14), "fp16 scaled"), (4096, (-100, 100), (-100, 0), "fp16 scaled")):
        choice, ratio = run(160, k, a_rng, b_rng)
        assert choice == want and ratio <= 1.0, (k, a_rng, b_rng, choice, ratio)
    # Dot products carried by a handful of terms (wide exponent ranges over short rows): the FP32 product barely rounds,
    # the pair's missing bit shows (ratio above 1), and the choice is the exact three-term split.
    for k, a_rng, b_rng in ((300, (-100, 100), (-100, 0)), (300, (-60, 60), (-60, 60))):
        choice, ratio = run(160, k, a_rng, b_rng)
        assert choice == "bf16" and ratio > 1.0, (k, a_rng, b_rng, choice, ratio)
    # (the threshold errs on the safe side: Type 4 over rows of 192 is sent the same way with the margin not yet gone)
    choice, ratio = run(160, 192, (-100, -35), (-100, -35))
    assert choice == "bf16" and 0.5 < ratio < 1.0
    n = 192
    poisoned = si.urand(n, n, 1, si.ID_A).copy()
    poisoned[5, 7] = np.nan
    assert split.automatic_choice(poisoned, si.urand(n, n, 1, si.ID_B)) == "bf16"
    huge = si.urand(n, n, 1, si.ID_A).copy()
    huge[5, 7] = 1e30                     # beyond the FP16 range as it is, an ordinary row maximum once scaled
    assert split.automatic_choice(huge, si.urand(n, n, 1, si.ID_B)) == "fp16 scaled"
