"""What one v_mfma_f32_32x32x16 does on the MI355X, through ecgemm_debug_mfma.

The method's accumulation discipline rests on these facts (section "Avoiding RZ during Tensor Core accumulation" is
about exactly this behaviour on another vendor's unit, where the answer differs).  They are measurements of the
hardware, not parity claims: the paper fixes none of them for AMD ("parity unpinned"); the CPU side of each check is
the paper's own mma_rn / mma_rz emulator or plain exact arithmetic.
"""
import numpy as np
import pytest

from oracle import mma_emulator as emu
from oracle import split

pytestmark = pytest.mark.gpu

ULP = 2.0 ** -23


def _to_bits(x, bf16):
    x = np.asarray(x, dtype=np.float32)
    return split.to_bf16_rn_bits(x) if bf16 else x.astype(np.float16).view(np.uint16)


def _run(A, B, C, bf16=False):
    """A: (p, 32, 16), B: (p, 16, 32), C: (p, 32, 32) -> D (p, 32, 32) via the documented lane layout."""
    import torch
    import paper_2203_03341_amd as ec
    A, B, C = (np.asarray(x, dtype=np.float32) for x in (A, B, C))
    p = A.shape[0]
    lane = np.arange(64)
    row, grp = lane % 32, lane // 32
    k_idx = 8 * grp[:, None] + np.arange(8)[None, :]                       # (64, 8)
    a = A[:, row[:, None], k_idx]                                           # (p, 64, 8): A(l % 32, 8 (l / 32) + e)
    b = B[:, k_idx, row[:, None]]                                           # B(8 (l / 32) + e, l % 32)
    v = np.arange(16)
    i_idx = 8 * (v[None, :] // 4) + 4 * grp[:, None] + v[None, :] % 4       # (64, 16)
    c = C[:, i_idx, row[:, None]]                                           # (p, 64, 16)
    ta = torch.from_numpy(_to_bits(a, bf16).view(np.int16).reshape(-1)).cuda()
    tb = torch.from_numpy(_to_bits(b, bf16).view(np.int16).reshape(-1)).cuda()
    tc = torch.from_numpy(np.ascontiguousarray(c).reshape(-1)).cuda()
    td = torch.empty_like(tc)
    h = ec.Handle()
    h.debug_mfma(bf16, p, ta, tb, tc, td)
    torch.cuda.synchronize()
    h.destroy()
    d = td.cpu().numpy().reshape(p, 64, 16)
    D = np.zeros((p, 32, 32), dtype=np.float32)
    D[:, i_idx, row[:, None]] = d
    return D


def _single(products, c0, bf16=False):
    """One output element: C(0, 0) = c0, products = {k: (a, b)} placed in row 0 of A and column 0 of B."""
    A = np.zeros((1, 32, 16), np.float32)
    B = np.zeros((1, 16, 32), np.float32)
    C = np.zeros((1, 32, 32), np.float32)
    C[0, 0, 0] = c0
    for k, (a, b) in products.items():
        A[0, 0, k], B[0, k, 0] = a, b
    return float(_run(A, B, C, bf16)[0, 0, 0])


@pytest.mark.parametrize("bf16", [False, True])
def test_lane_map_and_exact_small_integers(bf16):
    rng = np.random.default_rng(1)
    A = rng.integers(-7, 8, (5, 32, 16)).astype(np.float32)
    B = rng.integers(-7, 8, (5, 16, 32)).astype(np.float32)
    C = rng.integers(-50, 50, (5, 32, 32)).astype(np.float32)
    want = np.einsum("pik,pkj->pij", A.astype(np.int64), B.astype(np.int64)) + C.astype(np.int64)
    assert np.array_equal(_run(A, B, C, bf16).astype(np.int64), want)


def test_accumulate_rounds_to_nearest_even():
    p = lambda f: (f * 2.0 ** -10, 2.0 ** -13)          # a product of f ulps of 1.0
    assert _single({0: p(0.75)}, 1.0) == 1 + ULP         # round toward zero would return 1
    assert _single({0: p(0.5)}, 1.0) == 1.0              # tie to even (round half away would return 1 + ulp)
    assert _single({0: p(1.5)}, 1.0) == 1 + 2 * ULP      # tie to even upward
    assert _single({0: p(-0.125)}, 1.0) == 1.0           # round toward zero would return 1 - ulp / 2


def test_products_are_added_in_two_groups_of_eight():
    p = lambda f: (f * 2.0 ** -10, 2.0 ** -13)
    assert _single({0: p(0.3125), 1: p(0.3125)}, 1.0) == 1 + ULP      # same group: summed first, 0.625 ulp rounds up
    assert _single({0: p(0.3125), 8: p(0.3125)}, 1.0) == 1.0          # k = 0 and k = 8: two roundings, each down
    assert _single({k: p(0.09375) for k in range(8)}, 1.0) == 1 + ULP  # eight in one group: 0.75 ulp
    assert _single({k: p(0.0625) for k in range(16)}, 1.0) == 1.0      # 0.5 ulp per group: two ties to even


def test_addends_are_aligned_to_the_largest_and_cut_below_2_pow_minus_25():
    big = {0: (1024.0, 1024.0), 1: (-1024.0, 1024.0)}                  # +2^20 - 2^20
    assert _single({**big, 2: (2.0 ** -2, 2.0 ** -2)}, 0.0) == 2.0 ** -4    # 24 binary places below: kept
    assert _single({**big, 2: (2.0 ** -3, 2.0 ** -3)}, 0.0) == 0.0          # 26 places below: dropped
    assert _single({**big, 2: (0.75 * 2.0 ** -10, 2.0 ** -13)}, 1.0) == 1.0  # even the accumulator's guard bits go
    # the same small term among addends of its own size loses nothing: why corrections get their own accumulator
    assert _single({0: (0.75 * 2.0 ** -10, 2.0 ** -13)}, 2.0 ** -23) == 1.75 * 2.0 ** -23


def test_subnormal_inputs_and_outputs_are_kept():
    assert _single({0: (2.0 ** -20, 1024.0)}, 0.0) == 2.0 ** -10                  # FP16 subnormal operand
    assert _single({0: (2.0 ** -24, 2.0 ** -24)}, 0.0) == 2.0 ** -48
    assert _single({0: (2.0 ** -130, 2.0 ** 100)}, 0.0, bf16=True) == 2.0 ** -30  # BF16 subnormal operand
    assert _single({0: (2.0 ** -100, 2.0 ** -40)}, 0.0, bf16=True) == 2.0 ** -140  # FP32 subnormal result


def test_unit_resembles_the_rn_emulator_not_the_rz_one():
    """Chains of 64 instructions on uniform(-1, 1) FP16 data: the signed error against the exact sum has no drift
    toward zero (the paper's mma_rz model has one), and its size matches the mma_rn model."""
    rng = np.random.default_rng(2)
    p, steps = 8, 64
    A = rng.uniform(-1, 1, (steps, p, 32, 16)).astype(np.float16).astype(np.float32)
    B = rng.uniform(-1, 1, (steps, p, 16, 32)).astype(np.float16).astype(np.float32)
    hw = np.zeros((p, 32, 32), np.float32)
    for s in range(steps):
        hw = _run(A[s], B[s], hw)
    exact = np.einsum("spik,spkj->pij", A.astype(np.float64), B.astype(np.float64))
    rn = np.zeros((p, 32, 32), np.float32)
    rz = np.zeros((p, 32, 32), np.float32)
    for s in range(steps):
        for q in range(p):
            for half in (slice(0, 8), slice(8, 16)):
                rn[q] = emu.mma_rn(A[s, q][:, half], B[s, q][half, :], rn[q])
                rz[q] = emu.mma_rz(A[s, q][:, half], B[s, q][half, :], rz[q])
    toward_zero = lambda x: float(np.mean(np.sign(exact) * (x - exact)))     # negative = magnitude shrinks
    rms = lambda x: float(np.sqrt(np.mean((x - exact) ** 2)))
    assert toward_zero(rz) < -5 * abs(toward_zero(hw))
    assert rms(hw) < 0.5 * rms(rz) and 0.5 * rms(rn) < rms(hw) < 2.0 * rms(rn)
