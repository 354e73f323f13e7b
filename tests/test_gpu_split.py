"""Step 1 parity: the HIP split kernel against the numpy split, bit for bit, through the C-ABI."""
import numpy as np
import pytest

import seeded_inputs as si
from oracle import split
from gpu_util import pack_fp32_fragment_order, pack_fragment_order, to_device

pytestmark = pytest.mark.gpu


def _mode_id(mode):
    import paper_2203_03341_amd as ec
    if isinstance(mode, bool):
        return ec.MODE_BF16_FULL if mode else ec.MODE_FP16_SPLIT
    return {"unscaled": ec.MODE_FP16_UNSCALED, "markidis": ec.MODE_FP16_MARKIDIS, "plain16": ec.MODE_FP16_PLAIN,
            "plainbf": ec.MODE_BF16_PLAIN, "fp32": ec.MODE_FP32_MFMA}[mode]


def _expected(op, store, rows, depth, mode):
    X = store[:rows, :depth] if op == "N" else store[:depth, :rows].T
    X = np.ascontiguousarray(X, dtype=np.float32)
    if mode is True:
        parts = list(split.split_bf16x3(X))
    elif mode is False:
        parts = [p.view(np.uint16) for p in split.split_fp16(X)]
    elif mode in ("unscaled", "markidis"):
        parts = [p.view(np.uint16) for p in split.split_fp16(X, scaled=False)]
    elif mode == "fp32":
        return pack_fp32_fragment_order(X)
    elif mode == "plain16":
        parts = [split.to_fp16_rn(X).view(np.uint16)]
    else:
        parts = [split.to_bf16_rn_bits(X)]
    return pack_fragment_order(parts)


def _run(op, store, rows, depth, mode_bf16, offset_elems=0):
    import torch
    import paper_2203_03341_amd as ec
    mode = _mode_id(mode_bf16)
    h = ec.Handle()
    src = to_device(store)
    nbytes = ec.split_size(rows, depth, mode)
    packed = torch.full((nbytes // 2,), 0x7FFF, dtype=torch.int16, device="cuda")   # poison
    ld = store.shape[0]
    h.split(ec.OP_N if op == "N" else ec.OP_T, rows, depth, src, ld, mode, packed)
    torch.cuda.synchronize()
    got = packed.cpu().numpy().view(np.uint16)
    h.destroy()
    return got


CASES = [
    # (op, rows, depth, ld padding)
    ("N", 256, 256, 0), ("T", 256, 256, 0),
    ("N", 300, 77, 5), ("T", 300, 77, 3),
    ("N", 1, 1, 0), ("T", 1, 1, 0),
    ("N", 33, 1031, 1), ("T", 515, 40, 4), ("T", 70, 129, 1),
    # r-contiguous with a 16-byte aligned leading dimension (the 256-row kernel) and 1, 2, 3 rows past a multiple of 4
    ("N", 301, 77, 3), ("N", 1022, 70, 2), ("N", 515, 40, 1), ("N", 260, 33, 0),
]


@pytest.mark.parametrize("mode_bf16", [False, True])
@pytest.mark.parametrize("op,rows,depth,pad", CASES)
def test_split_matches_oracle_bitwise(op, rows, depth, pad, mode_bf16):
    sr, sc = (rows, depth) if op == "N" else (depth, rows)
    for kind in ("urand", "exp15", "exp100"):
        if kind == "urand":
            store = si.urand(sr, sc, seed=1, matrix_id=si.ID_A, ld=sr + pad)
        elif kind == "exp15":
            store = si.exp_rand(sr, sc, -15, 15, seed=2, matrix_id=si.ID_A, ld=sr + pad)
        else:
            store = si.exp_rand(sr, sc, -100, 100, seed=3, matrix_id=si.ID_A, ld=sr + pad)
        got = _run(op, store, rows, depth, mode_bf16)
        want = _expected(op, store, rows, depth, mode_bf16)
        assert got.shape == want.shape
        bad = np.flatnonzero(got != want)
        assert bad.size == 0, (kind, bad[:8], got[bad[:8]], want[bad[:8]])


@pytest.mark.parametrize("mode_bf16", [False, True])
def test_split_edge_values(mode_bf16):
    """Saturation, signed zeros, values that only the scaled residual can hold, FP32 subnormals, Inf, NaN."""
    vals = [0.0, -0.0, 65504.0, 65519.996, 65520.0, 65535.996, -65535.996, 2.0 ** -24, 2.0 ** -25, 2.0 ** -35,
            2.0 ** -36, 1.5 * 2.0 ** -36, 1e-45, -1e-40, 2.0 ** -126, 3.4028234e38, -3.4028234e38, 3.39e38,
            np.inf, -np.inf, 1.0, -1.0, 0.1, 2.0 ** -14, 2.0 ** -15, 1.9999999 * 2.0 ** -15, 6.1e-5, 100000.0, 1e30,
            2.0 ** 116, 2.0 ** 117, -2.0 ** 117, 1e36, -1e38]
    vals = np.array(vals, dtype=np.float32)
    rows, depth = 8, vals.size
    store = np.asfortranarray(np.tile(vals, (rows, 1)) * np.array([[1], [-1], [1], [-1], [1], [-1], [1], [-1]], np.float32))
    store = np.asfortranarray(store.astype(np.float32))
    for op in ("N", "T"):
        st = store if op == "N" else np.asfortranarray(store.T)
        got = _run(op, st, rows, depth, mode_bf16)
        want = _expected(op, st, rows, depth, mode_bf16)
        assert np.array_equal(got, want), np.flatnonzero(got != want)[:10]
    # NaN among ordinary values: where the oracle's parts are NaN the kernel's are (payload bits are not compared), and
    # every other position agrees bit for bit
    mixed = np.asfortranarray(np.tile(np.array([1.0, np.nan, -0.1, 65536.0, np.nan, 3.0e-5, -np.nan, 7.0], np.float32), (6, 1)))
    mixed[2, :] = np.nan
    for op in ("N", "T"):
        st = mixed if op == "N" else np.asfortranarray(mixed.T)
        got = _run(op, st, 6, 8, mode_bf16)
        want = _expected(op, st, 6, 8, mode_bf16)
        if mode_bf16:
            nan_of = lambda bits: ((bits & 0x7F80) == 0x7F80) & ((bits & 0x7F) != 0)
        else:
            nan_of = lambda bits: ((bits & 0x7C00) == 0x7C00) & ((bits & 0x3FF) != 0)
        want_nan = nan_of(want)
        assert want_nan.sum() == (3 if mode_bf16 else 2) * int(np.isnan(mixed).sum())
        assert np.array_equal(nan_of(got), want_nan)
        assert np.array_equal(got[~want_nan], want[~want_nan])


@pytest.mark.parametrize("mode", ["unscaled", "markidis", "plain16", "plainbf", "fp32"])
@pytest.mark.parametrize("op", ["N", "T"])
def test_split_of_comparison_methods(mode, op):
    """Markidis' unscaled residual (Eqs. corr-elm-1, corr-elm-2) and the plain conversions, bit for bit."""
    rows, depth = 300, 77
    sr, sc = (rows, depth) if op == "N" else (depth, rows)
    for store in (si.urand(sr, sc, 4, si.ID_A, ld=sr + 2), si.exp_rand(sr, sc, -20, 15, 5, si.ID_A, ld=sr + 1)):
        got = _run(op, store, rows, depth, mode)
        want = _expected(op, store, rows, depth, mode)
        assert got.shape == want.shape and np.array_equal(got, want)


@pytest.mark.parametrize("mode_bf16", [False, True])
def test_split_of_a_large_operand(mode_bf16):
    """2048 x 3000 in both orientations: every block position of a many-tile grid, bit for bit."""
    for op in ("N", "T"):
        rows, depth = 2048, 3000
        sr, sc = (rows, depth) if op == "N" else (depth, rows)
        store = si.exp_rand(sr, sc, -30, 20, 9, si.ID_B)
        got = _run(op, store, rows, depth, mode_bf16)
        assert np.array_equal(got, _expected(op, store, rows, depth, mode_bf16))
