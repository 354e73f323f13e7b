"""The seeded input generators (shared by the oracle side and the GPU side; they hold none of the method's arithmetic)."""
import numpy as np
import pytest

import seeded_inputs as si


def test_draws_are_pure_functions_of_seed_matrix_and_position():
    a = si.urand(37, 11, 5, si.ID_A)
    assert np.array_equal(a, si.urand(37, 11, 5, si.ID_A))
    assert not np.array_equal(a, si.urand(37, 11, 6, si.ID_A)) and not np.array_equal(a, si.urand(37, 11, 5, si.ID_B))
    # a larger leading dimension changes the storage, not the values; the padding rows hold NaN so that a stray read shows
    padded = si.urand(37, 11, 5, si.ID_A, ld=40)
    assert padded.shape == (40, 11) and padded.flags.f_contiguous
    assert np.array_equal(padded[:37], a) and np.all(np.isnan(padded[37:]))
    with pytest.raises(ValueError):
        si.urand(37, 11, 5, si.ID_A, ld=36)


def test_urand_and_exp_rand_have_the_papers_distributions():
    u = si.urand(1 << 16, 4, 1, si.ID_A)
    assert u.dtype == np.float32 and np.all(np.abs(u) < 1.0)
    assert abs(float(u.mean())) < 0.01 and abs(float((u.astype(np.float64) ** 2).mean()) - 1.0 / 3.0) < 0.01
    # exp_rand(a, b): sign * 1.mantissa * 2^e, e uniform over a .. b, all 23 mantissa bits random
    x = si.exp_rand(1 << 18, 1, -7, 12, 2, si.ID_B)[:, 0]
    mant, expo = np.frexp(x.astype(np.float64))          # |mant| in [0.5, 1): value = mant 2^expo
    e = expo - 1
    assert e.min() == -7 and e.max() == 12
    counts = np.bincount(e + 7, minlength=20)
    assert counts.min() > 0.9 * len(x) / 20 and counts.max() < 1.1 * len(x) / 20
    assert abs(float(np.mean(x > 0)) - 0.5) < 0.01
    bits = x.view(np.uint32) & np.uint32(0x7FFFFF)
    assert abs(float(np.mean(bits & 1)) - 0.5) < 0.01 and abs(float(np.mean(bits >> 22)) - 0.5) < 0.01
    with pytest.raises(ValueError):
        si.exp_rand(4, 4, -127, 0, 0, 0)
    r = si.randint(1000, 3, -15, 15, 0, si.ID_A)
    assert r.min() == -15 and r.max() == 15 and np.array_equal(r, np.round(r))


def test_row_samples():
    rows = si.sample_indices(1000, 64, seed=3)
    assert len(rows) == 64 and np.all(np.diff(rows) > 0) and rows.min() >= 0 and rows.max() < 1000
    assert np.array_equal(rows, si.sample_indices(1000, 64, seed=3)) and not np.array_equal(rows, si.sample_indices(1000, 64, seed=4))
    assert np.array_equal(si.sample_indices(10, 64, seed=0), np.arange(10))
    # one row out of every block of `stride` consecutive rows, the ragged last block included
    for n, stride in ((16384, 64), (2235, 64), (4095, 16), (5, 64), (64, 64), (65, 64)):
        strat = si.stratified_indices(n, stride, seed=7)
        blocks = -(-n // stride)
        assert len(strat) == blocks and np.array_equal(strat // stride, np.arange(blocks)) and strat.max() < n
        assert np.array_equal(strat, si.stratified_indices(n, stride, seed=7))
    assert not np.array_equal(si.stratified_indices(16384, 64, 7), si.stratified_indices(16384, 64, 8))
    assert len(np.unique(si.stratified_indices(16384, 64, 7) % 64)) > 32          # not the same offset in every block
