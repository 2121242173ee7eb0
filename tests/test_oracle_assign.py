"""Pins of the oracle's per-channel error table (paper Sec. 6.1) and of the greedy budgeted precision
assignment that stands in for the paper's ILP (Sec. 6): composition of the separately pinned
quantizer and decoder with numpy's mean, the 1-bit closed form, the quantizer's error bound,
exhaustive search on tiny instances, budget invariants."""
import itertools

import numpy as np
import pytest

from oracle import lowra_oracle as orc
from paper_2502_08141_amd import synth


def rows(N, K, seed):
    rng = np.random.default_rng(seed)
    return (rng.normal(0, 0.02, (N, K)) * rng.choice([0.2, 1.0, 5.0], size=(N, K // 64)).repeat(64, axis=1)).astype(np.float32)


def test_error_table_is_quantize_then_decode_then_numpy_mean():
    thr, mp, cbb = synth.shared_codebooks()
    W = rows(10, 320, 1)
    got = orc.channel_mse(W, thr, mp)
    for p, b in enumerate((1, 2, 4)):
        bits = np.full(10, b, np.uint8); cb = np.full(10, p, np.int32)
        packed, absmax = orc.quantize(W, bits, cb, thr)
        w32 = orc.dequantize(packed, absmax, bits, cb, mp, 320, "fp32")
        want = ((W - w32).astype(np.float32).astype(np.float64) ** 2).mean(axis=1)
        assert np.allclose(got[:, p], want, rtol=1e-12, atol=0)


def test_one_bit_closed_form_and_error_bound():
    """Levels -1/+1, threshold 0: the decoded weight is sign(w) * absmax, so the error is absmax - |w|."""
    thr, mp, cbb = synth.shared_codebooks()
    W = rows(6, 256, 2)
    got = orc.channel_mse(W, thr, mp)
    a = np.abs(W.reshape(6, 4, 64)).max(axis=2).repeat(64, axis=1)
    assert np.allclose(got[:, 0], ((a.astype(np.float64) - np.abs(W)) ** 2).mean(axis=1), rtol=1e-6)
    # midpoint thresholds on tables spanning [-1, 1]: |w32 - w| <= a * (largest level gap) / 2
    for p, b in enumerate((1, 2, 4)):
        gap = np.diff(mp[p, : 1 << b].astype(np.float64)).max()
        assert (got[:, p] <= ((a.astype(np.float64) * gap / 2) ** 2).mean(axis=1) * (1 + 1e-6)).all()
    assert (got[:, 2] < got[:, 1]).all() and (got[:, 1] < got[:, 0]).all()     # these tables: more bits, less error


def total_error(params, mse, bits):
    idx = np.searchsorted([1, 2, 4], bits)
    return float(np.sum(params.astype(np.float64) * mse[np.arange(len(bits)), idx].astype(np.float64)))


def test_greedy_matches_exhaustive_search_when_it_lands_on_the_budget():
    """Convex per-channel gains, equal channel sizes, a budget the greedy sequence meets exactly:
    the fractional-knapsack optimum is integral, so exhaustive search over 3^N assignments agrees."""
    rng = np.random.default_rng(4)
    N = 6
    params = np.full(N, 64, np.int64)
    for trial in range(6):
        g1 = rng.uniform(1.0, 2.0, N); g2 = g1 * rng.uniform(0.1, 0.45, N)      # gain per bit of 2->4 below that of 1->2
        m4 = rng.uniform(0.1, 0.2, N); m2 = m4 + 2 * g2; m1 = m2 + g1
        mse = np.stack([m1, m2, m4], axis=1).astype(np.float32)
        full = orc.assign_greedy(params, mse, 4.0)
        assert (full == 4).all()
        for budget_bits in range(N, 4 * N + 1):
            bits = orc.assign_greedy(params, mse, budget_bits / N)
            used = int(bits.sum())
            assert used <= budget_bits
            if used != budget_bits:
                continue                                                         # leftover budget: greedy need not be optimal
            best = min(total_error(params, mse, np.array(c, np.uint8))
                       for c in itertools.product((1, 2, 4), repeat=N) if sum(c) <= budget_bits)
            assert total_error(params, mse, bits) == pytest.approx(best, rel=1e-12)


def test_greedy_budget_invariants():
    rng = np.random.default_rng(6)
    N = 200
    params = rng.choice([4096, 11008], N).astype(np.int64)
    m4 = rng.uniform(1e-6, 2e-6, N); m2 = m4 * rng.uniform(3, 6, N); m1 = m2 * rng.uniform(2, 4, N)
    mse = np.stack([m1, m2, m4], axis=1).astype(np.float32)
    prev = None
    for bpp in (1.0, 1.15, 1.5, 2.0, 2.5, 4.0):
        bits = orc.assign_greedy(params, mse, bpp)
        assert set(np.unique(bits)) <= {1, 2, 4}
        used = float((params * bits).sum()); cap = bpp * float(params.sum())
        assert used <= cap * (1 + 1e-12)
        # maximal: no further upgrade with a positive gain fits
        for n in range(N):
            if bits[n] < 4:
                cost = params[n] * (1 if bits[n] == 1 else 2)
                assert used + cost > cap or mse[n, 0 if bits[n] == 1 else 1] <= mse[n, 1 if bits[n] == 1 else 2]
        err = total_error(params, mse, bits)
        assert prev is None or err <= prev
        prev = err
    assert (orc.assign_greedy(params, mse, 1.0) == 1).all() and (orc.assign_greedy(params, mse, 4.0) == 4).all()
    with pytest.raises(ValueError):
        orc.assign_greedy(params, mse, 0.9)


def test_greedy_skips_upgrades_that_do_not_help_and_breaks_ties_by_index():
    params = np.array([64, 64, 64], np.int64)
    mse = np.array([[1.0, 0.5, 0.5], [1.0, 0.5, 0.2], [1.0, 1.0, 0.1]], np.float32)
    assert orc.assign_greedy(params, mse, 4.0).tolist() == [2, 4, 1]      # channel 2's first upgrade gains nothing: it stays
    assert orc.assign_greedy(params, mse, 4.0 / 3).tolist() == [2, 1, 1]  # one bit to spend: the tie goes to channel 0
