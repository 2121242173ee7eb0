"""Pins of the oracle's mapping/threshold learner (weighted Lloyd-Max, paper Sec. 5 and App. G) and
of threshold averaging, against things other than the oracle itself: numpy's weighted average, scipy's
k-means (the unweighted Lloyd iteration), a brute-force fixed-point check, invariants, a hand-worked
group, and the paper's printed initial tables."""
import numpy as np
import pytest
from scipy.cluster.vq import kmeans2

from oracle import lowra_oracle as orc
from paper_2502_08141_amd import synth
from tests import tables_util


def listing(init_tables):
    """The paper's printed initial tables (App. F listing), printed 1-/2-bit thresholds included."""
    return tables_util.listing_tables(init_tables)


def normalised(W):
    """u = w * (1/absmax) per 64-group in fp32, and the per-element weights (the group's absmax)."""
    N, K = W.shape
    g = W.reshape(N, K // 64, 64)
    a = np.abs(g).max(axis=2).astype(np.float32)
    inv = np.where(a == 0, np.float32(0), np.float32(1) / np.where(a == 0, np.float32(1), a)).astype(np.float32)
    u = (g * inv[:, :, None]).astype(np.float32).reshape(N, K)
    return u, np.repeat(a, 64, axis=1)


def rows(N, K, seed, scale_spread=True):
    rng = np.random.default_rng(seed)
    W = rng.normal(0, 0.02, (N, K))
    if scale_spread:                       # blocks of very different magnitude, so the weighting matters
        W *= rng.choice([0.1, 1.0, 8.0], size=(N, K // 64)).repeat(64, axis=1)
    return W.astype(np.float32)


@pytest.mark.parametrize("b", [1, 2, 4])
def test_weighted_mse_never_increases(b, init_tables):
    thr0, mp0, cbb = listing(init_tables)
    W = rows(6, 512, seed=b)
    bits = np.full(6, b, np.uint8); cb = np.searchsorted(cbb, bits).astype(np.int32)
    _, _, mse, done = orc.learn_tables(W, bits, cb, thr0, mp0, iters=6)
    assert (np.diff(mse, axis=1) <= 1e-15).all()
    assert (mse[:, 1] < mse[:, 0]).all()          # the first centroid update strictly helps on random data
    assert (done >= 1).all()


def test_one_bit_is_the_weighted_mean_of_each_sign(init_tables):
    """1 bit, threshold 0: one iteration gives the absmax-weighted means of the non-positive and the
    positive normalised weights (numpy.average), and their midpoint as the threshold."""
    thr0, mp0, cbb = listing(init_tables)
    W = rows(5, 384, seed=7)
    bits = np.ones(5, np.uint8); cb = np.zeros(5, np.int32)
    thr, mp, mse, _ = orc.learn_tables(W, bits, cb, thr0, mp0, iters=1)
    u, a = normalised(W)
    for n in range(5):
        neg, pos = u[n] <= 0, u[n] > 0
        lo = np.average(u[n][neg].astype(np.float64), weights=a[n][neg].astype(np.float64))
        hi = np.average(u[n][pos].astype(np.float64), weights=a[n][pos].astype(np.float64))
        assert mp[n, 0] == np.float32(lo) and mp[n, 1] == np.float32(hi)
        assert thr[n, 0] == np.float32((np.float64(mp[n, 0]) + np.float64(mp[n, 1])) / 2)
        err = np.where(neg, u[n] - np.float64(mp[n, 0]), u[n] - np.float64(mp[n, 1])) ** 2
        assert mse[n, 1] == pytest.approx(np.average(err, weights=a[n].astype(np.float64)), rel=1e-12)
    assert np.isinf(thr[:, 1:]).all() and (mp[:, 2:] == 0).all()


@pytest.mark.parametrize("b,iters", [(2, 1), (2, 3), (4, 2)])
def test_equal_block_weights_reduce_to_plain_lloyd(b, iters, init_tables):
    """When every block has the same absmax the weighting drops out: scipy's kmeans2 (Lloyd's
    iteration from given centroids) gives the same levels."""
    thr0, mp0, cbb = listing(init_tables)
    rng = np.random.default_rng(11 * b + iters)
    K = 1024
    W = rng.uniform(-0.9, 0.9, (3, K))
    W[:, ::64] = 1.0                                   # absmax exactly 1 in every block: u == w
    W = W.astype(np.float32)
    bits = np.full(3, b, np.uint8); cb = np.searchsorted(cbb, bits).astype(np.int32)
    thr, mp, _, done = orc.learn_tables(W, bits, cb, thr0, mp0, iters=iters)
    assert (done == iters).all()
    init = mp0[cb[0], : 1 << b].astype(np.float64).reshape(-1, 1)
    for n in range(3):
        cent, _ = kmeans2(W[n].astype(np.float64).reshape(-1, 1), init.copy(), iter=iters, minit="matrix")
        assert np.allclose(mp[n, : 1 << b], cent.ravel(), rtol=0, atol=2e-7)


def test_fixed_point_condition_after_many_iterations(init_tables):
    """At convergence every level is the weighted centroid of the points nearer to it than to any
    other level (brute force over points and levels in fp64)."""
    thr0, mp0, cbb = listing(init_tables)
    W = rows(3, 256, seed=21)
    bits = np.full(3, 2, np.uint8); cb = np.ones(3, np.int32)
    thr, mp, mse, done = orc.learn_tables(W, bits, cb, thr0, mp0, iters=200)
    u, a = normalised(W)
    for n in range(3):
        lv = mp[n, :4].astype(np.float64)
        nearest = np.array([int(np.argmin([abs(x - l) for l in lv])) for x in u[n].astype(np.float64)])
        for j in range(4):
            sel = nearest == j
            cen = float(np.sum(a[n][sel].astype(np.float64) * u[n][sel]) / np.sum(a[n][sel].astype(np.float64)))
            assert lv[j] == pytest.approx(cen, abs=5e-6)
        assert done[n] < 200                       # the stopping rule fired: the MSE stopped going down


def test_scale_invariance_and_zero_rows(init_tables):
    thr0, mp0, cbb = listing(init_tables)
    W = rows(4, 320, seed=5)
    bits = np.array([1, 2, 4, 2], np.uint8); cb = np.searchsorted(cbb, bits).astype(np.int32)
    t1, m1, e1, _ = orc.learn_tables(W, bits, cb, thr0, mp0, iters=2)
    t2, m2, e2, _ = orc.learn_tables(W * np.float32(4.0), bits, cb, thr0, mp0, iters=2)     # exact scaling by a power of two
    assert np.array_equal(t1, t2) and np.array_equal(m1, m2) and np.allclose(e1, e2, rtol=1e-12)
    Z = W.copy(); Z[3] = 0
    t3, m3, e3, d3 = orc.learn_tables(Z, bits, cb, thr0, mp0, iters=2)
    assert np.array_equal(t3[3], thr0[1]) and np.array_equal(m3[3], mp0[1]) and (e3[3] == 0).all() and d3[3] == 0
    assert np.array_equal(t3[:3], t1[:3])


def test_hand_worked_group():
    """One 64-element block, 2 bits, levels (-1, 0, 0.5, 1): 16 x -4, 16 x -1, 16 x 2, 16 x 4 (absmax 4).
    u = -1, -0.25, 0.5, 1; thresholds -0.5, 0.25, 0.75 put -0.25 with level 0: levels become
    -1, -0.25, 0.5, 1, thresholds -0.625, 0.125, 0.75; mse 0.0625 * 16/64 = 1/64 -> 0."""
    W = np.repeat(np.array([-4.0, -1.0, 2.0, 4.0], np.float32), 16).reshape(1, 64)
    thr0, mp0 = tables_util.pad_tables([[-1.0, 0.0, 0.5, 1.0]])
    thr, mp, mse, done = orc.learn_tables(W, np.array([2], np.uint8), np.array([0], np.int32), thr0, mp0, iters=2)
    assert mp[0, :4].tolist() == [-1.0, -0.25, 0.5, 1.0]
    assert thr[0, :3].tolist() == [-0.625, 0.125, 0.75]
    assert mse[0].tolist() == [1.0 / 64, 0.0, 0.0] and done[0] == 2


def test_empty_bin_keeps_its_level():
    W = np.repeat(np.array([-4.0, 4.0], np.float32), 32).reshape(1, 64)
    thr0, mp0 = tables_util.pad_tables([[-1.0, -0.3, 0.3, 1.0]])
    thr, mp, mse, _ = orc.learn_tables(W, np.array([2], np.uint8), np.array([0], np.int32), thr0, mp0, iters=1)
    assert mp[0, :4].tolist() == [-1.0, np.float32(-0.3), np.float32(0.3), 1.0]


def test_paper_init_thresholds_are_nearest_level_binning(init_tables):
    """With the printed 2-bit tables the E-step of the first iteration is App. G's nearest-level rule."""
    thr0, mp0, cbb = listing(init_tables)
    W = rows(2, 256, seed=9, scale_spread=False)
    u, _ = normalised(W)
    lv = mp0[1, :4].astype(np.float64)
    for x in u.ravel()[:200].astype(np.float64):
        code = int(np.sum(thr0[1, :3] < np.float32(x)))
        assert code == int(np.argmin(np.abs(lv - x)))


def test_average_thresholds():
    rng = np.random.default_rng(3)
    bits = np.array([1, 2, 4, 2, 1, 2], np.uint8)
    thr = np.full((6, 16), np.inf, np.float32)
    for n, b in enumerate(bits):
        thr[n, : (1 << b) - 1] = np.sort(rng.uniform(-1, 1, (1 << b) - 1)).astype(np.float32)
    out = orc.average_thresholds(bits, thr)
    for b in (1, 2, 4):
        sel = bits == b
        want = thr[sel][:, : (1 << b) - 1].astype(np.float64).mean(axis=0).astype(np.float32)
        assert np.allclose(out[sel][:, : (1 << b) - 1], want[None, :], rtol=0, atol=1e-7)
        assert np.isinf(out[sel][:, (1 << b) - 1:]).all()
    assert np.isinf(thr[0, 1])                      # the input array is not modified
