"""GPU parity of the mapping/threshold learner (lowra_learn_tables, lowra_average_thresholds) against
the CPU oracle on the same seeded inputs.  The learner sums in fp32/fp64 in another order than the
oracle's fp64 element-order sums, so levels and thresholds (values in [-1, 1]) are compared to 5e-7
absolute, the weighted MSE to 5e-5 relative; the tables then have to reproduce through the quantizer."""
import numpy as np
import pytest
import torch

from oracle import lowra_oracle as orc
from paper_2502_08141_amd import lowra, synth
from tests import tables_util

pytestmark = pytest.mark.gpu

TABLE_ATOL = 5e-7          # measured: at most 1.2e-7 (one unit in the last place of a level near 1)


def listing_tables(init_tables):
    """The paper's printed initial tables (App. F listing), printed 1-/2-bit thresholds included."""
    return tables_util.listing_tables(init_tables)


def make_rows(N, K, seed, fractions):
    rng = np.random.default_rng(seed)
    W = rng.normal(0, 0.02, (N, K)) * rng.choice([0.1, 1.0, 8.0], size=(N, K // 64)).repeat(64, axis=1)
    bits = synth.assign_bits(N, fractions, np.random.default_rng([seed, 1]))
    return W.astype(np.float32), bits


def same_tables(got, want, nvalid):
    """Compare [N,16] tables on their used entries; the padding must match exactly."""
    for n in range(got.shape[0]):
        k = nvalid[n]
        assert np.allclose(got[n, :k], want[n, :k], rtol=0, atol=TABLE_ATOL), (n, got[n, :k], want[n, :k])
        assert np.array_equal(got[n, k:], want[n, k:])


CASES = {
    "small_mixed": (40, 512, 31, (0.3, 0.4, 0.3), 2),
    "ragged_K": (24, 320, 32, (0.3, 0.4, 0.3), 2),
    "one_block": (9, 64, 33, (0.34, 0.33, 0.33), 2),
    "long_rows": (16, 13824, 34, (0.5, 0.25, 0.25), 2),
    "iters1": (32, 1024, 35, (0.3, 0.4, 0.3), 1),
    "iters5": (32, 1024, 36, (0.3, 0.4, 0.3), 5),
    "iters0": (8, 256, 37, (0.3, 0.4, 0.3), 0),
    # the kernel is instantiated for 1, 2, 4 and 8 eighths of a block per thread (K up to 2048, 4096, 8192, 16384)
    "two_passes": (24, 4096, 38, (0.4, 0.4, 0.2), 2),
    "four_passes": (12, 6144, 39, (0.3, 0.4, 0.3), 3),
}


@pytest.mark.parametrize("name", list(CASES))
@pytest.mark.parametrize("family", ["listing", "quantile"])
def test_learn_tables_matches_oracle(name, family, init_tables):
    N, K, seed, fr, iters = CASES[name]
    print(f"[learner case {name} {family}]", flush=True)
    W, bits = make_rows(N, K, seed, fr)
    if name == "small_mixed":
        W[3] = 0                                   # a channel of zeros keeps its initial tables
    thr0, mp0, cbb = listing_tables(init_tables) if family == "listing" else synth.shared_codebooks()
    cb = np.searchsorted(cbb, bits).astype(np.int32)
    lay = lowra.Layout(K, bits, cb, cbb)
    thr, mp, mse = lowra.lowra_learn_tables(lay, torch.from_numpy(W).cuda(), torch.from_numpy(thr0).cuda(),
                                            torch.from_numpy(mp0).cuda(), iters)
    torch.cuda.synchronize()
    rthr, rmp, rmse, rdone = orc.learn_tables(W, bits, cb, thr0, mp0, iters)
    nl = (1 << bits.astype(np.int64))
    same_tables(mp.cpu().numpy(), rmp, nl)
    same_tables(thr.cpu().numpy(), rthr, nl - 1)
    got_mse = mse.cpu().numpy().astype(np.float64)
    assert np.allclose(got_mse, rmse, rtol=5e-5, atol=1e-9), np.abs(got_mse - rmse).max()
    assert (np.diff(got_mse, axis=1) <= 1e-7).all()           # never increases on the GPU either


def test_learned_tables_quantize_like_the_oracles(init_tables):
    """End to end: learn on the GPU, average the thresholds, quantize with one table per channel; the
    oracle, given the GPU's tables, produces the same codes (bit-exact), and the weighted error of
    the learned tables is below that of the initial ones."""
    N, K = 48, 1024
    W, bits = make_rows(N, K, 41, (0.3, 0.4, 0.3))
    thr0, mp0, cbb = listing_tables(init_tables)
    cb = np.searchsorted(cbb, bits).astype(np.int32)
    lay = lowra.Layout(K, bits, cb, cbb)
    Wd = torch.from_numpy(W).cuda()
    thr, mp, mse = lowra.lowra_learn_tables(lay, Wd, torch.from_numpy(thr0).cuda(), torch.from_numpy(mp0).cuda(), 2)
    before = thr.cpu().numpy()
    lowra.lowra_average_thresholds(lay, thr)
    torch.cuda.synchronize()
    want = orc.average_thresholds(bits, before)
    assert np.allclose(thr.cpu().numpy()[np.isfinite(want)], want[np.isfinite(want)], rtol=0, atol=1e-7)
    assert np.array_equal(np.isinf(thr.cpu().numpy()), np.isinf(want))
    per_channel = lowra.Layout(K, bits, np.arange(N, dtype=np.int32), bits)     # one table per channel
    packed, absmax = lowra.lowra_quantize(per_channel, Wd, thr)
    torch.cuda.synchronize()
    rp, ra = orc.quantize(W, bits, np.arange(N, dtype=np.int32), thr.cpu().numpy())
    assert np.array_equal(packed.cpu().numpy(), rp) and np.array_equal(absmax.cpu().numpy(), ra)
    m = mse.cpu().numpy()
    assert (m[:, 2] <= m[:, 0]).all() and (m[:, 2] < m[:, 0]).mean() > 0.9


def test_learner_rejects_what_it_cannot_do(init_tables):
    thr0, mp0, cbb = listing_tables(init_tables)
    bits = np.ones(8, np.uint8)
    lay = lowra.Layout(16384 + 64, bits, np.zeros(8, np.int32), cbb)
    W = torch.zeros((8, 16384 + 64), device="cuda")
    with pytest.raises(lowra.LowraError) as e:
        lowra.lowra_learn_tables(lay, W, torch.from_numpy(thr0).cuda(), torch.from_numpy(mp0).cuda(), 2)
    assert e.value.status == lowra.UNSUPPORTED
