"""GPU parity of the per-channel error table (lowra_channel_mse) against the CPU oracle.  The kernel
adds the squared fp32 differences in fp32 per thread and fp64 across threads, the oracle in fp64:
1e-5 relative."""
import numpy as np
import pytest
import torch

from oracle import lowra_oracle as orc
from paper_2502_08141_amd import lowra, synth
from tests import tables_util

pytestmark = pytest.mark.gpu


def rows(N, K, seed):
    rng = np.random.default_rng(seed)
    return (rng.normal(0, 0.02, (N, K)) * rng.choice([0.2, 1.0, 5.0], size=(N, K // 64)).repeat(64, axis=1)).astype(np.float32)


@pytest.mark.parametrize("N,K,seed", [(37, 512, 1), (5, 64, 2), (16, 4096, 3), (9, 13824, 4), (300, 320, 5)])
@pytest.mark.parametrize("family", ["quantile", "listing"])
def test_channel_mse_matches_oracle(N, K, seed, family, init_tables):
    print(f"[channel_mse {N}x{K} {family}]", flush=True)
    if family == "quantile":
        thr, mp, _ = synth.shared_codebooks()
    else:
        thr, mp, _ = tables_util.listing_tables(init_tables)
    W = rows(N, K, seed)
    if N > 4:
        W[2] = 0                                            # an all-zero channel has no error
    got = lowra.lowra_channel_mse(torch.from_numpy(W).cuda(), torch.from_numpy(thr).cuda(), torch.from_numpy(mp).cuda())
    torch.cuda.synchronize()
    want = orc.channel_mse(W, thr, mp)
    assert np.allclose(got.cpu().numpy().astype(np.float64), want, rtol=1e-5, atol=0)
    if N > 4:
        assert (got.cpu().numpy()[2] == 0).all()


def test_error_table_feeds_the_assignment_and_the_quantizer():
    """The table from the GPU, the greedy assignment from the library, a layout built from it: the
    mean width meets the budget and the quantizer's output for that layout matches the oracle's."""
    thr, mp, cbb = synth.shared_codebooks()
    N, K = 256, 1024
    W = rows(N, K, 9)
    mse = lowra.lowra_channel_mse(torch.from_numpy(W).cuda(), torch.from_numpy(thr).cuda(), torch.from_numpy(mp).cuda()).cpu().numpy()
    params = np.full(N, K, np.int64)
    bits = lowra.lowra_assign_precisions(params, mse, 1.5)
    assert np.array_equal(bits, orc.assign_greedy(params, mse, 1.5))
    assert bits.mean() <= 1.5 and bits.mean() > 1.45
    cb = np.searchsorted(cbb, bits).astype(np.int32)
    lay = lowra.Layout(K, bits, cb, cbb)
    packed, absmax = lowra.lowra_quantize(lay, torch.from_numpy(W).cuda(), torch.from_numpy(thr).cuda())
    torch.cuda.synchronize()
    rp, ra = orc.quantize(W, bits, cb, thr)
    assert np.array_equal(packed.cpu().numpy(), rp) and np.array_equal(absmax.cpu().numpy(), ra)


def test_equal_neighbouring_thresholds_and_padding_bin_like_the_oracle():
    """The 4-bit binning bisects the sorted thresholds: tables with equal neighbours (levels nobody can reach) and
    with +inf from some entry on (a coarser table in a 4-bit slot) give the counts of the definition -- the
    quantizer's codes bit for bit, the error table to its usual bar."""
    thr, mp, cbb = synth.shared_codebooks()
    thr, mp = thr.copy(), mp.copy()
    t4 = thr[2].copy()
    t4[3] = t4[4]; t4[8] = t4[9] = t4[10]                   # equal neighbours
    t4[12:] = np.inf                                        # a table that ends early
    thr[2] = t4
    N, K = 96, 1024
    W = rows(N, K, 11)
    W[5, :64] = np.float32(0.37) * np.sign(W[5, :64])       # many weights with the same normalised value
    bits = np.full(N, 4, np.uint8); bits[::3] = 2; bits[1::7] = 1
    cb = np.searchsorted(cbb, bits).astype(np.int32)
    lay = lowra.Layout(K, bits, cb, cbb)
    Wd, thr_d, mp_d = torch.from_numpy(W).cuda(), torch.from_numpy(thr).cuda(), torch.from_numpy(mp).cuda()
    packed, absmax = lowra.lowra_quantize(lay, Wd, thr_d)
    got = lowra.lowra_channel_mse(Wd, thr_d, mp_d)
    torch.cuda.synchronize()
    rp, ra = orc.quantize(W, bits, cb, thr)
    assert np.array_equal(packed.cpu().numpy(), rp) and np.array_equal(absmax.cpu().numpy(), ra)
    assert np.allclose(got.cpu().numpy().astype(np.float64), orc.channel_mse(W, thr, mp), rtol=1e-5, atol=0)
