"""GPU parity on one matrix larger than any of the configs: 66560 x 16384 (1.09 G weights).

Its fp32 form is 4.36 GB and its fp32 decode as large, the bf16 decode 2.18 GB: byte offsets pass
2^31 and 2^32 inside every buffer except the packed one.  K = 16384 is also the longest row the
learner takes.  The weights are drawn on the device (seeded); the oracle recomputes a sample of
channels, among them the first, the last and the ones on either side of the 2^31- and 2^32-byte
marks of W.  Each channel's codes, scales, decode, error table and learned tables depend on that
channel's row only, and column n of y on row n of the weights; the input gradient contracts over
all channels, so it is tied to the forward by the adjoint identity instead.
"""
import numpy as np
import pytest
import torch

from oracle import lowra_oracle as orc
from paper_2502_08141_amd import lowra, synth
from tests.gpu_util import REL_TOL, bf16_dev, bf16_host_bits, bf16_host_f64, rel_err

pytestmark = pytest.mark.gpu

N, K, R = 66560, 16384, 16


def test_large_matrix():
    print("[large] drawing W on the device", flush=True)
    gen = torch.Generator(device="cuda").manual_seed(20250211)
    W = torch.empty((N, K), dtype=torch.float32, device="cuda").normal_(0.0, 0.02, generator=gen)
    bits = synth.assign_bits(N, (0.4, 0.3, 0.3), np.random.default_rng([synth.SEED, 66560]))
    thr, mp, cbb = synth.shared_codebooks()
    cb = np.searchsorted(cbb, bits).astype(np.int32)
    lay = lowra.Layout(K, bits, cb, cbb)
    off = lowra.lowra_plan_rows(K, bits)
    thr_d, mp_d = torch.from_numpy(thr).cuda(), torch.from_numpy(mp).cuda()

    rng = np.random.default_rng([synth.SEED, 66561])
    marks = [0, 1, (1 << 31) // (4 * K) - 1, (1 << 31) // (4 * K), (1 << 32) // (4 * K) - 1, (1 << 32) // (4 * K), N - 2, N - 1]
    rows = np.unique(np.concatenate([np.array(marks), rng.choice(N, 40, replace=False)]))
    rows_d = torch.from_numpy(rows).cuda()
    Ws = W[rows_d].cpu().numpy()

    print("[large] quantize", flush=True)
    packed, absmax = lowra.lowra_quantize(lay, W, thr_d)
    torch.cuda.synchronize()
    rp, ra = orc.quantize(Ws, bits[rows], cb[rows], thr)
    assert np.array_equal(absmax[rows_d].cpu().numpy(), ra)
    packed_h = packed.cpu().numpy()
    got_rows = np.concatenate([packed_h[off[n]:off[n + 1]] for n in rows])
    assert np.array_equal(got_rows, rp)
    del packed_h

    print("[large] dequantize", flush=True)
    want16 = orc.dequantize(rp, ra, bits[rows], cb[rows], mp, K)
    want32 = orc.dequantize(rp, ra, bits[rows], cb[rows], mp, K, "fp32")
    out16 = lowra.lowra_dequantize(lay, packed, absmax, mp_d)
    torch.cuda.synchronize()
    assert np.array_equal(bf16_host_bits(out16[rows_d]), want16)
    del out16
    out32 = lowra.lowra_dequantize(lay, packed, absmax, mp_d, out_dtype=torch.float32)
    torch.cuda.synchronize()
    assert np.array_equal(out32[rows_d].cpu().numpy(), want32)
    del out32

    print("[large] error table and learner", flush=True)
    mse = lowra.lowra_channel_mse(W, thr_d, mp_d)
    torch.cuda.synchronize()
    assert np.allclose(mse[rows_d].cpu().numpy().astype(np.float64), orc.channel_mse(Ws, thr, mp), rtol=1e-5, atol=0)
    lthr, lmp, lmse = lowra.lowra_learn_tables(lay, W, thr_d, mp_d, 2)
    torch.cuda.synchronize()
    rthr, rmp, rmse, _ = orc.learn_tables(Ws, bits[rows], cb[rows], thr, mp, 2)
    assert np.allclose(lmp[rows_d].cpu().numpy(), rmp, rtol=0, atol=2e-6)
    assert np.allclose(lthr[rows_d].cpu().numpy(), rthr, rtol=0, atol=2e-6)
    assert np.allclose(lmse[rows_d].cpu().numpy().astype(np.float64), rmse, rtol=1e-4, atol=1e-9)
    del W, mse, lthr, lmp, lmse

    A = synth.to_bf16_bits(np.random.default_rng([synth.SEED, 66562]).normal(0.0, 0.01, size=(R, K)))
    B = synth.to_bf16_bits(np.random.default_rng([synth.SEED, 66563]).normal(0.0, 0.01, size=(N, R)))
    A_d, B_d = bf16_dev(A), bf16_dev(B)
    for M in (4, 24):                     # the small-token path and the GEMM path
        print(f"[large] linear, {M} tokens", flush=True)
        x = synth.to_bf16_bits(np.random.default_rng([synth.SEED, 66564, M]).normal(0.0, 1.0, size=(M, K)))
        dY = synth.to_bf16_bits(np.random.default_rng([synth.SEED, 66565, M]).normal(0.0, 1.0, size=(M, N)))
        x_d, dY_d = bf16_dev(x), bf16_dev(dY)
        y = lowra.lowra_linear_fwd(lay, packed, absmax, mp_d, x_d, A_d, B_d, 2.0)
        dX = lowra.lowra_linear_bwd_input(lay, packed, absmax, mp_d, dY_d, A_d, B_d, 2.0)
        torch.cuda.synchronize()
        ref = orc.linear_fwd(rp, ra, bits[rows], cb[rows], mp, x, A, np.ascontiguousarray(B[rows]), 2.0)
        yh = bf16_host_f64(y)
        assert rel_err(yh[:, rows], ref) <= REL_TOL
        # <dY, fwd(x)> == <bwd(dY), x>: both are the same bilinear form of the decoded weights
        dYf, xf, dXh = synth.bf16_bits_to_f64(dY), synth.bf16_bits_to_f64(x), bf16_host_f64(dX)
        lhs, rhs = float((dYf * yh).sum()), float((dXh * xf).sum())
        assert abs(lhs - rhs) <= 1e-2 * np.sqrt(float((yh * yh).sum()) * float((dYf * dYf).sum()))
        assert np.isfinite(dXh).all()
