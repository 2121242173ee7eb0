"""GPU parity at the full sizes of the benchmark configs, in the launch configuration bench.py times.

Quantize / dequantize are compared in full (bit exact).  The linear calls run on the whole token
batch; the oracle recomputes a seeded sample of token rows (each row of y / dX depends only on the
same row of x / dY), every column of each: the first and the last row of EVERY 256-token tile plus
two seeded rows inside it, so that every output tile of both GEMM grids (and the XCD-aware tile
order at the real grid size) has checked outputs.
"""
import numpy as np
import pytest
import torch

from oracle import lowra_oracle as orc
from paper_2502_08141_amd import lowra, synth
from tests.gpu_util import REL_TOL, DeviceLayer, bf16_host_bits, bf16_host_f64, oracle_state, rel_err

pytestmark = pytest.mark.gpu
TOKEN_TILE = 256


def sample_rows(M, key):
    """Both edges of every 256-token tile and two seeded rows strictly inside it."""
    rng = np.random.default_rng(key)
    rows = []
    for t0 in range(0, M, TOKEN_TILE):
        t1 = min(t0 + TOKEN_TILE, M)
        rows += [t0, t1 - 1]
        if t1 - t0 > 2:
            rows += list(t0 + 1 + rng.choice(t1 - t0 - 2, size=min(2, t1 - t0 - 2), replace=False))
    return np.unique(np.array(rows, dtype=np.int64))


@pytest.mark.parametrize("cfg", [2, 3, 4])
def test_full_config(cfg):
    print(f"[cfg {cfg}] generating", flush=True)
    L = synth.make_config(cfg)
    D = DeviceLayer(L)
    D.quantize()
    torch.cuda.synchronize()
    print(f"[cfg {cfg}] oracle quantize", flush=True)
    ref_packed, ref_absmax = oracle_state(L)
    assert np.array_equal(D.absmax.cpu().numpy(), ref_absmax)
    assert np.array_equal(D.packed.cpu().numpy(), ref_packed)
    assert D.layout.packed_bytes == int(round(L.mean_bits * L.N * L.K / 8))

    print(f"[cfg {cfg}] dequantize", flush=True)
    What = lowra.lowra_dequantize(D.layout, D.packed, D.absmax, D.mp)
    torch.cuda.synchronize()
    assert np.array_equal(bf16_host_bits(What), orc.dequantize(ref_packed, ref_absmax, L.bits, L.cb, L.mappings, L.K))
    del What

    rows = sample_rows(L.M, [synth.SEED, cfg, 77])
    assert set(rows // TOKEN_TILE) == set(range((L.M + TOKEN_TILE - 1) // TOKEN_TILE))
    print(f"[cfg {cfg}] forward", flush=True)
    y = lowra.lowra_linear_fwd(D.layout, D.packed, D.absmax, D.mp, D.x, D.A, D.B, L.s)
    torch.cuda.synchronize()
    ref = orc.linear_fwd(ref_packed, ref_absmax, L.bits, L.cb, L.mappings, L.x[rows], L.A, L.B, L.s)
    assert rel_err(bf16_host_f64(y[torch.from_numpy(rows).cuda()]), ref) <= REL_TOL
    del y
    print(f"[cfg {cfg}] backward", flush=True)
    dX = lowra.lowra_linear_bwd_input(D.layout, D.packed, D.absmax, D.mp, D.dY, D.A, D.B, L.s)
    torch.cuda.synchronize()
    ref = orc.linear_bwd_input(ref_packed, ref_absmax, L.bits, L.cb, L.mappings, L.dY[rows], L.A, L.B, L.s, L.K)
    assert rel_err(bf16_host_f64(dX[torch.from_numpy(rows).cuda()]), ref) <= REL_TOL


@pytest.mark.parametrize("r", [24, 64])      # 64: LoRA B is read in place by the input gradient's side product
def test_tall_ragged_tokens(r):
    """4130 tokens (not a multiple of 64) and 8200 channels: the input gradient's rank-r side product
    takes the 64-row workgroups with a split contraction (three slices, the last one ragged); sampled
    token rows around the block boundaries and the ragged end."""
    print(f"[tall ragged r={r}] generating", flush=True)
    L = synth.make_custom(8200, 1536, 4130, r, fractions=(0.5, 0.3, 0.2), seed=71)
    D = DeviceLayer(L)
    D.quantize()
    torch.cuda.synchronize()
    ref_packed, ref_absmax = oracle_state(L)
    rows = np.unique(np.concatenate([np.array([0, 63, 64, 4031, 4032, 4095, 4096, 4127, 4128, 4129]),
                                     np.random.default_rng([synth.SEED, 71]).choice(L.M, 14, replace=False)]))
    rows_d = torch.from_numpy(rows).cuda()
    y = lowra.lowra_linear_fwd(D.layout, D.packed, D.absmax, D.mp, D.x, D.A, D.B, L.s)
    dX = lowra.lowra_linear_bwd_input(D.layout, D.packed, D.absmax, D.mp, D.dY, D.A, D.B, L.s)
    torch.cuda.synchronize()
    ref = orc.linear_fwd(ref_packed, ref_absmax, L.bits, L.cb, L.mappings, L.x[rows], L.A, L.B, L.s)
    assert rel_err(bf16_host_f64(y[rows_d]), ref) <= REL_TOL
    ref = orc.linear_bwd_input(ref_packed, ref_absmax, L.bits, L.cb, L.mappings, L.dY[rows], L.A, L.B, L.s, L.K)
    assert rel_err(bf16_host_f64(dX[rows_d]), ref) <= REL_TOL
    # the LoRA term alone (s = large against a zero base would need another layout): compare the adapter gradients,
    # which read both side products, on sampled channels / input columns
    dA, dB = lowra.lowra_adapter_grads(D.layout, D.x, D.dY, D.A, D.B, L.s)
    torch.cuda.synchronize()
    nsel = np.array([0, 1, 4771, 8199]); ksel = np.array([0, 5, 800, 1535])
    _, rB = orc.adapter_grads(L.x, np.ascontiguousarray(L.dY[:, nsel]), L.A, np.ascontiguousarray(L.B[nsel]), L.s)
    assert rel_err(dB[torch.from_numpy(nsel).cuda()].cpu().numpy().astype(np.float64), rB) <= REL_TOL
    rA, _ = orc.adapter_grads(np.ascontiguousarray(L.x[:, ksel]), L.dY, np.ascontiguousarray(L.A[:, ksel]), L.B, L.s)
    assert rel_err(dA[:, torch.from_numpy(ksel).cuda()].cpu().numpy().astype(np.float64), rA) <= REL_TOL
