"""Seeded random shapes within the documented limits, each through quantize (bit-exact), the forward, the input
gradient and, where the rank allows, the adapter gradients, against the oracle at the linear calls' bar.  The shapes
are drawn to reach the code paths that fixed cases reach only by design: GEMM shapes with ragged tiles and any rank,
small-token shapes (K a multiple of 256 from 1024) with ranks that are no multiple of 8, and long contractions over
few output tiles (the input gradient's split contraction).  One seed per case, so a failure names its shape."""
import numpy as np
import pytest
import torch

from oracle import lowra_oracle as orc
from paper_2502_08141_amd import lowra, synth
from tests.gpu_util import REL_TOL, DeviceLayer, bf16_host_f64, oracle_state, rel_err

pytestmark = pytest.mark.gpu


def draw(ci):
    rng = np.random.default_rng([synth.SEED, 909, ci])
    kind = int(rng.integers(0, 3))
    if kind == 0:      # GEMM shapes
        N, K, M = int(rng.integers(1, 300)) * 8, int(rng.integers(1, 33)) * 64, int(rng.integers(17, 900))
        r = int(rng.choice([0, 5, 8, 16, 20, 24, 33, 64]))
    elif kind == 1:    # small-token streaming shapes
        N, K, M = int(rng.integers(2, 200)) * 8, int(rng.integers(4, 24)) * 256, int(rng.integers(1, 17))
        r = int(rng.choice([0, 5, 8, 16, 20, 32]))
    else:              # long contraction, few output tiles
        N, K, M = int(rng.integers(64, 600)) * 8, int(rng.integers(1, 9)) * 64, int(rng.integers(17, 600))
        r = int(rng.choice([0, 5, 8, 16, 20, 24, 33, 64]))
    fr = rng.dirichlet([1, 1, 1])
    fr = (float(fr[0] + fr[2]), float(fr[1]), 0.0) if rng.random() < 0.3 else tuple(float(v) for v in fr)
    per_channel = bool(rng.random() < 0.2) and kind != 1
    return N, K, M, r, fr, per_channel


@pytest.mark.parametrize("ci", range(48))
def test_random_shape(ci):
    N, K, M, r, fr, per_channel = draw(ci)
    print(f"[random shape {ci}] N={N} K={K} M={M} r={r} fractions=({fr[0]:.2f},{fr[1]:.2f},{fr[2]:.2f}) per_channel={per_channel}", flush=True)
    L = synth.make_custom(N, K, M, r, fractions=fr, seed=2000 + ci, per_channel_tables=per_channel)
    D = DeviceLayer(L)
    D.quantize()
    torch.cuda.synchronize()
    rp, ra = oracle_state(L)
    assert np.array_equal(D.packed.cpu().numpy(), rp) and np.array_equal(D.absmax.cpu().numpy(), ra)
    y = lowra.lowra_linear_fwd(D.layout, D.packed, D.absmax, D.mp, D.x, D.A, D.B, L.s)
    dX = lowra.lowra_linear_bwd_input(D.layout, D.packed, D.absmax, D.mp, D.dY, D.A, D.B, L.s)
    torch.cuda.synchronize()
    A, B = (L.A, L.B) if r else (None, None)
    assert rel_err(bf16_host_f64(y), orc.linear_fwd(rp, ra, L.bits, L.cb, L.mappings, L.x, A, B, L.s)) <= REL_TOL
    assert rel_err(bf16_host_f64(dX), orc.linear_bwd_input(rp, ra, L.bits, L.cb, L.mappings, L.dY, A, B, L.s, L.K)) <= REL_TOL
    if 0 < r <= 64:
        dA, dB = lowra.lowra_adapter_grads(D.layout, D.x, D.dY, D.A, D.B, L.s)
        torch.cuda.synchronize()
        oA, oB = orc.adapter_grads(L.x, L.dY, L.A, L.B, L.s)
        assert rel_err(dA.cpu().numpy().astype(np.float64), oA) <= REL_TOL
        assert rel_err(dB.cpu().numpy().astype(np.float64), oB) <= REL_TOL
