"""lowra_linear_fwd_static (the entry point that allocates nothing) against lowra_linear_fwd.

Both run the same kernels, so the outputs must be bit-identical; the existing entry point is itself
held to the oracle (2e-2 rule) by the other GPU tests, and the first case here repeats that check.
Two calls in a row share the GPU's static scratch: the second one is smaller (fewer tokens, a smaller
layer, another rank) and must not see anything of the first.
"""
import numpy as np
import pytest
import torch

from oracle import lowra_oracle as orc
from paper_2502_08141_amd import lowra, synth
from tests.gpu_util import REL_TOL, DeviceLayer, bf16_host_f64, rel_err

pytestmark = pytest.mark.gpu


def both(D, M):
    L = D.L
    x = D.x[:M].contiguous()
    want = lowra.lowra_linear_fwd(D.layout, D.packed, D.absmax, D.mp, x, D.A, D.B, L.s)
    y = torch.full((M, L.N), float("nan"), dtype=torch.bfloat16, device="cuda")
    got = lowra.lowra_linear_fwd_static(D.layout, D.packed, D.absmax, D.mp, x, D.A, D.B, L.s, y)
    torch.cuda.synchronize()
    return got, want


def test_static_scratch_entry_matches_workspace_entry():
    big = DeviceLayer(synth.make_custom(520, 1024, 300, 24, fractions=(0.4, 0.3, 0.3), seed=51)); big.quantize()
    small = DeviceLayer(synth.make_custom(264, 512, 40, 8, fractions=(0.5, 0.25, 0.25), seed=52)); small.quantize()
    # first call: 300 tokens, rank 24 (padded adapter copy + rank-r intermediate in the scratch), MFMA GEMM path
    got, want = both(big, 300)
    assert torch.equal(got, want)
    L = big.L
    rp, ra = orc.quantize(L.W, L.bits, L.cb, L.thresholds)
    ref = orc.linear_fwd(rp, ra, L.bits, L.cb, L.mappings, L.x, L.A, L.B, L.s)
    assert rel_err(bf16_host_f64(got), ref) <= REL_TOL
    # second call right after it, smaller in every respect
    got, want = both(small, 40)
    assert torch.equal(got, want)
    # and the small-token path (M <= 16) through the same scratch, after the larger calls
    got, want = both(big, 4)
    assert torch.equal(got, want)
    got, want = both(small, 1)
    assert torch.equal(got, want)


def test_static_scratch_entry_rejects_oversize():
    D = DeviceLayer(synth.make_custom(64, 128, 4, 64, seed=53)); D.quantize()
    M = 40000                                                      # 40000 x 64 bf16 > 4 MiB
    assert D.layout.workspace_bytes(lowra.OP_LINEAR_FWD, M, 64) > lowra.STATIC_SCRATCH_BYTES
    x = torch.zeros((M, 128), dtype=torch.bfloat16, device="cuda")
    y = torch.empty((M, 64), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(lowra.LowraError) as e:
        lowra.lowra_linear_fwd_static(D.layout, D.packed, D.absmax, D.mp, x, D.A, D.B, 2.0, y)
    assert e.value.status == lowra.WORKSPACE_TOO_SMALL
