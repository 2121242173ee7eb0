"""GPU parity on the full-model weight set (config 5): decoder layers 0 and 31, all seven matrices.

Each matrix is quantized on the GPU and compared bit for bit with the oracle; the small-token
forward and input gradient (token counts 1, 4, 16; LoRA rank 16) are compared with the fp64 oracle
on every output.  The token batches for 1 and 4 tokens are the leading rows of the 16-token draw.
"""
import numpy as np
import pytest
import torch

from oracle import lowra_oracle as orc
from paper_2502_08141_amd import lowra, synth
from tests.gpu_util import REL_TOL, DeviceLayer, bf16_host_f64, oracle_state, rel_err

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("layer", [0, synth.LLAMA7B_LAYERS - 1])
@pytest.mark.parametrize("idx", range(len(synth.LLAMA7B_LAYER)))
def test_config5_matrix(layer, idx):
    print(f"[cfg 5 layer {layer} matrix {synth.LLAMA7B_LAYER[idx][0]}] generating", flush=True)
    L = synth.make_cfg5_matrix(layer, idx, M=max(synth.CFG5_TOKENS))
    D = DeviceLayer(L)
    D.quantize()
    torch.cuda.synchronize()
    ref_packed, ref_absmax = oracle_state(L)
    assert np.array_equal(D.absmax.cpu().numpy(), ref_absmax)
    assert np.array_equal(D.packed.cpu().numpy(), ref_packed)
    for M in synth.CFG5_TOKENS:
        print(f"  forward, {M} token(s)", flush=True)
        x = D.x[:M].contiguous()
        y = lowra.lowra_linear_fwd(D.layout, D.packed, D.absmax, D.mp, x, D.A, D.B, L.s)   # PATH_AUTO: small-token kernel
        torch.cuda.synchronize()
        ref = orc.linear_fwd(ref_packed, ref_absmax, L.bits, L.cb, L.mappings, L.x[:M], L.A, L.B, L.s)
        assert rel_err(bf16_host_f64(y), ref) <= REL_TOL
        print(f"  input gradient, {M} token(s)", flush=True)
        dY = D.dY[:M].contiguous()
        dX = lowra.lowra_linear_bwd_input(D.layout, D.packed, D.absmax, D.mp, dY, D.A, D.B, L.s)   # PATH_AUTO: streaming kernel
        torch.cuda.synchronize()
        ref = orc.linear_bwd_input(ref_packed, ref_absmax, L.bits, L.cb, L.mappings, L.dY[:M], L.A, L.B, L.s, L.K)
        assert rel_err(bf16_host_f64(dX), ref) <= REL_TOL
