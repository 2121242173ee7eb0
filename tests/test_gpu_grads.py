"""GPU parity of the adapter gradients (lowra_adapter_grads) against the fp64 oracle.

dA and dB come out in fp32 from bf16 operands, with the rank-r intermediates rounded to bf16 as in
the two linear calls; the bar is the one of the linear outputs (max relative error 2e-2 with the
rms floor).  At the benchmark size the oracle recomputes a seeded sample of channels of dB and of
input columns of dA (row n of dB depends on column n of dY only, column k of dA on column k of x).
"""
import numpy as np
import pytest
import torch

from oracle import lowra_oracle as orc
from paper_2502_08141_amd import lowra, synth
from tests.gpu_util import REL_TOL, bf16_dev, rel_err

pytestmark = pytest.mark.gpu


def cases():
    return {
        "cfg1": lambda: synth.make_config(1),
        "ragged": lambda: synth.make_custom(520, 320, 300, 8, seed=41),
        "one_token": lambda: synth.make_custom(72, 64, 1, 5, seed=42),
        "rank64_chunks": lambda: synth.make_custom(264, 448, 1300, 64, seed=43),      # several token chunks, ragged last one
        "rank33_wide": lambda: synth.make_custom(1032, 1088, 515, 33, seed=44),
        "tall_ragged": lambda: synth.make_custom(136, 256, 4130, 24, seed=50),
        "tokens_256": lambda: synth.make_custom(128, 256, 256, 16, seed=45),          # exactly one chunk, no tail
        "tokens_257": lambda: synth.make_custom(128, 256, 257, 16, seed=46),          # one token past a stage boundary
    }


def run(L):
    layout = lowra.Layout(L.K, L.bits, L.cb, L.cb_bits)
    dA, dB = lowra.lowra_adapter_grads(layout, bf16_dev(L.x), bf16_dev(L.dY), bf16_dev(L.A), bf16_dev(L.B), L.s)
    torch.cuda.synchronize()
    return layout, dA, dB


@pytest.mark.parametrize("name", list(cases()))
def test_adapter_grads(name):
    print(f"[grads {name}]", flush=True)
    L = cases()[name]()
    _, dA, dB = run(L)
    rA, rB = orc.adapter_grads(L.x, L.dY, L.A, L.B, L.s)
    assert dA.shape == rA.shape and dB.shape == rB.shape
    assert rel_err(dA.cpu().numpy().astype(np.float64), rA) <= REL_TOL
    assert rel_err(dB.cpu().numpy().astype(np.float64), rB) <= REL_TOL


def test_adapter_grads_full_size_sampled():
    print("[grads cfg3] generating", flush=True)
    L = synth.make_config(3)
    _, dA, dB = run(L)
    rng = np.random.default_rng([synth.SEED, 3, 91])
    nsel = np.sort(rng.choice(L.N, 40, replace=False)); nsel[0], nsel[-1] = 0, L.N - 1
    ksel = np.sort(rng.choice(L.K, 40, replace=False)); ksel[0], ksel[-1] = 0, L.K - 1
    print("[grads cfg3] oracle dB sample", flush=True)
    _, rB = orc.adapter_grads(L.x, np.ascontiguousarray(L.dY[:, nsel]), L.A, np.ascontiguousarray(L.B[nsel]), L.s)
    assert rel_err(dB[torch.from_numpy(nsel).cuda()].cpu().numpy().astype(np.float64), rB) <= REL_TOL
    print("[grads cfg3] oracle dA sample", flush=True)
    rA, _ = orc.adapter_grads(np.ascontiguousarray(L.x[:, ksel]), L.dY, np.ascontiguousarray(L.A[:, ksel]), L.B, L.s)
    assert rel_err(dA[:, torch.from_numpy(ksel).cuda()].cpu().numpy().astype(np.float64), rA) <= REL_TOL


def test_adapter_grads_deterministic_and_workspace_reuse():
    L = synth.make_custom(264, 448, 700, 16, seed=47)
    layout = lowra.Layout(L.K, L.bits, L.cb, L.cb_bits)
    x, dY, A, B = bf16_dev(L.x), bf16_dev(L.dY), bf16_dev(L.A), bf16_dev(L.B)
    ws = torch.empty(layout.workspace_bytes(lowra.OP_ADAPTER_GRADS, L.M, L.r), dtype=torch.uint8, device="cuda")
    ws.fill_(0xFF)                                            # stale workspace contents must not matter
    a1, b1 = lowra.lowra_adapter_grads(layout, x, dY, A, B, L.s, workspace=ws)
    a2, b2 = lowra.lowra_adapter_grads(layout, x, dY, A, B, L.s, workspace=ws)
    torch.cuda.synchronize()
    assert torch.equal(a1, a2) and torch.equal(b1, b2)


def test_adapter_grads_edges_and_errors():
    L = synth.make_custom(72, 128, 4, 8, seed=48)
    layout = lowra.Layout(L.K, L.bits, L.cb, L.cb_bits)
    x, dY, A, B = bf16_dev(L.x), bf16_dev(L.dY), bf16_dev(L.A), bf16_dev(L.B)
    # no tokens: both gradients are zero
    dA, dB = lowra.lowra_adapter_grads(layout, x[:0], dY[:0], A, B, L.s)
    torch.cuda.synchronize()
    assert not dA.any() and not dB.any()
    # zero scale
    dA, dB = lowra.lowra_adapter_grads(layout, x, dY, A, B, 0.0)
    torch.cuda.synchronize()
    assert not dA.any() and not dB.any()
    # workspace too small
    small = torch.empty(16, dtype=torch.uint8, device="cuda")
    with pytest.raises(lowra.LowraError, match="workspace too small"):
        lowra.lowra_adapter_grads(layout, x, dY, A, B, L.s, workspace=small)
    # rank beyond the supported 64
    L2 = synth.make_custom(72, 128, 4, 100, seed=49)
    with pytest.raises(lowra.LowraError, match="unsupported"):
        lowra.lowra_adapter_grads(layout, bf16_dev(L2.x), bf16_dev(L2.dY), bf16_dev(L2.A), bf16_dev(L2.B), L2.s)


@pytest.mark.parametrize("name", ["ragged", "rank64_chunks", "rank33_wide", "tall_ragged"])
def test_adapter_grads_from_side_products(name):
    """The variant that takes s x A^T and s dY B from the workspaces of the step's two linear calls reads x and dY
    once; its results are those of the standalone call bit for bit (the same kernels on the same intermediates),
    and so meet the oracle to the same bar."""
    L = cases()[name]()
    print(f"[grads from side products {name}] N={L.N} K={L.K} M={L.M} r={L.r}", flush=True)
    layout = lowra.Layout(L.K, L.bits, L.cb, L.cb_bits)
    thr, mp = torch.from_numpy(L.thresholds).cuda(), torch.from_numpy(L.mappings).cuda()
    packed, absmax = lowra.lowra_quantize(layout, torch.from_numpy(L.W).cuda(), thr)
    x, dY, A, B = bf16_dev(L.x), bf16_dev(L.dY), bf16_dev(L.A), bf16_dev(L.B)
    ws_f = torch.empty(layout.workspace_bytes(lowra.OP_LINEAR_FWD, L.M, L.r), dtype=torch.uint8, device="cuda")
    ws_b = torch.empty(layout.workspace_bytes(lowra.OP_LINEAR_BWD_INPUT, L.M, L.r), dtype=torch.uint8, device="cuda")
    lowra.lowra_linear_fwd(layout, packed, absmax, mp, x, A, B, L.s, workspace=ws_f)
    lowra.lowra_linear_bwd_input(layout, packed, absmax, mp, dY, A, B, L.s, workspace=ws_b)
    st = lowra.lowra_linear_side_product(layout, lowra.OP_LINEAR_FWD, L.M, L.r, ws_f)
    su = lowra.lowra_linear_side_product(layout, lowra.OP_LINEAR_BWD_INPUT, L.M, L.r, ws_b)
    assert st is not None and su is not None and tuple(st.shape) == (L.M, 64)
    dA, dB = lowra.lowra_adapter_grads_from_side(layout, x, dY, L.r, st, su)
    rA, rB = lowra.lowra_adapter_grads(layout, x, dY, A, B, L.s)
    torch.cuda.synchronize()
    assert torch.equal(dA, rA) and torch.equal(dB, rB)
    oA, oB = orc.adapter_grads(L.x, L.dY, L.A, L.B, L.s)
    assert rel_err(dA.cpu().numpy().astype(np.float64), oA) <= REL_TOL
    assert rel_err(dB.cpu().numpy().astype(np.float64), oB) <= REL_TOL


def test_side_product_is_absent_where_no_call_leaves_one():
    L = synth.make_custom(72, 1024, 4, 8, seed=52)
    layout = lowra.Layout(L.K, L.bits, L.cb, L.cb_bits)
    ws = torch.empty(layout.workspace_bytes(lowra.OP_LINEAR_BWD_INPUT, 300, 100), dtype=torch.uint8, device="cuda")
    assert lowra.lowra_linear_side_product(layout, lowra.OP_LINEAR_FWD, L.M, L.r, ws) is None        # 4 tokens: a small-token kernel
    assert lowra.lowra_linear_side_product(layout, lowra.OP_LINEAR_FWD, 300, 0, ws) is None          # no rank-r term
    assert lowra.lowra_linear_side_product(layout, lowra.OP_LINEAR_FWD, 300, 100, ws) is None        # rank beyond 64
    assert lowra.lowra_linear_side_product(layout, lowra.OP_ADAPTER_GRADS, 300, 8, ws) is None       # not a linear call
    assert lowra.lowra_linear_side_product(layout, lowra.OP_LINEAR_BWD_INPUT, 300, 8, ws) is not None
