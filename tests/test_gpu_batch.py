"""GPU checks of the batched small-token forward (lowra_fwd_batch_*) and input gradient (lowra_bwd_batch_*, at the
end of the file).  Forward: every matrix of a batch must
come out as from its own lowra_linear_fwd call on the small-token path -- the same kernel body runs,
possibly with the contraction split over another number of wavefronts, so up to the fp32 summation
order: one bf16 step at most -- and within the 2e-2 rule of the fp64 oracle."""
import numpy as np
import pytest
import torch

from oracle import lowra_oracle as orc
from paper_2502_08141_amd import lowra, synth
from tests.gpu_util import REL_TOL, DeviceLayer, bf16_dev, bf16_host_f64, oracle_state, rel_err

pytestmark = pytest.mark.gpu

# (N, K, fractions): different widths, lengths and kernel instantiations in one batch
SHAPES = [(328, 1024, (0.34, 0.33, 0.33)), (136, 11008, (0.5, 0.5, 0.0)), (520, 4096, (0.5, 0.25, 0.25)),
          (4112, 1024, (0.3, 0.3, 0.4)), (264, 1024, (1.0, 0.0, 0.0))]


def build(M, r):
    layers = []
    for i, (N, K, fr) in enumerate(SHAPES):
        L = synth.make_custom(N, K, M, r, fractions=fr, seed=80 + i)
        D = DeviceLayer(L)
        D.quantize()
        layers.append(D)
    torch.cuda.synchronize()
    return layers


@pytest.mark.parametrize("M,r", [(1, 16), (4, 16), (16, 16), (3, 0), (16, 24)])
def test_batch_equals_single_calls_and_oracle(M, r):
    print(f"[batch M={M} r={r}]", flush=True)
    layers = build(M, r)
    mp = layers[0].mp
    items = [(D.layout, D.packed, D.absmax, D.x, D.A if r else None, D.B if r else None) for D in layers]
    batch = lowra.FwdBatch(items, mp, layers[0].L.s)
    ys = batch.run()
    torch.cuda.synchronize()
    for D, y in zip(layers, ys):
        L = D.L
        single = lowra.lowra_linear_fwd(D.layout, D.packed, D.absmax, mp, D.x, D.A, D.B, L.s)
        torch.cuda.synchronize()
        diff = (y.float() - single.float()).abs()
        assert bool((diff <= single.float().abs() * 2.0 ** -7 + 1e-6).all())
        rp, ra = oracle_state(L)
        ref = orc.linear_fwd(rp, ra, L.bits, L.cb, L.mappings, L.x, L.A if r else None, L.B if r else None, L.s)
        assert rel_err(bf16_host_f64(y), ref) <= REL_TOL
    # a second run into the same outputs, after they were cleared
    keep = [y.clone() for y in ys]
    for y in ys:
        y.zero_()
    batch.run()
    torch.cuda.synchronize()
    for y, k in zip(ys, keep):
        assert torch.equal(y.view(torch.int16), k.view(torch.int16))
    batch.close()


def test_batch_errors():
    layers = build(4, 16)
    mp = layers[0].mp
    items = [(D.layout, D.packed, D.absmax, D.x, D.A, D.B) for D in layers[:2]]
    with pytest.raises(lowra.LowraError, match="workspace too small"):
        lowra.FwdBatch(items, mp, 2.0, workspace=torch.empty(64, dtype=torch.uint8, device="cuda"))
    # 17 tokens: not a small-token shape
    L = synth.make_custom(328, 1024, 17, 16, seed=90)
    D = DeviceLayer(L); D.quantize()
    with pytest.raises(lowra.LowraError, match="unsupported"):
        lowra.FwdBatch([(D.layout, D.packed, D.absmax, D.x, D.A, D.B)], mp, 2.0)
    with pytest.raises(ValueError):
        lowra.FwdBatch([], mp, 2.0)


def test_batch_in_a_graph():
    """The run is launches only: it can be captured and replayed."""
    layers = build(4, 16)
    mp = layers[0].mp
    batch = lowra.FwdBatch([(D.layout, D.packed, D.absmax, D.x, D.A, D.B) for D in layers], mp, 2.0)
    ys = batch.run()
    torch.cuda.synchronize()
    want = [y.clone() for y in ys]
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        batch.run()
    for rep in range(3):
        for y in ys:
            y.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for y, w in zip(ys, want):
            assert torch.equal(y.view(torch.int16), w.view(torch.int16))
    batch.close()


# ---- the batched small-token input gradient (lowra_bwd_batch_*)
# Matrices of one batch share the codebooks' widths; K a multiple of 256 from 1024 up (the streaming kernel's shapes).
BWD_SHAPES = [(328, 1024, (0.34, 0.33, 0.33)), (136, 11008, (0.5, 0.5, 0.0)), (520, 4096, (0.5, 0.25, 0.25)),
              (4112, 1024, (0.3, 0.3, 0.4)), (264, 2304, (1.0, 0.0, 0.0)), (136, 4096, (0.0, 0.0, 1.0))]


def build_bwd(M, r):
    layers = []
    for i, (N, K, fr) in enumerate(BWD_SHAPES):
        D = DeviceLayer(synth.make_custom(N, K, M, r, fractions=fr, seed=180 + i))
        D.quantize()
        layers.append(D)
    torch.cuda.synchronize()
    return layers


@pytest.mark.parametrize("M,r", [(1, 16), (4, 16), (16, 32), (3, 0), (13, 24), (7, 5), (2, 20)])     # ranks 5 and 20: rows of B that are no multiple of 16 bytes
def test_bwd_batch_equals_single_calls_and_oracle(M, r):
    """Every matrix of a batch comes out as from its own lowra_linear_bwd_input call (the same kernel; the
    workgroup ranges, hence the order of the fp32 partial sums, differ: one bf16 step at most) and within
    the 2e-2 rule of the fp64 oracle."""
    print(f"[bwd batch M={M} r={r}]", flush=True)
    layers = build_bwd(M, r)
    mp = layers[0].mp
    items = [(D.layout, D.packed, D.absmax, D.dY, D.A if r else None, D.B if r else None) for D in layers]
    batch = lowra.BwdBatch(items, mp, layers[0].L.s)
    dXs = batch.run()
    torch.cuda.synchronize()
    for D, dX in zip(layers, dXs):
        L = D.L
        single = lowra.lowra_linear_bwd_input(D.layout, D.packed, D.absmax, mp, D.dY, D.A, D.B, L.s)
        torch.cuda.synchronize()
        diff = (dX.float() - single.float()).abs()
        assert bool((diff <= single.float().abs() * 2.0 ** -7 + 1e-5 * float(single.float().abs().max())).all())
        rp, ra = oracle_state(L)
        ref = orc.linear_bwd_input(rp, ra, L.bits, L.cb, L.mappings, L.dY, L.A if r else None, L.B if r else None, L.s, L.K)
        assert rel_err(bf16_host_f64(dX), ref) <= REL_TOL
    # a second run into the same outputs, after they were cleared: the partial slots are rewritten, nothing accumulates
    keep = [d.clone() for d in dXs]
    for d in dXs:
        d.zero_()
    batch.run()
    torch.cuda.synchronize()
    for d, k in zip(dXs, keep):
        assert torch.equal(d.view(torch.int16), k.view(torch.int16))
    batch.close()


def test_bwd_batch_errors():
    layers = build_bwd(4, 16)
    mp = layers[0].mp
    items = [(D.layout, D.packed, D.absmax, D.dY, D.A, D.B) for D in layers[:2]]
    with pytest.raises(lowra.LowraError, match="workspace too small"):
        lowra.BwdBatch(items, mp, 2.0, workspace=torch.empty(64, dtype=torch.uint8, device="cuda"))
    # K = 320 is not a shape of the streaming kernel
    D = DeviceLayer(synth.make_custom(520, 320, 4, 16, seed=190)); D.quantize()
    with pytest.raises(lowra.LowraError, match="unsupported"):
        lowra.BwdBatch([(D.layout, D.packed, D.absmax, D.dY, D.A, D.B)], mp, 2.0)
    # 17 tokens
    D = DeviceLayer(synth.make_custom(328, 1024, 17, 16, seed=191)); D.quantize()
    with pytest.raises(lowra.LowraError, match="unsupported"):
        lowra.BwdBatch([(D.layout, D.packed, D.absmax, D.dY, D.A, D.B)], mp, 2.0)


def test_bwd_batch_in_a_graph():
    """The run is launches only: it can be captured and replayed."""
    layers = build_bwd(4, 16)
    mp = layers[0].mp
    batch = lowra.BwdBatch([(D.layout, D.packed, D.absmax, D.dY, D.A, D.B) for D in layers], mp, 2.0)
    dXs = batch.run()
    torch.cuda.synchronize()
    want = [d.clone() for d in dXs]
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        batch.run()
    for rep in range(3):
        for d in dXs:
            d.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for d, w in zip(dXs, want):
            assert torch.equal(d.view(torch.int16), w.view(torch.int16))
    batch.close()
