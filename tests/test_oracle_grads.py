"""Pins of the oracle's adapter gradients: numpy's fp64 matmul, and finite differences of the
separately pinned forward oracle (the layer is linear in A and in B, so a difference quotient is the
derivative up to rounding)."""
import numpy as np

from oracle import lowra_oracle as orc
from paper_2502_08141_amd import synth


def case(seed=3):
    return synth.make_custom(24, 192, 10, 5, seed=seed)


def test_adapter_grads_are_the_matmul_formulas():
    L = case()
    f = synth.bf16_bits_to_f64
    x, dY, A, B = f(L.x), f(L.dY), f(L.A), f(L.B)
    dA, dB = orc.adapter_grads(L.x, L.dY, L.A, L.B, L.s)
    assert np.allclose(dB, L.s * dY.T @ (x @ A.T), rtol=1e-12, atol=1e-15)
    assert np.allclose(dA, L.s * (dY @ B).T @ x, rtol=1e-12, atol=1e-15)


def test_adapter_grads_are_the_derivatives_of_the_forward_oracle():
    """loss = sum(y * dY); d loss / d B[n,j] and d loss / d A[j,k] by difference quotients of
    orc.linear_fwd with perturbations that bf16 represents exactly."""
    L = case(5)
    rp, ra = orc.quantize(L.W, L.bits, L.cb, L.thresholds)
    f = synth.bf16_bits_to_f64
    dYf = f(L.dY)

    def loss(Abits, Bbits):
        return float(np.sum(orc.linear_fwd(rp, ra, L.bits, L.cb, L.mappings, L.x, Abits, Bbits, L.s) * dYf))

    dA, dB = orc.adapter_grads(L.x, L.dY, L.A, L.B, L.s)
    base = loss(L.A, L.B)
    rng = np.random.default_rng(0)
    for _ in range(6):
        n, j = int(rng.integers(L.N)), int(rng.integers(L.r))
        Bp = f(L.B).copy(); Bp[n, j] += 0.25                 # exact in bf16 for these magnitudes? re-round and use the realised step
        Bb = synth.to_bf16_bits(Bp); step = f(Bb)[n, j] - f(L.B)[n, j]
        assert abs((loss(L.A, Bb) - base) / step - dB[n, j]) <= 1e-9 * max(1.0, abs(dB[n, j]))
        jj, k = int(rng.integers(L.r)), int(rng.integers(L.K))
        Ap = f(L.A).copy(); Ap[jj, k] += 0.25
        Ab = synth.to_bf16_bits(Ap); step = f(Ab)[jj, k] - f(L.A)[jj, k]
        assert abs((loss(Ab, L.B) - base) / step - dA[jj, k]) <= 1e-9 * max(1.0, abs(dA[jj, k]))


def test_zero_scale_and_zero_gradient():
    L = case(7)
    dA, dB = orc.adapter_grads(L.x, L.dY, L.A, L.B, 0.0)
    assert not dA.any() and not dB.any()
    dA, dB = orc.adapter_grads(L.x, np.zeros_like(L.dY), L.A, L.B, L.s)
    assert not dA.any() and not dB.any()
