"""Pins for the oracle's linear steps L1 / L2 -- CPU only.

The loops in the oracle are checked against numpy's fp64 matmul on the decoded weights, special
cases that reduce to a plain GEMM, a hand-worked 2x2 example, and the adjoint identity.
"""
import numpy as np
import pytest

from oracle import lowra_oracle as orc
from paper_2502_08141_amd import synth

f64 = synth.bf16_bits_to_f64


def prepared(seed=0, N=40, K=192, M=9, r=5, s=2.0, per_channel=False):
    L = synth.make_custom(N, K, M, r, seed=seed, s=s, per_channel_tables=per_channel)
    packed, absmax = orc.quantize(L.W, L.bits, L.cb, L.thresholds)
    What = f64(orc.dequantize(packed, absmax, L.bits, L.cb, L.mappings, L.K))
    return L, packed, absmax, What


@pytest.mark.parametrize("seed,per_channel", [(0, False), (1, True)])
def test_forward_equals_numpy_matmul(seed, per_channel):
    L, packed, absmax, What = prepared(seed=seed, per_channel=per_channel)
    y = orc.linear_fwd(packed, absmax, L.bits, L.cb, L.mappings, L.x, L.A, L.B, L.s)
    want = f64(L.x) @ What.T + L.s * (f64(L.x) @ f64(L.A).T) @ f64(L.B).T
    assert np.allclose(y, want, rtol=1e-12, atol=1e-13)
    lora = L.s * (f64(L.x) @ f64(L.A).T) @ f64(L.B).T
    assert np.abs(lora).max() > 1e-4 * np.abs(want).max()      # the LoRA term is not lost in the noise


def test_backward_equals_numpy_matmul():
    L, packed, absmax, What = prepared(seed=2)
    dX = orc.linear_bwd_input(packed, absmax, L.bits, L.cb, L.mappings, L.dY, L.A, L.B, L.s, L.K)
    want = f64(L.dY) @ What + L.s * (f64(L.dY) @ f64(L.B)) @ f64(L.A)
    assert np.allclose(dX, want, rtol=1e-12, atol=1e-13)


def test_no_lora_reduces_to_plain_gemm():
    L, packed, absmax, What = prepared(seed=3)
    y0 = orc.linear_fwd(packed, absmax, L.bits, L.cb, L.mappings, L.x, L.A, L.B, 0.0)
    y1 = orc.linear_fwd(packed, absmax, L.bits, L.cb, L.mappings, L.x, None, None, 2.0)
    y2 = orc.linear_fwd(packed, absmax, L.bits, L.cb, L.mappings, L.x, L.A, np.zeros_like(L.B), 2.0)
    want = f64(L.x) @ What.T
    for y in (y0, y1, y2):
        assert np.allclose(y, want, rtol=1e-12, atol=1e-13)
    d0 = orc.linear_bwd_input(packed, absmax, L.bits, L.cb, L.mappings, L.dY, None, None, 2.0, L.K)
    assert np.allclose(d0, f64(L.dY) @ What, rtol=1e-12, atol=1e-13)


def test_hand_worked_tiny_linear():
    """N=2, K=64, M=1, r=1 with weights that decode exactly: row 0 = +-0.5 (1 bit), row 1 two-level
    2-bit pattern.  x = e_0 + 2 e_1, so y_n = What[n,0] + 2 What[n,1] + s * (x.A) * B[n]."""
    thr, mp, _ = synth.shared_codebooks()
    W = np.zeros((2, 64), np.float32)
    W[0] = -0.5; W[0, 0] = 0.5                     # 1-bit: decodes to +-0.5
    W[1] = -0.25; W[1, 1] = 0.25                   # 2-bit: levels +-1 only -> +-0.25
    bits = np.array([1, 2], np.uint8); cb = np.array([0, 1], np.int32)
    packed, absmax = orc.quantize(W, bits, cb, thr)
    x = np.zeros((1, 64)); x[0, 0] = 1; x[0, 1] = 2
    A = np.zeros((1, 64)); A[0, 0] = 3; A[0, 1] = 0.5          # x.A = 3 + 1 = 4
    B = np.array([[0.5], [-1.0]])
    y = orc.linear_fwd(packed, absmax, bits, cb, mp, synth.to_bf16_bits(x), synth.to_bf16_bits(A),
                       synth.to_bf16_bits(B), 0.5)
    assert y[0, 0] == 0.5 + 2 * -0.5 + 0.5 * 4 * 0.5          # = 0.5
    assert y[0, 1] == -0.25 + 2 * 0.25 + 0.5 * 4 * -1.0       # = -1.75
    dY = np.array([[1.0, 2.0]])
    dX = orc.linear_bwd_input(packed, absmax, bits, cb, mp, synth.to_bf16_bits(dY), synth.to_bf16_bits(A),
                              synth.to_bf16_bits(B), 0.5, 64)
    u = 1 * 0.5 + 2 * -1.0                                     # dY.B = -1.5
    assert dX[0, 0] == 1 * 0.5 + 2 * -0.25 + 0.5 * u * 3
    assert dX[0, 1] == 1 * -0.5 + 2 * 0.25 + 0.5 * u * 0.5
    assert dX[0, 2] == 1 * -0.5 + 2 * -0.25


def test_adjoint_identity():
    """The layer is linear in x, so <dY, fwd(x)> == <bwd(dY), x> up to fp64 round-off."""
    L, packed, absmax, _ = prepared(seed=4, N=56, K=256, M=7, r=6)
    y = orc.linear_fwd(packed, absmax, L.bits, L.cb, L.mappings, L.x, L.A, L.B, L.s)
    dX = orc.linear_bwd_input(packed, absmax, L.bits, L.cb, L.mappings, L.dY, L.A, L.B, L.s, L.K)
    lhs = float((f64(L.dY) * y).sum()); rhs = float((dX * f64(L.x)).sum())
    assert abs(lhs - rhs) <= 1e-11 * max(abs(lhs), abs(rhs), 1.0)


def test_token_rows_are_independent():
    """A row subset of x gives the same rows of y: what sampled checks at full size rely on."""
    L, packed, absmax, _ = prepared(seed=5, M=12)
    y = orc.linear_fwd(packed, absmax, L.bits, L.cb, L.mappings, L.x, L.A, L.B, L.s)
    rows = [1, 7, 10]
    ys = orc.linear_fwd(packed, absmax, L.bits, L.cb, L.mappings, L.x[rows], L.A, L.B, L.s)
    assert np.array_equal(ys, y[rows])
