"""Pins of the oracle's low-rank initialiser (loftq_init, best_rank_r).

The rank-r step is numpy's SVD; it is pinned by what the mathematics fixes without calling the SVD
again: exact recovery of a matrix of rank r, orthonormal rows, the Eckart-Young value through the
eigenvalues of the Gram matrix (another LAPACK routine), and no rank-r competitor doing better.
The alternation is pinned by its first step (quantization of W itself), by the residual it leaves
being what its outputs say, and by its objective: below plain quantization, not increasing (with
learned tables; nothing guarantees descent for an arbitrary quantizer)."""
import numpy as np

from oracle import lowra_oracle as orc
from paper_2502_08141_amd import synth


def layer(seed=1, N=96, K=256, fr=(0.4, 0.3, 0.3)):
    rng = np.random.default_rng(seed)
    # weights with some low-rank structure under the noise, like a trained layer
    W = rng.normal(0, 0.02, (N, K)) + 0.02 * rng.normal(0, 1, (N, 6)) @ rng.normal(0, 1, (6, K)) / np.sqrt(6)
    W = W.astype(np.float32)
    bits = synth.assign_bits(N, fr, np.random.default_rng([seed, 1]))
    thr0, mp0, cbb = synth.shared_codebooks()
    # per-channel tables from the learner (Sec. 5), as in the paper's pipeline: the quantile tables'
    # 1-bit levels of +-absmax leave an error larger than the weights, and the alternation then diverges
    thr, mp, _, _ = orc.learn_tables(W, bits, np.searchsorted(cbb, bits).astype(np.int32), thr0, mp0, 2)
    return W, bits, np.arange(N, dtype=np.int32), thr, mp


def test_best_rank_r_recovers_a_rank_r_matrix_and_has_orthonormal_rows():
    rng = np.random.default_rng(0)
    B0, A0 = rng.normal(size=(40, 5)), rng.normal(size=(5, 72))
    B, A = orc.best_rank_r(B0 @ A0, 5)
    assert np.allclose(B @ A, B0 @ A0, rtol=0, atol=1e-11)
    assert np.allclose(A @ A.T, np.eye(5), rtol=0, atol=1e-12)
    E = rng.normal(size=(40, 72))
    B, A = orc.best_rank_r(E, 7)
    assert np.allclose(B, E @ A.T) and np.allclose(A @ A.T, np.eye(7), atol=1e-12)


def test_best_rank_r_reaches_the_eckart_young_value_and_beats_competitors():
    rng = np.random.default_rng(2)
    E = rng.normal(size=(60, 48)) * rng.uniform(0.2, 3.0, size=(1, 48))
    r = 6
    B, A = orc.best_rank_r(E, r)
    got = np.linalg.norm(E - B @ A) ** 2
    ev = np.linalg.eigvalsh(E.T @ E)                      # ascending; squared singular values by another routine
    assert abs(got - ev[:-r].sum()) <= 1e-9 * ev.sum()
    for _ in range(50):                                   # projections onto other r-dimensional row spaces do worse
        Q, _ = np.linalg.qr(A.T + 0.3 * rng.normal(size=A.T.shape))
        assert np.linalg.norm(E - (E @ Q) @ Q.T) ** 2 >= got - 1e-9
    Q, _ = np.linalg.qr(rng.normal(size=(48, r)))
    assert np.linalg.norm(E - (E @ Q) @ Q.T) ** 2 > got


def test_first_step_quantizes_the_weights_themselves():
    W, bits, cb, thr, mp = layer(3)
    packed, absmax, A, B, obj = orc.loftq_init(W, bits, cb, thr, mp, 8, steps=1)
    rp, ra = orc.quantize(W, bits, cb, thr)
    assert np.array_equal(packed, rp) and np.array_equal(absmax, ra)
    E = W.astype(np.float64) - orc.dequantize(rp, ra, bits, cb, mp, W.shape[1], "fp32")
    B1, A1 = orc.best_rank_r(E, 8)
    assert np.allclose(B @ A, B1 @ A1, atol=1e-12) and abs(obj[0] - np.linalg.norm(E - B1 @ A1)) < 1e-12


def test_outputs_are_consistent_and_the_objective_behaves():
    for seed, r in ((4, 4), (5, 16)):
        W, bits, cb, thr, mp = layer(seed)
        K = W.shape[1]
        packed, absmax, A, B, obj = orc.loftq_init(W, bits, cb, thr, mp, r, steps=5)
        What = orc.dequantize(packed, absmax, bits, cb, mp, K, "fp32").astype(np.float64)
        assert abs(np.linalg.norm(W - What - B @ A) - obj[-1]) <= 1e-9          # the reported objective is the residual of the outputs
        assert A.shape == (r, K) and B.shape == (W.shape[0], r)
        rp, ra = orc.quantize(W, bits, cb, thr)
        plain = np.linalg.norm(W - orc.dequantize(rp, ra, bits, cb, mp, K, "fp32"))
        assert obj[0] < plain                                                    # the rank-r term absorbs part of the error
        assert (np.diff(obj) <= 1e-3 * obj[0]).all() and obj[-1] < obj[0]        # alternation does not make it worse
        # the last quantization is the quantization of W minus the previous step's product
        p4, a4, A4, B4, _ = orc.loftq_init(W, bits, cb, thr, mp, r, steps=4)
        rp, ra = orc.quantize((W.astype(np.float64) - B4 @ A4).astype(np.float32), bits, cb, thr)
        assert np.array_equal(packed, rp) and np.array_equal(absmax, ra)


def test_rank_zero_and_zero_steps_degenerate_cleanly():
    W, bits, cb, thr, mp = layer(6, N=16, K=128)
    packed, absmax, A, B, obj = orc.loftq_init(W, bits, cb, thr, mp, 0, steps=2)
    rp, ra = orc.quantize(W, bits, cb, thr)
    assert np.array_equal(packed, rp) and A.shape == (0, 128) and B.shape == (16, 0)
    assert abs(obj[0] - obj[1]) < 1e-15
