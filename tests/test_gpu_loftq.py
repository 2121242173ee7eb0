"""GPU checks of the alternating low-rank initialiser (lowra_loftq_init) against the oracle.

The oracle takes the rank-r fit from an exact SVD (the paper's definition); the library approximates
it by block power iteration on bf16 copies of the residual, so factors are not compared element by
element.  What is unique is compared exactly, the rest by properties with stated bounds:
  * one step: the quantized state is the oracle's quantization of W, bit for bit;
  * A has orthonormal rows (to the bf16 rounding of its entries, 4e-3) and B = E A^T for E = W - What of the
    returned state (2e-2 rule): B A is
    the projection of E onto a rank-r row space, whatever the subspace;
  * the objective |W - What - B A|_F of the returned state is within 2 % of the exact-SVD oracle's
    after five steps (two rounds per step) and below plain quantization;
  * the returned state is the quantization of W minus the previous step's product (run again with
    one step less), up to the rare code that the fp32 rounding of that residual moves across a
    threshold.
Tables come from the oracle's learner, as in the paper's pipeline (with the quantile tables' 1-bit
levels the alternation diverges, on the oracle as well).
"""
import numpy as np
import pytest
import torch

from oracle import lowra_oracle as orc
from paper_2502_08141_amd import lowra, synth
from tests.gpu_util import REL_TOL, bf16_dev, bf16_host_f64, rel_err

pytestmark = pytest.mark.gpu


# bounds of the flat-spectrum cases at the binding's default of 16 rounds per step: after five steps the library's fit
# must capture at least this fraction of the energy the exact rank-r fit of the same residual captures and end within
# 1e-3 of the exact-SVD alternation's objective (App. D takes the fit from an SVD); the first, cold-started step alone
# within 1.5e-3.  Observed after five steps: 1.0022 / 1.0033 with 4 rounds, 1.0013 / 1.0021 with 8, 1.0008 / 1.0005
# with 16, 0.9998 / 0.9994 with 32 (ranks 16 / 64); after one step 1.0009 / 1.0011 with 16 rounds, and with 2 rounds
# that step captures only 83 - 88 % of the best rank-r energy of a flat spectrum.
LOFTQ_ENERGY_FRACTION = 0.995
LOFTQ_OBJECTIVE_FACTOR = 1.001
LOFTQ_FIRST_STEP_FACTOR = 1.0015


def make(seed, N, K, fr, lowrank=True):
    rng = np.random.default_rng([synth.SEED, 404, seed])
    W = rng.normal(0, 0.02, (N, K))
    if lowrank:
        W = W + 0.02 * rng.normal(0, 1, (N, 6)) @ rng.normal(0, 1, (6, K)) / np.sqrt(6)
    W = W.astype(np.float32)
    bits = synth.assign_bits(N, fr, np.random.default_rng([synth.SEED, 405, seed]))
    thr0, mp0, cbb = synth.shared_codebooks()
    thr, mp, _, _ = orc.learn_tables(W, bits, np.searchsorted(cbb, bits).astype(np.int32), thr0, mp0, 2)
    return W, bits, np.arange(N, dtype=np.int32), bits.copy(), thr, mp


# A is the bf16 rounding of a matrix with orthonormal rows (fp32 substitution against an fp64 factor): entry (i, j) of
# A A^T - I is sum_k a_ik a_jk (d_ik + d_jk + d_ik d_jk) with |d| <= 2^-9, at most 2 x 2^-9 (1 + 2^-10) by Cauchy-Schwarz
# on unit rows; observed 4e-4 to 8e-4
ORTHONORMAL_TOL = 4e-3

NEAR_THRESHOLD = 8e-6   # in units of the normalised weight u in [-1, 1]: ~64 fp32 ulp at 1


def assert_state_is_quantization_of(packed, absmax, F64, bits, cb, thr):
    """The returned state must be the quantization of F = W - B A.  The library forms F in fp32 with
    another summation order than this fp64 reference (rank-r product accumulated in fp32), so F may
    differ by a few fp32 ulp of the product, which can move a weight across a threshold it almost
    touches.  Every code that differs from the oracle's must therefore belong to a weight whose
    normalised value lies within NEAR_THRESHOLD of one of its channel's thresholds, and differ by one
    bin; every group scale must agree to fp32 rounding of F."""
    N, K = F64.shape
    rp, ra = orc.quantize(F64.astype(np.float32), bits, cb, thr)
    assert np.allclose(absmax, ra, rtol=1e-6, atol=0)
    got, want = orc.unpack(packed, bits, K), orc.unpack(rp, bits, K)
    nn, kk = np.nonzero(got != want)
    print(f"    codes differing from the oracle's quantization of W - B A: {nn.size} of {N * K}", flush=True)
    assert nn.size <= 2e-3 * N * K
    if nn.size == 0:
        return
    assert np.all(np.abs(got[nn, kk].astype(np.int64) - want[nn, kk].astype(np.int64)) == 1)
    a = ra.astype(np.float64)[nn, kk // 64]
    u = F64[nn, kk] / a
    nthr = (1 << bits[nn].astype(np.int64)) - 1
    T = thr.astype(np.float64)[cb[nn]]                                     # [cases, 16]
    valid = np.arange(T.shape[1])[None, :] < nthr[:, None]
    dist = np.where(valid, np.abs(T - u[:, None]), np.inf).min(axis=1)
    assert dist.max() <= NEAR_THRESHOLD, (dist.max(), int(dist.argmax()))


CASES = {
    "mixed_r16": (1, 512, 512, (0.4, 0.3, 0.3), 16),
    "no4_r64": (2, 1024, 512, (0.5, 0.5, 0.0), 64),
    "ragged_r5": (3, 520, 320, (0.4, 0.3, 0.3), 5),
    "wide_r32": (4, 264, 1088, (0.3, 0.3, 0.4), 32),
}


def gpu_run(W, bits, cb, cbb, thr, mp, r, omega, steps, iters=2):
    lay = lowra.Layout(W.shape[1], bits, cb, cbb)
    out = lowra.lowra_loftq_init(lay, torch.from_numpy(W).cuda(), torch.from_numpy(thr).cuda(), torch.from_numpy(mp).cuda(), r,
                                 bf16_dev(omega), steps=steps, power_iterations=iters)
    torch.cuda.synchronize()
    packed, absmax, A, B = out
    return packed.cpu().numpy(), absmax.cpu().numpy(), bf16_host_f64(A), bf16_host_f64(B)


@pytest.mark.parametrize("name", list(CASES))
def test_loftq_init(name):
    print(f"[loftq {name}]", flush=True)
    seed, N, K, fr, r = CASES[name]
    W, bits, cb, cbb, thr, mp = make(seed, N, K, fr)
    W64 = W.astype(np.float64)
    omega = synth.to_bf16_bits(np.random.default_rng([synth.SEED, 406, seed]).normal(0, 1, (r, K)))

    # one step: quantization of W itself
    p1, a1, A1, B1 = gpu_run(W, bits, cb, cbb, thr, mp, r, omega, 1)
    rp, ra = orc.quantize(W, bits, cb, thr)
    assert np.array_equal(p1, rp) and np.array_equal(a1, ra)
    plain = np.linalg.norm(W64 - orc.dequantize(rp, ra, bits, cb, mp, K, "fp32"))

    p4, a4, A4, B4 = gpu_run(W, bits, cb, cbb, thr, mp, r, omega, 4)
    p5, a5, A5, B5 = gpu_run(W, bits, cb, cbb, thr, mp, r, omega, 5)
    # the factors: orthonormal rows, B = E A^T
    E = W64 - orc.dequantize(p5, a5, bits, cb, mp, K, "fp32")
    print(f"    |A A^T - I| max {np.abs(A5 @ A5.T - np.eye(r)).max():.2e}", flush=True)
    assert np.abs(A5 @ A5.T - np.eye(r)).max() <= ORTHONORMAL_TOL
    assert rel_err(B5, E @ A5.T) <= REL_TOL
    # the objective against the exact-SVD alternation
    *_, ref = orc.loftq_init(W, bits, cb, thr, mp, r, steps=5)
    obj5 = np.linalg.norm(E - B5 @ A5)
    obj1 = np.linalg.norm(W64 - orc.dequantize(p1, a1, bits, cb, mp, K, "fp32") - B1 @ A1)
    print(f"    plain {plain:.4f}  step 1 {obj1:.4f} (oracle {ref[0]:.4f})  step 5 {obj5:.4f} (oracle {ref[-1]:.4f})", flush=True)
    assert obj5 <= 1.02 * ref[-1]
    assert obj1 <= 1.06 * ref[0]
    assert obj5 < obj1 < plain
    # step 5 quantized W - B4 A4
    assert_state_is_quantization_of(p5, a5, W64 - B4 @ A4, bits, cb, thr)


FLAT_CASES = {
    # no planted low-rank part: the residual of quantization is noise-like, its spectrum flat, so the
    # top-r subspace is poorly separated -- the hard case for a power iteration
    "flat_r16": (11, 512, 512, (0.4, 0.3, 0.3), 16),
    "flat_r64": (12, 768, 512, (0.5, 0.5, 0.0), 64),
}


@pytest.mark.parametrize("name", list(FLAT_CASES))
def test_loftq_flat_spectrum(name):
    """Captured energy |B A|_F^2 and objective against the exact-SVD alternation on weights without a
    planted low-rank component (App. D takes the fit from an SVD)."""
    print(f"[loftq {name}]", flush=True)
    seed, N, K, fr, r = FLAT_CASES[name]
    W, bits, cb, cbb, thr, mp = make(seed, N, K, fr, lowrank=False)
    W64 = W.astype(np.float64)
    omega = synth.to_bf16_bits(np.random.default_rng([synth.SEED, 406, seed]).normal(0, 1, (r, K)))
    *_, ref = orc.loftq_init(W, bits, cb, thr, mp, r, steps=5)
    for steps in (1, 5):
        for iters in (2, 4, 8, 16):                                # the last one (the binding's default) is asserted
            p5, a5, A5, B5 = gpu_run(W, bits, cb, cbb, thr, mp, r, omega, steps, iters=iters)
            E = W64 - orc.dequantize(p5, a5, bits, cb, mp, K, "fp32")
            obj5 = np.linalg.norm(E - B5 @ A5)
            captured = np.linalg.norm(B5 @ A5) ** 2
            sv = np.linalg.svd(E, compute_uv=False)
            best = float((sv[:r] ** 2).sum())                     # Eckart-Young: the most any rank-r fit of this E captures
            print(f"    steps {steps} rounds {iters}: objective {obj5:.5f} (oracle {ref[steps - 1]:.5f}); captured energy {captured:.6f} of at most {best:.6f} "
                  f"({captured / best:.4f})", flush=True)
        if steps == 1:
            assert obj5 <= LOFTQ_FIRST_STEP_FACTOR * ref[0]
    assert captured >= LOFTQ_ENERGY_FRACTION * best
    assert obj5 <= LOFTQ_OBJECTIVE_FACTOR * ref[-1]


def test_loftq_rank_zero_and_errors():
    W, bits, cb, cbb, thr, mp = make(5, 64, 128, (0.4, 0.3, 0.3))
    lay = lowra.Layout(128, bits, cb, cbb)
    Wd, thr_d, mp_d = torch.from_numpy(W).cuda(), torch.from_numpy(thr).cuda(), torch.from_numpy(mp).cuda()
    packed, absmax, A, B = lowra.lowra_loftq_init(lay, Wd, thr_d, mp_d, 0, None, steps=3)
    torch.cuda.synchronize()
    rp, ra = orc.quantize(W, bits, cb, thr)
    assert np.array_equal(packed.cpu().numpy(), rp) and np.array_equal(absmax.cpu().numpy(), ra)
    assert A.shape == (0, 128) and B.shape == (64, 0)
    om = bf16_dev(synth.to_bf16_bits(np.random.default_rng(1).normal(0, 1, (8, 128))))
    with pytest.raises(lowra.LowraError, match="invalid argument"):
        lowra.lowra_loftq_init(lay, Wd, thr_d, mp_d, 8, om, steps=0)
    with pytest.raises(lowra.LowraError, match="workspace too small"):
        lowra.lowra_loftq_init(lay, Wd, thr_d, mp_d, 8, om, workspace=torch.empty(64, dtype=torch.uint8, device="cuda"))
    om100 = bf16_dev(synth.to_bf16_bits(np.random.default_rng(1).normal(0, 1, (100, 128))))
    with pytest.raises(lowra.LowraError, match="unsupported"):
        lowra.lowra_loftq_init(lay, Wd, thr_d, mp_d, 100, om100)


def test_loftq_zero_weights_stay_finite():
    """W = 0: nothing to fit; the vanishing pivots drop every row of A instead of dividing by zero."""
    W, bits, cb, cbb, thr, mp = make(6, 64, 128, (0.4, 0.3, 0.3))
    lay = lowra.Layout(128, bits, cb, cbb)
    om = bf16_dev(synth.to_bf16_bits(np.random.default_rng(2).normal(0, 1, (8, 128))))
    packed, absmax, A, B = lowra.lowra_loftq_init(lay, torch.zeros((64, 128), device="cuda"), torch.from_numpy(thr).cuda(),
                                                  torch.from_numpy(mp).cuda(), 8, om, steps=2)
    torch.cuda.synchronize()
    assert not absmax.any() and not A.float().abs().max() > 0 and not B.float().abs().max() > 0


def test_loftq_dependent_start_drops_a_row():
    """Two equal rows in the start: the second one's pivot vanishes in the factorisation of the Gram matrix, its row of
    A (and column of B) comes out zero in every round, and the other rows are still an orthonormal basis whose fit
    lowers the objective: a rank r - 1 fit, never a division by zero."""
    seed, N, K, fr, r = 7, 512, 512, (0.4, 0.3, 0.3), 16
    W, bits, cb, cbb, thr, mp = make(seed, N, K, fr)
    W64 = W.astype(np.float64)
    om = np.random.default_rng([synth.SEED, 406, seed]).normal(0, 1, (r, K))
    om[3] = om[2]
    p, a, A, B = gpu_run(W, bits, cb, cbb, thr, mp, r, synth.to_bf16_bits(om), 2, iters=4)
    assert np.isfinite(A).all() and np.isfinite(B).all()
    assert not A[3].any() and not B[:, 3].any()
    keep = [i for i in range(r) if i != 3]
    assert np.abs(A[keep] @ A[keep].T - np.eye(r - 1)).max() <= ORTHONORMAL_TOL
    E = W64 - orc.dequantize(p, a, bits, cb, mp, K, "fp32")
    assert rel_err(B[:, keep], E @ A[keep].T) <= REL_TOL
    rp, ra = orc.quantize(W, bits, cb, thr)
    plain = np.linalg.norm(W64 - orc.dequantize(rp, ra, bits, cb, mp, K, "fp32"))
    assert np.linalg.norm(E - B @ A) < plain


def test_loftq_full_size_objective():
    """Config 3 at full size with tables from the library's learner: the objective, computed on the
    device from the library's own fp32 decode, falls from plain quantization to step 1 to step 5."""
    print("[loftq cfg3] generating", flush=True)
    L = synth.make_config(3)
    lay0 = lowra.Layout(L.K, L.bits, L.cb, L.cb_bits)
    W = torch.from_numpy(L.W).cuda()
    thr, mp, _ = lowra.lowra_learn_tables(lay0, W, torch.from_numpy(L.thresholds).cuda(), torch.from_numpy(L.mappings).cuda(), 2)
    lay = lowra.Layout(L.K, L.bits, np.arange(L.N, dtype=np.int32), L.bits.copy())
    gen = torch.Generator(device="cuda").manual_seed(99)
    omega = torch.randn((64, L.K), generator=gen, device="cuda").bfloat16()

    def objective(packed, absmax, A, B):
        What = lowra.lowra_dequantize(lay, packed, absmax, mp, out_dtype=torch.float32)
        R = W - What
        if A is not None:
            R -= B.float() @ A.float()
        return float(torch.linalg.norm(R.double()))

    packed, absmax = lowra.lowra_quantize(lay, W, thr)
    plain = objective(packed, absmax, None, None)
    objs = []
    for steps in (1, 5):
        print(f"[loftq cfg3] {steps} step(s)", flush=True)
        packed, absmax, A, B = lowra.lowra_loftq_init(lay, W, thr, mp, 64, omega, steps=steps)
        torch.cuda.synchronize()
        objs.append(objective(packed, absmax, A, B))
        G = A.float() @ A.float().T
        assert float((G - torch.eye(64, device="cuda")).abs().max()) <= ORTHONORMAL_TOL
    print(f"    plain {plain:.3f}  step 1 {objs[0]:.3f}  step 5 {objs[1]:.3f}", flush=True)
    assert objs[1] < objs[0] < plain
