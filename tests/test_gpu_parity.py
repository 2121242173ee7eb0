"""GPU parity: the HIP path through the C ABI against the CPU oracle, on the same seeded inputs.

Codes, packing, absmax and dequantized values must match bit for bit; linear outputs and input
gradients within a max relative error of 2e-2 (bf16 operands and output, fp32 accumulation,
against the fp64 oracle).
"""
import numpy as np
import pytest
import torch

from oracle import lowra_oracle as orc
from paper_2502_08141_amd import lowra, synth
from tests.gpu_util import (REL_TOL, DeviceLayer, bf16_dev, bf16_host_bits, bf16_host_f64, big_entries_rel_err, oracle_state,
                            rel_err, rel_err_unfloored_p999)

pytestmark = pytest.mark.gpu


def layer_cases():
    return {
        "cfg1": lambda: synth.make_config(1),
        "cfg1_per_channel": lambda: synth.make_config(1, per_channel_tables=True),
        "ragged": lambda: synth.make_custom(520, 320, 300, 8, seed=11),
        "one_group": lambda: synth.make_custom(72, 64, 33, 0, seed=12),
        "rank100": lambda: synth.make_custom(264, 448, 70, 100, seed=13, per_channel_tables=True),
        "only4bit": lambda: synth.make_custom(128, 256, 40, 16, fractions=(0.0, 0.0, 1.0), seed=14),
        "only1bit": lambda: synth.make_custom(128, 256, 40, 16, fractions=(1.0, 0.0, 0.0), seed=15),
        # shapes with full 256x256 output tiles and a long contraction: the GEMM kernels' pipelined
        # main loops (mixed-width tiles, widths 1 and 2 alone, odd number of 64-wide groups, K tail)
        "tiles_mixed": lambda: synth.make_custom(512, 1024, 512, 64, fractions=(0.5, 0.25, 0.25), seed=21),
        "tiles_no4": lambda: synth.make_custom(512, 1024, 256, 8, fractions=(0.5, 0.5, 0.0), seed=22),
        "tiles_only1": lambda: synth.make_custom(256, 1152, 256, 0, fractions=(1.0, 0.0, 0.0), seed=23),
        "tiles_only2": lambda: synth.make_custom(256, 1024, 256, 0, fractions=(0.0, 1.0, 0.0), seed=24),
        # wavefronts that hold 4-bit rows next to narrower ones, and 4-bit rows alone: the lookup decode
        "tiles_lut_mix": lambda: synth.make_custom(512, 1024, 300, 16, fractions=(0.3, 0.3, 0.4), seed=28),
        "tiles_only4": lambda: synth.make_custom(256, 1024, 256, 0, fractions=(0.0, 0.0, 1.0), seed=29),
        # the paper's own data model at tile size (one table set per output channel, C = N > 64) with 4-bit
        # rows, several output tiles and a long contraction, for both linear calls
        "tiles_per_channel_lut": lambda: synth.make_custom(512, 1024, 300, 16, fractions=(0.4, 0.3, 0.3), seed=41,
                                                           per_channel_tables=True),
        "tiles_per_channel_no4": lambda: synth.make_custom(512, 1024, 300, 16, fractions=(0.5, 0.5, 0.0), seed=42,
                                                           per_channel_tables=True),
        # per-channel tables with mostly / only 4-bit rows: the forward keeps per-row tables of a tile in LDS as far as
        # they fit (the first wavefronts), the rest of the tile takes the general step; the input gradient stages the
        # tables of every 64-row step
        "tiles_per_channel_mostly4": lambda: synth.make_custom(512, 1024, 300, 16, fractions=(0.1, 0.1, 0.8), seed=48,
                                                               per_channel_tables=True),
        "tiles_per_channel_only4": lambda: synth.make_custom(256, 1024, 260, 8, fractions=(0.0, 0.0, 1.0), seed=49,
                                                             per_channel_tables=True),
        "tiles_oddG": lambda: synth.make_custom(512, 1088, 300, 16, fractions=(0.5, 0.5, 0.0), seed=25),
        # many output channels, K a multiple of 256, no 4-bit rows: the input-gradient kernel's staged
        # code pipeline (1-bit alone; 1-/2-bit mix with a ragged last channel step)
        "chan_only1": lambda: synth.make_custom(640, 512, 300, 8, fractions=(1.0, 0.0, 0.0), seed=26),
        "chan_mixed_ragged": lambda: synth.make_custom(1000, 768, 256, 16, fractions=(0.6, 0.4, 0.0), seed=27),
        # many output channels WITH 4-bit rows: the input gradient's lookup kernel over many full channel steps (the
        # variant without bounds), a ragged last step, and the hand-over to the general steps
        "chan_lut_many": lambda: synth.make_custom(1000, 768, 300, 16, fractions=(0.4, 0.3, 0.3), seed=51),
        "chan_lut_many_only4": lambda: synth.make_custom(1152, 512, 130, 0, fractions=(0.0, 0.0, 1.0), seed=52),
        # many tokens with a ragged end
        "tall_ragged": lambda: synth.make_custom(136, 256, 4130, 24, seed=30),
        # enough token rows that the rank-r side product takes 64 rows per workgroup (several rounds of 16-row ones)
        "tall_rank64": lambda: synth.make_custom(136, 320, 8200, 64, seed=31),
        "tall_longK": lambda: synth.make_custom(136, 1280, 4200, 64, seed=32),     # ten stages through that kernel's ring of four
        # small-token shapes (M <= 16 takes the bandwidth-bound path under PATH_AUTO)
        "tok1": lambda: synth.make_custom(328, 1024, 1, 16, seed=16),
        "tok4_longK": lambda: synth.make_custom(136, 11008, 4, 16, fractions=(0.5, 0.5, 0.0), seed=17),
        "tok16_r0": lambda: synth.make_custom(520, 4096, 16, 0, fractions=(0.5, 0.25, 0.25), seed=18),
        # the streaming small-token kernel: class sizes that need padding rows, three K-chunks with a short last one,
        # rank 24 (B fragment shorter than the MFMA step), one width only, 5 and 13 tokens
        "tok5_pad": lambda: synth.make_custom(1000, 2048, 5, 24, fractions=(0.37, 0.33, 0.3), seed=44),
        "tok13_chunks": lambda: synth.make_custom(264, 9216, 13, 8, fractions=(0.3, 0.3, 0.4), seed=45),
        "tok2_only4": lambda: synth.make_custom(136, 4096, 2, 16, fractions=(0.0, 0.0, 1.0), seed=46),
        "tok3_rank5": lambda: synth.make_custom(264, 2048, 3, 5, fractions=(0.4, 0.3, 0.3), seed=53),       # rows of B of 10 bytes
        "tok16_only1": lambda: synth.make_custom(4112, 4096, 16, 32, fractions=(1.0, 0.0, 0.0), seed=47),
    }


@pytest.fixture(scope="module", params=list(layer_cases()))
def case(request):
    print(f"[case {request.param}]", flush=True)
    L = layer_cases()[request.param]()
    D = DeviceLayer(L)
    D.quantize()
    torch.cuda.synchronize()
    D.ref_packed, D.ref_absmax = oracle_state(L)
    return D


def test_quantize_bit_exact(case):
    assert np.array_equal(case.absmax.cpu().numpy(), case.ref_absmax)
    assert np.array_equal(case.packed.cpu().numpy(), case.ref_packed)


def test_dequantize_bit_exact(case):
    L = case.L
    # decode the ORACLE's state so a quantizer mismatch cannot hide here
    packed = torch.from_numpy(case.ref_packed).cuda(); absmax = torch.from_numpy(case.ref_absmax).cuda()
    got16 = lowra.lowra_dequantize(case.layout, packed, absmax, case.mp)
    got32 = lowra.lowra_dequantize(case.layout, packed, absmax, case.mp, out_dtype=torch.float32)
    torch.cuda.synchronize()
    assert np.array_equal(bf16_host_bits(got16), orc.dequantize(case.ref_packed, case.ref_absmax, L.bits, L.cb, L.mappings, L.K))
    assert np.array_equal(got32.cpu().numpy(), orc.dequantize(case.ref_packed, case.ref_absmax, L.bits, L.cb, L.mappings, L.K, "fp32"))


@pytest.mark.parametrize("path", [lowra.PATH_GEMM, lowra.PATH_AUTO, lowra.PATH_GEMV])
def test_linear_fwd(case, path):
    L = case.L
    if path == lowra.PATH_GEMV and L.M > 16:
        pytest.skip("the streaming small-token kernel is forced only where a small-token kernel runs at all")
    packed = torch.from_numpy(case.ref_packed).cuda(); absmax = torch.from_numpy(case.ref_absmax).cuda()
    lowra.lowra_set_linear_path(path)
    try:
        y = lowra.lowra_linear_fwd(case.layout, packed, absmax, case.mp, case.x, case.A, case.B, L.s)
        torch.cuda.synchronize()
    finally:
        lowra.lowra_set_linear_path(lowra.PATH_AUTO)
    ref = orc.linear_fwd(case.ref_packed, case.ref_absmax, L.bits, L.cb, L.mappings, L.x,
                         L.A if L.r else None, L.B if L.r else None, L.s)
    got = bf16_host_f64(y)
    print(f"fwd path {path}: rel {rel_err(got, ref):.2e}, big entries {big_entries_rel_err(got, ref):.2e}, "
          f"unfloored p99.9 {rel_err_unfloored_p999(got, ref):.2e}", flush=True)
    assert rel_err(got, ref) <= REL_TOL
    assert big_entries_rel_err(got, ref) <= REL_TOL      # plain relative error wherever |ref| >= rms


# every plan the forward GEMM's planner can pick: one tile height for the whole output, or a lower one for the
# columns after the first 256 (a case with a single 256-channel column runs the first height alone)
FWD_TILINGS = [(256, 256, 0), (192, 192, 0), (128, 128, 0), (256, 192, 1), (256, 128, 1), (192, 128, 1)]


def test_linear_fwd_tilings_agree(case):
    """The result of the forward GEMM does not depend on how the output is tiled: every output is the same sum in the
    same order, so each plan must reproduce the planner's own choice bit for bit (which test_linear_fwd holds to the oracle)."""
    L = case.L
    packed = torch.from_numpy(case.ref_packed).cuda(); absmax = torch.from_numpy(case.ref_absmax).cuda()
    lowra.lowra_set_linear_path(lowra.PATH_GEMM)
    try:
        want = lowra.lowra_linear_fwd(case.layout, packed, absmax, case.mp, case.x, case.A, case.B, L.s)
        for plan in FWD_TILINGS:
            lowra.lowra_set_fwd_tiling(*plan)
            got = lowra.lowra_linear_fwd(case.layout, packed, absmax, case.mp, case.x, case.A, case.B, L.s)
            torch.cuda.synchronize()
            assert torch.equal(got.view(torch.int16), want.view(torch.int16)), plan
    finally:
        lowra.lowra_set_fwd_tiling(0, 0, 0)
        lowra.lowra_set_linear_path(lowra.PATH_AUTO)


@pytest.mark.parametrize("path", [lowra.PATH_GEMM, lowra.PATH_AUTO])
def test_linear_bwd_input(case, path):
    L = case.L
    packed = torch.from_numpy(case.ref_packed).cuda(); absmax = torch.from_numpy(case.ref_absmax).cuda()
    lowra.lowra_set_linear_path(path)
    try:
        dX = lowra.lowra_linear_bwd_input(case.layout, packed, absmax, case.mp, case.dY, case.A, case.B, L.s)
        torch.cuda.synchronize()
    finally:
        lowra.lowra_set_linear_path(lowra.PATH_AUTO)
    ref = orc.linear_bwd_input(case.ref_packed, case.ref_absmax, L.bits, L.cb, L.mappings, L.dY,
                               L.A if L.r else None, L.B if L.r else None, L.s, L.K)
    got = bf16_host_f64(dX)
    print(f"bwd path {path}: rel {rel_err(got, ref):.2e}, big entries {big_entries_rel_err(got, ref):.2e}, "
          f"unfloored p99.9 {rel_err_unfloored_p999(got, ref):.2e}", flush=True)
    assert rel_err(got, ref) <= REL_TOL
    assert big_entries_rel_err(got, ref) <= REL_TOL


# The small-token path applies the group scale to the group's fp32 dot product of unscaled bf16 levels;
# the GEMM path multiplies bf16(level * absmax), App. A.2's decode.  Same layer, two effective weight
# roundings: the two outputs may differ by the weight rounding (2^-9 relative per weight, averaging out
# over the contraction) plus the bf16 output rounding (2^-8 relative), never by more.
PATH_AGREE_TOL = 1e-2
# The streaming input gradient multiplies bf16(dY * absmax) by the unscaled bf16 level: two roundings per product (2^-9
# relative each) against the GEMM path's one, and a product's relative error does not average out over a sum of terms
# of random sign.  Measured: 1.0e-2 against the fp64 oracle and 1.5e-2 against the GEMM path, worst of 65536 outputs
# (the GEMM path: 0.4e-2 against the oracle).  The bound is the parity tolerance itself.
PATH_AGREE_TOL_BWD = REL_TOL


@pytest.mark.parametrize("M", [1, 4, 16])
def test_small_token_and_gemm_paths_agree(M):
    L = synth.make_custom(520, 4096, M, 16, fractions=(0.5, 0.25, 0.25), seed=43)
    D = DeviceLayer(L); D.quantize()
    out = {}
    for path in (lowra.PATH_GEMV, lowra.PATH_GEMV_GENERAL, lowra.PATH_GEMM):
        lowra.lowra_set_linear_path(path)
        try:
            out[path] = (bf16_host_f64(lowra.lowra_linear_fwd(D.layout, D.packed, D.absmax, D.mp, D.x, D.A, D.B, L.s)),
                         bf16_host_f64(lowra.lowra_linear_bwd_input(D.layout, D.packed, D.absmax, D.mp, D.dY, D.A, D.B, L.s)))
        finally:
            lowra.lowra_set_linear_path(lowra.PATH_AUTO)
    for path in (lowra.PATH_GEMV, lowra.PATH_GEMV_GENERAL):     # the streaming and the general small-token kernel
        for which in (0, 1):
            assert rel_err(out[path][which], out[lowra.PATH_GEMM][which]) <= (PATH_AGREE_TOL, PATH_AGREE_TOL_BWD)[which]


def test_adjoint_identity_on_gpu(case):
    """<dY, fwd(x)> == <bwd(dY), x> ties the two kernels to each other (both linear in their input)."""
    L = case.L
    y = bf16_host_f64(lowra.lowra_linear_fwd(case.layout, case.packed, case.absmax, case.mp, case.x, case.A, case.B, L.s))
    dX = bf16_host_f64(lowra.lowra_linear_bwd_input(case.layout, case.packed, case.absmax, case.mp, case.dY, case.A, case.B, L.s))
    lhs = float((synth.bf16_bits_to_f64(L.dY) * y).sum()); rhs = float((dX * synth.bf16_bits_to_f64(L.x)).sum())
    scale = np.sqrt(float((y * y).sum()) * float((synth.bf16_bits_to_f64(L.dY) ** 2).sum()))
    assert abs(lhs - rhs) <= 1e-2 * scale


def test_edge_cases_and_errors():
    thr, mp, cb_bits = synth.shared_codebooks()
    dthr, dmp = torch.from_numpy(thr).cuda(), torch.from_numpy(mp).cuda()
    # empty matrix
    lay0 = lowra.Layout(64, np.zeros(0, np.uint8), np.zeros(0, np.int32), cb_bits)
    assert lay0.packed_bytes == 0
    p, a = lowra.lowra_quantize(lay0, torch.empty((0, 64), device="cuda"), dthr)
    assert p.numel() == 0 and a.numel() == 0
    # zero tokens
    L = synth.make_custom(64, 128, 4, 4, seed=20)
    D = DeviceLayer(L); D.quantize()
    y = lowra.lowra_linear_fwd(D.layout, D.packed, D.absmax, D.mp, D.x[:0].contiguous(), D.A, D.B, 2.0)
    assert tuple(y.shape) == (0, 64)
    # all-zero weights: absmax 0, finite decode
    Dz = DeviceLayer(L); Dz.W.zero_(); Dz.quantize()
    out = lowra.lowra_dequantize(Dz.layout, Dz.packed, Dz.absmax, Dz.mp, out_dtype=torch.float32)
    torch.cuda.synchronize()
    assert float(Dz.absmax.abs().max()) == 0 and bool(torch.isfinite(out).all()) and float(out.abs().max()) == 0
    # error statuses
    with pytest.raises(lowra.LowraError) as e:
        lowra.Layout(100, L.bits, L.cb, L.cb_bits)                      # K % 64 != 0
    assert e.value.status == lowra.UNSUPPORTED
    with pytest.raises(lowra.LowraError) as e:
        lowra.Layout(128, np.full(8, 3, np.uint8), np.zeros(8, np.int32), cb_bits)   # 3-bit
    assert e.value.status == lowra.UNSUPPORTED
    with pytest.raises(lowra.LowraError) as e:
        lowra.Layout(128, np.full(8, 2, np.uint8), np.zeros(8, np.int32), cb_bits)   # table built for 1 bit
    assert e.value.status == lowra.INVALID_ARG
    with pytest.raises(lowra.LowraError) as e:                           # workspace too small
        lowra.lowra_linear_fwd(D.layout, D.packed, D.absmax, D.mp, D.x, D.A, D.B, 2.0,
                               workspace=torch.empty(16, dtype=torch.uint8, device="cuda"))
    assert e.value.status == lowra.WORKSPACE_TOO_SMALL
    with pytest.raises(lowra.LowraError) as e:                           # misaligned weight pointer
        Wm = torch.empty(L.N * L.K + 1, device="cuda")[1:].view(L.N, L.K)
        lowra.lowra_quantize(D.layout, Wm, D.thr)
    assert e.value.status == lowra.MISALIGNED


def test_runs_are_deterministic():
    D = DeviceLayer(synth.make_custom(264, 320, 130, 8, seed=21)); D.quantize()
    y1 = lowra.lowra_linear_fwd(D.layout, D.packed, D.absmax, D.mp, D.x, D.A, D.B, 2.0)
    y2 = lowra.lowra_linear_fwd(D.layout, D.packed, D.absmax, D.mp, D.x, D.A, D.B, 2.0)
    p2, a2 = lowra.lowra_quantize(D.layout, D.W, D.thr)
    torch.cuda.synchronize()
    assert torch.equal(y1, y2) and torch.equal(p2, D.packed) and torch.equal(a2, D.absmax)


def test_shared_thresholds_with_per_adapter_mappings():
    """Sec. 4.1, production variant: one quantized base (one set of thresholds), a decoding table per
    adapter.  The packed state is produced once; dequantize and the linear calls take each adapter's
    mappings as plain data and must match the oracle for each."""
    L = synth.make_custom(264, 512, 40, 16, seed=31)
    D = DeviceLayer(L)
    packed, absmax = D.quantize()
    torch.cuda.synchronize()
    rp, ra = oracle_state(L)
    assert np.array_equal(packed.cpu().numpy(), rp) and np.array_equal(absmax.cpu().numpy(), ra)
    rng = np.random.default_rng(5)
    for adapter in range(3):
        # the adapter's own levels: the shared ones nudged, still increasing within the used part of each row
        mp = L.mappings.copy()
        for c, b in enumerate(L.cb_bits):
            k = 1 << int(b)
            gap = np.diff(mp[c, :k]).min()
            mp[c, :k] += rng.uniform(-0.4, 0.4, k).astype(np.float32) * gap
        mp_d = torch.from_numpy(mp).cuda()
        got = lowra.lowra_dequantize(D.layout, packed, absmax, mp_d)
        y = lowra.lowra_linear_fwd(D.layout, packed, absmax, mp_d, D.x, D.A, D.B, L.s)
        dX = lowra.lowra_linear_bwd_input(D.layout, packed, absmax, mp_d, D.dY, D.A, D.B, L.s)
        torch.cuda.synchronize()
        assert np.array_equal(bf16_host_bits(got), orc.dequantize(rp, ra, L.bits, L.cb, mp, L.K))
        assert rel_err(bf16_host_f64(y), orc.linear_fwd(rp, ra, L.bits, L.cb, mp, L.x, L.A, L.B, L.s)) <= REL_TOL
        assert rel_err(bf16_host_f64(dX), orc.linear_bwd_input(rp, ra, L.bits, L.cb, mp, L.dY, L.A, L.B, L.s, L.K)) <= REL_TOL
