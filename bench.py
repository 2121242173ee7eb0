#!/usr/bin/env python3
"""Benchmark of the LowRA hot path on one MI355X.

A step is one pass of the whole path over config 3 (W 11008x4096 at 1.5 bits/param, 4096 tokens,
LoRA rank 64): quantize -> dequantize -> fused dequant-GEMM forward -> fused input gradient, all
through the C ABI, inputs resident in HBM.  Prints one JSON line.

  value      TFLOP/s of the step: base GEMM flops of forward + input gradient (2 * 2MNK) over the
             whole step time (quantize and dequantize included)
  roofline   the forward fused dequant-GEMM kernel alone, timed with HIP events recorded around its
             launch (lowra_set_kernel_timer), against the bf16 dense MFMA peak
  passes     per-pass times (ms: events around the call inside the step; kernel_ms: events around the
             kernel launch; stream_ms: per launch over 20 back-to-back launches rotating over 4
             buffer sets) and rates; the quantize and dequantize GB/s use stream_ms, against the HBM peak
  cpu_baseline  the CPU oracle on a bounded sample of the same workload
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
LOFTQ_ROUNDS = 16                                      # power-iteration rounds per step of the low-rank initialiser (the binding's default)
LOFTQ_BYTES_PER_WEIGHT = 82.0 + 10.0 * (2 * LOFTQ_ROUNDS + 1)   # 4 residuals W - B A 8 B, 5 quantize 4 B, 5 decode-and-subtract 6 B, 5 (2 rounds + 1) products with E or E^T 2 B
MFMA_BF16_PEAK_TFLOPS = 2500.0


def profiled_traffic_bytes(config: int):
    """HBM bytes per launch of the forward kernel from the committed rocprofv3 --pmc summary of this command
    (profiles/bench_config<N>_hbm_traffic.md, line `traffic_bytes_per_launch: <number>`); None when there is
    no such summary.  The counters need their own profiler runs, so the figure is read, not measured here."""
    path = os.path.join(ROOT, "profiles", f"bench_config{config}_hbm_traffic.md")
    try:
        with open(path) as f:
            for line in f:
                if line.strip().startswith("traffic_bytes_per_launch:"):
                    return float(line.split(":", 1)[1].split()[0])
    except OSError:
        pass
    return None


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--config", type=int, default=3, choices=[1, 2, 3, 4])
    ap.add_argument("--workload", choices=["train", "gemv"], default="train",
                    help="train: the step described above (the headline line); gemv: config 5, the small-token "
                         "forward streamed over the whole 32-layer weight set")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run a plain 256 MiB device copy: the known-size kernel that calibrates the "
                         "FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run of this command")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-gemv", action="store_true", help="skip the config-5 small-token leg of the default run")
    ap.add_argument("--no-other-configs", action="store_true", help="skip the kernel times of configs 2 and 4")
    ap.add_argument("--no-graph", action="store_true", help="gemv workload: skip the HIP-graph replays of the stream")
    ap.add_argument("--no-library-gemm", action="store_true", help="skip the library bf16 GEMM of the same shape (context figure)")
    ap.add_argument("--cpu-sample-rows", type=int, default=4096,
                    help="token rows of the forward and input gradient that the CPU oracle runs (the default, all of config 3, "
                         "is about 17 s on 16 cores)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        return 2

    import numpy as np
    import torch

    from paper_2502_08141_amd import lowra, synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)
    lowra.lib()
    if args.workload == "gemv":
        return gemv_stream(args, np, torch, lowra, synth)

    L = synth.make_config(args.config)
    N, K, M, r = L.N, L.K, L.M, L.r

    def dev16(a):
        return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).view(torch.bfloat16).cuda()

    lay = lowra.Layout(K, L.bits, L.cb, L.cb_bits)
    thr, mp = torch.from_numpy(L.thresholds).cuda(), torch.from_numpy(L.mappings).cuda()
    W = torch.from_numpy(L.W).cuda()
    x, dY, A, B = dev16(L.x), dev16(L.dY), dev16(L.A), dev16(L.B)
    packed = torch.empty(lay.packed_bytes, dtype=torch.uint8, device="cuda")
    absmax = torch.empty((N, K // 64), dtype=torch.float32, device="cuda")
    What = torch.empty((N, K), dtype=torch.bfloat16, device="cuda")
    y = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    dX = torch.empty((M, K), dtype=torch.bfloat16, device="cuda")
    ws = torch.empty(max(lay.workspace_bytes(lowra.OP_LINEAR_FWD, M, r),
                         lay.workspace_bytes(lowra.OP_LINEAR_BWD_INPUT, M, r), 16), dtype=torch.uint8, device="cuda")

    names = ["quantize", "dequantize", "linear_fwd", "linear_bwd_input"]

    def ev():
        e = torch.cuda.Event(enable_timing=True)
        e.record()          # creates the underlying hipEvent so its handle can be handed to the library
        return e

    def one_step(marks=None, kern=None):
        """One pass of the hot path.  With marks / kern: HIP events between the passes and around each
        pass's dominant kernel (the instrumented run); without: the four calls and nothing else."""
        if marks is None:
            lowra.lowra_quantize(lay, W, thr, packed, absmax)
            lowra.lowra_dequantize(lay, packed, absmax, mp, out=What)
            lowra.lowra_linear_fwd(lay, packed, absmax, mp, x, A, B, L.s, y=y, workspace=ws)
            lowra.lowra_linear_bwd_input(lay, packed, absmax, mp, dY, A, B, L.s, dX=dX, workspace=ws)
            return
        marks[0].record()
        lowra.lowra_set_kernel_timer(kern[4].cuda_event, kern[5].cuda_event)
        lowra.lowra_quantize(lay, W, thr, packed, absmax)
        marks[1].record()
        lowra.lowra_set_kernel_timer(kern[6].cuda_event, kern[7].cuda_event)
        lowra.lowra_dequantize(lay, packed, absmax, mp, out=What)
        marks[2].record()
        lowra.lowra_set_kernel_timer(kern[0].cuda_event, kern[1].cuda_event)
        lowra.lowra_linear_fwd(lay, packed, absmax, mp, x, A, B, L.s, y=y, workspace=ws)
        marks[3].record()
        lowra.lowra_set_kernel_timer(kern[2].cuda_event, kern[3].cuda_event)
        lowra.lowra_linear_bwd_input(lay, packed, absmax, mp, dY, A, B, L.s, dX=dX, workspace=ws)
        marks[4].record()
        lowra.lowra_set_kernel_timer(None, None)

    # The timed region is the K steps alone; the per-pass and per-kernel breakdown comes from an
    # instrumented run of up to 200 more steps right after it (13 event records per step cost time).
    n_inst = min(args.steps, 200)
    marks = [[ev() for _ in range(5)] for _ in range(n_inst)]
    kerns = [[ev() for _ in range(8)] for _ in range(n_inst)]
    torch.cuda.synchronize()
    for _ in range(args.warmup):
        one_step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        one_step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for i in range(n_inst):
        one_step(marks[i], kerns[i])
    torch.cuda.synchronize()

    # Bandwidth passes by the streaming protocol: events around 20 back-to-back launches that rotate
    # over 4 distinct buffer sets (footprint beyond the 256 MB memory-side cache), median of 5 repeats.
    def stream_ms(calls, n=20, reps=5):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        for c in calls:
            c()
        torch.cuda.synchronize()
        ts = []
        for _ in range(reps):
            e0.record()
            for i in range(n):
                calls[i % len(calls)]()
            e1.record()
            torch.cuda.synchronize()
            ts.append(e0.elapsed_time(e1) / n)
        return float(np.median(ts))

    Ws = [W] + [W.clone() for _ in range(3)]
    states = [(packed, absmax)] + [(torch.empty_like(packed), torch.empty_like(absmax)) for _ in range(3)]
    outs = [What] + [torch.empty_like(What) for _ in range(3)]
    q_stream_ms = stream_ms([lambda i=i: lowra.lowra_quantize(lay, Ws[i], thr, states[i][0], states[i][1]) for i in range(4)])
    deq_stream_ms = stream_ms([lambda i=i: lowra.lowra_dequantize(lay, states[i][0], states[i][1], mp, out=outs[i]) for i in range(4)])
    # beyond the step: the mapping/threshold learner on the same matrix (2 rounds), same streaming protocol
    learn_stream_ms = stream_ms([lambda i=i: lowra.lowra_learn_tables(lay, Ws[i], thr, mp, 2) for i in range(4)], n=8, reps=3)
    mse_stream_ms = stream_ms([lambda i=i: lowra.lowra_channel_mse(Ws[i], thr, mp) for i in range(4)], n=8, reps=3)
    del Ws, outs
    # beyond the step: adapter gradients dA, dB of the same layer (x and dY rotate over 4 copies)
    xs, dYs = [x] + [x.clone() for _ in range(3)], [dY] + [dY.clone() for _ in range(3)]
    ws_g = torch.empty(max(lay.workspace_bytes(lowra.OP_ADAPTER_GRADS, M, r), 16), dtype=torch.uint8, device="cuda")
    grads_stream_ms = stream_ms([lambda i=i: lowra.lowra_adapter_grads(lay, xs[i], dYs[i], A, B, L.s, workspace=ws_g) for i in range(4)],
                                n=8, reps=3) if r and r <= 64 else None
    gk = [[ev(), ev()] for _ in range(8)]
    if grads_stream_ms is not None:
        for i in range(8):
            lowra.lowra_set_kernel_timer(gk[i][0].cuda_event, gk[i][1].cuda_event)
            lowra.lowra_adapter_grads(lay, xs[i % 4], dYs[i % 4], A, B, L.s, workspace=ws_g)
        lowra.lowra_set_kernel_timer(None, None)
        torch.cuda.synchronize()
        grads_db_kernel_ms = float(np.median([a.elapsed_time(b) for a, b in gk]))
    # the same gradients from the rank-r intermediates that the step's two linear calls leave in their workspaces
    # (x and dY read once): one forward and one input-gradient call per copy fill them, untimed
    grads_side_ms = None
    if grads_stream_ms is not None:
        sides = []
        for i in range(4):
            wf = torch.empty(max(lay.workspace_bytes(lowra.OP_LINEAR_FWD, M, r), 16), dtype=torch.uint8, device="cuda")
            wb = torch.empty(max(lay.workspace_bytes(lowra.OP_LINEAR_BWD_INPUT, M, r), 16), dtype=torch.uint8, device="cuda")
            lowra.lowra_linear_fwd(lay, packed, absmax, mp, xs[i], A, B, L.s, y=y, workspace=wf)
            lowra.lowra_linear_bwd_input(lay, packed, absmax, mp, dYs[i], A, B, L.s, dX=dX, workspace=wb)
            sides.append((lowra.lowra_linear_side_product(lay, lowra.OP_LINEAR_FWD, M, r, wf),
                          lowra.lowra_linear_side_product(lay, lowra.OP_LINEAR_BWD_INPUT, M, r, wb)))
        if all(a is not None and b is not None for a, b in sides):
            grads_side_ms = stream_ms([lambda i=i: lowra.lowra_adapter_grads_from_side(lay, xs[i], dYs[i], r, sides[i][0], sides[i][1],
                                                                                        workspace=ws_g) for i in range(4)], n=8, reps=3)
        del sides
    del xs, dYs
    # beyond the step: alternating low-rank initialisation (5 steps, 2 power rounds each) of the same matrix
    loftq_ms = None
    if r and r <= 64:
        ws_l = torch.empty(max(lay.workspace_bytes(lowra.OP_LOFTQ_INIT, 0, r), 16), dtype=torch.uint8, device="cuda")
        omega = torch.randn((r, K), device="cuda", generator=torch.Generator(device="cuda").manual_seed(synth.SEED)).bfloat16()
        lq0, lq1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        ts = []
        for _ in range(4):
            lq0.record()
            lowra.lowra_loftq_init(lay, W, thr, mp, r, omega, steps=5, power_iterations=LOFTQ_ROUNDS, workspace=ws_l)
            lq1.record(); torch.cuda.synchronize()
            ts.append(lq0.elapsed_time(lq1))
        loftq_ms = float(np.median(ts[1:]))
        del ws_l

    ceil = measure_ceilings(np, torch, lowra)

    if args.copy_probe:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(2):
            dst.copy_(src)
        torch.cuda.synchronize()

    ms_per_step = (t1 - t0) * 1e3 / args.steps
    pass_ms = {n: float(np.mean([marks[i][j].elapsed_time(marks[i][j + 1]) for i in range(n_inst)]))
               for j, n in enumerate(names)}
    fwd_kernel_ms = float(np.mean([k[0].elapsed_time(k[1]) for k in kerns]))
    bwd_kernel_ms = float(np.mean([k[2].elapsed_time(k[3]) for k in kerns]))
    q_kernel_ms = float(np.mean([k[4].elapsed_time(k[5]) for k in kerns]))
    deq_kernel_ms = float(np.mean([k[6].elapsed_time(k[7]) for k in kerns]))

    base_flops = 2.0 * M * N * K
    lora_flops = 2.0 * M * r * (K + N)
    G = K // 64
    deq_bytes = lay.packed_bytes + 4 * N * G + 2 * N * K + mp.numel() * 4
    q_bytes = 4 * N * K + lay.packed_bytes + 4 * N * G
    value = 2 * base_flops / (ms_per_step * 1e-3) / 1e12
    fwd_tflops = base_flops / (fwd_kernel_ms * 1e-3) / 1e12
    out = {
        "metric": "fused dequant-GEMM TFLOP/s (fwd + input-gradient base flops over the whole step), "
                  f"{N}x{K} @{L.mean_bits:g} bits/param; dequant HBM GB/s in passes",
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"config {args.config}: W {N}x{K} fp32 N(0,0.02), group 64, {L.mean_bits:g} bits/param, "
                               f"x {M}x{K} bf16, LoRA rank {r}, quantize+dequantize+fwd+bwd-input",
                   "N": N, "K": K, "M": M, "r": r, "bits_per_param": L.mean_bits},
        "instrumented_ms_per_step": float(np.mean([marks[i][0].elapsed_time(marks[i][4]) for i in range(n_inst)])),
        "passes": {
            "quantize": {"ms": pass_ms["quantize"], "kernel_ms": q_kernel_ms, "stream_ms": q_stream_ms,
                         "GB/s_stream": q_bytes / q_stream_ms / 1e6, "GB/s_in_step": q_bytes / q_kernel_ms / 1e6,
                         "frac_hbm_peak_stream": q_bytes / q_stream_ms / 1e6 / HBM_PEAK_GBPS,
                         "frac_hbm_peak_in_step": q_bytes / q_kernel_ms / 1e6 / HBM_PEAK_GBPS,
                         "frac_copy_ceiling_stream": q_bytes / q_stream_ms / 1e6 / ceil["copy_GB/s"],
                         "frac_read_ceiling_stream": q_bytes / q_stream_ms / 1e6 / ceil["read_GB/s"]},
            "dequantize": {"ms": pass_ms["dequantize"], "kernel_ms": deq_kernel_ms, "stream_ms": deq_stream_ms,
                           "GB/s_stream": deq_bytes / deq_stream_ms / 1e6, "GB/s_in_step": deq_bytes / deq_kernel_ms / 1e6,
                           "frac_hbm_peak_stream": deq_bytes / deq_stream_ms / 1e6 / HBM_PEAK_GBPS,
                           "frac_hbm_peak_in_step": deq_bytes / deq_kernel_ms / 1e6 / HBM_PEAK_GBPS,
                           "frac_copy_ceiling_stream": deq_bytes / deq_stream_ms / 1e6 / ceil["copy_GB/s"]},
            "learn_tables": {"stream_ms": learn_stream_ms, "rounds": 2, "GB/s": 4.0 * N * K / learn_stream_ms / 1e6,
                             "frac_hbm_peak": 4.0 * N * K / learn_stream_ms / 1e6 / HBM_PEAK_GBPS,
                             "note": "not part of the step; 4 B/weight read once"},
            "channel_mse": {"stream_ms": mse_stream_ms, "GB/s": 4.0 * N * K / mse_stream_ms / 1e6,
                            "frac_hbm_peak": 4.0 * N * K / mse_stream_ms / 1e6 / HBM_PEAK_GBPS,
                            "note": "not part of the step; error table at 1, 2 and 4 bits, 4 B/weight read once"},
            "adapter_grads": None if grads_stream_ms is None else {
                "stream_ms": grads_stream_ms, "contraction_kernels_ms": grads_db_kernel_ms,
                "GB/s": 2.0 * M * (K + N) / grads_stream_ms / 1e6,
                "frac_hbm_peak": 2.0 * M * (K + N) / grads_stream_ms / 1e6 / HBM_PEAK_GBPS,
                "contraction_kernels_GB/s": 2.0 * M * (K + N) / grads_db_kernel_ms / 1e6,
                "from_side_products_ms": grads_side_ms,
                "from_side_products_GB/s": None if grads_side_ms is None else 2.0 * M * (K + N) / grads_side_ms / 1e6,
                "from_side_products_frac_hbm_peak": None if grads_side_ms is None else 2.0 * M * (K + N) / grads_side_ms / 1e6 / HBM_PEAK_GBPS,
                "note": "not part of the step; bytes = x and dY once (the standalone call reads each twice: once for the rank-r "
                        "intermediate, once for the gradient; from_side_products takes the intermediates from the workspaces "
                        "of the step's two linear calls and reads each once); contraction_kernels = the two token contractions dY^T (s t) and (s u)^T x, one launch, with their chunk sums"},
            "loftq_init": None if loftq_ms is None else {
                "ms": loftq_ms, "steps": 5, "power_iterations": LOFTQ_ROUNDS, "GB/s": LOFTQ_BYTES_PER_WEIGHT * N * K / loftq_ms / 1e6,
                "frac_hbm_peak": LOFTQ_BYTES_PER_WEIGHT * N * K / loftq_ms / 1e6 / HBM_PEAK_GBPS,
                "note": "not part of the step; bytes = the passes over N x K data the call makes by design (%d B per weight: "
                        "4 residuals W - B A 8 B, 5 quantize 4 B, 5 decode-and-subtract 6 B, 5 x (2 x rounds + 1) products with "
                        "E or E^T 2 B)" % LOFTQ_BYTES_PER_WEIGHT},
            "linear_fwd": {"ms": pass_ms["linear_fwd"], "kernel_ms": fwd_kernel_ms,
                           "TFLOP/s": base_flops / pass_ms["linear_fwd"] / 1e9,
                           "TFLOP/s_with_lora": (base_flops + lora_flops) / pass_ms["linear_fwd"] / 1e9},
            "linear_bwd_input": {"ms": pass_ms["linear_bwd_input"], "kernel_ms": bwd_kernel_ms,
                                 "TFLOP/s": base_flops / pass_ms["linear_bwd_input"] / 1e9,
                                 "kernel_TFLOP/s": base_flops / bwd_kernel_ms / 1e9,
                                 "kernel_frac_mfma_peak": base_flops / bwd_kernel_ms / 1e9 / MFMA_BF16_PEAK_TFLOPS,
                                 "kernel_frac_mfma_ceiling": base_flops / bwd_kernel_ms / 1e9 / ceil["mfma_bf16_TFLOP/s"],
                                 "kernel_frac_mfma_random_data_ceiling": base_flops / bwd_kernel_ms / 1e9 / ceil["mfma_bf16_random_data_TFLOP/s"]},
        },
        "ceilings": ceil,
        "roofline": {"kernel": "linear_fwd_kernel", "bound": "mfma", "achieved": fwd_tflops,
                     "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": fwd_tflops / MFMA_BF16_PEAK_TFLOPS,
                     "frac_of_mfma_ceiling": fwd_tflops / ceil["mfma_bf16_TFLOP/s"],
                     "frac_of_mfma_random_data_ceiling": fwd_tflops / ceil["mfma_bf16_random_data_TFLOP/s"],
                     "traffic": profiled_traffic_bytes(args.config), "kernel_ms": fwd_kernel_ms,
                     "algorithmic_flops_per_launch": base_flops, "algorithmic_hbm_bytes_per_launch":
                         2 * M * K + 2 * M * N + lay.packed_bytes + 4 * N * G + 2 * r * (K + N)},
    }

    if not args.no_library_gemm:
        # context, not a target: the rocm library's dense bf16 GEMM (through torch.matmul) on the same shape and the same
        # activations against the DEQUANTIZED weights -- what "dequantize, then the framework's matmul" (the paper's own
        # path) reaches on this chip at this size, with the same power-dependent clocks as the fused kernels
        out["ceilings"].update(library_gemm(np, torch, What, x, dY, base_flops))
        for key, t in (("frac_of_library_gemm", fwd_tflops), ):
            out["roofline"][key] = t / out["ceilings"]["library_bf16_gemm_fwd_TFLOP/s"]
        out["passes"]["linear_bwd_input"]["kernel_frac_of_library_gemm"] = \
            base_flops / bwd_kernel_ms / 1e9 / out["ceilings"]["library_bf16_gemm_bwd_TFLOP/s"]
    if not args.no_other_configs and args.config == 3:
        out["passes"]["other_configs"] = other_configs(np, torch, lowra, synth, ceil)
    if not args.no_gemv:
        # free the step's tensors first: config 5 keeps 2 GB of quantized state and draws 180 MB matrices
        del W, What, y, dX, x, dY, packed, absmax, states
        torch.cuda.empty_cache()
        g = gemv_measure(args, np, torch, lowra, synth, detailed=False)
        for per_tokens in g["tokens"].values():
            for v in per_tokens.values():
                if "GB/s" in v:
                    v["frac_read_ceiling"] = v["GB/s"] / ceil["read_GB/s"]
        out["passes"]["gemv_config5"] = g

    if not args.no_cpu_baseline:
        from oracle import lowra_oracle as orc

        rows = min(args.cpu_sample_rows, M)
        c0 = time.perf_counter()
        rp, ra = orc.quantize(L.W, L.bits, L.cb, L.thresholds)
        c1 = time.perf_counter()
        orc.dequantize(rp, ra, L.bits, L.cb, L.mappings, K)
        c2 = time.perf_counter()
        orc.linear_fwd(rp, ra, L.bits, L.cb, L.mappings, L.x[:rows], L.A, L.B, L.s)
        c3 = time.perf_counter()
        orc.linear_bwd_input(rp, ra, L.bits, L.cb, L.mappings, L.dY[:rows], L.A, L.B, L.s, K)
        c4 = time.perf_counter()
        orc.learn_tables(L.W[:1024], L.bits[:1024], L.cb[:1024], L.thresholds, L.mappings, 2)
        c5 = time.perf_counter()
        out["passes"]["learn_tables"]["cpu_oracle_ms"] = (c5 - c4) * 1e3 * (N / 1024)
        step_s = (c1 - c0) + (c2 - c1) + ((c3 - c2) + (c4 - c3)) * (M / rows)
        out["cpu_baseline"] = {
            "value": 2 * base_flops / step_s / 1e12, "unit": "TFLOP/s", "cores": orc.num_threads(), "kind": "oracle",
            "sample": f"full quantize ({c1 - c0:.2f} s) and dequantize ({c2 - c1:.2f} s); forward ({c3 - c2:.2f} s) and "
                      f"input gradient ({c4 - c3:.2f} s) on the first {rows} of {M} token rows, scaled by {M / rows:g}",
        }
    print(json.dumps(out))
    return 0


def other_configs(np, torch, lowra, synth, ceil):
    """Kernel times of the two fused GEMMs at configs 2 (4-bit rows present) and 4 (long contraction): random
    weights of the config's shape and width mix drawn on the GPU, 20 launches each through the timer hook."""
    res = {}
    gen = torch.Generator(device="cuda"); gen.manual_seed(synth.SEED + 1)
    thr_np, mp_np, cb_bits = synth.shared_codebooks()
    thr, mp = torch.from_numpy(thr_np).cuda(), torch.from_numpy(mp_np).cuda()
    for cfg in (2, 4):
        N, K, M, r, fr, _ = synth.CONFIGS[cfg]
        bits = synth.assign_bits(N, fr, np.random.default_rng([synth.SEED, cfg, 1]))
        cb = np.searchsorted(cb_bits, bits).astype(np.int32)
        lay = lowra.Layout(K, bits, cb, cb_bits)
        W = torch.randn((N, K), generator=gen, device="cuda") * 0.02
        packed, absmax = lowra.lowra_quantize(lay, W, thr)
        del W
        x = torch.randn((M, K), generator=gen, device="cuda").bfloat16()
        dY = torch.randn((M, N), generator=gen, device="cuda").bfloat16()
        A = (torch.randn((r, K), generator=gen, device="cuda") * 0.01).bfloat16()
        B = (torch.randn((N, r), generator=gen, device="cuda") * 0.01).bfloat16()
        y = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
        dX = torch.empty((M, K), dtype=torch.bfloat16, device="cuda")
        ws = torch.empty(max(lay.workspace_bytes(lowra.OP_LINEAR_FWD, M, r), lay.workspace_bytes(lowra.OP_LINEAR_BWD_INPUT, M, r), 16),
                         dtype=torch.uint8, device="cuda")
        n = 20
        ev = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(n)]
        for e in ev:
            for q in e:
                q.record()
        for it in range(5 + n):
            e = ev[max(it - 5, 0)]
            lowra.lowra_set_kernel_timer(e[0].cuda_event, e[1].cuda_event)
            lowra.lowra_linear_fwd(lay, packed, absmax, mp, x, A, B, 2.0, y=y, workspace=ws)
            lowra.lowra_set_kernel_timer(e[2].cuda_event, e[3].cuda_event)
            lowra.lowra_linear_bwd_input(lay, packed, absmax, mp, dY, A, B, 2.0, dX=dX, workspace=ws)
        lowra.lowra_set_kernel_timer(None, None)
        torch.cuda.synchronize()
        f_ms = float(np.median([e[0].elapsed_time(e[1]) for e in ev]))
        b_ms = float(np.median([e[2].elapsed_time(e[3]) for e in ev]))
        fl = 2.0 * M * N * K
        res[f"config{cfg}"] = {
            "shape": f"W {N}x{K}, {M} tokens, rank {r}, rows 1/2/4-bit {fr[0]:g}/{fr[1]:g}/{fr[2]:g}",
            "fwd_kernel_ms": f_ms, "fwd_kernel_TFLOP/s": fl / f_ms / 1e9, "fwd_frac_mfma_peak": fl / f_ms / 1e9 / MFMA_BF16_PEAK_TFLOPS,
            "bwd_kernel_ms": b_ms, "bwd_kernel_TFLOP/s": fl / b_ms / 1e9, "bwd_frac_mfma_peak": fl / b_ms / 1e9 / MFMA_BF16_PEAK_TFLOPS,
            "fwd_frac_mfma_ceiling": fl / f_ms / 1e9 / ceil["mfma_bf16_TFLOP/s"], "bwd_frac_mfma_ceiling": fl / b_ms / 1e9 / ceil["mfma_bf16_TFLOP/s"]}
        del packed, absmax, x, dY, y, dX, ws
    return res


def library_gemm(np, torch, What, x, dY, flops):
    """y = x What^T and dX = dY What with torch.matmul (the rocm GEMM library) on the step's own tensors: 200 warm-up
    launches (clocks settle), then the mean of 50."""
    res = {}
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for key, a, b in (("fwd", x, What.t()), ("bwd", dY, What)):
        out = torch.empty((a.shape[0], b.shape[1]), dtype=torch.bfloat16, device="cuda")
        for _ in range(200):
            torch.matmul(a, b, out=out)
        e0.record()
        for _ in range(50):
            torch.matmul(a, b, out=out)
        e1.record(); torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / 50
        res[f"library_bf16_gemm_{key}_ms"] = ms
        res[f"library_bf16_gemm_{key}_TFLOP/s"] = flops / ms / 1e9
        del out
    res["library_note"] = ("torch.matmul (rocm GEMM library) on the same shape, the step's activations and the dequantized "
                           "bf16 weights: the unfused path's GEMM, for context")
    return res


def measure_ceilings(np, torch, lowra):
    """The ceilings every fraction is also printed against, measured on this device in this run with the
    library's measurement kernels: a 1 GiB device copy and a 1 GiB streaming read (both far beyond the
    256 MB memory-side cache; 3 timed launches each after one warm-up) and a register-only loop of bf16
    MFMAs on every compute unit."""
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    nbytes = 1 << 30
    src = torch.empty(nbytes, dtype=torch.uint8, device="cuda").fill_(1)
    dst = torch.empty_like(src)
    out4 = torch.zeros(16, dtype=torch.uint8, device="cuda")

    def timed(fn, reps=3):
        fn(); torch.cuda.synchronize()
        ts = []
        for _ in range(reps):
            e0.record(); fn(); e1.record(); torch.cuda.synchronize()
            ts.append(e0.elapsed_time(e1))
        return float(np.median(ts))

    copy_ms = timed(lambda: lowra.lowra_measure_copy(dst, src))
    read_ms = timed(lambda: lowra.lowra_measure_read(src, out4))
    del src, dst
    flops = [0.0]

    def mfma():
        flops[0] = lowra.lowra_measure_mfma(4096, 20000, out4)
    mfma_ms = timed(mfma)
    const_flops = flops[0]

    def mfma_random():
        flops[0] = lowra.lowra_measure_mfma(4096, 20000, out4, random_operands=True)
    mfma_random_ms = timed(mfma_random)
    return {"copy_GB/s": 2.0 * nbytes / copy_ms / 1e6, "read_GB/s": nbytes / read_ms / 1e6,
            "mfma_bf16_TFLOP/s": const_flops / mfma_ms / 1e9,
            "mfma_bf16_random_data_TFLOP/s": flops[0] / mfma_random_ms / 1e9,
            "note": "measured in this run: 1 GiB device copy (read + write bytes), 1 GiB streaming read, "
                    "register-only v_mfma_f32_32x32x16_bf16 loop (4096 workgroups x 4 wavefronts x 20000 x 4) on constant "
                    "operands, and the same loop on pseudo-random bf16 operands that change with every instruction (the "
                    "matrix pipe's sustained rate depends on what the data toggles)"}


def gemv_measure(args, np, torch, lowra, synth, detailed: bool):
    """Config 5: quantize all 224 matrices of the 32-layer weight set, then the small-token forward and input gradient
    over them (token counts 1, 4, 16; LoRA rank 16): the whole set as ONE run of the batched entry point (the streaming
    kernels), and one library call per matrix, back to back on one stream.  The fp32 weights are drawn on the
    GPU (seeded) one decoder layer at a time; only the quantized state (about 2 GB) stays resident.  Bytes per pass:
    packed codes + absmax + x + y of every matrix.  detailed: also graph replays and smaller batches."""
    thr_np, mp_np, cb_bits = synth.shared_codebooks()
    thr, mp = torch.from_numpy(thr_np).cuda(), torch.from_numpy(mp_np).cuda()
    r = synth.CFG5_RANK
    gen = torch.Generator(device="cuda"); gen.manual_seed(synth.SEED)
    mats, mats16, q_ms, qb_ms, q_bytes = [], [], 0.0, 0.0, 0
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e2, e3 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    lora = {}
    for layer in range(synth.LLAMA7B_LAYERS):
        # the seven fp32 matrices of the layer are drawn first (0.81 GB, past the memory-side cache), then quantized
        # back to back between one pair of events: one synchronisation per layer
        todo = []
        for idx, (name, N, K) in enumerate(synth.LLAMA7B_LAYER):
            bits = synth.assign_bits(N, synth.CFG5_FRACTIONS, np.random.default_rng([synth.SEED, 5, 8 * layer + idx, 1]))
            cb = np.searchsorted(cb_bits, bits).astype(np.int32)
            lay = lowra.Layout(K, bits, cb, cb_bits)
            W = torch.randn((N, K), generator=gen, device="cuda") * 0.02
            packed = torch.empty(lay.packed_bytes, dtype=torch.uint8, device="cuda")
            absmax = torch.empty((N, K // 64), dtype=torch.float32, device="cuda")
            todo.append((lay, W, packed, absmax, bits, cb, N, K))
        e0.record()
        for lay, W, packed, absmax, bits, cb, N, K in todo:
            lowra.lowra_quantize(lay, W, thr, packed, absmax)
        e1.record()
        # the same seven matrices through the batched entry point: one launch, no gaps between matrices
        e2.record()
        lowra.lowra_quantize_batch([t[0] for t in todo], [t[1] for t in todo], [thr] * len(todo), [t[2] for t in todo], [t[3] for t in todo])
        e3.record(); torch.cuda.synchronize()
        if layer > 0:                   # layer 0 warms up
            q_ms += e0.elapsed_time(e1)
            qb_ms += e2.elapsed_time(e3)
            q_bytes += sum(4 * N * K + lay.packed_bytes + 4 * N * (K // 64) for lay, W, packed, absmax, bits, cb, N, K in todo)
        for lay, W, packed, absmax, bits, cb, N, K in todo:
            # the same weights with bf16 group scales (a second quantized state: codes differ where the rounded scale moves a weight across a threshold)
            lay16 = lowra.Layout(K, bits, cb, cb_bits).set_scale_dtype(torch.bfloat16)
            packed16, absmax16 = lowra.lowra_quantize(lay16, W, thr)
            mats16.append((lay16, packed16, absmax16, N, K))
            if (N, K) not in lora:
                lora[(N, K)] = ((torch.randn((r, K), generator=gen, device="cuda") * 0.01).bfloat16(),
                                (torch.randn((N, r), generator=gen, device="cuda") * 0.01).bfloat16())
            mats.append((lay, packed, absmax, N, K))
        del todo
    state_bytes = sum(m[0].packed_bytes + 4 * m[3] * (m[4] // 64) for m in mats)
    # (a run is 0.6-3.5 ms: with fewer repetitions the median still sits in the clock ramp after the host-side set-up)
    reps = 20 if not detailed else max(args.steps // 20, 3)
    res = {}
    for M in synth.CFG5_TOKENS:
        xs = {K: torch.randn((M, K), generator=gen, device="cuda").bfloat16() for K in {m[4] for m in mats}}
        ys = {N: torch.empty((M, N), dtype=torch.bfloat16, device="cuda") for N in {m[3] for m in mats}}
        ws = torch.empty(max(max(m[0].workspace_bytes(lowra.OP_LINEAR_FWD, M, r) for m in mats), 16),
                         dtype=torch.uint8, device="cuda")
        byts = state_bytes + sum(2 * M * (m[3] + m[4]) for m in mats)

        def rate(ms, **extra):
            return {"ms": ms, "GB/s": byts / ms / 1e6, "frac_hbm_peak": byts / ms / 1e6 / HBM_PEAK_GBPS, **extra}

        def stream():
            for lay, packed, absmax, N, K in mats:
                A, B = lora[(N, K)]
                lowra.lowra_linear_fwd(lay, packed, absmax, mp, xs[K], A, B, 2.0, y=ys[N], workspace=ws)

        def timed(fn, warm=10):
            for _ in range(warm):
                fn()
            torch.cuda.synchronize()
            ts = []
            for _ in range(reps):
                e0.record(); fn(); e1.record(); torch.cuda.synchronize()
                ts.append(e0.elapsed_time(e1))
            return float(np.median(ts))

        res[str(M)] = {}
        if detailed or M != 4:
            ms = timed(stream)
            res[str(M)]["one_call_per_matrix"] = rate(ms, us_per_matrix=ms * 1e3 / len(mats))

        # The same 224 calls captured once into a HIP graph and replayed: no host work between the
        # launches; with `branches` > 1 the calls are dealt round-robin onto parallel branches (each
        # with its own workspace and outputs), so independent matrices overlap their latency chains.
        def graph_ms(branches):
            side = [torch.cuda.Stream() for _ in range(branches - 1)]
            wss = [ws] + [torch.empty_like(ws) for _ in range(branches - 1)]
            ysb = [ys] + [{n: torch.empty_like(t) for n, t in ys.items()} for _ in range(branches - 1)]
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                main = torch.cuda.current_stream()
                for sd in side:
                    sd.wait_stream(main)
                for i, (lay, packed, absmax, N, K) in enumerate(mats):
                    b = i % branches
                    A, B = lora[(N, K)]
                    with torch.cuda.stream(main if b == 0 else side[b - 1]):
                        lowra.lowra_linear_fwd(lay, packed, absmax, mp, xs[K], A, B, 2.0, y=ysb[b][N], workspace=wss[b])
                for sd in side:
                    main.wait_stream(sd)
            t = timed(g.replay, warm=3)
            return rate(t, us_per_matrix=t * 1e3 / len(mats))

        if detailed and not args.no_graph:
            res[str(M)]["graph_1_branch"] = graph_ms(1)
            res[str(M)]["graph_4_branches"] = graph_ms(4)

        # The batched entry point (lowra_fwd_batch_*): the same matrices, same inputs, but the calls of a group
        # are one run of the streaming kernel.  Groups of one decoder layer by data dependence:
        # q,k,v | o | gate,up | down; a whole layer; all layers.
        def batched(groups):
            batches = []
            for grp in groups:
                items = [(mats[i][0], mats[i][1], mats[i][2], xs[mats[i][4]], *lora[(mats[i][3], mats[i][4])]) for i in grp]
                batches.append(lowra.FwdBatch(items, mp, 2.0))

            def run():
                for b in batches:
                    b.run()
            t = timed(run)
            kern = None
            if len(batches) == 1:       # the streaming kernel alone, through the library's timer hook
                k0, k1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                k0.record(); k1.record()
                ks = []
                for _ in range(reps):
                    lowra.lowra_set_kernel_timer(k0.cuda_event, k1.cuda_event)
                    run()
                    lowra.lowra_set_kernel_timer(None, None)
                    torch.cuda.synchronize()
                    ks.append(k0.elapsed_time(k1))
                kern = float(np.median(ks))
            for b in batches:
                b.close()
            out = rate(t, runs=len(groups))
            if kern is not None:
                out["kernel_ms"] = kern
                out["kernel_GB/s"] = byts / kern / 1e6
            return out

        nl, per = synth.LLAMA7B_LAYERS, len(synth.LLAMA7B_LAYER)
        if detailed:
            by_dep = [[per * l + i for i in g] for l in range(nl) for g in ((0, 1, 2), (3,), (4, 5), (6,))]
            by_layer = [[per * l + i for i in range(per)] for l in range(nl)]
            res[str(M)]["batched_by_dependence"] = batched(by_dep)
            res[str(M)]["batched_by_layer"] = batched(by_layer)
        res[str(M)]["batched_whole_set"] = batched([list(range(nl * per))])

        # The input gradient of the same matrices (dX = dY What + s (dY B) A for M tokens): the whole set as one run of
        # lowra_bwd_batch_* (the streaming kernel: every code read once), and one lowra_linear_bwd_input call per matrix.
        dys = {N: torch.randn((M, N), generator=gen, device="cuda").bfloat16() for N in {m[3] for m in mats}}
        bb = lowra.BwdBatch([(m[0], m[1], m[2], dys[m[3]], *lora[(m[3], m[4])]) for m in mats], mp, 2.0)
        t = timed(bb.run)
        k0, k1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        k0.record(); k1.record()
        ks = []
        for _ in range(reps):
            lowra.lowra_set_kernel_timer(k0.cuda_event, k1.cuda_event)
            bb.run()
            lowra.lowra_set_kernel_timer(None, None)
            torch.cuda.synchronize()
            ks.append(k0.elapsed_time(k1))
        kern = float(np.median(ks))
        bb.close()
        del bb
        res[str(M)]["input_gradient_whole_set"] = rate(t, runs=1, **{"kernel_ms": kern, "kernel_GB/s": byts / kern / 1e6})
        if M == 1:
            # bf16 group scales (2 instead of 4 bytes per 64 weights): the same two whole-set runs on that state
            state16 = sum(m[0].packed_bytes + 2 * m[3] * (m[4] // 64) for m in mats16)
            byts16 = state16 + sum(2 * M * (m[3] + m[4]) for m in mats16)
            fb = lowra.FwdBatch([(m[0], m[1], m[2], xs[m[4]], *lora[(m[3], m[4])]) for m in mats16], mp, 2.0)
            tf = timed(fb.run)
            fb.close(); del fb
            bb = lowra.BwdBatch([(m[0], m[1], m[2], dys[m[3]], *lora[(m[3], m[4])]) for m in mats16], mp, 2.0)
            tb = timed(bb.run)
            bb.close(); del bb
            res[str(M)]["bf16_scales"] = {
                "quantized_state_bytes": state16, "algorithmic_bytes_per_weight": state16 / 6.476e9,
                "batched_whole_set": {"ms": tf, "GB/s": byts16 / tf / 1e6, "frac_hbm_peak": byts16 / tf / 1e6 / HBM_PEAK_GBPS},
                "input_gradient_whole_set": {"ms": tb, "GB/s": byts16 / tb / 1e6, "frac_hbm_peak": byts16 / tb / 1e6 / HBM_PEAK_GBPS},
                "note": "the kernels are bound by instruction issue and the LDS pipe, not by bytes: the time stays, the state shrinks by 10 %"}
        if detailed or M != 4:
            wsb = torch.empty(max(max(m[0].workspace_bytes(lowra.OP_LINEAR_BWD_INPUT, M, r) for m in mats), 16),
                              dtype=torch.uint8, device="cuda")
            dxs = {K: torch.empty((M, K), dtype=torch.bfloat16, device="cuda") for K in {m[4] for m in mats}}

            def stream_bwd():
                for lay, packed, absmax, N, K in mats:
                    A, B = lora[(N, K)]
                    lowra.lowra_linear_bwd_input(lay, packed, absmax, mp, dys[N], A, B, 2.0, dX=dxs[K], workspace=wsb)
            ms = timed(stream_bwd)
            res[str(M)]["input_gradient_one_call_per_matrix"] = rate(ms, us_per_matrix=ms * 1e3 / len(mats))
            del wsb
    return {
        "workload": "config 5: 224 matrices, 6.476 G weights, 50/25/25 % of 1/2/4-bit rows, LoRA rank 16",
        "quantized_state_bytes": state_bytes, "algorithmic_bytes_per_weight": state_bytes / 6.476e9,
        "tokens": res,
        "quantize_all": {"ms": qb_ms, "GB/s": q_bytes / qb_ms / 1e6, "frac_hbm_peak": q_bytes / qb_ms / 1e6 / HBM_PEAK_GBPS,
                         "one_call_per_matrix": {"ms": q_ms, "GB/s": q_bytes / q_ms / 1e6, "frac_hbm_peak": q_bytes / q_ms / 1e6 / HBM_PEAK_GBPS},
                         "note": "31 of 32 layers timed (the first warms up), one synchronisation per layer: the seven matrices of a layer as one lowra_quantize_batch call (one launch); one_call_per_matrix: seven lowra_quantize calls back to back"},
    }


def gemv_stream(args, np, torch, lowra, synth) -> int:
    g = gemv_measure(args, np, torch, lowra, synth, detailed=True)
    ceil = measure_ceilings(np, torch, lowra)
    best = g["tokens"]["1"]["batched_whole_set"]
    out = {
        "metric": "small-token dequant-GEMV stream GB/s over the 32-layer Llama-7B-shaped weight set @2.0 bits/param",
        "value": best["GB/s"], "unit": "GB/s", "n_gpus": 1, "higher_is_better": True, "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": g["workload"] + ", whole set as one batched run, 1 token",
                   "quantized_state_bytes": g["quantized_state_bytes"]},
        "tokens": g["tokens"], "quantize_all": g["quantize_all"], "ceilings": ceil,
        "roofline": {"kernel": "gemv_stream_kernel", "bound": "hbm", "achieved": best["GB/s"], "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": best["frac_hbm_peak"], "frac_of_read_ceiling": best["GB/s"] / ceil["read_GB/s"],
                     "traffic": None},
    }
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
