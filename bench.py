#!/usr/bin/env python3
"""Benchmark of the LowRA hot path on one MI355X.

A step is one pass of the whole path over config 3 (W 11008x4096 at 1.5 bits/param, 4096 tokens,
LoRA rank 64): quantize -> dequantize -> fused dequant-GEMM forward -> fused input gradient, all
through the C ABI, inputs resident in HBM.  Prints one JSON line.

  value      TFLOP/s of the step: base GEMM flops of forward + input gradient (2 * 2MNK) over the
             whole step time (quantize and dequantize included)
  roofline   the forward fused dequant-GEMM kernel alone, timed with HIP events recorded around its
             launch (lowra_set_kernel_timer), against the bf16 dense MFMA peak
  passes     per-pass times and rates, incl. the dequantize pass in GB/s against the HBM peak
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
MFMA_BF16_PEAK_TFLOPS = 2500.0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=3, choices=[1, 2, 3, 4])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-rows", type=int, default=256)
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

    def one_step(marks, kern):
        marks[0].record()
        lowra.lowra_quantize(lay, W, thr, packed, absmax)
        marks[1].record()
        lowra.lowra_dequantize(lay, packed, absmax, mp, out=What)
        marks[2].record()
        lowra.lowra_set_kernel_timer(kern[0].cuda_event, kern[1].cuda_event)
        lowra.lowra_linear_fwd(lay, packed, absmax, mp, x, A, B, L.s, y=y, workspace=ws)
        marks[3].record()
        lowra.lowra_set_kernel_timer(kern[2].cuda_event, kern[3].cuda_event)
        lowra.lowra_linear_bwd_input(lay, packed, absmax, mp, dY, A, B, L.s, dX=dX, workspace=ws)
        marks[4].record()
        lowra.lowra_set_kernel_timer(None, None)

    marks = [[ev() for _ in range(5)] for _ in range(args.steps)]
    kerns = [[ev() for _ in range(4)] for _ in range(args.steps)]
    wm, wk = [ev() for _ in range(5)], [ev() for _ in range(4)]
    torch.cuda.synchronize()
    for _ in range(args.warmup):
        one_step(wm, wk)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        one_step(marks[i], kerns[i])
    torch.cuda.synchronize()
    t1 = time.perf_counter()

    ms_per_step = (t1 - t0) * 1e3 / args.steps
    pass_ms = {n: float(np.mean([marks[i][j].elapsed_time(marks[i][j + 1]) for i in range(args.steps)]))
               for j, n in enumerate(names)}
    fwd_kernel_ms = float(np.mean([k[0].elapsed_time(k[1]) for k in kerns]))
    bwd_kernel_ms = float(np.mean([k[2].elapsed_time(k[3]) for k in kerns]))

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
        "passes": {
            "quantize": {"ms": pass_ms["quantize"], "GB/s": q_bytes / pass_ms["quantize"] / 1e6,
                         "frac_hbm_peak": q_bytes / pass_ms["quantize"] / 1e6 / HBM_PEAK_GBPS},
            "dequantize": {"ms": pass_ms["dequantize"], "GB/s": deq_bytes / pass_ms["dequantize"] / 1e6,
                           "frac_hbm_peak": deq_bytes / pass_ms["dequantize"] / 1e6 / HBM_PEAK_GBPS},
            "linear_fwd": {"ms": pass_ms["linear_fwd"], "kernel_ms": fwd_kernel_ms,
                           "TFLOP/s": base_flops / pass_ms["linear_fwd"] / 1e9,
                           "TFLOP/s_with_lora": (base_flops + lora_flops) / pass_ms["linear_fwd"] / 1e9},
            "linear_bwd_input": {"ms": pass_ms["linear_bwd_input"], "kernel_ms": bwd_kernel_ms,
                                 "TFLOP/s": base_flops / pass_ms["linear_bwd_input"] / 1e9,
                                 "kernel_TFLOP/s": base_flops / bwd_kernel_ms / 1e9},
        },
        "roofline": {"kernel": "linear_fwd_kernel", "bound": "mfma", "achieved": fwd_tflops,
                     "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": fwd_tflops / MFMA_BF16_PEAK_TFLOPS,
                     "traffic": None, "kernel_ms": fwd_kernel_ms},
    }

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
        step_s = (c1 - c0) + (c2 - c1) + ((c3 - c2) + (c4 - c3)) * (M / rows)
        out["cpu_baseline"] = {
            "value": 2 * base_flops / step_s / 1e12, "unit": "TFLOP/s", "cores": orc.num_threads(), "kind": "oracle",
            "sample": f"full quantize ({c1 - c0:.2f} s) and dequantize ({c2 - c1:.2f} s); forward ({c3 - c2:.2f} s) and "
                      f"input gradient ({c4 - c3:.2f} s) on the first {rows} of {M} token rows, scaled by {M / rows:g}",
        }
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
