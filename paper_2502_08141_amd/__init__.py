"""MI355X-native LowRA hot path: mixed-precision quantize / dequantize and the dequant-fused LoRA linear.

`paper_2502_08141_amd.lowra` is the thin binding over the C-ABI HIP library (csrc/, include/lowra.h);
`paper_2502_08141_amd.synth` holds the seeded input generators.  Nothing here falls back to the CPU.
"""
__all__ = ["lowra", "synth"]
