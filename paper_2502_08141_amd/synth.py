"""Seeded synthetic inputs for the LowRA hot path -- inputs only, none of the method's arithmetic.

Both the CPU oracle's tests and the HIP path's tests/benchmark draw their inputs here, so the two
sides see identical bytes.  Nothing in this module quantizes, packs, decodes or multiplies
matrices.  Everything is numpy on the host; bf16 tensors are uint16 bit patterns.

The shapes stand in for the paper's workloads: LLaMA-2-7B/13B linear layers (4096x4096,
11008x4096, 5120x13824; Sec. 6.1), 64-element groups (Sec. 4.1), precisions {1,2,4} (Sec. 6.2),
LoRA rank 64 and bf16 training (App. I).  The real weights and datasets are not used.

Recipe: numpy.random.default_rng([8141, cfg, stream]) with stream 0: W, 1: precision assignment,
2: x, 3: A, 4: B, 5: dY, 6: outlier positions; config 5 adds the key 8*layer + matrix.
"""
from __future__ import annotations

from dataclasses import dataclass
from statistics import NormalDist

import numpy as np
import torch

TABLE_STRIDE = 16
GROUP = 64
SEED = 8141


def to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round an fp32/fp64 array to bf16 with torch's CPU cast and return the uint16 bit patterns."""
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16).copy()


def bf16_bits_to_f64(h: np.ndarray) -> np.ndarray:
    return (h.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def normal_quantile_levels(b: int) -> np.ndarray:
    """2^b levels at standard-normal quantiles, scaled so the end levels are -1 and +1 (fp64)."""
    n = 1 << b
    inv = NormalDist().inv_cdf
    q = np.array([inv((j + 0.5) / n) for j in range(n)], dtype=np.float64)
    return q / inv(1.0 - 0.5 / n)


def _input_tables(levels_list):
    """The threshold / mapping tables that the generated inputs carry: per-codebook levels stacked into ([C,16]
    thresholds padded with +inf, [C,16] mappings padded with 0), the thresholds halfway between consecutive levels.
    Input data only: both the oracle and the library receive these tables as arguments."""
    C = len(levels_list)
    thr = np.full((C, TABLE_STRIDE), np.inf, dtype=np.float32)
    mp = np.zeros((C, TABLE_STRIDE), dtype=np.float32)
    for c, lv in enumerate(levels_list):
        lv = np.asarray(lv, dtype=np.float64)
        mp[c, : lv.size] = lv.astype(np.float32)
        thr[c, : lv.size - 1] = ((lv[:-1] + lv[1:]) / 2.0).astype(np.float32)
    return thr, mp


def shared_codebooks():
    """The three per-precision codebooks of the configs: index 0 -> 1 bit, 1 -> 2 bits, 2 -> 4 bits."""
    thr, mp = _input_tables([normal_quantile_levels(b) for b in (1, 2, 4)])
    cb_bits = np.array([1, 2, 4], dtype=np.uint8)
    return thr, mp, cb_bits


def assign_bits(N: int, fractions, rng) -> np.ndarray:
    """Seeded per-output-channel precision: a random permutation cut into 1-, 2- and 4-bit runs."""
    f1, f2, f4 = fractions
    n1, n2 = int(round(f1 * N)), int(round(f2 * N))
    perm = rng.permutation(N)
    bits = np.full(N, 4, dtype=np.uint8)
    bits[perm[:n1]] = 1
    bits[perm[n1:n1 + n2]] = 2
    if f4 == 0.0:
        bits[perm[n1 + n2:]] = 2
    return bits


@dataclass
class Layer:
    name: str
    N: int
    K: int
    M: int
    r: int
    s: float
    W: np.ndarray            # fp32 [N,K]
    bits: np.ndarray         # uint8 [N]
    cb: np.ndarray           # int32 [N]
    cb_bits: np.ndarray      # uint8 [C]
    thresholds: np.ndarray   # fp32 [C,16]
    mappings: np.ndarray     # fp32 [C,16]
    x: np.ndarray            # uint16 (bf16) [M,K]
    dY: np.ndarray           # uint16 (bf16) [M,N]
    A: np.ndarray            # uint16 (bf16) [r,K]
    B: np.ndarray            # uint16 (bf16) [N,r]

    @property
    def mean_bits(self) -> float:
        return float(self.bits.astype(np.float64).mean())


CONFIGS = {
    # cfg: (N, K, M, r, (f1, f2, f4), weight law)
    1: (256, 512, 16, 8, (0.25, 0.50, 0.25), "normal"),
    2: (4096, 4096, 2048, 64, (0.50, 0.25, 0.25), "outliers"),
    3: (11008, 4096, 4096, 64, (0.50, 0.50, 0.0), "normal"),
    4: (5120, 13824, 4096, 64, (0.85, 0.15, 0.0), "student_t"),
}
# config 5: one decoder layer's matrices, (name, N, K); 32 such layers.
LLAMA7B_LAYER = [("q", 4096, 4096), ("k", 4096, 4096), ("v", 4096, 4096), ("o", 4096, 4096),
                 ("gate", 11008, 4096), ("up", 11008, 4096), ("down", 4096, 11008)]
LLAMA7B_LAYERS = 32
CFG5_FRACTIONS = (0.50, 0.25, 0.25)
CFG5_TOKENS = (1, 4, 16)
CFG5_RANK = 16


def _weights(N, K, law, key):
    rng = np.random.default_rng(key + [0])
    if law == "student_t":
        W = 0.02 * rng.standard_t(4, size=(N, K)) / np.sqrt(2.0)
    else:
        W = rng.normal(0.0, 0.02, size=(N, K))
    if law == "outliers":
        cnt = int(0.001 * N * K)
        pos = np.random.default_rng(key + [6]).choice(N * K, size=cnt, replace=False)
        W.reshape(-1)[pos] *= 10.0
    return W.astype(np.float32)


def _layer(name, key, N, K, M, r, s, fractions, law, per_channel_tables=False, want_w=True):
    bits = assign_bits(N, fractions, np.random.default_rng(key + [1]))
    thr, mp, cb_bits = shared_codebooks()
    cb = np.searchsorted(cb_bits, bits).astype(np.int32)
    if per_channel_tables:  # the paper's own data model: one table set per output channel (C == N)
        thr, mp, cb_bits = thr[cb].copy(), mp[cb].copy(), bits.copy()
        cb = np.arange(N, dtype=np.int32)
    W = _weights(N, K, law, key) if want_w else np.zeros((0, K), np.float32)
    x = to_bf16_bits(np.random.default_rng(key + [2]).normal(0.0, 1.0, size=(M, K)))
    dY = to_bf16_bits(np.random.default_rng(key + [5]).normal(0.0, 1.0, size=(M, N)))
    A = to_bf16_bits(np.random.default_rng(key + [3]).normal(0.0, 0.01, size=(r, K)))
    B = to_bf16_bits(np.random.default_rng(key + [4]).normal(0.0, 0.01, size=(N, r)))
    return Layer(name, N, K, M, r, s, W, bits, cb, cb_bits, thr, mp, x, dY, A, B)


def make_config(cfg: int, M: int | None = None, per_channel_tables: bool = False) -> Layer:
    """Configs 1-4.  M overrides the token count (a row subset is NOT a prefix of the full draw)."""
    N, K, M0, r, fr, law = CONFIGS[cfg]
    return _layer(f"cfg{cfg}", [SEED, cfg], N, K, M if M is not None else M0, r, 2.0, fr, law,
                  per_channel_tables=per_channel_tables)


def make_cfg5_matrix(layer: int, idx: int, M: int = 16) -> Layer:
    """Config 5: matrix idx (0..6) of decoder layer `layer` (0..31)."""
    name, N, K = LLAMA7B_LAYER[idx]
    return _layer(f"cfg5.L{layer}.{name}", [SEED, 5, 8 * layer + idx], N, K, M, CFG5_RANK, 2.0,
                  CFG5_FRACTIONS, "normal")


def make_custom(N, K, M, r, fractions=(0.34, 0.33, 0.33), seed=0, s=2.0, law="normal",
                per_channel_tables=False) -> Layer:
    """Free-form case for edge-shape tests."""
    return _layer(f"custom{seed}", [SEED, 99, seed], N, K, M, r, s, fractions, law,
                  per_channel_tables=per_channel_tables)
