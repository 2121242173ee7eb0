"""Helpers for the GPU parity tests: move seeded inputs to the device, run the oracle beside."""
import numpy as np
import torch

from oracle import lowra_oracle as orc
from paper_2502_08141_amd import lowra

REL_TOL = 2e-2   # max relative error allowed for linear outputs and gradients (bf16 vs fp64 oracle)


def bf16_dev(bits_u16: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(bits_u16).view(np.int16)).view(torch.bfloat16).cuda()


def bf16_host_bits(t: torch.Tensor) -> np.ndarray:
    return t.detach().cpu().view(torch.int16).numpy().view(np.uint16)


def bf16_host_f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().cpu().to(torch.float64).numpy()


class DeviceLayer:
    """A synth.Layer on the GPU plus its layout handle."""

    def __init__(self, L):
        self.L = L
        self.layout = lowra.Layout(L.K, L.bits, L.cb, L.cb_bits)
        self.thr = torch.from_numpy(L.thresholds).cuda()
        self.mp = torch.from_numpy(L.mappings).cuda()
        self.W = torch.from_numpy(L.W).cuda()
        self.x = bf16_dev(L.x); self.dY = bf16_dev(L.dY)
        self.A = bf16_dev(L.A) if L.r else None
        self.B = bf16_dev(L.B) if L.r else None

    def quantize(self):
        self.packed, self.absmax = lowra.lowra_quantize(self.layout, self.W, self.thr)
        return self.packed, self.absmax


def oracle_state(L):
    return orc.quantize(L.W, L.bits, L.cb, L.thresholds)


def rel_err(got: np.ndarray, ref: np.ndarray) -> float:
    """max |got - ref| / max(|ref|, rms(ref)): the floor keeps near-zero outputs from blowing up the ratio."""
    rms = float(np.sqrt(np.mean(ref * ref))) if ref.size else 1.0
    den = np.maximum(np.abs(ref), max(rms, 1e-30))
    return float((np.abs(got - ref) / den).max()) if ref.size else 0.0


def rel_err_unfloored_p999(got: np.ndarray, ref: np.ndarray) -> float:
    """99.9th percentile of the plain element-wise relative error |got - ref| / |ref| (no floor): reported
    beside rel_err, which is the asserted bound; entries with ref == 0 are left out."""
    nz = ref != 0
    if not nz.any():
        return 0.0
    return float(np.quantile(np.abs(got[nz] - ref[nz]) / np.abs(ref[nz]), 0.999))


def big_entries_rel_err(got: np.ndarray, ref: np.ndarray) -> float:
    """max plain relative error over the entries with |ref| >= rms(ref), where no floor acts."""
    rms = float(np.sqrt(np.mean(ref * ref))) if ref.size else 0.0
    sel = np.abs(ref) >= max(rms, 1e-30)
    return float((np.abs(got[sel] - ref[sel]) / np.abs(ref[sel])).max()) if sel.any() else 0.0
