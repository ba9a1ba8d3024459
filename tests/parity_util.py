"""Helpers shared by the GPU parity tests (comparison rules only)."""
import numpy as np
import torch

from paper_2412_14363_amd import workloads as wl

# bf16 outputs: max relative error 1e-2 against the oracle's fp64 evaluation of
# the fp32 formula.  Outputs near zero are measured against a floor of
# 2^-6 * rms(y) instead of their own magnitude (a sum of signed terms can cancel
# to far below the size of its terms, where a relative error says nothing).
REL_TOL = 1e-2


def y_within_tolerance(y_gpu_bf16: torch.Tensor, y_ref: np.ndarray):
    y = wl.bits_to_f64(wl.bf16_bits(y_gpu_bf16.cpu()))
    rms = float(np.sqrt(np.mean(y_ref ** 2))) if y_ref.size else 0.0
    denom = np.maximum(np.abs(y_ref), 2.0 ** -6 * rms)
    denom = np.where(denom == 0, 1.0, denom)
    rel = np.abs(y - y_ref) / denom
    return float(rel.max()) if rel.size else 0.0


def unpack_nibbles(p: np.ndarray, cols: int) -> np.ndarray:
    lo = (p & 0xF).astype(np.int8)
    hi = (p >> 4).astype(np.int8)
    out = np.empty((p.shape[0], p.shape[1] * 2), np.int8)
    out[:, 0::2] = lo - 8
    out[:, 1::2] = np.where(hi > 7, hi - 16, hi)
    return out[:, :cols]
