"""Seeded synthetic inputs for the ResQ mixed-precision linear layer.

This module only draws random numbers and shapes them; it holds none of the
method's arithmetic (no quantizer, no GEMM, no Hadamard) and imports neither
the HIP binding nor the CPU oracle, so both sides can be fed from it.

Every tensor is produced on the CPU with a seeded ``torch.Generator`` and cast
to bf16 before anything else sees it.  bf16 tensors are handed to numpy users
as their raw 16-bit patterns (``bf16_bits``).

The shapes are those of Llama-3-8B / Llama-3-70B / Qwen2.5-72B linear layers;
the value structure follows the paper's description of projected activations:
a few channels roughly 20x larger than the rest (Introduction), captured by the
high-precision group after the PCA projection (Section 4.2), and a random
orthogonal rotation inside each group that makes the coefficients close to
Gaussian (Lemma 4.1).  Heavy-tailed cases use Student-t (df=3) draws.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Optional

import numpy as np
import torch


@dataclass(frozen=True)
class LayerShape:
    """One linear layer: ``M`` tokens, ``K`` input features, ``N`` output
    features, ``r`` = width of the high-precision (INT8) group, columns [0, r)."""
    name: str
    M: int
    K: int
    N: int
    r: int
    act: str = "normal"          # "normal" | "student_t3"
    outliers: str = "none"       # "none" | "first4" | "one_percent_hi"
    rotate: bool = False         # random orthogonal rotation inside each group
    hadamard: bool = False       # online Walsh-Hadamard on columns [r, K) first
    seed: int = 0


# The five workload families named by the build's baseline description.
TINY = LayerShape("tiny", M=16, K=256, N=256, r=32, outliers="first4")
OPROJ_PREFILL = LayerShape("llama3_8b_o_proj_prefill", M=2048, K=4096, N=4096, r=512,
                           outliers="one_percent_hi", rotate=True)
MLP_GATE_UP = LayerShape("llama3_8b_gate_up_prefill", M=4096, K=4096, N=14336, r=512,
                         act="student_t3")
MLP_DOWN = LayerShape("llama3_8b_down_prefill", M=4096, K=14336, N=4096, r=1792,
                      act="student_t3", hadamard=True)


# Side paths of Section 4.3 on Llama-3-8B head shapes (2048 tokens, 8 K/V heads, d_head 128,
# an eighth of each head in 8 bits): the K and the V entries of 2048 tokens, one row per head,
# quantized asymmetrically per head; N = 0 marks a workload without a GEMM.
KV_CACHE_QUANT = LayerShape("llama3_8b_kv_cache_quant", M=2048 * 8 * 2, K=128, N=0, r=16,
                            act="student_t3", seed=7)

# The online projection of queries (32 heads) and keys (8 heads) after RoPE onto the cache
# basis U_C, in 8 bits: one row per token and head, K = N = d_head, every column high.
UC_PROJ = LayerShape("llama3_8b_uc_proj_prefill", M=2048 * (32 + 8), K=128, N=128, r=128, seed=8)


def chunk_shape(which: str, M: int) -> LayerShape:
    """A prefill chunk (or a large generation batch) of M tokens on a Llama-3-8B layer: few
    128 x 128 output tiles, the regime between the generation stage and a full prefill."""
    if which == "o_proj":
        return LayerShape(f"llama3_8b_o_proj_m{M}", M=M, K=4096, N=4096, r=512,
                          outliers="one_percent_hi", rotate=True)
    if which == "down":
        return LayerShape(f"llama3_8b_down_m{M}", M=M, K=14336, N=4096, r=1792,
                          act="student_t3", hadamard=True)
    raise ValueError(which)


def decode_shape(M: int) -> LayerShape:
    return LayerShape(f"llama3_70b_up_decode_m{M}", M=M, K=8192, N=28672, r=1024,
                      outliers="one_percent_hi")


def qwen_mlp_shape(r: int) -> LayerShape:
    return LayerShape(f"qwen2.5_72b_mlp_prefill_r{r}", M=8192, K=8192, N=29568, r=r,
                      act="student_t3")


def _gen(seed: int) -> torch.Generator:
    g = torch.Generator(device="cpu")
    g.manual_seed(int(seed))
    return g


def random_orthogonal(n: int, seed: int) -> torch.Tensor:
    """Q factor of a seeded Gaussian matrix, columns sign-fixed so that the
    result does not depend on the QR routine's sign convention.  fp32 [n, n]."""
    if n == 0:
        return torch.zeros(0, 0)
    a = torch.randn(n, n, generator=_gen(seed), dtype=torch.float64)
    q, rr = torch.linalg.qr(a)
    q = q * torch.sign(torch.diagonal(rr)).unsqueeze(0)
    return q.to(torch.float32)


def _draw(kind: str, rows: int, cols: int, g: torch.Generator) -> torch.Tensor:
    z = torch.randn(rows, cols, generator=g, dtype=torch.float32)
    if kind == "normal":
        return z
    if kind == "student_t3":
        # t_3 = z / sqrt(chi2_3 / 3), chi2_3 = sum of three squared normals
        c = torch.randn(rows, cols, 3, generator=g, dtype=torch.float32).square_().sum(-1)
        return z / torch.sqrt(c / 3.0)
    raise ValueError(kind)


def make_activations(shape: LayerShape, rows: Optional[int] = None) -> torch.Tensor:
    """bf16 ``[M, K]`` activations, already in the projected basis.

    ``rows`` overrides ``M`` (the first ``rows`` rows of the same stream are not
    guaranteed to equal a prefix of the full draw; callers that want a sample
    of a big workload slice the full tensor instead)."""
    M = shape.M if rows is None else rows
    K, r = shape.K, shape.r
    g = _gen(shape.seed)
    x = _draw(shape.act, M, K, g)
    if shape.outliers == "first4":
        x[:, :4] *= 20.0
    elif shape.outliers == "one_percent_hi":
        n_out = math.ceil(0.01 * K)
        if r > 0:
            n_out = min(n_out, r)
            perm = torch.randperm(r, generator=_gen(shape.seed + 100))[:n_out]
        else:
            perm = torch.randperm(K, generator=_gen(shape.seed + 100))[:n_out]
        x[:, perm] *= 20.0
    elif shape.outliers != "none":
        raise ValueError(shape.outliers)
    if shape.rotate:
        if r > 0:
            x[:, :r] = x[:, :r] @ random_orthogonal(r, shape.seed + 1)
        if K - r > 0:
            x[:, r:] = x[:, r:] @ random_orthogonal(K - r, shape.seed + 2)
    return x.to(torch.bfloat16).contiguous()


def make_weights(shape: LayerShape, rows: Optional[int] = None) -> torch.Tensor:
    """bf16 ``[N, K]`` weights (out_features, in_features), N(0, 0.02^2)."""
    N = shape.N if rows is None else rows
    g = _gen(shape.seed + 7)
    w = torch.randn(N, shape.K, generator=g, dtype=torch.float32) * 0.02
    return w.to(torch.bfloat16).contiguous()


def bf16_bits(t: torch.Tensor) -> np.ndarray:
    """Raw 16-bit patterns of a CPU bf16 tensor as a uint16 numpy array."""
    assert t.dtype == torch.bfloat16
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)


def bits_to_bf16(a: np.ndarray) -> torch.Tensor:
    """Inverse of :func:`bf16_bits`."""
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).view(torch.bfloat16)


def bits_to_f64(a: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns to float64."""
    u32 = a.astype(np.uint32) << np.uint32(16)
    return u32.view(np.float32).astype(np.float64)


def random_small_case(seed: int, M: int, K: int, N: int, r: int, *, act: str = "normal",
                      outliers: str = "none") -> tuple[torch.Tensor, torch.Tensor]:
    """Small seeded (X, W) pair for randomized parity cases."""
    s = LayerShape(f"rand{seed}", M=M, K=K, N=N, r=r, act=act, outliers=outliers, seed=seed)
    return make_activations(s), make_weights(s)
