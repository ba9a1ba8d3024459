"""ctypes front end of the CPU oracle (``resq_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by the tests, the smoke check and the
benchmark's cpu_baseline leg, never by the product path.  It builds the C file
with gcc on first use and passes numpy arrays straight through; the only
arithmetic done here is composing the oracle's steps in the paper's order
(Section 4.1: quantize activations and weights per group, two integer GEMMs,
sum of the dequantized products) and the textbook SNR.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass
from pathlib import Path
from typing import Optional

import numpy as np

_HERE = Path(__file__).resolve().parent
_SRC = _HERE / "resq_oracle.c"
_LIB = _HERE / "libresq_oracle.so"
_lib = None


def build(force: bool = False) -> Path:
    """Compile the oracle with gcc (plain C11 + OpenMP, strict IEEE arithmetic)."""
    if force or not _LIB.exists() or _LIB.stat().st_mtime < _SRC.stat().st_mtime:
        tmp = _LIB.with_suffix(f".tmp{os.getpid()}.so")
        cmd = ["gcc", "-std=c11", "-O2", "-fopenmp", "-fPIC", "-shared", "-ffp-contract=off",
               "-fno-fast-math", "-Wall", "-Wextra", "-o", str(tmp), str(_SRC), "-lm"]
        subprocess.run(cmd, check=True)
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = C.CDLL(str(_LIB))
        i64, p = C.c_int64, C.c_void_p
        lib.oracle_num_threads.restype = C.c_int
        lib.oracle_round_bf16.argtypes = [p, i64, p]
        lib.oracle_quantize_act.argtypes = [p, i64, i64, i64, i64, p, p, p, p]
        lib.oracle_quantize_weights.argtypes = [p, i64, i64, i64, i64, p, p, p, p]
        lib.oracle_pack_nibbles.argtypes = [p, i64, i64, i64, p]
        lib.oracle_odd_code_sums.argtypes = [p, i64, i64, p]
        lib.oracle_gemm_i64.argtypes = [p, i64, p, i64, i64, i64, i64, p]
        lib.oracle_gemm_i64.restype = i64
        lib.oracle_dequant.argtypes = [p, p, p, p, p, p, i64, i64, p]
        lib.oracle_hadamard.argtypes = [p, p, i64, i64, i64, i64, i64, i64]
        lib.oracle_quantize_act_asym.argtypes = [p, i64, i64, i64, i64, p, p, p, p, p, p]
        lib.oracle_gemm_u8i8_i64.argtypes = [p, i64, p, i64, i64, i64, i64, p]
        lib.oracle_dequant_asym.argtypes = [p, p, p, p, p, p, p, p, p, p, i64, i64, p]
        for f in ("oracle_round_bf16", "oracle_quantize_act", "oracle_quantize_weights",
                  "oracle_pack_nibbles", "oracle_odd_code_sums", "oracle_dequant",
                  "oracle_hadamard"):
            getattr(lib, f).restype = None
        _lib = lib
    return _lib


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _c(a: np.ndarray, dtype) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def round_bf16(y: np.ndarray) -> np.ndarray:
    """fp64 -> nearest bf16 bit patterns (ties to even)."""
    y = _c(y, np.float64)
    out = np.empty(y.shape, np.uint16)
    _load().oracle_round_bf16(_ptr(y), y.size, _ptr(out))
    return out


def quantize_act(x_bits: np.ndarray, r: int):
    """Eq. 2 per token.  Returns (q_hi int8 [M,r], q_lo int8 [M,K-r], s_hi f32 [M], s_lo f32 [M])."""
    x_bits = _c(x_bits, np.uint16)
    M, K = x_bits.shape
    q_hi = np.zeros((M, r), np.int8)
    q_lo = np.zeros((M, K - r), np.int8)
    s_hi = np.ones(M, np.float32)
    s_lo = np.ones(M, np.float32)
    _load().oracle_quantize_act(_ptr(x_bits), K, M, K, r, _ptr(q_hi), _ptr(q_lo), _ptr(s_hi),
                                _ptr(s_lo))
    return q_hi, q_lo, s_hi, s_lo


def quantize_weights(w_bits: np.ndarray, r: int):
    """Eq. 3 per output channel.  Returns (w_hi int8 [N,r], w_lo int8 [N,K-r],
    sw_hi fp16 bits [N], sw_lo fp16 bits [N])."""
    w_bits = _c(w_bits, np.uint16)
    N, K = w_bits.shape
    w_hi = np.zeros((N, r), np.int8)
    w_lo = np.zeros((N, K - r), np.int8)
    one = np.float16(1.0).view(np.uint16)
    sw_hi = np.full(N, one, np.uint16)
    sw_lo = np.full(N, one, np.uint16)
    _load().oracle_quantize_weights(_ptr(w_bits), K, N, K, r, _ptr(w_hi), _ptr(w_lo),
                                    _ptr(sw_hi), _ptr(sw_lo))
    return w_hi, w_lo, sw_hi, sw_lo


def pack_nibbles(codes: np.ndarray, ld_out: Optional[int] = None) -> np.ndarray:
    """4-bit codes, one per byte, -> two per byte: even element in bits 0..3 as
    code + 8, odd element in bits 4..7 in two's complement; padding bytes 0x08."""
    codes = _c(codes, np.int8)
    rows, cols = codes.shape
    assert cols % 2 == 0
    ld = cols // 2 if ld_out is None else int(ld_out)
    assert ld >= cols // 2
    out = np.empty((rows, ld), np.uint8)
    _load().oracle_pack_nibbles(_ptr(codes), rows, cols, ld, _ptr(out))
    return out


def odd_code_sums(codes: np.ndarray) -> np.ndarray:
    """Per row, the sum of the codes in odd positions, int32."""
    codes = _c(codes, np.int8)
    rows, cols = codes.shape
    out = np.zeros(rows, np.int32)
    _load().oracle_odd_code_sums(_ptr(codes), rows, cols, _ptr(out))
    return out


def gemm_i64(a: np.ndarray, b: np.ndarray) -> np.ndarray:
    """acc[m,n] = sum_k a[m,k] b[n,k], exact; asserts every result fits int32."""
    a = _c(a, np.int8)
    b = _c(b, np.int8)
    M, Kc = a.shape
    N, Kb = b.shape
    assert Kc == Kb
    acc = np.zeros((M, N), np.int64)
    if Kc > 0:
        bad = _load().oracle_gemm_i64(_ptr(a), Kc, _ptr(b), Kc, M, N, Kc, _ptr(acc))
        assert bad == 0, f"{bad} accumulators do not fit int32"
    return acc


def dequant(acc_hi, acc_lo, s_hi, s_lo, sw_hi, sw_lo) -> np.ndarray:
    """y = A_hi s_hi sw_hi + A_lo s_lo sw_lo in fp64; a None accumulator is an empty group."""
    ref = acc_hi if acc_hi is not None else acc_lo
    M, N = ref.shape
    y = np.empty((M, N), np.float64)
    ah = None if acc_hi is None else _c(acc_hi, np.int64)
    al = None if acc_lo is None else _c(acc_lo, np.int64)
    sh, sl = _c(s_hi, np.float32), _c(s_lo, np.float32)
    wh, wl = _c(sw_hi, np.uint16), _c(sw_lo, np.uint16)
    _load().oracle_dequant(_ptr(ah), _ptr(al), _ptr(sh), _ptr(sl), _ptr(wh), _ptr(wl), M, N,
                           _ptr(y))
    return y


def hadamard(x_bits: np.ndarray, c0: int, c1: int, block: int) -> np.ndarray:
    """Block-diagonal orthonormal Walsh-Hadamard on columns [c0, c1); bf16 bits in and out."""
    x_bits = _c(x_bits, np.uint16)
    M, K = x_bits.shape
    assert 0 <= c0 <= c1 <= K and block > 0 and (block & (block - 1)) == 0
    assert (c1 - c0) % block == 0
    y = np.empty_like(x_bits)
    _load().oracle_hadamard(_ptr(x_bits), _ptr(y), K, M, K, c0, c1, block)
    return y


@dataclass
class LayerResult:
    q_hi: np.ndarray      # int8 [M, r]
    q_lo: np.ndarray      # int8 [M, K-r], one code per byte
    s_hi: np.ndarray      # f32 [M]
    s_lo: np.ndarray      # f32 [M]
    w_hi: np.ndarray      # int8 [N, r]
    w_lo: np.ndarray      # int8 [N, K-r]
    sw_hi: np.ndarray     # fp16 bits [N]
    sw_lo: np.ndarray     # fp16 bits [N]
    acc_hi: np.ndarray    # int64 [M, N]
    acc_lo: np.ndarray    # int64 [M, N]
    y: np.ndarray         # f64 [M, N]


def linear(x_bits: np.ndarray, w_bits: np.ndarray, r: int, weights=None) -> LayerResult:
    """The whole layer, steps in the paper's order (Eq. 2, Eq. 3, Eq. 4).
    ``weights`` may carry an earlier ``quantize_weights`` result for reuse."""
    K = x_bits.shape[1]
    q_hi, q_lo, s_hi, s_lo = quantize_act(x_bits, r)
    w_hi, w_lo, sw_hi, sw_lo = weights if weights is not None else quantize_weights(w_bits, r)
    acc_hi = gemm_i64(q_hi, w_hi)
    acc_lo = gemm_i64(q_lo, w_lo)
    y = dequant(acc_hi if r > 0 else None, acc_lo if K - r > 0 else None, s_hi, s_lo, sw_hi,
                sw_lo)
    return LayerResult(q_hi, q_lo, s_hi, s_lo, w_hi, w_lo, sw_hi, sw_lo, acc_hi, acc_lo, y)


# ---- asymmetric activations (the other branch of Eq. 1) ---------------------

def quantize_act_asym(x_bits: np.ndarray, r: int):
    """Eq. 2 per token with the asymmetric quantizer of Eq. 1.  Returns
    (q_hi uint8 [M,r] in 0..255, q_lo uint8 [M,K-r] in 0..15, s_hi, s_lo, z_hi, z_lo f32 [M])."""
    x_bits = _c(x_bits, np.uint16)
    M, K = x_bits.shape
    q_hi = np.zeros((M, r), np.uint8)
    q_lo = np.zeros((M, K - r), np.uint8)
    s_hi, s_lo = np.ones(M, np.float32), np.ones(M, np.float32)
    z_hi, z_lo = np.zeros(M, np.float32), np.zeros(M, np.float32)
    _load().oracle_quantize_act_asym(_ptr(x_bits), K, M, K, r, _ptr(q_hi), _ptr(q_lo), _ptr(s_hi),
                                     _ptr(s_lo), _ptr(z_hi), _ptr(z_lo))
    return q_hi, q_lo, s_hi, s_lo, z_hi, z_lo


def kv_cache_row_bytes(d_head: int, r: int) -> int:
    """Bytes of one cache row (one head of one token): r codes of 8 bits, d_head - r codes of 4
    bits, and scale and zero-point of both groups in fp32."""
    return r + (d_head - r) // 2 + 16


def pack_kv_cache(q_hi: np.ndarray, q_lo: np.ndarray, s_hi, z_hi, s_lo, z_lo) -> np.ndarray:
    """Compact storage of mixed-precision K/V cache entries (Section 5.1 and Appendix C: the
    cache is quantized per head, asymmetrically, an eighth of the channels in 8 bits).  One row
    per head of a token, no padding:
        bytes [0, r)                 the 8-bit codes of Eq. 1's asymmetric branch, 0..255
        bytes [r, r + (d - r)/2)     the 4-bit codes, 0..15, channel r + 2j in bits 0..3 of byte j,
                                     channel r + 2j + 1 in bits 4..7
        then four little-endian fp32: s_hi, z_hi, s_lo, z_lo   (x ~ code * s + z per group)
    The codes and parameters are those of quantize_act_asym on rows of d_head columns."""
    q_hi, q_lo = _c(q_hi, np.uint8), _c(q_lo, np.uint8)
    rows, r = q_hi.shape
    kl = q_lo.shape[1]
    assert kl % 2 == 0 and q_lo.shape[0] == rows
    out = np.zeros((rows, r + kl // 2 + 16), np.uint8)
    out[:, :r] = q_hi
    out[:, r:r + kl // 2] = q_lo[:, 0::2] | (q_lo[:, 1::2] << 4)
    params = np.stack([np.asarray(v, np.float32) for v in (s_hi, z_hi, s_lo, z_lo)], axis=1)
    out[:, r + kl // 2:] = params.astype("<f4").view(np.uint8).reshape(rows, 16)
    return out


def dequantize_kv_cache(cache: np.ndarray, d_head: int, r: int) -> np.ndarray:
    """What a reader of the cache reconstructs (Eq. 1): code * s + z per group, in fp64."""
    cache = _c(cache, np.uint8)
    rows = cache.shape[0]
    kl = d_head - r
    par = cache[:, r + kl // 2:r + kl // 2 + 16].copy().view("<f4").astype(np.float64)
    x = np.zeros((rows, d_head), np.float64)
    x[:, :r] = cache[:, :r].astype(np.float64) * par[:, 0:1] + par[:, 1:2]
    lo = cache[:, r:r + kl // 2]
    x[:, r + 0::2] = (lo & 15).astype(np.float64) * par[:, 2:3] + par[:, 3:4]
    x[:, r + 1::2] = (lo >> 4).astype(np.float64) * par[:, 2:3] + par[:, 3:4]
    return x


def gemm_u8i8_i64(a: np.ndarray, b: np.ndarray) -> np.ndarray:
    """acc[m,n] = sum_k a[m,k] b[n,k] for unsigned a and signed b, exact in int64."""
    a = _c(a, np.uint8)
    b = _c(b, np.int8)
    M, Kc = a.shape
    N, Kb = b.shape
    assert Kc == Kb
    acc = np.zeros((M, N), np.int64)
    if Kc > 0:
        _load().oracle_gemm_u8i8_i64(_ptr(a), Kc, _ptr(b), Kc, M, N, Kc, _ptr(acc))
    return acc


def dequant_asym(acc_hi, acc_lo, s_hi, s_lo, z_hi, z_lo, wsum_hi, wsum_lo, sw_hi, sw_lo):
    """y = sum over groups of sw (s A + z wsum) in fp64; a None accumulator is an empty group."""
    ref = acc_hi if acc_hi is not None else acc_lo
    M, N = ref.shape
    y = np.empty((M, N), np.float64)
    ah = None if acc_hi is None else _c(acc_hi, np.int64)
    al = None if acc_lo is None else _c(acc_lo, np.int64)
    arrs = [_c(v, np.float32) for v in (s_hi, s_lo, z_hi, z_lo)]
    wsh, wsl = _c(wsum_hi, np.int64), _c(wsum_lo, np.int64)
    wh, wl = _c(sw_hi, np.uint16), _c(sw_lo, np.uint16)
    _load().oracle_dequant_asym(_ptr(ah), _ptr(al), *[_ptr(v) for v in arrs], _ptr(wsh), _ptr(wsl),
                                _ptr(wh), _ptr(wl), M, N, _ptr(y))
    return y


@dataclass
class AsymLayerResult:
    q_hi: np.ndarray      # uint8 [M, r], 0..255
    q_lo: np.ndarray      # uint8 [M, K-r], 0..15
    s_hi: np.ndarray
    s_lo: np.ndarray
    z_hi: np.ndarray      # f32 [M]: min of the group
    z_lo: np.ndarray
    wsum_hi: np.ndarray   # int64 [N]: sums of the weight codes
    wsum_lo: np.ndarray
    acc_hi: np.ndarray    # int64 [M, N], sums over the unsigned codes
    acc_lo: np.ndarray
    y: np.ndarray         # f64 [M, N]


def linear_asym(x_bits: np.ndarray, w_bits: np.ndarray, r: int, weights=None) -> AsymLayerResult:
    """The layer with per-token asymmetric activations (Section 5.1) and the same
    symmetric per-channel weights."""
    K = x_bits.shape[1]
    q_hi, q_lo, s_hi, s_lo, z_hi, z_lo = quantize_act_asym(x_bits, r)
    w_hi, w_lo, sw_hi, sw_lo = weights if weights is not None else quantize_weights(w_bits, r)
    acc_hi = gemm_u8i8_i64(q_hi, w_hi)
    acc_lo = gemm_u8i8_i64(q_lo, w_lo)
    wsum_hi = w_hi.sum(axis=1, dtype=np.int64)
    wsum_lo = w_lo.sum(axis=1, dtype=np.int64)
    y = dequant_asym(acc_hi if r > 0 else None, acc_lo if K - r > 0 else None, s_hi, s_lo, z_hi,
                     z_lo, wsum_hi, wsum_lo, sw_hi, sw_lo)
    return AsymLayerResult(q_hi, q_lo, s_hi, s_lo, z_hi, z_lo, wsum_hi, wsum_lo, acc_hi, acc_lo, y)


def swiglu(y: np.ndarray) -> np.ndarray:
    """Gated pair epilogue of the MLP front (the activation function that precedes the
    down_proj input, Section 4.3): columns 2c and 2c+1 of ``y`` are the gate and the up
    output of feature c; returns silu(gate) * up, silu(x) = x / (1 + exp(-x)), in fp64."""
    y = np.asarray(y, np.float64)
    gate, up = y[:, 0::2], y[:, 1::2]
    return gate / (1.0 + np.exp(-gate)) * up


def snr_db(ref: np.ndarray, approx: np.ndarray) -> float:
    """10 log10( sum ref^2 / sum (ref - approx)^2 ), fp64."""
    ref = np.asarray(ref, np.float64)
    err = ref - np.asarray(approx, np.float64)
    den = float(np.sum(err * err))
    num = float(np.sum(ref * ref))
    return float("inf") if den == 0.0 else 10.0 * np.log10(num / den)
