"""Python binding of the C ABI in ``include/resq.h``.

Argument marshalling only: every function here has the name of the C entry
point it calls, takes torch tensors (device memory and streams are the only
things torch is used for), checks their dtype/device, and passes raw pointers.
All arithmetic runs in the HIP kernels.  There is no CPU fallback: if the
library cannot be loaded, importing the symbols raises.
"""
from __future__ import annotations

import ctypes as C
from typing import Optional

import torch

from . import build as _build

RESQ_OK = 0
STATUS_NAMES = {0: "RESQ_OK", 1: "RESQ_ERR_NULL", 2: "RESQ_ERR_SHAPE", 3: "RESQ_ERR_ALIGN",
                4: "RESQ_ERR_BUFFER", 5: "RESQ_ERR_HIP"}

# every symbol include/resq.h declares: name -> (restype, argtypes)
_i64, _p, _sz = C.c_int64, C.c_void_p, C.c_size_t
SYMBOLS = {
    "resq_status_string": (C.c_char_p, [C.c_int]),
    "resq_time_next_kernel": (C.c_int, [_p, _p]),
    "resq_act_hi_ld": (_i64, [_i64, _i64]),
    "resq_act_lo_ld": (_i64, [_i64, _i64]),
    "resq_packed_weight_bytes": (_sz, [_i64, _i64, _i64]),
    "resq_hadamard_block": (_i64, [_i64]),
    "resq_quantize_act": (C.c_int, [_p, _i64, _i64, _i64, _i64, _p, _p, _p, _p, _p, _p]),
    "resq_hadamard_quantize_act": (C.c_int, [_p, _i64, _i64, _i64, _i64, _i64, _p, _p, _p, _p, _p, _p, _i64, _p]),
    "resq_quantize_act_asym": (C.c_int, [_p, _i64, _i64, _i64, _i64, _i64, _p, _p, _p, _p, _p, _p, _p, _p]),
    "resq_hadamard_quantize_act_asym": (C.c_int, [_p, _i64, _i64, _i64, _i64, _i64, _p, _p, _p, _p, _p, _p, _p, _p, _i64, _p]),
    "resq_gemm_mixed_asym": (C.c_int, [_p, _p, _p, _p, _p, _p, _p, _i64, _p, _i64, _i64, _i64, _p, _i64, _p, _p, _p]),
    "resq_gemm_mixed_plan": (C.c_int, [_i64, _i64, _i64, _i64, C.POINTER(C.c_int), C.POINTER(C.c_int), C.POINTER(C.c_int)]),
    "resq_quantize_gemm_mixed": (C.c_int, [_p, _i64, _i64, _p, _i64, _i64, _i64, _p, _i64, _p]),
    "resq_gemm_mixed_swiglu": (C.c_int, [_p, _p, _p, _p, _p, _i64, _p, _i64, _i64, _i64, _p, _i64, _p]),
    "resq_gram_accumulate": (C.c_int, [_p, _i64, _i64, _i64, _p, _i64, _p]),
    "resq_sym_eig_workspace_bytes": (_sz, [_i64]),
    "resq_sym_eig": (C.c_int, [_p, _i64, _i64, C.c_int, _p, _p, _i64, _p, _sz, _p]),
    "resq_sym_eig_static": (C.c_int, [_p, _i64, _i64, C.c_int, _p, _p, _i64, _p]),
    "resq_project_rows": (C.c_int, [_p, C.c_int, _i64, _i64, _i64, _p, _i64, _i64, _p, C.c_int, _i64, _p]),
    "resq_project_heads": (C.c_int, [_p, _i64, _i64, _i64, _p, _p, _i64, _p]),
    "resq_kv_cache_row_bytes": (_sz, [_i64, _i64]),
    "resq_quantize_kv_cache": (C.c_int, [_p, _i64, _i64, _i64, _i64, _p, _i64, _p]),
    "resq_dequantize_kv_cache": (C.c_int, [_p, _i64, _i64, _i64, _i64, _p, _i64, _p]),
    "resq_pack_weights": (C.c_int, [_p, _i64, _i64, _i64, _i64, _p, _sz, _p]),
    "resq_unpack_weights": (C.c_int, [_p, _i64, _i64, _i64, _p, _p, _p, _p, _p]),
    "resq_gemm_mixed": (C.c_int, [_p, _p, _p, _p, _p, _i64, _p, _i64, _i64, _i64, _p, _i64, _p, _p, _p]),
    "resq_online_hadamard": (C.c_int, [_p, _p, _i64, _i64, _i64, _i64, _i64, _i64, _p]),
}

_lib = None


class ResqError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = lib().resq_status_string(status).decode()
        super().__init__(f"{where}: {msg}")


def lib() -> C.CDLL:
    """The loaded HIP library (built on first use if no library is there)."""
    global _lib
    if _lib is None:
        path = _build.ensure_built()
        handle = C.CDLL(str(path))
        for name, (res, args) in SYMBOLS.items():
            fn = getattr(handle, name)  # AttributeError if the symbol is missing
            fn.restype = res
            fn.argtypes = args
        _lib = handle
    return _lib


def _check(status: int, where: str) -> None:
    if status != RESQ_OK:
        raise ResqError(status, where)


def _dev(t: Optional[torch.Tensor], dtype, name: str):
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError(f"{name} must live in device memory")
    if t.dtype != dtype:
        raise ValueError(f"{name} must be {dtype}, got {t.dtype}")
    return t.data_ptr()


def _check_layer_buffers(where: str, act: "ActCodes", packed: torch.Tensor, N: int, n_out: int,
                         y: torch.Tensor, dbg=(), want_asym: bool = False) -> None:
    """Sizes the kernels rely on: a mismatch would make them read or write past a buffer."""
    M, K, r = act.M, act.K, act.r
    need = resq_packed_weight_bytes(N, K, r)
    if need == 0:
        raise ValueError(f"{where}: invalid (N, K, r) = ({N}, {K}, {r})")
    if packed.numel() < need:
        raise ValueError(f"{where}: packed holds {packed.numel()} bytes, (N, K, r) = ({N}, {K}, {r}) needs {need}")
    if act.asym != want_asym:
        raise ValueError(f"{where}: the activation codes are {'asymmetric' if act.asym else 'symmetric'}; "
                         f"use resq_gemm_mixed{'_asym' if act.asym else ''}")
    if tuple(y.shape) != (M, n_out):
        raise ValueError(f"{where}: y must be [{M}, {n_out}], got {tuple(y.shape)}")
    for name, t in dbg:
        if t is not None and (tuple(t.shape) != (M, N) or not t.is_contiguous()):
            raise ValueError(f"{where}: {name} must be a contiguous [{M}, {N}] tensor")
    if act.q_hi.shape != (M, act.ld_hi) or act.q_lo.shape != (M, act.ld_lo) or act.ld_hi != resq_act_hi_ld(K, r) \
            or act.ld_lo != resq_act_lo_ld(K, r):
        raise ValueError(f"{where}: activation code buffers do not match (M, K, r) = ({M}, {K}, {r})")


def _stream(stream) -> int:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


# ---- layout queries ---------------------------------------------------------

def resq_act_hi_ld(K: int, r: int) -> int:
    return int(lib().resq_act_hi_ld(K, r))


def resq_act_lo_ld(K: int, r: int) -> int:
    return int(lib().resq_act_lo_ld(K, r))


def resq_packed_weight_bytes(N: int, K: int, r: int) -> int:
    return int(lib().resq_packed_weight_bytes(N, K, r))


def resq_hadamard_block(width: int) -> int:
    return int(lib().resq_hadamard_block(width))


# ---- buffers ----------------------------------------------------------------

class ActCodes:
    """Device buffers resq_quantize_act writes and resq_gemm_mixed reads."""

    def __init__(self, M: int, K: int, r: int, device="cuda"):
        self.M, self.K, self.r = M, K, r
        self.ld_hi, self.ld_lo = resq_act_hi_ld(K, r), resq_act_lo_ld(K, r)
        if self.ld_hi < 0:
            raise ValueError("invalid (K, r)")
        self.q_hi = torch.empty((M, self.ld_hi), dtype=torch.int8, device=device)
        self.q_lo = torch.empty((M, self.ld_lo), dtype=torch.uint8, device=device)
        self.s_hi = torch.empty(M, dtype=torch.float32, device=device)
        self.s_lo = torch.empty(M, dtype=torch.float32, device=device)
        self.lo_sum = torch.empty(M, dtype=torch.int32, device=device)
        # asymmetric codes only (resq_quantize_act_asym): real value of the stored code 0
        self.c_hi = torch.empty(M, dtype=torch.float32, device=device)
        self.c_lo = torch.empty(M, dtype=torch.float32, device=device)
        self.asym = False


def alloc_packed(N: int, K: int, r: int, device="cuda") -> torch.Tensor:
    nbytes = resq_packed_weight_bytes(N, K, r)
    if nbytes == 0:
        raise ValueError("invalid (N, K, r)")
    return torch.empty(nbytes, dtype=torch.uint8, device=device)


# ---- the entry points -------------------------------------------------------

def resq_quantize_act(x: torch.Tensor, r: int, out: Optional[ActCodes] = None,
                      stream=None) -> ActCodes:
    M, K = x.shape
    if x.stride(1) != 1:
        raise ValueError("x must be row-major")
    if out is None:
        out = ActCodes(M, K, r, x.device)
    st = lib().resq_quantize_act(_dev(x, torch.bfloat16, "x"), x.stride(0), M, K, r,
                                 out.q_hi.data_ptr() if r > 0 else None,
                                 out.q_lo.data_ptr() if K - r > 0 else None,
                                 out.s_hi.data_ptr() if r > 0 else None,
                                 out.s_lo.data_ptr() if K - r > 0 else None,
                                 out.lo_sum.data_ptr() if K - r > 0 else None, _stream(stream))
    _check(st, "resq_quantize_act")
    return out


def resq_hadamard_quantize_act(x: torch.Tensor, r: int, block: int = 0,
                               out: Optional[ActCodes] = None,
                               x_rot: Optional[torch.Tensor] = None, stream=None) -> ActCodes:
    M, K = x.shape
    if x.stride(1) != 1:
        raise ValueError("x must be row-major")
    if x_rot is not None and x_rot.stride(1) != 1:
        raise ValueError("x_rot must be row-major")
    if out is None:
        out = ActCodes(M, K, r, x.device)
    st = lib().resq_hadamard_quantize_act(
        _dev(x, torch.bfloat16, "x"), x.stride(0), M, K, r, block,
        out.q_hi.data_ptr() if r > 0 else None, out.q_lo.data_ptr(),
        out.s_hi.data_ptr() if r > 0 else None, out.s_lo.data_ptr(), out.lo_sum.data_ptr(),
        _dev(x_rot, torch.bfloat16, "x_rot"), x_rot.stride(0) if x_rot is not None else 0,
        _stream(stream))
    _check(st, "resq_hadamard_quantize_act")
    return out


def resq_quantize_act_asym(x: torch.Tensor, r: int, hadamard_block: int = 0,
                           out: Optional[ActCodes] = None, stream=None) -> ActCodes:
    M, K = x.shape
    if x.stride(1) != 1:
        raise ValueError("x must be row-major")
    if out is None:
        out = ActCodes(M, K, r, x.device)
    hi, lo = r > 0, K - r > 0
    st = lib().resq_quantize_act_asym(
        _dev(x, torch.bfloat16, "x"), x.stride(0), M, K, r, hadamard_block,
        out.q_hi.data_ptr() if hi else None, out.q_lo.data_ptr() if lo else None,
        out.s_hi.data_ptr() if hi else None, out.s_lo.data_ptr() if lo else None,
        out.c_hi.data_ptr() if hi else None, out.c_lo.data_ptr() if lo else None,
        out.lo_sum.data_ptr() if lo else None, _stream(stream))
    _check(st, "resq_quantize_act_asym")
    out.asym = True
    return out


def resq_gemm_mixed_plan(M: int, N: int, K: int, r: int):
    """(kernel, token_groups, runs) that resq_gemm_mixed uses for this shape; host only."""
    k, tg, sk = C.c_int(), C.c_int(), C.c_int()
    _check(lib().resq_gemm_mixed_plan(M, N, K, r, C.byref(k), C.byref(tg), C.byref(sk)), "resq_gemm_mixed_plan")
    return k.value, tg.value, sk.value


def resq_quantize_gemm_mixed(x: torch.Tensor, packed: torch.Tensor, N: int, r: int,
                             y: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    M, K = x.shape
    if x.stride(1) != 1:
        raise ValueError("x must be row-major")
    if y is None:
        y = torch.empty((M, N), dtype=torch.bfloat16, device=x.device)
    if y.stride(1) != 1:
        raise ValueError("y must be row-major")
    need = resq_packed_weight_bytes(N, K, r)
    if need == 0 or packed.numel() < need or tuple(y.shape) != (M, N):
        raise ValueError(f"resq_quantize_gemm_mixed: packed ({packed.numel()} bytes, needs {need}) or y "
                         f"{tuple(y.shape)} do not match (M, N, K, r) = ({M}, {N}, {K}, {r})")
    st = lib().resq_quantize_gemm_mixed(
        _dev(x, torch.bfloat16, "x"), x.stride(0), M, _dev(packed, torch.uint8, "packed"), N, K, r,
        _dev(y, torch.bfloat16, "y"), y.stride(0), _stream(stream))
    _check(st, "resq_quantize_gemm_mixed")
    return y


def resq_hadamard_quantize_act_asym(x: torch.Tensor, r: int, block: int = 0,
                                    out: Optional[ActCodes] = None,
                                    x_rot: Optional[torch.Tensor] = None, stream=None) -> ActCodes:
    M, K = x.shape
    if x.stride(1) != 1:
        raise ValueError("x must be row-major")
    if x_rot is not None and x_rot.stride(1) != 1:
        raise ValueError("x_rot must be row-major")
    if out is None:
        out = ActCodes(M, K, r, x.device)
    hi = r > 0
    st = lib().resq_hadamard_quantize_act_asym(
        _dev(x, torch.bfloat16, "x"), x.stride(0), M, K, r, block,
        out.q_hi.data_ptr() if hi else None, out.q_lo.data_ptr(),
        out.s_hi.data_ptr() if hi else None, out.s_lo.data_ptr(),
        out.c_hi.data_ptr() if hi else None, out.c_lo.data_ptr(), out.lo_sum.data_ptr(),
        _dev(x_rot, torch.bfloat16, "x_rot"), x_rot.stride(0) if x_rot is not None else 0,
        _stream(stream))
    _check(st, "resq_hadamard_quantize_act_asym")
    out.asym = True
    return out


def resq_gemm_mixed_asym(act: ActCodes, packed: torch.Tensor, N: int,
                         y: Optional[torch.Tensor] = None,
                         dbg_acc_hi: Optional[torch.Tensor] = None,
                         dbg_acc_lo: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    M, K, r = act.M, act.K, act.r
    if y is None:
        y = torch.empty((M, N), dtype=torch.bfloat16, device=packed.device)
    if y.stride(1) != 1:
        raise ValueError("y must be row-major")
    _check_layer_buffers("resq_gemm_mixed_asym", act, packed, N, N, y,
                         (("dbg_acc_hi", dbg_acc_hi), ("dbg_acc_lo", dbg_acc_lo)), want_asym=True)
    hi, lo = r > 0, K - r > 0
    st = lib().resq_gemm_mixed_asym(
        act.q_hi.data_ptr() if hi else None, act.q_lo.data_ptr() if lo else None,
        act.s_hi.data_ptr() if hi else None, act.s_lo.data_ptr() if lo else None,
        act.c_hi.data_ptr() if hi else None, act.c_lo.data_ptr() if lo else None,
        act.lo_sum.data_ptr() if lo else None, M, _dev(packed, torch.uint8, "packed"), N, K, r,
        _dev(y, torch.bfloat16, "y"), y.stride(0), _dev(dbg_acc_hi, torch.int32, "dbg_acc_hi"),
        _dev(dbg_acc_lo, torch.int32, "dbg_acc_lo"), _stream(stream))
    _check(st, "resq_gemm_mixed_asym")
    return y


def resq_pack_weights(w: torch.Tensor, r: int, packed: Optional[torch.Tensor] = None,
                      stream=None) -> torch.Tensor:
    N, K = w.shape
    if w.stride(1) != 1:
        raise ValueError("w must be row-major [N, K]")
    if packed is None:
        packed = alloc_packed(N, K, r, w.device)
    st = lib().resq_pack_weights(_dev(w, torch.bfloat16, "w"), w.stride(0), N, K, r,
                                 _dev(packed, torch.uint8, "packed"), packed.numel(),
                                 _stream(stream))
    _check(st, "resq_pack_weights")
    return packed


def resq_unpack_weights(packed: torch.Tensor, N: int, K: int, r: int, stream=None):
    dev = packed.device
    need = resq_packed_weight_bytes(N, K, r)
    if need == 0 or packed.numel() < need:
        raise ValueError(f"resq_unpack_weights: packed holds {packed.numel()} bytes, (N, K, r) = ({N}, {K}, {r}) needs {need}")
    w_hi = torch.empty((N, r), dtype=torch.int8, device=dev)
    w_lo = torch.empty((N, K - r), dtype=torch.int8, device=dev)
    sw_hi = torch.empty(N, dtype=torch.int16, device=dev)
    sw_lo = torch.empty(N, dtype=torch.int16, device=dev)
    st = lib().resq_unpack_weights(_dev(packed, torch.uint8, "packed"), N, K, r,
                                   w_hi.data_ptr() if r > 0 else None,
                                   w_lo.data_ptr() if K - r > 0 else None,
                                   sw_hi.data_ptr() if r > 0 else None,
                                   sw_lo.data_ptr() if K - r > 0 else None, _stream(stream))
    _check(st, "resq_unpack_weights")
    return w_hi, w_lo, sw_hi, sw_lo


def resq_gemm_mixed(act: ActCodes, packed: torch.Tensor, N: int, y: Optional[torch.Tensor] = None,
                    dbg_acc_hi: Optional[torch.Tensor] = None,
                    dbg_acc_lo: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    M, K, r = act.M, act.K, act.r
    if y is None:
        y = torch.empty((M, N), dtype=torch.bfloat16, device=packed.device)
    if y.stride(1) != 1:
        raise ValueError("y must be row-major")
    _check_layer_buffers("resq_gemm_mixed", act, packed, N, N, y,
                         (("dbg_acc_hi", dbg_acc_hi), ("dbg_acc_lo", dbg_acc_lo)))
    st = lib().resq_gemm_mixed(act.q_hi.data_ptr() if r > 0 else None,
                               act.q_lo.data_ptr() if K - r > 0 else None,
                               act.s_hi.data_ptr() if r > 0 else None,
                               act.s_lo.data_ptr() if K - r > 0 else None,
                               act.lo_sum.data_ptr() if K - r > 0 else None, M,
                               _dev(packed, torch.uint8, "packed"), N, K, r,
                               _dev(y, torch.bfloat16, "y"), y.stride(0),
                               _dev(dbg_acc_hi, torch.int32, "dbg_acc_hi"),
                               _dev(dbg_acc_lo, torch.int32, "dbg_acc_lo"), _stream(stream))
    _check(st, "resq_gemm_mixed")
    return y


def resq_gemm_mixed_swiglu(act: ActCodes, packed: torch.Tensor, N2: int,
                           y: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """packed: 2F interleaved (gate, up) channels; returns y [M, F] = silu(gate) * up."""
    M, K, r = act.M, act.K, act.r
    if y is None:
        y = torch.empty((M, N2 // 2), dtype=torch.bfloat16, device=packed.device)
    if y.stride(1) != 1:
        raise ValueError("y must be row-major")
    if N2 % 2:
        raise ValueError("resq_gemm_mixed_swiglu: N2 must be even (interleaved gate and up rows)")
    _check_layer_buffers("resq_gemm_mixed_swiglu", act, packed, N2, N2 // 2, y)
    hi, lo = r > 0, K - r > 0
    st = lib().resq_gemm_mixed_swiglu(
        act.q_hi.data_ptr() if hi else None, act.q_lo.data_ptr() if lo else None,
        act.s_hi.data_ptr() if hi else None, act.s_lo.data_ptr() if lo else None,
        act.lo_sum.data_ptr() if lo else None, M, _dev(packed, torch.uint8, "packed"), N2, K, r,
        _dev(y, torch.bfloat16, "y"), y.stride(0), _stream(stream))
    _check(st, "resq_gemm_mixed_swiglu")
    return y


def resq_gram_accumulate(x: torch.Tensor, c: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """c (fp32 [K, K], zeros when not given) += x^T x for x bf16 [T, K]."""
    T, K = x.shape
    if x.stride(1) != 1:
        raise ValueError("x must be row-major")
    if c is None:
        c = torch.zeros((K, K), dtype=torch.float32, device=x.device)
    st = lib().resq_gram_accumulate(_dev(x, torch.bfloat16, "x"), x.stride(0), T, K,
                                    _dev(c, torch.float32, "c"), c.stride(0), _stream(stream))
    _check(st, "resq_gram_accumulate")
    return c


def resq_sym_eig(c: torch.Tensor, sweeps: int = 12, stream=None):
    """Eigenvalues (decreasing, fp32 [K]) and eigenvectors (columns of fp32 [K, K]) of the symmetric c."""
    K = c.shape[0]
    nbytes = lib().resq_sym_eig_workspace_bytes(K)
    work = torch.empty(max(nbytes, 1), dtype=torch.uint8, device=c.device)
    lam = torch.empty(K, dtype=torch.float32, device=c.device)
    p = torch.empty((K, K), dtype=torch.float32, device=c.device)
    st = lib().resq_sym_eig(_dev(c, torch.float32, "c"), c.stride(0), K, sweeps, lam.data_ptr(), p.data_ptr(),
                            p.stride(0), work.data_ptr(), nbytes, _stream(stream))
    _check(st, "resq_sym_eig")
    return lam, p


def resq_sym_eig_static(c: torch.Tensor, lam: torch.Tensor, p: torch.Tensor, sweeps: int = 12, stream=None):
    """resq_sym_eig into caller-provided outputs (lam fp32 [K], p fp32 [K, K]) on the library's
    built-in scratch area (K <= 512): the call itself allocates nothing."""
    K = c.shape[0]
    if tuple(lam.shape) != (K,) or tuple(p.shape) != (K, K) or p.stride(1) != 1:
        raise ValueError("lam must be [K] and p a row-major [K, K]")
    st = lib().resq_sym_eig_static(_dev(c, torch.float32, "c"), c.stride(0), K, sweeps, _dev(lam, torch.float32, "lam"),
                                   _dev(p, torch.float32, "p"), p.stride(0), _stream(stream))
    _check(st, "resq_sym_eig_static")
    return lam, p


def resq_project_rows(a: torch.Tensor, u: torch.Tensor, out: Optional[torch.Tensor] = None,
                      out_dtype=None, stream=None) -> torch.Tensor:
    """out = a @ u; a bf16 or fp32 [rows, K] (a column block of a wider matrix is fine), u fp32
    [K, J]; out bf16 or fp32 [rows, J] (a column block of a wider matrix is fine)."""
    rows, K = a.shape
    J = u.shape[1]
    if a.stride(1) != 1 or u.stride(1) != 1 or u.shape[0] != K:
        raise ValueError("a, u must be row-major with matching inner size")
    if a.dtype not in (torch.bfloat16, torch.float32):
        raise ValueError("a must be bf16 or fp32")
    if out is None:
        out = torch.empty((rows, J), dtype=out_dtype or a.dtype, device=a.device)
    if out.stride(1) != 1 or out.dtype not in (torch.bfloat16, torch.float32):
        raise ValueError("out must be row-major bf16 or fp32")
    st = lib().resq_project_rows(_dev(a, a.dtype, "a"), int(a.dtype == torch.bfloat16), a.stride(0), rows, K,
                                 _dev(u, torch.float32, "u"), u.stride(0), J,
                                 _dev(out, out.dtype, "out"), int(out.dtype == torch.bfloat16), out.stride(0),
                                 _stream(stream))
    _check(st, "resq_project_rows")
    return out


def resq_project_heads(x: torch.Tensor, packed: torch.Tensor, y: Optional[torch.Tensor] = None,
                       stream=None) -> torch.Tensor:
    """x: bf16 [rows, d_head] (one row per token and head); packed: resq_pack_weights of the
    [d_head, d_head] matrix of output-channel rows with r = d_head; returns bf16 [rows, d_head]."""
    rows, d = x.shape
    if x.stride(1) != 1:
        raise ValueError("x must be row-major")
    if y is None:
        y = torch.empty((rows, d), dtype=torch.bfloat16, device=x.device)
    if y.stride(1) != 1:
        raise ValueError("y must be row-major")
    need = resq_packed_weight_bytes(d, d, d)
    if need == 0 or packed.numel() < need or tuple(y.shape) != (rows, d):
        raise ValueError(f"resq_project_heads: packed ({packed.numel()} bytes, needs {need}) or y {tuple(y.shape)} "
                         f"do not match rows = {rows}, d_head = {d}")
    st = lib().resq_project_heads(_dev(x, torch.bfloat16, "x"), x.stride(0), rows, d,
                                  _dev(packed, torch.uint8, "packed"),
                                  _dev(y, torch.bfloat16, "y"), y.stride(0),
                                  _stream(stream))
    _check(st, "resq_project_heads")
    return y


def resq_kv_cache_row_bytes(d_head: int, r: int) -> int:
    return int(lib().resq_kv_cache_row_bytes(d_head, r))


def resq_quantize_kv_cache(x: torch.Tensor, r: int, cache: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """x: bf16 [rows, d_head] (one row per token and head) -> uint8 [rows, row_bytes] compact cache rows."""
    rows, d = x.shape
    if x.stride(1) != 1:
        raise ValueError("x must be row-major")
    need = resq_kv_cache_row_bytes(d, r)
    if need == 0:
        raise ValueError(f"invalid (d_head, r) = ({d}, {r})")
    if cache is None:
        cache = torch.empty((rows, need), dtype=torch.uint8, device=x.device)
    if cache.dim() != 2 or cache.shape[0] != rows or cache.stride(1) != 1 or cache.shape[1] < need:
        raise ValueError(f"cache must be a row-major [{rows}, >= {need}] byte tensor")
    st = lib().resq_quantize_kv_cache(_dev(x, torch.bfloat16, "x"), x.stride(0), rows, d, r,
                                      _dev(cache, torch.uint8, "cache"), cache.stride(0), _stream(stream))
    _check(st, "resq_quantize_kv_cache")
    return cache


def resq_dequantize_kv_cache(cache: torch.Tensor, d_head: int, r: int, out: Optional[torch.Tensor] = None,
                             stream=None) -> torch.Tensor:
    """The reader: bf16 [rows, d_head] = code * s + z of every channel."""
    rows = cache.shape[0]
    need = resq_kv_cache_row_bytes(d_head, r)
    if need == 0 or cache.dim() != 2 or cache.stride(1) != 1 or cache.shape[1] < need:
        raise ValueError(f"cache must be a row-major [rows, >= {need}] byte tensor for (d_head, r) = ({d_head}, {r})")
    if out is None:
        out = torch.empty((rows, d_head), dtype=torch.bfloat16, device=cache.device)
    if tuple(out.shape) != (rows, d_head) or out.stride(1) != 1:
        raise ValueError(f"out must be a row-major [{rows}, {d_head}] tensor")
    st = lib().resq_dequantize_kv_cache(_dev(cache, torch.uint8, "cache"), cache.stride(0), rows, d_head, r,
                                        _dev(out, torch.bfloat16, "out"), out.stride(0), _stream(stream))
    _check(st, "resq_dequantize_kv_cache")
    return out


def resq_online_hadamard(x: torch.Tensor, col_begin: int, col_end: int, block: int = 0,
                         out: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    M, K = x.shape
    if x.stride(1) != 1:
        raise ValueError("x must be row-major")
    if out is None:
        out = torch.empty_like(x)
    if out.stride() != x.stride():
        raise ValueError("out must have x's layout")
    st = lib().resq_online_hadamard(_dev(x, torch.bfloat16, "x"), _dev(out, torch.bfloat16, "out"),
                                    x.stride(0), M, K, col_begin, col_end, block, _stream(stream))
    _check(st, "resq_online_hadamard")
    return out
