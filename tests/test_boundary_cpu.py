"""Host-side checks of the C ABI that need no GPU: the library loads, exports
every symbol the header declares, answers the layout queries, and turns bad
arguments into status codes before anything is launched."""
import ctypes as C
import re
from pathlib import Path

import pytest

from paper_2412_14363_amd import binding

ROOT = Path(__file__).resolve().parent.parent


def declared_symbols():
    text = (ROOT / "include" / "resq.h").read_text()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(resq_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_symbols()
    assert len(names) >= 10
    handle = C.CDLL(str(binding._build.ensure_built()))
    for n in names:
        assert hasattr(handle, n), f"{n} declared in resq.h but not exported"
    assert sorted(binding.SYMBOLS) == names


def test_layout_queries():
    assert binding.resq_act_hi_ld(256, 32) == 128
    assert binding.resq_act_lo_ld(256, 32) == 128          # 224 codes -> 256 -> 128 bytes
    assert binding.resq_act_hi_ld(4096, 512) == 512
    assert binding.resq_act_lo_ld(4096, 512) == 1792
    assert binding.resq_act_hi_ld(4096, 0) == 0 and binding.resq_act_lo_ld(4096, 4096) == 0
    assert binding.resq_act_hi_ld(10, 3) == -1             # K - r odd
    assert binding.resq_act_lo_ld(8, 9) == -1
    # 8192 x 28672, r = 1024: 4.5 bits per weight plus two fp16 scales and three int32 sums per channel
    assert binding.resq_packed_weight_bytes(28672, 8192, 1024) == 28672 * (1024 + 3584) + 16 * 28672
    # N is padded to 256 rows
    assert binding.resq_packed_weight_bytes(29568, 8192, 1024) == 29696 * (1024 + 3584 + 16)
    assert binding.resq_packed_weight_bytes(0, 8, 0) == 0
    assert binding.resq_hadamard_block(12544) == 256
    assert binding.resq_hadamard_block(14336) == 2048
    assert binding.resq_hadamard_block(1 << 20) == 8192
    assert binding.resq_hadamard_block(7) == 1 and binding.resq_hadamard_block(0) == 0


def test_status_strings():
    L = binding.lib()
    for code, name in binding.STATUS_NAMES.items():
        assert L.resq_status_string(code).decode().startswith(name)
    assert b"unknown" in L.resq_status_string(99)


P = 0x10000   # a plausible, aligned, never dereferenced address


def test_quantize_act_rejects_bad_arguments():
    f = binding.lib().resq_quantize_act
    assert f(P, 256, 0, 256, 32, P, P, P, P, P, None) == 2         # M < 1
    assert f(P, 256, 4, 256, 257, P, P, P, P, P, None) == 2        # r > K
    assert f(P, 256, 4, 256, 33, P, P, P, P, P, None) == 2         # K - r odd
    assert f(P, 255, 4, 256, 32, P, P, P, P, P, None) == 2         # ldx < K
    assert f(None, 256, 4, 256, 32, P, P, P, P, P, None) == 1
    assert f(P, 256, 4, 256, 32, None, P, P, P, P, None) == 1
    assert f(P, 256, 4, 256, 32, P, P, P, None, P, None) == 1
    assert f(P, 256, 4, 256, 32, P, P, P, P, None, None) == 1      # lo_sum missing
    assert f(P, 256, 4, 256, 256, P, None, P, None, None, None) != 1   # r = K: low pointers may be null
    assert f(P, 256, 4, 256, 32, P + 8, P, P, P, P, None) == 3
    assert f(P + 1, 256, 4, 256, 32, P, P, P, P, P, None) == 3


def test_pack_and_gemm_reject_bad_arguments():
    L = binding.lib()
    need = binding.resq_packed_weight_bytes(256, 256, 32)
    assert L.resq_pack_weights(P, 256, 256, 256, 32, P, need - 1, None) == 4
    assert L.resq_pack_weights(P, 256, 256, 256, 32, P + 16, need, None) == 3
    assert L.resq_pack_weights(None, 256, 256, 256, 32, P, need, None) == 1
    assert L.resq_pack_weights(P, 100, 256, 256, 32, P, need, None) == 2
    g = L.resq_gemm_mixed
    assert g(P, P, P, P, P, 16, P, 256, 256, 32, P, 255, None, None, None) == 2   # ldy < N
    assert g(P, P, P, P, P, 16, None, 256, 256, 32, P, 256, None, None, None) == 1
    assert g(None, P, P, P, P, 16, P, 256, 256, 32, P, 256, None, None, None) == 1
    assert g(P, P, P, P, None, 16, P, 256, 256, 32, P, 256, None, None, None) == 1
    assert g(P, P + 4, P, P, P, 16, P, 256, 256, 32, P, 256, None, None, None) == 3
    assert g(P, P, P, P, P, 16, P, 256, 256, 31, P, 256, None, None, None) == 2
    u = L.resq_unpack_weights
    assert u(None, 256, 256, 32, P, P, P, P, None) == 1
    assert u(P, 256, 256, 32, P, None, P, P, None) == 1


def test_hadamard_rejects_bad_arguments():
    h = binding.lib().resq_online_hadamard
    assert h(P, P, 512, 4, 512, 0, 512, 3, None) == 2              # not a power of two
    assert h(P, P, 512, 4, 512, 0, 512, 1024, None) == 2           # does not divide the width
    assert h(P, P, 512, 4, 512, 0, 768, 0, None) == 2              # col_end > K
    assert h(P, P, 512, 4, 512, 8, 8, 0, None) == 2                # empty range
    assert h(None, P, 512, 4, 512, 0, 512, 0, None) == 1
    assert h(P, P, 512, 4, 512, 4, 260, 0, None) == 3              # col_begin not a multiple of 8
    assert h(P + 2, P, 512, 4, 512, 0, 512, 0, None) == 3


def test_hadamard_quantize_rejects_bad_arguments():
    f = binding.lib().resq_hadamard_quantize_act
    ok = (P, 1024, 4, 1024, 256)
    assert f(*ok, 3, P, P, P, P, P, None, 0, None) == 2            # block not a power of two
    assert f(*ok, 1024, P, P, P, P, P, None, 0, None) == 2         # block > 512
    assert f(*ok, 4, P, P, P, P, P, None, 0, None) == 2            # block < 8
    assert f(P, 1024, 4, 1024, 128, 256, P, P, P, P, P, None, 0, None) == 2   # block does not divide r
    assert f(P, 1024, 4, 1024, 1024, 0, P, P, P, P, P, None, 0, None) == 2    # empty low group
    assert f(P, 16384, 4, 8192 + 2048, 2048, 0, P, P, P, P, P, None, 0, None) == 2   # default block 8192
    assert f(*ok, 256, P, P, P, P, P, P, 1000, None) == 2          # ld_rot < K
    assert f(*ok, 256, P, P, P, P, P, P + 8, 1024, None) == 3      # x_rot not 16-byte aligned
    assert f(P + 2, 1024, 4, 1024, 256, 256, P, P, P, P, P, None, 0, None) == 3      # needs the vector path
    assert f(None, 1024, 4, 1024, 256, 256, P, P, P, P, P, None, 0, None) == 1
    assert f(*ok, 256, P, P, P, P, None, None, 0, None) == 1       # lo_sum missing


def test_asym_entry_points_reject_bad_arguments():
    q = binding.lib().resq_quantize_act_asym
    assert q(P, 256, 4, 256, 32, 0, P, P, P, P, P, P, P, None) != 1
    assert q(P, 256, 4, 256, 32, 0, P, P, P, P, None, P, P, None) == 1     # c_hi missing
    assert q(P, 256, 4, 256, 32, 0, P, P, P, P, P, None, P, None) == 1     # c_lo missing
    assert q(P, 256, 4, 256, 256, 0, P, None, P, None, P, None, None, None) != 1   # r = K
    assert q(P, 256, 4, 256, 32, 64, P, P, P, P, P, P, P, None) == 2       # block does not divide r
    assert q(P, 256, 4, 256, 33, 0, P, P, P, P, P, P, P, None) == 2        # K - r odd
    assert q(P, 256, 4, 256, 32, 0, P, P, P, P, P + 2, P, P, None) == 3
    h = binding.lib().resq_hadamard_quantize_act_asym
    ok = (P, 1024, 4, 1024, 256)
    assert h(*ok, 3, P, P, P, P, P, P, P, None, 0, None) == 2              # block not a power of two
    assert h(*ok, 256, P, P, P, P, None, P, P, None, 0, None) == 1         # c_hi missing
    assert h(*ok, 256, P, P, P, P, P, P, P, P, 1000, None) == 2            # ld_rot < K
    assert h(*ok, 256, P, P, P, P, P, P, P, P + 8, 1024, None) == 3        # x_rot not 16-byte aligned
    assert h(P + 2, 1024, 4, 1024, 256, 256, P, P, P, P, P, P, P, None, 0, None) == 3   # needs the vector path
    g = binding.lib().resq_gemm_mixed_asym
    assert g(P, P, P, P, None, P, P, 16, P, 256, 256, 32, P, 256, None, None, None) == 1
    assert g(P, P, P, P, P, None, P, 16, P, 256, 256, 32, P, 256, None, None, None) == 1
    assert g(P, P, P, P, P, P, P, 16, P, 256, 256, 32, P, 255, None, None, None) == 2


def test_swiglu_entry_point_rejects_bad_arguments():
    g = binding.lib().resq_gemm_mixed_swiglu
    assert g(P, P, P, P, P, 16, P, 255, 256, 32, P, 256, None) == 2          # odd channel count
    assert g(P, P, P, P, P, 16, P, 256, 256, 32, P, 127, None) == 2          # ldy < N2 / 2
    assert g(P, P, P, P, P, 16, None, 256, 256, 32, P, 128, None) == 1
    assert g(P, P, P, P, None, 16, P, 256, 256, 32, P, 128, None) == 1


def test_project_heads_rejects_bad_arguments():
    g = binding.lib().resq_project_heads
    assert g(P, 128, 64, 96, P, P, 128, None) == 2                           # d_head not 64 / 128
    assert g(P, 120, 64, 128, P, P, 128, None) == 2                          # ldx < d_head
    assert g(P, 128, 64, 128, P, P, 100, None) == 2                          # ldy < d_head
    assert g(P, 128, -1, 128, P, P, 128, None) == 2
    assert g(None, 128, 64, 128, P, P, 128, None) == 1
    assert g(P, 128, 64, 128, None, P, 128, None) == 1
    assert g(P, 132, 64, 128, P, P, 128, None) == 3                          # rows not 16-byte aligned
    assert g(P + 8, 128, 64, 128, P, P, 128, None) == 3
    assert g(P, 128, 0, 128, P, P, 128, None) == 0                           # no rows: nothing to do


def test_basis_entry_points_reject_bad_arguments():
    L = binding.lib()
    g = L.resq_gram_accumulate
    assert g(P, 128, 10, 128, P, 120, None) == 2                             # ldc < K
    assert g(P, 128, 10, 124, P, 128, None) == 3                             # K % 8 != 0
    assert g(None, 128, 10, 128, P, 128, None) == 1
    assert g(None, 128, 0, 128, None, 128, None) == 0                        # no tokens: nothing to do
    e = L.resq_sym_eig
    assert L.resq_sym_eig_workspace_bytes(7) == 0 and L.resq_sym_eig_workspace_bytes(64) >= 2 * 64 * 64 * 8
    assert L.resq_sym_eig_workspace_bytes(8194) == 0                         # two rows must fit LDS
    assert e(P, 8194, 8194, 8, P, P, 8194, P, 1 << 40, None) == 2
    assert e(P, 63, 63, 8, P, P, 63, P, 1 << 30, None) == 2                  # odd order
    assert e(P, 64, 64, 0, P, P, 64, P, 1 << 30, None) == 2                  # no sweeps
    assert e(P, 64, 64, 8, P, P, 64, P, 100, None) == 4                      # workspace too small
    assert e(P, 64, 64, 8, P, P, 64, None, 1 << 30, None) == 1
    es = L.resq_sym_eig_static                                              # the variant on the built-in scratch area
    assert es(P, 514, 514, 8, P, P, 514, None) == 4                          # beyond its 512: nothing is launched
    assert es(P, 64, 63, 8, P, P, 64, None) == 2 and es(None, 64, 64, 8, P, P, 64, None) == 1
    assert es(P, 64, 64, 8, P + 2, P, 64, None) == 3
    r = L.resq_project_rows
    assert r(P, 1, 64, 8, 64, P, 60, 64, P, 1, 64, None) == 2                # ldu < J
    assert r(P, 1, 64, 8, 64, P, 64, 60, P, 1, 64, None) == 3                # J % 8 != 0
    assert r(P, 1, 64, 8, 64, None, 64, 64, P, 1, 64, None) == 1
    assert r(P, 1, 64, 0, 64, P, 64, 64, P, 1, 64, None) == 0


def test_binding_fails_loudly_without_device_tensors():
    import torch
    x = torch.zeros(4, 256, dtype=torch.bfloat16)
    with pytest.raises((ValueError, RuntimeError)):
        binding.resq_quantize_act(x, 32)


def test_kv_cache_entry_points_reject_bad_arguments():
    L = binding.lib()
    assert L.resq_kv_cache_row_bytes(128, 16) == 16 + 56 + 16 == 88
    assert L.resq_kv_cache_row_bytes(64, 0) == 32 + 16 and L.resq_kv_cache_row_bytes(64, 64) == 64 + 16
    assert L.resq_kv_cache_row_bytes(100, 16) == 0 and L.resq_kv_cache_row_bytes(128, 12) == 0
    assert L.resq_kv_cache_row_bytes(1024, 128) == 0 and L.resq_kv_cache_row_bytes(128, 136) == 0
    q, dq = L.resq_quantize_kv_cache, L.resq_dequantize_kv_cache
    assert q(P, 128, 10, 100, 16, P, 88, None) == 2 and q(P, 120, 10, 128, 16, P, 88, None) == 2
    assert q(P, 128, 10, 128, 16, P, 80, None) == 4                        # row_bytes too small
    assert q(None, 128, 10, 128, 16, P, 88, None) == 1 and q(P, 128, 10, 128, 16, None, 88, None) == 1
    assert q(P + 2, 128, 10, 128, 16, P, 88, None) == 3 and q(P, 128, 10, 128, 16, P + 1, 88, None) == 3
    assert q(P, 128, 10, 128, 16, P, 90, None) == 3                        # row_bytes % 4
    assert q(P, 128, 0, 128, 16, P, 88, None) == 0                         # no rows: nothing to do
    assert dq(P, 80, 10, 128, 16, P, 128, None) == 4 and dq(P, 88, 10, 128, 16, None, 128, None) == 1
    assert dq(P, 88, 10, 128, 16, P, 120, None) == 2 and dq(P, 88, 0, 128, 16, P, 128, None) == 0


def test_binding_rejects_buffers_that_do_not_fit_the_shape():
    # the kernels trust (M, N, K, r): the binding checks the buffers against them before any call
    import torch
    M, K, N, r = 4, 256, 64, 32
    act = binding.ActCodes(M, K, r, device="cpu")
    packed = torch.zeros(binding.resq_packed_weight_bytes(N, K, r), dtype=torch.uint8)
    with pytest.raises(ValueError, match="packed holds"):
        binding.resq_gemm_mixed(act, packed[:-16], N)
    with pytest.raises(ValueError, match="packed holds"):
        binding.resq_gemm_mixed(act, packed, 8 * N)                      # more channels than were packed
    with pytest.raises(ValueError, match="y must be"):
        binding.resq_gemm_mixed(act, packed, N, y=torch.zeros(M, N - 8, dtype=torch.bfloat16))
    with pytest.raises(ValueError, match="dbg_acc_hi"):
        binding.resq_gemm_mixed(act, packed, N, dbg_acc_hi=torch.zeros(M, N - 1, dtype=torch.int32))
    with pytest.raises(ValueError, match="symmetric"):
        binding.resq_gemm_mixed_asym(act, packed, N)                     # symmetric codes into the asymmetric entry
    act.asym = True
    with pytest.raises(ValueError, match="asymmetric"):
        binding.resq_gemm_mixed(act, packed, N)
    act.asym = False
    with pytest.raises(ValueError, match="even"):
        binding.resq_gemm_mixed_swiglu(act, packed, N + 1)
    with pytest.raises(ValueError, match="packed holds"):
        binding.resq_unpack_weights(packed[:100], N, K, r)
    other = binding.ActCodes(M, 2 * K, r, device="cpu")
    other.K = K                                                          # buffers of another row length
    with pytest.raises(ValueError, match="activation code buffers"):
        binding.resq_gemm_mixed(other, packed, N)


def test_quantize_gemm_mixed_rejects_bad_arguments():
    f = binding.lib().resq_quantize_gemm_mixed
    P256 = P - P % 256 + 256
    assert f(P, 512, 17, P256, 256, 512, 64, P, 256, None) == 2       # more than 16 tokens
    assert f(P, 512, 0, P256, 256, 512, 64, P, 256, None) == 2        # no token
    assert f(P, 500, 4, P256, 256, 512, 64, P, 256, None) == 2        # ldx < K
    assert f(P, 512, 4, P256, 256, 512, 64, P, 200, None) == 2        # ldy < N
    assert f(P, 65536, 16, P256, 256, 65536, 8192, P, 256, None) == 2  # 16 rows of that length do not fit LDS
    assert f(None, 512, 4, P256, 256, 512, 64, P, 256, None) == 1
    assert f(P, 512, 4, None, 256, 512, 64, P, 256, None) == 1
    assert f(P, 512, 4, P256, 256, 512, 64, None, 256, None) == 1
    assert f(P + 2, 512, 4, P256, 256, 512, 64, P, 256, None) == 3    # x not 16-byte aligned
    assert f(P, 516, 4, P256, 256, 512, 64, P, 256, None) == 3        # ldx not a multiple of 8
    assert f(P, 512, 4, P256, 256, 508, 64, P, 256, None) == 3        # K not a multiple of 8
    assert f(P, 512, 4, P256 + 16, 256, 512, 64, P, 256, None) == 3   # packed not 256-byte aligned


# shapes that take every (token groups, runs) pair of the chunked weight-streaming kernel; the GPU
# parity tests run the same list
STREAM_PLAN_SHAPES = [
    ((17, 256, 40, 32), (1, 1, 1)), ((17, 4096, 40, 512), (1, 1, 2)), ((17, 8192, 130, 1024), (1, 1, 4)),
    ((17, 53248, 16, 6656), (1, 1, 8)), ((130, 520, 4100, 64), (1, 2, 1)), ((17, 14336, 8208, 1792), (1, 2, 2)),
    ((60, 520, 16400, 64), (1, 4, 1)),
]


def test_gemm_mixed_plan():
    plan = binding.resq_gemm_mixed_plan
    # the benchmark's workloads
    assert plan(2048, 4096, 4096, 512) == (2, 0, 0)            # o_proj prefill: tiled
    assert plan(1, 28672, 8192, 1024) == (0, 1, 1)             # decode, wide layer: one run per group
    assert plan(9, 28672, 8192, 1024) == (0, 1, 1)
    assert plan(16, 28672, 8192, 1024) == (1, 1, 1)            # ... ten tokens and more: codes chunked through LDS
    assert plan(16, 8192, 8192, 1024)[0] == 0                  # not on a layer the caches hold
    assert plan(1, 4096, 4096, 512) == (0, 1, 8)               # narrow layer: reduction axis cut
    assert plan(16, 8192, 28672, 3584) == (1, 1, 4)            # code rows too long to re-read per wavefront
    assert plan(64, 28672, 8192, 1024) == (1, 4, 1)            # batched decode, wide layer: one slice
    assert plan(64, 4096, 4096, 512) == (1, 1, 2)              # ... narrow layer: four slices of 16 tokens
    assert plan(256, 4096, 4096, 512)[0] == 1                  # few tiles: the streaming kernel in slices ...
    assert plan(384, 4096, 4096, 512) == (3, 0, 2)             # ... until tiles of 64 tokens are estimated faster (192 tiles: two rings)
    assert plan(1024, 4096, 4096, 512) == (3, 0, 1)            # 512 of them: still those, one ring
    assert plan(1025, 1024, 4096, 512) == (3, 0, 2)            # above 1024 tokens always tiled
    assert plan(1025, 4096, 4096, 512) == (2, 0, 0)            # more than 512 tiles of 64 tokens: 128 x 128 tiles
    assert plan(65, 14336, 4096, 512) == (3, 0, 2)             # a wide layer: tiles from 65 tokens on
    for shape, want in STREAM_PLAN_SHAPES:
        M, K, N, r = shape
        assert plan(M, N, K, r) == want, shape
    f = binding.lib().resq_gemm_mixed_plan
    import ctypes
    a, b, c = ctypes.c_int(), ctypes.c_int(), ctypes.c_int()
    assert f(0, 256, 256, 32, ctypes.byref(a), ctypes.byref(b), ctypes.byref(c)) == 2
    assert f(4, 256, 256, 33, ctypes.byref(a), ctypes.byref(b), ctypes.byref(c)) == 2
    assert f(4, 256, 256, 32, None, ctypes.byref(b), ctypes.byref(c)) == 1
