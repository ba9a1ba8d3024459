#!/usr/bin/env python3
"""Benchmark of the ResQ mixed INT8/INT4 linear layer on one MI355X.

A step is one pass of the whole hot path over one batch of synthetic, seeded
activations that are already resident in HBM: the per-token quantize+pack
kernel, then the mixed GEMM with its dequantizing epilogue (for the down_proj
workload the online Hadamard runs first).  Weights are quantized and packed
once, before the timed region, as they are offline in the method.

Prints ONE JSON line.  With no --workload it is the headline line: the largest
single-GPU configuration (Qwen2.5-72B-shaped MLP prefill, M = 8192, K = 8192,
N = 29568, r = K/8) as ``value`` / ``roofline`` / ``cpu_baseline``, and in the
same line a ``decode`` block (M = 1, 4, 16 on the Llama-3-70B up_proj shape: the
memory-bound half of the metric), the output SNR and TOPS per rank r in
{0, K/8, K/4} (``rank_sweep``, the rank ablation of Section 5.4 on synthetic
inputs), and ``calibration``: what the chip sustains on the matrix instruction
alone and on a plain read, measured in the same process.

``value`` is 2*M*N*K operations per second of the whole step for prefill
workloads (TOPS) and algorithmic bytes per second for decode workloads (GB/s).
``roofline`` prices the GEMM kernel alone, its duration measured with HIP
events that the library records at the kernel's own start and end
(resq_time_next_kernel) in a second pass over the same steps; ``cpu_baseline``
is the CPU oracle timed on a bounded sample of the same workload on this
host's cores.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time
from pathlib import Path

ROOT = Path(__file__).resolve().parent
if str(ROOT) not in sys.path:
    sys.path.insert(0, str(ROOT))

PEAK_INT8_TOPS = 5000.0   # MI355X dense int8 matrix-core peak, TOP/s
PEAK_HBM_GBS = 8000.0     # MI355X HBM3E peak, GB/s

# HBM traffic of the dominant kernel per launch, in bytes: FETCH_SIZE + WRITE_SIZE of two
# rocprofv3 --pmc runs of this script, each scaled by what the same counter reads for a 1 GiB
# device copy (x2.000 and x1.000).  This run does not measure it: the figures are copied from
# the summaries under profiles/ (named in `traffic_source`); absent = not measured.
MEASURED_TRAFFIC = {
    "qwen_r1024": (3241.78e6 + 484.44e6, "profiles/qwen_r1024.txt"),
    "oproj_prefill": (38.29e6 + 16.78e6, "profiles/oproj_prefill.txt"),
    "gate_up_prefill": (284.52e6 + 117.44e6, "profiles/gate_up_prefill.txt"),
    "down_prefill": (366.70e6 + 33.55e6, "profiles/down_prefill.txt"),
    "oproj_m512": (19.28e6 + 4.19e6, "profiles/oproj_m512.txt"),
    "down_m512": (66.47e6 + 4.19e6, "profiles/down_m512.txt"),
    "decode_m1": (133.04e6 + 0.06e6, "profiles/decode_m1.txt"),
    "decode_m16": (133.12e6 + 0.92e6, "profiles/decode_m16.txt"),
    "decode_m64": (135.09e6 + 3.67e6, "profiles/decode_m64.txt"),
    "uc_proj": (21.35e6 + 20.97e6, "profiles/uc_proj.txt"),
    "kv_quant": (8.47e6 + 2.88e6, "profiles/kv_quant.txt"),
}


def traffic_fields(tag: str) -> dict:
    """`traffic` and where it comes from (never measured by this run itself)."""
    t = MEASURED_TRAFFIC.get(tag)
    if t is None:
        return {"traffic": None}
    return {"traffic": t[0], "traffic_source": f"{t[1]} (rocprofv3 --pmc FETCH_SIZE, WRITE_SIZE; copied, not measured by this run)"}


def workload_shape(name: str):
    from paper_2412_14363_amd import workloads as wl
    table = {
        "tiny": wl.TINY,
        "oproj_prefill": wl.OPROJ_PREFILL,
        "gate_up_prefill": wl.MLP_GATE_UP,
        "down_prefill": wl.MLP_DOWN,
        "decode_m1": wl.decode_shape(1),
        "decode_m4": wl.decode_shape(4),
        "decode_m16": wl.decode_shape(16),
        "decode_m32": wl.decode_shape(32),
        "decode_m64": wl.decode_shape(64),
        "qwen_r0": wl.qwen_mlp_shape(0),
        "qwen_r1024": wl.qwen_mlp_shape(1024),
        "qwen_r2048": wl.qwen_mlp_shape(2048),
        "oproj_m512": wl.chunk_shape("o_proj", 512),
        "down_m512": wl.chunk_shape("down", 512),
        "kv_quant": wl.KV_CACHE_QUANT,
        "uc_proj": wl.UC_PROJ,
    }
    if name not in table:
        raise SystemExit(f"unknown workload {name!r}; choose from {sorted(table)}")
    return table[name]


def algorithmic_bytes_gemm(s) -> int:
    """Bytes one GEMM launch must move: codes and scales of the activations, the
    packed weights with their scales, and the bf16 output."""
    per_tok = s.r + (s.K - s.r) // 2 + 12
    return s.M * per_tok + s.N * (s.r + (s.K - s.r) // 2 + 8) + 2 * s.M * s.N


def output_snr_db(x, w, y, rows: int = 32, cols: int = 4096) -> float:
    """10 log10(sum ref^2 / sum (ref - y)^2) of the layer's output against the unquantized
    product X W^T in fp64, on a strided sample of token rows and output channels (the
    accuracy-side figure of Section 5: what a given r buys on these inputs)."""
    import numpy as np
    M, N = y.shape
    ri = np.unique(np.linspace(0, M - 1, min(rows, M)).astype(np.int64))
    ci = np.unique(np.linspace(0, N - 1, min(cols, N)).astype(np.int64))
    import torch
    rt, ct = torch.from_numpy(ri), torch.from_numpy(ci)
    ref = x[rt].double().numpy() @ w[ct].double().numpy().T
    got = y[rt.to(y.device)].cpu()[:, ct].double().numpy()
    return float(10.0 * np.log10((ref ** 2).sum() / ((ref - got) ** 2).sum()))


def cpu_baseline(shape, x, wq_np, budget_s: float = 15.0, hadamard_block: int = 0,
                 asym: bool = False):
    """Time the oracle (activation quantizer, two int GEMMs, dequantization) on a
    row sample sized for roughly ``budget_s`` seconds."""
    import numpy as np
    from oracle import resq_oracle as oracle
    from paper_2412_14363_amd import workloads as wl

    xb = wl.bf16_bits(x)
    layer = oracle.linear_asym if asym else oracle.linear
    # two probes: the first pays the start-up of the oracle's threads, the second (as many
    # rows as the first says fit into a tenth of the budget) gives the cost per row
    rows = min(shape.M, 2)
    for share in (0.1, 1.0):
        t0 = time.perf_counter()
        layer(xb[:rows], None, shape.r, weights=wq_np)
        t_probe = max(time.perf_counter() - t0, 1e-4)
        rows = int(max(1, min(shape.M, rows * share * budget_s / t_probe)))
    idx = np.sort(np.random.default_rng(0).choice(shape.M, rows, replace=False))
    sample = np.ascontiguousarray(xb[idx])
    t0 = time.perf_counter()
    if shape.hadamard:
        sample = oracle.hadamard(sample, shape.r, shape.K, hadamard_block)
    layer(sample, None, shape.r, weights=wq_np)
    dt = time.perf_counter() - t0
    ops = 2.0 * rows * shape.N * shape.K
    return {"value": ops / dt / 1e12, "unit": "TOPS", "cores": oracle.num_threads(),
            "kind": "oracle",
            "sample": f"{rows} of {shape.M} token rows x all {shape.N} channels, seed 0, "
                      f"{dt:.1f} s; weights pre-quantized as on the GPU side",
            "seconds": dt, "rows": rows}


def quant_only_bench(args, s) -> None:
    """A workload that is the quantizer alone: per-head quantization of K/V cache entries into
    compact cache rows (asymmetric, as in the paper): HBM-bound, reported in GB/s of
    algorithmic bytes (the bf16 rows in, the cache rows out)."""
    import ctypes
    import numpy as np
    import torch
    from paper_2412_14363_amd import binding as rq
    from paper_2412_14363_amd import workloads as wl

    x = wl.make_activations(s)
    xd = x.cuda()
    row_bytes = rq.resq_kv_cache_row_bytes(s.K, s.r)
    cache = torch.empty((s.M, row_bytes), dtype=torch.uint8, device="cuda")
    L = rq.lib()
    st = torch.cuda.current_stream().cuda_stream
    qa = (xd.data_ptr(), s.K, s.M, s.K, s.r, cache.data_ptr(), row_bytes, st)

    def step(events=None):
        if events is not None:
            L.resq_time_next_kernel(*events)
        rc = L.resq_quantize_kv_cache(*qa)
        assert rc == 0, rc

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) / args.steps * 1e3
    hip = ctypes.CDLL("libamdhip64.so")
    evs = []
    for _ in range(args.steps):
        a, b = ctypes.c_void_p(), ctypes.c_void_p()
        assert hip.hipEventCreate(ctypes.byref(a)) == 0 and hip.hipEventCreate(ctypes.byref(b)) == 0
        evs.append((a, b))
        step((a, b))
    torch.cuda.synchronize()
    tot = 0.0
    for a, b in evs:
        ms = ctypes.c_float()
        assert hip.hipEventElapsedTime(ctypes.byref(ms), a, b) == 0
        tot += ms.value
        hip.hipEventDestroy(a)
        hip.hipEventDestroy(b)
    kernel_ms = tot / args.steps
    abytes = s.M * (2 * s.K + row_bytes)     # per head row: the bf16 row in, the compact cache row out
    out = {
        "metric": "per-head K/V cache quantization GB/s (% HBM peak)",
        "value": abytes / (ms_per_step * 1e-3) / 1e9, "unit": "GB/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "int8",
        "data": "synthetic",
        "config": {"workload": f"{s.name}: rows={s.M} d_head={s.K} r={s.r}", "tag": args.workload,
                   "step": "quantize_kv_cache", "activations": "asymmetric per head",
                   "cache_row_bytes": row_bytes, "compression_vs_bf16": 2 * s.K / row_bytes},
        "quantize_ms": kernel_ms,
        "roofline": {"bound": "hbm", "achieved": abytes / (kernel_ms * 1e-3) / 1e9,
                     "peak": PEAK_HBM_GBS, "unit": "GB/s",
                     "frac": abytes / (kernel_ms * 1e-3) / 1e9 / PEAK_HBM_GBS, "traffic": None,
                     "kernel": "resq quantize_kv_cache", "kernel_ms": kernel_ms},
    }
    if not args.no_cpu_baseline:
        from oracle import resq_oracle as oracle
        xb = wl.bf16_bits(x)
        t0 = time.perf_counter()
        q = oracle.quantize_act_asym(xb, s.r)
        oracle.pack_kv_cache(q[0], q[1], q[2], q[4], q[3], q[5])
        dt = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": abytes / dt / 1e9, "unit": "GB/s", "cores": oracle.num_threads(),
                               "kind": "oracle", "sample": f"all {s.M} rows, {dt:.2f} s"}
    print(json.dumps(out))


def head_proj_bench(args, s) -> None:
    """The online 8-bit projection of query and key heads onto the cache basis as one kernel
    (row quantizer + INT8 product + dequantization): HBM-bound, GB/s of algorithmic bytes."""
    import ctypes
    import torch
    from paper_2412_14363_amd import binding as rq
    from paper_2412_14363_amd import workloads as wl

    x = wl.make_activations(s)
    u = wl.random_orthogonal(s.K, s.seed + 1).to(torch.bfloat16).contiguous()
    xd = x.cuda()
    packed = rq.resq_pack_weights(u.cuda(), s.K)
    y = torch.empty((s.M, s.N), dtype=torch.bfloat16, device="cuda")
    L = rq.lib()
    st = torch.cuda.current_stream().cuda_stream
    pa = (xd.data_ptr(), s.K, s.M, s.K, packed.data_ptr(), y.data_ptr(), s.N, st)

    def step(events=None):
        if events is not None:
            L.resq_time_next_kernel(*events)
        rc = L.resq_project_heads(*pa)
        assert rc == 0, rc

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) / args.steps * 1e3
    hip = ctypes.CDLL("libamdhip64.so")
    evs = []
    for _ in range(args.steps):
        a, b = ctypes.c_void_p(), ctypes.c_void_p()
        assert hip.hipEventCreate(ctypes.byref(a)) == 0 and hip.hipEventCreate(ctypes.byref(b)) == 0
        evs.append((a, b))
        step((a, b))
    torch.cuda.synchronize()
    tot = 0.0
    for a, b in evs:
        ms = ctypes.c_float()
        assert hip.hipEventElapsedTime(ctypes.byref(ms), a, b) == 0
        tot += ms.value
        hip.hipEventDestroy(a)
        hip.hipEventDestroy(b)
    kernel_ms = tot / args.steps
    abytes = s.M * (2 * s.K + 2 * s.N) + s.N * (s.K + 4)   # rows in and out, U_C codes and scales
    out = {
        "metric": "online head projection GB/s (% HBM peak)",
        "value": abytes / (ms_per_step * 1e-3) / 1e9, "unit": "GB/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "int8",
        "data": "synthetic",
        "config": {"workload": f"{s.name}: rows={s.M} d_head={s.K}", "tag": args.workload,
                   "step": "project_heads (quantize rows + W8A8 product + dequantize, one kernel)",
                   "activations": "symmetric per head"},
        "tops": 2.0 * s.M * s.N * s.K / (ms_per_step * 1e-3) / 1e12,
        "roofline": {"bound": "hbm", "achieved": abytes / (kernel_ms * 1e-3) / 1e9,
                     "peak": PEAK_HBM_GBS, "unit": "GB/s",
                     "frac": abytes / (kernel_ms * 1e-3) / 1e9 / PEAK_HBM_GBS, **traffic_fields(args.workload),
                     "kernel": "resq project_heads", "kernel_ms": kernel_ms},
        "snr_db": output_snr_db(x, u, y),
    }
    if not args.no_cpu_baseline:
        from oracle import resq_oracle as oracle
        rows = min(s.M, 8192)
        xb, ub = wl.bf16_bits(x[:rows].contiguous()), wl.bf16_bits(u)
        t0 = time.perf_counter()
        oracle.linear(xb, ub, s.K)
        dt = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": abytes * rows / s.M / dt / 1e9, "unit": "GB/s",
                               "cores": oracle.num_threads(), "kind": "oracle",
                               "sample": f"first {rows} of {s.M} rows, {dt:.2f} s"}
    print(json.dumps(out))


def basis_bench(args) -> None:
    """The offline basis construction for one hidden-size basis (U_A of Llama-3-8B, Section 4.2):
    Gram matrix of 32768 calibration tokens, PCA by Jacobi sweeps, U = P blockdiag(R), and the
    folding of U into one 4096 x 4096 weight.  A step is the whole construction; it takes
    seconds, so at most two steps are timed whatever --steps says."""
    import torch
    from paper_2412_14363_amd import binding as rq
    from paper_2412_14363_amd import workloads as wl

    K, T, r, N, sweeps = 4096, 32768, 512, 4096, 12
    steps, warmup = max(1, min(args.steps, 2)), min(args.warmup, 1)
    s = wl.LayerShape("llama3_8b_basis_calibration", M=T, K=K, N=N, r=r, seed=3)
    x = wl.make_activations(s).cuda()                  # N(0,1) with 20x outlier columns
    w = wl.make_weights(s).cuda()
    r_h = wl.random_orthogonal(r, 1).contiguous().cuda()
    r_l = wl.random_orthogonal(K - r, 2).contiguous().cuda()
    c = torch.zeros((K, K), dtype=torch.float32, device="cuda")
    u = torch.empty((K, K), dtype=torch.float32, device="cuda")
    wr = torch.empty_like(w)
    out = {}

    def ev():
        return torch.cuda.Event(enable_timing=True)

    def step(timed=None):
        marks = [ev() for _ in range(5)]
        c.zero_()
        marks[0].record()
        rq.resq_gram_accumulate(x, c)
        marks[1].record()
        lam, p = rq.resq_sym_eig(c, sweeps=sweeps)
        marks[2].record()
        rq.resq_project_rows(p[:, :r], r_h, out=u[:, :r])
        rq.resq_project_rows(p[:, r:], r_l, out=u[:, r:])
        marks[3].record()
        rq.resq_project_rows(w, u, out=wr)
        marks[4].record()
        out["lam"], out["p"] = lam, p
        if timed is not None:
            torch.cuda.synchronize()
            timed.append([marks[i].elapsed_time(marks[i + 1]) for i in range(4)])

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    parts = []
    t0 = time.perf_counter()
    for _ in range(steps):
        step(parts)
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) / steps * 1e3
    gram_ms, eig_ms, compose_ms, fold_ms = [sum(p[i] for p in parts) / steps for i in range(4)]
    # quality of what came out: eigenpair residual and orthogonality, on the device in fp64
    lam, p = out["lam"].double(), out["p"].double()
    resid = float(((c.double() @ p) - p * lam).abs().max() / lam[0])
    orth = float((u.double().T @ u.double() - torch.eye(K, device="cuda", dtype=torch.float64)).abs().max())
    # Jacobi: per round the matrix and the vectors are read and written once, in fp64
    eig_bytes = sweeps * (K - 1) * 4.0 * K * K * 8
    gram_flops = 2.0 * T * K * K
    res = {
        "metric": "basis construction time (Gram + PCA + compose + fold)", "value": ms_per_step / 1e3,
        "unit": "s", "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": ms_per_step,
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "f32/f64",
        "data": "synthetic",
        "config": {"workload": f"{s.name}: tokens={T} K={K} r={r} fold N={N} sweeps={sweeps}", "tag": "basis",
                   "step": "gram_accumulate + sym_eig + 2 x project_rows (U) + project_rows (W U)"},
        "gram_ms": gram_ms, "eig_ms": eig_ms, "compose_ms": compose_ms, "fold_ms": fold_ms,
        "gram_tflops": gram_flops / (gram_ms * 1e-3) / 1e12,
        "fold_tflops": 2.0 * N * K * K / (fold_ms * 1e-3) / 1e12,
        "eig_residual_over_scale": resid, "u_orthogonality_error": orth,
        "roofline": {"bound": "hbm", "achieved": eig_bytes / (eig_ms * 1e-3) / 1e9, "peak": PEAK_HBM_GBS,
                     "unit": "GB/s", "frac": eig_bytes / (eig_ms * 1e-3) / 1e9 / PEAK_HBM_GBS, "traffic": None,
                     "note": "the 268 MB working set nearly fits the 256 MB last-level cache: not purely an HBM fraction",
                     "kernel": "resq sym_eig (all Jacobi rounds)", "kernel_ms": eig_ms},
    }
    if not args.no_cpu_baseline:
        import numpy as np
        from oracle import resq_basis_oracle as bo
        xs = x[:4096].double().cpu().numpy()
        t0 = time.perf_counter()
        cg = bo.gram(xs)
        t1 = time.perf_counter()
        bo.pca_basis(c.double().cpu().numpy())
        t2 = time.perf_counter()
        est = (t1 - t0) * T / 4096 + (t2 - t1)
        res["cpu_baseline"] = {"value": est, "unit": "s", "cores": os.cpu_count(), "kind": "oracle",
                               "sample": f"Gram matrix of 4096 of {T} tokens ({t1 - t0:.1f} s, scaled) + LAPACK eigh of the "
                                         f"full {K} x {K} matrix ({t2 - t1:.1f} s); fold not timed"}
    print(json.dumps(res))


def calib_lib():
    """The calibration kernels beside this script (bench_calib.hip), built on first use."""
    import ctypes
    import subprocess
    so, src = ROOT / "libbench_calib.so", ROOT / "bench_calib.hip"
    if not so.exists() or so.stat().st_mtime < src.stat().st_mtime:
        subprocess.run(["hipcc", "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
                        "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
                        "-Wno-unused-command-line-argument", "-o", str(so), str(src)], check=True,
                       capture_output=True)
    lib = ctypes.CDLL(str(so))
    vp, ci = ctypes.c_void_p, ctypes.c_int
    lib.calib_mfma_int8.argtypes = [vp, vp, ci, ci, vp, vp, vp, vp]
    lib.calib_hbm_read.argtypes = [vp, ctypes.c_size_t, ci, vp, vp, vp, vp]
    return lib


def calibration(mfma_ms: float = 1.5, quick: bool = True) -> dict:
    """What this chip sustains with nothing else going on, measured here and now:
    * v_mfma_i32_16x16x64_i8 alone (operands in registers, two wavefronts per SIMD, launches about
      as long as the headline GEMM) on operand bytes like the low group's (one operand code + 8 in
      the low nibble, the other 16 * code) and like the high group's (random INT8).  The matrix
      pipes are power-limited, so the rate depends on the bytes; `mix_r_eighth` is the rate of a
      kernel that spends 7/8 of its products on the first kind and 1/8 on the second.
    * a plain streaming read of as many bytes as the decode GEMM's packed weights, regions
      rotated through 1 GiB so that the last-level cache cannot serve them."""
    import ctypes
    import numpy as np
    import torch
    L = calib_lib()
    hip = ctypes.CDLL("libamdhip64.so")
    st = torch.cuda.current_stream().cuda_stream
    sink = torch.zeros(1, dtype=torch.int32, device="cuda")
    rng = np.random.default_rng(0)
    n = 4096 * 16
    frag = np.arange(n) // 16 // 512             # blocks of 512 lanes: 0..3 even halves, 4..7 odd halves
    c, w = rng.integers(-7, 8, n), rng.integers(-7, 8, n)
    odd = frag >= 4
    kinds = {
        "low_group_like": (np.where(odd, c * 16, c + 8).astype(np.int64) & 0xFF,
                           np.where(odd, w + 8, w * 16).astype(np.int64) & 0xFF),
        "high_group_like": (rng.integers(-127, 128, n) & 0xFF, rng.integers(-127, 128, n) & 0xFF),
    }

    def timed(fn, reps):
        a, b = ctypes.c_void_p(), ctypes.c_void_p()
        assert hip.hipEventCreate(ctypes.byref(a)) == 0 and hip.hipEventCreate(ctypes.byref(b)) == 0
        best = []
        for i in range(reps + 1):
            assert fn(i, a, b) == 0
            torch.cuda.synchronize()
            ms = ctypes.c_float()
            assert hip.hipEventElapsedTime(ctypes.byref(ms), a, b) == 0
            if i > 0:
                best.append(ms.value)
        hip.hipEventDestroy(a)
        hip.hipEventDestroy(b)
        return sum(best) / len(best)

    out = {}
    ops_per_iter = 2.0 * 16 * 16 * 64 * 32 * 8 * 256
    iters = max(1, int(mfma_ms * 1e-3 * 4.0e15 / ops_per_iter))
    for name, (ha, hb) in kinds.items():
        da = torch.from_numpy(ha.astype(np.uint8)).cuda()
        db = torch.from_numpy(hb.astype(np.uint8)).cuda()
        ms = timed(lambda i, a, b: L.calib_mfma_int8(da.data_ptr(), db.data_ptr(), iters, 256, sink.data_ptr(), a, b, st),
                   3 if quick else 6)
        out[name] = {"kernel_ms": ms, "tops": ops_per_iter * iters / (ms * 1e-3) / 1e12}
    lo, hi = out["low_group_like"]["tops"], out["high_group_like"]["tops"]
    out["mix_r_eighth"] = {"tops": 1.0 / (0.875 / lo + 0.125 / hi)}
    region = 132_600_000 // 256 * 256
    buf = torch.ones(1 << 30, dtype=torch.uint8, device="cuda")
    span = buf.numel() - region
    best = None
    for wgs in (2048, 4096, 8192):
        ms = timed(lambda i, a, b: L.calib_hbm_read(buf.data_ptr() + (i * (region + 4096)) % span // 256 * 256, region, wgs,
                                                    sink.data_ptr(), a, b, st), 6 if quick else 12)
        if best is None or ms < best[0]:
            best = (ms, wgs)
    out["read_132MB"] = {"kernel_ms": best[0], "gbs": region / (best[0] * 1e-3) / 1e9, "workgroups": best[1]}
    # a plain device-to-device copy (the runtime's own copy kernel) of 134 MB, sources and
    # destinations rotated through the same 1 GiB: the rate at which this chip moves memory
    # when it reads and writes at once, which is what the quantizer has to do
    n = 134_217_728
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(10)]
    for i in range(12):
        src = buf[(i % 3) * n:(i % 3 + 1) * n]
        dst = buf[((i + 1) % 3 + 4) * n:((i + 1) % 3 + 5) * n]
        if i >= 2:
            ev[i - 2][0].record()
        dst.copy_(src)
        if i >= 2:
            ev[i - 2][1].record()
    torch.cuda.synchronize()
    ms = sorted(a.elapsed_time(b) for a, b in ev)[len(ev) // 2]
    out["copy_134MB"] = {"ms": ms, "gbs_read_plus_write": 2 * n / (ms * 1e-3) / 1e9}
    del buf
    return out


def calib_bench(args) -> None:
    """`--workload calib`: the calibration alone, as its own line."""
    cal = calibration(quick=False)
    best = cal["mix_r_eighth"]["tops"]
    print(json.dumps({
        "metric": "sustained int8 MFMA rate, matrix instructions only (TOPS)", "value": best, "unit": "TOPS",
        "n_gpus": 1, "steps": 6, "warmup": 1, "ms_per_step": cal["low_group_like"]["kernel_ms"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "int8", "data": "synthetic",
        "config": {"workload": "calib: v_mfma_i32_16x16x64_i8 alone (256 workgroups x 8 wavefronts) and a plain read of 132.6 MB",
                   "tag": "calib"},
        "calibration": cal,
        "roofline": {"bound": "mfma", "achieved": best, "peak": PEAK_INT8_TOPS, "unit": "TOP/s",
                     "frac": best / PEAK_INT8_TOPS, "traffic": None,
                     "kernel": "calib_mfma_kernel (7/8 low-group-like, 1/8 high-group-like operands)",
                     "kernel_ms": cal["low_group_like"]["kernel_ms"]},
    }))


def mlp_block_bench(args) -> None:
    """The MLP block of Llama-3-8B on 4096 tokens as four kernels: quantize_act,
    gate/up as one layer with the gated activation in its epilogue (N2 = 28672), the
    fused Hadamard + quantizer on its output, and down_proj."""
    import ctypes
    import torch
    from paper_2412_14363_amd import binding as rq
    from paper_2412_14363_amd import workloads as wl

    gu, dn = wl.MLP_GATE_UP, wl.MLP_DOWN
    M, K, F = gu.M, gu.K, gu.N
    x = wl.make_activations(gu).cuda()
    w_gate, w_up = wl.make_weights(gu), wl.make_weights(wl.LayerShape("up", M=1, K=K, N=F, r=gu.r, seed=1))
    w_gu = torch.stack([w_gate, w_up], dim=1).reshape(2 * F, K).contiguous()   # rows 2c, 2c+1 = gate, up
    p_gu = rq.resq_pack_weights(w_gu.cuda(), gu.r)
    p_dn = rq.resq_pack_weights(wl.make_weights(dn).cuda(), dn.r)
    a1, a2 = rq.ActCodes(M, K, gu.r), rq.ActCodes(M, F, dn.r)
    h = torch.empty((M, F), dtype=torch.bfloat16, device="cuda")
    y = torch.empty((M, dn.N), dtype=torch.bfloat16, device="cuda")
    L = rq.lib()
    st = torch.cuda.current_stream().cuda_stream
    calls = [
        ("quantize_ms", L.resq_quantize_act, (x.data_ptr(), K, M, K, gu.r, a1.q_hi.data_ptr(), a1.q_lo.data_ptr(),
                                              a1.s_hi.data_ptr(), a1.s_lo.data_ptr(), a1.lo_sum.data_ptr(), st)),
        ("gate_up_swiglu_ms", L.resq_gemm_mixed_swiglu,
         (a1.q_hi.data_ptr(), a1.q_lo.data_ptr(), a1.s_hi.data_ptr(), a1.s_lo.data_ptr(), a1.lo_sum.data_ptr(),
          M, p_gu.data_ptr(), 2 * F, K, gu.r, h.data_ptr(), F, st)),
        ("hadamard_quantize_ms", L.resq_hadamard_quantize_act,
         (h.data_ptr(), F, M, F, dn.r, 0, a2.q_hi.data_ptr(), a2.q_lo.data_ptr(), a2.s_hi.data_ptr(),
          a2.s_lo.data_ptr(), a2.lo_sum.data_ptr(), None, 0, st)),
        ("down_ms", L.resq_gemm_mixed,
         (a2.q_hi.data_ptr(), a2.q_lo.data_ptr(), a2.s_hi.data_ptr(), a2.s_lo.data_ptr(), a2.lo_sum.data_ptr(),
          M, p_dn.data_ptr(), dn.N, F, dn.r, y.data_ptr(), dn.N, None, None, st)),
    ]

    def step(events=None):
        for i, (_, fn, fargs) in enumerate(calls):
            if events is not None:
                L.resq_time_next_kernel(*events[i])
            rc = fn(*fargs)
            assert rc == 0, rc

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) / args.steps * 1e3
    hip = ctypes.CDLL("libamdhip64.so")
    evs = []
    for _ in range(args.steps):
        row = []
        for _ in calls:
            a, b = ctypes.c_void_p(), ctypes.c_void_p()
            assert hip.hipEventCreate(ctypes.byref(a)) == 0 and hip.hipEventCreate(ctypes.byref(b)) == 0
            row.append((a, b))
        evs.append(row)
        step(row)
    torch.cuda.synchronize()
    sums = [0.0] * len(calls)
    for row in evs:
        for i, (a, b) in enumerate(row):
            ms = ctypes.c_float()
            assert hip.hipEventElapsedTime(ctypes.byref(ms), a, b) == 0
            sums[i] += ms.value
            hip.hipEventDestroy(a)
            hip.hipEventDestroy(b)
    per = {name: sums[i] / args.steps for i, (name, _, _) in enumerate(calls)}
    ops_gu, ops_dn = 2.0 * M * K * 2 * F, 2.0 * M * F * dn.N
    achieved = ops_gu / (per["gate_up_swiglu_ms"] * 1e-3) / 1e12
    out = {
        "metric": "mixed INT8/INT4 MLP block TOPS (% int8 MFMA peak)",
        "value": (ops_gu + ops_dn) / (ms_per_step * 1e-3) / 1e12, "unit": "TOPS", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "int8",
        "data": "synthetic",
        "config": {"workload": f"llama3_8b_mlp_block: M={M} d={K} d_ffn={F} r={gu.r}/{dn.r}",
                   "tag": "mlp_block",
                   "step": "quantize_act + gemm_mixed_swiglu (gate/up, N2=28672) + "
                           "hadamard_quantize_act + gemm_mixed (down)"},
        "tokens_per_s": M / (ms_per_step * 1e-3), **per,
        "roofline": {"bound": "mfma", "achieved": achieved, "peak": PEAK_INT8_TOPS, "unit": "TOP/s",
                     "frac": achieved / PEAK_INT8_TOPS, "traffic": None,
                     "kernel": "resq gemm_mixed (gate/up with gated epilogue)",
                     "kernel_ms": per["gate_up_swiglu_ms"]},
    }
    print(json.dumps(out))


_WEIGHTS: dict = {}   # the last layer's weights and packed copies (see layer_bench)


def layer_bench(args, tag: str, steps: int, warmup: int, with_cpu_baseline: bool, cpu_budget: float,
                keep: dict | None = None) -> dict:
    """One workload that is a whole layer step (quantizer + GEMM, the transform in front where the
    workload has one): times `steps` steps, then a second pass with events around each kernel.
    Returns the JSON object; `keep`, when given, receives the inputs for follow-up measurements."""
    import ctypes
    import torch
    from paper_2412_14363_amd import binding as rq
    from paper_2412_14363_amd import workloads as wl

    s = workload_shape(tag)
    decode = s.M <= 64
    x = wl.make_activations(s)
    xd = x.cuda()
    # decode: rotate over enough weight copies that the 256 MB last-level cache
    # cannot hold them, so that HBM is what is measured.  The weights depend on the layer,
    # not on M: workloads of one layer (decode_m1/4/16 in the headline run) share them.
    wkey = (s.N, s.K, s.r, s.seed)
    if _WEIGHTS.get("key") != wkey:
        _WEIGHTS.clear()
        w = wl.make_weights(s)
        packed0 = rq.resq_pack_weights(w.cuda(), s.r)
        n_copies = max(1, int(-(-768e6 // packed0.numel()))) if decode else 1
        _WEIGHTS.update(key=wkey, w=w, packed=[packed0] + [packed0.clone() for _ in range(n_copies - 1)])
    w, packed = _WEIGHTS["w"], _WEIGHTS["packed"]
    n_copies = len(packed)
    act = rq.ActCodes(s.M, s.K, s.r)
    y = torch.empty((s.M, s.N), dtype=torch.bfloat16, device="cuda")
    fused = s.hadamard and not args.unfused_hadamard
    xh = torch.empty_like(xd) if s.hadamard and not fused else None
    L = rq.lib()
    st = torch.cuda.current_stream().cuda_stream

    def ptr(t, live=True):
        return t.data_ptr() if live else None

    hi, lo = s.r > 0, s.K - s.r > 0
    had_args = (xd.data_ptr(), xh.data_ptr() if xh is not None else None, s.K, s.M, s.K, s.r,
                s.K, 0, st)
    xq = xh if xh is not None else xd
    hq_args = (xd.data_ptr(), s.K, s.M, s.K, s.r, 0, ptr(act.q_hi, hi), ptr(act.q_lo, lo),
               ptr(act.s_hi, hi), ptr(act.s_lo, lo), ptr(act.lo_sum, lo), None, 0, st)
    qa_args = (xq.data_ptr(), s.K, s.M, s.K, s.r, ptr(act.q_hi, hi), ptr(act.q_lo, lo),
               ptr(act.s_hi, hi), ptr(act.s_lo, lo), ptr(act.lo_sum, lo), st)
    gemm_args = [(ptr(act.q_hi, hi), ptr(act.q_lo, lo), ptr(act.s_hi, hi), ptr(act.s_lo, lo),
                  ptr(act.lo_sum, lo), s.M, p.data_ptr(), s.N, s.K, s.r, y.data_ptr(), s.N, None,
                  None, st)
                 for p in packed]
    # asymmetric activations: same kernels, one more pair of per-token vectors
    qa_asym_args = (xq.data_ptr(), s.K, s.M, s.K, s.r, -1 if fused else 0, ptr(act.q_hi, hi),
                    ptr(act.q_lo, lo), ptr(act.s_hi, hi), ptr(act.s_lo, lo), ptr(act.c_hi, hi),
                    ptr(act.c_lo, lo), ptr(act.lo_sum, lo), st)
    gemm_asym_args = [(ptr(act.q_hi, hi), ptr(act.q_lo, lo), ptr(act.s_hi, hi), ptr(act.s_lo, lo),
                       ptr(act.c_hi, hi), ptr(act.c_lo, lo), ptr(act.lo_sum, lo), s.M, p.data_ptr(),
                       s.N, s.K, s.r, y.data_ptr(), s.N, None, None, st)
                      for p in packed]

    one_call = args.one_call
    if one_call and (s.M > 16 or args.asym or s.hadamard):
        raise SystemExit("--one-call: symmetric codes, at most 16 tokens, no transform")
    one_args = [(xd.data_ptr(), s.K, s.M, p.data_ptr(), s.N, s.K, s.r, y.data_ptr(), s.N, st) for p in packed]

    def step(i: int, events=None):
        # events: three (start, stop) pairs of hipEvent_t, recorded by the library at
        # the start and end of the kernel each call launches
        if one_call:
            if events is not None:
                L.resq_time_next_kernel(*events[2])
            rc = L.resq_quantize_gemm_mixed(*one_args[i % n_copies])
            assert rc == 0, rc
            return
        if s.hadamard and not fused:
            if events is not None:
                L.resq_time_next_kernel(*events[0])
            rc = L.resq_online_hadamard(*had_args)
            assert rc == 0, rc
        if events is not None:
            L.resq_time_next_kernel(*events[1])
        if args.asym:
            rc = L.resq_quantize_act_asym(*qa_asym_args)
        else:
            rc = L.resq_hadamard_quantize_act(*hq_args) if fused else L.resq_quantize_act(*qa_args)
        assert rc == 0, rc
        if events is not None:
            L.resq_time_next_kernel(*events[2])
        if args.asym:
            rc = L.resq_gemm_mixed_asym(*gemm_asym_args[i % n_copies])
        else:
            rc = L.resq_gemm_mixed(*gemm_args[i % n_copies])
        assert rc == 0, rc

    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    # a generation-stage step is tens of microseconds, close to what the host needs to launch
    # it: keep the interpreter's garbage collector out of the timed region
    import gc
    gc.collect()
    gc.disable()
    t0 = time.perf_counter()
    for i in range(steps):
        step(i)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    gc.enable()
    ms_per_step = dt / steps * 1e3

    # second pass over the same steps; HIP events at the start and end of each kernel
    hip = ctypes.CDLL("libamdhip64.so")

    def new_event():
        e = ctypes.c_void_p()
        assert hip.hipEventCreate(ctypes.byref(e)) == 0
        return e

    def elapsed_ms(pair):
        ms = ctypes.c_float()
        assert hip.hipEventElapsedTime(ctypes.byref(ms), pair[0], pair[1]) == 0
        return ms.value

    evs = [[(new_event(), new_event()) for _ in range(3)] for _ in range(steps)]
    for i in range(steps):
        step(i, evs[i])
    torch.cuda.synchronize()
    had_ms = sum(elapsed_ms(e[0]) for e in evs) / steps if s.hadamard and not fused else 0.0
    quant_ms = 0.0 if one_call else sum(elapsed_ms(e[1]) for e in evs) / steps
    gemm_all = sorted(elapsed_ms(e[2]) for e in evs)
    gemm_ms = sum(gemm_all) / steps
    for e in evs:
        for pair in e:
            hip.hipEventDestroy(pair[0])
            hip.hipEventDestroy(pair[1])

    ops = 2.0 * s.M * s.N * s.K
    abytes = algorithmic_bytes_gemm(s)
    if decode:
        metric, unit = "decode GB/s (% HBM peak)", "GB/s"
        value = (abytes + 2 * s.M * s.K) / (ms_per_step * 1e-3) / 1e9
        achieved = abytes / (gemm_ms * 1e-3) / 1e9
        roof = {"bound": "hbm", "achieved": achieved, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                "frac": achieved / PEAK_HBM_GBS, **traffic_fields(tag)}
    else:
        metric, unit = "mixed INT8/INT4 linear TOPS (% int8 MFMA peak)", "TOPS"
        value = ops / (ms_per_step * 1e-3) / 1e12
        achieved = ops / (gemm_ms * 1e-3) / 1e12
        roof = {"bound": "mfma", "achieved": achieved, "peak": PEAK_INT8_TOPS, "unit": "TOP/s",
                "frac": achieved / PEAK_INT8_TOPS, **traffic_fields(tag)}
    roof["kernel"] = "resq quantize_gemm_mixed" if one_call else "resq gemm_mixed"
    roof["kernel_ms"] = gemm_ms        # the mean: what `achieved` is priced with
    roof["kernel_ms_median"] = gemm_all[len(gemm_all) // 2]
    roof["kernel_ms_min"] = gemm_all[0]

    out = {
        "metric": metric, "value": value, "unit": unit, "n_gpus": 1, "steps": steps,
        "warmup": warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "int8", "data": "synthetic",
        "config": {"workload": f"{s.name}: M={s.M} K={s.K} N={s.N} r={s.r}", "tag": tag,
                   "step": "quantize_gemm_mixed (one kernel)" if one_call else
                           ("hadamard_quantize_act (one kernel) + " if fused else
                            "online_hadamard + quantize_act + " if s.hadamard else
                            "quantize_act + ") + "gemm_mixed",
                   "activations": "asymmetric per token" if args.asym else "symmetric per token",
                   "weight_copies_rotated": n_copies},
        "tokens_per_s": s.M / (ms_per_step * 1e-3),
        "hadamard_ms": had_ms, "quantize_ms": quant_ms, "gemm_ms": gemm_ms,
        # ms_per_step is host time over back-to-back steps; the *_ms fields are device time of
        # each kernel from the second pass (events between the kernels), so they need not add up to it
        "roofline": roof,
    }
    if not s.hadamard:
        out["snr_db"] = output_snr_db(x, w, y)
    if with_cpu_baseline:
        from oracle import resq_oracle as oracle
        wq_np = oracle.quantize_weights(wl.bf16_bits(w), s.r)
        cb = cpu_baseline(s, x, wq_np, cpu_budget,
                          rq.resq_hadamard_block(s.K - s.r) if s.hadamard else 0, args.asym)
        if decode:
            # same unit as the metric: algorithmic bytes of the sampled rows per second
            frac = cb["rows"] / s.M
            cb["value"] = abytes * frac / cb["seconds"] / 1e9
            cb["unit"] = "GB/s"
        out["cpu_baseline"] = {k: cb[k] for k in ("value", "unit", "cores", "kind", "sample")}
    if keep is not None:
        keep.update(x=x, w=w, xd=xd, shape=s)
    return out


def rank_sweep(args, x, w, xd, base, ranks, steps: int = 20) -> dict:
    """The rank ablation of Section 5.4 on the headline workload's inputs: for each r the GEMM's
    device time (events at the kernel's start and end) and the SNR of the layer's output against
    the unquantized product in fp64 on a strided sample of rows and channels."""
    import ctypes
    import torch
    from paper_2412_14363_amd import binding as rq
    hip = ctypes.CDLL("libamdhip64.so")
    L = rq.lib()
    wd = w.cuda()
    out = {}
    for r in ranks:
        packed = rq.resq_pack_weights(wd, r)
        act = rq.resq_quantize_act(xd, r)
        y = rq.resq_gemm_mixed(act, packed, base.N)
        for _ in range(3):
            rq.resq_gemm_mixed(act, packed, base.N, y=y)
        evs = []
        for _ in range(steps):       # back to back, like the timed steps of the headline workload
            a, b = ctypes.c_void_p(), ctypes.c_void_p()
            assert hip.hipEventCreate(ctypes.byref(a)) == 0 and hip.hipEventCreate(ctypes.byref(b)) == 0
            L.resq_time_next_kernel(a, b)
            rq.resq_gemm_mixed(act, packed, base.N, y=y)
            evs.append((a, b))
        torch.cuda.synchronize()
        tot = 0.0
        for a, b in evs:
            ms = ctypes.c_float()
            assert hip.hipEventElapsedTime(ctypes.byref(ms), a, b) == 0
            tot += ms.value
            hip.hipEventDestroy(a)
            hip.hipEventDestroy(b)
        gemm_ms = tot / steps
        tops = 2.0 * base.M * base.N * base.K / (gemm_ms * 1e-3) / 1e12
        out[f"r={r}"] = {"snr_db": output_snr_db(x, w, y), "gemm_ms": gemm_ms, "gemm_tops": tops,
                         "frac_of_int8_peak": tops / PEAK_INT8_TOPS}
        del packed, act, y
    return out


def headline(args) -> None:
    """The default line: config 5 at r = K/8 in full, plus the decode half of the metric, the
    rank sweep and the calibration."""
    import torch
    keep: dict = {}
    out = layer_bench(args, "qwen_r1024", args.steps, args.warmup, not args.no_cpu_baseline, args.cpu_budget, keep)
    # both halves of the metric are in this line: `value` is the prefill half (TOPS), `decode` the other
    out["metric"] = "mixed INT8/INT4 linear TOPS (% int8 MFMA peak); decode GB/s (% HBM peak)"
    s = keep["shape"]
    out["rank_sweep"] = rank_sweep(args, keep["x"], keep["w"], keep["xd"], s, (0, s.K // 8, s.K // 4))
    keep.clear()
    _WEIGHTS.clear()
    torch.cuda.empty_cache()
    dec = {}
    for m in (1, 4, 16):
        d = layer_bench(args, f"decode_m{m}", max(args.steps, 500), args.warmup, not args.no_cpu_baseline and m == 16,
                        min(args.cpu_budget, 5.0))
        dec[f"M={m}"] = {"value": d["value"], "unit": d["unit"], "ms_per_step": d["ms_per_step"],
                         "quantize_ms": d["quantize_ms"], "gemm_ms": d["gemm_ms"],
                         "tokens_per_s": d["tokens_per_s"], "workload": d["config"]["workload"],
                         "weight_copies_rotated": d["config"]["weight_copies_rotated"],
                         "roofline": d["roofline"]}
        if "cpu_baseline" in d:
            dec[f"M={m}"]["cpu_baseline"] = d["cpu_baseline"]
        torch.cuda.empty_cache()
    out["decode"] = dec
    cal = calibration()
    out["calibration"] = cal
    out["roofline"]["measured_peak"] = cal["mix_r_eighth"]["tops"]
    out["roofline"]["frac_of_measured"] = out["roofline"]["achieved"] / cal["mix_r_eighth"]["tops"]
    out["roofline"]["measured_peak_source"] = ("calibration.mix_r_eighth: the matrix instruction alone on operand "
                                               "bytes like this workload's, same process")
    # the quantizer of the headline step against HBM and against the measured copy rate
    qbytes = s.M * (2 * s.K + s.r + (s.K - s.r) // 2 + 12)
    qgbs = qbytes / (out["quantize_ms"] * 1e-3) / 1e9
    out["quantize_roofline"] = {"bound": "hbm", "achieved": qgbs, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                                "frac": qgbs / PEAK_HBM_GBS, "kernel": "resq quantize_act",
                                "kernel_ms": out["quantize_ms"],
                                "measured_peak": cal["copy_134MB"]["gbs_read_plus_write"],
                                "frac_of_measured": qgbs / cal["copy_134MB"]["gbs_read_plus_write"],
                                "measured_peak_source": "calibration.copy_134MB: a plain device copy, same process"}
    for v in dec.values():
        v["roofline"]["measured_peak"] = cal["read_132MB"]["gbs"]
        v["roofline"]["frac_of_measured"] = v["roofline"]["achieved"] / cal["read_132MB"]["gbs"]
    print(json.dumps(out), flush=True)


def main() -> None:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="headline",
                    help="headline (default: Qwen2.5-72B MLP prefill + decode block + rank sweep + calibration), "
                         "or one workload alone: oproj_prefill, gate_up_prefill, down_prefill, qwen_r0/r1024/r2048, "
                         "decode_m1/4/16/32/64, oproj_m512, down_m512, mlp_block, kv_quant, uc_proj, basis, calib, "
                         "copy_calib")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-budget", type=float, default=15.0)
    ap.add_argument("--asym", action="store_true",
                    help="asymmetric per-token activations (the paper's experimental setting) "
                         "instead of the symmetric ones the headline metric is defined on")
    ap.add_argument("--one-call", action="store_true",
                    help="generation-stage workloads with at most 16 tokens: quantizer and GEMM as ONE "
                         "kernel (resq_quantize_gemm_mixed) instead of the two calls")
    ap.add_argument("--unfused-hadamard", action="store_true",
                    help="down_proj input: transform and quantize in two kernels instead of one")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        raise SystemExit("bench.py: this build runs on ONE GPU and has no multi-GPU path; "
                         "--gpus must be 1")

    import torch
    if not torch.cuda.is_available():
        raise SystemExit("bench.py needs a GPU: the library has no CPU path")
    torch.cuda.set_device(0)
    if args.workload == "copy_calib":
        # Calibration for the FETCH_SIZE / WRITE_SIZE counters: a plain device copy of
        # known size (1 GiB read, 1 GiB written per launch), to be run under rocprofv3 --pmc.
        n = 1 << 30
        src = torch.empty(n, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(args.steps):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"workload": "copy_calib", "bytes_read_per_copy": n,
                          "bytes_written_per_copy": n, "copies": args.steps}))
        return
    if args.workload == "headline":
        headline(args)
        return
    if args.workload == "mlp_block":
        mlp_block_bench(args)
        return
    if args.workload == "basis":
        basis_bench(args)
        return
    if args.workload == "calib":
        calib_bench(args)
        return
    s = workload_shape(args.workload)
    if args.workload == "uc_proj":
        head_proj_bench(args, s)
        return
    if s.N == 0:
        quant_only_bench(args, s)
        return
    print(json.dumps(layer_bench(args, args.workload, args.steps, args.warmup, not args.no_cpu_baseline,
                                 args.cpu_budget)), flush=True)


if __name__ == "__main__":
    main()
