#!/usr/bin/env python3
"""Benchmark of the ResQ mixed INT8/INT4 linear layer on one MI355X.

A step is one pass of the whole hot path over one batch of synthetic, seeded
activations that are already resident in HBM: the per-token quantize+pack
kernel, then the mixed GEMM with its dequantizing epilogue (for the down_proj
workload the online Hadamard runs first).  Weights are quantized and packed
once, before the timed region, as they are offline in the method.

Prints ONE JSON line.  ``value`` is 2*M*N*K operations per second of the whole
step for prefill workloads (TOPS) and algorithmic bytes per second for decode
workloads (GB/s).  ``roofline`` prices the GEMM kernel alone, its duration
measured with HIP events that the library records at the kernel's own start and
end (resq_time_next_kernel) in a second pass over the same steps;
``cpu_baseline`` is the CPU oracle timed on a bounded sample of the same
workload on this host's cores.
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

# HBM traffic of the GEMM kernel per launch, in bytes: FETCH_SIZE + WRITE_SIZE of two
# rocprofv3 --pmc runs, each scaled by what the same counter reads for a 1 GiB device copy
# (x2.000 and x1.000; the summaries are under profiles/).  Absent = not measured.
MEASURED_TRAFFIC = {
    "oproj_prefill": 38.42e6 + 16.78e6,
    "gate_up_prefill": 265.88e6 + 117.44e6,
    "down_prefill": 265.08e6 + 33.55e6,
    "qwen_r1024": 2194.69e6 + 484.44e6,
    "oproj_m512": 19.27e6 + 4.19e6,
    "down_m512": 66.45e6 + 4.19e6,
    "decode_m16": 133.61e6 + 0.92e6,
    "decode_m64": 134.98e6 + 3.67e6,
    "kv_quant": 8.47e6 + 9.04e6,
    "uc_proj": 21.35e6 + 20.97e6,
}


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
    """A workload that is the quantizer alone (per-head quantization of K/V cache entries,
    asymmetric as in the paper): HBM-bound, reported in GB/s of algorithmic bytes."""
    import ctypes
    import numpy as np
    import torch
    from paper_2412_14363_amd import binding as rq
    from paper_2412_14363_amd import workloads as wl

    x = wl.make_activations(s)
    xd = x.cuda()
    act = rq.ActCodes(s.M, s.K, s.r)
    L = rq.lib()
    st = torch.cuda.current_stream().cuda_stream
    qa = (xd.data_ptr(), s.K, s.M, s.K, s.r, 0, act.q_hi.data_ptr(), act.q_lo.data_ptr(),
          act.s_hi.data_ptr(), act.s_lo.data_ptr(), act.c_hi.data_ptr(), act.c_lo.data_ptr(),
          act.lo_sum.data_ptr(), st)

    def step(events=None):
        if events is not None:
            L.resq_time_next_kernel(*events)
        rc = L.resq_quantize_act_asym(*qa)
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
    # per row: the bf16 row in; padded codes, two scales, two offsets and one sum out
    abytes = s.M * (2 * s.K + act.ld_hi + act.ld_lo + 20)
    out = {
        "metric": "per-head K/V cache quantization GB/s (% HBM peak)",
        "value": abytes / (ms_per_step * 1e-3) / 1e9, "unit": "GB/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "int8",
        "data": "synthetic",
        "config": {"workload": f"{s.name}: rows={s.M} d_head={s.K} r={s.r}", "tag": args.workload,
                   "step": "quantize_act_asym", "activations": "asymmetric per head"},
        "quantize_ms": kernel_ms,
        "roofline": {"bound": "hbm", "achieved": abytes / (kernel_ms * 1e-3) / 1e9,
                     "peak": PEAK_HBM_GBS, "unit": "GB/s",
                     "frac": abytes / (kernel_ms * 1e-3) / 1e9 / PEAK_HBM_GBS, "traffic": MEASURED_TRAFFIC.get(args.workload),
                     "kernel": "resq quantize_act (short rows)", "kernel_ms": kernel_ms},
    }
    if not args.no_cpu_baseline:
        from oracle import resq_oracle as oracle
        xb = wl.bf16_bits(x)
        t0 = time.perf_counter()
        oracle.quantize_act_asym(xb, s.r)
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
                     "frac": abytes / (kernel_ms * 1e-3) / 1e9 / PEAK_HBM_GBS, "traffic": MEASURED_TRAFFIC.get(args.workload),
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


def mfma_ceiling_bench(args) -> None:
    """Not a workload of the method: what this chip sustains on v_mfma_i32_32x32x32_i8 alone,
    for operand bytes like the GEMM's (all zero; INT4 codes widened to the high nibble and the
    offset low nibble; random INT8 codes) and launches about as long as the GEMM's.  The matrix
    pipes are power-limited, so this, not the nominal 5 POPS, is what the GEMM can approach."""
    import ctypes
    import numpy as np
    import torch
    from paper_2412_14363_amd import binding as rq

    L = rq.lib()
    st = torch.cuda.current_stream().cuda_stream
    rng = np.random.default_rng(0)
    kinds = {
        "zeros": np.zeros(2048 * 16, np.uint8),
        "int4_widened": np.where(np.arange(2048 * 16) % 32 < 16,
                                 (rng.integers(-7, 8, 2048 * 16) * 16) & 0xFF,          # weight-like: code << 4
                                 rng.integers(1, 16, 2048 * 16)).astype(np.uint8),      # activation-like: code + 8
        "random_int8": (rng.integers(-127, 128, 2048 * 16) & 0xFF).astype(np.uint8),
    }
    sink = torch.zeros(1, dtype=torch.int32, device="cuda")
    hip = ctypes.CDLL("libamdhip64.so")
    wgs = 256                                  # one workgroup of four wavefronts per compute unit, as the GEMM
    out_rows = {}
    for name, host in kinds.items():
        dev = torch.from_numpy(host).cuda()
        for label, iters in (("35us", 290), ("200us", 1650), ("1500us", 12400)):
            for _ in range(2):
                assert L.resq_probe_mfma_int8(dev.data_ptr(), iters, wgs, sink.data_ptr(), st) == 0
            torch.cuda.synchronize()
            a, b = ctypes.c_void_p(), ctypes.c_void_p()
            assert hip.hipEventCreate(ctypes.byref(a)) == 0 and hip.hipEventCreate(ctypes.byref(b)) == 0
            tot, reps = 0.0, 5
            for _ in range(reps):
                L.resq_time_next_kernel(a, b)
                assert L.resq_probe_mfma_int8(dev.data_ptr(), iters, wgs, sink.data_ptr(), st) == 0
                torch.cuda.synchronize()
                ms = ctypes.c_float()
                assert hip.hipEventElapsedTime(ctypes.byref(ms), a, b) == 0
                tot += ms.value
            hip.hipEventDestroy(a)
            hip.hipEventDestroy(b)
            ms_avg = tot / reps
            ops = 2.0 * 32 ** 3 * 8 * 4 * iters * wgs
            out_rows[f"{name}_{label}"] = {"kernel_ms": ms_avg, "tops": ops / (ms_avg * 1e-3) / 1e12}
    best = out_rows["int4_widened_200us"]["tops"]
    print(json.dumps({
        "metric": "sustained int8 MFMA rate, matrix instructions only (TOPS)", "value": best, "unit": "TOPS",
        "n_gpus": 1, "steps": 5, "warmup": 2, "ms_per_step": out_rows["int4_widened_200us"]["kernel_ms"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "int8", "data": "synthetic",
        "config": {"workload": "mfma_ceiling: 256 workgroups x 4 wavefronts, 8 accumulator tiles each", "tag": "mfma_ceiling"},
        "rates": out_rows,
        "roofline": {"bound": "mfma", "achieved": best, "peak": PEAK_INT8_TOPS, "unit": "TOP/s",
                     "frac": best / PEAK_INT8_TOPS, "traffic": None, "kernel": "resq probe_mfma_int8 (int4_widened, 200 us)",
                     "kernel_ms": out_rows["int4_widened_200us"]["kernel_ms"]},
    }))


def hbm_ceiling_bench(args) -> None:
    """Not a workload of the method: the rate of a plain streaming read, for a launch that reads
    as many bytes as the decode GEMM does (the 132 MB of packed weights of the Llama-3-70B up_proj,
    rotated over regions that the last-level cache cannot hold) and for one long read of 3 GiB."""
    import ctypes
    import torch
    from paper_2412_14363_amd import binding as rq

    L = rq.lib()
    st = torch.cuda.current_stream().cuda_stream
    hip = ctypes.CDLL("libamdhip64.so")
    region = 132_600_000 // 256 * 256
    buf = torch.ones(3 << 30, dtype=torch.uint8, device="cuda")
    sink = torch.zeros(1, dtype=torch.int32, device="cuda")
    rows = {}

    def timed(offset, nbytes, wgs, reps):
        a, b = ctypes.c_void_p(), ctypes.c_void_p()
        assert hip.hipEventCreate(ctypes.byref(a)) == 0 and hip.hipEventCreate(ctypes.byref(b)) == 0
        tot = 0.0
        for i in range(reps + 2):
            off = (offset + i * (region + 4096)) % (buf.numel() - nbytes) // 256 * 256 if nbytes == region else 0
            L.resq_time_next_kernel(a, b)
            assert L.resq_probe_hbm_read(buf.data_ptr() + off, nbytes, wgs, sink.data_ptr(), st) == 0
            torch.cuda.synchronize()
            ms = ctypes.c_float()
            assert hip.hipEventElapsedTime(ctypes.byref(ms), a, b) == 0
            if i >= 2:
                tot += ms.value
        hip.hipEventDestroy(a)
        hip.hipEventDestroy(b)
        return tot / reps

    for wgs in (1024, 2048, 4096, 8192):
        ms = timed(0, region, wgs, 12)
        rows[f"read_132MB_{wgs}wg"] = {"kernel_ms": ms, "gbs": region / (ms * 1e-3) / 1e9}
    for wgs in (4096, 16384):
        ms = timed(0, buf.numel(), wgs, 3)
        rows[f"read_3GiB_{wgs}wg"] = {"kernel_ms": ms, "gbs": buf.numel() / (ms * 1e-3) / 1e9}
    best = max(v["gbs"] for k, v in rows.items() if k.startswith("read_132MB"))
    print(json.dumps({
        "metric": "plain streaming read GB/s", "value": best, "unit": "GB/s", "n_gpus": 1, "steps": 12, "warmup": 2,
        "ms_per_step": region / best / 1e6, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u8", "data": "synthetic",
        "config": {"workload": "hbm_ceiling: one launch reads 132.6 MB (regions rotated through 3 GiB), or all 3 GiB", "tag": "hbm_ceiling"},
        "rates": rows,
        "roofline": {"bound": "hbm", "achieved": best, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": best / PEAK_HBM_GBS,
                     "traffic": None, "kernel": "resq probe_hbm_read (132.6 MB per launch)", "kernel_ms": region / best / 1e6},
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


def main() -> None:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="oproj_prefill")
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
    from paper_2412_14363_amd import binding as rq
    from paper_2412_14363_amd import workloads as wl

    if args.workload == "mlp_block":
        mlp_block_bench(args)
        return
    if args.workload == "basis":
        basis_bench(args)
        return
    if args.workload == "mfma_ceiling":
        mfma_ceiling_bench(args)
        return
    if args.workload == "hbm_ceiling":
        hbm_ceiling_bench(args)
        return
    s = workload_shape(args.workload)
    if args.workload == "uc_proj":
        head_proj_bench(args, s)
        return
    if s.N == 0:
        quant_only_bench(args, s)
        return
    decode = s.M <= 64
    x = wl.make_activations(s)
    w = wl.make_weights(s)
    xd = x.cuda()
    # decode: rotate over enough weight copies that the 256 MB last-level cache
    # cannot hold them, so that HBM is what is measured
    n_copies = 1
    packed0 = rq.resq_pack_weights(w.cuda(), s.r)
    if decode:
        n_copies = max(1, int(-(-768e6 // packed0.numel())))
    packed = [packed0] + [packed0.clone() for _ in range(n_copies - 1)]
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

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3

    # second pass over the same steps; HIP events at the start and end of each kernel
    import ctypes
    hip = ctypes.CDLL("libamdhip64.so")

    def new_event():
        e = ctypes.c_void_p()
        assert hip.hipEventCreate(ctypes.byref(e)) == 0
        return e

    def elapsed_ms(pair):
        ms = ctypes.c_float()
        assert hip.hipEventElapsedTime(ctypes.byref(ms), pair[0], pair[1]) == 0
        return ms.value

    evs = [[(new_event(), new_event()) for _ in range(3)] for _ in range(args.steps)]
    for i in range(args.steps):
        step(i, evs[i])
    torch.cuda.synchronize()
    had_ms = sum(elapsed_ms(e[0]) for e in evs) / args.steps if s.hadamard and not fused else 0.0
    quant_ms = 0.0 if one_call else sum(elapsed_ms(e[1]) for e in evs) / args.steps
    gemm_all = sorted(elapsed_ms(e[2]) for e in evs)
    gemm_ms = sum(gemm_all) / args.steps
    for e in evs:
        for pair in e:
            hip.hipEventDestroy(pair[0])
            hip.hipEventDestroy(pair[1])

    ops = 2.0 * s.M * s.N * s.K
    abytes = algorithmic_bytes_gemm(s)
    traffic = MEASURED_TRAFFIC.get(args.workload)
    if decode:
        metric, unit = "decode GB/s (% HBM peak)", "GB/s"
        value = (abytes + 2 * s.M * s.K) / (ms_per_step * 1e-3) / 1e9
        achieved = abytes / (gemm_ms * 1e-3) / 1e9
        roof = {"bound": "hbm", "achieved": achieved, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                "frac": achieved / PEAK_HBM_GBS, "traffic": traffic}
    else:
        metric, unit = "mixed INT8/INT4 linear TOPS (% int8 MFMA peak)", "TOPS"
        value = ops / (ms_per_step * 1e-3) / 1e12
        achieved = ops / (gemm_ms * 1e-3) / 1e12
        roof = {"bound": "mfma", "achieved": achieved, "peak": PEAK_INT8_TOPS, "unit": "TOP/s",
                "frac": achieved / PEAK_INT8_TOPS, "traffic": traffic}
    roof["kernel"] = "resq quantize_gemm_mixed" if one_call else "resq gemm_mixed"
    roof["kernel_ms"] = gemm_ms        # the mean: what `achieved` is priced with
    roof["kernel_ms_median"] = gemm_all[len(gemm_all) // 2]
    roof["kernel_ms_min"] = gemm_all[0]

    out = {
        "metric": metric, "value": value, "unit": unit, "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "int8", "data": "synthetic",
        "config": {"workload": f"{s.name}: M={s.M} K={s.K} N={s.N} r={s.r}", "tag": args.workload,
                   "step": "quantize_gemm_mixed (one kernel)" if one_call else
                           ("hadamard_quantize_act (one kernel) + " if fused else
                            "online_hadamard + quantize_act + " if s.hadamard else
                            "quantize_act + ") + "gemm_mixed",
                   "activations": "asymmetric per token" if args.asym else "symmetric per token",
                   "weight_copies_rotated": n_copies},
        "tokens_per_s": s.M / (ms_per_step * 1e-3),
        "hadamard_ms": had_ms, "quantize_ms": quant_ms, "gemm_ms": gemm_ms,
        "roofline": roof,
    }
    if not s.hadamard:
        out["snr_db"] = output_snr_db(x, w, y)
    if not args.no_cpu_baseline:
        from oracle import resq_oracle as oracle
        wq_np = oracle.quantize_weights(wl.bf16_bits(w), s.r)
        cb = cpu_baseline(s, x, wq_np, args.cpu_budget,
                          rq.resq_hadamard_block(s.K - s.r) if s.hadamard else 0, args.asym)
        if decode:
            # same unit as the metric: algorithmic bytes of the sampled rows per second
            frac = cb["rows"] / s.M
            cb["value"] = abytes * frac / cb["seconds"] / 1e9
            cb["unit"] = "GB/s"
        out["cpu_baseline"] = {k: cb[k] for k in ("value", "unit", "cores", "kind", "sample")}
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
