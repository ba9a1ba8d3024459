// Measurement aid, not part of the method: the rate at which this chip sustains
// v_mfma_i32_32x32x32_i8 with NOTHING else going on (operands resident in
// registers, eight independent accumulator tiles per wavefront, one wavefront per
// SIMD as in the tiled GEMM), for operand bytes supplied by the caller.  The matrix
// pipes are limited by power, so the rate depends on how many operand bits toggle:
// the benchmark compares all-zero, widened-INT4-like and random INT8 operands, which
// is the ceiling that the GEMM's fraction of the nominal peak has to be read against.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "resq_gemm.hip.h"

namespace resq {

constexpr int kProbeThreads = 256;
constexpr int kProbeOperandBytes = 2048 * 16;  // caller's buffer: 2048 16-byte fragments

// 2 * 32^3 * 8 operations per wavefront and iteration
__global__ __launch_bounds__(kProbeThreads) void probe_mfma_int8_kernel(int iters, const v4i* __restrict__ data,
                                                                       int* __restrict__ sink) {
    v16i acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][v] = 0;
    v4i a[2], b[4];
#pragma unroll
    for (int i = 0; i < 2; ++i) a[i] = data[(threadIdx.x + 256 * i) & 2047];
#pragma unroll
    for (int i = 0; i < 4; ++i) b[i] = data[(threadIdx.x + 256 * (i + 2)) & 2047];
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int i = 0; i < 2; ++i)
                acc[j * 2 + i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(b[j], a[i], acc[j * 2 + i], 0, 0, 0);
    }
    int s = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) s += acc[i][v];
    if (s == 0x7fffffff) sink[0] = s;  // keeps the loop alive; practically never true
}

// The same for HBM: a plain streaming read of `n16` 16-byte words, four loads in flight per
// lane, results folded into a value that is practically never stored: what a kernel that
// must read this many bytes once (the generation-stage GEMM: its packed weights) can reach.
__global__ __launch_bounds__(kProbeThreads) void probe_hbm_read_kernel(const uint4* __restrict__ p, size_t n16,
                                                                      uint32_t* __restrict__ sink) {
    size_t i = (size_t)blockIdx.x * kProbeThreads * 4 + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * kProbeThreads * 4;
    uint32_t acc = 0;
    for (; i < n16; i += stride) {
        uint4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u] = i + kProbeThreads * u < n16 ? p[i + kProbeThreads * u] : make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
        for (int u = 0; u < 4; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    }
    if (acc == 0x12345678u) sink[0] = acc;
}

}  // namespace resq
