// Calibration kernels for bench.py (not part of the library, nothing of the method):
// what this chip sustains on the int8 matrix instruction alone and on a plain streaming
// read, so that the benchmark can quote its kernels against the measured ceilings next to
// the nominal peaks.  The matrix pipes are power-limited: the rate depends on the operand
// bytes, which the caller supplies.
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

typedef int v4i __attribute__((ext_vector_type(4)));

constexpr int kThreads = 512;  // two wavefronts per SIMD, as in the tiled GEMM

// 16 accumulator tiles per wavefront, 4 x 4 operand fragments, even and odd halves like the
// GEMM's widened nibbles: 32 x v_mfma_i32_16x16x64_i8 per iteration and wavefront
__global__ __launch_bounds__(kThreads) void calib_mfma_kernel(int iters, const v4i* __restrict__ a_bytes,
                                                             const v4i* __restrict__ b_bytes, int* __restrict__ sink) {
    const int t = threadIdx.x;
    v4i acc[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = (v4i){0, 0, 0, 0};
    v4i a[2][4], b[2][4];
#pragma unroll
    for (int e = 0; e < 2; ++e)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            a[e][i] = a_bytes[(t + kThreads * (4 * e + i)) & 4095];
            b[e][i] = b_bytes[(t + kThreads * (4 * e + i)) & 4095];
        }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int e = 0; e < 2; ++e)
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    acc[j * 4 + i] = __builtin_amdgcn_mfma_i32_16x16x64_i8(b[e][j], a[e][i], acc[j * 4 + i], 0, 0, 0);
    }
    int s = 0;
#pragma unroll
    for (int i = 0; i < 16; ++i) s += acc[i][0] + acc[i][1] + acc[i][2] + acc[i][3];
    if (s == 0x7fffffff) sink[0] = s;  // keeps the loop alive; practically never true
}

// plain streaming read of n16 16-byte words, four loads in flight per lane
__global__ __launch_bounds__(256) void calib_read_kernel(const uint4* __restrict__ p, size_t n16,
                                                         uint32_t* __restrict__ sink) {
    size_t i = (size_t)blockIdx.x * 256 * 4 + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * 256 * 4;
    uint32_t acc = 0;
    for (; i < n16; i += stride) {
        uint4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u] = i + 256 * u < n16 ? p[i + 256 * u] : make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
        for (int u = 0; u < 4; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    }
    if (acc == 0x12345678u) sink[0] = acc;
}

extern "C" {

// a_bytes, b_bytes: device, 64 KiB each (4096 fragments of 16 bytes), 16-byte aligned; sink: one int, device.
// The two events (hipEvent_t, may be null) are recorded at the kernel's own start and end.
// Operations per launch: 2 * 16 * 16 * 64 * 32 * 8 * iters * workgroups.
int calib_mfma_int8(const void* a_bytes, const void* b_bytes, int iters, int workgroups, int* sink,
                    void* start_event, void* stop_event, void* stream) {
    if (!a_bytes || !b_bytes || !sink || iters < 1 || workgroups < 1) return 1;
    hipExtLaunchKernelGGL(calib_mfma_kernel, dim3((unsigned)workgroups), dim3(kThreads), 0,
                          static_cast<hipStream_t>(stream), static_cast<hipEvent_t>(start_event),
                          static_cast<hipEvent_t>(stop_event), 0, iters, static_cast<const v4i*>(a_bytes),
                          static_cast<const v4i*>(b_bytes), sink);
    return hipGetLastError() == hipSuccess ? 0 : 5;
}

// reads the first bytes / 16 * 16 bytes of buf (device, 16-byte aligned) once
int calib_hbm_read(const void* buf, size_t bytes, int workgroups, int* sink, void* start_event,
                   void* stop_event, void* stream) {
    if (!buf || !sink || bytes < 16 || workgroups < 1) return 1;
    hipExtLaunchKernelGGL(calib_read_kernel, dim3((unsigned)workgroups), dim3(256), 0,
                          static_cast<hipStream_t>(stream), static_cast<hipEvent_t>(start_event),
                          static_cast<hipEvent_t>(stop_event), 0, static_cast<const uint4*>(buf), bytes / 16,
                          reinterpret_cast<uint32_t*>(sink));
    return hipGetLastError() == hipSuccess ? 0 : 5;
}

}  // extern "C"
