// Online block Walsh-Hadamard transform (Section 4.3, projection U_D applied
// to the down_proj input at run time):
//   y[c0 + g b + j] = (1 / sqrt(b)) * sum_i x[c0 + g b + i] * (-1)^popcount(i & j)
// for every block g of b columns (b a power of two) of [c0, c1).
//
// One wavefront transforms a span of 512 * I consecutive columns of one row,
// held entirely in registers: element e = i * 512 + lane * 8 + j of the span
// sits in register (i, j) of lane `lane`, so global accesses are 16 bytes per
// lane and coalesced.  Butterfly stage p pairs elements that differ in bit p:
// bits 0..2 are register-to-register, bits 3..8 cross lanes (one shuffle per
// value), bits 9.. are register-to-register again.  Only stages p < log2(b)
// run, so a span covers several whole blocks when b < 512 * I.  HBM-bound: one
// read and one write of the transformed columns.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

namespace resq {

constexpr int kHadThreads = 256;

struct HadArgs {
    const uint16_t* x;
    uint16_t* y;
    int64_t ld, M;
    int K, c0, c1;
    int log2b;
    int spans_per_row;
    float scale;  // 1 / sqrt(b)
};

// value of lane (l ^ MASK): data-parallel-primitive moves inside a row of 16
// lanes where the pattern has one (quad permutes for 1 and 2, a rotation by 8),
// the swizzle unit inside 32 lanes, a general shuffle across the two halves
template <int MASK>
__device__ __forceinline__ float lane_xor(float x) {
    const int xi = __float_as_int(x);
    int r;
    if constexpr (MASK == 1) r = __builtin_amdgcn_update_dpp(xi, xi, 0xB1, 0xF, 0xF, false);       // quad_perm [1,0,3,2]
    else if constexpr (MASK == 2) r = __builtin_amdgcn_update_dpp(xi, xi, 0x4E, 0xF, 0xF, false);  // quad_perm [2,3,0,1]
    else if constexpr (MASK == 8) r = __builtin_amdgcn_update_dpp(xi, xi, 0x128, 0xF, 0xF, false); // row_ror:8
    else if constexpr (MASK == 4) r = __builtin_amdgcn_ds_swizzle(xi, 0x101F);                     // xor 4 within 32
    else if constexpr (MASK == 16) r = __builtin_amdgcn_ds_swizzle(xi, 0x401F);                    // xor 16 within 32
    else r = __float_as_int(__shfl_xor(x, MASK));
    return __int_as_float(r);
}

template <int I>
__global__ __launch_bounds__(kHadThreads) void hadamard_kernel(const HadArgs a) {
    const int lane = threadIdx.x & 63;
    const int64_t item = (int64_t)blockIdx.x * (kHadThreads / 64) + (threadIdx.x >> 6);
    const int64_t m = item / a.spans_per_row;
    const int span = (int)(item % a.spans_per_row);
    if (m >= a.M) return;
    const int span_cols = 512 * I;
    const int base = a.c0 + span * span_cols;
    const uint16_t* xr = a.x + m * a.ld;
    uint16_t* yr = a.y + m * a.ld;

    float v[I][8];
#pragma unroll
    for (int i = 0; i < I; ++i) {
        const int col = base + i * 512 + lane * 8;
        uint4 w = make_uint4(0u, 0u, 0u, 0u);
        if (col < a.c1) w = *reinterpret_cast<const uint4*>(xr + col);
        const uint32_t ww[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
        for (int j = 0; j < 8; ++j)
            v[i][j] = __uint_as_float((j & 1) ? (ww[j >> 1] & 0xFFFF0000u) : (ww[j >> 1] << 16));
    }

    // stages inside a lane's 8-vector (bits 0..2)
#pragma unroll
    for (int p = 0; p < 3; ++p) {
        if (p < a.log2b) {
#pragma unroll
            for (int i = 0; i < I; ++i)
#pragma unroll
                for (int j = 0; j < 8; ++j)
                    if (!(j & (1 << p))) {
                        const float lo = v[i][j], hi = v[i][j | (1 << p)];
                        v[i][j] = lo + hi;
                        v[i][j | (1 << p)] = lo - hi;
                    }
        }
    }
    // stages across lanes (bits 3..8): new = partner + sign * own, sign = -1 in
    // the upper lane of a pair
    auto lane_stage = [&](auto m) __attribute__((always_inline)) {
        constexpr int MASK = decltype(m)::value;
        const float sign = (lane & MASK) ? -1.0f : 1.0f;
#pragma unroll
        for (int i = 0; i < I; ++i)
#pragma unroll
            for (int j = 0; j < 8; ++j) v[i][j] = lane_xor<MASK>(v[i][j]) + sign * v[i][j];
    };
    if (a.log2b > 3) lane_stage(std::integral_constant<int, 1>{});
    if (a.log2b > 4) lane_stage(std::integral_constant<int, 2>{});
    if (a.log2b > 5) lane_stage(std::integral_constant<int, 4>{});
    if (a.log2b > 6) lane_stage(std::integral_constant<int, 8>{});
    if (a.log2b > 7) lane_stage(std::integral_constant<int, 16>{});
    if (a.log2b > 8) lane_stage(std::integral_constant<int, 32>{});
    // stages across a lane's vectors (bits 9..)
#pragma unroll
    for (int p = 9; (1 << (p - 9)) < I; ++p) {
        if (p < a.log2b) {
            const int bit = 1 << (p - 9);
#pragma unroll
            for (int i = 0; i < I; ++i)
                if (!(i & bit)) {
#pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        const float lo = v[i][j], hi = v[i | bit][j];
                        v[i][j] = lo + hi;
                        v[i | bit][j] = lo - hi;
                    }
                }
        }
    }

#pragma unroll
    for (int i = 0; i < I; ++i) {
        const int col = base + i * 512 + lane * 8;
        if (col < a.c1) {
            uint32_t o[4];
#pragma unroll
            for (int j = 0; j < 8; j += 2) {
                uint32_t lo = __float_as_uint(v[i][j] * a.scale);
                uint32_t hi = __float_as_uint(v[i][j + 1] * a.scale);
                lo += 0x7FFFu + ((lo >> 16) & 1u);  // round to nearest even bf16
                hi += 0x7FFFu + ((hi >> 16) & 1u);
                o[j >> 1] = (lo >> 16) | (hi & 0xFFFF0000u);
            }
            *reinterpret_cast<uint4*>(yr + col) = make_uint4(o[0], o[1], o[2], o[3]);
        }
    }
}

// copies columns [0, c0) and [c1, K) of every row when y is a different buffer
__global__ __launch_bounds__(kHadThreads) void hadamard_copy_rest_kernel(const HadArgs a) {
    const int64_t m = blockIdx.x;
    const uint16_t* xr = a.x + m * a.ld;
    uint16_t* yr = a.y + m * a.ld;
    for (int k = threadIdx.x; k < a.c0; k += kHadThreads) yr[k] = xr[k];
    for (int k = a.c1 + threadIdx.x; k < a.K; k += kHadThreads) yr[k] = xr[k];
}

}  // namespace resq
