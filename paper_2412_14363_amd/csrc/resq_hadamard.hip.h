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

// ---- pieces shared with the fused transform + quantize kernel ------------------
// A lane holds 8 consecutive columns (16 bytes of bf16); column bits 0..2 select
// the register, bits 3..8 the lane.

__device__ __forceinline__ void unpack8_bf16(const uint4& w, float (&v)[8]) {
    const uint32_t ww[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
    for (int j = 0; j < 8; ++j)
        v[j] = __uint_as_float((j & 1) ? (ww[j >> 1] & 0xFFFF0000u) : (ww[j >> 1] << 16));
}

// butterfly stages of column bits 0..2 (those below log2b)
__device__ __forceinline__ void wht_in_lane(float (&v)[8], int log2b) {
#pragma unroll
    for (int p = 0; p < 3; ++p) {
        if (p < log2b) {
#pragma unroll
            for (int j = 0; j < 8; ++j)
                if (!(j & (1 << p))) {
                    const float lo = v[j], hi = v[j | (1 << p)];
                    v[j] = lo + hi;
                    v[j | (1 << p)] = lo - hi;
                }
        }
    }
}

// one butterfly stage across lanes: new = partner + sign * own, sign = -1 in
// the upper lane of a pair
template <int MASK>
__device__ __forceinline__ void wht_lane_stage(float (&v)[8], int lane) {
    const float sign = (lane & MASK) ? -1.0f : 1.0f;
#pragma unroll
    for (int j = 0; j < 8; ++j) v[j] = lane_xor<MASK>(v[j]) + sign * v[j];
}

// butterfly stages of column bits 3..8 (those below log2b); every lane of the
// wavefront must call this
__device__ __forceinline__ void wht_across_lanes(float (&v)[8], int log2b, int lane) {
    if (log2b > 3) wht_lane_stage<1>(v, lane);
    if (log2b > 4) wht_lane_stage<2>(v, lane);
    if (log2b > 5) wht_lane_stage<4>(v, lane);
    if (log2b > 6) wht_lane_stage<8>(v, lane);
    if (log2b > 7) wht_lane_stage<16>(v, lane);
    if (log2b > 8) wht_lane_stage<32>(v, lane);
}

// scale, round to bf16 (nearest even: the hardware conversion), pack
typedef float v2f_had __attribute__((ext_vector_type(2)));
typedef __bf16 v2bf_had __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint4 pack8_bf16(const float (&v)[8], float scale) {
    uint32_t o[4];
#pragma unroll
    for (int j = 0; j < 8; j += 2) {
        const v2bf_had r = __builtin_convertvector((v2f_had){v[j] * scale, v[j + 1] * scale}, v2bf_had);
        o[j >> 1] = *reinterpret_cast<const uint32_t*>(&r);
    }
    return make_uint4(o[0], o[1], o[2], o[3]);
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
        unpack8_bf16(w, v[i]);
    }
#pragma unroll
    for (int i = 0; i < I; ++i) wht_in_lane(v[i], a.log2b);
#pragma unroll
    for (int i = 0; i < I; ++i) wht_across_lanes(v[i], a.log2b, lane);
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
        if (col < a.c1) *reinterpret_cast<uint4*>(yr + col) = pack8_bf16(v[i], a.scale);
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
