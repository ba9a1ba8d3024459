// Offline construction of the projection basis (Section 4.2): the dense products.
//
//   gram:    C[i][j] += sum_t X[t][i] X[t][j]      covariance of the calibration activations
//   project: Y[i][j]  = sum_t A[i][t] U[t][j]      rows of A (activations, weights, P_h, P_l)
//                                                  expressed in a basis / rotated inside a group
//
// Both are C(i, j) = sum_t A(i, t) B(t, j) with fp32 accumulation on the fp32
// matrix-core instruction v_mfma_f32_32x32x2_f32 (bf16 inputs are widened exactly,
// so a Gram matrix of bf16 data loses nothing before the accumulation; the basis
// itself must stay fp32: a bf16 U would be orthogonal to 2^-9 only).  Lane l of
// that instruction supplies A(i = l % 32, t = l / 32) and B(t = l / 32, j = l % 32):
// with both tiles stored t-major in LDS (As[t][i], Bs[t][j]) an operand is one
// conflict-free ds_read_b32, and the Gram matrix needs no transposition at all
// (its A(i, t) = X[t][i] is t-major in memory already).
//
// Workgroup: 4 wavefronts, 128 x 128 outputs (a wavefront 64 x 64 = 2 x 2 matrix
// tiles), reduction in chunks of 16 through two LDS buffers, the next chunk
// travelling through registers while this one is multiplied; one barrier per chunk.
// Roofline: fp32 matrix (157.3 TFLOP/s); 2 I J T flops.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "resq_gemm.hip.h"

namespace resq {

typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int kBasisThreads = 256;
constexpr int kBasisTile = 128;   // outputs per workgroup, each way
constexpr int kBasisChunk = 16;   // reduction steps per LDS buffer
constexpr int kBasisPitch = kBasisTile + 4;  // floats; rows 16-byte aligned

struct BasisGemmArgs {
    const void* a;   // A_TRANS: [T][lda] (element (i, t) at a[t * lda + i]); else [I][lda]
    const void* b;   // [T][ldb]
    void* c;         // [I][ldc], fp32 or bf16
    int64_t lda, ldb, ldc;
    int64_t I, J, T;
    int64_t t_per_slice;  // reduction steps per blockIdx.z (a multiple of kBasisChunk)
    int accumulate;       // fp32 output only: add to what is there (atomically when the reduction is sliced)
};

template <bool BF16>
__device__ __forceinline__ void load8(const void* base, int64_t elem, bool live, float (&v)[8]) {
    if (!live) {
#pragma unroll
        for (int k = 0; k < 8; ++k) v[k] = 0.0f;
        return;
    }
    if constexpr (BF16) {
        const uint4 w = *reinterpret_cast<const uint4*>(static_cast<const uint16_t*>(base) + elem);
        const uint32_t ww[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
        for (int k = 0; k < 8; ++k)
            v[k] = __uint_as_float((k & 1) ? (ww[k >> 1] & 0xFFFF0000u) : (ww[k >> 1] << 16));
    } else {
        const float4 lo = *reinterpret_cast<const float4*>(static_cast<const float*>(base) + elem);
        const float4 hi = *reinterpret_cast<const float4*>(static_cast<const float*>(base) + elem + 4);
        v[0] = lo.x; v[1] = lo.y; v[2] = lo.z; v[3] = lo.w;
        v[4] = hi.x; v[5] = hi.y; v[6] = hi.z; v[7] = hi.w;
    }
}

// Requires lda, ldb multiples of 8 elements and 16-byte (bf16) / 32-byte... aligned bases
// (checked on the host); I, J, T arbitrary.
template <bool A_TRANS, bool A_BF16, bool B_BF16, bool OUT_BF16>
__global__ __launch_bounds__(kBasisThreads) void basis_gemm_kernel(const BasisGemmArgs g) {
    __shared__ __attribute__((aligned(16))) float lds_a[2][kBasisChunk][kBasisPitch];
    __shared__ __attribute__((aligned(16))) float lds_b[2][kBasisChunk][kBasisPitch];
    const int t = threadIdx.x, lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int wi = wave >> 1, wj = wave & 1;
    const int64_t i0 = (int64_t)blockIdx.y * kBasisTile, j0 = (int64_t)blockIdx.x * kBasisTile;
    const int64_t t_begin = (int64_t)blockIdx.z * g.t_per_slice;
    const int64_t t_end = t_begin + g.t_per_slice < g.T ? t_begin + g.t_per_slice : g.T;

    // loaders: a t-major source gives thread (row t / 16 of the chunk, 8 columns); an
    // i-major A gives thread (row i = t % 128, 8 consecutive reduction steps)
    const int lr = t >> 4, lc = (t & 15) * 8;      // t-major: chunk row, first column
    const int ar = t & 127, at = (t >> 7) * 8;     // i-major A: tile row, first step
    float ra[8], rb[8];
    auto fetch = [&](int64_t tc) {
        if constexpr (A_TRANS) {
            const int64_t tt = tc + lr, i = i0 + lc;
            load8<A_BF16>(g.a, tt * g.lda + i, tt < t_end && i < g.I, ra);   // I % 8 == 0 in this form
        } else {
            const int64_t i = i0 + ar, tt = tc + at;
            load8<A_BF16>(g.a, i * g.lda + tt, i < g.I && tt + 8 <= t_end, ra);
            if (i < g.I && tt < t_end && tt + 8 > t_end) {   // ragged end of the reduction axis
#pragma unroll
                for (int k = 0; k < 8; ++k) {
                    ra[k] = 0.0f;
                    if (tt + k < t_end) {
                        if constexpr (A_BF16) ra[k] = __uint_as_float((uint32_t)static_cast<const uint16_t*>(g.a)[i * g.lda + tt + k] << 16);
                        else ra[k] = static_cast<const float*>(g.a)[i * g.lda + tt + k];
                    }
                }
            }
        }
        const int64_t tt = tc + lr, j = j0 + lc;
        load8<B_BF16>(g.b, tt * g.ldb + j, tt < t_end && j < g.J, rb);       // J % 8 == 0
    };
    auto stash = [&](int buf) {
        if constexpr (A_TRANS) {
            *reinterpret_cast<float4*>(&lds_a[buf][lr][lc]) = make_float4(ra[0], ra[1], ra[2], ra[3]);
            *reinterpret_cast<float4*>(&lds_a[buf][lr][lc + 4]) = make_float4(ra[4], ra[5], ra[6], ra[7]);
        } else {
#pragma unroll
            for (int k = 0; k < 8; ++k) lds_a[buf][at + k][ar] = ra[k];
        }
        *reinterpret_cast<float4*>(&lds_b[buf][lr][lc]) = make_float4(rb[0], rb[1], rb[2], rb[3]);
        *reinterpret_cast<float4*>(&lds_b[buf][lr][lc + 4]) = make_float4(rb[4], rb[5], rb[6], rb[7]);
    };

    v16f acc[2][2];
#pragma unroll
    for (int p = 0; p < 2; ++p)
#pragma unroll
        for (int q = 0; q < 2; ++q)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[p][q][v] = 0.0f;

    const int ol = lane & 31, oh = lane >> 5;
    int buf = 0;
    if (t_begin < t_end) {
        fetch(t_begin);
        stash(0);
    }
    __syncthreads();
    for (int64_t tc = t_begin; tc < t_end; tc += kBasisChunk) {
        const bool more = tc + kBasisChunk < t_end;
        if (more) fetch(tc + kBasisChunk);
#pragma unroll
        for (int s = 0; s < kBasisChunk; s += 2) {
            float fa[2], fb[2];
#pragma unroll
            for (int p = 0; p < 2; ++p) fa[p] = lds_a[buf][s + oh][wi * 64 + p * 32 + ol];
#pragma unroll
            for (int q = 0; q < 2; ++q) fb[q] = lds_b[buf][s + oh][wj * 64 + q * 32 + ol];
#pragma unroll
            for (int p = 0; p < 2; ++p)
#pragma unroll
                for (int q = 0; q < 2; ++q)
                    acc[p][q] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[p], fb[q], acc[p][q], 0, 0, 0);
        }
        if (more) stash(buf ^ 1);  // last read in the previous iteration, before its barrier
        __syncthreads();
        buf ^= 1;
    }

    // acc[p][q][v]: row 8 (v / 4) + 4 (lane / 32) + v % 4, column lane % 32 of matrix tile (p, q)
#pragma unroll
    for (int p = 0; p < 2; ++p) {
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            const int64_t j = j0 + wj * 64 + q * 32 + ol;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int64_t i = i0 + wi * 64 + p * 32 + 8 * (v >> 2) + 4 * oh + (v & 3);
                if (i < g.I && j < g.J) {
                    if constexpr (OUT_BF16) {
                        static_cast<uint16_t*>(g.c)[i * g.ldc + j] = (uint16_t)pack_bf16(acc[p][q][v], 0.0f);
                    } else {
                        float* dst = static_cast<float*>(g.c) + i * g.ldc + j;
                        if (!g.accumulate) *dst = acc[p][q][v];
                        else if (gridDim.z == 1) *dst += acc[p][q][v];
                        else atomicAdd(dst, acc[p][q][v]);
                    }
                }
            }
        }
    }
}

}  // namespace resq
