// Weight-streaming variant of the mixed INT8/INT4 layer for M <= 16 tokens
// (Section 4.1, Eq. 4; the generation stage, which the paper's introduction
// calls memory-bound).  The packed weights are read from HBM exactly once, in
// 1 KiB blocks that are already one operand of the 16x16x64 int8 matrix-core
// instruction (16 channels x 64 bytes, see resq_layout.h): lane l loads row
// l % 16, 16-byte piece l / 16 straight into operand registers, no LDS in
// between, and a wavefront walks the contiguous blocks of one 16-channel group
// (all high blocks, then all low blocks) with eight loads in flight.  One
// workgroup of eight wavefronts runs per compute unit, and groups are dealt
// round-robin over compute units first, so that every unit streams the same
// number of bytes.  The activation codes of all tokens (at most a few tens of
// KiB) sit in LDS for the whole kernel.  The matrix cores are nearly idle here; they are used because
// the vector ALU could not keep up with 8 TB/s of nibbles at M = 16.
//
// Roofline: HBM.  Algorithmic bytes = the packed weight buffer.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "resq_gemm.hip.h"
#include "resq_layout.h"

namespace resq {

constexpr int kDecodeThreads = 512;
constexpr int kDecodeMaxM = 16;
constexpr int kDecodeDepth = 8;      // weight loads in flight per wavefront
constexpr int kDecodeRowPad = 16;    // LDS row padding: 16 token rows hit 16 different bank groups

struct DecodeArgs {
    const uint8_t* q_hi;
    const uint8_t* q_lo;
    int64_t ld_hi, ld_lo;
    const float* s_hi;
    const float* s_lo;
    const int32_t* lo_sum;
    const float* c_hi;  // asymmetric activation codes only (else null): per token, the real
    const float* c_lo;  // value that the stored code 0 of the group stands for
    const uint8_t* packed;
    WeightLayout L;
    int M;
    uint16_t* y;
    int64_t ldy;
    int32_t* dbg_hi;
    int32_t* dbg_lo;
    int swiglu;       // 1: channels 2c, 2c+1 = gate and up row of feature c; y[m, c] = silu(gate) * up
    int groups;       // ceil(N / 16)
    int lds_row;      // bytes of one token row in LDS
};

template <bool DBG>
__global__ __launch_bounds__(kDecodeThreads) void gemm_decode_kernel(const DecodeArgs a) {
    extern __shared__ __attribute__((aligned(16))) uint8_t act[];  // [M][lds_row]
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int hi_blocks = (int)a.L.hi_blocks, blocks = (int)(a.L.hi_blocks + a.L.lo_blocks);
    const int hi_units = (int)(a.L.kh_pad / 16), row_units = hi_units + (int)(a.L.kl_pad / 32);
    const int lane_off = (lane & 15) * kRowBytes + (lane >> 4) * 16;

    // start the weight stream of this wave's first group before anything else
    int group = wave * gridDim.x + blockIdx.x;
    uint4 ring[kDecodeDepth];
    {
        const uint4* wp = reinterpret_cast<const uint4*>(
            a.packed + (int64_t)(group < a.groups ? group : 0) * a.L.group_bytes + lane_off);
#pragma unroll
        for (int i = 0; i < kDecodeDepth; ++i)
            if (group < a.groups && i < blocks) ring[i] = wp[i * (kBlockBytes / 16)];
    }

    // activation codes of every token -> LDS (row = high codes, then packed low codes);
    // 16-byte unit u of token m, up to twelve loads in flight per thread
    constexpr int FILL = 12;
    const int units = a.M * row_units;
    for (int u0 = t; u0 < units; u0 += FILL * kDecodeThreads) {
        uint4 v[FILL];
#pragma unroll
        for (int q = 0; q < FILL; ++q) {
            const int u = u0 + q * kDecodeThreads;
            v[q] = make_uint4(0u, 0u, 0u, 0u);
            if (u < units) {
                const int m = u / row_units, c = u - m * row_units;
                v[q] = c < hi_units
                           ? *reinterpret_cast<const uint4*>(a.q_hi + m * a.ld_hi + c * 16)
                           : *reinterpret_cast<const uint4*>(a.q_lo + m * a.ld_lo + (c - hi_units) * 16);
            }
        }
#pragma unroll
        for (int q = 0; q < FILL; ++q) {
            const int u = u0 + q * kDecodeThreads;
            if (u < units) {
                const int m = u / row_units, c = u - m * row_units;
                *reinterpret_cast<uint4*>(act + m * a.lds_row + c * 16) = v[q];
            }
        }
    }
    __syncthreads();

    // lane l supplies token l % 16 (zero operand past M), piece l / 16 of each 64-byte chunk
    const int tok = lane & 15;
    const bool tok_live = tok < a.M;
    const uint8_t* arow = act + (tok_live ? tok : 0) * a.lds_row + (lane >> 4) * 16;
    const v4i zero = {0, 0, 0, 0};
    const uint16_t* sw_hi = reinterpret_cast<const uint16_t*>(a.packed + a.L.scale_off);
    const uint16_t* sw_lo = sw_hi + a.L.n_pad;
    const int32_t* even_sum = reinterpret_cast<const int32_t*>(a.packed + a.L.scale_off + 4 * a.L.n_pad);
    const bool has_hi = a.L.r > 0, has_lo = a.L.K - a.L.r > 0;
    const float sth = (has_hi && tok_live) ? a.s_hi[tok] : 0.f;
    const float stl = (has_lo && tok_live) ? a.s_lo[tok] : 0.f;
    const int ca = (has_lo && tok_live) ? a.lo_sum[tok] : 0;
    // asymmetric activations: zero-point term c[m] * wsum[n] * sw[n] per group
    const bool asym = a.c_hi != nullptr || a.c_lo != nullptr;
    const float cth = (asym && has_hi && tok_live) ? a.c_hi[tok] : 0.f;
    const float ctl = (asym && has_lo && tok_live) ? a.c_lo[tok] : 0.f;
    const int32_t* wsum_hi = even_sum + a.L.n_pad;
    const int32_t* wsum_lo = even_sum + 2 * a.L.n_pad;

    for (; group < a.groups; group += 8 * gridDim.x) {
        const uint4* wp = reinterpret_cast<const uint4*>(a.packed + (int64_t)group * a.L.group_bytes + lane_off);
        v4i acc_hi = {0, 0, 0, 0}, acc_lo = {0, 0, 0, 0};
        for (int b0 = 0; b0 < blocks; b0 += kDecodeDepth) {
#pragma unroll
            for (int i = 0; i < kDecodeDepth; ++i) {
                const int b = b0 + i;
                if (b < blocks) {
                    const uint4 wq = ring[i];
                    if (b + kDecodeDepth < blocks) ring[i] = wp[(b + kDecodeDepth) * (kBlockBytes / 16)];
                    const v4i w = {(int)wq.x, (int)wq.y, (int)wq.z, (int)wq.w};
                    v4i p = *reinterpret_cast<const v4i*>(arow + b * kRowBytes);
                    if (!tok_live) p = zero;
                    if (b < hi_blocks) {
                        acc_hi = __builtin_amdgcn_mfma_i32_16x16x64_i8(w, p, acc_hi, 0, 0, 0);
                    } else {
                        // see resq_gemm.hip.h: one operand of each product carries an offset of 8
                        acc_lo = __builtin_amdgcn_mfma_i32_16x16x64_i8(
                            w & (int)0xF0F0F0F0, tok_live ? (p & (int)0x0F0F0F0F) : zero, acc_lo, 0, 0, 0);
                        acc_lo = __builtin_amdgcn_mfma_i32_16x16x64_i8(
                            w & (int)0x0F0F0F0F, p & (int)0xF0F0F0F0, acc_lo, 0, 0, 0);
                    }
                }
            }
        }
        // the next group's first loads go out before this group's epilogue
        const int next = group + 8 * gridDim.x;
        if (next < a.groups) {
            const uint4* np = reinterpret_cast<const uint4*>(a.packed + (int64_t)next * a.L.group_bytes + lane_off);
#pragma unroll
            for (int i = 0; i < kDecodeDepth; ++i)
                if (i < blocks) ring[i] = np[i * (kBlockBytes / 16)];
        }

        // lane l now holds token l % 16, channels 16 group + 4 (l / 16) + {0..3}
        if (!tok_live) continue;
        const int64_t n = (int64_t)group * 16 + (lane >> 4) * 4;
        const uint2 sch = *reinterpret_cast<const uint2*>(sw_hi + n);
        const uint2 scl = *reinterpret_cast<const uint2*>(sw_lo + n);
        const int4 es = *reinterpret_cast<const int4*>(even_sum + n);
        const float snh[4] = {fp16_bits_to_f32(sch.x & 0xFFFFu), fp16_bits_to_f32(sch.x >> 16),
                              fp16_bits_to_f32(sch.y & 0xFFFFu), fp16_bits_to_f32(sch.y >> 16)};
        const float snl[4] = {fp16_bits_to_f32(scl.x & 0xFFFFu), fp16_bits_to_f32(scl.x >> 16),
                              fp16_bits_to_f32(scl.y & 0xFFFFu), fp16_bits_to_f32(scl.y >> 16)};
        const int ev[4] = {es.x, es.y, es.z, es.w};
        float out[4];
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int a_hi = acc_hi[v];
            const int a_lo = (acc_lo[v] - 128 * (ev[v] + ca)) >> 4;  // exact
            out[v] = (float)a_hi * (sth * snh[v]) + (float)a_lo * (stl * snl[v]);
            if (asym)
                out[v] += cth * ((float)wsum_hi[n + v] * snh[v]) + ctl * ((float)wsum_lo[n + v] * snl[v]);
            if constexpr (DBG) {
                if (n + v < a.L.N) {
                    if (a.dbg_hi) a.dbg_hi[(int64_t)tok * a.L.N + n + v] = a_hi;
                    if (a.dbg_lo) a.dbg_lo[(int64_t)tok * a.L.N + n + v] = a_lo;
                }
            }
        }
        if (a.swiglu) {
            // two (gate, up) pairs per lane -> two outputs
            const int64_t c = n >> 1, c_end = a.L.N >> 1;
            uint16_t* d2 = a.y + (int64_t)tok * a.ldy + c;
            const uint32_t pair = pack_bf16(silu_f32(out[0]) * out[1], silu_f32(out[2]) * out[3]);
            if (c + 1 < c_end && ((reinterpret_cast<uintptr_t>(a.y) & 3) == 0) && (a.ldy % 2 == 0)) {
                *reinterpret_cast<uint32_t*>(d2) = pair;
            } else {
                if (c < c_end) d2[0] = (uint16_t)pair;
                if (c + 1 < c_end) d2[1] = (uint16_t)(pair >> 16);
            }
            continue;
        }
        uint16_t* dst = a.y + (int64_t)tok * a.ldy + n;
        if (n + 3 < a.L.N && ((reinterpret_cast<uintptr_t>(a.y) & 7) == 0) && (a.ldy % 4 == 0)) {
            *reinterpret_cast<uint2*>(dst) = make_uint2(pack_bf16(out[0], out[1]), pack_bf16(out[2], out[3]));
        } else {
#pragma unroll
            for (int v = 0; v < 4; ++v)
                if (n + v < a.L.N) dst[v] = (uint16_t)pack_bf16(out[v], 0.f);
        }
    }
}

}  // namespace resq
