// The online projection of queries and keys onto the basis of the K/V cache
// (Section 4.3: after the position embedding every head is multiplied by the
// d_head x d_head matrix U_C, with 8-bit weights and 8-bit activations): one
// kernel that reads the bf16 head rows, quantizes each row to INT8 with its own
// scale (Eq. 1, symmetric), multiplies by the packed INT8 codes of U_C on the
// matrix cores and writes the dequantized bf16 rows.  The result is that of the
// row quantizer followed by the mixed GEMM with r = K = N = d_head; the codes
// never go to memory.
//
// A wavefront owns 16 rows at a time.  Lane l holds a quarter of row l % 16:
// the d_head / 4 consecutive columns from (l / 16) d_head / 4 on, which it
// loads with 16-byte loads (the wavefront reads 16 whole rows, contiguous when
// the rows are), reduces (|max| over its quarter, then two exchanges inside the
// four lanes of the row) and quantizes in registers.  Both operands of the
// 16x16x64 int8 matrix instruction want 16 consecutive bytes of the reduction
// axis per lane and step; which 16 columns a (lane quarter, step) pair stands
// for is free as long as both operands agree, so step s takes columns
// (l / 16) d_head / 4 + 16 s of the activation row and of the weight row: no
// exchange between lanes.  The whole of U_C (d_head^2 bytes) is copied to LDS
// once per workgroup (while the first rows are quantized) and from there into
// registers once per wavefront; column
// slot c of tile j stands for channel (d_head / 16) c + j, so that a lane ends
// with d_head / 16 consecutive channels of a row and a store instruction writes
// four whole rows.  The next 16 rows are loaded while these are multiplied and written.
//
// Roofline: HBM (2 d_head bytes read and 2 d_head written per row); the row
// quantizer's vector-ALU work is of the same order.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "resq_gemm.hip.h"
#include "resq_quantize.hip.h"

namespace resq {

constexpr int kHeadProjThreads = 256;

struct HeadProjArgs {
    const uint16_t* x;  // bf16 [rows, ldx]
    int64_t ldx;
    int64_t rows;
    const uint8_t* packed;  // pack_weights image of U_C^T as [N = D][K = D], r = D
    WeightLayout L;
    uint16_t* y;  // bf16 [rows, ldy]
    int64_t ldy;
    int vec_store;  // y and ldy allow D / 16-byte stores
};

template <int D>
__global__ __launch_bounds__(kHeadProjThreads) void head_project_kernel(const HeadProjArgs a) {
    static_assert(D == 64 || D == 128, "d_head");
    constexpr int KS = D / 64;     // steps of the reduction axis
    constexpr int NT = D / 16;     // 16-channel tiles = consecutive channels per lane
    constexpr int UNITS = D / 32;  // 16-byte loads of a lane's quarter row
    constexpr int kWaves = kHeadProjThreads / 64;
    __shared__ __attribute__((aligned(16))) uint8_t wlds[(D / 16) * 2 * kBlockBytes];
    const int t = threadIdx.x, lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int c = lane & 15, q = lane >> 4;
    const int64_t tiles = (a.rows + 15) / 16;
    const int64_t stride = (int64_t)gridDim.x * kWaves;

    auto load_tile = [&](int64_t tile, uint4 (&v)[UNITS]) {
        const int64_t row_raw = tile * 16 + c;
        const int64_t row = row_raw < a.rows ? row_raw : a.rows - 1;  // rows past the end: computed, not stored
        const uint4* src = reinterpret_cast<const uint4*>(a.x + row * a.ldx + (D / 4) * q);
#pragma unroll
        for (int u = 0; u < UNITS; ++u) v[u] = src[u];
    };

    int64_t tile = (int64_t)blockIdx.x * kWaves + wave;
    uint4 v[UNITS];
    if (tile < tiles) load_tile(tile, v);

    // quantize the 16 x D values a wavefront holds: row scale and the operand of each step
    auto quantize_tile = [&](const uint4 (&rowv)[UNITS], v4i (&qa)[KS], float& st) {
        float amax = 0.0f;
#pragma unroll
        for (int u = 0; u < UNITS; ++u) amax = fmaxf(amax, absmax8(rowv[u]));
        amax = fmaxf(amax, lane_xor<16>(amax));
        amax = fmaxf(amax, lane_xor<32>(amax));
        st = group_scale(amax, kQmaxHi);
        const float inv = 1.0f / st;
        float unused = 0.0f;
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            uint32_t c0[8], c1[8];
            quant8<false>(rowv[2 * s], st, inv, c0, unused);
            quant8<false>(rowv[2 * s + 1], st, inv, c1, unused);
            qa[s] = (v4i){(int)pack_low_bytes(c0[0], c0[1], c0[2], c0[3]), (int)pack_low_bytes(c0[4], c0[5], c0[6], c0[7]),
                          (int)pack_low_bytes(c1[0], c1[1], c1[2], c1[3]), (int)pack_low_bytes(c1[4], c1[5], c1[6], c1[7])};
        }
    };

    // U_C: the D / 16 channel groups of the packed image, two high blocks each (the
    // second one is padding when D = 64), are contiguous.  They go to LDS by direct
    // loads (1 KiB per wavefront and instruction), and the first tile is quantized
    // while those are in flight.
    constexpr int kStageLoads = (D / 16) * 2 / kWaves;  // blocks per wavefront
    static_assert(kStageLoads * kWaves == (D / 16) * 2, "whole blocks per wavefront");
#pragma unroll
    for (int i = 0; i < kStageLoads; ++i) {
        const int blk = wave + i * kWaves;
        load_to_lds_16B(a.packed + blk * kBlockBytes + lane * 16, wlds + blk * kBlockBytes);
    }
    uint32_t sw_bits[NT / 2];  // the lane's NT consecutive fp16 channel scales
    {
        const uint8_t* swp = a.packed + a.L.scale_off + 2 * NT * c;
        if constexpr (NT == 8) {
            const uint4 w4 = *reinterpret_cast<const uint4*>(swp);
            sw_bits[0] = w4.x; sw_bits[1] = w4.y; sw_bits[2] = w4.z; sw_bits[3] = w4.w;
        } else {
            const uint2 w2 = *reinterpret_cast<const uint2*>(swp);
            sw_bits[0] = w2.x; sw_bits[1] = w2.y;
        }
    }
    v4i qa[KS];
    float st = 1.0f;
    if (tile < tiles) quantize_tile(v, qa, st);
    wait_loads_and_barrier<0>();
    // fragment (j, s) = channel NT c + j, bytes D/4 q + 16 s .. + 16 of its row
    v4i wfrag[NT][KS];
    float sw[NT];
#pragma unroll
    for (int j = 0; j < NT; ++j) {
        const int n = NT * c + j;
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            const int b = (D / 4) * q + 16 * s;
            wfrag[j][s] = *reinterpret_cast<const v4i*>(
                wlds + (n / 16) * (2 * kBlockBytes) + (b / kRowBytes) * kBlockBytes + (n % 16) * kRowBytes + b % kRowBytes);
        }
        sw[j] = fp16_bits_to_f32((sw_bits[j / 2] >> (16 * (j & 1))) & 0xFFFFu);
    }

    // v is free once its codes exist: the next 16 rows load while these are multiplied and
    // written, and are quantized at the end of the iteration
    for (; tile < tiles; tile += stride) {
        const bool more = tile + stride < tiles;
        if (more) load_tile(tile + stride, v);

        v4i acc[NT];
#pragma unroll
        for (int j = 0; j < NT; ++j) {
            acc[j] = (v4i){0, 0, 0, 0};
#pragma unroll
            for (int s = 0; s < KS; ++s)
                acc[j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(qa[s], wfrag[j][s], acc[j], 0, 0, 0);
        }

        // acc[j][i]: row 4 q + i of the tile, channel NT c + j; the scale of that row sits
        // in lane (row) of the wavefront
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int tr = 4 * q + i;
            const float srow = __int_as_float(__builtin_amdgcn_ds_bpermute(4 * tr, __float_as_int(st)));
            const int64_t orow = tile * 16 + tr;
            uint32_t o[NT / 2];
#pragma unroll
            for (int j = 0; j < NT; j += 2)
                o[j / 2] = pack_bf16((float)acc[j][i] * (srow * sw[j]), (float)acc[j + 1][i] * (srow * sw[j + 1]));
            if (orow < a.rows) {
                uint16_t* dst = a.y + orow * a.ldy + NT * c;
                if (a.vec_store) {
                    if constexpr (NT == 8) *reinterpret_cast<uint4*>(dst) = make_uint4(o[0], o[1], o[2], o[3]);
                    else *reinterpret_cast<uint2*>(dst) = make_uint2(o[0], o[1]);
                } else {
#pragma unroll
                    for (int j = 0; j < NT; ++j) dst[j] = (uint16_t)(o[j / 2] >> (16 * (j & 1)));
                }
            }
        }
        if (more) quantize_tile(v, qa, st);
    }
}

}  // namespace resq
