// Tiled mixed INT8/INT4 GEMM with dequantizing epilogue (Section 4.1, Eq. 4):
//   A_hi = q_hi * w_hi^T over the high group, A_lo = q_lo * w_lo^T over the low
//   group, y = bf16(A_hi * s_hi[m] * sw_hi[n] + A_lo * s_lo[m] * sw_lo[n]).
//
// One workgroup of 4 wavefronts owns a 128 (tokens) x 256 (channels) output
// tile; each wavefront owns 64 x 128 of it as 4 x 8 tiles of the 16x16x64 int8
// matrix-core instruction.  The reduction axis is walked in stages of 128 bytes
// per row: a stage of the high group is 128 int8 codes, a stage of the low
// group 256 nibble codes, so the global->LDS copy is the same for both.  LDS
// holds operand images ("chunks", see resq_layout.h) that a wavefront reads
// with one conflict-free 16-byte-per-lane load each.
//
// The low group: a lane's 16 packed bytes hold 32 codes.  (p << 4) & 0xF0F0F0F0
// puts the even codes, p & 0xF0F0F0F0 the odd codes, into the high nibble of
// each byte, i.e. 16 * code as int8, for activations and weights alike; the two
// results feed two matrix-core instructions.  The accumulator therefore holds
// 256 * A_lo, and an arithmetic shift by 8 recovers A_lo exactly.
//
// The two groups have different scale pairs, so they cannot share an integer
// accumulator: after the high stages the int32 tile is scaled into an fp32
// tile that stays in registers, the int32 tile is cleared for the low stages,
// and the output is written once.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "resq_layout.h"

namespace resq {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef float v4f __attribute__((ext_vector_type(4)));

constexpr int kGemmThreads = 256;
constexpr int kBM = 128;
constexpr int kBN = 256;
constexpr int kStageABytes = kBM * 128;  // 16 KiB
constexpr int kStageBBytes = kBN * 128;  // 32 KiB
constexpr int kStageBytes = kStageABytes + kStageBBytes;
constexpr int kAUnits = kStageABytes / 16 / kGemmThreads;  // 16-byte units per thread: 4
constexpr int kBUnits = kStageBBytes / 16 / kGemmThreads;  // 8

struct GemmArgs {
    const uint8_t* q_hi;
    const uint8_t* q_lo;
    int64_t ld_hi, ld_lo;
    const float* s_hi;
    const float* s_lo;
    const uint8_t* packed;
    WeightLayout L;
    int64_t M;
    uint16_t* y;
    int64_t ldy;
    int32_t* dbg_hi;
    int32_t* dbg_lo;
    int stages_hi, stages_lo;
    int tiles_m, tiles_n;
};

__device__ __forceinline__ float fp16_bits_to_f32(uint32_t h) {
    return __uint_as_float((((h >> 10) & 0x1Fu) + 112u) << 23 | (h & 0x3FFu) << 13);
}

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// blockIdx -> (tile_m, tile_n).  Consecutive workgroup ids land on different
// XCDs (8 of them, each with its own L2), so ids are first regrouped per XCD
// and each XCD then walks a compact band of the tile grid.
__device__ __forceinline__ void tile_of_block(const GemmArgs& a, int& tm, int& tn) {
    const int total = a.tiles_m * a.tiles_n;
    int id = blockIdx.x;
    if (total % 8 == 0) id = (id % 8) * (total / 8) + id / 8;
    tn = id / a.tiles_m;
    tm = id % a.tiles_m;
}

__global__ __launch_bounds__(kGemmThreads) void gemm_mixed_kernel(const GemmArgs a) {
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];  // 2 stages
    const int t = threadIdx.x;
    const int lane = t & 63;
    const int wave = t >> 6;
    const int wm = wave >> 1;  // 0..1: 64-token half of the tile
    const int wn = wave & 1;   // 0..1: 128-channel half of the tile
    int tile_m, tile_n;
    tile_of_block(a, tile_m, tile_n);
    const int64_t m0 = (int64_t)tile_m * kBM;
    const int64_t n0 = (int64_t)tile_n * kBN;
    const int stages = a.stages_hi + a.stages_lo;

    // ---- global -> register -> LDS copy of one stage -------------------------
    // A (activation codes): unit e = t + 256 i is the 16 bytes of LDS at 16 e,
    // i.e. token row (e % 16) of 16-row block (e / 128), sub-chunk (e / 16) % 4
    // of chunk (e / 64) % 2.  B (weights): the stage is 16 contiguous 2 KiB
    // pieces, one per 16-channel block, already in operand order.
    int64_t a_row_off_hi[kAUnits], a_row_off_lo[kAUnits];
#pragma unroll
    for (int i = 0; i < kAUnits; ++i) {
        const int e = t + kGemmThreads * i;
        int64_t row = m0 + (e >> 7) * 16 + (e & 15);
        row = row < a.M ? row : a.M - 1;
        const int col = ((e >> 6) & 1) * 64 + ((e >> 4) & 3) * 16;
        a_row_off_hi[i] = row * a.ld_hi + col;
        a_row_off_lo[i] = row * a.ld_lo + col;
    }
    const uint8_t* b_base[kBUnits];
#pragma unroll
    for (int i = 0; i < kBUnits; ++i) {
        const int e = t + kGemmThreads * i;
        b_base[i] = a.packed + (n0 / 16 + (e >> 7)) * a.L.block_bytes + (e & 127) * 16;
    }
    uint4 ra[kAUnits], rb[kBUnits];
    auto load_stage = [&](int s) {
        if (s < a.stages_hi) {
#pragma unroll
            for (int i = 0; i < kAUnits; ++i)
                ra[i] = *reinterpret_cast<const uint4*>(a.q_hi + a_row_off_hi[i] + (int64_t)s * 128);
#pragma unroll
            for (int i = 0; i < kBUnits; ++i)
                rb[i] = *reinterpret_cast<const uint4*>(b_base[i] + (int64_t)s * 2 * kChunkBytes);
        } else {
            const int sl = s - a.stages_hi;
#pragma unroll
            for (int i = 0; i < kAUnits; ++i)
                ra[i] = *reinterpret_cast<const uint4*>(a.q_lo + a_row_off_lo[i] + (int64_t)sl * 128);
#pragma unroll
            for (int i = 0; i < kBUnits; ++i)
                rb[i] = *reinterpret_cast<const uint4*>(
                    b_base[i] + (a.L.hi_chunks + (int64_t)sl * 2) * kChunkBytes);
        }
    };
    auto store_stage = [&](int buf) {
        uint8_t* sa = lds + buf * kStageBytes;
        uint8_t* sb = sa + kStageABytes;
#pragma unroll
        for (int i = 0; i < kAUnits; ++i)
            *reinterpret_cast<uint4*>(sa + (t + kGemmThreads * i) * 16) = ra[i];
#pragma unroll
        for (int i = 0; i < kBUnits; ++i)
            *reinterpret_cast<uint4*>(sb + (t + kGemmThreads * i) * 16) = rb[i];
    };

    // ---- accumulators: acc[j][i] is channels 16 j.., tokens 16 i.. of the wave tile;
    // lane l holds token (l % 16) and channels 4 (l / 16) + {0,1,2,3}
    v4i acc[8][4];
    v4f part[8][4];
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            acc[j][i] = (v4i){0, 0, 0, 0};
            part[j][i] = (v4f){0.f, 0.f, 0.f, 0.f};
        }

    // per-lane coordinates of the epilogue
    const int64_t tok0 = m0 + wm * 64 + (lane & 15);
    const int64_t ch0 = n0 + wn * 128 + (lane >> 4) * 4;
    const uint16_t* sw_hi = reinterpret_cast<const uint16_t*>(a.packed + a.L.scale_off);
    const uint16_t* sw_lo = sw_hi + a.L.n_pad;

    auto fold = [&](const float* s_tok, const uint16_t* s_ch, int32_t* dbg, int shift) {
        float st[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int64_t m = tok0 + 16 * i;
            st[i] = m < a.M ? s_tok[m] : 0.0f;
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int64_t n = ch0 + 16 * j;  // < n_pad always
            const uint2 sc = *reinterpret_cast<const uint2*>(s_ch + n);
            const float sn[4] = {fp16_bits_to_f32(sc.x & 0xFFFFu), fp16_bits_to_f32(sc.x >> 16),
                                 fp16_bits_to_f32(sc.y & 0xFFFFu), fp16_bits_to_f32(sc.y >> 16)};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int64_t m = tok0 + 16 * i;
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int iv = acc[j][i][v] >> shift;
                    part[j][i][v] += (float)iv * (st[i] * sn[v]);
                    if (dbg && m < a.M && n + v < a.L.N) dbg[m * a.L.N + n + v] = iv;
                    acc[j][i][v] = 0;
                }
            }
        }
    };

    if (stages > 0) {
        load_stage(0);
        store_stage(0);
    }
    __syncthreads();

    for (int s = 0; s < stages; ++s) {
        const int buf = s & 1;
        if (s + 1 < stages) load_stage(s + 1);
        const uint8_t* sa = lds + buf * kStageBytes;
        const uint8_t* sb = sa + kStageABytes;
        if (s < a.stages_hi) {
#pragma unroll
            for (int c = 0; c < 2; ++c) {
                v4i fa[4];
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    fa[i] = *reinterpret_cast<const v4i*>(sa + ((wm * 4 + i) * 2 + c) * kChunkBytes + lane * 16);
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const v4i fb = *reinterpret_cast<const v4i*>(sb + ((wn * 8 + j) * 2 + c) * kChunkBytes + lane * 16);
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        acc[j][i] = __builtin_amdgcn_mfma_i32_16x16x64_i8(fb, fa[i], acc[j][i], 0, 0, 0);
                }
            }
        } else {
#pragma unroll
            for (int c = 0; c < 2; ++c) {
                v4i fe[4], fo[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const v4i p = *reinterpret_cast<const v4i*>(sa + ((wm * 4 + i) * 2 + c) * kChunkBytes + lane * 16);
                    fe[i] = (p << 4) & (int)0xF0F0F0F0;
                    fo[i] = p & (int)0xF0F0F0F0;
                }
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const v4i p = *reinterpret_cast<const v4i*>(sb + ((wn * 8 + j) * 2 + c) * kChunkBytes + lane * 16);
                    const v4i be = (p << 4) & (int)0xF0F0F0F0;
                    const v4i bo = p & (int)0xF0F0F0F0;
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        acc[j][i] = __builtin_amdgcn_mfma_i32_16x16x64_i8(be, fe[i], acc[j][i], 0, 0, 0);
                        acc[j][i] = __builtin_amdgcn_mfma_i32_16x16x64_i8(bo, fo[i], acc[j][i], 0, 0, 0);
                    }
                }
            }
        }
        if (s + 1 < stages) store_stage(buf ^ 1);
        if (s + 1 == a.stages_hi) fold(a.s_hi, sw_hi, a.dbg_hi, 0);
        __syncthreads();
    }
    if (a.stages_lo > 0) fold(a.s_lo, sw_lo, a.dbg_lo, 8);

    // ---- write y once --------------------------------------------------------
    const bool vec_ok = ((reinterpret_cast<uintptr_t>(a.y) & 7) == 0) && (a.ldy % 4 == 0);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int64_t m = tok0 + 16 * i;
        if (m >= a.M) continue;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int64_t n = ch0 + 16 * j;
            uint16_t o[4];
#pragma unroll
            for (int v = 0; v < 4; ++v) o[v] = f32_to_bf16_rne(part[j][i][v]);
            uint16_t* dst = a.y + m * a.ldy + n;
            if (vec_ok && n + 3 < a.L.N) {
                *reinterpret_cast<uint2*>(dst) =
                    make_uint2((uint32_t)o[0] | ((uint32_t)o[1] << 16), (uint32_t)o[2] | ((uint32_t)o[3] << 16));
            } else {
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    if (n + v < a.L.N) dst[v] = o[v];
            }
        }
    }
}

}  // namespace resq
