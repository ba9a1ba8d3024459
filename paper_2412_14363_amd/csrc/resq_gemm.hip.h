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
// Global -> LDS copies use the direct-to-LDS load (16 bytes per lane, the LDS
// destination is a wave-uniform base plus 16 * lane), so no registers are spent
// on staging; three LDS buffers keep two stages in flight behind the one being
// multiplied, with one workgroup barrier per stage.  The three buffers are
// separate __shared__ arrays and the stage loop is unrolled by three so that
// every LDS access names its array statically: the compiler then only waits
// for the loads that fill the buffer it is about to read.
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

#include <type_traits>

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
constexpr int kAChunksPerWave = kStageABytes / kChunkBytes / 4;  // 4
constexpr int kBChunksPerWave = kStageBBytes / kChunkBytes / 4;  // 8
constexpr int kLoadsPerStage = kAChunksPerWave + kBChunksPerWave;  // per lane

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

// Wait until at most N of this wave's vector-memory loads are outstanding, then
// join the workgroup barrier.  Written as one asm statement with a memory
// clobber: the compiler may not move LDS accesses across it, and, unlike
// __syncthreads(), it does not drain the loads of the stages still in flight.
template <int N>
__device__ __forceinline__ void wait_loads_and_barrier() {
    asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(N) : "memory");
}

__device__ __forceinline__ void load_to_lds_16B(const uint8_t* g, uint8_t* lds_wave_base) {
    __builtin_amdgcn_global_load_lds(
        (const __attribute__((address_space(1))) void*)g,
        (__attribute__((address_space(3))) void*)lds_wave_base, 16, 0, 0);
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

// 16-byte LDS read whose completion the compiler does not track: the caller
// pairs it with lds_wait<N>() on the same register before using the value.
// (Reads the compiler can see would each be preceded by a wait for every
// direct-to-LDS load in flight, which would serialize the pipeline.)
template <int OFF>
__device__ __forceinline__ void lds_read16(v4i& dst, uint32_t addr) {
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=&v"(dst) : "v"(addr), "n"(OFF));
}
// Wait until every LDS read has returned.  The twelve registers are tied to
// the wait as in/out operands so that no use of them can be scheduled above it.
__device__ __forceinline__ void lds_wait_all(v4i& a0, v4i& a1, v4i& a2, v4i& a3, v4i& b0, v4i& b1,
                                             v4i& b2, v4i& b3, v4i& b4, v4i& b5, v4i& b6,
                                             v4i& b7) {
    asm volatile("s_waitcnt lgkmcnt(0)"
                 : "+v"(a0), "+v"(a1), "+v"(a2), "+v"(a3), "+v"(b0), "+v"(b1), "+v"(b2), "+v"(b3),
                   "+v"(b4), "+v"(b5), "+v"(b6), "+v"(b7));
}

template <bool DBG>
__global__ __launch_bounds__(kGemmThreads) void gemm_mixed_kernel(const GemmArgs a) {
    __shared__ __attribute__((aligned(1024))) uint8_t lds[3 * kStageBytes];

    const int t = threadIdx.x;
    const int lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int wm = wave >> 1;  // 0..1: 64-token half of the tile
    const int wn = wave & 1;   // 0..1: 128-channel half of the tile
    int tile_m, tile_n;
    tile_of_block(a, tile_m, tile_n);
    const int64_t m0 = (int64_t)tile_m * kBM;
    const int64_t n0 = (int64_t)tile_n * kBN;

    // ---- what this lane copies per stage ---------------------------------------
    // Wave w fills chunks 4w..4w+3 of the A image and 8w..8w+7 of the B image.
    // A chunk q (= 16-token block q/2, 64-byte half q%2): lane l fetches token row
    // (l % 16), 16-byte piece (l / 16); rows past M are clamped to the last row
    // (their results are never stored).  A B chunk is 1 KiB contiguous in HBM.
    const uint8_t* a_src[kAChunksPerWave];
    const uint8_t* b_src[kBChunksPerWave];
    auto set_sources = [&](const uint8_t* q, int64_t ld, int64_t b_chunk0) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < kAChunksPerWave; ++i) {
            const int chunk = wave * kAChunksPerWave + i;
            int64_t row = m0 + (chunk >> 1) * 16 + (lane & 15);
            row = row < a.M ? row : a.M - 1;
            a_src[i] = q + row * ld + (chunk & 1) * 64 + (lane >> 4) * 16;
        }
#pragma unroll
        for (int i = 0; i < kBChunksPerWave; ++i) {
            const int chunk = wave * kBChunksPerWave + i;
            b_src[i] = a.packed + (n0 / 16 + (chunk >> 1)) * a.L.block_bytes +
                       (b_chunk0 + (chunk & 1)) * kChunkBytes + lane * 16;
        }
    };
    auto issue_stage = [&](int s, int buf) __attribute__((always_inline)) {
        uint8_t* dst = lds + buf * kStageBytes;
#pragma unroll
        for (int i = 0; i < kAChunksPerWave; ++i)
            load_to_lds_16B(a_src[i] + (int64_t)s * 128,
                            dst + (wave * kAChunksPerWave + i) * kChunkBytes);
#pragma unroll
        for (int i = 0; i < kBChunksPerWave; ++i)
            load_to_lds_16B(b_src[i] + (int64_t)s * 2 * kChunkBytes,
                            dst + kStageABytes + (wave * kBChunksPerWave + i) * kChunkBytes);
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

    // LDS byte addresses of this lane's operand pieces in buffer 0
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t*)lds;
    const uint32_t a_addr0 = lds0 + wm * 4 * 2 * kChunkBytes + lane * 16;
    const uint32_t b_addr0 = lds0 + kStageABytes + wn * 8 * 2 * kChunkBytes + lane * 16;

    // fragments of one 64-byte chunk: 4 activation pieces, 8 weight pieces
    struct Frags {
        v4i fa[4];
        v4i fb[8];
    };
    // issue the 12 reads of chunk C of the stage in buffer `buf`
    auto read_chunk = [&](auto chunk, Frags& f, int buf) __attribute__((always_inline)) {
        constexpr int C = decltype(chunk)::value;
        const uint32_t aa = a_addr0 + buf * kStageBytes, bb = b_addr0 + buf * kStageBytes;
        lds_read16<(0 * 2 + C) * kChunkBytes>(f.fa[0], aa);
        lds_read16<(1 * 2 + C) * kChunkBytes>(f.fa[1], aa);
        lds_read16<(2 * 2 + C) * kChunkBytes>(f.fa[2], aa);
        lds_read16<(3 * 2 + C) * kChunkBytes>(f.fa[3], aa);
        lds_read16<(0 * 2 + C) * kChunkBytes>(f.fb[0], bb);
        lds_read16<(1 * 2 + C) * kChunkBytes>(f.fb[1], bb);
        lds_read16<(2 * 2 + C) * kChunkBytes>(f.fb[2], bb);
        lds_read16<(3 * 2 + C) * kChunkBytes>(f.fb[3], bb);
        lds_read16<(4 * 2 + C) * kChunkBytes>(f.fb[4], bb);
        lds_read16<(5 * 2 + C) * kChunkBytes>(f.fb[5], bb);
        lds_read16<(6 * 2 + C) * kChunkBytes>(f.fb[6], bb);
        lds_read16<(7 * 2 + C) * kChunkBytes>(f.fb[7], bb);
    };
    auto wait_chunk = [&](Frags& f) __attribute__((always_inline)) {
        lds_wait_all(f.fa[0], f.fa[1], f.fa[2], f.fa[3], f.fb[0], f.fb[1], f.fb[2], f.fb[3],
                     f.fb[4], f.fb[5], f.fb[6], f.fb[7]);
    };
    auto mma_chunk = [&](auto is_lo, Frags& f) __attribute__((always_inline)) {
        if constexpr (decltype(is_lo)::value) {
            v4i fe[4], fo[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                fe[i] = (f.fa[i] << 4) & (int)0xF0F0F0F0;
                fo[i] = f.fa[i] & (int)0xF0F0F0F0;
            }
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const v4i be = (f.fb[j] << 4) & (int)0xF0F0F0F0;
                const v4i bo = f.fb[j] & (int)0xF0F0F0F0;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    acc[j][i] = __builtin_amdgcn_mfma_i32_16x16x64_i8(be, fe[i], acc[j][i], 0, 0, 0);
                    acc[j][i] = __builtin_amdgcn_mfma_i32_16x16x64_i8(bo, fo[i], acc[j][i], 0, 0, 0);
                }
            }
        } else {
#pragma unroll
            for (int j = 0; j < 8; ++j)
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    acc[j][i] = __builtin_amdgcn_mfma_i32_16x16x64_i8(f.fb[j], f.fa[i], acc[j][i], 0, 0, 0);
        }
    };

    // One group's stages; the buffer of stage s is s % 3, and up to two stages
    // are in flight behind the one being multiplied.  At the top of stage s
    // every wave waits for its own loads of stage s (those of stage s + 1 may
    // stay in flight) and joins the barrier: stage s is then visible to all,
    // and every wave is done with stage s - 1, whose buffer the loads of stage
    // s + 2 then overwrite.  Each stage is two chunks; the reads of the second
    // are issued before the matrix instructions of the first, which hide them.
    auto run_group = [&](auto is_lo, int stages) __attribute__((always_inline)) {
        using C0 = std::integral_constant<int, 0>;
        using C1 = std::integral_constant<int, 1>;
        wait_loads_and_barrier<0>();  // the previous group's buffers are no longer read
        issue_stage(0, 0);
        if (stages > 1) issue_stage(1, 1);
        int buf = 0;
        for (int s = 0; s < stages; ++s) {
            const int prv = buf == 0 ? 2 : buf - 1;
            if (s + 1 < stages) wait_loads_and_barrier<kLoadsPerStage>();
            else wait_loads_and_barrier<0>();
            if (s + 2 < stages) issue_stage(s + 2, prv);
            Frags x, y;
            read_chunk(C0{}, x, buf);
            wait_chunk(x);
            read_chunk(C1{}, y, buf);
            mma_chunk(is_lo, x);
            wait_chunk(y);
            mma_chunk(is_lo, y);
            buf = buf == 2 ? 0 : buf + 1;
        }
    };

    // per-lane coordinates of the epilogue
    const int64_t tok0 = m0 + wm * 64 + (lane & 15);
    const int64_t ch0 = n0 + wn * 128 + (lane >> 4) * 4;
    const uint16_t* sw_hi = reinterpret_cast<const uint16_t*>(a.packed + a.L.scale_off);
    const uint16_t* sw_lo = sw_hi + a.L.n_pad;

    // part += (acc >> shift) * s_tok[m] * s_ch[n]; acc = 0
    auto fold = [&](const float* s_tok, const uint16_t* s_ch, int32_t* dbg, int shift) __attribute__((always_inline)) {
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
                    if constexpr (DBG) {
                        if (dbg && m < a.M && n + v < a.L.N) dbg[m * a.L.N + n + v] = iv;
                    }
                    acc[j][i][v] = 0;
                }
                // keep the fp32 tile in accumulation registers while the other
                // group's loop needs the ordinary ones for operands
                asm volatile("" : "+a"(part[j][i]));
            }
        }
    };

    if (a.stages_hi > 0) {
        set_sources(a.q_hi, a.ld_hi, 0);
        run_group(std::false_type{}, a.stages_hi);
        fold(a.s_hi, sw_hi, a.dbg_hi, 0);
    }
    if (a.stages_lo > 0) {
        set_sources(a.q_lo, a.ld_lo, a.L.hi_chunks);
        run_group(std::true_type{}, a.stages_lo);
        fold(a.s_lo, sw_lo, a.dbg_lo, 8);
    }

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
