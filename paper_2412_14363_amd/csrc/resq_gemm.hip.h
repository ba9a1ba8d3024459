// Tiled mixed INT8/INT4 GEMM with dequantizing epilogue (Section 4.1, Eq. 4):
//   A_hi = q_hi * w_hi^T over the high group, A_lo = q_lo * w_lo^T over the low
//   group, y = bf16(A_hi * s_hi[m] * sw_hi[n] + A_lo * s_lo[m] * sw_lo[n]).
//
// Tiling.  One workgroup of 4 wavefronts owns a 128 (tokens) x 256 (channels)
// output tile; each wavefront owns 64 x 128 of it as 2 x 4 tiles of the
// 32x32x32 int8 matrix-core instruction, the weights as its first operand so
// that a lane ends up with four consecutive channels of one token.
//
// Stages.  The reduction axis is walked in stages of 64 bytes per row: 64 int8
// codes of the high group or 128 nibble codes of the low group, i.e. two
// matrix-core steps of 32 bytes.  High and low stages form one sequence; the
// global->LDS copy is the same for both.  Six LDS buffers of 24 KiB hold the
// stage being multiplied, the next one, and up to four in flight.
//
// Global -> LDS.  The direct-to-LDS load moves 16 bytes per lane to a
// wave-uniform LDS base plus 16 * lane, so the LDS image is fixed by which
// global address each lane asks for.  A block (16 rows x 64 bytes) is stored
// with piece kc (16 bytes) of row r at unit 4 r + (kc ^ (r >> 2)): four
// consecutive lanes fetch one row's 64 contiguous bytes, and the 16 lanes that
// later read the same piece of 16 different rows hit 16 different bank groups.
//
// LDS -> registers.  Operand reads are issued as untracked ds_read_b128 (inline
// asm) and paired with an explicit wait: reads the compiler can see would each
// be preceded by a wait for every direct-to-LDS load still in flight.
//
// Software pipeline.  Low steps: read(k+2) | widen(k+1) | multiply(k), so that
// the matrix instructions of step k never wait for the vector ALU work of
// their own operands.  High steps need no widening: read(k+1) lands in the
// operand registers themselves while step k is multiplied.  The epilogue's
// per-channel and per-token constants (3.5 KiB) are fetched into LDS by the
// first loads of the kernel.
//
// The low group.  A lane's 16 packed bytes hold 32 codes, and each nibble is
// widened to an int8 operand with one AND (the vector ALU has room for about
// four instructions per matrix instruction, so every one counts).  In an
// activation byte the low nibble is c_even + 8 and the high nibble c_odd; in a
// weight byte the high nibble is w_even and the low nibble w_odd + 8.  Then
//   (pa & 0x0F) * (pw & 0xF0) = (c_even + 8) * 16 w_even
//   (pa & 0xF0) * (pw & 0x0F) = 16 c_odd * (w_odd + 8)
// feed two matrix-core instructions, and the accumulator ends as
//   16 * A_lo + 128 * (sum_even w[n] + sum_odd c[m]);
// the two sums are known per channel (packed with the weights) and per token
// (written by the quantizer), so A_lo is recovered exactly.
//
// Two scale pairs, one output write.  Each group has its own int32 tile in
// accumulation registers (2 x 128 per lane); both are folded into the output
// at the end, and y is written once, through LDS so that every store
// instruction writes whole 256-byte row segments.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>
#include <utility>

#include "resq_layout.h"

namespace resq {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int kGemmThreads = 256;
constexpr int kBM = 128;
constexpr int kBN = 256;
constexpr int kStageABytes = kBM * kRowBytes;  // 8 KiB = 8 blocks
constexpr int kStageBBytes = kBN * kRowBytes;  // 16 KiB = 16 blocks
constexpr int kStageBytes = kStageABytes + kStageBBytes;
constexpr int kNumBuf = 6;
constexpr int kPrefetch = kNumBuf - 1;  // stages requested ahead of the one being multiplied
constexpr int kLoadsPerStage = (kBM + kBN) / kRowsPerBlock / 4;  // per lane: 6
constexpr int kOutRowBytes = 128 * 2 + 16;  // one wave-tile row of bf16 in LDS, padded
// After the stage buffers: the tile's per-channel and per-token constants of the
// epilogue, copied there by the first loads of the kernel.
constexpr int kMetaOff = kNumBuf * kStageBytes;
constexpr int kMetaSwHi = 0;       // fp16 [256] high-group weight scales
constexpr int kMetaSwLo = 512;     // fp16 [256] low-group weight scales
constexpr int kMetaEven = 1024;    // int32 [256] even-column code sums of the low group
constexpr int kMetaSHi = 2048;     // fp32 [128] high-group token scales
constexpr int kMetaSLo = 2560;     // fp32 [128] low-group token scales
constexpr int kMetaLoSum = 3072;   // int32 [128] odd-column code sums of the low group
// only for asymmetric activation codes:
constexpr int kMetaWsumHi = 3584;  // int32 [256] sums of the high weight codes
constexpr int kMetaWsumLo = 4608;  // int32 [256] sums of the low weight codes
constexpr int kMetaCHi = 5632;     // fp32 [128] real value of the stored high code 0, per token
constexpr int kMetaCLo = 6144;     // fp32 [128] the same for the low group
constexpr int kMetaBytes = 6656;

struct GemmArgs {
    const uint8_t* q_hi;
    const uint8_t* q_lo;
    int64_t ld_hi, ld_lo;
    const float* s_hi;
    const float* s_lo;
    const int32_t* lo_sum;  // per token: sum of the low codes in odd columns
    const float* c_hi;      // asymmetric activation codes only (else null): per token, the real
    const float* c_lo;      // value that the stored code 0 of the group stands for
    const uint8_t* packed;
    WeightLayout L;
    int64_t M;
    uint16_t* y;
    int64_t ldy;
    int32_t* dbg_hi;
    int32_t* dbg_lo;
    int stages_hi, stages_lo;
    int tiles_m, tiles_n;
    int swiglu;  // 1: channels 2c and 2c+1 are the gate and the up row of feature c; y[m, c] = silu(gate) * up
};

// x * sigmoid(x) with the hardware exponential and reciprocal (well inside the
// output tolerance)
__device__ __forceinline__ float silu_f32(float x) {
    return x * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.44269504f * x));
}

__device__ __forceinline__ float fp16_bits_to_f32(uint32_t h) {
    return __uint_as_float((((h >> 10) & 0x1Fu) + 112u) << 23 | (h & 0x3FFu) << 13);
}

typedef int v2i __attribute__((ext_vector_type(2)));
typedef _Float16 v4h __attribute__((ext_vector_type(4)));

// two fp32 -> two bf16 (round to nearest even) in one dword, low half first
typedef float v2f __attribute__((ext_vector_type(2)));
typedef __bf16 v2bf __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
    const v2bf r = __builtin_convertvector((v2f){lo, hi}, v2bf);
    return *reinterpret_cast<const uint32_t*>(&r);
}

// Wait until at most N of this wave's vector-memory loads are outstanding, then
// join the workgroup barrier.  One asm statement with a memory clobber: the
// compiler may not move LDS accesses across it, and, unlike __syncthreads(),
// it does not drain the loads of the stages still in flight.
template <int N>
__device__ __forceinline__ void wait_loads_and_barrier() {
    asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(N) : "memory");
}
// the same with N = 6 * later, later = 0..4 stages allowed to stay in flight
__device__ __forceinline__ void wait_stage_and_barrier(int later) {
    if (later >= 4) wait_loads_and_barrier<4 * kLoadsPerStage>();
    else if (later == 3) wait_loads_and_barrier<3 * kLoadsPerStage>();
    else if (later == 2) wait_loads_and_barrier<2 * kLoadsPerStage>();
    else if (later == 1) wait_loads_and_barrier<1 * kLoadsPerStage>();
    else wait_loads_and_barrier<0>();
}

// direct-to-LDS loads: lane l's 16 (4) bytes land at lds_wave_base + 16 (4) * l
__device__ __forceinline__ void load_to_lds_16B(const void* g, uint8_t* lds_wave_base) {
    __builtin_amdgcn_global_load_lds(
        (const __attribute__((address_space(1))) void*)g,
        (__attribute__((address_space(3))) void*)lds_wave_base, 16, 0, 0);
}
__device__ __forceinline__ void load_to_lds_4B(const void* g, uint8_t* lds_wave_base) {
    __builtin_amdgcn_global_load_lds(
        (const __attribute__((address_space(1))) void*)g,
        (__attribute__((address_space(3))) void*)lds_wave_base, 4, 0, 0);
}

// untracked LDS reads (the compiler does not know these touch LDS)
template <int OFF>
__device__ __forceinline__ void lds_read16(v4i& dst, uint32_t addr) {
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=&v"(dst) : "v"(addr), "n"(OFF));
}
template <int OFF>
__device__ __forceinline__ void lds_read8(v2i& dst, uint32_t addr) {
    asm volatile("ds_read_b64 %0, %1 offset:%2" : "=&v"(dst) : "v"(addr), "n"(OFF));
}
template <int OFF>
__device__ __forceinline__ void lds_read4(int& dst, uint32_t addr) {
    asm volatile("ds_read_b32 %0, %1 offset:%2" : "=&v"(dst) : "v"(addr), "n"(OFF));
}

// packed fragments of one reduction step as read from LDS:
// 2 activation tiles and 4 weight tiles of 32 rows x 32 bytes
struct Packed {
    v4i fa[2];
    v4i fb[4];
};
// matrix-core operands of one reduction step: for a low step the even-code and
// odd-code halves of every fragment; for a high step only the e members are used
struct Operands {
    v4i ae[2], ao[2];
    v4i be[4], bo[4];
};

// Wait until every LDS read has returned.  The registers are tied to the wait
// as in/out operands so that no use of them can be scheduled above it.
__device__ __forceinline__ void lds_wait_all(Packed& f) {
    asm volatile("s_waitcnt lgkmcnt(0)"
                 : "+v"(f.fa[0]), "+v"(f.fa[1]), "+v"(f.fb[0]), "+v"(f.fb[1]), "+v"(f.fb[2]),
                   "+v"(f.fb[3]));
}

// Wait until at most N LDS reads are outstanding (they return in order); ties the
// e members of an operand set, which high steps read into directly.
template <int N>
__device__ __forceinline__ void lds_wait_operands(Operands& u) {
    asm volatile("s_waitcnt lgkmcnt(%6)"
                 : "+v"(u.ae[0]), "+v"(u.ae[1]), "+v"(u.be[0]), "+v"(u.be[1]), "+v"(u.be[2]), "+v"(u.be[3])
                 : "n"(N));
}

// blockIdx -> (tile_m, tile_n).  Consecutive workgroup ids land on different
// XCDs (8 of them, 32 compute units and one L2 each), and an XCD runs its
// workgroups in id order, 32 at a time.  When the grid allows it, the 32 tiles
// an XCD works on together form an 8 x 4 patch (1024 tokens x 1024 channels),
// so that each activation stage is fetched into that L2 once per 4 tiles and
// each weight stage once per 8; the 8 XCDs take neighbouring patches.
__device__ __forceinline__ void tile_of_block(const GemmArgs& a, int& tm, int& tn) {
    const int total = a.tiles_m * a.tiles_n;
    const int id = blockIdx.x;
    if (total % 256 == 0 && a.tiles_m % 8 == 0 && a.tiles_n % 4 == 0) {
        const int xcd = id & 7, k = id >> 3;
        const int patch = (k >> 5) * 8 + xcd, within = k & 31;
        const int patches_m = a.tiles_m >> 3;
        tm = (patch % patches_m) * 8 + (within & 7);
        tn = (patch / patches_m) * 4 + (within >> 3);
    } else if (total % 8 == 0) {
        const int lin = (id & 7) * (total >> 3) + (id >> 3);
        tn = lin / a.tiles_m;
        tm = lin % a.tiles_m;
    } else {
        tn = id / a.tiles_m;
        tm = id % a.tiles_m;
    }
}

template <int N>
using IC = std::integral_constant<int, N>;
// f(IC<0>), f(IC<1>), ..., f(IC<N-1>)
template <class F, int... Is>
__device__ __forceinline__ void static_for_impl(F&& f, std::integer_sequence<int, Is...>) {
    (f(IC<Is>{}), ...);
}
template <int N, class F>
__device__ __forceinline__ void static_for(F&& f) {
    static_for_impl(f, std::make_integer_sequence<int, N>{});
}

template <bool DBG>
__global__ __launch_bounds__(kGemmThreads) void gemm_mixed_kernel(const GemmArgs a) {
    __shared__ __attribute__((aligned(1024))) uint8_t lds[kMetaOff + kMetaBytes];

    const int t = threadIdx.x;
    const int lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int wm = wave >> 1;  // 0..1: 64-token half of the tile
    const int wn = wave & 1;   // 0..1: 128-channel half of the tile
    int tile_m, tile_n;
    tile_of_block(a, tile_m, tile_n);
    const int64_t m0 = (int64_t)tile_m * kBM;
    const int64_t n0 = (int64_t)tile_n * kBN;
    const int S_hi = a.stages_hi, S_lo = a.stages_lo, S = S_hi + S_lo;
    const uint16_t* sw_hi = reinterpret_cast<const uint16_t*>(a.packed + a.L.scale_off);
    const uint16_t* sw_lo = sw_hi + a.L.n_pad;
    const int32_t* even_sum = reinterpret_cast<const int32_t*>(a.packed + a.L.scale_off + 4 * a.L.n_pad);
    const bool asym = a.c_hi != nullptr || a.c_lo != nullptr;

    // ---- epilogue constants -> LDS ---------------------------------------------
    // These are the oldest loads of every wave, so the first wait for a stage
    // covers them.  Token rows past M repeat the last row (never stored).
    if (wave == 0) {
        load_to_lds_16B((lane < 32 ? sw_hi : sw_lo) + n0 + (lane & 31) * 8, lds + kMetaOff + kMetaSwHi);
        if (asym) load_to_lds_16B(even_sum + a.L.n_pad + n0 + lane * 4, lds + kMetaOff + kMetaWsumHi);
    } else if (wave == 1) {
        load_to_lds_16B(even_sum + n0 + lane * 4, lds + kMetaOff + kMetaEven);
        if (asym) load_to_lds_16B(even_sum + 2 * a.L.n_pad + n0 + lane * 4, lds + kMetaOff + kMetaWsumLo);
    } else {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            int64_t m = m0 + h * 64 + lane;
            m = m < a.M ? m : a.M - 1;
            if (wave == 2) {
                if (S_hi > 0) load_to_lds_4B(a.s_hi + m, lds + kMetaOff + kMetaSHi + h * 256);
                if (S_lo > 0) load_to_lds_4B(a.s_lo + m, lds + kMetaOff + kMetaSLo + h * 256);
            } else {
                if (S_lo > 0) load_to_lds_4B(a.lo_sum + m, lds + kMetaOff + kMetaLoSum + h * 256);
                if (asym && S_hi > 0) load_to_lds_4B(a.c_hi + m, lds + kMetaOff + kMetaCHi + h * 256);
                if (asym && S_lo > 0) load_to_lds_4B(a.c_lo + m, lds + kMetaOff + kMetaCLo + h * 256);
            }
        }
    }

    // ---- global -> LDS copy --------------------------------------------------
    // One load instruction fills one block: lane l fetches row l / 4, piece
    // (l % 4) ^ (l / 16).  Wave w copies A blocks 2w, 2w+1 and B blocks 4w..4w+3
    // of each stage.  Token rows past M are clamped to the last row (their
    // results are never stored).  The weight blocks of one 16-channel group are
    // contiguous over all stages, high ones first.  Every address is a
    // wave-uniform base (scalar registers, advanced per stage) plus a 32-bit
    // per-lane offset that never changes.
    uint32_t a_voff_hi[2], a_voff_lo[2], b_voff;
    const uint8_t* a_base_hi = a.q_hi + m0 * a.ld_hi;
    const uint8_t* a_base_lo = a.q_lo + m0 * a.ld_lo - (int64_t)S_hi * kRowBytes;
    const uint8_t* b_base = a.packed + (n0 / 16 + wave * 4) * a.L.group_bytes;
    {
        const int r = lane >> 2, kc = (lane & 3) ^ (lane >> 4);
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            int64_t row = (wave * 2 + i) * 16 + r;
            row = m0 + row < a.M ? row : a.M - 1 - m0;
            a_voff_hi[i] = (uint32_t)(row * a.ld_hi + kc * 16);
            a_voff_lo[i] = (uint32_t)(row * a.ld_lo + kc * 16);
        }
        b_voff = r * kRowBytes + kc * 16;
    }
    // load K of stage sg (0 .. S-1, high stages first) into buffer buf; K = 0, 1: A blocks, 2..5: B blocks
    auto issue_load = [&](auto k, int sg, int buf) __attribute__((always_inline)) {
        constexpr int K = decltype(k)::value;
        uint8_t* dst = lds + buf * kStageBytes;
        if constexpr (K < 2) {
            const bool lo = sg >= S_hi;
            const uint8_t* base = (lo ? a_base_lo : a_base_hi) + (int64_t)sg * kRowBytes;
            load_to_lds_16B(base + (lo ? a_voff_lo[K] : a_voff_hi[K]), dst + (wave * 2 + K) * kBlockBytes);
        } else {
            const uint8_t* base = b_base + (K - 2) * a.L.group_bytes + (int64_t)sg * kBlockBytes;
            // the lane offset is made opaque here so that it is not folded into a per-lane
            // 64-bit pointer outside the loop: the load takes a scalar base plus a 32-bit offset
            uint32_t voff = b_voff;
            asm volatile("" : "+v"(voff));
            load_to_lds_16B(base + voff, dst + kStageABytes + (wave * 4 + K - 2) * kBlockBytes);
        }
    };

    // ---- accumulators ----------------------------------------------------------
    // One int32 tile per group, both in accumulation registers for the whole
    // kernel (2 x 128), folded into the output together at the end.
    // acc[j][i]: channels 32 j.., tokens 32 i.. of the wave tile.  Lane l holds
    // token (l % 32) and, in element v, channel 8 (v / 4) + 4 (l / 32) + v % 4.
    v16i acc_hi[4][2], acc_lo[4][2];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                acc_hi[j][i][v] = 0;
                acc_lo[j][i][v] = 0;
            }

    // The tile that a loop does not touch stays where it is, in accumulation
    // registers: stating so in every stage keeps the register allocator from
    // moving it to ordinary registers and back around the loops (128 moves a time).
    auto park = [&](v16i (&acc)[4][2]) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int i = 0; i < 2; ++i) asm volatile("" : "+a"(acc[j][i]));
    };

    // ---- LDS -> register reads ---------------------------------------------------
    // An operand tile is 32 rows x 64 bytes (two blocks).  In step st (0, 1) of a
    // stage lane l supplies row (l % 32), piece 2 st + l / 32.
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t*)lds;
    uint32_t a_off[2], b_off[2];
    {
        const int R = lane & 31, r = R & 15, g = lane >> 5;
#pragma unroll
        for (int st = 0; st < 2; ++st) {
            const int kc = 2 * st + g;
            const uint32_t off = (R >> 4) * kBlockBytes + (4 * r + (kc ^ (r >> 2))) * 16;
            a_off[st] = lds0 + wm * (4 * kBlockBytes) + off;
            b_off[st] = lds0 + kStageABytes + wn * (8 * kBlockBytes) + off;
        }
    }
    // read K of a step: K = 0, 1: activation fragments, 2..5: weight fragments
    auto read_frag = [&](auto k, Packed& f, uint32_t aa, uint32_t bb) __attribute__((always_inline)) {
        constexpr int K = decltype(k)::value;
        if constexpr (K < 2) lds_read16<K * 2 * kBlockBytes>(f.fa[K], aa);
        else lds_read16<(K - 2) * 2 * kBlockBytes>(f.fb[K - 2], bb);
    };
    // the same read into the e members of an operand set (high steps need no widening)
    auto read_operand = [&](auto k, Operands& u, uint32_t aa, uint32_t bb) __attribute__((always_inline)) {
        constexpr int K = decltype(k)::value;
        if constexpr (K < 2) lds_read16<K * 2 * kBlockBytes>(u.ae[K], aa);
        else lds_read16<(K - 2) * 2 * kBlockBytes>(u.be[K - 2], bb);
    };
    // piece P (0..11) of the widening of one low step's fragments: one AND over a fragment
    auto widen_piece = [&](auto p, const Packed& f, Operands& u) __attribute__((always_inline)) {
        constexpr int P = decltype(p)::value;
        if constexpr (P < 2) u.ae[P] = f.fa[P] & (int)0x0F0F0F0F;           // even columns: code + 8
        else if constexpr (P < 4) u.ao[P - 2] = f.fa[P - 2] & (int)0xF0F0F0F0;  // odd columns: 16 * code
        else if constexpr (P < 8) u.be[P - 4] = f.fb[P - 4] & (int)0xF0F0F0F0;  // even columns: 16 * code
        else u.bo[P - 8] = f.fb[P - 8] & (int)0x0F0F0F0F;                        // odd columns: code + 8
    };
    // matrix instruction Q of a step (8 per high step, 16 per low step), in an
    // order that keeps two instructions on the same accumulator eight apart
    auto mfma = [&](auto q, const Operands& u, v16i (&acc)[4][2]) __attribute__((always_inline)) {
        constexpr int Q = decltype(q)::value;
        constexpr int j = (Q & 7) >> 1, i = Q & 1;
        if constexpr (Q < 8)
            acc[j][i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(u.be[j], u.ae[i], acc[j][i], 0, 0, 0);
        else
            acc[j][i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(u.bo[j], u.ao[i], acc[j][i], 0, 0, 0);
    };

    // ---- epilogue pieces -------------------------------------------------------------
    // Lane coordinates inside the tile: token tl + 32 i, channel cl + 32 j + 8 vq + vr.
    const int tl = wm * 64 + (lane & 31);
    const int cl = wn * 128 + (lane >> 5) * 4;
    uint8_t* const out_stage = lds + wave * (64 * kOutRowBytes);

    // Fold both integer tiles into the output:
    //   y = A_hi * s_hi[m] * sw_hi[n] + A_lo * s_lo[m] * sw_lo[n]
    // A_hi is its accumulator; A_lo = (acc_lo - 128 * (even_sum[n] + lo_sum[m])) / 16,
    // an exact division whose 1/16 is folded into the scale outside the debug
    // kernel (same fp32 product).  The result is rounded to bf16 and staged in
    // LDS, row-padded, for the row-segment stores.  The constants come from LDS
    // (no direct-to-LDS load is in flight any more: ordinary loads).
    // ASYM (asymmetric activation codes, stored minus 2^(N-1)): each group gains the
    // zero-point term c[m] * wsum[n] * sw[n], c the real value of the stored code 0
    // and wsum the sum of the channel's weight codes (Eq. 1 inserted into Eq. 4).
    // GLU (gated pair epilogue): the lane's four consecutive channels are two (gate, up)
    // pairs; silu(gate) * up of each goes out, so the staged row is half as wide.
    auto fold = [&](auto has_hi, auto has_lo, auto is_asym, auto is_glu) __attribute__((always_inline)) {
        constexpr bool HI_ON = decltype(has_hi)::value, LO_ON = decltype(has_lo)::value;
        constexpr bool ASYM = decltype(is_asym)::value, GLU = decltype(is_glu)::value;
        const uint8_t* meta = lds + kMetaOff;
        float st_hi[2] = {0.f, 0.f}, st_lo[2] = {0.f, 0.f}, ct_hi[2] = {0.f, 0.f}, ct_lo[2] = {0.f, 0.f};
        int ca[2] = {0, 0};
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            if constexpr (HI_ON) st_hi[i] = *reinterpret_cast<const float*>(meta + kMetaSHi + (tl + 32 * i) * 4);
            if constexpr (ASYM && HI_ON) ct_hi[i] = *reinterpret_cast<const float*>(meta + kMetaCHi + (tl + 32 * i) * 4);
            if constexpr (ASYM && LO_ON) ct_lo[i] = *reinterpret_cast<const float*>(meta + kMetaCLo + (tl + 32 * i) * 4);
            if constexpr (LO_ON) {
                st_lo[i] = *reinterpret_cast<const float*>(meta + kMetaSLo + (tl + 32 * i) * 4);
                if constexpr (!DBG) st_lo[i] *= 0.0625f;
                ca[i] = 128 * *reinterpret_cast<const int*>(meta + kMetaLoSum + (tl + 32 * i) * 4);
            }
        }
        // debug dump of the integer sums: row pointers and the number of valid columns from cl on
        int32_t* dbg_row_hi[2] = {nullptr, nullptr};
        int32_t* dbg_row_lo[2] = {nullptr, nullptr};
        bool dbg_ok[2] = {false, false};
        int dbg_cols = 0;
        if constexpr (DBG) {
            dbg_cols = (int)(a.L.N - n0 - cl);
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int64_t m = m0 + tl + 32 * i;
                dbg_ok[i] = m < a.M;
                dbg_row_hi[i] = a.dbg_hi + m * a.L.N + n0 + cl;
                dbg_row_lo[i] = a.dbg_lo + m * a.L.N + n0 + cl;
            }
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
#pragma unroll
            for (int vq = 0; vq < 4; ++vq) {
                const int c = cl + 32 * j + 8 * vq;
                float sn_hi[4] = {0.f, 0.f, 0.f, 0.f}, sn_lo[4] = {0.f, 0.f, 0.f, 0.f};
                float zw_hi[4] = {0.f, 0.f, 0.f, 0.f}, zw_lo[4] = {0.f, 0.f, 0.f, 0.f};  // wsum[n] * sw[n]
                v4i ev = {0, 0, 0, 0};
                if constexpr (HI_ON) {
                    const v4h h = *reinterpret_cast<const v4h*>(meta + kMetaSwHi + c * 2);
#pragma unroll
                    for (int vr = 0; vr < 4; ++vr) sn_hi[vr] = (float)h[vr];
                    if constexpr (ASYM) {
                        const v4i ws = *reinterpret_cast<const v4i*>(meta + kMetaWsumHi + c * 4);
#pragma unroll
                        for (int vr = 0; vr < 4; ++vr) zw_hi[vr] = (float)ws[vr] * sn_hi[vr];
                    }
                }
                if constexpr (LO_ON) {
                    const v4h h = *reinterpret_cast<const v4h*>(meta + kMetaSwLo + c * 2);
#pragma unroll
                    for (int vr = 0; vr < 4; ++vr) sn_lo[vr] = (float)h[vr];
                    ev = *reinterpret_cast<const v4i*>(meta + kMetaEven + c * 4);
                    if constexpr (ASYM) {
                        const v4i ws = *reinterpret_cast<const v4i*>(meta + kMetaWsumLo + c * 4);
#pragma unroll
                        for (int vr = 0; vr < 4; ++vr) zw_lo[vr] = (float)ws[vr] * sn_lo[vr];
                    }
                }
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                    float val[4];
#pragma unroll
                    for (int vr = 0; vr < 4; ++vr) {
                        const int v = vq * 4 + vr;
                        val[vr] = 0.f;
                        if constexpr (HI_ON) {
                            const int ih = acc_hi[j][i][v];
                            val[vr] = (float)ih * (st_hi[i] * sn_hi[vr]);
                            if constexpr (ASYM) val[vr] += ct_hi[i] * zw_hi[vr];
                            if constexpr (DBG) {
                                if (a.dbg_hi && dbg_ok[i] && 32 * j + 8 * vq + vr < dbg_cols)
                                    dbg_row_hi[i][32 * j + 8 * vq + vr] = ih;
                            }
                        }
                        if constexpr (LO_ON) {
                            int il = acc_lo[j][i][v] - (ev[vr] * 128 + ca[i]);
                            if constexpr (DBG) il >>= 4;
                            val[vr] += (float)il * (st_lo[i] * sn_lo[vr]);
                            if constexpr (ASYM) val[vr] += ct_lo[i] * zw_lo[vr];
                            if constexpr (DBG) {
                                if (a.dbg_lo && dbg_ok[i] && 32 * j + 8 * vq + vr < dbg_cols)
                                    dbg_row_lo[i][32 * j + 8 * vq + vr] = il;
                            }
                        }
                    }
                    const int row = 32 * i + (lane & 31);
                    const int col = 32 * j + 8 * vq + 4 * (lane >> 5);
                    if constexpr (GLU)
                        *reinterpret_cast<uint32_t*>(out_stage + row * kOutRowBytes + col) =
                            pack_bf16(silu_f32(val[0]) * val[1], silu_f32(val[2]) * val[3]);
                    else
                        *reinterpret_cast<uint2*>(out_stage + row * kOutRowBytes + col * 2) =
                            make_uint2(pack_bf16(val[0], val[1]), pack_bf16(val[2], val[3]));
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // ---- main loop ---------------------------------------------------------------
    {
        Packed px, py;
        Operands ux, uy;
        const int ahead = S < kPrefetch ? S : kPrefetch;
        for (int i = 0; i < ahead; ++i)
            static_for<kLoadsPerStage>([&](auto k) __attribute__((always_inline)) { issue_load(k, i, i); });
        wait_stage_and_barrier(ahead - 1);  // stage 0 (and the epilogue constants) have landed everywhere
        if (S_hi > 0) {
            // high stages read straight into the operand registers
            static_for<6>([&](auto k) __attribute__((always_inline)) { read_operand(k, ux, a_off[0], b_off[0]); });
        } else {
            static_for<6>([&](auto k) __attribute__((always_inline)) { read_frag(k, px, a_off[0], b_off[0]); });
            lds_wait_all(px);
            static_for<6>([&](auto k) __attribute__((always_inline)) { read_frag(k, py, a_off[1], b_off[1]); });
            static_for<12>([&](auto p) __attribute__((always_inline)) { widen_piece(p, px, ux); });
        }

        int buf = 0;
        // A low stage = two pipeline slots (reduction steps) of 16 matrix
        // instructions.  ISSUE: this stage requests stage sg + kPrefetch (every
        // stage but the last kPrefetch ones).  A slot is a fixed sequence of groups,
        // one matrix instruction each, with the slot's other work dealt out among
        // them so that it issues in the shadow of the matrix pipeline (about four
        // vector ALU instructions, or a read and a load, fit behind one matrix
        // instruction):
        //   slot 0: multiply step 0 | wait + barrier after 4 groups | then per group one
        //           LDS read of the next stage's step 0 and one piece of step 1's widening
        //   slot 1: multiply step 1 | per group one LDS read of the next stage's step 1 and
        //           one piece of the next step 0's widening
        // and the stage's six global loads at even distances after the barrier.
        // Invariant at entry: ux = operands of (sg, step 0); the reads of (sg, step 1)
        // into py are in flight.
        auto stage_lo = [&](auto issue, int sg) __attribute__((always_inline)) {
            constexpr bool ISSUE = decltype(issue)::value;
            constexpr int NM = 16;               // matrix instructions per step
            constexpr int PRE = 4;               // ... of which this many go before the barrier
            constexpr int LD_EVERY = (NM - PRE) / 3;  // a global load every so many groups, three per slot
            const int nxt = buf == kNumBuf - 1 ? 0 : buf + 1;
            const int prv = buf == 0 ? kNumBuf - 1 : buf - 1;
            const uint32_t shift = nxt * kStageBytes;
            park(acc_hi);
            __builtin_amdgcn_sched_barrier(0);
            static_for<PRE>([&](auto q) __attribute__((always_inline)) { mfma(q, ux, acc_lo); });
            __builtin_amdgcn_sched_barrier(0);
            // stage sg + 1 has landed everywhere, and every wave is done with stage sg - 1;
            // stages sg + 2 .. sg + 4 may stay in flight
            if constexpr (ISSUE) {
                wait_loads_and_barrier<3 * kLoadsPerStage>();
            } else {
                const int rem = S - 2 - sg;
                wait_stage_and_barrier(rem > 3 ? 3 : rem);
            }
            lds_wait_all(py);
            __builtin_amdgcn_sched_barrier(0);
            static_for<NM - PRE>([&](auto g) __attribute__((always_inline)) {
                constexpr int G = decltype(g)::value;
                mfma(IC<PRE + G>{}, ux, acc_lo);
                // past the last stage the reads fetch stale LDS: harmless
                if constexpr (G < 6) read_frag(g, px, a_off[0] + shift, b_off[0] + shift);
                widen_piece(g, py, uy);
                if constexpr (ISSUE && G % LD_EVERY == LD_EVERY - 1)
                    issue_load(IC<G / LD_EVERY>{}, sg + kPrefetch, prv);
                __builtin_amdgcn_sched_barrier(0);
            });
            static_for<PRE>([&](auto q) __attribute__((always_inline)) { mfma(q, uy, acc_lo); });
            __builtin_amdgcn_sched_barrier(0);
            lds_wait_all(px);
            __builtin_amdgcn_sched_barrier(0);
            static_for<NM - PRE>([&](auto g) __attribute__((always_inline)) {
                constexpr int G = decltype(g)::value;
                mfma(IC<PRE + G>{}, uy, acc_lo);
                if constexpr (G < 6) read_frag(g, py, a_off[1] + shift, b_off[1] + shift);
                widen_piece(g, px, ux);
                if constexpr (ISSUE && G % LD_EVERY == LD_EVERY - 1)
                    issue_load(IC<3 + G / LD_EVERY>{}, sg + kPrefetch, prv);
                __builtin_amdgcn_sched_barrier(0);
            });
            buf = nxt;
        };
        // A high stage needs no widening, so its reads go straight into the operand
        // registers of the step after the one being multiplied (ux and uy take
        // turns) and the Packed sets are not used.  Invariant at entry: the reads
        // of (sg, step 0) into ux have been issued.  Per slot, 8 matrix
        // instructions M0..M7 with the 6 reads of the next step behind M0..M5 and
        // the waits placed so that each instruction only waits for its own
        // operands (activations first, then the weight fragments in order):
        //   before M0: <= 3 reads of this step outstanding; before M2: <= 2, and so
        //   on, each plus the reads of the next step issued by then.
        auto stage_hi = [&](auto issue, int sg) __attribute__((always_inline)) {
            constexpr bool ISSUE = decltype(issue)::value;
            const int nxt = buf == kNumBuf - 1 ? 0 : buf + 1;
            const int prv = buf == 0 ? kNumBuf - 1 : buf - 1;
            const uint32_t here = buf * kStageBytes, shift = nxt * kStageBytes;
            park(acc_lo);
            auto slot = [&](auto second, Operands& use, Operands& fill, uint32_t aa, uint32_t bb) __attribute__((always_inline)) {
                constexpr bool SECOND = decltype(second)::value;
                __builtin_amdgcn_sched_barrier(0);
                lds_wait_operands<3>(use);
                mfma(IC<0>{}, use, acc_hi);
                read_operand(IC<0>{}, fill, aa, bb);
                __builtin_amdgcn_sched_barrier(0);
                mfma(IC<1>{}, use, acc_hi);
                read_operand(IC<1>{}, fill, aa, bb);
                __builtin_amdgcn_sched_barrier(0);
                if constexpr (!SECOND) {
                    // stage sg + 1 has landed everywhere, and every wave is done with stage sg - 1;
                    // stages sg + 2 .. sg + 4 may stay in flight
                    if constexpr (ISSUE) {
                        wait_loads_and_barrier<3 * kLoadsPerStage>();
                    } else {
                        const int rem = S - 2 - sg;
                        wait_stage_and_barrier(rem > 3 ? 3 : rem);
                    }
                }
                lds_wait_operands<2 + 2>(use);
                mfma(IC<2>{}, use, acc_hi);
                read_operand(IC<2>{}, fill, aa, bb);
                __builtin_amdgcn_sched_barrier(0);
                mfma(IC<3>{}, use, acc_hi);
                read_operand(IC<3>{}, fill, aa, bb);
                if constexpr (ISSUE) issue_load(IC<SECOND ? 3 : 0>{}, sg + kPrefetch, prv);
                __builtin_amdgcn_sched_barrier(0);
                lds_wait_operands<1 + 4>(use);
                mfma(IC<4>{}, use, acc_hi);
                read_operand(IC<4>{}, fill, aa, bb);
                __builtin_amdgcn_sched_barrier(0);
                mfma(IC<5>{}, use, acc_hi);
                read_operand(IC<5>{}, fill, aa, bb);
                if constexpr (ISSUE) issue_load(IC<SECOND ? 4 : 1>{}, sg + kPrefetch, prv);
                __builtin_amdgcn_sched_barrier(0);
                lds_wait_operands<0 + 6>(use);
                mfma(IC<6>{}, use, acc_hi);
                __builtin_amdgcn_sched_barrier(0);
                mfma(IC<7>{}, use, acc_hi);
                if constexpr (ISSUE) issue_load(IC<SECOND ? 5 : 2>{}, sg + kPrefetch, prv);
                __builtin_amdgcn_sched_barrier(0);
            };
            // slot 0 multiplies (sg, step 0) and reads (sg, step 1); slot 1 multiplies that
            // and reads (sg + 1, step 0) -- stale LDS past the last stage, harmless
            slot(std::false_type{}, ux, uy, a_off[1] + here, b_off[1] + here);
            slot(std::true_type{}, uy, ux, a_off[0] + shift, b_off[0] + shift);
            buf = nxt;
        };
        using YES = std::true_type;
        using NO = std::false_type;
        const int issue_end = S - kPrefetch;  // stages below this one request a later stage
        int sg = 0;
        if (S_hi > 0) {
            // The last high stage reads the first low step like a high one (its packed
            // bytes land in ux), so that the loops need no stage of a mixed kind; they
            // are widened in place afterwards.
            for (; sg < S_hi && sg < issue_end; ++sg) stage_hi(YES{}, sg);
            for (; sg < S_hi; ++sg) stage_hi(NO{}, sg);
            lds_wait_operands<0>(ux);  // the packed bytes of the first low step (or stale ones)
            if (S_lo > 0) {
                static_for<6>([&](auto k) __attribute__((always_inline)) {
                    read_frag(k, py, a_off[1] + buf * kStageBytes, b_off[1] + buf * kStageBytes);
                });
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                    ux.ao[i] = ux.ae[i] & (int)0xF0F0F0F0;
                    ux.ae[i] = ux.ae[i] & (int)0x0F0F0F0F;
                }
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    ux.bo[j] = ux.be[j] & (int)0x0F0F0F0F;
                    ux.be[j] = ux.be[j] & (int)0xF0F0F0F0;
                }
            }
        }
        if (S_lo > 0) {
            for (; sg < issue_end; ++sg) stage_lo(YES{}, sg);
            for (; sg < S; ++sg) stage_lo(NO{}, sg);
            lds_wait_all(py);  // reads past the last stage: let them land
        }
        wait_loads_and_barrier<0>();  // every wave is done reading the stage buffers
        if (a.swiglu) {  // symmetric codes only (checked on the host)
            if (S_hi > 0 && S_lo > 0) fold(YES{}, YES{}, NO{}, YES{});
            else if (S_hi > 0) fold(YES{}, NO{}, NO{}, YES{});
            else fold(NO{}, YES{}, NO{}, YES{});
        } else if (asym) {
            if (S_hi > 0 && S_lo > 0) fold(YES{}, YES{}, YES{}, NO{});
            else if (S_hi > 0) fold(YES{}, NO{}, YES{}, NO{});
            else fold(NO{}, YES{}, YES{}, NO{});
        } else {
            if (S_hi > 0 && S_lo > 0) fold(YES{}, YES{}, NO{}, NO{});
            else if (S_hi > 0) fold(YES{}, NO{}, NO{}, NO{});
            else fold(NO{}, YES{}, NO{}, NO{});
        }
    }

    // ---- write y once --------------------------------------------------------
    // The wave's 64 x 128 bf16 tile sits in LDS; each store instruction writes
    // four whole 256-byte row segments.
    __syncthreads();
    const bool fast = ((reinterpret_cast<uintptr_t>(a.y) & 15) == 0) && (a.ldy % 8 == 0) &&
                      (n0 + kBN <= a.L.N);
    if (a.swiglu) {
        // 64 x 64 outputs per wave: eight 128-byte row segments per store instruction
        const int64_t n_out = a.L.N / 2;
#pragma unroll
        for (int it = 0; it < 8; ++it) {
            const int row = it * 8 + (lane >> 3);
            const int64_t m = m0 + wm * 64 + row;
            const int64_t n = n0 / 2 + wn * 64 + (lane & 7) * 8;
            const uint4 v = *reinterpret_cast<const uint4*>(out_stage + row * kOutRowBytes + (lane & 7) * 16);
            if (m >= a.M) continue;
            if (fast) {
                *reinterpret_cast<uint4*>(a.y + m * a.ldy + n) = v;
            } else {
                const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    if (n + e < n_out) a.y[m * a.ldy + n + e] = (uint16_t)(w[e >> 1] >> (16 * (e & 1)));
            }
        }
        return;
    }
#pragma unroll
    for (int it = 0; it < 16; ++it) {
        const int row = it * 4 + (lane >> 4);
        const int64_t m = m0 + wm * 64 + row;
        const int64_t n = n0 + wn * 128 + (lane & 15) * 8;
        const uint4 v = *reinterpret_cast<const uint4*>(out_stage + row * kOutRowBytes + (lane & 15) * 16);
        if (m >= a.M) continue;
        if (fast) {
            *reinterpret_cast<uint4*>(a.y + m * a.ldy + n) = v;
        } else {
            const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int e = 0; e < 8; ++e)
                if (n + e < a.L.N) a.y[m * a.ldy + n + e] = (uint16_t)(w[e >> 1] >> (16 * (e & 1)));
        }
    }
}

}  // namespace resq
