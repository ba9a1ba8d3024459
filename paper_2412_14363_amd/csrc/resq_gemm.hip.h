// Tiled mixed INT8/INT4 GEMM with dequantizing epilogue (Section 4.1, Eq. 4):
//   A_hi = q_hi * w_hi^T over the high group, A_lo = q_lo * w_lo^T over the low
//   group, y = bf16(A_hi * s_hi[m] * sw_hi[n] + A_lo * s_lo[m] * sw_lo[n]).
//
// Tiling.  One workgroup of 8 wavefronts owns a 128 (tokens) x 256 (channels)
// output tile; each wavefront owns 64 x 64 of it as 2 x 2 tiles of the
// 32x32x32 int8 matrix-core instruction, the weights as its first operand so
// that a lane ends up with four consecutive channels of one token.  Two
// wavefronts share a SIMD (256 registers each): while one waits for the matrix
// pipe, the other issues its vector-ALU, LDS and memory instructions, which a
// single wavefront per SIMD cannot hide behind its own matrix instructions
// (measured: about five other instructions fit behind one matrix instruction
// of a lone wavefront, and the low group needs more).
//
// Stages.  The reduction axis is walked in stages of 64 bytes per row: 64 int8
// codes of the high group or 128 nibble codes of the low group, i.e. two
// matrix-core steps of 32 bytes.  High and low stages form one sequence; the
// global->LDS copy is the same for both.  Six LDS buffers of 24 KiB hold the
// stage being multiplied, the next one, and up to four in flight.
//
// Global -> LDS.  Buffer loads with the LDS flag move 16 bytes per lane to a
// wave-uniform LDS base plus 16 * lane, so the LDS image is fixed by which
// global address each lane asks for; the address is a buffer resource (scalar
// registers, fixed per tile) plus a per-lane offset that never changes plus a
// scalar offset that advances per stage, so a load costs no vector-ALU work
// (and measurably less issue time than the same load with a 64-bit address).
// A block (16 rows x 64 bytes) is stored with piece kc (16 bytes) of row r at
// unit 4 r + (kc ^ (r >> 2)): four consecutive lanes fetch one row's 64
// contiguous bytes, and the 16 lanes that later read the same piece of 16
// different rows hit 16 different bank groups.
//
// LDS -> registers.  Operand reads are issued as untracked ds_read_b128 (inline
// asm) and paired with an explicit wait: reads the compiler can see would each
// be preceded by a wait for every direct-to-LDS load still in flight.
//
// Software pipeline.  Low steps: read(k+2) | widen(k+1) | multiply(k), so that
// the matrix instructions of step k never wait for the vector ALU work of
// their own operands.  High steps need no widening: the reads of a whole stage
// land in operand registers while the stage before it is multiplied.  The
// epilogue's per-channel and per-token constants (3.5 KiB) are fetched into
// LDS by the first loads of the kernel.
//
// The low group.  A lane's 16 packed bytes hold 32 codes, and each nibble is
// widened to an int8 operand with one AND.  In an activation byte the low
// nibble is c_even + 8 and the high nibble c_odd; in a weight byte the high
// nibble is w_even and the low nibble w_odd + 8.  Then
//   (pa & 0x0F) * (pw & 0xF0) = (c_even + 8) * 16 w_even
//   (pa & 0xF0) * (pw & 0x0F) = 16 c_odd * (w_odd + 8)
// feed two matrix-core instructions, and the accumulator ends as
//   16 * A_lo + 128 * (sum_even w[n] + sum_odd c[m]);
// the two sums are known per channel (packed with the weights) and per token
// (written by the quantizer), so A_lo is recovered exactly.
//
// Two scale pairs, one output write.  Each group has its own int32 tile in
// accumulation registers (2 x 64 per lane); both are folded into the output
// at the end, and y is written once, through LDS so that every store
// instruction writes whole 512-byte row segments.
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

constexpr int kGemmThreads = 512;  // 8 wavefronts, two per SIMD
constexpr int kBM = 128;
constexpr int kBN = 256;
constexpr int kStageABytes = kBM * kRowBytes;  // 8 KiB = 8 blocks
constexpr int kStageBBytes = kBN * kRowBytes;  // 16 KiB = 16 blocks
constexpr int kStageBytes = kStageABytes + kStageBBytes;
constexpr int kNumBuf = 6;
constexpr int kPrefetch = kNumBuf - 1;  // stages requested ahead of the one being multiplied
constexpr int kLoadsPerStage = (kBM + kBN) / kRowsPerBlock / 8;  // per wavefront: 3 (one activation block, two weight blocks)
constexpr int kOutRowBytes = kBN * 2 + 16;  // one tile row of bf16 in LDS, padded
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
// 2 activation tiles and 2 weight tiles of 32 rows x 32 bytes
struct Packed {
    v4i fa[2];
    v4i fb[2];
};
// matrix-core operands of one low reduction step: the even-code and the odd-code half of
// every fragment
struct Operands {
    Packed e, o;
};

// Wait until at most N LDS reads of this wavefront are outstanding (they return in order).
// The four fragments are tied to the wait as in/out operands so that no use of them can be
// scheduled above it.
template <int N>
__device__ __forceinline__ void lds_wait(v4i& a0, v4i& a1, v4i& b0, v4i& b1) {
    asm volatile("s_waitcnt lgkmcnt(%4)" : "+v"(a0), "+v"(a1), "+v"(b0), "+v"(b1) : "n"(N));
}

// buffer resource over all of memory from `base` on (raw, no stride, no bounds): the loads
// below address base + per-lane offset + scalar offset
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* base) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, 0x7FFFFFFF, 0x00020000);
}
// direct-to-LDS buffer load: lane l's 16 bytes at base + voff + soff land at lds_wave_base + 16 l
__device__ __forceinline__ void buffer_load_to_lds_16B(__amdgpu_buffer_rsrc_t rsrc, uint32_t voff, uint32_t soff,
                                                       uint8_t* lds_wave_base) {
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (__attribute__((address_space(3))) void*)lds_wave_base, 16,
                                             (int)voff, (int)soff, 0, 0);
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
    const int wm = wave >> 2;  // 0..1: 64-token half of the tile
    const int wn = wave & 3;   // 0..3: 64-channel quarter of the tile
    int tile_m, tile_n;
    tile_of_block(a, tile_m, tile_n);
    const int64_t m0 = (int64_t)tile_m * kBM;
    const int64_t n0 = (int64_t)tile_n * kBN;
    const int S_hi = a.stages_hi, S_lo = a.stages_lo, S = S_hi + S_lo;  // S_hi and S_lo are even
    const uint16_t* sw_hi = reinterpret_cast<const uint16_t*>(a.packed + a.L.scale_off);
    const uint16_t* sw_lo = sw_hi + a.L.n_pad;
    const int32_t* even_sum = reinterpret_cast<const int32_t*>(a.packed + a.L.scale_off + 4 * a.L.n_pad);
    const bool asym = a.c_hi != nullptr || a.c_lo != nullptr;

    // ---- epilogue constants -> LDS ---------------------------------------------
    // These are the oldest loads of their waves, so the first wait for a stage
    // covers them.  Token rows past M repeat the last row (never stored).
    if (wave == 0) {
        load_to_lds_16B((lane < 32 ? sw_hi : sw_lo) + n0 + (lane & 31) * 8, lds + kMetaOff + kMetaSwHi);
        if (asym) load_to_lds_16B(even_sum + a.L.n_pad + n0 + lane * 4, lds + kMetaOff + kMetaWsumHi);
    } else if (wave == 1) {
        load_to_lds_16B(even_sum + n0 + lane * 4, lds + kMetaOff + kMetaEven);
        if (asym) load_to_lds_16B(even_sum + 2 * a.L.n_pad + n0 + lane * 4, lds + kMetaOff + kMetaWsumLo);
    } else if (wave < 4) {
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
    // (l % 4) ^ (l / 16).  Wave w copies A block w and B blocks 2w, 2w+1 of each
    // stage.  Token rows past M are clamped to the last row (their results are
    // never stored).  The weight blocks of one 16-channel group are contiguous
    // over all stages, high ones first.  Every address is a buffer resource
    // (wave-uniform, fixed) plus a per-lane offset that never changes plus a
    // scalar offset that depends on the stage alone.
    uint32_t a_voff_hi, a_voff_lo, b_voff[2];
    {
        const int r = lane >> 2, kc = (lane & 3) ^ (lane >> 4);
        int64_t row = wave * 16 + r;
        row = m0 + row < a.M ? row : a.M - 1 - m0;
        a_voff_hi = (uint32_t)(row * a.ld_hi + kc * 16);
        a_voff_lo = (uint32_t)(row * a.ld_lo + kc * 16);
        b_voff[0] = r * kRowBytes + kc * 16;
        b_voff[1] = b_voff[0] + (uint32_t)a.L.group_bytes;
    }
    // the low rows are addressed by the global stage index too: their resource starts S_hi stages early
    const __amdgpu_buffer_rsrc_t rs_a_hi = make_rsrc(a.q_hi + m0 * a.ld_hi);
    const __amdgpu_buffer_rsrc_t rs_a_lo = make_rsrc(a.q_lo + m0 * a.ld_lo - (int64_t)S_hi * kRowBytes);
    const __amdgpu_buffer_rsrc_t rs_b = make_rsrc(a.packed + (n0 / 16 + wave * 2) * a.L.group_bytes);
    // load K of stage sg (0 .. S-1, high stages first) into buffer buf; K = 0: the A block, 1, 2: the B blocks
    auto issue_load = [&](auto k, int sg, int buf) __attribute__((always_inline)) {
        constexpr int K = decltype(k)::value;
        uint8_t* dst = lds + buf * kStageBytes;
        if constexpr (K == 0) {
            const bool lo = sg >= S_hi;
            buffer_load_to_lds_16B(lo ? rs_a_lo : rs_a_hi, lo ? a_voff_lo : a_voff_hi, (uint32_t)sg * kRowBytes,
                                   dst + wave * kBlockBytes);
        } else {
            buffer_load_to_lds_16B(rs_b, b_voff[K - 1], (uint32_t)sg * kBlockBytes,
                                   dst + kStageABytes + (wave * 2 + K - 1) * kBlockBytes);
        }
    };
    // the same for a stage known to be a low one (no selection of the activation rows)
    auto issue_load_lo = [&](auto k, int sg, int buf) __attribute__((always_inline)) {
        constexpr int K = decltype(k)::value;
        uint8_t* dst = lds + buf * kStageBytes;
        if constexpr (K == 0)
            buffer_load_to_lds_16B(rs_a_lo, a_voff_lo, (uint32_t)sg * kRowBytes, dst + wave * kBlockBytes);
        else
            buffer_load_to_lds_16B(rs_b, b_voff[K - 1], (uint32_t)sg * kBlockBytes,
                                   dst + kStageABytes + (wave * 2 + K - 1) * kBlockBytes);
    };

    // ---- accumulators ----------------------------------------------------------
    // One int32 tile per group, both in accumulation registers for the whole
    // kernel (2 x 64), folded into the output together at the end.
    // acc[j][i]: channels 32 j.., tokens 32 i.. of the wave tile.  Lane l holds
    // token (l % 32) and, in element v, channel 8 (v / 4) + 4 (l / 32) + v % 4.
    v16i acc_hi[2][2], acc_lo[2][2];
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                acc_hi[j][i][v] = 0;
                acc_lo[j][i][v] = 0;
            }

    // The tile that a loop does not touch stays where it is, in accumulation
    // registers: stating so in every stage keeps the register allocator from
    // moving it to ordinary registers and back around the loops.
    auto park = [&](v16i (&acc)[2][2]) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < 2; ++j)
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
            b_off[st] = lds0 + kStageABytes + wn * (4 * kBlockBytes) + off;
        }
    }
    // read K of a step: K = 0, 1: activation fragments, 2, 3: weight fragments
    auto read_frag = [&](auto k, Packed& f, uint32_t aa, uint32_t bb) __attribute__((always_inline)) {
        constexpr int K = decltype(k)::value;
        if constexpr (K < 2) lds_read16<K * 2 * kBlockBytes>(f.fa[K], aa);
        else lds_read16<(K - 2) * 2 * kBlockBytes>(f.fb[K - 2], bb);
    };
    // piece P (0..7) of the widening of one low step's fragments: one AND over a fragment
    auto widen_piece = [&](auto p, const Packed& f, Operands& u) __attribute__((always_inline)) {
        constexpr int P = decltype(p)::value;
        if constexpr (P < 2) u.e.fa[P] = f.fa[P] & (int)0x0F0F0F0F;               // even columns: code + 8
        else if constexpr (P < 4) u.e.fb[P - 2] = f.fb[P - 2] & (int)0xF0F0F0F0;  // even columns: 16 * code
        else if constexpr (P < 6) u.o.fa[P - 4] = f.fa[P - 4] & (int)0xF0F0F0F0;  // odd columns: 16 * code
        else u.o.fb[P - 6] = f.fb[P - 6] & (int)0x0F0F0F0F;                        // odd columns: code + 8
    };
    // matrix instruction Q of a low step (8 of them): the four products of the even halves,
    // then those of the odd halves, so that two instructions on one accumulator are four apart
    auto mfma_lo = [&](auto q, const Operands& u) __attribute__((always_inline)) {
        constexpr int Q = decltype(q)::value;
        constexpr int j = (Q >> 1) & 1, i = Q & 1;
        if constexpr (Q < 4)
            acc_lo[j][i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(u.e.fb[j], u.e.fa[i], acc_lo[j][i], 0, 0, 0);
        else
            acc_lo[j][i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(u.o.fb[j], u.o.fa[i], acc_lo[j][i], 0, 0, 0);
    };
    // matrix instruction Q of a high step (4 of them), operands as they were read
    auto mfma_hi = [&](auto q, const Packed& f) __attribute__((always_inline)) {
        constexpr int Q = decltype(q)::value;
        constexpr int j = (Q >> 1) & 1, i = Q & 1;
        acc_hi[j][i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(f.fb[j], f.fa[i], acc_hi[j][i], 0, 0, 0);
    };

    // ---- epilogue pieces -------------------------------------------------------------
    // Lane coordinates inside the tile: token tl + 32 i, channel cl + 32 j + 8 vq + vr.
    const int tl = wm * 64 + (lane & 31);
    const int cl = wn * 64 + (lane >> 5) * 4;

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
        for (int j = 0; j < 2; ++j) {
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
                    const int row = tl + 32 * i;
                    const int col = cl + 32 * j + 8 * vq;
                    if constexpr (GLU)
                        *reinterpret_cast<uint32_t*>(lds + row * kOutRowBytes + col) =
                            pack_bf16(silu_f32(val[0]) * val[1], silu_f32(val[2]) * val[3]);
                    else
                        *reinterpret_cast<uint2*>(lds + row * kOutRowBytes + col * 2) =
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
        // the four register sets of the high stages: two stages' worth of operands, used as read
        Packed& h0 = px;
        Packed& h1 = py;
        Packed& h2 = ux.e;
        Packed& h3 = uy.e;
        const int ahead = S < kPrefetch ? S : kPrefetch;
        for (int i = 0; i < ahead; ++i)
            static_for<kLoadsPerStage>([&](auto k) __attribute__((always_inline)) { issue_load(k, i, i); });
        wait_stage_and_barrier(ahead - 1);  // stage 0 (and the epilogue constants) have landed everywhere
        static_for<4>([&](auto k) __attribute__((always_inline)) { read_frag(k, px, a_off[0], b_off[0]); });
        static_for<4>([&](auto k) __attribute__((always_inline)) { read_frag(k, py, a_off[1], b_off[1]); });
        if (S_hi == 0) {
            lds_wait<4>(px.fa[0], px.fa[1], px.fb[0], px.fb[1]);
            static_for<8>([&](auto p) __attribute__((always_inline)) { widen_piece(p, px, ux); });
        }

        int buf = 0;
        // A low stage = two pipeline slots (reduction steps) of 8 matrix
        // instructions.  ISSUE: this stage requests stage sg + kPrefetch (every
        // stage but the last kPrefetch ones).  A slot is a fixed sequence of groups,
        // one matrix instruction each, with the slot's other work dealt out among
        // them so that it issues while the SIMD's matrix pipe is busy with this or
        // the other wavefront's instructions:
        //   slot 0: multiply step 0 | wait + barrier after 2 groups | then the four LDS reads
        //           of the next stage's step 0 and the widening of step 1
        //   slot 1: multiply step 1 | the four LDS reads of the next stage's step 1 and the
        //           widening of the next step 0
        // and the stage's three global loads after the barrier.
        // Invariant at entry: ux = operands of (sg, step 0); the reads of (sg, step 1)
        // into py are in flight.
        auto stage_lo = [&](auto issue, int sg) __attribute__((always_inline)) {
            constexpr bool ISSUE = decltype(issue)::value;
            const int nxt = buf == kNumBuf - 1 ? 0 : buf + 1;
            const int prv = buf == 0 ? kNumBuf - 1 : buf - 1;
            const uint32_t shift = nxt * kStageBytes;
            park(acc_hi);
            __builtin_amdgcn_sched_barrier(0);
            mfma_lo(IC<0>{}, ux);
            mfma_lo(IC<1>{}, ux);
            __builtin_amdgcn_sched_barrier(0);
            // stage sg + 1 has landed everywhere, and every wave is done with stage sg - 1;
            // stages sg + 2 .. sg + 4 may stay in flight
            if constexpr (ISSUE) {
                wait_loads_and_barrier<3 * kLoadsPerStage>();
            } else {
                const int rem = S - 2 - sg;
                wait_stage_and_barrier(rem > 3 ? 3 : rem);
            }
            lds_wait<0>(py.fa[0], py.fa[1], py.fb[0], py.fb[1]);
            __builtin_amdgcn_sched_barrier(0);
            static_for<6>([&](auto g) __attribute__((always_inline)) {
                constexpr int G = decltype(g)::value;
                mfma_lo(IC<2 + G>{}, ux);
                // past the last stage the reads fetch stale LDS: harmless
                if constexpr (G < 4) read_frag(g, px, a_off[0] + shift, b_off[0] + shift);
                widen_piece(g, py, uy);
                if constexpr (G == 4) widen_piece(IC<6>{}, py, uy);
                if constexpr (G == 5) widen_piece(IC<7>{}, py, uy);
                if constexpr (ISSUE && G == 4) issue_load_lo(IC<0>{}, sg + kPrefetch, prv);
                __builtin_amdgcn_sched_barrier(0);
            });
            mfma_lo(IC<0>{}, uy);
            read_frag(IC<0>{}, py, a_off[1] + shift, b_off[1] + shift);
            __builtin_amdgcn_sched_barrier(0);
            mfma_lo(IC<1>{}, uy);
            read_frag(IC<1>{}, py, a_off[1] + shift, b_off[1] + shift);
            if constexpr (ISSUE) issue_load_lo(IC<1>{}, sg + kPrefetch, prv);
            __builtin_amdgcn_sched_barrier(0);
            lds_wait<2>(px.fa[0], px.fa[1], px.fb[0], px.fb[1]);   // px is older than the two reads of py
            __builtin_amdgcn_sched_barrier(0);
            static_for<6>([&](auto g) __attribute__((always_inline)) {
                constexpr int G = decltype(g)::value;
                mfma_lo(IC<2 + G>{}, uy);
                if constexpr (G < 2) read_frag(IC<2 + G>{}, py, a_off[1] + shift, b_off[1] + shift);
                widen_piece(g, px, ux);
                if constexpr (G == 4) widen_piece(IC<6>{}, px, ux);
                if constexpr (G == 5) widen_piece(IC<7>{}, px, ux);
                if constexpr (ISSUE && G == 3) issue_load_lo(IC<2>{}, sg + kPrefetch, prv);
                __builtin_amdgcn_sched_barrier(0);
            });
            buf = nxt;
        };
        // A high stage needs no widening: 2 x 4 matrix instructions on the fragments as they
        // were read.  Its eight reads were issued during the stage before it (after that
        // stage's barrier, which says that this stage has landed), into the register sets
        // (u0, u1); this stage issues the next stage's reads into (f0, f1).  The last high
        // stage thereby leaves the packed bytes of the first low stage in px and py.
        // Invariant at entry: the reads of (sg, step 0) into u0 and of (sg, step 1) into u1
        // have been issued, in this order.
        auto stage_hi = [&](Packed& u0, Packed& u1, Packed& f0, Packed& f1, int sg) __attribute__((always_inline)) {
            const int nxt = buf == kNumBuf - 1 ? 0 : buf + 1;
            const int prv = buf == 0 ? kNumBuf - 1 : buf - 1;
            const uint32_t shift = nxt * kStageBytes;
            const bool issue = sg + kPrefetch < S;
            park(acc_lo);
            __builtin_amdgcn_sched_barrier(0);
            lds_wait<4>(u0.fa[0], u0.fa[1], u0.fb[0], u0.fb[1]);
            mfma_hi(IC<0>{}, u0);
            mfma_hi(IC<1>{}, u0);
            __builtin_amdgcn_sched_barrier(0);
            // stage sg + 1 has landed everywhere, and every wave is done with stage sg - 1
            {
                const int rem = S - 2 - sg;
                wait_stage_and_barrier(rem > 3 ? 3 : rem);
            }
            __builtin_amdgcn_sched_barrier(0);
            mfma_hi(IC<2>{}, u0);
            read_frag(IC<0>{}, f0, a_off[0] + shift, b_off[0] + shift);
            read_frag(IC<1>{}, f0, a_off[0] + shift, b_off[0] + shift);
            __builtin_amdgcn_sched_barrier(0);
            mfma_hi(IC<3>{}, u0);
            read_frag(IC<2>{}, f0, a_off[0] + shift, b_off[0] + shift);
            read_frag(IC<3>{}, f0, a_off[0] + shift, b_off[0] + shift);
            if (issue) issue_load(IC<0>{}, sg + kPrefetch, prv);
            __builtin_amdgcn_sched_barrier(0);
            lds_wait<4>(u1.fa[0], u1.fa[1], u1.fb[0], u1.fb[1]);   // u1 is older than the four reads of f0
            mfma_hi(IC<0>{}, u1);
            read_frag(IC<0>{}, f1, a_off[1] + shift, b_off[1] + shift);
            read_frag(IC<1>{}, f1, a_off[1] + shift, b_off[1] + shift);
            __builtin_amdgcn_sched_barrier(0);
            mfma_hi(IC<1>{}, u1);
            read_frag(IC<2>{}, f1, a_off[1] + shift, b_off[1] + shift);
            read_frag(IC<3>{}, f1, a_off[1] + shift, b_off[1] + shift);
            if (issue) issue_load(IC<1>{}, sg + kPrefetch, prv);
            __builtin_amdgcn_sched_barrier(0);
            mfma_hi(IC<2>{}, u1);
            __builtin_amdgcn_sched_barrier(0);
            mfma_hi(IC<3>{}, u1);
            if (issue) issue_load(IC<2>{}, sg + kPrefetch, prv);
            __builtin_amdgcn_sched_barrier(0);
            buf = nxt;
        };
        using YES = std::true_type;
        using NO = std::false_type;
        const int issue_end = S - kPrefetch;  // stages below this one request a later stage
        int sg = 0;
        if (S_hi > 0) {
            // S_hi is even: the sets alternate (px, py) -> (h2, h3) -> (px, py), and the last
            // high stage reads the first low stage (or stale bytes) into px and py
            for (; sg < S_hi; sg += 2) {
                stage_hi(h0, h1, h2, h3, sg);
                stage_hi(h2, h3, h0, h1, sg + 1);
            }
            if (S_lo > 0) {
                lds_wait<4>(px.fa[0], px.fa[1], px.fb[0], px.fb[1]);
                static_for<8>([&](auto p) __attribute__((always_inline)) { widen_piece(p, px, ux); });
            }
        }
        if (S_lo > 0) {
            for (; sg < issue_end; ++sg) stage_lo(YES{}, sg);
            for (; sg < S; ++sg) stage_lo(NO{}, sg);
        }
        // reads past the last stage: let them land
        lds_wait<0>(px.fa[0], px.fa[1], px.fb[0], px.fb[1]);
        lds_wait<0>(py.fa[0], py.fa[1], py.fb[0], py.fb[1]);
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
    // The 128 x 256 bf16 tile sits in LDS; wave w stores rows 16 w .. 16 w + 15, two
    // whole 512-byte row segments per store instruction.
    __syncthreads();
    const bool fast = ((reinterpret_cast<uintptr_t>(a.y) & 15) == 0) && (a.ldy % 8 == 0) &&
                      (n0 + kBN <= a.L.N);
    if (a.swiglu) {
        // 128 outputs per row: four 256-byte row segments per store instruction
        const int64_t n_out = a.L.N / 2;
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            const int row = wave * 16 + it * 4 + (lane >> 4);
            const int64_t m = m0 + row;
            const int64_t n = n0 / 2 + (lane & 15) * 8;
            const uint4 v = *reinterpret_cast<const uint4*>(lds + row * kOutRowBytes + (lane & 15) * 16);
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
    for (int it = 0; it < 8; ++it) {
        const int row = wave * 16 + it * 2 + (lane >> 5);
        const int64_t m = m0 + row;
        const int64_t n = n0 + (lane & 31) * 8;
        const uint4 v = *reinterpret_cast<const uint4*>(lds + row * kOutRowBytes + (lane & 31) * 16);
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
