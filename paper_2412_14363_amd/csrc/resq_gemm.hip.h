// Tiled mixed INT8/INT4 GEMM with dequantizing epilogue (Section 4.1, Eq. 4):
//   A_hi = q_hi * w_hi^T over the high group, A_lo = q_lo * w_lo^T over the low
//   group, y = bf16(A_hi * s_hi[m] * sw_hi[n] + A_lo * s_lo[m] * sw_lo[n]).
//
// Tiling.  One workgroup of 4 wavefronts owns a 128 (tokens) x 128 (channels)
// output tile; each wavefront owns 64 x 64 of it as 4 x 4 tiles of the
// 16x16x64 int8 matrix-core instruction, the weights as its first operand so
// that a lane ends up with four consecutive channels of one token.  (Under the
// chip's power limit this instruction sustains 16-20 % more operations per
// second than the 32x32x32 one on the same operands: it moves a quarter of the
// accumulator registers per instruction for half the products.)  TWO workgroups
// share a compute unit (half of its LDS and registers each), so two wavefronts
// share a SIMD (256 registers each): while one waits for the matrix pipe, the
// other issues its vector-ALU, LDS and memory instructions, which a single
// wavefront per SIMD cannot hide behind its own matrix instructions (measured:
// about five other instructions fit behind one matrix instruction of a lone
// wavefront, and the low group needs more); and since the two are independent
// workgroups, one's prologue, epilogue and barrier waits are the other's
// matrix time.  (One workgroup of 8 wavefronts on a 128 x 256 tile, the same
// wavefront tiles and registers, moves a quarter less through L2 per product
// but leaves the compute unit idle at both ends of every tile: measured 10-17 %
// slower on the Llama-3-8B MLP shapes, 0-3 % on the Qwen2.5-72B one.)
//
// Stages.  The reduction axis is walked in stages of 64 bytes per row: 64 int8
// codes of the high group or 128 nibble codes of the low group, one reduction
// step of the matrix-core instruction (two for nibbles: even and odd columns).  High and low stages form one sequence; the
// global->LDS copy is the same for both.  Four LDS buffers of 16 KiB hold the
// stage being multiplied, the next one, and two in flight.
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
// Software pipeline.  The eight fragment reads of stage k+1 are issued while
// stage k is multiplied.  A low stage multiplies widened copies: the four
// activation fragments of the whole stage and one weight fragment at a time;
// the next weight fragment is widened behind the products of the current one,
// the next stage's activation fragments in place behind the last products
// that read their predecessors.  High stages multiply the fragments as read.  The
// epilogue's per-channel and per-token constants (2.5 KiB, 4.5 KiB with
// asymmetric codes) are fetched into LDS by the first loads of the kernel.
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

constexpr int kGemmThreads = 256;  // 4 wavefronts, one per SIMD; two workgroups share a compute unit
constexpr int kBM = 128;
constexpr int kBN = 128;
constexpr int kStageABytes = kBM * kRowBytes;  // 8 KiB = 8 blocks
constexpr int kStageBBytes = kBN * kRowBytes;  // 8 KiB = 8 blocks
constexpr int kStageBytes = kStageABytes + kStageBBytes;
constexpr int kNumBuf = 4;
constexpr int kPrefetch = kNumBuf - 1;  // stages requested ahead of the one being multiplied
constexpr int kLoadsPerStage = (kBM + kBN) / kRowsPerBlock / 4;  // per wavefront: 4 (two activation blocks, two weight blocks)
constexpr int kOutRowBytes = kBN * 2 + 16;  // one tile row of bf16 in LDS, padded
// After the stage buffers: the tile's per-channel and per-token constants of the
// epilogue, copied there by the first loads of the kernel.
constexpr int kMetaOff = kNumBuf * kStageBytes;
constexpr int kMetaSwHi = 0;       // fp16 [128] high-group weight scales
constexpr int kMetaSwLo = 256;     // fp16 [128] low-group weight scales
constexpr int kMetaEven = 512;     // int32 [128] even-column code sums of the low group
constexpr int kMetaSHi = 1024;     // fp32 [128] high-group token scales
constexpr int kMetaSLo = 1536;     // fp32 [128] low-group token scales
constexpr int kMetaLoSum = 2048;   // int32 [128] odd-column code sums of the low group
// only for asymmetric activation codes:
constexpr int kMetaWsumHi = 2560;  // int32 [128] sums of the high weight codes
constexpr int kMetaWsumLo = 3072;  // int32 [128] sums of the low weight codes
constexpr int kMetaCHi = 3584;     // fp32 [128] real value of the stored high code 0, per token
constexpr int kMetaCLo = 4096;     // fp32 [128] the same for the low group
constexpr int kMetaBytes = 4608;
// two workgroups fit the 160 KiB of a compute unit
static_assert(2 * (kMetaOff + kMetaBytes) <= 160 * 1024, "LDS of two resident workgroups");

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

// the fragments of one stage as read from LDS: 4 activation and 4 weight fragments of
// 16 rows x 64 bytes, 16 bytes per lane each (row l % 16, piece l / 16)
struct Raw {
    v4i a[4];
    v4i b[4];
};

// Wait until at most N LDS reads of this wavefront are outstanding (they return in order).
// The fragments are tied to the wait as in/out operands so that no use of them can be
// scheduled above it.
template <int N>
__device__ __forceinline__ void lds_wait(v4i (&f)[4]) {
    asm volatile("s_waitcnt lgkmcnt(%4)" : "+v"(f[0]), "+v"(f[1]), "+v"(f[2]), "+v"(f[3]) : "n"(N));
}

// acc += b * a^T on the int8 matrix cores (b: 16 channels x 64 bytes, a: 16 tokens x 64 bytes), the
// accumulator tile in place in accumulation registers.  Written as assembly because the
// compiler, given the builtin, renames the 32 four-register tiles from instruction to
// instruction and runs out of registers.  Nothing here tells the compiler how long the
// instruction takes: two of them on one tile are kept at least four instructions apart by the
// loops below, and the epilogue waits before it reads the tiles.
__device__ __forceinline__ void mfma_16x16x64(v4i& acc, const v4i& b, const v4i& a) {
    asm volatile("v_mfma_i32_16x16x64_i8 %0, %1, %2, %0" : "+a"(acc) : "v"(b), "v"(a));
}

// Keeps the instructions that compute x where they are written, between the assembly
// statements around them: the matrix instruction above is opaque to the compiler, which
// therefore neither knows that an operand written by the vector ALU needs two wait states
// before a matrix instruction may read it, nor has a reason to keep the widening spread
// out between the matrix instructions.
__device__ __forceinline__ void pin(v4i& x) { asm volatile("" : "+v"(x)); }

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
// workgroups in id order, 64 at a time (two per compute unit).  When the grid
// allows it, the 64 tiles an XCD works on together form an 8 x 8 patch (1024
// tokens x 1024 channels), so that each activation stage and each weight stage
// is fetched into that L2 once per 8 tiles; the 8 XCDs take neighbouring patches.
__device__ __forceinline__ void tile_of_block(const GemmArgs& a, int& tm, int& tn) {
    const int total = a.tiles_m * a.tiles_n;
    const int id = blockIdx.x;
    if (total % 512 == 0 && a.tiles_m % 8 == 0 && a.tiles_n % 8 == 0) {
        const int xcd = id & 7, k = id >> 3;
        const int patch = (k >> 6) * 8 + xcd, within = k & 63;
        const int patches_m = a.tiles_m >> 3;
        tm = (patch % patches_m) * 8 + (within & 7);
        tn = (patch / patches_m) * 8 + (within >> 3);
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

// Second launch bound: two workgroups per compute unit, i.e. two wavefronts per SIMD with
// 256 registers each (128 vector + 128 accumulation).
template <bool DBG>
__global__ __launch_bounds__(kGemmThreads, 2) void gemm_mixed_kernel(const GemmArgs a) {
    __shared__ __attribute__((aligned(1024))) uint8_t lds[kMetaOff + kMetaBytes];

    const int t = threadIdx.x;
    const int lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int wm = wave >> 1;  // 0..1: 64-token half of the tile
    const int wn = wave & 1;   // 0..1: 64-channel half of the tile
    int tile_m, tile_n;
    tile_of_block(a, tile_m, tile_n);
    const int64_t m0 = (int64_t)tile_m * kBM;
    const int64_t n0 = (int64_t)tile_n * kBN;
    // the grid covers the padded channel count (a multiple of 256, which keeps the patches of
    // tile_of_block whole): a tile that holds padding channels only has nothing to do
    if (n0 >= a.L.N) return;
    const int S_hi = a.stages_hi, S_lo = a.stages_lo, S = S_hi + S_lo;  // S_hi and S_lo are even
    const uint16_t* sw_hi = reinterpret_cast<const uint16_t*>(a.packed + a.L.scale_off);
    const uint16_t* sw_lo = sw_hi + a.L.n_pad;
    const int32_t* even_sum = reinterpret_cast<const int32_t*>(a.packed + a.L.scale_off + 4 * a.L.n_pad);
    const bool asym = a.c_hi != nullptr || a.c_lo != nullptr;

    // ---- epilogue constants -> LDS ---------------------------------------------
    // These are the oldest loads of their waves, so the first wait for a stage
    // covers them.  Token rows past M repeat the last row (never stored).
    // (a load to LDS places an active lane's bytes at the base plus 16 x its lane number)
    if (wave == 0) {
        if (lane < 32) {
            load_to_lds_16B((lane < 16 ? sw_hi : sw_lo) + n0 + (lane & 15) * 8, lds + kMetaOff + kMetaSwHi);
            if (asym) load_to_lds_16B(even_sum + a.L.n_pad + n0 + lane * 4, lds + kMetaOff + kMetaWsumHi);
        }
    } else if (wave == 1) {
        if (lane < 32) {
            load_to_lds_16B(even_sum + n0 + lane * 4, lds + kMetaOff + kMetaEven);
            if (asym) load_to_lds_16B(even_sum + 2 * a.L.n_pad + n0 + lane * 4, lds + kMetaOff + kMetaWsumLo);
        }
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
    // (l % 4) ^ (l / 16).  Wave w copies A blocks 2w, 2w+1 and B blocks 2w, 2w+1 of
    // each stage.  Token rows past M are clamped to the last row (their results are
    // never stored).  The weight blocks of one 16-channel group are contiguous
    // over all stages, high ones first.  Every address is a buffer resource
    // (wave-uniform, fixed) plus a per-lane offset that never changes plus a
    // scalar offset that depends on the stage alone.
    uint32_t a_voff_hi[2], a_voff_lo[2], b_voff[2];
    {
        const int r = lane >> 2, kc = (lane & 3) ^ (lane >> 4);
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            int64_t row = (wave * 2 + h) * 16 + r;
            row = m0 + row < a.M ? row : a.M - 1 - m0;
            a_voff_hi[h] = (uint32_t)(row * a.ld_hi + kc * 16);
            a_voff_lo[h] = (uint32_t)(row * a.ld_lo + kc * 16);
        }
        b_voff[0] = r * kRowBytes + kc * 16;
        b_voff[1] = b_voff[0] + (uint32_t)a.L.group_bytes;
    }
    // the low rows are addressed by the global stage index too: their resource starts S_hi stages early
    const __amdgpu_buffer_rsrc_t rs_a_hi = make_rsrc(a.q_hi + m0 * a.ld_hi);
    const __amdgpu_buffer_rsrc_t rs_a_lo = make_rsrc(a.q_lo + m0 * a.ld_lo - (int64_t)S_hi * kRowBytes);
    const __amdgpu_buffer_rsrc_t rs_b = make_rsrc(a.packed + (n0 / 16 + wave * 2) * a.L.group_bytes);
    // load K of stage sg (0 .. S-1, high stages first) into buffer buf; K = 0, 1: the A blocks, 2, 3: the B blocks
    auto issue_load = [&](auto k, int sg, int buf) __attribute__((always_inline)) {
        constexpr int K = decltype(k)::value;
        uint8_t* dst = lds + buf * kStageBytes;
        if constexpr (K < 2) {
            const bool lo = sg >= S_hi;
            buffer_load_to_lds_16B(lo ? rs_a_lo : rs_a_hi, lo ? a_voff_lo[K] : a_voff_hi[K], (uint32_t)sg * kRowBytes,
                                   dst + (wave * 2 + K) * kBlockBytes);
        } else {
            buffer_load_to_lds_16B(rs_b, b_voff[K - 2], (uint32_t)sg * kBlockBytes,
                                   dst + kStageABytes + (wave * 2 + K - 2) * kBlockBytes);
        }
    };
    // the same for a stage known to be a low one (no selection of the activation rows)
    auto issue_load_lo = [&](auto k, int sg, int buf) __attribute__((always_inline)) {
        constexpr int K = decltype(k)::value;
        uint8_t* dst = lds + buf * kStageBytes;
        if constexpr (K < 2)
            buffer_load_to_lds_16B(rs_a_lo, a_voff_lo[K], (uint32_t)sg * kRowBytes, dst + (wave * 2 + K) * kBlockBytes);
        else
            buffer_load_to_lds_16B(rs_b, b_voff[K - 2], (uint32_t)sg * kBlockBytes,
                                   dst + kStageABytes + (wave * 2 + K - 2) * kBlockBytes);
    };

    // ---- accumulators ----------------------------------------------------------
    // One int32 tile per group, both in accumulation registers for the whole
    // kernel (2 x 64), folded into the output together at the end.
    // acc[j][i]: channels 16 j.., tokens 16 i.. of the wave tile.  Lane l holds
    // token (l % 16) and, in element v, channel 4 (l / 16) + v.
    v4i acc_hi[4][4], acc_lo[4][4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            acc_hi[j][i] = (v4i){0, 0, 0, 0};
            acc_lo[j][i] = (v4i){0, 0, 0, 0};
        }

    // The tile that a loop does not touch stays where it is, in accumulation
    // registers: stating so in every stage keeps the register allocator from
    // moving it to ordinary registers and back around the loops.
    auto park = [&](v4i (&acc)[4][4]) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int i = 0; i < 4; ++i) asm volatile("" : "+a"(acc[j][i]));
    };

    // ---- LDS -> register reads ---------------------------------------------------
    // A fragment is one block (16 rows x 64 bytes): lane l supplies row l % 16, piece l / 16.
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t*)lds;
    uint32_t a_off, b_off;
    {
        const int r = lane & 15, kc = lane >> 4;
        const uint32_t off = (4 * r + (kc ^ (r >> 2))) * 16;
        a_off = lds0 + wm * (4 * kBlockBytes) + off;
        b_off = lds0 + kStageABytes + wn * (4 * kBlockBytes) + off;
    }
    // read K of a stage: K = 0..3: activation fragments, 4..7: weight fragments
    auto read_frag = [&](auto k, Raw& f, uint32_t aa, uint32_t bb) __attribute__((always_inline)) {
        constexpr int K = decltype(k)::value;
        if constexpr (K < 4) lds_read16<K * kBlockBytes>(f.a[K], aa);
        else lds_read16<(K - 4) * kBlockBytes>(f.b[K - 4], bb);
    };

    // ---- epilogue pieces -------------------------------------------------------------
    // Lane coordinates inside the tile: token tl + 16 i, channel cl + 16 j + v.
    const int tl = wm * 64 + (lane & 15);
    const int cl = wn * 64 + (lane >> 4) * 4;

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
        float st_hi[4], st_lo[4], ct_hi[4], ct_lo[4];
        int ca[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            st_hi[i] = st_lo[i] = ct_hi[i] = ct_lo[i] = 0.f;
            ca[i] = 0;
            if constexpr (HI_ON) st_hi[i] = *reinterpret_cast<const float*>(meta + kMetaSHi + (tl + 16 * i) * 4);
            if constexpr (ASYM && HI_ON) ct_hi[i] = *reinterpret_cast<const float*>(meta + kMetaCHi + (tl + 16 * i) * 4);
            if constexpr (ASYM && LO_ON) ct_lo[i] = *reinterpret_cast<const float*>(meta + kMetaCLo + (tl + 16 * i) * 4);
            if constexpr (LO_ON) {
                st_lo[i] = *reinterpret_cast<const float*>(meta + kMetaSLo + (tl + 16 * i) * 4);
                if constexpr (!DBG) st_lo[i] *= 0.0625f;
                ca[i] = 128 * *reinterpret_cast<const int*>(meta + kMetaLoSum + (tl + 16 * i) * 4);
            }
        }
        // debug dump of the integer sums: row pointers and the number of valid columns from cl on
        int32_t* dbg_row_hi[4] = {nullptr, nullptr, nullptr, nullptr};
        int32_t* dbg_row_lo[4] = {nullptr, nullptr, nullptr, nullptr};
        bool dbg_ok[4] = {false, false, false, false};
        int dbg_cols = 0;
        if constexpr (DBG) {
            dbg_cols = (int)(a.L.N - n0 - cl);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int64_t m = m0 + tl + 16 * i;
                dbg_ok[i] = m < a.M;
                dbg_row_hi[i] = a.dbg_hi + m * a.L.N + n0 + cl;
                dbg_row_lo[i] = a.dbg_lo + m * a.L.N + n0 + cl;
            }
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int c = cl + 16 * j;
            float sn_hi[4] = {0.f, 0.f, 0.f, 0.f}, sn_lo[4] = {0.f, 0.f, 0.f, 0.f};
            float zw_hi[4] = {0.f, 0.f, 0.f, 0.f}, zw_lo[4] = {0.f, 0.f, 0.f, 0.f};  // wsum[n] * sw[n]
            v4i ev = {0, 0, 0, 0};
            if constexpr (HI_ON) {
                const v4h h = *reinterpret_cast<const v4h*>(meta + kMetaSwHi + c * 2);
#pragma unroll
                for (int v = 0; v < 4; ++v) sn_hi[v] = (float)h[v];
                if constexpr (ASYM) {
                    const v4i ws = *reinterpret_cast<const v4i*>(meta + kMetaWsumHi + c * 4);
#pragma unroll
                    for (int v = 0; v < 4; ++v) zw_hi[v] = (float)ws[v] * sn_hi[v];
                }
            }
            if constexpr (LO_ON) {
                const v4h h = *reinterpret_cast<const v4h*>(meta + kMetaSwLo + c * 2);
#pragma unroll
                for (int v = 0; v < 4; ++v) sn_lo[v] = (float)h[v];
                ev = *reinterpret_cast<const v4i*>(meta + kMetaEven + c * 4);
                if constexpr (ASYM) {
                    const v4i ws = *reinterpret_cast<const v4i*>(meta + kMetaWsumLo + c * 4);
#pragma unroll
                    for (int v = 0; v < 4; ++v) zw_lo[v] = (float)ws[v] * sn_lo[v];
                }
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                float val[4];
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    val[v] = 0.f;
                    if constexpr (HI_ON) {
                        const int ih = acc_hi[j][i][v];
                        val[v] = (float)ih * (st_hi[i] * sn_hi[v]);
                        if constexpr (ASYM) val[v] += ct_hi[i] * zw_hi[v];
                        if constexpr (DBG) {
                            if (a.dbg_hi && dbg_ok[i] && 16 * j + v < dbg_cols) dbg_row_hi[i][16 * j + v] = ih;
                        }
                    }
                    if constexpr (LO_ON) {
                        int il = acc_lo[j][i][v] - (ev[v] * 128 + ca[i]);
                        if constexpr (DBG) il >>= 4;
                        val[v] += (float)il * (st_lo[i] * sn_lo[v]);
                        if constexpr (ASYM) val[v] += ct_lo[i] * zw_lo[v];
                        if constexpr (DBG) {
                            if (a.dbg_lo && dbg_ok[i] && 16 * j + v < dbg_cols) dbg_row_lo[i][16 * j + v] = il;
                        }
                    }
                }
                const int row = tl + 16 * i;
                if constexpr (GLU)
                    *reinterpret_cast<uint32_t*>(lds + row * kOutRowBytes + c) =
                        pack_bf16(silu_f32(val[0]) * val[1], silu_f32(val[2]) * val[3]);
                else
                    *reinterpret_cast<uint2*>(lds + row * kOutRowBytes + c * 2) =
                        make_uint2(pack_bf16(val[0], val[1]), pack_bf16(val[2], val[3]));
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // ---- main loop ---------------------------------------------------------------
    {
        // Two sets of fragments as read from LDS: the stage being multiplied and the next one,
        // taking turns (the numbers of high and of low stages are even).  Low stages multiply
        // widened copies: the activation fragments of the whole stage (aw_e, aw_o: even and odd
        // columns) and the two halves of one weight fragment at a time (bw_e, bw_o).
        Raw p0, p1;
        v4i aw_e[4], aw_o[4], bw_e, bw_o;
        const int ahead = S < kPrefetch ? S : kPrefetch;
        for (int i = 0; i < ahead; ++i)
            static_for<kLoadsPerStage>([&](auto k) __attribute__((always_inline)) { issue_load(k, i, i); });
        wait_stage_and_barrier(ahead - 1);  // stage 0 (and the epilogue constants) have landed everywhere
        static_for<8>([&](auto k) __attribute__((always_inline)) { read_frag(k, p0, a_off, b_off); });

        // widening of a low stage's fragments: one AND over a fragment each
        auto widen_a = [&](auto i_, auto odd, const Raw& f) __attribute__((always_inline)) {
            constexpr int I = decltype(i_)::value;
            if constexpr (!decltype(odd)::value) {
                aw_e[I] = f.a[I] & (int)0x0F0F0F0F;  // even columns: code + 8
                pin(aw_e[I]);
            } else {
                aw_o[I] = f.a[I] & (int)0xF0F0F0F0;  // odd columns: 16 * code
                pin(aw_o[I]);
            }
        };
        using YES = std::true_type;
        using NO = std::false_type;

        int buf = 0;
        // A low stage: 4 weight fragments x (4 even + 4 odd) products.  Invariant at entry: cur
        // has landed; aw_e, aw_o hold the widened activation fragments of this stage and bw_e
        // the even half of weight fragment 0.  Each half of a weight fragment is widened while
        // the other half of the fragment before it is multiplied.  After the barrier the eight
        // reads of the next stage go out (into nx) and the three global loads of stage
        // sg + kPrefetch; during fragment 3 the next stage's activation fragments are widened
        // in place, each right after the last instruction that reads its predecessor.
        auto stage_lo = [&](auto steady, Raw& cur, Raw& nx, int sg) __attribute__((always_inline)) {
            // STEADY: stage sg + kPrefetch exists (known to the caller), so the loads and the wait are unconditional
            constexpr bool STEADY = decltype(steady)::value;
            const int nbuf = buf == kNumBuf - 1 ? 0 : buf + 1;
            const int prv = buf == 0 ? kNumBuf - 1 : buf - 1;
            const uint32_t shift = nbuf * kStageBytes;
            const bool issue = STEADY || sg + kPrefetch < S;
            park(acc_hi);
            static_for<4>([&](auto j_) __attribute__((always_inline)) {
                constexpr int J = decltype(j_)::value;
                static_for<8>([&](auto p_) __attribute__((always_inline)) {
                    constexpr int P = decltype(p_)::value;
                    constexpr int I = P & 3;
                    __builtin_amdgcn_sched_barrier(0);
                    if constexpr (P < 4) mfma_16x16x64(acc_lo[J][I], bw_e, aw_e[I]);
                    else mfma_16x16x64(acc_lo[J][I], bw_o, aw_o[I]);
                    if constexpr (J == 0 && P == 5) {
                        // stage sg + 1 has landed everywhere, and every wave is done with stage sg - 1;
                        // stages sg + 2 .. sg + 4 may stay in flight.  Six products in, the waves
                        // that ran late in the last stage have caught up (measured: 3 % faster on
                        // an all-low layer than a barrier after the second product)
                        __builtin_amdgcn_sched_barrier(0);
                        if constexpr (STEADY) {
                            wait_loads_and_barrier<(kPrefetch - 2) * kLoadsPerStage>();
                        } else {
                            const int rem = S - 2 - sg;
                            wait_stage_and_barrier(rem > kPrefetch - 2 ? kPrefetch - 2 : rem);
                        }
                    }
                    // the halves of the weight fragments: odd columns code + 8, even columns 16 * code
                    if constexpr (P == 1) {
                        bw_o = cur.b[J] & (int)0x0F0F0F0F;
                        pin(bw_o);
                    }
                    if constexpr (P == 5) {
                        if constexpr (J < 3) bw_e = cur.b[J + 1] & (int)0xF0F0F0F0;
                        else bw_e = nx.b[0] & (int)0xF0F0F0F0;
                        pin(bw_e);
                    }
                    // the reads of the next stage (stale LDS past the last stage: harmless), weight
                    // fragments first, one behind every other product from the barrier on: spaced
                    // like this they leave LDS cycles to the incoming global loads
                    {
                        constexpr int G = J * 8 + P - 6;
                        if constexpr (G >= 0 && G < 16 && G % 2 == 0) {
                            read_frag(IC<(G < 8 ? G / 2 + 4 : G / 2 - 4)>{}, nx, a_off + shift, b_off + shift);
                        }
                    }
                    if constexpr (J == 1 && P == 3) { if (issue) issue_load_lo(IC<0>{}, sg + kPrefetch, prv); }
                    if constexpr (J == 1 && P == 7) { if (issue) issue_load_lo(IC<1>{}, sg + kPrefetch, prv); }
                    if constexpr (J == 2 && P == 3) { if (issue) issue_load_lo(IC<2>{}, sg + kPrefetch, prv); }
                    if constexpr (J == 2 && P == 6) { if (issue) issue_load_lo(IC<3>{}, sg + kPrefetch, prv); }
                    if constexpr (J == 2 && P == 7) {
                        lds_wait<0>(nx.b);
                        lds_wait<0>(nx.a);
                    }
                    if constexpr (J == 3) {
                        // aw_e[I] was last read by product (3, even, I), aw_o[I] by (3, odd, I)
                        if constexpr (P >= 1 && P <= 4) widen_a(IC<P - 1>{}, NO{}, nx);
                        if constexpr (P >= 6) widen_a(IC<P - 6>{}, YES{}, nx);
                    }
                });
            });
            __builtin_amdgcn_sched_barrier(0);
            widen_a(IC<2>{}, YES{}, nx);
            widen_a(IC<3>{}, YES{}, nx);
            buf = nbuf;
        };
        // A high stage needs no widening: 4 x 4 products on the fragments as they were read.
        // Invariant at entry: the eight reads of this stage into cur have been issued.
        auto stage_hi = [&](auto steady, Raw& cur, Raw& nx, int sg) __attribute__((always_inline)) {
            constexpr bool STEADY = decltype(steady)::value;  // as in stage_lo
            const int nbuf = buf == kNumBuf - 1 ? 0 : buf + 1;
            const int prv = buf == 0 ? kNumBuf - 1 : buf - 1;
            const uint32_t shift = nbuf * kStageBytes;
            const bool issue = STEADY || sg + kPrefetch < S;
            park(acc_lo);
            __builtin_amdgcn_sched_barrier(0);
            lds_wait<0>(cur.a);
            lds_wait<0>(cur.b);
            static_for<4>([&](auto j_) __attribute__((always_inline)) {
                constexpr int J = decltype(j_)::value;
                static_for<4>([&](auto i_) __attribute__((always_inline)) {
                    constexpr int I = decltype(i_)::value;
                    __builtin_amdgcn_sched_barrier(0);
                    mfma_16x16x64(acc_hi[J][I], cur.b[J], cur.a[I]);
                    if constexpr (J == 0 && I == 3) {
                        __builtin_amdgcn_sched_barrier(0);
                        if constexpr (STEADY) {
                            wait_loads_and_barrier<(kPrefetch - 2) * kLoadsPerStage>();
                        } else {
                            const int rem = S - 2 - sg;
                            wait_stage_and_barrier(rem > kPrefetch - 2 ? kPrefetch - 2 : rem);
                        }
                    }
                    if constexpr (J == 1) read_frag(IC<I>{}, nx, a_off + shift, b_off + shift);
                    if constexpr (J == 2) read_frag(IC<I + 4>{}, nx, a_off + shift, b_off + shift);
                    if constexpr (J == 3 && I == 0) { if (issue) issue_load(IC<0>{}, sg + kPrefetch, prv); }
                    if constexpr (J == 3 && I == 1) { if (issue) issue_load(IC<1>{}, sg + kPrefetch, prv); }
                    if constexpr (J == 3 && I == 2) { if (issue) issue_load(IC<2>{}, sg + kPrefetch, prv); }
                    if constexpr (J == 3 && I == 3) { if (issue) issue_load(IC<3>{}, sg + kPrefetch, prv); }
                });
            });
            __builtin_amdgcn_sched_barrier(0);
            buf = nbuf;
        };
        int sg = 0;
        for (; sg < S_hi && sg + 1 + kPrefetch < S; sg += 2) {
            stage_hi(YES{}, p0, p1, sg);
            stage_hi(YES{}, p1, p0, sg + 1);
        }
        for (; sg < S_hi; sg += 2) {
            stage_hi(NO{}, p0, p1, sg);
            stage_hi(NO{}, p1, p0, sg + 1);
        }
        if (S_lo > 0) {
            // p0 holds the first low stage, as read: widen its activation fragments and weight fragment 0
            lds_wait<0>(p0.a);
            lds_wait<0>(p0.b);
            static_for<4>([&](auto i_) __attribute__((always_inline)) {
                widen_a(i_, NO{}, p0);
                widen_a(i_, YES{}, p0);
            });
            bw_e = p0.b[0] & (int)0xF0F0F0F0;
            pin(bw_e);
            asm volatile("s_nop 4" ::: "memory");  // wait states between the widening and the first product
            for (; sg + 1 + kPrefetch < S; sg += 2) {
                stage_lo(YES{}, p0, p1, sg);
                stage_lo(YES{}, p1, p0, sg + 1);
            }
            for (; sg < S; sg += 2) {
                stage_lo(NO{}, p0, p1, sg);
                stage_lo(NO{}, p1, p0, sg + 1);
            }
        }
        // the reads past the last stage went into p0: let them land before its registers are reused
        lds_wait<0>(p0.a);
        lds_wait<0>(p0.b);
        wait_loads_and_barrier<0>();  // every wave is done reading the stage buffers
        asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");  // the last matrix instructions have written their tiles
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
    // The 128 x 128 bf16 tile sits in LDS; wave w stores rows 32 w .. 32 w + 31, four
    // whole 256-byte row segments per store instruction.
    __syncthreads();
    const bool fast = ((reinterpret_cast<uintptr_t>(a.y) & 15) == 0) && (a.ldy % 8 == 0) &&
                      (n0 + kBN <= a.L.N);
    if (a.swiglu) {
        // 64 outputs per row: eight 128-byte row segments per store instruction
        const int64_t n_out = a.L.N / 2;
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            const int row = wave * 32 + it * 8 + (lane >> 3);
            const int64_t m = m0 + row;
            const int64_t n = n0 / 2 + (lane & 7) * 8;
            const uint4 v = *reinterpret_cast<const uint4*>(lds + row * kOutRowBytes + (lane & 7) * 16);
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
        const int row = wave * 32 + it * 4 + (lane >> 4);
        const int64_t m = m0 + row;
        const int64_t n = n0 + (lane & 15) * 8;
        const uint4 v = *reinterpret_cast<const uint4*>(lds + row * kOutRowBytes + (lane & 15) * 16);
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
