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
// Software pipeline, per reduction step k:  read(k+2) | transform(k+1) | multiply(k)
// where transform widens nibbles for a low step (and is a register copy for a
// high step), so that the matrix instructions of step k never wait for the
// vector ALU work of their own operands.
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
// Two scale pairs, one output write.  After the last high step the int32 tile is
// scaled into an fp32 tile that stays in (accumulation) registers, the int32
// tile is cleared for the low steps, and y is written once, through LDS so that
// every store instruction writes whole 256-byte row segments.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

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

struct GemmArgs {
    const uint8_t* q_hi;
    const uint8_t* q_lo;
    int64_t ld_hi, ld_lo;
    const float* s_hi;
    const float* s_lo;
    const int32_t* lo_sum;  // per token: sum of the low codes in odd columns
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
// the same with N = 6 * later, later = 0..3 stages allowed to stay in flight
__device__ __forceinline__ void wait_stage_and_barrier(int later) {
    if (later >= 4) wait_loads_and_barrier<4 * kLoadsPerStage>();
    else if (later == 3) wait_loads_and_barrier<3 * kLoadsPerStage>();
    else if (later == 2) wait_loads_and_barrier<2 * kLoadsPerStage>();
    else if (later == 1) wait_loads_and_barrier<1 * kLoadsPerStage>();
    else wait_loads_and_barrier<0>();
}

__device__ __forceinline__ void load_to_lds_16B(const uint8_t* g, uint8_t* lds_wave_base) {
    __builtin_amdgcn_global_load_lds(
        (const __attribute__((address_space(1))) void*)g,
        (__attribute__((address_space(3))) void*)lds_wave_base, 16, 0, 0);
}

template <int OFF>
__device__ __forceinline__ void lds_read16(v4i& dst, uint32_t addr) {
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=&v"(dst) : "v"(addr), "n"(OFF));
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

template <bool DBG>
__global__ __launch_bounds__(kGemmThreads) void gemm_mixed_kernel(const GemmArgs a) {
    __shared__ __attribute__((aligned(1024))) uint8_t lds[kNumBuf * kStageBytes];

    const int t = threadIdx.x;
    const int lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int wm = wave >> 1;  // 0..1: 64-token half of the tile
    const int wn = wave & 1;   // 0..1: 128-channel half of the tile
    int tile_m, tile_n;
    tile_of_block(a, tile_m, tile_n);
    const int64_t m0 = (int64_t)tile_m * kBM;
    const int64_t n0 = (int64_t)tile_n * kBN;
    const int S_hi = a.stages_hi, S = a.stages_hi + a.stages_lo;

    // ---- global -> LDS copy --------------------------------------------------
    // One load instruction fills one block: lane l fetches row l / 4, piece
    // (l % 4) ^ (l / 16).  Wave w copies A blocks 2w, 2w+1 and B blocks 4w..4w+3
    // of each stage.  Token rows past M are clamped to the last row (their
    // results are never stored).  The weight blocks of one 16-channel group are
    // contiguous over all stages, high ones first.
    const uint8_t* a_src_hi[2];
    const uint8_t* a_src_lo[2];
    const uint8_t* b_src[4];
    {
        const int r = lane >> 2, kc = (lane & 3) ^ (lane >> 4);
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            int64_t row = m0 + (wave * 2 + i) * 16 + r;
            row = row < a.M ? row : a.M - 1;
            a_src_hi[i] = a.q_hi + row * a.ld_hi + kc * 16;
            a_src_lo[i] = a.q_lo + row * a.ld_lo + kc * 16 - (int64_t)S_hi * kRowBytes;
        }
#pragma unroll
        for (int i = 0; i < 4; ++i)
            b_src[i] = a.packed + (n0 / 16 + wave * 4 + i) * a.L.group_bytes + r * kRowBytes + kc * 16;
    }
    // request stage sg (0 .. S-1, high stages first) into buffer buf
    auto issue_stage = [&](int sg, int buf) __attribute__((always_inline)) {
        uint8_t* dst = lds + buf * kStageBytes;
        const bool lo = sg >= S_hi;
#pragma unroll
        for (int i = 0; i < 2; ++i)
            load_to_lds_16B((lo ? a_src_lo[i] : a_src_hi[i]) + (int64_t)sg * kRowBytes,
                            dst + (wave * 2 + i) * kBlockBytes);
#pragma unroll
        for (int i = 0; i < 4; ++i)
            load_to_lds_16B(b_src[i] + (int64_t)sg * kBlockBytes,
                            dst + kStageABytes + (wave * 4 + i) * kBlockBytes);
    };

    // ---- accumulators ----------------------------------------------------------
    // acc[j][i]: channels 32 j.., tokens 32 i.. of the wave tile.  Lane l holds
    // token (l % 32) and, in element v, channel 8 (v / 4) + 4 (l / 32) + v % 4.
    v16i acc[4][2];
    v16f part[4][2];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                acc[j][i][v] = 0;
                part[j][i][v] = 0.f;
            }

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
    auto read_step = [&](auto step, Packed& f, int buf) __attribute__((always_inline)) {
        constexpr int ST = decltype(step)::value;
        const uint32_t aa = a_off[ST] + buf * kStageBytes, bb = b_off[ST] + buf * kStageBytes;
        lds_read16<0 * 2 * kBlockBytes>(f.fa[0], aa);
        lds_read16<1 * 2 * kBlockBytes>(f.fa[1], aa);
        lds_read16<0 * 2 * kBlockBytes>(f.fb[0], bb);
        lds_read16<1 * 2 * kBlockBytes>(f.fb[1], bb);
        lds_read16<2 * 2 * kBlockBytes>(f.fb[2], bb);
        lds_read16<3 * 2 * kBlockBytes>(f.fb[3], bb);
    };
    auto transform = [&](auto is_lo, const Packed& p, Operands& u) __attribute__((always_inline)) {
        if constexpr (decltype(is_lo)::value) {
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                u.ae[i] = p.fa[i] & (int)0x0F0F0F0F;  // even columns: code + 8
                u.ao[i] = p.fa[i] & (int)0xF0F0F0F0;  // odd columns: 16 * code
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                u.be[j] = p.fb[j] & (int)0xF0F0F0F0;  // even columns: 16 * code
                u.bo[j] = p.fb[j] & (int)0x0F0F0F0F;  // odd columns: code + 8
            }
        } else {
#pragma unroll
            for (int i = 0; i < 2; ++i) u.ae[i] = p.fa[i];
#pragma unroll
            for (int j = 0; j < 4; ++j) u.be[j] = p.fb[j];
        }
    };
    // matrix instructions FIRST .. LAST-1 of a step, in an order that keeps two
    // instructions on the same accumulator eight apart
    auto multiply = [&](auto is_lo, auto first, auto last, const Operands& u) __attribute__((always_inline)) {
        constexpr int FIRST = decltype(first)::value, LAST = decltype(last)::value;
#pragma unroll
        for (int q = FIRST; q < LAST; ++q) {
            const int j = (q & 7) >> 1, i = q & 1;
            if (q < 8)
                acc[j][i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(u.be[j], u.ae[i], acc[j][i], 0, 0, 0);
            else
                acc[j][i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(u.bo[j], u.ao[i], acc[j][i], 0, 0, 0);
        }
    };

    // per-lane coordinates of the epilogue
    const int64_t tok0 = m0 + wm * 64 + (lane & 31);
    const int64_t ch0 = n0 + wn * 128 + (lane >> 5) * 4;
    const uint16_t* sw_hi = reinterpret_cast<const uint16_t*>(a.packed + a.L.scale_off);
    const uint16_t* sw_lo = sw_hi + a.L.n_pad;

    // part += A * s_tok[m] * s_ch[n]; acc = 0, where A is the group's integer sum:
    // the accumulator itself for the high group; for the low group
    // (acc - 128 * (even_sum[n] + lo_sum[m])) / 16, an exact division whose 1/16
    // is folded into the scale outside the debug kernel (same fp32 product).
    const int32_t* even_sum = reinterpret_cast<const int32_t*>(a.packed + a.L.scale_off + 4 * a.L.n_pad);
    auto fold = [&](auto is_lo, const float* s_tok, const uint16_t* s_ch, int32_t* dbg) __attribute__((always_inline)) {
        constexpr bool LOW = decltype(is_lo)::value;
        float st[2];
        int ca[2] = {0, 0};
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int64_t m = tok0 + 32 * i;
            st[i] = m < a.M ? s_tok[m] : 0.0f;
            if constexpr (LOW) {
                ca[i] = m < a.M ? a.lo_sum[m] * 128 : 0;
                if constexpr (!DBG) st[i] *= 0.0625f;
            }
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
#pragma unroll
            for (int vq = 0; vq < 4; ++vq) {
                const int64_t n = ch0 + 32 * j + 8 * vq;  // < n_pad always
                const uint2 sc = *reinterpret_cast<const uint2*>(s_ch + n);
                const float sn[4] = {fp16_bits_to_f32(sc.x & 0xFFFFu), fp16_bits_to_f32(sc.x >> 16),
                                     fp16_bits_to_f32(sc.y & 0xFFFFu), fp16_bits_to_f32(sc.y >> 16)};
                int cw[4] = {0, 0, 0, 0};
                if constexpr (LOW) {
                    const int4 e = *reinterpret_cast<const int4*>(even_sum + n);
                    cw[0] = e.x * 128; cw[1] = e.y * 128; cw[2] = e.z * 128; cw[3] = e.w * 128;
                }
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                    const int64_t m = tok0 + 32 * i;
#pragma unroll
                    for (int vr = 0; vr < 4; ++vr) {
                        const int v = vq * 4 + vr;
                        int iv = acc[j][i][v];
                        if constexpr (LOW) {
                            iv -= cw[vr] + ca[i];
                            if constexpr (DBG) iv >>= 4;
                        }
                        part[j][i][v] += (float)iv * (st[i] * sn[vr]);
                        if constexpr (DBG) {
                            if (dbg && m < a.M && n + vr < a.L.N) dbg[m * a.L.N + n + vr] = iv;
                        }
                        acc[j][i][v] = 0;
                    }
                }
            }
        }
        // keep the fp32 tile in accumulation registers while the low steps need
        // the ordinary ones for operands
        if constexpr (!LOW) {
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int i = 0; i < 2; ++i) asm volatile("" : "+a"(part[j][i]));
        }
    };

    // ---- main loop ---------------------------------------------------------------
    using T0 = std::integral_constant<int, 0>;
    using T1 = std::integral_constant<int, 1>;
    using HI = std::false_type;
    using LO = std::true_type;
    {
        Packed px, py;
        Operands ux, uy;
        const int ahead = S < kPrefetch ? S : kPrefetch;
        for (int i = 0; i < ahead; ++i) issue_stage(i, i);
        wait_stage_and_barrier(ahead - 1);  // stage 0 has landed everywhere
        read_step(T0{}, px, 0);
        lds_wait_all(px);
        read_step(T1{}, py, 0);
        if (S_hi > 0) transform(HI{}, px, ux);
        else transform(LO{}, px, ux);

        int buf = 0;
        // One stage = two pipeline slots; `cur` is the kind of this stage's steps,
        // `next` the kind of the next stage's first step.  In each slot the first
        // two matrix instructions are issued before anything else, so that the
        // waits, the barrier and the issue of reads and loads run in their shadow.
        using N0 = std::integral_constant<int, 0>;
        using N2 = std::integral_constant<int, 2>;
        // Scheduling pattern of the second part of a slot: the vector ALU can
        // issue about four instructions in the shadow of one matrix instruction,
        // and only if they sit between two matrix instructions, so the widening
        // of the next step's operands is spread evenly, four per matrix
        // instruction, instead of being bunched at the front.
        auto spread = [&](auto is_lo) __attribute__((always_inline)) {
            constexpr int PAIRS = decltype(is_lo)::value ? 12 : 6;
#pragma unroll
            for (int q = 0; q < PAIRS; ++q) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // one matrix instruction
                __builtin_amdgcn_sched_group_barrier(0x002, 4, 0);  // four vector ALU instructions
            }
        };
        auto stage = [&](auto cur, auto next, int sg) __attribute__((always_inline)) {
            using NM = std::integral_constant<int, decltype(cur)::value ? 16 : 8>;
            const int nxt = buf == kNumBuf - 1 ? 0 : buf + 1;
            const int prv = buf == 0 ? kNumBuf - 1 : buf - 1;
            // invariant: ux = operands of (sg, step 0); py = reads of (sg, step 1) in flight
            __builtin_amdgcn_sched_barrier(0);
            multiply(cur, N0{}, N2{}, ux);
            __builtin_amdgcn_sched_barrier(0);
            // stage sg + 1 has landed everywhere, and every wave is done with stage sg - 1;
            // stages sg + 2 .. sg + 4 may stay in flight
            const int rem = S - 2 - sg;
            wait_stage_and_barrier(rem > 3 ? 3 : rem);
            lds_wait_all(py);
            read_step(T0{}, px, nxt);  // past the last stage: a harmless read of stale LDS
            __builtin_amdgcn_sched_barrier(0);
            if (sg + kPrefetch < S) issue_stage(sg + kPrefetch, prv);
            transform(cur, py, uy);
            multiply(cur, N2{}, NM{}, ux);
            spread(cur);
            __builtin_amdgcn_sched_barrier(0);
            multiply(cur, N0{}, N2{}, uy);
            __builtin_amdgcn_sched_barrier(0);
            lds_wait_all(px);
            read_step(T1{}, py, nxt);
            __builtin_amdgcn_sched_barrier(0);
            transform(next, px, ux);
            multiply(cur, N2{}, NM{}, uy);
            spread(cur);
            __builtin_amdgcn_sched_barrier(0);
            buf = nxt;
        };
        if (S_hi > 0) {
            for (int sg = 0; sg + 1 < S_hi; ++sg) stage(HI{}, HI{}, sg);
            stage(HI{}, LO{}, S_hi - 1);
            fold(HI{}, a.s_hi, sw_hi, a.dbg_hi);
        }
        for (int sg = S_hi; sg < S; ++sg) stage(LO{}, LO{}, sg);
        if (a.stages_lo > 0) fold(LO{}, a.s_lo, sw_lo, a.dbg_lo);
    }

    // ---- write y once --------------------------------------------------------
    wait_loads_and_barrier<0>();  // every wave is done reading the stage buffers
    const bool fast = ((reinterpret_cast<uintptr_t>(a.y) & 15) == 0) && (a.ldy % 8 == 0) &&
                      (n0 + kBN <= a.L.N);
    if (fast) {
        // wave tile (64 tokens x 128 channels, bf16) -> LDS, row-padded; then each
        // store instruction writes four whole 256-byte row segments
        uint8_t* mine = lds + wave * (64 * kOutRowBytes);
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int vq = 0; vq < 4; ++vq) {
                    const uint32_t lo = pack_bf16(part[j][i][vq * 4 + 0], part[j][i][vq * 4 + 1]);
                    const uint32_t hi = pack_bf16(part[j][i][vq * 4 + 2], part[j][i][vq * 4 + 3]);
                    const int row = 32 * i + (lane & 31);
                    const int col = 32 * j + 8 * vq + 4 * (lane >> 5);
                    *reinterpret_cast<uint2*>(mine + row * kOutRowBytes + col * 2) = make_uint2(lo, hi);
                }
        __syncthreads();
#pragma unroll
        for (int it = 0; it < 16; ++it) {
            const int row = it * 4 + (lane >> 4);
            const int64_t m = m0 + wm * 64 + row;
            const uint4 v = *reinterpret_cast<const uint4*>(mine + row * kOutRowBytes + (lane & 15) * 16);
            if (m < a.M)
                *reinterpret_cast<uint4*>(a.y + m * a.ldy + n0 + wn * 128 + (lane & 15) * 8) = v;
        }
    } else {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int64_t m = tok0 + 32 * i;
            if (m >= a.M) continue;
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int vq = 0; vq < 4; ++vq) {
                    const int64_t n = ch0 + 32 * j + 8 * vq;
#pragma unroll
                    for (int vr = 0; vr < 4; ++vr)
                        if (n + vr < a.L.N)
                            a.y[m * a.ldy + n + vr] = (uint16_t)pack_bf16(part[j][i][vq * 4 + vr], 0.f);
                }
        }
    }
}

}  // namespace resq
