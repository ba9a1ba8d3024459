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
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int kGemmThreads = 256;
constexpr int kBM = 128;
constexpr int kBN = 256;
constexpr int kStageABytes = kBM * kRowBytes;  // 16 KiB = 8 blocks
constexpr int kStageBBytes = kBN * kRowBytes;  // 32 KiB = 16 blocks
constexpr int kStageBytes = kStageABytes + kStageBBytes;
constexpr int kLoadsPerStage = (kBM + kBN) / kRowsPerBlock * 2 / 4;  // per lane: 12

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

// 16-byte LDS read whose completion the compiler does not track: the caller
// pairs it with lds_wait_all() on the same registers before using the values.
// (Reads the compiler can see would each be preceded by a wait for every
// direct-to-LDS load in flight, which would serialize the pipeline.)
template <int OFF>
__device__ __forceinline__ void lds_read16(v4i& dst, uint32_t addr) {
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=&v"(dst) : "v"(addr), "n"(OFF));
}

// fragments of one reduction step: 2 activation tiles, 4 weight tiles (32 rows x 32 bytes each)
struct Frags {
    v4i fa[2];
    v4i fb[4];
};

// Wait until every LDS read has returned.  The registers are tied to the wait
// as in/out operands so that no use of them can be scheduled above it.
__device__ __forceinline__ void lds_wait_all(Frags& f) {
    asm volatile("s_waitcnt lgkmcnt(0)"
                 : "+v"(f.fa[0]), "+v"(f.fa[1]), "+v"(f.fb[0]), "+v"(f.fb[1]), "+v"(f.fb[2]),
                   "+v"(f.fb[3]));
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

    // ---- global -> LDS copy --------------------------------------------------
    // One load instruction fills half a block (1 KiB): LDS unit q = lane + 64 h
    // receives row r(q), 16-byte piece kc(q) of the block, so eight consecutive
    // lanes fetch one whole 128-byte line of a row.  Wave w copies A blocks
    // 2w, 2w+1 and B blocks 4w..4w+3 of each stage.  Token rows past M are
    // clamped to the last row (their results are never stored).
    const int r_lo = (lane >> 4) * 2 + ((lane >> 3) & 1);                 // row for h = 0; + 8 for h = 1
    const int kc_h0 = (lane & 7) ^ (lane >> 4);                           // piece for h = 0
    const int kc_h1 = (lane & 7) ^ ((lane >> 4) + 4);                     // piece for h = 1
    const uint8_t* a_src[4];
    const uint8_t* b_src[8];
    auto set_sources = [&](const uint8_t* q, int64_t ld, int64_t first_block) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int blk = wave * 2 + (i >> 1), h = i & 1;
            int64_t row = m0 + blk * 16 + r_lo + 8 * h;
            row = row < a.M ? row : a.M - 1;
            a_src[i] = q + row * ld + (h ? kc_h1 : kc_h0) * 16;
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int blk = wave * 4 + (i >> 1), h = i & 1;
            b_src[i] = a.packed + (n0 / 16 + blk) * a.L.group_bytes + first_block * kBlockBytes +
                       (r_lo + 8 * h) * kRowBytes + (h ? kc_h1 : kc_h0) * 16;
        }
    };
    auto issue_stage = [&](int s, int buf) __attribute__((always_inline)) {
        uint8_t* dst = lds + buf * kStageBytes;
#pragma unroll
        for (int i = 0; i < 4; ++i)
            load_to_lds_16B(a_src[i] + (int64_t)s * kRowBytes, dst + (wave * 4 + i) * 1024);
#pragma unroll
        for (int i = 0; i < 8; ++i)
            load_to_lds_16B(b_src[i] + (int64_t)s * kBlockBytes,
                            dst + kStageABytes + (wave * 8 + i) * 1024);
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
    // An operand tile is 32 rows x 128 bytes (two blocks).  In reduction step s4
    // lane l supplies row (l % 32), piece 2 s4 + l / 32.  off[s4] is the byte
    // offset of that piece inside the tile.
    uint32_t a_off[4], b_off[4];
    {
        const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t*)lds;
        const int R = lane & 31, r = R & 15, g = lane >> 5;
#pragma unroll
        for (int s4 = 0; s4 < 4; ++s4) {
            const int kc = 2 * s4 + g;
            const uint32_t off = (R >> 4) * kBlockBytes + ((r >> 1) * 16 + (r & 1) * 8 + (kc ^ (r >> 1))) * 16;
            a_off[s4] = lds0 + wm * (4 * kBlockBytes) + off;
            b_off[s4] = lds0 + kStageABytes + wn * (8 * kBlockBytes) + off;
        }
    }
    auto read_step = [&](auto step, Frags& f, int buf) __attribute__((always_inline)) {
        constexpr int S4 = decltype(step)::value;
        const uint32_t aa = a_off[S4] + buf * kStageBytes, bb = b_off[S4] + buf * kStageBytes;
        lds_read16<0 * 2 * kBlockBytes>(f.fa[0], aa);
        lds_read16<1 * 2 * kBlockBytes>(f.fa[1], aa);
        lds_read16<0 * 2 * kBlockBytes>(f.fb[0], bb);
        lds_read16<1 * 2 * kBlockBytes>(f.fb[1], bb);
        lds_read16<2 * 2 * kBlockBytes>(f.fb[2], bb);
        lds_read16<3 * 2 * kBlockBytes>(f.fb[3], bb);
    };
    auto mma_step = [&](auto is_lo, Frags& f) __attribute__((always_inline)) {
        if constexpr (decltype(is_lo)::value) {
            v4i ae[2], ao[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                ae[i] = (f.fa[i] << 4) & (int)0xF0F0F0F0;
                ao[i] = f.fa[i] & (int)0xF0F0F0F0;
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const v4i be = (f.fb[j] << 4) & (int)0xF0F0F0F0;
                const v4i bo = f.fb[j] & (int)0xF0F0F0F0;
#pragma unroll
                for (int i = 0; i < 2; ++i)
                    acc[j][i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(be, ae[i], acc[j][i], 0, 0, 0);
#pragma unroll
                for (int i = 0; i < 2; ++i)
                    acc[j][i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(bo, ao[i], acc[j][i], 0, 0, 0);
            }
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int i = 0; i < 2; ++i)
                    acc[j][i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(f.fb[j], f.fa[i], acc[j][i], 0, 0, 0);
        }
    };

    // One group's stages; the buffer of stage s is s % 3, and up to two stages
    // are in flight behind the one being multiplied.  At the top of stage s
    // every wave waits for its own loads of stage s (those of stage s + 1 may
    // stay in flight) and joins the barrier: stage s is then visible to all,
    // and every wave is done with stage s - 1, whose buffer the loads of stage
    // s + 2 then overwrite.  A stage is four reduction steps; the reads of a
    // step are issued before the matrix instructions of the previous one.
    auto run_group = [&](auto is_lo, int stages) __attribute__((always_inline)) {
        using S0 = std::integral_constant<int, 0>;
        using S1 = std::integral_constant<int, 1>;
        using S2 = std::integral_constant<int, 2>;
        using S3 = std::integral_constant<int, 3>;
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
            read_step(S0{}, x, buf);
            lds_wait_all(x);
            read_step(S1{}, y, buf);
            mma_step(is_lo, x);
            __builtin_amdgcn_sched_barrier(0);
            lds_wait_all(y);
            read_step(S2{}, x, buf);
            mma_step(is_lo, y);
            __builtin_amdgcn_sched_barrier(0);
            lds_wait_all(x);
            read_step(S3{}, y, buf);
            mma_step(is_lo, x);
            __builtin_amdgcn_sched_barrier(0);
            lds_wait_all(y);
            mma_step(is_lo, y);
            __builtin_amdgcn_sched_barrier(0);
            buf = buf == 2 ? 0 : buf + 1;
        }
    };

    // per-lane coordinates of the epilogue
    const int64_t tok0 = m0 + wm * 64 + (lane & 31);
    const int64_t ch0 = n0 + wn * 128 + (lane >> 5) * 4;
    const uint16_t* sw_hi = reinterpret_cast<const uint16_t*>(a.packed + a.L.scale_off);
    const uint16_t* sw_lo = sw_hi + a.L.n_pad;

    // part += (acc >> shift) * s_tok[m] * s_ch[n]; acc = 0
    auto fold = [&](const float* s_tok, const uint16_t* s_ch, int32_t* dbg, int shift) __attribute__((always_inline)) {
        float st[2];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int64_t m = tok0 + 32 * i;
            st[i] = m < a.M ? s_tok[m] : 0.0f;
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
#pragma unroll
            for (int vq = 0; vq < 4; ++vq) {
                const int64_t n = ch0 + 32 * j + 8 * vq;  // < n_pad always
                const uint2 sc = *reinterpret_cast<const uint2*>(s_ch + n);
                const float sn[4] = {fp16_bits_to_f32(sc.x & 0xFFFFu), fp16_bits_to_f32(sc.x >> 16),
                                     fp16_bits_to_f32(sc.y & 0xFFFFu), fp16_bits_to_f32(sc.y >> 16)};
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                    const int64_t m = tok0 + 32 * i;
#pragma unroll
                    for (int vr = 0; vr < 4; ++vr) {
                        const int v = vq * 4 + vr;
                        const int iv = acc[j][i][v] >> shift;
                        part[j][i][v] += (float)iv * (st[i] * sn[vr]);
                        if constexpr (DBG) {
                            if (dbg && m < a.M && n + vr < a.L.N) dbg[m * a.L.N + n + vr] = iv;
                        }
                        acc[j][i][v] = 0;
                    }
                }
            }
        }
        // keep the fp32 tile in accumulation registers while the other group's
        // loop needs the ordinary ones for operands
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int i = 0; i < 2; ++i) asm volatile("" : "+a"(part[j][i]));
    };

    if (a.stages_hi > 0) {
        set_sources(a.q_hi, a.ld_hi, 0);
        run_group(std::false_type{}, a.stages_hi);
        fold(a.s_hi, sw_hi, a.dbg_hi, 0);
    }
    if (a.stages_lo > 0) {
        set_sources(a.q_lo, a.ld_lo, a.L.hi_blocks);
        run_group(std::true_type{}, a.stages_lo);
        fold(a.s_lo, sw_lo, a.dbg_lo, 8);
    }

    // ---- write y once --------------------------------------------------------
    const bool vec_ok = ((reinterpret_cast<uintptr_t>(a.y) & 7) == 0) && (a.ldy % 4 == 0);
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int64_t m = tok0 + 32 * i;
        if (m >= a.M) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
#pragma unroll
            for (int vq = 0; vq < 4; ++vq) {
                const int64_t n = ch0 + 32 * j + 8 * vq;
                uint16_t o[4];
#pragma unroll
                for (int vr = 0; vr < 4; ++vr) o[vr] = f32_to_bf16_rne(part[j][i][vq * 4 + vr]);
                uint16_t* dst = a.y + m * a.ldy + n;
                if (vec_ok && n + 3 < a.L.N) {
                    *reinterpret_cast<uint2*>(dst) =
                        make_uint2((uint32_t)o[0] | ((uint32_t)o[1] << 16), (uint32_t)o[2] | ((uint32_t)o[3] << 16));
                } else {
#pragma unroll
                    for (int vr = 0; vr < 4; ++vr)
                        if (n + vr < a.L.N) dst[vr] = o[vr];
                }
            }
        }
    }
}

}  // namespace resq
