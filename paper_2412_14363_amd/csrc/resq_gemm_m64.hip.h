// The tiled mixed INT8/INT4 GEMM (Section 4.1, Eq. 4) on 64 (tokens) x 128
// (channels) tiles, for token counts at which the 128 x 128 tiles of
// resq_gemm.hip.h are fewer than the compute units can take.  Same operands,
// same LDS image of a block, same loads, same nibble arithmetic and the same
// epilogue as there; what differs:
//
// Tiling.  A wavefront owns 32 x 64 outputs: 2 activation fragments x 4 weight
// fragments of the 16x16x64 instruction, 2 x 32 accumulation registers.  A
// stage is 12 KiB (4 activation blocks, 8 weight blocks), three loads per
// wavefront.  Half the products per stage and wavefront means half the time
// per stage: six stage buffers (five stages ahead) keep about the same
// distance in time between a load and its use (more were measured to bring
// nothing); two workgroups still share a compute unit.
//
// Low stages.  With two activation fragments the two products on one
// accumulator tile (even and odd columns) would be two instructions apart in
// the order of the wide kernel; here a stage runs all even-column products
// first and then all odd-column ones (eight apart).  Each half of a weight
// fragment is widened behind the first product of the half before it, into
// one of two registers taking turns.  The widened activation fragments exist
// twice: the next stage's are written while this stage's are multiplied.
//
// Two rings (KS = 2), for layers with at most one such tile per compute unit: a
// single wavefront per SIMD cannot keep the matrix pipe busy by itself, so a
// second set of four wavefronts works on the same tile, taking every other
// pair of stages through a ring of stage buffers of its own; at the end the
// two sets exchange half of their integer tiles through LDS (integer sums:
// exact in any order) and each folds and stores half of the channels.
#pragma once
#include "resq_gemm.hip.h"

namespace resq {

constexpr int kBM64 = 64;
constexpr int kStageABytes64 = kBM64 * kRowBytes;              // 4 KiB = 4 blocks
constexpr int kStageBytes64 = kStageABytes64 + kStageBBytes;   // 12 KiB
constexpr int kLoadsPerStage64 = (kBM64 + kBN) / kRowsPerBlock / 4;  // per wavefront: 3 (one activation block, two weight blocks)
// stage buffers per ring: six for one ring (two workgroups per compute unit), five for each of two
constexpr int num_buf64(int ks) { return ks == 1 ? 6 : 5; }
constexpr int kXchgBytes64 = 8 * 8192;  // KS = 2: eight wavefronts hand over eight four-register tiles each
static_assert(2 * (num_buf64(1) * kStageBytes64 + kMetaBytes) <= 160 * 1024, "LDS of two resident workgroups");
static_assert(2 * num_buf64(2) * kStageBytes64 + kMetaBytes <= 160 * 1024, "LDS of one workgroup with two rings");
static_assert(kBM64 * kOutRowBytes <= num_buf64(1) * kStageBytes64, "the staged output tile fits the stage buffers");
static_assert(kXchgBytes64 + kBM64 * kOutRowBytes <= 2 * num_buf64(2) * kStageBytes64, "exchange area and staged tile fit the rings");

// the fragments of one stage as read from LDS: 2 activation and 4 weight fragments
struct Raw64 {
    v4i a[2];
    v4i b[4];
};
// the activation fragments of a low stage, widened: even columns (code + 8), odd columns (16 * code)
struct Wide64 {
    v4i e[2];
    v4i o[2];
};

// as lds_wait, on two fragments
template <int N>
__device__ __forceinline__ void lds_wait(v4i (&f)[2]) {
    asm volatile("s_waitcnt lgkmcnt(%2)" : "+v"(f[0]), "+v"(f[1]) : "n"(N));
}

// wait until at most `later` (0 .. MAXLATER) stages of LOADS loads each are outstanding, then the barrier
template <int LOADS, int MAXLATER>
__device__ __forceinline__ void wait_stages_and_barrier(int later) {
    if constexpr (MAXLATER > 0) {
        if (later >= MAXLATER) wait_loads_and_barrier<MAXLATER * LOADS>();
        else wait_stages_and_barrier<LOADS, MAXLATER - 1>(later);
    } else {
        wait_loads_and_barrier<0>();
    }
}

// KS = 1: four wavefronts, the whole reduction axis.  KS = 2: eight wavefronts in two halves, each
// half with a ring of its own walking every other PAIR of stages (pairs 0, 2, 4, ... and 1, 3, 5, ...;
// a pair is all high or all low since both stage counts are even); at the end the halves swap
// half of their integer tiles through LDS and each folds and stores half of the channels.
template <bool DBG, int KS>
__global__ __launch_bounds__(kGemmThreads * KS, KS == 1 ? 2 : 1) void gemm_mixed_m64_kernel(const GemmArgs a) {
    constexpr int kNumBuf64 = num_buf64(KS);
    constexpr int kPrefetch64 = kNumBuf64 - 1;  // stages requested ahead of the one being multiplied
    constexpr int kRingBytes = kNumBuf64 * kStageBytes64;
    constexpr int kMetaOff64 = KS * kRingBytes;
    __shared__ __attribute__((aligned(1024))) uint8_t lds[kMetaOff64 + kMetaBytes];

    const int t = threadIdx.x;
    const int lane = t & 63;
    const int wave_wg = __builtin_amdgcn_readfirstlane(t >> 6);   // 0 .. 4 KS - 1
    const int half = KS == 1 ? 0 : wave_wg >> 2;                   // which ring, which pairs of stages
    const int wave = wave_wg & 3;
    const int wm = wave >> 1;  // 0..1: 32-token half of the tile
    const int wn = wave & 1;   // 0..1: 64-channel half of the tile
    uint8_t* const ring = lds + half * kRingBytes;
    int tile_m, tile_n;
    tile_of_block(a, tile_m, tile_n);  // a.tiles_m counts 64-token tiles here
    const int64_t m0 = (int64_t)tile_m * kBM64;
    const int64_t n0 = (int64_t)tile_n * kBN;
    if (n0 >= a.L.N) return;  // a tile of padding channels only
    // all stages of the layer (both counts even), and this half's share of them, in its own numbering
    const int S_hi_all = a.stages_hi, S_all = S_hi_all + a.stages_lo;
    const int S_hi = KS == 1 ? S_hi_all : 2 * ((S_hi_all / 2 - half + 1) / 2);
    const int S = KS == 1 ? S_all : 2 * ((S_all / 2 - half + 1) / 2);
    const int S_lo = S - S_hi;
    const bool any_hi = S_hi_all > 0, any_lo = S_all > S_hi_all;  // the layer has a high (low) group
    // this half's stage k is stage ... of the layer
    auto layer_stage = [&](int k) __attribute__((always_inline)) {
        return KS == 1 ? k : 4 * (k >> 1) + 2 * half + (k & 1);
    };
    const uint16_t* sw_hi = reinterpret_cast<const uint16_t*>(a.packed + a.L.scale_off);
    const uint16_t* sw_lo = sw_hi + a.L.n_pad;
    const int32_t* even_sum = reinterpret_cast<const int32_t*>(a.packed + a.L.scale_off + 4 * a.L.n_pad);
    const bool asym = a.c_hi != nullptr || a.c_lo != nullptr;

    // ---- epilogue constants -> LDS (the oldest loads of their waves) ------------
    // Token rows past M repeat the last row (never stored).
    if (half != 0) {
        // the first ring's wavefronts fetch them
    } else if (wave == 0) {
        if (lane < 32) {
            load_to_lds_16B((lane < 16 ? sw_hi : sw_lo) + n0 + (lane & 15) * 8, lds + kMetaOff64 + kMetaSwHi);
            if (asym) load_to_lds_16B(even_sum + a.L.n_pad + n0 + lane * 4, lds + kMetaOff64 + kMetaWsumHi);
        }
    } else if (wave == 1) {
        if (lane < 32) {
            load_to_lds_16B(even_sum + n0 + lane * 4, lds + kMetaOff64 + kMetaEven);
            if (asym) load_to_lds_16B(even_sum + 2 * a.L.n_pad + n0 + lane * 4, lds + kMetaOff64 + kMetaWsumLo);
        }
    } else {
        int64_t m = m0 + lane;
        m = m < a.M ? m : a.M - 1;
        if (wave == 2) {
            if (any_hi) load_to_lds_4B(a.s_hi + m, lds + kMetaOff64 + kMetaSHi);
            if (any_lo) load_to_lds_4B(a.s_lo + m, lds + kMetaOff64 + kMetaSLo);
        } else {
            if (any_lo) load_to_lds_4B(a.lo_sum + m, lds + kMetaOff64 + kMetaLoSum);
            if (asym && any_hi) load_to_lds_4B(a.c_hi + m, lds + kMetaOff64 + kMetaCHi);
            if (asym && any_lo) load_to_lds_4B(a.c_lo + m, lds + kMetaOff64 + kMetaCLo);
        }
    }

    // ---- global -> LDS copy: wave w copies A block w and B blocks 2w, 2w+1 of each stage ----
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
    const __amdgpu_buffer_rsrc_t rs_a_lo = make_rsrc(a.q_lo + m0 * a.ld_lo - (int64_t)S_hi_all * kRowBytes);
    const __amdgpu_buffer_rsrc_t rs_b = make_rsrc(a.packed + (n0 / 16 + wave * 2) * a.L.group_bytes);
    // load K of this half's stage sg (high stages first) into buffer buf of its ring; K = 0: the A block, 1, 2: the B blocks
    auto issue_load = [&](auto k, int sg, int buf) __attribute__((always_inline)) {
        constexpr int K = decltype(k)::value;
        uint8_t* dst = ring + buf * kStageBytes64;
        const uint32_t g = (uint32_t)layer_stage(sg);
        if constexpr (K == 0) {
            const bool lo = sg >= S_hi;
            buffer_load_to_lds_16B(lo ? rs_a_lo : rs_a_hi, lo ? a_voff_lo : a_voff_hi, g * kRowBytes,
                                   dst + wave * kBlockBytes);
        } else {
            buffer_load_to_lds_16B(rs_b, b_voff[K - 1], g * kBlockBytes,
                                   dst + kStageABytes64 + (wave * 2 + K - 1) * kBlockBytes);
        }
    };
    // the same for a stage known to be a low one
    auto issue_load_lo = [&](auto k, int sg, int buf) __attribute__((always_inline)) {
        constexpr int K = decltype(k)::value;
        uint8_t* dst = ring + buf * kStageBytes64;
        const uint32_t g = (uint32_t)layer_stage(sg);
        if constexpr (K == 0)
            buffer_load_to_lds_16B(rs_a_lo, a_voff_lo, g * kRowBytes, dst + wave * kBlockBytes);
        else
            buffer_load_to_lds_16B(rs_b, b_voff[K - 1], g * kBlockBytes,
                                   dst + kStageABytes64 + (wave * 2 + K - 1) * kBlockBytes);
    };

    // ---- accumulators: acc[j][i]: channels 16 j.., tokens 16 i.. of the wave tile ----
    v4i acc_hi[4][2], acc_lo[4][2];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            acc_hi[j][i] = (v4i){0, 0, 0, 0};
            acc_lo[j][i] = (v4i){0, 0, 0, 0};
        }
    auto park = [&](v4i (&acc)[4][2]) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int i = 0; i < 2; ++i) asm volatile("" : "+a"(acc[j][i]));
    };

    // ---- LDS -> register reads: lane l supplies row l % 16, piece l / 16 of a block ----
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t*)ring;
    uint32_t a_off, b_off;
    {
        const int r = lane & 15, kc = lane >> 4;
        const uint32_t off = (4 * r + (kc ^ (r >> 2))) * 16;
        a_off = lds0 + wm * (2 * kBlockBytes) + off;
        b_off = lds0 + kStageABytes64 + wn * (4 * kBlockBytes) + off;
    }
    // read K of a stage: K = 0, 1: activation fragments, 2..5: weight fragments
    auto read_frag = [&](auto k, Raw64& f, uint32_t aa, uint32_t bb) __attribute__((always_inline)) {
        constexpr int K = decltype(k)::value;
        if constexpr (K < 2) lds_read16<K * kBlockBytes>(f.a[K], aa);
        else lds_read16<(K - 2) * kBlockBytes>(f.b[K - 2], bb);
    };

    // ---- epilogue: as in the wide kernel, on two token fragments ---------------------
    const int tl = wm * 32 + (lane & 15);
    const int cl = wn * 64 + (lane >> 4) * 4;
    // KS = 2: this half folds the weight fragments J0, J0 + 1 only, and the tile is staged behind the exchange area
    uint8_t* const staged = lds + (KS == 1 ? 0 : kXchgBytes64);
    auto fold = [&](auto has_hi, auto has_lo, auto is_asym, auto is_glu, auto j0_) __attribute__((always_inline)) {
        constexpr bool HI_ON = decltype(has_hi)::value, LO_ON = decltype(has_lo)::value;
        constexpr bool ASYM = decltype(is_asym)::value, GLU = decltype(is_glu)::value;
        constexpr int J0 = decltype(j0_)::value;
        const uint8_t* meta = lds + kMetaOff64;
        float st_hi[2], st_lo[2], ct_hi[2], ct_lo[2];
        int ca[2];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
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
        int32_t* dbg_row_hi[2] = {nullptr, nullptr};
        int32_t* dbg_row_lo[2] = {nullptr, nullptr};
        bool dbg_ok[2] = {false, false};
        int dbg_cols = 0;
        if constexpr (DBG) {
            dbg_cols = (int)(a.L.N - n0 - cl);
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int64_t m = m0 + tl + 16 * i;
                dbg_ok[i] = m < a.M;
                dbg_row_hi[i] = a.dbg_hi + m * a.L.N + n0 + cl;
                dbg_row_lo[i] = a.dbg_lo + m * a.L.N + n0 + cl;
            }
        }
#pragma unroll
        for (int j = J0; j < J0 + 4 / KS; ++j) {
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
            for (int i = 0; i < 2; ++i) {
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
                    *reinterpret_cast<uint32_t*>(staged + row * kOutRowBytes + c) =
                        pack_bf16(silu_f32(val[0]) * val[1], silu_f32(val[2]) * val[3]);
                else
                    *reinterpret_cast<uint2*>(staged + row * kOutRowBytes + c * 2) =
                        make_uint2(pack_bf16(val[0], val[1]), pack_bf16(val[2], val[3]));
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // ---- main loop ---------------------------------------------------------------
    {
        Raw64 p0, p1;     // the stage being multiplied and the next one, as read, taking turns
        Wide64 w0, w1;    // their widened activation fragments (low stages)
        v4i bw[2];        // the halves of the weight fragments of a low stage, taking turns
        const int ahead = S < kPrefetch64 ? S : kPrefetch64;
        for (int i = 0; i < ahead; ++i)
            static_for<kLoadsPerStage64>([&](auto k) __attribute__((always_inline)) { issue_load(k, i, i); });
        wait_stages_and_barrier<kLoadsPerStage64, kPrefetch64 - 1>(ahead - 1);  // stage 0 and the constants have landed
        static_for<6>([&](auto k) __attribute__((always_inline)) { read_frag(k, p0, a_off, b_off); });

        using YES = std::true_type;
        using NO = std::false_type;
        int buf = 0;
        // A low stage: 16 products in 8 groups (g = 4 * half + weight fragment) of two (the
        // activation fragments).  Invariant at entry: cur has landed, wc holds its widened
        // activation fragments and bw[0] the even half of weight fragment 0.  After the
        // barrier: the six reads of the next stage (activation fragments first), which are
        // widened into wn as they land, and the three loads of stage sg + kPrefetch64.
        auto stage_lo = [&](auto steady, Raw64& cur, Raw64& nx, Wide64& wc, Wide64& wn_, int sg) __attribute__((always_inline)) {
            // STEADY: stage sg + kPrefetch64 exists (known to the caller): loads and wait unconditional
            constexpr bool STEADY = decltype(steady)::value;
            const int nbuf = buf == kNumBuf64 - 1 ? 0 : buf + 1;
            const int prv = buf == 0 ? kNumBuf64 - 1 : buf - 1;
            const uint32_t shift = nbuf * kStageBytes64;
            const bool issue = STEADY || sg + kPrefetch64 < S;
            park(acc_hi);
            static_for<16>([&](auto s_) __attribute__((always_inline)) {
                constexpr int SL = decltype(s_)::value;
                constexpr int G = SL >> 1, I = SL & 1, J = G & 3;
                __builtin_amdgcn_sched_barrier(0);
                if constexpr (G < 4) mfma_16x16x64(acc_lo[J][I], bw[G & 1], wc.e[I]);
                else mfma_16x16x64(acc_lo[J][I], bw[G & 1], wc.o[I]);
                if constexpr (I == 0) {
                    // the half for the next group (weights: even columns 16 * code, odd columns code + 8)
                    constexpr int GN = G + 1;
                    if constexpr (GN < 8) bw[GN & 1] = cur.b[GN & 3] & (GN < 4 ? (int)0xF0F0F0F0 : (int)0x0F0F0F0F);
                    else bw[0] = nx.b[0] & (int)0xF0F0F0F0;
                    pin(bw[GN & 1]);
                }
                if constexpr (SL == 1) asm volatile("s_nop 0");  // keeps the widening two instructions ahead of its product
                if constexpr (SL == 3) {
                    // stage sg + 1 has landed everywhere, and every wave is done with stage sg - 1
                    __builtin_amdgcn_sched_barrier(0);
                    if constexpr (STEADY) {
                        wait_loads_and_barrier<(kPrefetch64 - 2) * kLoadsPerStage64>();
                    } else {
                        const int rem = S - 2 - sg;
                        wait_stages_and_barrier<kLoadsPerStage64, kPrefetch64 - 2>(rem);
                    }
                }
                if constexpr (SL >= 4 && SL <= 9) read_frag(IC<SL - 4>{}, nx, a_off + shift, b_off + shift);
                if constexpr (SL == 10) { if (issue) issue_load_lo(IC<0>{}, sg + kPrefetch64, prv); }
                if constexpr (SL == 12) { if (issue) issue_load_lo(IC<1>{}, sg + kPrefetch64, prv); }
                if constexpr (SL == 14) { if (issue) issue_load_lo(IC<2>{}, sg + kPrefetch64, prv); }
                // the next stage's activation fragments (the first two reads) and, before slot 14
                // reads it, its weight fragments
                if constexpr (SL == 9) {
                    lds_wait<4>(nx.a);
                    wn_.e[0] = nx.a[0] & (int)0x0F0F0F0F;
                    pin(wn_.e[0]);
                }
                if constexpr (SL == 11) {
                    wn_.e[1] = nx.a[1] & (int)0x0F0F0F0F;
                    pin(wn_.e[1]);
                }
                if constexpr (SL == 13) {
                    lds_wait<0>(nx.b);
                    wn_.o[0] = nx.a[0] & (int)0xF0F0F0F0;
                    pin(wn_.o[0]);
                }
                if constexpr (SL == 15) {
                    wn_.o[1] = nx.a[1] & (int)0xF0F0F0F0;
                    pin(wn_.o[1]);
                }
            });
            __builtin_amdgcn_sched_barrier(0);
            buf = nbuf;
        };
        // A high stage: 4 x 2 products on the fragments as read.  Invariant at entry: the six
        // reads of this stage into cur have been issued.
        auto stage_hi = [&](auto steady, Raw64& cur, Raw64& nx, int sg) __attribute__((always_inline)) {
            constexpr bool STEADY = decltype(steady)::value;
            const int nbuf = buf == kNumBuf64 - 1 ? 0 : buf + 1;
            const int prv = buf == 0 ? kNumBuf64 - 1 : buf - 1;
            const uint32_t shift = nbuf * kStageBytes64;
            const bool issue = STEADY || sg + kPrefetch64 < S;
            park(acc_lo);
            __builtin_amdgcn_sched_barrier(0);
            lds_wait<0>(cur.a);
            lds_wait<0>(cur.b);
            static_for<8>([&](auto s_) __attribute__((always_inline)) {
                constexpr int SL = decltype(s_)::value;
                constexpr int J = SL >> 1, I = SL & 1;
                __builtin_amdgcn_sched_barrier(0);
                mfma_16x16x64(acc_hi[J][I], cur.b[J], cur.a[I]);
                if constexpr (SL == 1) {
                    __builtin_amdgcn_sched_barrier(0);
                    if constexpr (STEADY) {
                        wait_loads_and_barrier<(kPrefetch64 - 2) * kLoadsPerStage64>();
                    } else {
                        const int rem = S - 2 - sg;
                        wait_stages_and_barrier<kLoadsPerStage64, kPrefetch64 - 2>(rem);
                    }
                }
                if constexpr (SL >= 2) read_frag(IC<SL - 2>{}, nx, a_off + shift, b_off + shift);
                if constexpr (SL == 3) { if (issue) issue_load(IC<0>{}, sg + kPrefetch64, prv); }
                if constexpr (SL == 5) { if (issue) issue_load(IC<1>{}, sg + kPrefetch64, prv); }
                if constexpr (SL == 7) { if (issue) issue_load(IC<2>{}, sg + kPrefetch64, prv); }
            });
            __builtin_amdgcn_sched_barrier(0);
            buf = nbuf;
        };
        int sg = 0;
        for (; sg < S_hi && sg + 1 + kPrefetch64 < S; sg += 2) {
            stage_hi(YES{}, p0, p1, sg);
            stage_hi(YES{}, p1, p0, sg + 1);
        }
        for (; sg < S_hi; sg += 2) {
            stage_hi(NO{}, p0, p1, sg);
            stage_hi(NO{}, p1, p0, sg + 1);
        }
        if (S_lo > 0) {
            // p0 holds the first low stage, as read: widen its activation fragments and half a weight fragment
            lds_wait<0>(p0.a);
            lds_wait<0>(p0.b);
            static_for<2>([&](auto i_) __attribute__((always_inline)) {
                constexpr int I = decltype(i_)::value;
                w0.e[I] = p0.a[I] & (int)0x0F0F0F0F;
                pin(w0.e[I]);
                w0.o[I] = p0.a[I] & (int)0xF0F0F0F0;
                pin(w0.o[I]);
            });
            bw[0] = p0.b[0] & (int)0xF0F0F0F0;
            pin(bw[0]);
            asm volatile("s_nop 4" ::: "memory");  // wait states between the widening and the first product
            for (; sg + 1 + kPrefetch64 < S; sg += 2) {
                stage_lo(YES{}, p0, p1, w0, w1, sg);
                stage_lo(YES{}, p1, p0, w1, w0, sg + 1);
            }
            for (; sg < S; sg += 2) {
                stage_lo(NO{}, p0, p1, w0, w1, sg);
                stage_lo(NO{}, p1, p0, w1, w0, sg + 1);
            }
        }
        // the reads past the last stage went into p0: let them land before its registers are reused
        lds_wait<0>(p0.a);
        lds_wait<0>(p0.b);
        if constexpr (KS == 2) {
            // Every stage holds one workgroup barrier, and the first half may have one pair of
            // stages more than this one: join its two barriers.
            if (S < 2 * ((S_all / 2 + 1) / 2)) {
                wait_loads_and_barrier<0>();
                wait_loads_and_barrier<0>();
            }
        }
        wait_loads_and_barrier<0>();  // every wave is done reading the stage buffers
        asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");  // the last matrix instructions have written their tiles
        if constexpr (KS == 2) {
            // The first half folds weight fragments 0, 1 and the second 2, 3: wavefront (half, w)
            // hands the other two of its own (both integer sets, 8 tiles of 1 KiB) to wavefront
            // (1 - half, w) and adds what that one hands over.  Integer sums: exact in any order.
            auto tile_at = [&](int slot, int idx) __attribute__((always_inline)) {
                return reinterpret_cast<v4i*>(lds + slot * 8192 + idx * 1024 + lane * 16);
            };
            auto send = [&](auto j0_) __attribute__((always_inline)) {
                constexpr int J0 = decltype(j0_)::value;
                const int slot = (1 - half) * 4 + wave;
#pragma unroll
                for (int jj = 0; jj < 2; ++jj)
#pragma unroll
                    for (int i = 0; i < 2; ++i) {
                        *tile_at(slot, jj * 2 + i) = acc_hi[J0 + jj][i];
                        *tile_at(slot, 4 + jj * 2 + i) = acc_lo[J0 + jj][i];
                    }
            };
            auto receive = [&](auto j0_) __attribute__((always_inline)) {
                constexpr int J0 = decltype(j0_)::value;
                const int slot = half * 4 + wave;
#pragma unroll
                for (int jj = 0; jj < 2; ++jj)
#pragma unroll
                    for (int i = 0; i < 2; ++i) {
                        acc_hi[J0 + jj][i] += *tile_at(slot, jj * 2 + i);
                        acc_lo[J0 + jj][i] += *tile_at(slot, 4 + jj * 2 + i);
                    }
            };
            if (half == 0) send(IC<2>{}); else send(IC<0>{});
            __syncthreads();
            if (half == 0) receive(IC<0>{}); else receive(IC<2>{});
        }
        auto fold_from = [&](auto j0_) __attribute__((always_inline)) {
            if (a.swiglu) {  // symmetric codes only (checked on the host)
                if (any_hi && any_lo) fold(YES{}, YES{}, NO{}, YES{}, j0_);
                else if (any_hi) fold(YES{}, NO{}, NO{}, YES{}, j0_);
                else fold(NO{}, YES{}, NO{}, YES{}, j0_);
            } else if (asym) {
                if (any_hi && any_lo) fold(YES{}, YES{}, YES{}, NO{}, j0_);
                else if (any_hi) fold(YES{}, NO{}, YES{}, NO{}, j0_);
                else fold(NO{}, YES{}, YES{}, NO{}, j0_);
            } else {
                if (any_hi && any_lo) fold(YES{}, YES{}, NO{}, NO{}, j0_);
                else if (any_hi) fold(YES{}, NO{}, NO{}, NO{}, j0_);
                else fold(NO{}, YES{}, NO{}, NO{}, j0_);
            }
        };
        if (KS == 1 || half == 0) fold_from(IC<0>{});
        else fold_from(IC<2>{});
    }

    // ---- write y once: each wavefront of the workgroup stores 16 / KS rows of the staged tile ----
    constexpr int kRowsPerWave = 16 / KS;
    __syncthreads();
    const bool fast = ((reinterpret_cast<uintptr_t>(a.y) & 15) == 0) && (a.ldy % 8 == 0) &&
                      (n0 + kBN <= a.L.N);
    if (a.swiglu) {
        const int64_t n_out = a.L.N / 2;
#pragma unroll
        for (int it = 0; it < kRowsPerWave / 8; ++it) {
            const int row = wave_wg * kRowsPerWave + it * 8 + (lane >> 3);
            const int64_t m = m0 + row;
            const int64_t n = n0 / 2 + (lane & 7) * 8;
            const uint4 v = *reinterpret_cast<const uint4*>(staged + row * kOutRowBytes + (lane & 7) * 16);
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
    for (int it = 0; it < kRowsPerWave / 4; ++it) {
        const int row = wave_wg * kRowsPerWave + it * 4 + (lane >> 4);
        const int64_t m = m0 + row;
        const int64_t n = n0 + (lane & 15) * 8;
        const uint4 v = *reinterpret_cast<const uint4*>(staged + row * kOutRowBytes + (lane & 15) * 16);
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
