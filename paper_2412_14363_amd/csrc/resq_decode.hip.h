// Weight-streaming variant of the mixed INT8/INT4 layer for M <= 16 tokens
// (Section 4.1, Eq. 4; the generation stage, which the paper's introduction
// calls memory-bound).  The packed weights are read from HBM exactly once, in
// 1 KiB blocks that are already one operand of the 16x16x64 int8 matrix-core
// instruction (16 channels x 64 bytes, see resq_layout.h): lane l loads row
// l % 16, 16-byte piece l / 16 straight into operand registers, no LDS in
// between, and a wavefront walks the contiguous blocks of one 16-channel group
// (all high blocks, then all low blocks) with a ring of eight loads in flight,
// of which it only ever waits for the oldest (see stream_run for what that takes).
// One workgroup of eight wavefronts runs per compute unit, and groups are dealt
// round-robin over compute units first, so that every unit streams the same
// number of bytes.  The activation codes of all tokens (at most a few tens of
// KiB) are read from L2 as they are needed.  The matrix cores are nearly idle here; they are used because
// the vector ALU could not keep up with 8 TB/s of nibbles at M = 16.
//
// Roofline: HBM.  Algorithmic bytes = the packed weight buffer.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "resq_gemm.hip.h"
#include "resq_layout.h"
#include "resq_quantize.hip.h"

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
    // quantizer fused in front (kernels built with FUSED): the bf16 activations, [M][ldx];
    // q_hi .. lo_sum above are not read then
    const uint16_t* x;
    int64_t ldx;
    int fuse_rows;    // rows quantized at a time: 1, 2, 4 or 8
};

constexpr int kFusedScratchFloats = 3 * 16 + 8 * 3;  // LDS beside the token rows, see fill_act_quantize

// Epilogue of the weight-streaming kernels for one lane: token `tok`, channels
// n .. n + 3, the two integer sums of each.  Dequantizes (Eq. 4), adds the
// zero-point term of asymmetric activation codes, applies the gated pair
// epilogue when asked, writes bf16 (and the integer sums in the debug build).
// The per-token and per-channel constants it needs are a separate step, so that
// a kernel can ask for them before it starts on the weights: they then arrive
// under the stream instead of as two dependent memory round trips after it
// (measured: 2 to 6 % on the short runs of the kernel that cuts the reduction
// axis, nothing on the long runs of the plain one, which therefore asks late).
struct EpilogueConsts {
    float sth, stl, cth, ctl;
    int ca;
    float snh[4], snl[4];
    int ev[4];
    int wsh[4], wsl[4];  // asymmetric activation codes only
};
__device__ __forceinline__ EpilogueConsts load_epilogue_consts(const DecodeArgs& a, int tok, int64_t n) {
    const uint16_t* sw_hi = reinterpret_cast<const uint16_t*>(a.packed + a.L.scale_off);
    const uint16_t* sw_lo = sw_hi + a.L.n_pad;
    const int32_t* even_sum = reinterpret_cast<const int32_t*>(a.packed + a.L.scale_off + 4 * a.L.n_pad);
    const int32_t* wsum_hi = even_sum + a.L.n_pad;
    const int32_t* wsum_lo = even_sum + 2 * a.L.n_pad;
    const bool has_hi = a.L.r > 0, has_lo = a.L.K - a.L.r > 0;
    const bool asym = a.c_hi != nullptr || a.c_lo != nullptr;
    EpilogueConsts c;
    c.sth = has_hi ? a.s_hi[tok] : 0.f;
    c.stl = has_lo ? a.s_lo[tok] : 0.f;
    c.ca = has_lo ? a.lo_sum[tok] : 0;
    c.cth = (asym && has_hi) ? a.c_hi[tok] : 0.f;
    c.ctl = (asym && has_lo) ? a.c_lo[tok] : 0.f;
    const uint2 sch = *reinterpret_cast<const uint2*>(sw_hi + n);
    const uint2 scl = *reinterpret_cast<const uint2*>(sw_lo + n);
    const int4 es = *reinterpret_cast<const int4*>(even_sum + n);
    c.snh[0] = fp16_bits_to_f32(sch.x & 0xFFFFu);
    c.snh[1] = fp16_bits_to_f32(sch.x >> 16);
    c.snh[2] = fp16_bits_to_f32(sch.y & 0xFFFFu);
    c.snh[3] = fp16_bits_to_f32(sch.y >> 16);
    c.snl[0] = fp16_bits_to_f32(scl.x & 0xFFFFu);
    c.snl[1] = fp16_bits_to_f32(scl.x >> 16);
    c.snl[2] = fp16_bits_to_f32(scl.y & 0xFFFFu);
    c.snl[3] = fp16_bits_to_f32(scl.y >> 16);
    c.ev[0] = es.x;
    c.ev[1] = es.y;
    c.ev[2] = es.z;
    c.ev[3] = es.w;
#pragma unroll
    for (int v = 0; v < 4; ++v) {
        c.wsh[v] = asym ? wsum_hi[n + v] : 0;
        c.wsl[v] = asym ? wsum_lo[n + v] : 0;
    }
    return c;
}

template <bool DBG>
__device__ __forceinline__ void stream_epilogue(const DecodeArgs& a, int tok, int64_t n, const EpilogueConsts& c,
                                                v4i acc_hi, v4i acc_lo) {
    const bool asym = a.c_hi != nullptr || a.c_lo != nullptr;
    float out[4];
#pragma unroll
    for (int v = 0; v < 4; ++v) {
        const int a_hi = acc_hi[v];
        const int a_lo = (acc_lo[v] - 128 * (c.ev[v] + c.ca)) >> 4;  // exact
        out[v] = (float)a_hi * (c.sth * c.snh[v]) + (float)a_lo * (c.stl * c.snl[v]);
        if (asym) out[v] += c.cth * ((float)c.wsh[v] * c.snh[v]) + c.ctl * ((float)c.wsl[v] * c.snl[v]);
        if constexpr (DBG) {
            if (n + v < a.L.N) {
                if (a.dbg_hi) a.dbg_hi[(int64_t)tok * a.L.N + n + v] = a_hi;
                if (a.dbg_lo) a.dbg_lo[(int64_t)tok * a.L.N + n + v] = a_lo;
            }
        }
    }
    if (a.swiglu) {
        // two (gate, up) pairs per lane -> two outputs
        const int64_t ch = n >> 1, ch_end = a.L.N >> 1;
        uint16_t* d2 = a.y + (int64_t)tok * a.ldy + ch;
        const uint32_t pair = pack_bf16(silu_f32(out[0]) * out[1], silu_f32(out[2]) * out[3]);
        if (ch + 1 < ch_end && ((reinterpret_cast<uintptr_t>(a.y) & 3) == 0) && (a.ldy % 2 == 0)) {
            *reinterpret_cast<uint32_t*>(d2) = pair;
        } else {
            if (ch < ch_end) d2[0] = (uint16_t)pair;
            if (ch + 1 < ch_end) d2[1] = (uint16_t)(pair >> 16);
        }
        return;
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
template <bool DBG>
__device__ __forceinline__ void stream_epilogue(const DecodeArgs& a, int tok, int64_t n, v4i acc_hi,
                                                v4i acc_lo) {
    stream_epilogue<DBG>(a, tok, n, load_epilogue_consts(a, tok, n), acc_hi, acc_lo);
}

// The per-token quantizer (Section 4.1 Eq. 2, symmetric) run by the workgroup itself on
// the M bf16 rows of a.x, codes straight into the LDS rows: with a handful of tokens
// every workgroup can afford to redo it, which saves a kernel launch in front of the
// weight stream.  The arithmetic is the quantizer kernel's (absmax8, group_scale,
// quant8), so the codes, scales and sums are the ones resq_quantize_act would have
// written.  R = a.fuse_rows (1, 2, 4 or 8) rows are in flight at a time, each with a team
// of 512 / R threads that holds the whole row in registers (at most kFusedUnits 16-byte
// loads per thread, all issued before the first is used: one memory latency per batch
// of rows, not per row), reduces its maxima through LDS and quantizes from registers.
// scal: [3][16] floats = s_hi, s_lo, lo_sum (as int) per token, then reduction scratch.
// Requires K, r, ldx multiples of 8, 16-byte aligned rows, K / 8 <= kFusedUnits * 512 / R.
constexpr int kFusedUnits = 16;
__device__ __forceinline__ void fill_act_quantize(const DecodeArgs& a, uint8_t* act, float* scal, int t) {
    constexpr int kWaves = kDecodeThreads / 64;
    const int lane = t & 63, wave = t >> 6;
    const int K = (int)a.L.K, r = (int)a.L.r;
    const int nunits = K >> 3, hi_units = r >> 3;
    const int R = a.fuse_rows, T = kDecodeThreads / R, WT = T / 64;
    const int team = t / T, tt = t - team * T;
    float* red = scal + 3 * 16;                                      // [8 waves][2]
    int* red_sum = reinterpret_cast<int*>(scal + 3 * 16 + kWaves * 2);  // [8 waves]
    for (int m0 = 0; m0 < a.M; m0 += R) {   // the same trip count for every thread
        const int m = m0 + team;
        const bool live = m < a.M;
        const uint4* row = reinterpret_cast<const uint4*>(a.x + (int64_t)(live ? m : a.M - 1) * a.ldx);
        uint4 v[kFusedUnits];
#pragma unroll
        for (int i = 0; i < kFusedUnits; ++i) {
            const int u = tt + i * T;
            v[i] = make_uint4(0u, 0u, 0u, 0u);
            if (i * T >= nunits) continue;   // the same for every thread
            if (u < nunits) v[i] = row[u];
        }
        float ah = 0.0f, al = 0.0f;
#pragma unroll
        for (int i = 0; i < kFusedUnits; ++i) {
            if (i * T >= nunits) break;
            const int u = tt + i * T;
            const float x = absmax8(v[i]);   // zero past the row
            if (u < hi_units) ah = fmaxf(ah, x);
            else al = fmaxf(al, x);
        }
        ah = wave_max(ah);
        al = wave_max(al);
        if (lane == 0) {
            red[wave * 2] = ah;
            red[wave * 2 + 1] = al;
        }
        __syncthreads();
        ah = 0.0f;
        al = 0.0f;
        for (int w = 0; w < WT; ++w) {
            ah = fmaxf(ah, red[(team * WT + w) * 2]);
            al = fmaxf(al, red[(team * WT + w) * 2 + 1]);
        }
        const float sh = group_scale(ah, kQmaxHi), sl = group_scale(al, kQmaxLo);
        const float inv_h = 1.0f / sh, inv_l = 1.0f / sl;
        if (tt == 0 && live) {
            scal[m] = sh;
            scal[16 + m] = sl;
        }
        uint8_t* arow = act + (live ? m : 0) * a.lds_row;
        uint8_t* alow = arow + a.L.kh_pad;
        float odd_f = 0.0f, unused = 0.0f;
#pragma unroll
        for (int i = 0; i < kFusedUnits; ++i) {
            if (i * T >= nunits) break;
            const int u = tt + i * T;
            if (u < nunits && live) {
                uint32_t c[8];
                if (u < hi_units) {
                    quant8<false>(v[i], sh, inv_h, c, unused);
                    *reinterpret_cast<uint2*>(arow + u * 8) =
                        make_uint2(pack_low_bytes(c[0], c[1], c[2], c[3]), pack_low_bytes(c[4], c[5], c[6], c[7]));
                } else {
                    quant8<true>(v[i], sl, inv_l, c, odd_f);
                    uint32_t by[4];
#pragma unroll
                    for (int k = 0; k < 4; ++k) by[k] = (c[2 * k + 1] << 4) | c[2 * k];
                    *reinterpret_cast<uint32_t*>(alow + (u - hi_units) * 4) = pack_low_bytes(by[0], by[1], by[2], by[3]);
                }
            }
        }
        if (live) {   // zero codes in the padding of both parts of the row
            for (int b = r + 8 * tt; b < (int)a.L.kh_pad; b += 8 * T)
                *reinterpret_cast<uint2*>(arow + b) = make_uint2(0u, 0u);
            for (int b = (K - r) / 2 + 4 * tt; b < (int)(a.L.kl_pad / 2); b += 4 * T)
                *reinterpret_cast<uint32_t*>(alow + b) = 0x08080808u;
        }
        const int odd = wave_sum((int)odd_f);
        if (lane == 0) red_sum[wave] = odd;
        __syncthreads();
        if (tt == 0 && live) {
            int sum = 0;
            for (int w = 0; w < WT; ++w) sum += red_sum[team * WT + w];
            reinterpret_cast<int*>(scal)[32 + m] = sum;
        }
    }
    __syncthreads();
}

// the arguments as the epilogue reads them: with the fused quantizer the per-token
// constants sit in LDS
template <bool FUSED>
__device__ __forceinline__ DecodeArgs epilogue_args(const DecodeArgs& a, const float* scal) {
    DecodeArgs e = a;
    if constexpr (FUSED) {
        e.s_hi = scal;
        e.s_lo = scal + 16;
        e.lo_sum = reinterpret_cast<const int32_t*>(scal + 32);
    }
    return e;
}

// Where a wavefront's activation operand comes from: straight from the code rows in memory
// through a second ring beside the weight ring (no LDS, no barrier: the first matrix
// instruction waits for nothing but its own two loads; the code rows are a few KiB per
// token, stay in L2, and every wavefront reads its part of them once per group), or from
// LDS rows into which the workgroup itself has quantized the bf16 activations.
enum : int { kActQuantize = 1, kActDirect = 2 };

// lane's pointers to its 16-byte piece of block 0 of the high and of the low codes of its
// token (the low pointer moved back by the high blocks, so that both take the block index)
struct ActPieces {
    const uint8_t* hi;
    const uint8_t* lo;
    int hi_blocks;
    __device__ __forceinline__ uint4 operator()(int b) const {
        return *reinterpret_cast<const uint4*>((b < hi_blocks ? hi : lo) + (int64_t)b * kRowBytes);
    }
};
__device__ __forceinline__ ActPieces act_pieces(const DecodeArgs& a, int lane, bool tok_live) {
    const int tok = tok_live ? (lane & 15) : 0;
    ActPieces p;
    p.hi_blocks = (int)a.L.hi_blocks;
    p.hi = a.q_hi + (int64_t)tok * a.ld_hi + (lane >> 4) * 16;
    p.lo = a.q_lo + (int64_t)tok * a.ld_lo + (lane >> 4) * 16 - (int64_t)p.hi_blocks * kRowBytes;
    return p;
}

// A 16-byte piece of the packed weights, read with the non-temporal hint: the weights pass
// through once per call, and without the hint they push the tokens' code rows, which every
// wavefront reads again and again, out of the caches (measured on the 132 MB up projection
// at M = 1: 5.5 -> 6.2 TB/s).
typedef unsigned int v4u_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 load_weights_16B(const uint4* p) {
    const v4u_t v = __builtin_nontemporal_load(reinterpret_cast<const v4u_t*>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
}

// One run of a wavefront: blocks [b_begin, b_end) of a channel group meet the tokens'
// codes; the sums go to acc_hi / acc_lo.  On entry ring[i] (and aring[i], when the codes
// come straight from memory) holds block b_begin + i for every i < min(kDecodeDepth,
// b_end - b_begin); wp points at the lane's piece of the group's block 0.  While a turn of
// kDecodeDepth blocks is multiplied, the loads of the turn after it go out, slot by slot.
// Turns whose blocks are all of one kind and whose refills all exist are straight-line
// code without a branch, in loops of their own: only then does the compiler count the
// outstanding loads exactly and wait for just the oldest one, instead of draining the
// ring at every turn (it gives up at the joins of conditional loads).  Nothing here
// depends on the lane: lanes of tokens past M carry token 0's codes and produce sums in
// output columns that are never stored.
template <bool DIRECT>
__device__ __forceinline__ void stream_run(uint4 (&ring)[kDecodeDepth], uint4 (&aring)[DIRECT ? kDecodeDepth : 1],
                                           const uint4* wp, const ActPieces& piece, const uint8_t* arow,
                                           int b_begin, int b_end, int hi_blocks, v4i& acc_hi, v4i& acc_lo) {
    constexpr int D = kDecodeDepth;
    auto product = [&](bool hi, const uint4& wq, const v4i& p) __attribute__((always_inline)) {
        const v4i w = {(int)wq.x, (int)wq.y, (int)wq.z, (int)wq.w};
        if (hi) {
            acc_hi = __builtin_amdgcn_mfma_i32_16x16x64_i8(w, p, acc_hi, 0, 0, 0);
        } else {
            // see resq_gemm.hip.h: one operand of each product carries an offset of 8
            acc_lo = __builtin_amdgcn_mfma_i32_16x16x64_i8(w & (int)0xF0F0F0F0, p & (int)0x0F0F0F0F, acc_lo, 0, 0, 0);
            acc_lo = __builtin_amdgcn_mfma_i32_16x16x64_i8(w & (int)0x0F0F0F0F, p & (int)0xF0F0F0F0, acc_lo, 0, 0, 0);
        }
    };
    // KIND 0: all high, 1: all low, 2: the turn that holds the boundary
    auto full_turn = [&](auto kind, int b0) __attribute__((always_inline)) {
        constexpr int KIND = decltype(kind)::value;
#pragma unroll
        for (int i = 0; i < D; ++i) {
            const int b = b0 + i;
            v4i p;
            if constexpr (DIRECT) p = v4i{(int)aring[i].x, (int)aring[i].y, (int)aring[i].z, (int)aring[i].w};
            else p = *reinterpret_cast<const v4i*>(arow + b * kRowBytes);
            product(KIND == 0 || (KIND == 2 && b < hi_blocks), ring[i], p);
            // the slot is refilled only after its product has been issued: old and new value
            // never live side by side, so the ring stays in the same registers from turn to
            // turn (a copy of a register just loaded would wait for that load)
            __builtin_amdgcn_sched_barrier(0);
            ring[i] = load_weights_16B(&wp[(b + D) * (kBlockBytes / 16)]);
            if constexpr (DIRECT) aring[i] = piece(b + D);
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    // The ring was filled a moment ago under conditions; waiting for all of it here costs
    // next to nothing (its loads went out back to back) and hands the loops below a state
    // the compiler can count from.  vmcnt(0), other counters untouched.
    __builtin_amdgcn_s_waitcnt(0x0F70);
    int b0 = b_begin;
    while (b0 + D <= hi_blocks && b0 + 2 * D <= b_end) {
        full_turn(std::integral_constant<int, 0>{}, b0);
        b0 += D;
    }
    if (b0 < hi_blocks && b0 + 2 * D <= b_end) {
        full_turn(std::integral_constant<int, 2>{}, b0);
        b0 += D;
    }
    while (b0 >= hi_blocks && b0 + 2 * D <= b_end) {
        full_turn(std::integral_constant<int, 1>{}, b0);
        b0 += D;
    }
    // the last turns: some refills, then none
    for (; b0 < b_end; b0 += D) {
#pragma unroll
        for (int i = 0; i < D; ++i) {
            const int b = b0 + i;
            if (b < b_end) {
                const uint4 wq = ring[i];
                v4i p;
                if constexpr (DIRECT) {
                    const uint4 pq = aring[i];
                    p = v4i{(int)pq.x, (int)pq.y, (int)pq.z, (int)pq.w};
                } else {
                    p = *reinterpret_cast<const v4i*>(arow + b * kRowBytes);
                }
                if (b + D < b_end) {
                    ring[i] = load_weights_16B(&wp[(b + D) * (kBlockBytes / 16)]);
                    if constexpr (DIRECT) aring[i] = piece(b + D);
                }
                product(b < hi_blocks, wq, p);
            }
        }
    }
}

template <bool DBG, int ACT>
__global__ __launch_bounds__(kDecodeThreads) void gemm_decode_kernel(const DecodeArgs a) {
    extern __shared__ __attribute__((aligned(16))) uint8_t act[];  // kActQuantize: [M][lds_row]
    constexpr bool DIRECT = ACT == kActDirect;
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int hi_blocks = (int)a.L.hi_blocks, blocks = (int)(a.L.hi_blocks + a.L.lo_blocks);
    const int lane_off = (lane & 15) * kRowBytes + (lane >> 4) * 16;
    // lane l supplies token l % 16 (token 0 again past M: those output columns are never stored), piece l / 16 of each 64-byte chunk
    const int tok = lane & 15;
    const bool tok_live = tok < a.M;
    const ActPieces piece = act_pieces(a, lane, tok_live);

    // start the weight stream of this wave's first group before anything else
    int group = wave * gridDim.x + blockIdx.x;
    uint4 ring[kDecodeDepth], aring[DIRECT ? kDecodeDepth : 1];
    {
        const uint4* wp = reinterpret_cast<const uint4*>(
            a.packed + (int64_t)(group < a.groups ? group : 0) * a.L.group_bytes + lane_off);
#pragma unroll
        for (int i = 0; i < kDecodeDepth; ++i) {
            if (group < a.groups && i < blocks) {
                ring[i] = load_weights_16B(&wp[i * (kBlockBytes / 16)]);
                if constexpr (DIRECT) aring[i] = piece(i);
            }
        }
    }

    float* scal = reinterpret_cast<float*>(act + ((a.M * a.lds_row + 15) & ~15));
    if constexpr (ACT == kActQuantize) fill_act_quantize(a, act, scal, t);
    const DecodeArgs ea = epilogue_args<ACT == kActQuantize>(a, scal);

    const uint8_t* arow = act + (tok_live ? tok : 0) * a.lds_row + (lane >> 4) * 16;
    for (; group < a.groups; group += 8 * gridDim.x) {
        const uint4* wp = reinterpret_cast<const uint4*>(a.packed + (int64_t)group * a.L.group_bytes + lane_off);
        v4i acc_hi = {0, 0, 0, 0}, acc_lo = {0, 0, 0, 0};
        stream_run<DIRECT>(ring, aring, wp, piece, arow, 0, blocks, hi_blocks, acc_hi, acc_lo);
        // the next group's first loads go out before this group's epilogue
        const int next = group + 8 * gridDim.x;
        if (next < a.groups) {
            const uint4* np = reinterpret_cast<const uint4*>(a.packed + (int64_t)next * a.L.group_bytes + lane_off);
#pragma unroll
            for (int i = 0; i < kDecodeDepth; ++i)
                if (i < blocks) {
                    ring[i] = load_weights_16B(&np[i * (kBlockBytes / 16)]);
                    if constexpr (DIRECT) aring[i] = piece(i);
                }
        }

        // lane l now holds token l % 16, channels 16 group + 4 (l / 16) + {0..3}
        if (!tok_live) continue;
        stream_epilogue<DBG>(ea, tok, (int64_t)group * 16 + (lane >> 4) * 4, acc_hi, acc_lo);
    }
}

// ---------------------------------------------------------------------------
// The same for layers with few output channels (o_proj, down_proj: N / 16 groups
// are fewer than the wavefronts the chip needs in flight to keep HBM busy): the
// reduction axis of a group is cut into SK contiguous runs of blocks, one per
// wavefront of a workgroup, whose integer sums meet in LDS; the wavefront of the
// first run adds them and runs the epilogue.  A workgroup owns 8 / SK groups at
// a time ("a set"); sets are dealt round-robin over workgroups.  Exact: integer
// addition in any order.
// ---------------------------------------------------------------------------
template <bool DBG, int SK, int ACT>
__global__ __launch_bounds__(kDecodeThreads) void gemm_decode_splitk_kernel(const DecodeArgs a) {
    static_assert(SK == 2 || SK == 4 || SK == 8, "runs per group");
    constexpr int kWaves = kDecodeThreads / 64;
    constexpr int G = kWaves / SK;  // groups per set
    extern __shared__ __attribute__((aligned(16))) uint8_t act[];  // kActQuantize: [M][lds_row]; then the partial sums
    constexpr bool DIRECT = ACT == kActDirect;
    const int t = threadIdx.x, lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int gsel = wave / SK, part = wave % SK;
    const int hi_blocks = (int)a.L.hi_blocks, blocks = (int)(a.L.hi_blocks + a.L.lo_blocks);
    const int b_begin = (int)((int64_t)blocks * part / SK), b_end = (int)((int64_t)blocks * (part + 1) / SK);
    const int lane_off = (lane & 15) * kRowBytes + (lane >> 4) * 16;
    v4i* partial = reinterpret_cast<v4i*>(act + (DIRECT ? 0 : ((a.M * a.lds_row + 15) & ~15)));  // [kWaves][2][64]
    const int sets = (a.groups + G - 1) / G;
    const int tok = lane & 15;
    const bool tok_live = tok < a.M;
    const ActPieces piece = act_pieces(a, lane, tok_live);

    // start the weight stream of this wave's first run before anything else
    int set = blockIdx.x;
    uint4 ring[kDecodeDepth], aring[DIRECT ? kDecodeDepth : 1];
    {
        const int group = set * G + gsel;
        const bool live = set < sets && group < a.groups;
        const uint4* wp = reinterpret_cast<const uint4*>(
            a.packed + (int64_t)(live ? group : 0) * a.L.group_bytes + lane_off);
#pragma unroll
        for (int i = 0; i < kDecodeDepth; ++i) {
            if (live && b_begin + i < b_end) {
                ring[i] = load_weights_16B(&wp[(b_begin + i) * (kBlockBytes / 16)]);
                if constexpr (DIRECT) aring[i] = piece(b_begin + i);
            }
        }
    }

    float* scal = reinterpret_cast<float*>(partial + kWaves * 2 * 64);
    if constexpr (ACT == kActQuantize) fill_act_quantize(a, act, scal, t);
    const DecodeArgs ea = epilogue_args<ACT == kActQuantize>(a, scal);

    const uint8_t* arow = act + (tok_live ? tok : 0) * a.lds_row + (lane >> 4) * 16;
    for (; set < sets; set += gridDim.x) {  // the same trip count for every wavefront of a workgroup
        const int group = set * G + gsel;
        const bool live = group < a.groups;
        const uint4* wp = reinterpret_cast<const uint4*>(
            a.packed + (int64_t)(live ? group : 0) * a.L.group_bytes + lane_off);
        v4i acc_hi = {0, 0, 0, 0}, acc_lo = {0, 0, 0, 0};
        // the wavefront that will run the epilogue asks for its constants behind the first weight loads
        const int64_t n0 = (int64_t)(live ? group : 0) * 16 + (lane >> 4) * 4;
        EpilogueConsts ec;
        if (part == 0) ec = load_epilogue_consts(ea, tok_live ? tok : 0, n0);
        if (live) stream_run<DIRECT>(ring, aring, wp, piece, arow, b_begin, b_end, hi_blocks, acc_hi, acc_lo);
        // the next set's first loads go out before the sums are exchanged
        {
            const int nset = set + gridDim.x;
            const int ngroup = nset * G + gsel;
            if (nset < sets && ngroup < a.groups) {
                const uint4* np = reinterpret_cast<const uint4*>(a.packed + (int64_t)ngroup * a.L.group_bytes + lane_off);
#pragma unroll
                for (int i = 0; i < kDecodeDepth; ++i)
                    if (b_begin + i < b_end) {
                        ring[i] = load_weights_16B(&np[(b_begin + i) * (kBlockBytes / 16)]);
                        if constexpr (DIRECT) aring[i] = piece(b_begin + i);
                    }
            }
        }
        if (part != 0) {
            partial[(wave * 2 + 0) * 64 + lane] = acc_hi;
            partial[(wave * 2 + 1) * 64 + lane] = acc_lo;
        }
        __syncthreads();
        if (part == 0 && live) {
#pragma unroll
            for (int k = 1; k < SK; ++k) {
                acc_hi += partial[((wave + k) * 2 + 0) * 64 + lane];
                acc_lo += partial[((wave + k) * 2 + 1) * 64 + lane];
            }
            // lane l now holds token l % 16, channels 16 group + 4 (l / 16) + {0..3}
            if (tok_live) stream_epilogue<DBG>(ea, tok, n0, ec, acc_hi, acc_lo);
        }
        __syncthreads();  // the partial sums are read before the next set overwrites them
    }
}

// ---------------------------------------------------------------------------
// The same for 17 .. 64 tokens (batched generation), and for up to 16 tokens of
// a reduction axis too long for LDS: still one pass over the packed weights,
// each 1 KiB block going from HBM into operand registers once and meeting every
// group of 16 tokens there (TG = 1, 2 or 4 groups, one accumulator pair each;
// eight groups do not fit the registers next to the weight ring, and a spill in
// the loop would wait for the whole ring on the shared load counter).  The
// activation codes do not fit LDS whole, so the wavefronts walk the reduction
// axis in chunks of kChunkBlocks blocks; a chunk of all tokens' codes sits in
// LDS as the 16-row x 64-byte blocks of the tiled kernel (piece kc of row r at
// unit 4 r + (kc ^ (r >> 2)), so the 16 lanes that read one piece of 16 rows
// hit 16 bank groups), fetched by direct-to-LDS loads one chunk ahead: one
// barrier per chunk.  As in the kernel above the reduction axis of a group can
// be cut into SK runs, one per wavefront (SK * TG <= 8: LDS holds the chunks of
// all runs); a workgroup owns 8 / SK groups at a time.
// ---------------------------------------------------------------------------
constexpr int kChunkBlocks = 8;
static_assert(kChunkBlocks == kDecodeDepth, "a chunk fills the weight ring exactly once");
constexpr int kStreamMaxM = 64;

// NT: the weights are read with the non-temporal hint (one token slice on a layer too large
// for the caches: nobody reads them again)
template <bool DBG, int TG, int SK, bool NT = false>
__global__ __launch_bounds__(kDecodeThreads) void gemm_stream_kernel(const DecodeArgs a_in) {
    static_assert(TG * 16 <= kStreamMaxM && SK * TG <= 8, "LDS holds two chunks of every run");
    // blockIdx.y selects a slice of TG * 16 tokens (more tokens than that: every slice
    // streams the weights for itself, out of the last-level cache after the first)
    DecodeArgs a = a_in;
    {
        const int tok0 = (int)blockIdx.y * (TG * 16);
        a.M = a_in.M - tok0 < TG * 16 ? a_in.M - tok0 : TG * 16;
        if (a.q_hi) a.q_hi += (int64_t)tok0 * a.ld_hi;
        if (a.q_lo) a.q_lo += (int64_t)tok0 * a.ld_lo;
        if (a.s_hi) a.s_hi += tok0;
        if (a.s_lo) a.s_lo += tok0;
        if (a.lo_sum) a.lo_sum += tok0;
        if (a.c_hi) a.c_hi += tok0;
        if (a.c_lo) a.c_lo += tok0;
        a.y += (int64_t)tok0 * a.ldy;
        if (a.dbg_hi) a.dbg_hi += (int64_t)tok0 * a.L.N;
        if (a.dbg_lo) a.dbg_lo += (int64_t)tok0 * a.L.N;
    }
    extern __shared__ __attribute__((aligned(1024))) uint8_t act[];  // [2][SK][kChunkBlocks][TG] blocks
    constexpr int kWaves = kDecodeThreads / 64;
    constexpr int G = kWaves / SK;  // groups per set
    constexpr int kRunBytes = kChunkBlocks * TG * kBlockBytes;  // one run's chunk
    constexpr int kBufBytes = SK * kRunBytes;
    constexpr int kFetches = SK * TG;  // direct-to-LDS loads per wavefront and chunk
    const int t = threadIdx.x, lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int gsel = wave / SK, part = wave % SK;
    const int hi_blocks = (int)a.L.hi_blocks, blocks = (int)(a.L.hi_blocks + a.L.lo_blocks);
    // run `part` covers blocks [run_begin(part), run_begin(part + 1)); every run walks the
    // same number of chunks (the longest run's)
    auto run_begin = [&](int p) { return (int)((int64_t)blocks * p / SK); };
    const int b_begin = run_begin(part), b_end = run_begin(part + 1);
    const int chunks = ((blocks + SK - 1) / SK + kChunkBlocks - 1) / kChunkBlocks;
    const int lane_off = (lane & 15) * kRowBytes + (lane >> 4) * 16;
    // operand read: lane l supplies token l % 16, piece l / 16 of a block
    const int rr = lane & 15, rk = lane >> 4;
    const int read_off = part * kRunBytes + (4 * rr + (rk ^ (rr >> 2))) * 16;
    // the partial sums of the runs meet in the chunk buffers once the last chunk is done with
    v4i* partial = reinterpret_cast<v4i*>(act);  // [kWaves][TG][2][64]
    static_assert(kWaves * TG * 2 * 64 * 16 <= 2 * kBufBytes, "partial sums fit the chunk buffers");

    // Chunk loader: fetch f = q * kWaves + wave of a chunk step is block i of run p for
    // token group g, f = (p * kChunkBlocks + i) * TG + g.  Lane l brings row l / 4, piece
    // (l % 4) ^ (l / 16) of that block, which lands at unit l: the layout read above.
    const int f_r = lane >> 2, f_kc = (lane & 3) ^ (lane >> 4);
    // (Buffer loads, not global ones: a global load to LDS counts for the compiler as an access
    // through a flat address, after which it waits for every load in flight before any
    // use of a loaded register.)
    const __amdgpu_buffer_rsrc_t rs_hi = make_rsrc(a.q_hi), rs_lo = make_rsrc(a.q_lo);
    auto fetch_one = [&](int q, int c, int buf, bool all) __attribute__((always_inline)) {
        const int f = q * kWaves + wave;
        const int g = f % TG, i = (f / TG) % kChunkBlocks, p = f / (TG * kChunkBlocks);
        int b = run_begin(p) + c * kChunkBlocks + i;
        if (!all && b >= run_begin(p + 1)) return;
        b = b < blocks ? b : blocks - 1;  // a block past the end of its run: valid memory, never read from LDS
        int m = g * 16 + f_r;
        m = m < a.M ? m : a.M - 1;  // rows past M repeat the last token (never stored)
        const bool hi = b < hi_blocks;
        const uint32_t voff = hi ? (uint32_t)(m * (int)a.ld_hi + b * kRowBytes + f_kc * 16)
                                 : (uint32_t)(m * (int)a.ld_lo + (b - hi_blocks) * kRowBytes + f_kc * 16);
        buffer_load_to_lds_16B(hi ? rs_hi : rs_lo, voff, 0, act + buf * kBufBytes + f * kBlockBytes);
    };
    auto fetch_chunk = [&](int c, int buf) {
#pragma unroll
        for (int q = 0; q < kFetches; ++q) fetch_one(q, c, buf, false);
        asm volatile("" ::: "memory");  // later loads stay behind these
    };
    // the same without conditions, for chunk steps that are straight-line code
    auto fetch_chunk_all = [&](int c, int buf) __attribute__((always_inline)) {
#pragma unroll
        for (int q = 0; q < kFetches; ++q) fetch_one(q, c, buf, true);
        asm volatile("" ::: "memory");
    };
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t*)act;

    auto load_w = [](const uint4* ptr) __attribute__((always_inline)) {
        if constexpr (NT) return load_weights_16B(ptr);
        else return *ptr;
    };
    const int sets = (a.groups + G - 1) / G;
    for (int set = blockIdx.x; set < sets; set += gridDim.x) {
        const int group = set * G + gsel;
        const bool live = group < a.groups;
        const uint4* wp = reinterpret_cast<const uint4*>(
            a.packed + (int64_t)(live ? group : 0) * a.L.group_bytes + lane_off);
        uint4 ring[kDecodeDepth];
#pragma unroll
        for (int i = 0; i < kDecodeDepth; ++i)
            if (live && b_begin + i < b_end) ring[i] = load_w(&wp[(b_begin + i) * (kBlockBytes / 16)]);
        __syncthreads();  // every wavefront is done with the LDS buffers of the previous set
        fetch_chunk(0, 0);
        wait_loads_and_barrier<0>();

        v4i acc_hi[TG], acc_lo[TG];
#pragma unroll
        for (int g = 0; g < TG; ++g) {
            acc_hi[g] = (v4i){0, 0, 0, 0};
            acc_lo[g] = (v4i){0, 0, 0, 0};
        }
        // Chunk steps of a run that has all eight blocks of this chunk and of the next, all of
        // one kind: straight-line code in loops of their own (see stream_run for why), the
        // activation fragments read by instructions the compiler does not track, so that it
        // does not make every LDS read wait for the chunk loads in flight.
        constexpr int PGs = TG < 4 ? TG : 4;            // groups per pass
        constexpr int PASSESs = TG / PGs;               // passes per block
        auto wait_frags = [&](v4i (&f)[PGs]) __attribute__((always_inline)) {
            if constexpr (PGs == 1) asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(f[0]));
            else if constexpr (PGs == 2) asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(f[0]), "+v"(f[1]));
            else asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(f[0]), "+v"(f[1]), "+v"(f[2]), "+v"(f[3]));
        };
        auto steady_step = [&](auto kind, int c) __attribute__((always_inline)) {
            constexpr int KIND = decltype(kind)::value;  // 0: high blocks, 1: low blocks, 2: both
            fetch_chunk_all(c + 1, (c + 1) & 1);
            const uint32_t cur = lds0 + (c & 1) * kBufBytes + read_off;
            const int first = b_begin + c * kChunkBlocks;
            v4i p[PGs], pn[PGs];
            static_for<PGs>([&](auto g_) __attribute__((always_inline)) {
                constexpr int g = decltype(g_)::value;
                lds_read16<g * kBlockBytes>(p[g], cur);
            });
            wait_frags(p);
            static_for<kChunkBlocks>([&](auto i_) __attribute__((always_inline)) {
                constexpr int i = decltype(i_)::value;
                static_for<PASSESs>([&](auto h_) __attribute__((always_inline)) {
                    constexpr int h = decltype(h_)::value;
                    constexpr int kLast = kChunkBlocks * PASSESs - 1, step = i * PASSESs + h;
                    if constexpr (step < kLast) {
                        constexpr int ni = (step + 1) / PASSESs, nh = (step + 1) % PASSESs;
                        static_for<PGs>([&](auto g_) __attribute__((always_inline)) {
                            constexpr int g = decltype(g_)::value;
                            lds_read16<(ni * TG + nh * PGs + g) * kBlockBytes>(pn[g], cur);
                        });
                    }
                    const v4i w = {(int)ring[i].x, (int)ring[i].y, (int)ring[i].z, (int)ring[i].w};
                    if (KIND == 0 || (KIND == 2 && first + i < hi_blocks)) {
#pragma unroll
                        for (int g = 0; g < PGs; ++g)
                            acc_hi[h * PGs + g] = __builtin_amdgcn_mfma_i32_16x16x64_i8(w, p[g], acc_hi[h * PGs + g], 0, 0, 0);
                    } else {
                        // see resq_gemm.hip.h: one operand of each product carries an offset of 8
                        const v4i we = w & (int)0xF0F0F0F0, wo = w & (int)0x0F0F0F0F;
#pragma unroll
                        for (int g = 0; g < PGs; ++g) {
                            acc_lo[h * PGs + g] = __builtin_amdgcn_mfma_i32_16x16x64_i8(
                                we, p[g] & (int)0x0F0F0F0F, acc_lo[h * PGs + g], 0, 0, 0);
                            acc_lo[h * PGs + g] = __builtin_amdgcn_mfma_i32_16x16x64_i8(
                                wo, p[g] & (int)0xF0F0F0F0, acc_lo[h * PGs + g], 0, 0, 0);
                        }
                    }
                    __builtin_amdgcn_sched_barrier(0);
                    if constexpr (step < kLast) {
                        wait_frags(pn);
#pragma unroll
                        for (int g = 0; g < PGs; ++g) p[g] = pn[g];
                    }
                });
                // the slot is refilled once its last product has been issued
                ring[i] = load_w(&wp[(first + i + kDecodeDepth) * (kBlockBytes / 16)]);
                __builtin_amdgcn_sched_barrier(0);
            });
            // the next chunk's codes have landed; the eight weight loads behind them stay in flight
            wait_loads_and_barrier<kDecodeDepth>();
        };
        __builtin_amdgcn_s_waitcnt(0x0F70);  // nothing in flight here (the wait above): tells the compiler so
        int c = 0;
        auto steady = [&](int cc) { return live && b_begin + (cc + 2) * kChunkBlocks <= b_end; };
        while (steady(c) && b_begin + (c + 1) * kChunkBlocks <= hi_blocks) {
            steady_step(std::integral_constant<int, 0>{}, c);
            ++c;
        }
        if (steady(c) && b_begin + c * kChunkBlocks < hi_blocks) {
            steady_step(std::integral_constant<int, 2>{}, c);
            ++c;
        }
        while (steady(c) && b_begin + c * kChunkBlocks >= hi_blocks) {
            steady_step(std::integral_constant<int, 1>{}, c);
            ++c;
        }
        for (; c < chunks; ++c) {
            // the other buffer was last read in chunk c - 1, before the barrier that ended it
            if (c + 1 < chunks) fetch_chunk(c + 1, (c + 1) & 1);
            const uint8_t* cur = act + (c & 1) * kBufBytes + read_off;
            const int first = b_begin + c * kChunkBlocks, last = first + kChunkBlocks;
            // A block meets the token groups PG at a time; the fragments of the next PG
            // groups are read while these are multiplied.  KIND 0: a full chunk of high
            // blocks; 1: a full chunk of low blocks; 2: anything else (the chunk that holds
            // the boundary between the groups, a partial last chunk).
            constexpr int PG = TG < 4 ? TG : 4;         // groups per pass
            constexpr int PASSES = TG / PG;             // passes per block
            auto chunk_body = [&](auto kind) __attribute__((always_inline)) {
                constexpr int KIND = decltype(kind)::value;
                v4i p[PG], pn[PG];
#pragma unroll
                for (int g = 0; g < PG; ++g) p[g] = *reinterpret_cast<const v4i*>(cur + g * kBlockBytes);
#pragma unroll
                for (int i = 0; i < kChunkBlocks; ++i) {
                    const int b = first + i;  // kChunkBlocks == kDecodeDepth: ring slot i
                    const uint4 wq = ring[i];
                    if (b + kDecodeDepth < b_end) ring[i] = load_w(&wp[(b + kDecodeDepth) * (kBlockBytes / 16)]);
                    const v4i w = {(int)wq.x, (int)wq.y, (int)wq.z, (int)wq.w};
                    const bool hi_block = KIND == 0 || (KIND == 2 && b < hi_blocks && b < b_end);
                    const bool lo_block = KIND == 1 || (KIND == 2 && b >= hi_blocks && b < b_end);
#pragma unroll
                    for (int h = 0; h < PASSES; ++h) {
                        constexpr int kLast = kChunkBlocks * PASSES - 1;
                        const int step = i * PASSES + h;
                        if (step < kLast) {
                            const int ni = (step + 1) / PASSES, nh = (step + 1) % PASSES;
#pragma unroll
                            for (int g = 0; g < PG; ++g)
                                pn[g] = *reinterpret_cast<const v4i*>(cur + (ni * TG + nh * PG + g) * kBlockBytes);
                        }
                        if (hi_block) {
#pragma unroll
                            for (int g = 0; g < PG; ++g)
                                acc_hi[h * PG + g] = __builtin_amdgcn_mfma_i32_16x16x64_i8(w, p[g], acc_hi[h * PG + g], 0, 0, 0);
                        }
                        if (lo_block) {
                            // see resq_gemm.hip.h: one operand of each product carries an offset of 8
                            const v4i we = w & (int)0xF0F0F0F0, wo = w & (int)0x0F0F0F0F;
#pragma unroll
                            for (int g = 0; g < PG; ++g) {
                                acc_lo[h * PG + g] = __builtin_amdgcn_mfma_i32_16x16x64_i8(
                                    we, p[g] & (int)0x0F0F0F0F, acc_lo[h * PG + g], 0, 0, 0);
                                acc_lo[h * PG + g] = __builtin_amdgcn_mfma_i32_16x16x64_i8(
                                    wo, p[g] & (int)0xF0F0F0F0, acc_lo[h * PG + g], 0, 0, 0);
                            }
                        }
                        __builtin_amdgcn_sched_barrier(0);
                        if (step < kLast) {
#pragma unroll
                            for (int g = 0; g < PG; ++g) p[g] = pn[g];
                        }
                    }
                }
            };
            if (live && first < b_end) {
                if (last <= hi_blocks && last <= b_end) chunk_body(std::integral_constant<int, 0>{});
                else if (first >= hi_blocks && last <= b_end) chunk_body(std::integral_constant<int, 1>{});
                else chunk_body(std::integral_constant<int, 2>{});
            }
            // The next chunk's codes must have landed; the weight loads issued after them
            // (eight, when the run goes on for two more chunks) may stay in flight.
            if (live && last + kDecodeDepth <= b_end) wait_loads_and_barrier<kDecodeDepth>();
            else wait_loads_and_barrier<0>();
        }
        if constexpr (SK > 1) {
            if (part != 0) {
#pragma unroll
                for (int g = 0; g < TG; ++g) {
                    partial[((wave * TG + g) * 2 + 0) * 64 + lane] = acc_hi[g];
                    partial[((wave * TG + g) * 2 + 1) * 64 + lane] = acc_lo[g];
                }
            }
            __syncthreads();
            if (part == 0) {
#pragma unroll
                for (int k = 1; k < SK; ++k) {
#pragma unroll
                    for (int g = 0; g < TG; ++g) {
                        acc_hi[g] += partial[(((wave + k) * TG + g) * 2 + 0) * 64 + lane];
                        acc_lo[g] += partial[(((wave + k) * TG + g) * 2 + 1) * 64 + lane];
                    }
                }
            }
        }
        if (!live || part != 0) continue;  // the barriers of the next set are reached all the same
#pragma unroll
        for (int g = 0; g < TG; ++g) {
            const int tok = g * 16 + (lane & 15);
            if (tok < a.M)
                stream_epilogue<DBG>(a, tok, (int64_t)group * 16 + (lane >> 4) * 4, acc_hi[g], acc_lo[g]);
            __builtin_amdgcn_sched_barrier(0);  // one token group at a time: keeps the registers few
        }
    }
}

}  // namespace resq
