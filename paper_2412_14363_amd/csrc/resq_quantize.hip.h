// Quantizer kernels: per-token activation quantization (Section 4.1 Eq. 2) and
// offline per-output-channel weight quantization + packing (Eq. 3), both with
// the symmetric quantizer of Section 3 Eq. 1.
//
// Arithmetic contract (what makes the integer codes reproducible bit for bit):
//   amax  = max |x| over the group                (exact: bf16 -> fp32 is exact)
//   scale = amax / qmax                           (fp32 IEEE division; 1 if amax == 0)
//   code  = clip(rint(x / scale), -qmax, qmax)    (fp32 IEEE division, ties to even)
// The per-token kernels multiply by the reciprocal of the scale and redo with the
// division every element whose quotient comes close to a half-integer or is not
// finite (see quant8), which yields exactly these codes.  Do not build this file
// with fast-math.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "resq_hadamard.hip.h"
#include "resq_layout.h"

namespace resq {

constexpr int kQuantThreads = 256;

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t b) { return __uint_as_float(b << 16); }

__device__ __forceinline__ int quant_code(float x, float scale, int qmax) {
    float q = rintf(x / scale);
    q = fminf(fmaxf(q, -(float)qmax), (float)qmax);
    return (int)q;
}

// Butterfly reductions over the 64 lanes of a wavefront; the lane exchanges are
// the cheap ones of the transform kernel (DPP moves, swizzles) where they exist.
// G = 16, 32 or 64: the reduction runs inside aligned groups of G lanes.
template <int G = 64>
__device__ __forceinline__ float wave_max(float a) {
    a = fmaxf(a, lane_xor<1>(a));
    a = fmaxf(a, lane_xor<2>(a));
    a = fmaxf(a, lane_xor<4>(a));
    a = fmaxf(a, lane_xor<8>(a));
    if constexpr (G > 16) a = fmaxf(a, lane_xor<16>(a));
    if constexpr (G > 32) a = fmaxf(a, lane_xor<32>(a));
    return a;
}
template <int G = 64>
__device__ __forceinline__ int wave_sum(int v) {
    v += __float_as_int(lane_xor<1>(__int_as_float(v)));
    v += __float_as_int(lane_xor<2>(__int_as_float(v)));
    v += __float_as_int(lane_xor<4>(__int_as_float(v)));
    v += __float_as_int(lane_xor<8>(__int_as_float(v)));
    if constexpr (G > 16) v += __float_as_int(lane_xor<16>(__int_as_float(v)));
    if constexpr (G > 32) v += __float_as_int(lane_xor<32>(__int_as_float(v)));
    return v;
}

// max over the 256 threads of a block of two non-negative floats at once
__device__ __forceinline__ void block_max2(float& a, float& b, float* red /* [8] in LDS */) {
    a = wave_max(a);
    b = wave_max(b);
    const int wave = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) {
        red[wave] = a;
        red[4 + wave] = b;
    }
    __syncthreads();
    a = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    b = fmaxf(fmaxf(red[4], red[5]), fmaxf(red[6], red[7]));
}

// max over the 256 threads of a block of four floats at once
__device__ __forceinline__ void block_max4(float (&a)[4], float* red /* [16] in LDS */) {
#pragma unroll
    for (int i = 0; i < 4; ++i) a[i] = wave_max(a[i]);
    const int wave = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0)
#pragma unroll
        for (int i = 0; i < 4; ++i) red[4 * i + wave] = a[i];
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 4; ++i)
        a[i] = fmaxf(fmaxf(red[4 * i], red[4 * i + 1]), fmaxf(red[4 * i + 2], red[4 * i + 3]));
}

// Asymmetric branch of Section 3 Eq. 1: z = min, s = (max - min) / (2^N - 1),
// code = clip(rint((x - z) / s), 0, 2^N - 1), difference and quotient in fp32.
// A constant group has s = 1.
__device__ __forceinline__ float asym_scale(float mn, float mx, int levels) {
    const float range = mx - mn;
    return range == 0.0f ? 1.0f : range / (float)levels;
}
__device__ __forceinline__ int quant_code_asym(float x, float zero, float scale, int levels) {
    float q = rintf((x - zero) / scale);
    q = fminf(fmaxf(q, 0.0f), (float)levels);
    return (int)q;
}

// sum over the 256 threads of a block
__device__ __forceinline__ int block_sum(int v, int* red /* [4] in LDS */) {
    v = wave_sum(v);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    return red[0] + red[1] + red[2] + red[3];
}

__device__ __forceinline__ float group_scale(float amax, int qmax) {
    return amax == 0.0f ? 1.0f : amax / (float)qmax;
}

// largest |.| of the eight bf16 values in a 16-byte vector, as a float
typedef unsigned short v2us __attribute__((ext_vector_type(2)));
__device__ __forceinline__ float absmax8(const uint4& v) {
    // non-negative bf16 patterns order like unsigned integers: packed 16-bit max
    auto as2 = [](uint32_t w) { w &= 0x7FFF7FFFu; return *reinterpret_cast<v2us*>(&w); };
    const v2us m = __builtin_elementwise_max(__builtin_elementwise_max(as2(v.x), as2(v.y)),
                                             __builtin_elementwise_max(as2(v.z), as2(v.w)));
    return bf16_bits_to_f32(max((uint32_t)m[0], (uint32_t)m[1]));
}

// ---------------------------------------------------------------------------
// Activations, vectorized: one workgroup per token.  The row is read once (16
// bytes per lane, coalesced), kept in registers across the absmax reduction,
// then quantized and stored.  (One wavefront per token, without LDS or barrier,
// was measured slower at every size: fewer, fatter waves hide less latency.)
// Requires K, r, ldx multiples of 8 and x 16-byte aligned; ITERS * 2048 >= K.
//
// The division x / scale is what the quantizer is defined by, but a correctly
// rounded fp32 division costs about ten instructions per element, as much time
// as the memory traffic of this kernel.  So: t = x * (1 / scale) is within a
// few ulp of the correctly rounded quotient, and rint(t) equals rint(x / scale)
// whenever t is further than that from every half-integer.  Elements within
// qmax * 2^-20 of a half-integer (|t| <= qmax, so at least 8 ulp of t) are
// redone with the true division, in branches that are taken only by the
// wavefronts that hold such an element, for the element slots that hold one.
// The codes are therefore exactly those of the definition.  (bf16 inputs make
// exact ties common: about 2 in 10^4 elements of a 4096-wide row, 1 in 10^3 of
// a 128-wide one, so the branches are not rare, but cheap on average.)
// ---------------------------------------------------------------------------
// Eight elements at once.  On return the low bits of u[j] hold the two's
// complement code of element j (plus 8 for even j when LOW, the offset-binary
// storage of even columns) and odd_sum has gained the codes of the odd elements.
// Adding 1.5 * 2^23 to t rounds it to an integer, ties to even, in the low
// mantissa bits of the sum, so rounding, conversion and the offset cost one add.
template <bool LOW>
__device__ __forceinline__ void quant8(const uint4& v, float scale, float inv, uint32_t (&u)[8],
                                       float& odd_sum) {
    constexpr float kMagic = 12582912.0f;  // 1.5 * 2^23, bit pattern 0x4B400000
    constexpr int qmax = LOW ? kQmaxLo : kQmaxHi;
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
    float xs[8], rr[8];
    bool near_tie[8], any_tie = false;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        xs[j] = __uint_as_float((j & 1) ? (w[j >> 1] & 0xFFFF0000u) : (w[j >> 1] << 16));
        const float magic = kMagic + ((LOW && !(j & 1)) ? 8.0f : 0.0f);
        const float t = xs[j] * inv;
        const float uf = t + magic;
        rr[j] = uf - kMagic;                    // rint(t) (+ 8), exact
        // negated <= so that a quotient that is not finite (a row whose scale is so small that its
        // reciprocal overflows) is redone with the division as well
        near_tie[j] = !(fabsf(t - (uf - magic)) <= 0.5f - (LOW ? 8.0f : 128.0f) * 9.5367431640625e-07f);
        any_tie |= near_tie[j];
        u[j] = __float_as_uint(uf);
    }
    // Wave-uniform branches.  With short rows (one attention head) a wavefront holds a
    // near-tie more often than not, so the redo is per element slot: one division for
    // the slots in which some lane has one, not eight.
    if (__builtin_amdgcn_ballot_w64(any_tie) != 0) {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            if (__builtin_amdgcn_ballot_w64(near_tie[j]) != 0) {
                const int c = quant_code(xs[j], scale, qmax) + ((LOW && !(j & 1)) ? 8 : 0);
                u[j] = (uint32_t)c;
                rr[j] = (float)c;
            }
        }
    }
    if (LOW) odd_sum += (rr[1] + rr[3]) + (rr[5] + rr[7]);
}

// The same for the asymmetric quantizer.  Codes are STORED minus 2^(N-1) (int8 for
// the high group; for the low group a two's-complement nibble in odd columns and
// the plain code 0..15, i.e. stored value + 8, in even columns), so that the GEMM
// sees the operands it sees for symmetric codes.  On return the low bits of u[j]
// hold that stored value and odd_sum has gained the stored values of the odd elements.
template <bool LOW>
__device__ __forceinline__ void quant8_asym(const uint4& v, float zero, float scale, float inv,
                                            uint32_t (&u)[8], float& odd_sum) {
    constexpr float kMagic = 12582912.0f;  // 1.5 * 2^23
    constexpr int levels = LOW ? 15 : 255;
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
    float ds[8], rr[8];
    bool near_tie[8], any_tie = false;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const float x = __uint_as_float((j & 1) ? (w[j >> 1] & 0xFFFF0000u) : (w[j >> 1] << 16));
        const float off = LOW ? ((j & 1) ? 8.0f : 0.0f) : 128.0f;  // stored = code - off
        ds[j] = x - zero;
        const float t = ds[j] * inv;
        const float uf = t + (kMagic - off);
        rr[j] = uf - kMagic;                    // rint(t) - off, exact
        near_tie[j] = !(fabsf(t - (uf - (kMagic - off))) <= 0.5f - (LOW ? 16.0f : 256.0f) * 9.5367431640625e-07f);
        any_tie |= near_tie[j];
        u[j] = __float_as_uint(uf);
    }
    if (__builtin_amdgcn_ballot_w64(any_tie) != 0) {  // wave-uniform, then per element slot
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            if (__builtin_amdgcn_ballot_w64(near_tie[j]) != 0) {
                float q = rintf(ds[j] / scale);
                q = fminf(fmaxf(q, 0.0f), (float)levels);
                const int c = (int)q - (LOW ? ((j & 1) ? 8 : 0) : 128);
                u[j] = (uint32_t)c;
                rr[j] = (float)c;
            }
        }
    }
    if (LOW) odd_sum += (rr[1] + rr[3]) + (rr[5] + rr[7]);
}

// low bytes of four registers -> one dword
__device__ __forceinline__ uint32_t pack_low_bytes(uint32_t a, uint32_t b, uint32_t c, uint32_t d) {
    return __builtin_amdgcn_perm(b, a, 0x0c0c0400u) | __builtin_amdgcn_perm(d, c, 0x04000c0cu);
}

// Optional block Walsh-Hadamard transform of the low group in front of the
// quantizer (the online projection of the down_proj input, Section 4.3): the
// rotated row never goes to memory unless the caller asks for it.
struct RotateArgs {
    int log2b;          // 0: no transform; else log2 of the block size, 3..9
    float scale;        // 1 / sqrt(block)
    uint16_t* x_rot;    // null, or bf16 [M, ld_rot]: receives columns [r, K) of the rotated row
    int64_t ld_rot;
};

// ASYM: the asymmetric quantizer; c_hi / c_lo [M] receive z + 2^(N-1) s, the real
// value that the stored code 0 stands for (what the GEMM's epilogue needs).
template <int ITERS, bool ROTATE, bool ASYM>
__global__ __launch_bounds__(kQuantThreads) void quantize_act_vec_kernel(
    const uint16_t* __restrict__ x, int64_t ldx, int K, int r, int8_t* __restrict__ q_hi,
    int64_t ld_hi, uint8_t* __restrict__ q_lo, int64_t ld_lo, float* __restrict__ s_hi,
    float* __restrict__ s_lo, int32_t* __restrict__ lo_sum, const RotateArgs rot,
    float* __restrict__ c_hi, float* __restrict__ c_lo) {
    constexpr int RT = kQuantThreads;     // threads per row
    __shared__ float red[16];
    __shared__ int red_sum[4];
    const int t = threadIdx.x;
    const int64_t m = blockIdx.x;
    const int nunits = K >> 3;
    const int hi_units = r >> 3;
    const uint4* row = reinterpret_cast<const uint4*>(x + m * ldx);

    uint4 v[ITERS];
#pragma unroll
    for (int i = 0; i < ITERS; ++i) {
        const int u = t + i * RT;
        v[i] = u < nunits ? row[u] : make_uint4(0u, 0u, 0u, 0u);
    }
    if constexpr (ROTATE) {
        // The same butterflies, in the same order, as the stand-alone transform
        // kernel, followed by its rounding to bf16: the codes are those of
        // quantizing that kernel's output.  A block is block/8 consecutive lanes
        // (r and K - r are multiples of the block), so a wavefront may hold lanes
        // of the high group too: they take part in the exchanges and keep their
        // own values.
        const int lane = t & 63;
#pragma unroll
        for (int i = 0; i < ITERS; ++i) {
            const int u = t + i * RT;
            float f[8];
            unpack8_bf16(v[i], f);
            wht_in_lane(f, rot.log2b);
            wht_across_lanes(f, rot.log2b, lane);
            if (u >= hi_units && u < nunits) {
                v[i] = pack8_bf16(f, rot.scale);
                if (rot.x_rot) *reinterpret_cast<uint4*>(rot.x_rot + m * rot.ld_rot + (int64_t)u * 8) = v[i];
            }
        }
    }
    float sh, sl, zh = 0.0f, zl = 0.0f;
    if constexpr (ASYM) {
        // max and -min of both groups in one reduction
        const float inf = __builtin_huge_valf();
        float ext[4] = {-inf, -inf, -inf, -inf};  // max_h, -min_h, max_l, -min_l
#pragma unroll
        for (int i = 0; i < ITERS; ++i) {
            const int u = t + i * RT;
            if (u < nunits) {
                float f[8];
                unpack8_bf16(v[i], f);
                const float mx = fmaxf(fmaxf(fmaxf(f[0], f[1]), fmaxf(f[2], f[3])),
                                       fmaxf(fmaxf(f[4], f[5]), fmaxf(f[6], f[7])));
                const float mn = fminf(fminf(fminf(f[0], f[1]), fminf(f[2], f[3])),
                                       fminf(fminf(f[4], f[5]), fminf(f[6], f[7])));
                const int g = u < hi_units ? 0 : 2;
                ext[g] = fmaxf(ext[g], mx);
                ext[g + 1] = fmaxf(ext[g + 1], -mn);
            }
        }
        block_max4(ext, red);
        zh = -ext[1];
        zl = -ext[3];
        sh = r > 0 ? asym_scale(zh, ext[0], 255) : 1.0f;
        sl = K - r > 0 ? asym_scale(zl, ext[2], 15) : 1.0f;
        if (t == 0) {
            if (r > 0) c_hi[m] = zh + 128.0f * sh;
            if (K - r > 0) c_lo[m] = zl + 8.0f * sl;
        }
    } else {
        float amax_h = 0.0f, amax_l = 0.0f;
#pragma unroll
        for (int i = 0; i < ITERS; ++i) {
            const int u = t + i * RT;
            if (u < nunits) {
                const float a = absmax8(v[i]);
                if (u < hi_units) amax_h = fmaxf(amax_h, a);
                else amax_l = fmaxf(amax_l, a);
            }
        }
        block_max2(amax_h, amax_l, red);
        sh = group_scale(amax_h, kQmaxHi);
        sl = group_scale(amax_l, kQmaxLo);
    }
    const float inv_h = 1.0f / sh, inv_l = 1.0f / sl;
    if (t == 0) {
        if (r > 0) s_hi[m] = sh;
        if (K - r > 0) s_lo[m] = sl;
    }

    int8_t* qh = q_hi + m * ld_hi;
    uint8_t* ql = q_lo + m * ld_lo;
    float odd_f = 0.0f;  // low codes of odd columns (small integers, exact in fp32)
#pragma unroll
    for (int i = 0; i < ITERS; ++i) {
        const int u = t + i * RT;
        if (u < nunits) {
            uint32_t c[8];
            if (u < hi_units) {
                if constexpr (ASYM) quant8_asym<false>(v[i], zh, sh, inv_h, c, odd_f);
                else quant8<false>(v[i], sh, inv_h, c, odd_f);
                *reinterpret_cast<uint2*>(qh + (int64_t)u * 8) =
                    make_uint2(pack_low_bytes(c[0], c[1], c[2], c[3]), pack_low_bytes(c[4], c[5], c[6], c[7]));
            } else {
                if constexpr (ASYM) quant8_asym<true>(v[i], zl, sl, inv_l, c, odd_f);
                else quant8<true>(v[i], sl, inv_l, c, odd_f);
                // byte k = (even code + 8) | (odd code << 4); the even value is 1..15 in
                // its low byte already, and only the low byte of by[k] is kept
                uint32_t by[4];
#pragma unroll
                for (int k = 0; k < 4; ++k) by[k] = (c[2 * k + 1] << 4) | c[2 * k];
                *reinterpret_cast<uint32_t*>(ql + (int64_t)(u - hi_units) * 4) =
                    pack_low_bytes(by[0], by[1], by[2], by[3]);
            }
        }
    }
    int odd_sum = (int)odd_f;
    // zero codes in the padding of both rows
    for (int64_t b = (int64_t)r + 8 * t; b < ld_hi; b += 8 * RT)
        *reinterpret_cast<uint2*>(qh + b) = make_uint2(0u, 0u);
    for (int64_t b = (int64_t)(K - r) / 2 + 4 * t; b < ld_lo; b += 4 * RT)
        *reinterpret_cast<uint32_t*>(ql + b) = 0x08080808u;
    odd_sum = block_sum(odd_sum, red_sum);
    if (t == 0 && K - r > 0) lo_sum[m] = odd_sum;
}

// ---------------------------------------------------------------------------
// The fused transform + quantizer for blocks of 256 (the down_proj input of the
// Llama models: 12544 = 49 * 256 low columns), with the first five butterfly
// stages on the bf16 matrix cores.  The vector-ALU butterflies of the kernel
// above cost about 30 instructions per element, which makes that kernel
// ALU-bound at twice the time its memory traffic takes.
//
// H_256 = H_8 (x) H_32: column e = 32 a + c of a block, a = 0..7, c = 0..31.  A
// wavefront takes a span of 512 low columns (two blocks, 16 rows rho = 8 g + a of
// 32 columns).  Lane l loads the 8 consecutive columns c = 8 q .. 8 q + 7 of row
// rho = l % 16, q = l / 16: exactly the B operand of v_mfma_f32_16x16x32_bf16
// (B[k = c][j = rho]), with A[i = c'][k = c] = H_32[c'][c] / 16 made in registers
// (+-2^-4 is exact in bf16, the inputs are bf16, the sums accumulate in fp32).  Two
// instructions (c' = 0..15 and 16..31) leave lane l with D[c' = 16 d + 4 q + v][rho],
// d = 0, 1, v = 0..3: four consecutive output columns 32 rho + 16 d + 4 q + v per d.
// The remaining H_8 over a runs across lanes: the row that lane l loads is chosen so
// that a sits in lane bits 0, 1 and 3 (g in bit 2), whose exchanges (lane ^ 1, ^ 2,
// ^ 8) are data-parallel-primitive modifiers of the arithmetic instruction itself.
// A butterfly stage is new = partner + s own, s = -1 in the upper lane of a pair
// = s (own + s partner): the stage computes own + s partner in ONE multiply-add
// (v_fmac_f32 with the exchange as its DPP modifier, written as inline assembly) and
// leaves the factor s pending; partners of later stages share it, so the pending
// factors multiply up to one sign per lane, which goes into the quantizer's scale
// (symmetric codes) or is applied once at the end.
// The eight values are then rounded to bf16 and go through the same
// quantizer arithmetic as everywhere else (column parity = v parity, as in a unit
// of eight consecutive columns), so the codes are exactly those of quantizing
// the rotated row, which the caller can have written out (x_rot) to check.  The
// fp32 sums are taken in another order than the stand-alone transform kernel takes
// them, so a rotated value may round to the neighbouring bf16 there.
//
// HI: units of 8 high columns per thread; LO: spans per wavefront.
// Requires r <= 2048 HI, K - r <= 2048 LO, r and K - r multiples of 256.
// ---------------------------------------------------------------------------
typedef __bf16 v8bf_q __attribute__((ext_vector_type(8)));
typedef float v4f_q __attribute__((ext_vector_type(4)));

template <int HI, int LO, bool ASYM>
__global__ __launch_bounds__(kQuantThreads) void hadamard256_quantize_kernel(
    const uint16_t* __restrict__ x, int64_t ldx, int K, int r, int8_t* __restrict__ q_hi,
    int64_t ld_hi, uint8_t* __restrict__ q_lo, int64_t ld_lo, float* __restrict__ s_hi,
    float* __restrict__ s_lo, int32_t* __restrict__ lo_sum, const RotateArgs rot,
    float* __restrict__ c_hi, float* __restrict__ c_lo) {
    constexpr int RT = kQuantThreads;
    __shared__ float red[16];
    __shared__ int red_sum[4];
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int64_t m = blockIdx.x;
    const int hi_units = r >> 3;
    const int lo_cols = K - r;
    const uint16_t* row = x + m * ldx;
    const int q = lane >> 4;
    // the lane's row of the span: a = lane bits 0, 1, 3; g = lane bit 2
    const int rho = (lane & 3) | ((lane & 8) >> 1) | ((lane & 4) << 1);
    const int cp = lane & 15;   // row c' (and 16 + c') of H_32 that this lane supplies
    // pending sign of the lane after the three exchange stages
    const bool neg = (__builtin_popcount(lane & 11) & 1) != 0;
    const uint32_t flip = neg ? 0x80008000u : 0u;
    const float m1 = (lane & 1) ? -1.0f : 1.0f, m2 = (lane & 2) ? -1.0f : 1.0f, m8 = (lane & 8) ? -1.0f : 1.0f;

    uint4 vh[HI], vl[LO];
#pragma unroll
    for (int i = 0; i < HI; ++i) {
        const int u = t + i * RT;
        vh[i] = u < hi_units ? *reinterpret_cast<const uint4*>(row + (int64_t)u * 8) : make_uint4(0u, 0u, 0u, 0u);
    }
    // rows c' = rho and 16 + rho of H_32 / 16, columns c = 8 q .. 8 q + 7
    uint32_t h0[4], h1[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        uint32_t w0 = 0, w1 = 0;
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            const int c = 8 * q + 2 * k + e;
            const uint32_t s0 = (uint32_t)__builtin_popcount(cp & c) & 1u;
            const uint32_t s1 = (uint32_t)__builtin_popcount((16 + cp) & c) & 1u;
            w0 |= (0x3D80u | (s0 << 15)) << (16 * e);
            w1 |= (0x3D80u | (s1 << 15)) << (16 * e);
        }
        h0[k] = w0;
        h1[k] = w1;
    }
    const v8bf_q ha0 = __builtin_bit_cast(v8bf_q, make_uint4(h0[0], h0[1], h0[2], h0[3]));
    const v8bf_q ha1 = __builtin_bit_cast(v8bf_q, make_uint4(h1[0], h1[1], h1[2], h1[3]));
    // column of the lane's first output of span s, relative to r: + 16 d + v
    const int out_col = 32 * rho + 4 * q;
    // every load of the row is issued before the first product (addresses past the row are
    // clamped into it and the loaded value replaced by zero)
#pragma unroll
    for (int i = 0; i < LO; ++i) {
        const int col = (wave + 4 * i) * 512 + 32 * rho + 8 * q;
        vl[i] = *reinterpret_cast<const uint4*>(row + r + (col < lo_cols ? col : lo_cols - 8));
    }
#pragma unroll
    for (int i = 0; i < LO; ++i) {
        const int s = wave + 4 * i;
        const int col = s * 512 + 32 * rho + 8 * q;
        const uint4 raw = col < lo_cols ? vl[i] : make_uint4(0u, 0u, 0u, 0u);
        const v4f_q zero = {0.0f, 0.0f, 0.0f, 0.0f};
        const v4f_q d0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ha0, __builtin_bit_cast(v8bf_q, raw), zero, 0, 0, 0);
        const v4f_q d1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ha1, __builtin_bit_cast(v8bf_q, raw), zero, 0, 0, 0);
        float f[8] = {d0[0], d0[1], d0[2], d0[3], d1[0], d1[1], d1[2], d1[3]};
        // own + s * partner for all eight values, the exchange as a modifier of the
        // multiply-add (the compiler keeps a separate move in front of it).  The wait states in
        // front cover a write of these registers or of the execution mask just before.
#define RESQ_H8_STAGE(CTRL, MUL)                                                                         \
        asm volatile("s_nop 4\n\t"                                                                        \
                     "v_fmac_f32_dpp %0, %0, %8 " CTRL " row_mask:0xf bank_mask:0xf\n\t"                   \
                     "v_fmac_f32_dpp %1, %1, %8 " CTRL " row_mask:0xf bank_mask:0xf\n\t"                   \
                     "v_fmac_f32_dpp %2, %2, %8 " CTRL " row_mask:0xf bank_mask:0xf\n\t"                   \
                     "v_fmac_f32_dpp %3, %3, %8 " CTRL " row_mask:0xf bank_mask:0xf\n\t"                   \
                     "v_fmac_f32_dpp %4, %4, %8 " CTRL " row_mask:0xf bank_mask:0xf\n\t"                   \
                     "v_fmac_f32_dpp %5, %5, %8 " CTRL " row_mask:0xf bank_mask:0xf\n\t"                   \
                     "v_fmac_f32_dpp %6, %6, %8 " CTRL " row_mask:0xf bank_mask:0xf\n\t"                   \
                     "v_fmac_f32_dpp %7, %7, %8 " CTRL " row_mask:0xf bank_mask:0xf"                        \
                     : "+v"(f[0]), "+v"(f[1]), "+v"(f[2]), "+v"(f[3]), "+v"(f[4]), "+v"(f[5]), "+v"(f[6]),  \
                       "+v"(f[7])                                                                        \
                     : "v"(MUL))
        RESQ_H8_STAGE("quad_perm:[1,0,3,2]", m1);
        RESQ_H8_STAGE("quad_perm:[2,3,0,1]", m2);
        RESQ_H8_STAGE("row_ror:8", m8);
#undef RESQ_H8_STAGE
        vl[i] = pack8_bf16(f, 1.0f);   // the rotated values times the pending sign
        if constexpr (ASYM) vl[i] = make_uint4(vl[i].x ^ flip, vl[i].y ^ flip, vl[i].z ^ flip, vl[i].w ^ flip);
        const int oc = s * 512 + out_col;
        if (rot.x_rot && oc < lo_cols) {
            const uint32_t fx = ASYM ? 0u : flip;
            uint16_t* dst = rot.x_rot + m * rot.ld_rot + r + oc;
            *reinterpret_cast<uint2*>(dst) = make_uint2(vl[i].x ^ fx, vl[i].y ^ fx);
            *reinterpret_cast<uint2*>(dst + 16) = make_uint2(vl[i].z ^ fx, vl[i].w ^ fx);
        }
    }

    float sh, sl, zh = 0.0f, zl = 0.0f;
    if constexpr (ASYM) {
        const float inf = __builtin_huge_valf();
        float ext[4] = {-inf, -inf, -inf, -inf};  // max_h, -min_h, max_l, -min_l
        auto take = [&](const uint4& v, int g) __attribute__((always_inline)) {
            float f[8];
            unpack8_bf16(v, f);
            const float mx = fmaxf(fmaxf(fmaxf(f[0], f[1]), fmaxf(f[2], f[3])),
                                   fmaxf(fmaxf(f[4], f[5]), fmaxf(f[6], f[7])));
            const float mn = fminf(fminf(fminf(f[0], f[1]), fminf(f[2], f[3])),
                                   fminf(fminf(f[4], f[5]), fminf(f[6], f[7])));
            ext[g] = fmaxf(ext[g], mx);
            ext[g + 1] = fmaxf(ext[g + 1], -mn);
        };
#pragma unroll
        for (int i = 0; i < HI; ++i)
            if (t + i * RT < hi_units) take(vh[i], 0);
#pragma unroll
        for (int i = 0; i < LO; ++i)
            if ((wave + 4 * i) * 512 + out_col < lo_cols) take(vl[i], 2);
        block_max4(ext, red);
        zh = -ext[1];
        zl = -ext[3];
        sh = r > 0 ? asym_scale(zh, ext[0], 255) : 1.0f;
        sl = asym_scale(zl, ext[2], 15);
        if (t == 0) {
            if (r > 0) c_hi[m] = zh + 128.0f * sh;
            c_lo[m] = zl + 8.0f * sl;
        }
    } else {
        float amax_h = 0.0f, amax_l = 0.0f;
#pragma unroll
        for (int i = 0; i < HI; ++i) amax_h = fmaxf(amax_h, absmax8(vh[i]));   // zeros past the group
#pragma unroll
        for (int i = 0; i < LO; ++i) amax_l = fmaxf(amax_l, absmax8(vl[i]));   // zeros past the row
        block_max2(amax_h, amax_l, red);
        sh = group_scale(amax_h, kQmaxHi);
        sl = group_scale(amax_l, kQmaxLo);
    }
    const float inv_h = 1.0f / sh, inv_l = 1.0f / sl;
    if (t == 0) {
        if (r > 0) s_hi[m] = sh;
        s_lo[m] = sl;
    }

    int8_t* qh = q_hi + m * ld_hi;
    uint8_t* ql = q_lo + m * ld_lo;
    float odd_f = 0.0f, unused = 0.0f;
#pragma unroll
    for (int i = 0; i < HI; ++i) {
        const int u = t + i * RT;
        if (u < hi_units) {
            uint32_t c[8];
            if constexpr (ASYM) quant8_asym<false>(vh[i], zh, sh, inv_h, c, unused);
            else quant8<false>(vh[i], sh, inv_h, c, unused);
            *reinterpret_cast<uint2*>(qh + (int64_t)u * 8) =
                make_uint2(pack_low_bytes(c[0], c[1], c[2], c[3]), pack_low_bytes(c[4], c[5], c[6], c[7]));
        }
    }
#pragma unroll
    for (int i = 0; i < LO; ++i) {
        const int oc = (wave + 4 * i) * 512 + out_col;
        if (oc < lo_cols) {   // the last span may hold one block only: its upper 8 rows are idle
            uint32_t c[8];
            if constexpr (ASYM) quant8_asym<true>(vl[i], zl, sl, inv_l, c, odd_f);
            else quant8<true>(vl[i], neg ? -sl : sl, neg ? -inv_l : inv_l, c, odd_f);   // x / s = (-x) / (-s)
            uint32_t by[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) by[k] = (c[2 * k + 1] << 4) | c[2 * k];
            const uint32_t w = pack_low_bytes(by[0], by[1], by[2], by[3]);
            uint8_t* dst = ql + (oc >> 1);
            *reinterpret_cast<uint16_t*>(dst) = (uint16_t)w;          // columns oc .. oc + 3
            *reinterpret_cast<uint16_t*>(dst + 8) = (uint16_t)(w >> 16);  // columns oc + 16 .. oc + 19
        }
    }
    int odd_sum = (int)odd_f;
    for (int64_t b = (int64_t)r + 8 * t; b < ld_hi; b += 8 * RT)
        *reinterpret_cast<uint2*>(qh + b) = make_uint2(0u, 0u);
    for (int64_t b = (int64_t)lo_cols / 2 + 4 * t; b < ld_lo; b += 4 * RT)
        *reinterpret_cast<uint32_t*>(ql + b) = 0x08080808u;
    odd_sum = block_sum(odd_sum, red_sum);
    if (t == 0) lo_sum[m] = odd_sum;
}

// ---------------------------------------------------------------------------
// Activations, short rows (K <= 512, e.g. one attention head of a K/V cache
// entry, Section 4.3): a group of G = 16, 32 or 64 lanes per row (G * 8 >= K),
// so 256 / G rows per workgroup, one 8-element unit per lane, reductions inside
// the group: no LDS, no barrier.  Same arithmetic and the same outputs as the
// kernel above.
// ---------------------------------------------------------------------------
template <bool ASYM, int G>
__global__ __launch_bounds__(kQuantThreads) void quantize_act_short_kernel(
    const uint16_t* __restrict__ x, int64_t ldx, int64_t M, int K, int r, int8_t* __restrict__ q_hi,
    int64_t ld_hi, uint8_t* __restrict__ q_lo, int64_t ld_lo, float* __restrict__ s_hi,
    float* __restrict__ s_lo, int32_t* __restrict__ lo_sum, float* __restrict__ c_hi,
    float* __restrict__ c_lo) {
    const int gl = threadIdx.x & (G - 1);  // lane inside the group
    const int64_t m_raw = (int64_t)blockIdx.x * (kQuantThreads / G) + threadIdx.x / G;
    // every lane of a wavefront runs the exchanges and the votes below; groups past
    // the last row work on the last row and store nothing
    const bool row_live = m_raw < M;
    const int64_t m = row_live ? m_raw : M - 1;
    const int nunits = K >> 3, hi_units = r >> 3;
    const bool live = gl < nunits, high = gl < hi_units;
    const uint4 v = live ? reinterpret_cast<const uint4*>(x + m * ldx)[gl] : make_uint4(0u, 0u, 0u, 0u);

    float sh, sl, zh = 0.0f, zl = 0.0f;
    if constexpr (ASYM) {
        const float inf = __builtin_huge_valf();
        float mx = -inf, nmn = -inf;
        if (live) {
            float f[8];
            unpack8_bf16(v, f);
            mx = fmaxf(fmaxf(fmaxf(f[0], f[1]), fmaxf(f[2], f[3])), fmaxf(fmaxf(f[4], f[5]), fmaxf(f[6], f[7])));
            nmn = -fminf(fminf(fminf(f[0], f[1]), fminf(f[2], f[3])), fminf(fminf(f[4], f[5]), fminf(f[6], f[7])));
        }
        const float mx_h = wave_max<G>(high ? mx : -inf), nmn_h = wave_max<G>(high ? nmn : -inf);
        const float mx_l = wave_max<G>(live && !high ? mx : -inf);
        const float nmn_l = wave_max<G>(live && !high ? nmn : -inf);
        zh = -nmn_h;
        zl = -nmn_l;
        sh = r > 0 ? asym_scale(zh, mx_h, 255) : 1.0f;
        sl = K - r > 0 ? asym_scale(zl, mx_l, 15) : 1.0f;
        if (gl == 0 && row_live) {
            if (r > 0) c_hi[m] = zh + 128.0f * sh;
            if (K - r > 0) c_lo[m] = zl + 8.0f * sl;
        }
    } else {
        const float a = live ? absmax8(v) : 0.0f;
        sh = group_scale(wave_max<G>(high ? a : 0.0f), kQmaxHi);
        sl = group_scale(wave_max<G>(high ? 0.0f : a), kQmaxLo);
    }
    if (gl == 0 && row_live) {
        if (r > 0) s_hi[m] = sh;
        if (K - r > 0) s_lo[m] = sl;
    }
    int8_t* qh = q_hi + m * ld_hi;
    uint8_t* ql = q_lo + m * ld_lo;
    float odd_f = 0.0f;
    // the branch on `high` is not wave-uniform, and the quantizer votes across the
    // wavefront: run both kinds for every lane's vote, keep the own kind's result
    uint32_t ch[8], cl8[8];
    float odd_dummy = 0.0f;
    if (hi_units > 0) {
        if constexpr (ASYM) quant8_asym<false>(v, zh, sh, 1.0f / sh, ch, odd_dummy);
        else quant8<false>(v, sh, 1.0f / sh, ch, odd_dummy);
    }
    if (nunits > hi_units) {
        if constexpr (ASYM) quant8_asym<true>(v, zl, sl, 1.0f / sl, cl8, odd_f);
        else quant8<true>(v, sl, 1.0f / sl, cl8, odd_f);
    }
    const int odd_sum = wave_sum<G>(live && !high ? (int)odd_f : 0);
    if (!row_live) return;
    if (live && high) {
        *reinterpret_cast<uint2*>(qh + (int64_t)gl * 8) =
            make_uint2(pack_low_bytes(ch[0], ch[1], ch[2], ch[3]), pack_low_bytes(ch[4], ch[5], ch[6], ch[7]));
    } else if (live) {
        uint32_t by[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) by[k] = (cl8[2 * k + 1] << 4) | cl8[2 * k];
        *reinterpret_cast<uint32_t*>(ql + (int64_t)(gl - hi_units) * 4) = pack_low_bytes(by[0], by[1], by[2], by[3]);
    }
    // zero codes in the padding of both rows
    for (int64_t b = (int64_t)r + 8 * gl; b < ld_hi; b += 8 * G)
        *reinterpret_cast<uint2*>(qh + b) = make_uint2(0u, 0u);
    for (int64_t b = (int64_t)(K - r) / 2 + 4 * gl; b < ld_lo; b += 4 * G)
        *reinterpret_cast<uint32_t*>(ql + b) = 0x08080808u;
    if (gl == 0 && K - r > 0) lo_sum[m] = odd_sum;
}

// ---------------------------------------------------------------------------
// Compact K/V cache rows (Section 5.1 and Appendix C: the cache is quantized per
// head with the asymmetric quantizer of Eq. 1, an eighth of the channels in 8
// bits).  One row per head of a token, no padding:
//   r bytes: the 8-bit codes, 0..255 | (d - r) / 2 bytes: the 4-bit codes, 0..15,
//   channel r + 2j in bits 0..3, r + 2j + 1 in bits 4..7 | fp32 s_hi, z_hi, s_lo, z_lo
// with x ~ code * s + z per group: r + (d - r) / 2 + 16 bytes for 2 d bytes of bf16.
// The quantizer is the short-row kernel above (G lanes per row, no LDS, no
// barrier); its stored codes (code - 2^(N-1), the GEMM's operand form) become the
// codes of Eq. 1 with one XOR per four bytes.
// ---------------------------------------------------------------------------
template <int G>
__global__ __launch_bounds__(kQuantThreads) void quantize_kv_cache_kernel(
    const uint16_t* __restrict__ x, int64_t ldx, int64_t rows, int d, int r, uint8_t* __restrict__ cache,
    int64_t row_bytes) {
    const int gl = threadIdx.x & (G - 1);  // lane inside the group
    const int64_t m_raw = (int64_t)blockIdx.x * (kQuantThreads / G) + threadIdx.x / G;
    // every lane of a wavefront runs the exchanges and the votes below; groups past
    // the last row work on the last row and store nothing
    const bool row_live = m_raw < rows;
    const int64_t m = row_live ? m_raw : rows - 1;
    const int nunits = d >> 3, hi_units = r >> 3;
    const bool live = gl < nunits, high = gl < hi_units;
    const uint4 v = live ? reinterpret_cast<const uint4*>(x + m * ldx)[gl] : make_uint4(0u, 0u, 0u, 0u);

    const float inf = __builtin_huge_valf();
    float mx = -inf, nmn = -inf;
    if (live) {
        float f[8];
        unpack8_bf16(v, f);
        mx = fmaxf(fmaxf(fmaxf(f[0], f[1]), fmaxf(f[2], f[3])), fmaxf(fmaxf(f[4], f[5]), fmaxf(f[6], f[7])));
        nmn = -fminf(fminf(fminf(f[0], f[1]), fminf(f[2], f[3])), fminf(fminf(f[4], f[5]), fminf(f[6], f[7])));
    }
    const float mx_h = wave_max<G>(high ? mx : -inf), nmn_h = wave_max<G>(high ? nmn : -inf);
    const float mx_l = wave_max<G>(live && !high ? mx : -inf);
    const float nmn_l = wave_max<G>(live && !high ? nmn : -inf);
    // an absent group: scale 1, zero-point 0
    const float zh = r > 0 ? -nmn_h : 0.0f, zl = d - r > 0 ? -nmn_l : 0.0f;
    const float sh = r > 0 ? asym_scale(zh, mx_h, 255) : 1.0f;
    const float sl = d - r > 0 ? asym_scale(zl, mx_l, 15) : 1.0f;
    // the branch on `high` is not wave-uniform, and the quantizer votes across the
    // wavefront: run both kinds for every lane's vote, keep the own kind's result
    uint32_t ch[8], cl8[8];
    float odd_dummy = 0.0f;
    if (hi_units > 0) quant8_asym<false>(v, zh, sh, 1.0f / sh, ch, odd_dummy);
    if (nunits > hi_units) quant8_asym<true>(v, zl, sl, 1.0f / sl, cl8, odd_dummy);
    if (!row_live) return;
    uint8_t* row = cache + m * row_bytes;
    if (live && high) {
        // stored = code - 128 in the low byte: flipping bit 7 gives the code
        uint32_t* dst = reinterpret_cast<uint32_t*>(row + gl * 8);   // rows are 4-byte aligned
        dst[0] = pack_low_bytes(ch[0], ch[1], ch[2], ch[3]) ^ 0x80808080u;
        dst[1] = pack_low_bytes(ch[4], ch[5], ch[6], ch[7]) ^ 0x80808080u;
    } else if (live) {
        // even channels are stored as the code already, odd ones as code - 8 in two's complement
        uint32_t by[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) by[k] = ((cl8[2 * k + 1] << 4) | (cl8[2 * k] & 0xFu)) ^ 0x80u;
        *reinterpret_cast<uint32_t*>(row + r + (gl - hi_units) * 4) = pack_low_bytes(by[0], by[1], by[2], by[3]);
    }
    if (gl == 0) {
        float* par = reinterpret_cast<float*>(row + r + (d - r) / 2);
        par[0] = sh;
        par[1] = zh;
        par[2] = sl;
        par[3] = zl;
    }
}

__device__ __forceinline__ uint32_t pack_bf16_pair(float lo, float hi) {
    const v2bf_had r = __builtin_convertvector((v2f_had){lo, hi}, v2bf_had);   // round to nearest even
    return *reinterpret_cast<const uint32_t*>(&r);
}

// The reader of such rows: x[m, k] = bf16(code * s + z) (Eq. 1), one lane per eight channels.
template <int G>
__global__ __launch_bounds__(kQuantThreads) void dequantize_kv_cache_kernel(
    const uint8_t* __restrict__ cache, int64_t row_bytes, int64_t rows, int d, int r, uint16_t* __restrict__ x,
    int64_t ldx) {
    const int gl = threadIdx.x & (G - 1);
    const int64_t m = (int64_t)blockIdx.x * (kQuantThreads / G) + threadIdx.x / G;
    const int nunits = d >> 3, hi_units = r >> 3;
    if (m >= rows || gl >= nunits) return;
    const uint8_t* row = cache + m * row_bytes;
    const float* par = reinterpret_cast<const float*>(row + r + (d - r) / 2);
    float f[8];
    if (gl < hi_units) {
        const uint32_t* src = reinterpret_cast<const uint32_t*>(row + gl * 8);
        const uint32_t c0 = src[0], c1 = src[1];
        const float s = par[0], z = par[1];
#pragma unroll
        for (int k = 0; k < 8; ++k) f[k] = fmaf((float)(((k < 4 ? c0 : c1) >> (8 * (k & 3))) & 0xFFu), s, z);
    } else {
        const uint32_t c = *reinterpret_cast<const uint32_t*>(row + r + (gl - hi_units) * 4);
        const float s = par[2], z = par[3];
#pragma unroll
        for (int k = 0; k < 8; ++k) f[k] = fmaf((float)((c >> (4 * k)) & 0xFu), s, z);
    }
    uint4 o;
    o.x = pack_bf16_pair(f[0], f[1]);
    o.y = pack_bf16_pair(f[2], f[3]);
    o.z = pack_bf16_pair(f[4], f[5]);
    o.w = pack_bf16_pair(f[6], f[7]);
    reinterpret_cast<uint4*>(x + m * ldx)[gl] = o;
}

// ---------------------------------------------------------------------------
// Activations, any K, r (K - r even) and alignment: two passes over the row
// with 2-byte loads.  Correct everywhere, fast nowhere.
// ---------------------------------------------------------------------------
template <bool ASYM>
__global__ __launch_bounds__(kQuantThreads) void quantize_act_generic_kernel(
    const uint16_t* __restrict__ x, int64_t ldx, int K, int r, int8_t* __restrict__ q_hi,
    int64_t ld_hi, uint8_t* __restrict__ q_lo, int64_t ld_lo, float* __restrict__ s_hi,
    float* __restrict__ s_lo, int32_t* __restrict__ lo_sum, float* __restrict__ c_hi,
    float* __restrict__ c_lo) {
    __shared__ float red[16];
    __shared__ int red_sum[4];
    const int64_t m = blockIdx.x;
    const int t = threadIdx.x;
    const uint16_t* row = x + m * ldx;
    float sh, sl, zh = 0.0f, zl = 0.0f;
    if constexpr (ASYM) {
        const float inf = __builtin_huge_valf();
        float ext[4] = {-inf, -inf, -inf, -inf};  // max_h, -min_h, max_l, -min_l
        for (int k = t; k < K; k += kQuantThreads) {
            const float a = bf16_bits_to_f32(row[k]);
            const int g = k < r ? 0 : 2;
            ext[g] = fmaxf(ext[g], a);
            ext[g + 1] = fmaxf(ext[g + 1], -a);
        }
        block_max4(ext, red);
        zh = -ext[1];
        zl = -ext[3];
        sh = r > 0 ? asym_scale(zh, ext[0], 255) : 1.0f;
        sl = K - r > 0 ? asym_scale(zl, ext[2], 15) : 1.0f;
        if (t == 0) {
            if (r > 0) c_hi[m] = zh + 128.0f * sh;
            if (K - r > 0) c_lo[m] = zl + 8.0f * sl;
        }
    } else {
        float amax_h = 0.0f, amax_l = 0.0f;
        for (int k = t; k < K; k += kQuantThreads) {
            const float a = bf16_bits_to_f32(row[k] & 0x7FFFu);
            if (k < r) amax_h = fmaxf(amax_h, a);
            else amax_l = fmaxf(amax_l, a);
        }
        block_max2(amax_h, amax_l, red);
        sh = group_scale(amax_h, kQmaxHi);
        sl = group_scale(amax_l, kQmaxLo);
    }
    if (t == 0) {
        if (r > 0) s_hi[m] = sh;
        if (K - r > 0) s_lo[m] = sl;
    }
    // stored codes: symmetric codes as they are; asymmetric codes minus 2^(N-1)
    auto code_hi = [&](float v) {
        if constexpr (ASYM) return quant_code_asym(v, zh, sh, 255) - 128;
        else return quant_code(v, sh, kQmaxHi);
    };
    auto code_lo = [&](float v) {
        if constexpr (ASYM) return quant_code_asym(v, zl, sl, 15) - 8;
        else return quant_code(v, sl, kQmaxLo);
    };
    int8_t* qh = q_hi + m * ld_hi;
    uint8_t* ql = q_lo + m * ld_lo;
    for (int64_t k = t; k < ld_hi; k += kQuantThreads)
        qh[k] = k < r ? (int8_t)code_hi(bf16_bits_to_f32(row[k])) : (int8_t)0;
    const int pairs = (K - r) / 2;
    int odd_sum = 0;
    for (int64_t j = t; j < ld_lo; j += kQuantThreads) {
        uint32_t byte = 0x08u;
        if (j < pairs) {
            const int c0 = code_lo(bf16_bits_to_f32(row[r + 2 * j]));
            const int c1 = code_lo(bf16_bits_to_f32(row[r + 2 * j + 1]));
            odd_sum += c1;
            byte = (uint32_t)((c0 + 8) & 0xF) | ((uint32_t)(c1 & 0xF) << 4);
        }
        ql[j] = (uint8_t)byte;
    }
    odd_sum = block_sum(odd_sum, red_sum);
    if (t == 0 && K - r > 0) lo_sum[m] = odd_sum;
}

// ---------------------------------------------------------------------------
// Weights (offline): one block per padded output channel.
// ---------------------------------------------------------------------------

// smallest positive normal fp16 >= s after clamping s to [2^-14, 65504]
__device__ __forceinline__ uint16_t fp16_round_up(float s) {
    s = fminf(fmaxf(s, 6.103515625e-05f), 65504.0f);
    const uint32_t u = __float_as_uint(s);
    uint32_t h = (((u >> 23) - 112u) << 10) | ((u & 0x7FFFFFu) >> 13);
    if (u & 0x1FFFu) h += 1u;
    return (uint16_t)h;
}
__device__ __forceinline__ float fp16_normal_to_f32(uint32_t h) {
    return __uint_as_float((((h >> 10) & 0x1Fu) + 112u) << 23 | (h & 0x3FFu) << 13);
}

__global__ __launch_bounds__(kQuantThreads) void pack_weights_kernel(
    const uint16_t* __restrict__ w, int64_t ldw, WeightLayout L, uint8_t* __restrict__ packed) {
    __shared__ float red[8];
    __shared__ int red_sum[4];
    const int64_t n = blockIdx.x;  // 0 .. n_pad - 1
    const int t = threadIdx.x;
    const int K = (int)L.K, r = (int)L.r;
    uint16_t* sw_hi = reinterpret_cast<uint16_t*>(packed + L.scale_off);
    uint16_t* sw_lo = sw_hi + L.n_pad;
    const bool live = n < L.N;
    const uint16_t* row = w + (live ? n : 0) * ldw;

    // rows that can be read 16 bytes at a time (every vector then lies inside one group)
    const bool vec = (reinterpret_cast<uintptr_t>(w) & 15) == 0 && ldw % 8 == 0 && K % 8 == 0 && r % 8 == 0;
    const uint4* row4 = reinterpret_cast<const uint4*>(row);
    // eight consecutive weights from column k on (zero where the row or the group has ended)
    auto load8 = [&](int k, int end, uint16_t (&e)[8]) __attribute__((always_inline)) {
        if (vec) {
            uint4 v = make_uint4(0u, 0u, 0u, 0u);
            if (k < end) v = row4[k >> 3];
            const uint32_t ww[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int j = 0; j < 8; ++j) e[j] = (uint16_t)(ww[j >> 1] >> (16 * (j & 1)));
        } else {
#pragma unroll
            for (int j = 0; j < 8; ++j) e[j] = k + j < end ? row[k + j] : (uint16_t)0;
        }
    };
    float amax_h = 0.0f, amax_l = 0.0f;
    if (live) {
        if (vec) {
            for (int u = t; u < (K >> 3); u += kQuantThreads) {
                const float a = absmax8(row4[u]);
                if (u < (r >> 3)) amax_h = fmaxf(amax_h, a);
                else amax_l = fmaxf(amax_l, a);
            }
        } else {
            for (int k = t; k < K; k += kQuantThreads) {
                const float a = bf16_bits_to_f32(row[k] & 0x7FFFu);
                if (k < r) amax_h = fmaxf(amax_h, a);
                else amax_l = fmaxf(amax_l, a);
            }
        }
    }
    block_max2(amax_h, amax_l, red);
    const uint16_t hh = fp16_round_up(group_scale(amax_h, kQmaxHi));
    const uint16_t hl = fp16_round_up(group_scale(amax_l, kQmaxLo));
    const float sh = fp16_normal_to_f32(hh), sl = fp16_normal_to_f32(hl);
    if (t == 0) {
        sw_hi[n] = (live && r > 0) ? hh : (uint16_t)0x3C00u;      // 1.0
        sw_lo[n] = (live && K - r > 0) ? hl : (uint16_t)0x3C00u;
    }
    // high group: units of 16 codes
    int sum_hi = 0, sum_lo_odd = 0;
    for (int u = t; u < (int)(L.kh_pad / 16); u += kQuantThreads) {
        uint32_t out[4] = {0u, 0u, 0u, 0u};
        if (live) {
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                uint16_t e[8];
                load8(u * 16 + q * 8, r, e);
#pragma unroll
                for (int jj = 0; jj < 8; ++jj) {
                    const int j = q * 8 + jj, k = u * 16 + j;
                    if (k < r) {
                        const int c = quant_code(bf16_bits_to_f32(e[jj]), sh, kQmaxHi);
                        sum_hi += c;
                        out[j >> 2] |= (uint32_t)(c & 0xFF) << (8 * (j & 3));
                    }
                }
            }
        }
        *reinterpret_cast<uint4*>(packed + hi_byte_offset(L, n, (int64_t)u * 16)) =
            make_uint4(out[0], out[1], out[2], out[3]);
    }
    // low group: units of 32 codes = 16 bytes; byte = (even code) << 4 | (odd code + 8)
    int even_sum = 0;
    for (int u = t; u < (int)(L.kl_pad / 32); u += kQuantThreads) {
        uint32_t out[4] = {0x08080808u, 0x08080808u, 0x08080808u, 0x08080808u};
        if (live) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                uint16_t e[8];
                load8(r + u * 32 + q * 8, K, e);
#pragma unroll
                for (int jj = 0; jj < 8; ++jj) {
                    const int j = q * 8 + jj, k = r + u * 32 + j;
                    if (k < K) {
                        const int c = quant_code(bf16_bits_to_f32(e[jj]), sl, kQmaxLo);
                        if (j & 1) {
                            sum_lo_odd += c;
                            out[j >> 3] = (out[j >> 3] & ~(0xFu << (4 * (j & 7) - 4))) |
                                          ((uint32_t)((c + 8) & 0xF) << (4 * (j & 7) - 4));
                        } else {
                            even_sum += c;
                            out[j >> 3] |= (uint32_t)(c & 0xF) << (4 * (j & 7) + 4);
                        }
                    }
                }
            }
        }
        *reinterpret_cast<uint4*>(packed + lo_byte_offset(L, n, (int64_t)u * 16)) =
            make_uint4(out[0], out[1], out[2], out[3]);
    }
    even_sum = block_sum(even_sum, red_sum);
    __syncthreads();
    sum_lo_odd = block_sum(sum_lo_odd, red_sum);
    __syncthreads();
    sum_hi = block_sum(sum_hi, red_sum);
    if (t == 0) {
        int32_t* sums = reinterpret_cast<int32_t*>(packed + L.scale_off + 4 * L.n_pad);
        sums[n] = even_sum;
        sums[L.n_pad + n] = sum_hi;
        sums[2 * L.n_pad + n] = even_sum + sum_lo_odd;
    }
}

__global__ __launch_bounds__(kQuantThreads) void unpack_weights_kernel(
    const uint8_t* __restrict__ packed, WeightLayout L, int8_t* __restrict__ w_hi,
    int8_t* __restrict__ w_lo, uint16_t* __restrict__ sw_hi, uint16_t* __restrict__ sw_lo) {
    const int64_t n = blockIdx.x;  // 0 .. N - 1
    const int t = threadIdx.x;
    const int r = (int)L.r, kl = (int)(L.K - L.r);
    const uint16_t* s = reinterpret_cast<const uint16_t*>(packed + L.scale_off);
    if (t == 0) {
        if (r > 0) sw_hi[n] = s[n];
        if (kl > 0) sw_lo[n] = s[L.n_pad + n];
    }
    for (int k = t; k < r; k += kQuantThreads)
        w_hi[n * r + k] = (int8_t)packed[hi_byte_offset(L, n, k)];
    for (int k = t; k < kl; k += kQuantThreads) {
        const uint32_t byte = packed[lo_byte_offset(L, n, k / 2)];
        // even column: bits 4..7, two's complement; odd column: bits 0..3, code + 8
        w_lo[n * (int64_t)kl + k] = (k & 1) ? (int8_t)((int)(byte & 0xFu) - 8)
                                            : (int8_t)((int)((byte >> 4) ^ 8u) - 8);
    }
}

}  // namespace resq
