/*
 * CPU oracle for the ResQ mixed-precision quantized linear layer.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what
 * the layer computes, written from the paper (ResQ, arXiv 2412.14363) so that
 * the GPU library can be checked against it.  Only the test-suite, the smoke
 * check and the benchmark's cpu_baseline leg may call it; the product path
 * never does.  It shares no code, header, table or helper with the HIP path.
 *
 * Every routine takes the steps in the paper's order, with no blocking, no
 * fusion and no reordering; OpenMP only spreads independent rows over cores.
 *
 * Conventions fixed where the paper is silent (each is also listed in the
 * design notes):
 *   - columns [0, r) form the high-precision group (H = 8 bits), columns
 *     [r, K) the low-precision group (L = 4 bits)        (Section 4.1, Eq. 2)
 *   - symmetric quantizer, zero-point 0, scale = max|x| / (2^(N-1) - 1),
 *     computed per token for activations and per output channel for weights
 *     (Section 3 Eq. 1; Section 5.1 "Implementation details")
 *   - the round in Eq. 1 is round-half-to-even of the fp32 quotient x / s;
 *     the clip is to [-(2^(N-1)-1), 2^(N-1)-1]
 *   - an all-zero group gets scale 1
 *   - the asymmetric branch of Eq. 1 (activations only, the setting of Section
 *     5.1): z = min, s = (max - min) / (2^N - 1), unsigned codes 0 .. 2^N - 1,
 *     the difference x - z and the quotient both rounded to fp32
 *   - weight scales are stored in fp16, rounded toward +inf from the fp32
 *     quotient (so that no code can exceed the clip) and clamped to the fp16
 *     normal range; weight codes are computed with the stored value
 *   - 4-bit codes are packed two per byte: the even element in bits 0..3 as
 *     code + 8 (offset binary, 1..15), the odd element in bits 4..7 in two's
 *     complement; a padding byte holds two zero codes, i.e. 0x08
 *
 * Pins: every function here is checked in tests/test_oracle_pins.py against
 * invariants, closed forms, library routines and exact brute force; none is
 * "parity unpinned".  The paper prints no worked numeric example, so no
 * end-to-end value is pinned to a printed number.
 */
#include <math.h>
#include <stdint.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define QMAX_H 127 /* 2^(8-1) - 1, Eq. 1 with N = 8 */
#define QMAX_L 7   /* 2^(4-1) - 1, Eq. 1 with N = 4 */

int oracle_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ---- number formats ---------------------------------------------------- */

static float bf16_to_f32(uint16_t b) {
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

/* fp16 bit pattern of a positive normal number -> float (exact) */
static float fp16_normal_to_f32(uint16_t h) {
    uint32_t e = (uint32_t)(h >> 10) & 0x1Fu;
    uint32_t m = (uint32_t)h & 0x3FFu;
    uint32_t u = ((e - 15u + 127u) << 23) | (m << 13);
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

/* smallest positive normal fp16 that is >= s, after clamping s to the fp16
 * normal range [2^-14, 65504] */
static uint16_t f32_to_fp16_up(float s) {
    const float lo = 6.103515625e-05f; /* 2^-14 */
    const float hi = 65504.0f;
    if (!(s > lo)) s = lo;
    if (s > hi) s = hi;
    uint32_t u;
    memcpy(&u, &s, sizeof u);
    uint32_t e = (u >> 23) & 0xFFu;          /* biased fp32 exponent, 113..142 */
    uint32_t m = u & 0x7FFFFFu;
    uint32_t h = ((e - 127u + 15u) << 10) | (m >> 13);
    if (m & 0x1FFFu) h += 1u;                /* discard bits set: next fp16 up */
    return (uint16_t)h;
}

/* round a double to the nearest bf16 (ties to even), directly, no float step */
static uint16_t f64_to_bf16(double d) {
    if (d == 0.0 || !isfinite(d)) {
        float f = (float)d;
        uint32_t u;
        memcpy(&u, &f, sizeof u);
        return (uint16_t)(u >> 16);
    }
    int e;
    (void)frexp(d, &e);          /* |d| = f * 2^e, f in [0.5, 1) */
    int q = e - 8;               /* bf16 keeps 8 significant bits: quantum 2^(e-8) */
    if (q < -133) q = -133;      /* bf16 subnormal quantum 2^-133 */
    double n = nearbyint(ldexp(d, -q));
    float f = (float)ldexp(n, q); /* exact: at most 8 significant bits */
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    return (uint16_t)(u >> 16);
}

void oracle_round_bf16(const double* y, int64_t n, uint16_t* out) {
    for (int64_t i = 0; i < n; ++i) out[i] = f64_to_bf16(y[i]);
}

/* ---- the quantizer (Section 3, Eq. 1, symmetric branch) ---------------- */

/* scale of one group: max|x| / qmax in fp32; 1 for an all-zero group */
static float group_scale_bf16(const uint16_t* v, int64_t n, int qmax) {
    float amax = 0.0f;
    for (int64_t k = 0; k < n; ++k) {
        float a = fabsf(bf16_to_f32(v[k]));
        if (a > amax) amax = a;
    }
    if (amax == 0.0f) return 1.0f;
    return amax / (float)qmax;
}

/* integer code of x: round-half-to-even of the fp32 quotient, then clip */
static int quant_code(float x, float s, int qmax) {
    volatile float t = x / s;      /* volatile: the quotient is rounded to fp32 */
    float q = nearbyintf(t);       /* default rounding mode: ties to even */
    if (q > (float)qmax) q = (float)qmax;
    if (q < -(float)qmax) q = -(float)qmax;
    return (int)q;
}

/*
 * Mixed-precision activation quantization (Section 4.1, Eq. 2), per token
 * (Section 5.1): columns [0, r) -> 8-bit codes with scale s_hi[m], columns
 * [r, K) -> 4-bit codes with scale s_lo[m].  Codes are returned one per byte.
 *   x     bf16 bits [M, ldx]        q_hi int8 [M, r]     q_lo int8 [M, K - r]
 */
void oracle_quantize_act(const uint16_t* x, int64_t ldx, int64_t M, int64_t K, int64_t r,
                         int8_t* q_hi, int8_t* q_lo, float* s_hi, float* s_lo) {
    const int64_t kl = K - r;
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        const uint16_t* row = x + m * ldx;
        if (r > 0) {
            float s = group_scale_bf16(row, r, QMAX_H);
            s_hi[m] = s;
            for (int64_t k = 0; k < r; ++k)
                q_hi[m * r + k] = (int8_t)quant_code(bf16_to_f32(row[k]), s, QMAX_H);
        }
        if (kl > 0) {
            float s = group_scale_bf16(row + r, kl, QMAX_L);
            s_lo[m] = s;
            for (int64_t k = 0; k < kl; ++k)
                q_lo[m * kl + k] = (int8_t)quant_code(bf16_to_f32(row[r + k]), s, QMAX_L);
        }
    }
}

/*
 * Asymmetric branch of Eq. 1 (Section 3), the setting of the paper's own
 * experiments for activations (Section 5.1, per token), applied to each group
 * of Eq. 2 separately:
 *   z = min(x),  s = (max(x) - min(x)) / (2^N - 1),
 *   code = clip(round((x - z) / s), 0, 2^N - 1),   x ~ code * s + z.
 * The difference and the quotient are fp32 IEEE operations, the round is half
 * to even, as for the symmetric branch; a constant group (max = min) gets s = 1
 * and codes 0.  Codes are returned unsigned, one per byte.
 */
static void quantize_group_asym(const uint16_t* v, int64_t n, int levels, uint8_t* q, float* s_out,
                                float* z_out) {
    float mn = bf16_to_f32(v[0]), mx = mn;
    for (int64_t k = 1; k < n; ++k) {
        float a = bf16_to_f32(v[k]);
        if (a < mn) mn = a;
        if (a > mx) mx = a;
    }
    volatile float range = mx - mn;
    float s = range == 0.0f ? 1.0f : range / (float)levels;
    for (int64_t k = 0; k < n; ++k) {
        volatile float d = bf16_to_f32(v[k]) - mn; /* volatile: rounded to fp32 */
        volatile float t = d / s;
        float c = nearbyintf(t);
        if (c < 0.0f) c = 0.0f;
        if (c > (float)levels) c = (float)levels;
        q[k] = (uint8_t)c;
    }
    *s_out = s;
    *z_out = mn;
}

void oracle_quantize_act_asym(const uint16_t* x, int64_t ldx, int64_t M, int64_t K, int64_t r,
                              uint8_t* q_hi, uint8_t* q_lo, float* s_hi, float* s_lo,
                              float* z_hi, float* z_lo) {
    const int64_t kl = K - r;
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        const uint16_t* row = x + m * ldx;
        if (r > 0) quantize_group_asym(row, r, 255, q_hi + m * r, s_hi + m, z_hi + m);
        if (kl > 0) quantize_group_asym(row + r, kl, 15, q_lo + m * kl, s_lo + m, z_lo + m);
    }
}

/*
 * Integer GEMM of unsigned activation codes with signed weight codes:
 * acc[m, n] = sum_k a[m, k] * b[n, k], exact in int64 (Eq. 4 with the codes of
 * the asymmetric quantizer).
 */
void oracle_gemm_u8i8_i64(const uint8_t* a, int64_t lda, const int8_t* b, int64_t ldb, int64_t M,
                          int64_t N, int64_t Kc, int64_t* acc) {
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        for (int64_t n = 0; n < N; ++n) {
            int64_t s = 0;
            for (int64_t k = 0; k < Kc; ++k)
                s += (int64_t)a[m * lda + k] * (int64_t)b[n * ldb + k];
            acc[m * N + n] = s;
        }
    }
}

/*
 * Dequantization with asymmetric activations: inserting x ~ q s + z (Eq. 1)
 * and w ~ c sw into Eq. 4 gives, per group,
 *   y[m, n] += sw[n] * ( s[m] * sum_k q[m, k] c[n, k]  +  z[m] * sum_k c[n, k] ),
 * evaluated in fp64 from the fp32 scales and zero-points.  acc_* are the sums
 * over the unsigned codes, wsum_* the per-channel sums of the weight codes.
 */
void oracle_dequant_asym(const int64_t* acc_hi, const int64_t* acc_lo, const float* s_hi,
                         const float* s_lo, const float* z_hi, const float* z_lo,
                         const int64_t* wsum_hi, const int64_t* wsum_lo, const uint16_t* sw_hi,
                         const uint16_t* sw_lo, int64_t M, int64_t N, double* y) {
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        for (int64_t n = 0; n < N; ++n) {
            double v = 0.0;
            if (acc_hi)
                v += (double)fp16_normal_to_f32(sw_hi[n]) *
                     ((double)s_hi[m] * (double)acc_hi[m * N + n] +
                      (double)z_hi[m] * (double)wsum_hi[n]);
            if (acc_lo)
                v += (double)fp16_normal_to_f32(sw_lo[n]) *
                     ((double)s_lo[m] * (double)acc_lo[m * N + n] +
                      (double)z_lo[m] * (double)wsum_lo[n]);
            y[m * N + n] = v;
        }
    }
}

/*
 * Mixed-precision weight quantization along the input dimension (Section 4.1,
 * Eq. 3), per output channel, symmetric (Section 5.1), round-to-nearest.
 * W is [N, K] (out_features, in_features).  Scales are fp16 bit patterns,
 * rounded up as described in the header; codes use the stored scale.
 */
void oracle_quantize_weights(const uint16_t* w, int64_t ldw, int64_t N, int64_t K, int64_t r,
                             int8_t* w_hi, int8_t* w_lo, uint16_t* sw_hi, uint16_t* sw_lo) {
    const int64_t kl = K - r;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        const uint16_t* row = w + n * ldw;
        if (r > 0) {
            uint16_t h = f32_to_fp16_up(group_scale_bf16(row, r, QMAX_H));
            float s = fp16_normal_to_f32(h);
            sw_hi[n] = h;
            for (int64_t k = 0; k < r; ++k)
                w_hi[n * r + k] = (int8_t)quant_code(bf16_to_f32(row[k]), s, QMAX_H);
        }
        if (kl > 0) {
            uint16_t h = f32_to_fp16_up(group_scale_bf16(row + r, kl, QMAX_L));
            float s = fp16_normal_to_f32(h);
            sw_lo[n] = h;
            for (int64_t k = 0; k < kl; ++k)
                w_lo[n * kl + k] = (int8_t)quant_code(bf16_to_f32(row[r + k]), s, QMAX_L);
        }
    }
}

/*
 * Pack 4-bit codes two per byte: element 2j in bits 0..3 of byte j as code + 8
 * (offset binary), element 2j+1 in bits 4..7 in two's complement.  Each output
 * row has ld_out bytes; bytes past cols/2 hold two zero codes (0x08), which add
 * nothing to a dot product.  cols must be even.
 */
void oracle_pack_nibbles(const int8_t* codes, int64_t rows, int64_t cols, int64_t ld_out,
                         uint8_t* out) {
    for (int64_t i = 0; i < rows; ++i) {
        uint8_t* o = out + i * ld_out;
        memset(o, 0x08, (size_t)ld_out);
        for (int64_t j = 0; j < cols / 2; ++j) {
            uint8_t a = (uint8_t)(codes[i * cols + 2 * j] + 8) & 0xFu;
            uint8_t b = (uint8_t)codes[i * cols + 2 * j + 1] & 0xFu;
            o[j] = (uint8_t)(a | (b << 4));
        }
    }
}

/*
 * Per row, the sum of the codes in odd positions (1, 3, 5, ...).  The GPU
 * quantizer emits this number per token next to the packed low codes.
 */
void oracle_odd_code_sums(const int8_t* codes, int64_t rows, int64_t cols, int32_t* out) {
    for (int64_t i = 0; i < rows; ++i) {
        int32_t s = 0;
        for (int64_t k = 1; k < cols; k += 2) s += codes[i * cols + k];
        out[i] = s;
    }
}

/* ---- the two integer GEMMs (Section 4.1, Eq. 4) ------------------------ */

/*
 * acc[m, n] = sum_k a[m, k] * b[n, k], exact in int64.  Returns how many
 * results do not fit an int32 (the GPU accumulates in int32).
 */
int64_t oracle_gemm_i64(const int8_t* a, int64_t lda, const int8_t* b, int64_t ldb,
                        int64_t M, int64_t N, int64_t Kc, int64_t* acc) {
    int64_t overflow = 0;
#pragma omp parallel for schedule(static) reduction(+ : overflow)
    for (int64_t m = 0; m < M; ++m) {
        for (int64_t n = 0; n < N; ++n) {
            int64_t s = 0;
            for (int64_t k = 0; k < Kc; ++k)
                s += (int64_t)a[m * lda + k] * (int64_t)b[n * ldb + k];
            acc[m * N + n] = s;
            if (s > INT32_MAX || s < INT32_MIN) overflow += 1;
        }
    }
    return overflow;
}

/*
 * Dequantized layer output (Eq. 1's "* s" factor applied to both operands of
 * each product of Eq. 4):
 *   y[m, n] = A_hi[m, n] * s_hi[m] * sw_hi[n] + A_lo[m, n] * s_lo[m] * sw_lo[n]
 * in fp64 from the fp32 activation scales and fp16 weight scales.  A group of
 * width zero is passed as a null accumulator and contributes nothing.
 */
void oracle_dequant(const int64_t* acc_hi, const int64_t* acc_lo, const float* s_hi,
                    const float* s_lo, const uint16_t* sw_hi, const uint16_t* sw_lo, int64_t M,
                    int64_t N, double* y) {
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        for (int64_t n = 0; n < N; ++n) {
            double v = 0.0;
            if (acc_hi)
                v += (double)acc_hi[m * N + n] *
                     ((double)s_hi[m] * (double)fp16_normal_to_f32(sw_hi[n]));
            if (acc_lo)
                v += (double)acc_lo[m * N + n] *
                     ((double)s_lo[m] * (double)fp16_normal_to_f32(sw_lo[n]));
            y[m * N + n] = v;
        }
    }
}

/* ---- online Hadamard (Section 4.3, projection U_D) --------------------- */

/*
 * y[m, c0 + g*b + j] = (1/sqrt(b)) * sum_i x[m, c0 + g*b + i] * H_b[i, j]
 * for every block g of b columns inside [c0, c1), with H_b the Sylvester
 * (natural-order) Hadamard matrix H_b[i, j] = (-1)^popcount(i & j).  Written
 * as the matrix product it is, in fp64, result rounded to bf16.  Columns
 * outside [c0, c1) are copied.  b must be a power of two dividing c1 - c0.
 */
void oracle_hadamard(const uint16_t* x, uint16_t* y, int64_t ld, int64_t M, int64_t K,
                     int64_t c0, int64_t c1, int64_t b) {
    const double inv = 1.0 / sqrt((double)b);
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        const uint16_t* xr = x + m * ld;
        uint16_t* yr = y + m * ld;
        for (int64_t k = 0; k < c0; ++k) yr[k] = xr[k];
        for (int64_t k = c1; k < K; ++k) yr[k] = xr[k];
        for (int64_t g0 = c0; g0 < c1; g0 += b) {
            for (int64_t j = 0; j < b; ++j) {
                double s = 0.0;
                for (int64_t i = 0; i < b; ++i) {
                    double v = (double)bf16_to_f32(xr[g0 + i]);
                    s += (__builtin_popcountll((unsigned long long)(i & j)) & 1) ? -v : v;
                }
                yr[g0 + j] = f64_to_bf16(s * inv);
            }
        }
    }
}
