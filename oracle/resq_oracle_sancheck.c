/*
 * TEST INFRASTRUCTURE: runs every entry point of the oracle (resq_oracle.c, included below
 * as it is) once on small ragged shapes with heap buffers of exactly the documented sizes,
 * for a build with -fsanitize=address,undefined: an access past a buffer, a signed
 * overflow, a misaligned or out-of-range conversion in the oracle ends the program.
 * It checks only what Section 3, Eq. 1 fixes at a glance (codes inside their ranges);
 * the values are pinned by tests/test_oracle_pins.py.  Exit code 0 = clean.
 */
#include "resq_oracle.c"

#include <stdio.h>
#include <stdlib.h>

static uint32_t rng_state = 12345u;
static uint32_t rng(void) {
    rng_state = rng_state * 1664525u + 1013904223u;
    return rng_state >> 8;
}
/* a bf16 bit pattern of a finite number of moderate size, a zero now and then */
static uint16_t rand_bf16(void) {
    uint32_t r = rng();
    if ((r & 63u) == 0) return 0;
    uint16_t sign = (uint16_t)((r >> 6 & 1u) << 15);
    uint16_t expo = (uint16_t)(120 + (r >> 7) % 12);
    return (uint16_t)(sign | (uint16_t)(expo << 7) | (uint16_t)(r >> 12 & 0x7Fu));
}
static void* xmalloc(size_t n) {
    void* p = malloc(n ? n : 1);
    if (!p) exit(3);
    return p;
}

static int run_case(int64_t M, int64_t N, int64_t K, int64_t r, int64_t ld_extra) {
    const int64_t kl = K - r, ldx = K + ld_extra, ldw = K + ld_extra;
    uint16_t* x = xmalloc((size_t)(M * ldx) * 2);
    uint16_t* w = xmalloc((size_t)(N * ldw) * 2);
    for (int64_t i = 0; i < M * ldx; ++i) x[i] = rand_bf16();
    for (int64_t i = 0; i < N * ldw; ++i) w[i] = rand_bf16();
    for (int64_t k = 0; k < K; ++k) x[k] = 0;                 /* an all-zero token */
    int8_t* q_hi = xmalloc((size_t)(M * r));
    int8_t* q_lo = xmalloc((size_t)(M * kl));
    float* s_hi = xmalloc((size_t)M * 4);
    float* s_lo = xmalloc((size_t)M * 4);
    oracle_quantize_act(x, ldx, M, K, r, q_hi, q_lo, s_hi, s_lo);
    int bad = 0;
    for (int64_t i = 0; i < M * r; ++i) bad |= q_hi[i] < -QMAX_H;   /* -128 is never a code */
    for (int64_t i = 0; i < M * kl; ++i) bad |= q_lo[i] < -QMAX_L || q_lo[i] > QMAX_L;

    uint8_t* u_hi = xmalloc((size_t)(M * r));
    uint8_t* u_lo = xmalloc((size_t)(M * kl));
    float* t_hi = xmalloc((size_t)M * 4);
    float* t_lo = xmalloc((size_t)M * 4);
    float* z_hi = xmalloc((size_t)M * 4);
    float* z_lo = xmalloc((size_t)M * 4);
    oracle_quantize_act_asym(x, ldx, M, K, r, u_hi, u_lo, t_hi, t_lo, z_hi, z_lo);
    for (int64_t i = 0; i < M * kl; ++i) bad |= u_lo[i] > 15;

    int8_t* w_hi = xmalloc((size_t)(N * r));
    int8_t* w_lo = xmalloc((size_t)(N * kl));
    uint16_t* sw_hi = xmalloc((size_t)N * 2);
    uint16_t* sw_lo = xmalloc((size_t)N * 2);
    oracle_quantize_weights(w, ldw, N, K, r, w_hi, w_lo, sw_hi, sw_lo);
    for (int64_t i = 0; i < N * kl; ++i) bad |= w_lo[i] < -QMAX_L || w_lo[i] > QMAX_L;

    if (kl > 0) {
        const int64_t ld_out = kl / 2 + 3;
        uint8_t* packed = xmalloc((size_t)(M * ld_out));
        oracle_pack_nibbles(q_lo, M, kl, ld_out, packed);
        int32_t* sums = xmalloc((size_t)M * 4);
        oracle_odd_code_sums(q_lo, M, kl, sums);
        free(packed);
        free(sums);
    }
    int64_t* a_hi = r > 0 ? xmalloc((size_t)(M * N) * 8) : NULL;
    int64_t* a_lo = kl > 0 ? xmalloc((size_t)(M * N) * 8) : NULL;
    int64_t over = 0;
    if (r > 0) over += oracle_gemm_i64(q_hi, r, w_hi, r, M, N, r, a_hi);
    if (kl > 0) over += oracle_gemm_i64(q_lo, kl, w_lo, kl, M, N, kl, a_lo);
    bad |= over != 0;
    double* y = xmalloc((size_t)(M * N) * 8);
    oracle_dequant(a_hi, a_lo, s_hi, s_lo, sw_hi, sw_lo, M, N, y);
    uint16_t* yb = xmalloc((size_t)(M * N) * 2);
    oracle_round_bf16(y, M * N, yb);

    int64_t* ws_hi = xmalloc((size_t)N * 8);
    int64_t* ws_lo = xmalloc((size_t)N * 8);
    for (int64_t n = 0; n < N; ++n) {
        ws_hi[n] = ws_lo[n] = 0;
        for (int64_t k = 0; k < r; ++k) ws_hi[n] += w_hi[n * r + k];
        for (int64_t k = 0; k < kl; ++k) ws_lo[n] += w_lo[n * kl + k];
    }
    if (r > 0) oracle_gemm_u8i8_i64(u_hi, r, w_hi, r, M, N, r, a_hi);
    if (kl > 0) oracle_gemm_u8i8_i64(u_lo, kl, w_lo, kl, M, N, kl, a_lo);
    oracle_dequant_asym(a_hi, a_lo, t_hi, t_lo, z_hi, z_lo, ws_hi, ws_lo, sw_hi, sw_lo, M, N, y);

    /* the transform on the low columns, block = largest power of two dividing their number */
    if (kl > 0) {
        int64_t b = kl & (-kl);
        uint16_t* xr = xmalloc((size_t)(M * ldx) * 2);
        for (int64_t i = 0; i < M * ldx; ++i) xr[i] = 0;
        oracle_hadamard(x, xr, ldx, M, K, r, K, b);
        free(xr);
    }
    free(x); free(w); free(q_hi); free(q_lo); free(s_hi); free(s_lo); free(u_hi); free(u_lo);
    free(t_hi); free(t_lo); free(z_hi); free(z_lo); free(w_hi); free(w_lo); free(sw_hi); free(sw_lo);
    free(a_hi); free(a_lo); free(y); free(yb); free(ws_hi); free(ws_lo);
    return bad;
}

int main(void) {
    int bad = 0;
    bad |= run_case(16, 256, 256, 32, 0);     /* the tiny configuration */
    bad |= run_case(5, 7, 90, 30, 6);         /* ragged, strided rows */
    bad |= run_case(3, 9, 64, 0, 0);          /* uniform INT4 */
    bad |= run_case(3, 9, 64, 64, 2);         /* uniform INT8 */
    bad |= run_case(1, 1, 2, 0, 0);           /* the smallest legal layer */
    bad |= run_case(2, 17, 520, 8, 8);
    if (oracle_num_threads() < 1) bad = 1;
    printf(bad ? "oracle sanitizer check: FAILED\n" : "oracle sanitizer check: clean\n");
    return bad ? 1 : 0;
}
