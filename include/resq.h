/*
 * resq.h - C ABI of the MI355X (gfx950) ResQ mixed-precision linear layer.
 *
 * ResQ (arXiv 2412.14363) keeps r of the K input coefficients of a linear
 * layer in 8 bits and the other K - r in 4 bits, for activations and weights
 * alike, and evaluates the layer as two integer GEMMs between operands of the
 * same precision whose dequantized results are added (Section 4.1, Eq. 2-4).
 * This library is that inference path: per-token activation quantization,
 * offline weight quantization and packing, the fused two-GEMM kernel with its
 * dequantizing epilogue, and the online Hadamard transform of the down_proj
 * input (Section 4.3).
 *
 * Conventions common to every call
 *   - Columns [0, r) of the K axis are the high-precision (INT8) group, columns
 *     [r, K) the low-precision (INT4) group.  r = 0 and r = K are legal; the
 *     pointers of an empty group may be null.  K - r must be even.
 *   - The quantizer is the symmetric one of Section 3, Eq. 1: zero-point 0,
 *     scale = max|x| / (2^(N-1) - 1) over the group (127 for N = 8, 7 for
 *     N = 4), code = clip(round_half_even(x / scale)), fp32 IEEE division.
 *     A group that is all zero has scale 1.
 *   - Every pointer is a DEVICE pointer owned by the caller unless marked
 *     "host".  The library allocates nothing and never synchronizes: work is
 *     enqueued on `stream` (a hipStream_t passed as void*; null = the default
 *     stream) and results are ready when that stream reaches them.
 *   - Every function returns a resq_status.  Arguments are checked on the host
 *     before anything is launched; on any status other than RESQ_OK nothing
 *     was enqueued (RESQ_ERR_HIP excepted: the runtime refused a launch).
 *   - bf16 tensors are row-major with a leading dimension given in ELEMENTS.
 *   - Inputs are expected to be finite; NaN or infinity give unspecified codes.
 */
#ifndef RESQ_H
#define RESQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum resq_status {
    RESQ_OK = 0,
    RESQ_ERR_NULL = 1,   /* a required pointer is null                               */
    RESQ_ERR_SHAPE = 2,  /* M, N, K < 1, r outside [0, K], K - r odd, ld too small,
                            bad Hadamard block, size beyond a documented limit        */
    RESQ_ERR_ALIGN = 3,  /* a pointer or leading dimension breaks a stated alignment  */
    RESQ_ERR_BUFFER = 4, /* packed-weight buffer smaller than resq_packed_weight_bytes */
    RESQ_ERR_HIP = 5     /* the HIP runtime reported an error at launch               */
} resq_status;

/* Static, human-readable name of a status code (host pointer, never null). */
const char* resq_status_string(int status);

/*
 * Measurement aid: the next quantize, GEMM or Hadamard kernel that THIS host
 * thread launches through the library records the two events (hipEvent_t passed
 * as void*, created by the caller) exactly at the kernel's start and end, so
 * that hipEventElapsedTime(start, stop) is the kernel's own duration without
 * the gaps that events recorded around a launch include.  One-shot: the request
 * is consumed by that launch.  The helper kernels of resq_pack_weights and
 * resq_unpack_weights are not timed.
 */
int resq_time_next_kernel(void* start_event, void* stop_event);

/* ---- layout queries (pure host functions) ------------------------------- */

/*
 * Bytes per token row of the two activation code arrays written by
 * resq_quantize_act and read by resq_gemm_mixed.  High codes are int8, one per
 * byte, the row padded with zero codes to a multiple of 128 codes.  Low codes
 * are nibbles, two per byte: column r + 2j in bits 0..3 of byte j as code + 8
 * (offset binary, 1..15) and column r + 2j + 1 in bits 4..7 in two's
 * complement, so that each of the two can be widened for the int8 matrix cores
 * with a single AND; the row is padded with zero codes (bytes 0x08) to a
 * multiple of 256 codes.  Zero codes add nothing to Eq. 4's sums.  Both return
 * 0 for an empty group and -1 for an invalid (K, r).
 */
int64_t resq_act_hi_ld(int64_t K, int64_t r);
int64_t resq_act_lo_ld(int64_t K, int64_t r);

/*
 * Size in bytes of the packed weight buffer of an [N, K] layer with a high
 * group of width r; 0 for invalid arguments.  The layout is private to the
 * library (tiled for the matrix cores; read it back with resq_unpack_weights):
 * N is padded to a multiple of 256 rows, the high group to a multiple of 128
 * and the low group to a multiple of 256 codes, all with zero codes, followed
 * by two fp16 scale vectors and three int32 sums of codes per channel (16 bytes
 * per channel in all).
 */
size_t resq_packed_weight_bytes(int64_t N, int64_t K, int64_t r);

/*
 * Default block size of the online Hadamard transform over `width` columns:
 * the largest power of two that divides width, at most 8192 (Sylvester
 * Hadamard matrices exist only for powers of two, so a width such as
 * 12544 = 49 * 256 is covered by a block-diagonal transform, which is still
 * orthogonal).  Returns 0 for width < 1.
 */
int64_t resq_hadamard_block(int64_t width);

/* ---- the hot path -------------------------------------------------------- */

/*
 * Per-token mixed-precision activation quantization (Section 4.1 Eq. 2 with
 * the quantizer of Section 3 Eq. 1, per token as in Section 5.1).
 *   x      bf16 [M, ldx], ldx >= K                      (read)
 *   q_hi   int8  [M, resq_act_hi_ld(K, r)]              (written, padding zeroed)
 *   q_lo   uint8 [M, resq_act_lo_ld(K, r)]              (written, padding = zero codes)
 *   s_hi, s_lo   fp32 [M] scales of the two groups      (written)
 *   lo_sum int32 [M]: per token, the sum of the low codes of the odd columns
 *          r + 1, r + 3, ...                            (written)
 *          resq_gemm_mixed needs it to undo the offset of the nibbles that are
 *          stored as code + 8 (see resq_act_lo_ld)
 * One read of x; the absmax, the division, the rounding and the packing are
 * fused.  Alignment: none required; x 16-byte aligned with ldx, K and r
 * multiples of 8 selects the vectorized path.  q_hi and q_lo must be 16-byte
 * aligned.  Limits: K <= 2^20.
 */
int resq_quantize_act(const void* x, int64_t ldx, int64_t M, int64_t K, int64_t r,
                      int8_t* q_hi, uint8_t* q_lo, float* s_hi, float* s_lo, int32_t* lo_sum,
                      void* stream);

/*
 * The online Hadamard projection of the low group (Section 4.3, U_D; see
 * resq_online_hadamard) fused with resq_quantize_act: the codes, scales and
 * lo_sum are exactly those of
 *   resq_online_hadamard(x, t, ..., col_begin = r, col_end = K, block)
 *   resq_quantize_act(t, ...)
 * (same butterflies in the same order, same rounding of the rotated values to
 * bf16 before they are quantized), but the rotated row is not written to memory
 * and read back: one read of x in all.  Blocks of 256 (the Llama down_proj
 * inputs) take most of their sums on the bf16 matrix cores, in another order:
 * there a rotated value may be the neighbouring bf16 of the stand-alone
 * transform's (both within rounding of the exact transform), and the codes are
 * exactly those of resq_quantize_act on the rotated row that x_rot receives.
 *   block   power of two in [8, 512] dividing both r and K - r (a block is held
 *           by one wavefront); 0 selects resq_hadamard_block(K - r).  Other
 *           sizes: RESQ_ERR_SHAPE, use the two calls above.
 *   x_rot   null, or bf16 [M, ld_rot] (ld_rot >= K, 16-byte aligned, ld_rot a
 *           multiple of 8): receives columns [r, K) of the rotated rows, for
 *           inspection and parity checks; columns [0, r) are not touched.
 * Needs the vectorized path: x 16-byte aligned, ldx, K, r multiples of 8,
 * K <= 16384, or with blocks of 256 r <= 4096 and K - r <= 26624 (else
 * RESQ_ERR_ALIGN).  Other arguments as resq_quantize_act.
 */
int resq_hadamard_quantize_act(const void* x, int64_t ldx, int64_t M, int64_t K, int64_t r,
                               int64_t block, int8_t* q_hi, uint8_t* q_lo, float* s_hi,
                               float* s_lo, int32_t* lo_sum, void* x_rot, int64_t ld_rot,
                               void* stream);

/*
 * Per-token quantization with the ASYMMETRIC branch of Section 3 Eq. 1, the
 * setting of the paper's own experiments for activations (Section 5.1), applied
 * to each group separately:
 *   z = min(x), s = (max(x) - min(x)) / (2^N - 1), code = clip(round((x - z) / s), 0, 2^N - 1)
 * with x - z and the quotient in fp32 and the round half to even; a constant
 * group has s = 1.  Codes are STORED minus 2^(N-1) in the layouts of
 * resq_quantize_act (int8 for the high group; for the low group the plain code
 * 0..15 in bits 0..3 for even columns, a two's-complement nibble of code - 8 in
 * bits 4..7 for odd columns), so that the matrix cores see the operands they see
 * for symmetric codes; padding is the stored code 0.
 *   s_hi, s_lo   fp32 [M] scales                                     (written)
 *   c_hi, c_lo   fp32 [M]: z + 2^(N-1) s, the real value that the stored code 0
 *                stands for, i.e. x ~ stored * s + c                 (written)
 *   lo_sum       as in resq_quantize_act, over the stored values     (written)
 *   hadamard_block  0: none; > 0: the block Walsh-Hadamard transform of the low
 *                group first, in the same kernel, under the conditions of
 *                resq_hadamard_quantize_act; < 0: the same with the default block
 * Other arguments, alignment and limits as resq_quantize_act.  Feed the result
 * to resq_gemm_mixed_asym.
 */
int resq_quantize_act_asym(const void* x, int64_t ldx, int64_t M, int64_t K, int64_t r,
                           int64_t hadamard_block, int8_t* q_hi, uint8_t* q_lo, float* s_hi,
                           float* s_lo, float* c_hi, float* c_lo, int32_t* lo_sum, void* stream);

/*
 * resq_quantize_act_asym with the block Walsh-Hadamard transform of the low
 * group in front (the down_proj input with asymmetric codes, Sections 4.3 and
 * 5.1) and the optional inspection output of resq_hadamard_quantize_act:
 * block, x_rot, ld_rot as there, everything else as resq_quantize_act_asym.
 */
int resq_hadamard_quantize_act_asym(const void* x, int64_t ldx, int64_t M, int64_t K, int64_t r,
                                    int64_t block, int8_t* q_hi, uint8_t* q_lo, float* s_hi,
                                    float* s_lo, float* c_hi, float* c_lo, int32_t* lo_sum,
                                    void* x_rot, int64_t ld_rot, void* stream);

/*
 * Offline weight quantization and packing (Section 4.1 Eq. 3; per output
 * channel, symmetric, round-to-nearest, Section 5.1).
 *   w       bf16 [N, ldw], ldw >= K: (out_features, in_features)   (read)
 *   packed  resq_packed_weight_bytes(N, K, r) bytes, 256-byte aligned (written)
 * The per-channel scale of each group is stored as fp16, rounded toward +inf
 * from max|w| / qmax and clamped to [2^-14, 65504]; the codes are computed
 * with the stored value, so |w - code * scale| <= scale / 2 holds for it.
 * packed_bytes is the capacity of `packed`.
 */
int resq_pack_weights(const void* w, int64_t ldw, int64_t N, int64_t K, int64_t r,
                      void* packed, size_t packed_bytes, void* stream);

/*
 * Inverse of the packing, for inspection and parity checks: plain row-major
 * codes (one per byte) and the stored fp16 scale bit patterns.
 *   w_hi int8 [N, r]   w_lo int8 [N, K - r]   sw_hi, sw_lo uint16 [N]   (written)
 */
int resq_unpack_weights(const void* packed, int64_t N, int64_t K, int64_t r, int8_t* w_hi,
                        int8_t* w_lo, uint16_t* sw_hi, uint16_t* sw_lo, void* stream);

/*
 * The layer (Section 4.1 Eq. 4): for every token m and output channel n
 *   A_hi[m, n] = sum_{k <  r} q_hi[m, k] * w_hi[n, k]       (int8 x int8 -> int32)
 *   A_lo[m, n] = sum_{k >= r} q_lo[m, k] * w_lo[n, k]       (int4 x int4 -> int32)
 *   y[m, n]    = bf16( A_hi * s_hi[m] * sw_hi[n] + A_lo * s_lo[m] * sw_lo[n] )
 * Both sums run on the int8 matrix cores (nibbles are widened in registers)
 * inside one kernel; y is written once.  The integer sums are exact: the call
 * accepts r <= 132104 and K - r <= 2^20, so neither 128 * 127 * r (stored asymmetric
 * codes reach -128) nor the widened low sum 1680 * (K - r) can reach 2^31 (larger
 * groups: RESQ_ERR_SHAPE).
 *   q_hi, q_lo, s_hi, s_lo, lo_sum   as written by resq_quantize_act for the same K, r
 *   packed                   as written by resq_pack_weights for the same N, K, r
 *   y        bf16 [M, ldy], ldy >= N                         (written)
 *   dbg_acc_hi, dbg_acc_lo   int32 [M, N] each, or null: when given, the two
 *                            integer accumulators are written as well
 * Shapes with M <= 64 take weight-streaming kernels bound by HBM bandwidth
 * (the packed weights cross HBM once; the code rows of up to 16 tokens are
 * read as they are needed while they are short enough to stay in cache, else
 * and up to 64 tokens they are chunked through LDS; layers with
 * few output channels split the reduction axis over wavefronts), larger M the
 * tiled matrix-core kernel (128 x 128 tiles, or 64 x 128 where those are at
 * most 512), except that up to 1024 tokens go through the streaming kernel in
 * slices of 16 to 64 tokens where that is estimated faster (few tiles, each
 * walking the whole reduction axis alone); the integer accumulators are
 * identical.
 * Alignment: q_hi, q_lo 16 bytes; packed 256 bytes; y 2 bytes.
 */
int resq_gemm_mixed(const int8_t* q_hi, const uint8_t* q_lo, const float* s_hi,
                    const float* s_lo, const int32_t* lo_sum, int64_t M, const void* packed,
                    int64_t N, int64_t K,
                    int64_t r, void* y, int64_t ldy, int32_t* dbg_acc_hi, int32_t* dbg_acc_lo,
                    void* stream);

/*
 * Which kernel resq_gemm_mixed (and its variants) runs for a shape: host only,
 * no device call.  For callers that want to know, and for tests.
 *   kernel        0: weight-streaming kernel for at most 16 tokens
 *                 1: weight-streaming kernel with the activation codes chunked
 *                    through LDS, in slices of 16 * token_groups tokens (also
 *                    for 10 to 16 tokens on wide layers of 64 MB and more)
 *                 2: tiled matrix-core kernel, 128 x 128 tiles
 *                 3: tiled matrix-core kernel, 64 (tokens) x 128 tiles, where
 *                    those are at most 512                           (written)
 *   token_groups  1, 2 or 4 for kernel 1 (1 for kernel 0, 0 for kernels 2, 3) (written)
 *   runs          parts into which the reduction axis of a channel group (kernels
 *                 0, 1: 1..8) or of a tile (kernel 3: 2 where the tiles are at
 *                 most 256, else 1) is cut across wavefronts; 0 for kernel 2 (written)
 * Errors as resq_gemm_mixed for the shape; RESQ_ERR_NULL for a null output.
 */
int resq_gemm_mixed_plan(int64_t M, int64_t N, int64_t K, int64_t r, int* kernel, int* token_groups,
                         int* runs);

/*
 * The layer in ONE call for the generation stage (a handful of tokens, Section 1:
 * memory-bound): resq_quantize_act (Section 4.1 Eq. 2) and resq_gemm_mixed
 * (Eq. 4) in one kernel.  Every workgroup of the weight-streaming kernel
 * quantizes the M token rows itself, straight into the LDS rows that the kernel
 * reads its activation codes from, while its first weight blocks are on their
 * way: the codes never go to memory and the launch of the quantizer is saved.
 * y is bit-identical to the two calls (same quantizer arithmetic, same integer
 * sums, same epilogue).
 *   x        bf16 [M, ldx], ldx >= K                          (read)
 *   M        1..16 tokens whose code rows fit LDS (M * (padded row bytes) <=
 *            140 KiB; K = 8192 with r = 1024 takes 16), else RESQ_ERR_SHAPE: use
 *            the two calls
 *   packed, N, K, r, y, ldy   as in resq_gemm_mixed
 * Alignment: x 16 bytes and ldx, K, r multiples of 8 (else RESQ_ERR_ALIGN); packed
 * 256 bytes; y 2 bytes.  Symmetric codes, no gated epilogue, no debug outputs.
 */
int resq_quantize_gemm_mixed(const void* x, int64_t ldx, int64_t M, const void* packed, int64_t N,
                             int64_t K, int64_t r, void* y, int64_t ldy, void* stream);

/*
 * The gate and up projections of an MLP block as ONE layer with the gated
 * activation in its epilogue, so that the down_proj input (which Section 4.3
 * transforms and quantizes next) is written directly instead of two [M, F]
 * tensors that another kernel would read back:
 *   y[m, c] = bf16( silu(z[m, 2c]) * z[m, 2c + 1] ),  silu(x) = x / (1 + exp(-x)),
 * z the dequantized output of resq_gemm_mixed (in fp32, not rounded to bf16 in
 * between).  `packed` holds N2 = 2 F channels packed by resq_pack_weights from a
 * weight matrix whose rows 2c and 2c + 1 are the gate row and the up row of
 * feature c (the caller interleaves them); y is bf16 [M, ldy], ldy >= N2 / 2.
 * Symmetric activation codes; no accumulator dump.  Other arguments, alignment
 * and kernel choice as resq_gemm_mixed.
 */
int resq_gemm_mixed_swiglu(const int8_t* q_hi, const uint8_t* q_lo, const float* s_hi,
                           const float* s_lo, const int32_t* lo_sum, int64_t M, const void* packed,
                           int64_t N2, int64_t K, int64_t r, void* y, int64_t ldy, void* stream);

/*
 * Offline construction of the projection basis (Section 4.2), three steps.
 *
 * 1. The covariance (Gram) matrix of calibration activations, accumulated over
 *    calls:  c[i][j] += sum_t x[t][i] x[t][j]   (fp32 accumulation of exact bf16
 *    products on the fp32 matrix cores; the caller zeroes c before the first
 *    call).  When the token axis is cut over workgroups their sums meet by
 *    atomic adds, so the last bits depend on the order of arrival.
 *      x   bf16 [T, ldx], ldx >= K        (read)    T = 0 does nothing
 *      c   fp32 [K, ldc], ldc >= K        (read and written)
 *    Alignment: x 16 bytes, ldx % 8 == 0, K % 8 == 0 (else RESQ_ERR_ALIGN).
 */
int resq_gram_accumulate(const void* x, int64_t ldx, int64_t T, int64_t K, float* c, int64_t ldc,
                         void* stream);

/*
 * 2. PCA: eigenvalues and eigenvectors of the symmetric matrix c (its symmetric
 *    part is taken), by cyclic Jacobi rotations in fp64.  eigvals[k] decrease
 *    with k and column k of p is the unit eigenvector of eigvals[k], so that the
 *    high-precision subspace P_h of Section 4.2 (largest eigenvalues) is the
 *    first r columns, as this library's column convention wants it (the paper
 *    orders them increasingly and keeps the last r).  Signs of the vectors, and
 *    bases inside a repeated eigenvalue, are whatever the rotations give.
 *      c        fp32 [K, ldc]                        (read)
 *      K        even, 2 .. 8192 (else RESQ_ERR_SHAPE; two fp64 rows sit in LDS)
 *      sweeps   Jacobi sweeps, 1 .. 64.  Convergence is quadratic at the end: 12
 *               sweeps bring every off-diagonal element of a K = 4096 covariance
 *               below 2^-40 of its diagonal neighbours.  The count is fixed so
 *               that the call never has to wait for the device; sweeps after one
 *               that found nothing to rotate cost only their empty launches
 *      eigvals  fp32 [K]                             (written)
 *      p        fp32 [K, ldp], ldp >= K              (written)
 *      workspace  device memory, 256-byte aligned, resq_sym_eig_workspace_bytes(K)
 *               bytes (else RESQ_ERR_BUFFER); contents meaningless afterwards
 */
size_t resq_sym_eig_workspace_bytes(int64_t K);
int resq_sym_eig(const float* c, int64_t ldc, int64_t K, int sweeps, float* eigvals, float* p,
                 int64_t ldp, void* workspace, size_t workspace_bytes, void* stream);

/*
 * resq_sym_eig for callers that cannot allocate device memory and have no workspace to pass
 * (code under HIP graph capture, serving loops and harnesses that forbid hipMalloc, a basis
 * refreshed between requests): the same kernels on the same arguments, with the workspace in
 * a device array that is part of the library (4.2 MB on every GPU the library has run this
 * call on, held until the process ends).  The call allocates and frees nothing.
 *   K   even, 2 .. 512 (head-size and small hidden-size bases); larger: RESQ_ERR_BUFFER,
 *       nothing is launched
 * Results are those of resq_sym_eig bit for bit.  All calls on one GPU share the one array:
 * calls that overlap on a GPU (different streams or host threads) race, and its contents
 * after a call are meaningless (every call initializes what it reads).  RESQ_ERR_HIP if the
 * array's address cannot be obtained on the current device.
 */
int resq_sym_eig_static(const float* c, int64_t ldc, int64_t K, int sweeps, float* eigvals, float* p,
                        int64_t ldp, void* stream);

/*
 * 3. Rows expressed in a basis:  out[i][j] = sum_k a[i][k] u[k][j]  (fp32
 *    accumulation on the fp32 matrix cores).  This one product serves every
 *    remaining step: U_h = P_h R_h and U_l = P_l R_l (the definition of U in
 *    Section 4.2: a = a column block of p, u = a random orthogonal matrix passed
 *    in by the caller, out = a column block of U), the folding of U into the
 *    weights W U (Section 4.3; W as [out_features, in_features]) and the
 *    projection X U of activations.
 *      a    bf16 or fp32 (a_is_bf16) [rows, lda], lda >= K      (read)
 *      u    fp32 [K, ldu], ldu >= J                             (read)
 *      out  bf16 (rounded to nearest even) or fp32 (out_is_bf16) [rows, ldo], ldo >= J
 *    Alignment: a, u 16 bytes; lda % 8 == 0, ldu % 8 == 0, J % 8 == 0.  rows = 0
 *    does nothing.
 */
int resq_project_rows(const void* a, int a_is_bf16, int64_t lda, int64_t rows, int64_t K,
                      const float* u, int64_t ldu, int64_t J, void* out, int out_is_bf16,
                      int64_t ldo, void* stream);

/*
 * The online projection of queries and keys onto the basis of the K/V cache
 * (Section 4.3: after the position embedding each head is multiplied by the
 * d_head x d_head matrix U_C, with 8-bit weights and 8-bit activations), as one
 * kernel: every row of x (one head of one token) is quantized to INT8 with its
 * own symmetric scale (Section 3 Eq. 1), multiplied by the INT8 codes of U_C
 * and dequantized (Section 4.1 Eq. 4 with every column in the high group).
 * The result equals resq_quantize_act followed by resq_gemm_mixed with
 * K = N = r = d_head; the activation codes never go to memory.
 *   x        bf16 [rows, ldx], ldx >= d_head                 (read)
 *   rows     tokens x heads; 0 is allowed and does nothing (no pointer is looked at)
 *   d_head   64 or 128 (else RESQ_ERR_SHAPE: use the two calls above)
 *   packed   resq_pack_weights of the [d_head, d_head] matrix whose row n is
 *            column n of U_C (the weight of output channel n), r = d_head
 *   y        bf16 [rows, ldy], ldy >= d_head                 (written)
 * Alignment: x 16 bytes and ldx % 8 == 0 (else RESQ_ERR_ALIGN); packed 256
 * bytes; y 2 bytes (rows aligned to d_head / 8 bytes are written with wider stores).
 */
int resq_project_heads(const void* x, int64_t ldx, int64_t rows, int64_t d_head, const void* packed,
                       void* y, int64_t ldy, void* stream);

/*
 * The layer for asymmetric activation codes (resq_quantize_act_asym): inserting
 * x ~ stored * s + c (Section 3 Eq. 1) and w ~ code * sw into Section 4.1 Eq. 4
 * gives, per group,
 *   y[m, n] += sw[n] * ( s[m] * A[m, n] + c[m] * wsum[n] ),
 * A the integer sum over the stored codes (what dbg_acc_* receive) and wsum[n]
 * the sum of channel n's weight codes of that group, which resq_pack_weights
 * keeps in the packed buffer.  Same kernels as resq_gemm_mixed plus one
 * multiply-add per group in the epilogue; all other arguments as there.
 */
int resq_gemm_mixed_asym(const int8_t* q_hi, const uint8_t* q_lo, const float* s_hi,
                         const float* s_lo, const float* c_hi, const float* c_lo,
                         const int32_t* lo_sum, int64_t M, const void* packed, int64_t N, int64_t K,
                         int64_t r, void* y, int64_t ldy, int32_t* dbg_acc_hi, int32_t* dbg_acc_lo,
                         void* stream);

/*
 * Mixed-precision K/V cache entries (Section 5.1 and Appendix C: keys and values are
 * quantized per head with the asymmetric quantizer of Section 3, Eq. 1, an eighth of the
 * channels of a head in 8 bits, the rest in 4), in a compact row per head of a token:
 *   bytes [0, r)                      8-bit codes 0..255 of channels [0, r)
 *   bytes [r, r + (d_head - r) / 2)   4-bit codes 0..15: channel r + 2j in bits 0..3 of
 *                                     byte j, channel r + 2j + 1 in bits 4..7
 *   then fp32 s_hi, z_hi, s_lo, z_lo  scale and zero-point of both groups: a reader
 *                                     reconstructs x ~ code * s + z (a group without
 *                                     channels has s = 1, z = 0)
 * resq_kv_cache_row_bytes = r + (d_head - r) / 2 + 16 (88 bytes for d_head = 128, r = 16,
 * against 256 bytes of bf16), or 0 for an invalid pair.  Codes, scales and zero-points are
 * those of resq_quantize_act_asym on rows of d_head columns (z = min, s = (max - min) /
 * (2^N - 1), round half to even), stored here as Eq. 1 defines them.
 *   x       bf16 [rows, ldx], ldx >= d_head; one row per token and head       (read / written)
 *   cache   [rows, row_bytes] bytes, row_bytes >= resq_kv_cache_row_bytes     (written / read)
 *   d_head  multiple of 8, 8 .. 512; r multiple of 8, 0 .. d_head (else RESQ_ERR_SHAPE);
 *           rows = 0 does nothing
 * resq_dequantize_kv_cache is the reader: x[m, k] = bf16(code * s + z), the multiply-add in
 * fp32.  Errors: RESQ_ERR_BUFFER for a row_bytes too small; RESQ_ERR_ALIGN unless x is
 * 16-byte aligned, ldx % 8 == 0, cache 4-byte aligned and row_bytes % 4 == 0.
 */
size_t resq_kv_cache_row_bytes(int64_t d_head, int64_t r);
int resq_quantize_kv_cache(const void* x, int64_t ldx, int64_t rows, int64_t d_head, int64_t r, void* cache,
                           int64_t row_bytes, void* stream);
int resq_dequantize_kv_cache(const void* cache, int64_t row_bytes, int64_t rows, int64_t d_head, int64_t r,
                             void* x, int64_t ldx, void* stream);

/*
 * Online Hadamard projection of the down_proj input (Section 4.3, U_D):
 *   y[m, c0 + g*b + j] = (1/sqrt(b)) * sum_i x[m, c0 + g*b + i] * H_b[i, j]
 * for each block g of b columns in [col_begin, col_end), H_b the Sylvester
 * (natural-order) Hadamard matrix; other columns are copied.  fp32 butterflies,
 * bf16 in and out; y may alias x (in place).
 *   x, y   bf16 [M, ld], ld >= K
 *   block  power of two dividing col_end - col_begin, <= 8192;
 *          0 selects resq_hadamard_block(col_end - col_begin)
 * Errors: RESQ_ERR_ALIGN unless x and y are 16-byte aligned and ld, col_begin and
 * col_end - col_begin are multiples of 8 (rows are moved 16 bytes per lane).
 */
int resq_online_hadamard(const void* x, void* y, int64_t ld, int64_t M, int64_t K,
                         int64_t col_begin, int64_t col_end, int64_t block, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* RESQ_H */
