// Data layout of the quantized operands in HBM, shared by every kernel of the
// library (and by nothing else).
//
// Activation codes (written by the quantize kernel, read by the GEMMs) are
// plain row-major per token:
//   q_hi  int8  [M, kh_pad]      kh_pad = round_up(r, 128)
//   q_lo  uint8 [M, kl_pad / 2]  kl_pad = round_up(K - r, 256), two nibbles per
//                                byte, even column in bits 0..3
// Padding codes are zero.
//
// Packed weights are tiled for the 16x16x64 int8 matrix-core instruction.  Its
// operand register holds, in lane l, 16 consecutive bytes of the reduction axis
// for row (l % 16), sub-chunk (l / 16).  A "chunk" is the 1 KiB image of one
// such operand: 16 weight rows x 64 bytes, stored sub-chunk-major,
//   byte offset = ((kc * 16) + row) * 16 + byte,   kc in 0..3, row in 0..15,
// so that a wavefront reads it with one fully coalesced 16-byte-per-lane load
// (lane l reads offset 16 * l) straight into operand registers or into LDS.
// A chunk of the high group covers 64 int8 codes per row, a chunk of the low
// group 128 nibble codes per row (byte j of a row's 64 holds codes 2j, 2j+1,
// as in the activation rows).
//
// The buffer is
//   for each block of 16 output channels (n_pad / 16 of them):
//       kh_pad / 64 high chunks, then kl_pad / 128 low chunks
//   fp16 sw_hi[n_pad], fp16 sw_lo[n_pad]
// with n_pad = round_up(N, 256); padding rows hold zero codes and scale 1.
#pragma once
#include <stdint.h>

namespace resq {

constexpr int kQmaxHi = 127;  // 2^(8-1) - 1  (Section 3, Eq. 1, N = 8)
constexpr int kQmaxLo = 7;    // 2^(4-1) - 1  (Section 3, Eq. 1, N = 4)

constexpr int kHiPad = 128;     // codes; one LDS stage of the tiled GEMM = 128 bytes per row
constexpr int kLoPad = 256;     // codes (= 128 bytes per row)
constexpr int kNPad = 256;      // output channels; the widest GEMM tile
constexpr int kRowsPerBlock = 16;
constexpr int kChunkBytes = 1024;

__host__ __device__ inline int64_t round_up(int64_t a, int64_t b) { return (a + b - 1) / b * b; }

struct WeightLayout {
    int64_t N, K, r;
    int64_t kh_pad, kl_pad, n_pad;
    int64_t hi_chunks, lo_chunks;  // per 16-row block
    int64_t block_bytes;           // bytes of one 16-row block
    int64_t scale_off;             // byte offset of sw_hi; sw_lo follows at + 2 * n_pad
    int64_t total_bytes;
};

__host__ __device__ inline WeightLayout make_weight_layout(int64_t N, int64_t K, int64_t r) {
    WeightLayout L;
    L.N = N; L.K = K; L.r = r;
    L.kh_pad = round_up(r, kHiPad);
    L.kl_pad = round_up(K - r, kLoPad);
    L.n_pad = round_up(N, kNPad);
    L.hi_chunks = L.kh_pad / 64;
    L.lo_chunks = L.kl_pad / 128;
    L.block_bytes = (L.hi_chunks + L.lo_chunks) * kChunkBytes;
    L.scale_off = (L.n_pad / kRowsPerBlock) * L.block_bytes;
    L.total_bytes = L.scale_off + 4 * L.n_pad;
    return L;
}

// byte offset of the 16-byte unit holding, for output channel n, bytes
// [16 * u, 16 * u + 16) of its padded high row (u counts 16-byte units)
__host__ __device__ inline int64_t hi_unit_offset(const WeightLayout& L, int64_t n, int64_t u) {
    return (n / kRowsPerBlock) * L.block_bytes + (u / 4) * kChunkBytes +
           ((u % 4) * 16 + (n % kRowsPerBlock)) * 16;
}
// same for the packed low row (unit u = bytes [16u, 16u+16) = codes [32u, 32u+32))
__host__ __device__ inline int64_t lo_unit_offset(const WeightLayout& L, int64_t n, int64_t u) {
    return (n / kRowsPerBlock) * L.block_bytes + (L.hi_chunks + u / 4) * kChunkBytes +
           ((u % 4) * 16 + (n % kRowsPerBlock)) * 16;
}

}  // namespace resq
