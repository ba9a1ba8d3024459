// Data layout of the quantized operands in HBM, shared by every kernel of the
// library (and by nothing else).
//
// Activation codes (written by the quantize kernel, read by the GEMMs) are
// plain row-major per token:
//   q_hi  int8  [M, kh_pad]      kh_pad = round_up(r, 128)
//   q_lo  uint8 [M, kl_pad / 2]  kl_pad = round_up(K - r, 256), two nibbles per
//                                byte: bits 0..3 = code of the even column + 8,
//                                bits 4..7 = code of the odd column (two's
//                                complement)
// Padding codes are zero (a padding byte of q_lo is 0x08).
//
// Packed weights use the same two row formats, cut into blocks that a GEMM
// stage consumes whole: a "block" is 16 output channels x 64 bytes of one
// group's row (64 int8 codes of the high group, or 128 nibble codes of the low
// group), row-major, 1 KiB, contiguous in HBM: exactly one operand of the
// 16x16x64 matrix-core instruction, or half of a 32x32x32 one.  The buffer is
//   for each group of 16 output channels (n_pad / 16 of them):
//       kh_pad / 64 high blocks, then kl_pad / 128 low blocks
//   fp16 sw_hi[n_pad], fp16 sw_lo[n_pad], int32 even_sum[n_pad]
// with n_pad = round_up(N, 256); padding rows hold zero codes and scale 1.
// A weight byte of the low group pairs the other way round than an activation
// byte: bits 4..7 = code of the even column (two's complement), bits 0..3 =
// code of the odd column + 8, so that every product of the widened nibbles
// pairs one offset operand with one signed operand (see resq_gemm.hip.h);
// even_sum[n] is the sum of channel n's low codes in even columns.
// So channel n, byte b of its padded high row lives at
//   (n / 16) * group_bytes + (b / 64) * 1024 + (n % 16) * 64 + b % 64
// and byte b of its packed low row at the same place past the high blocks.
#pragma once
#include <stdint.h>

namespace resq {

constexpr int kQmaxHi = 127;  // 2^(8-1) - 1  (Section 3, Eq. 1, N = 8)
constexpr int kQmaxLo = 7;    // 2^(4-1) - 1  (Section 3, Eq. 1, N = 4)

constexpr int kHiPad = 128;     // codes
constexpr int kLoPad = 256;     // codes (= 128 bytes per row)
constexpr int kNPad = 256;      // output channels; the widest GEMM tile
constexpr int kRowsPerBlock = 16;
constexpr int kRowBytes = 64;   // bytes of one row inside a block
constexpr int kBlockBytes = kRowsPerBlock * kRowBytes;  // 1024

__host__ __device__ inline int64_t round_up(int64_t a, int64_t b) { return (a + b - 1) / b * b; }

struct WeightLayout {
    int64_t N, K, r;
    int64_t kh_pad, kl_pad, n_pad;
    int64_t hi_blocks, lo_blocks;  // per group of 16 channels
    int64_t group_bytes;           // bytes of one group of 16 channels
    int64_t scale_off;             // byte offset of the per-channel constants, n_pad entries each:
                                   //   fp16 sw_hi at + 0, fp16 sw_lo at + 2 n_pad,
                                   //   int32 even_sum (low codes of even columns) at + 4 n_pad,
                                   //   int32 wsum_hi at + 8 n_pad, int32 wsum_lo at + 12 n_pad
                                   //   (sums of all codes of a group: the zero-point term of
                                   //   asymmetric activations)
    int64_t total_bytes;
};

__host__ __device__ inline WeightLayout make_weight_layout(int64_t N, int64_t K, int64_t r) {
    WeightLayout L;
    L.N = N; L.K = K; L.r = r;
    L.kh_pad = round_up(r, kHiPad);
    L.kl_pad = round_up(K - r, kLoPad);
    L.n_pad = round_up(N, kNPad);
    L.hi_blocks = L.kh_pad / kRowBytes;
    L.lo_blocks = L.kl_pad / (2 * kRowBytes);
    L.group_bytes = (L.hi_blocks + L.lo_blocks) * kBlockBytes;
    L.scale_off = (L.n_pad / kRowsPerBlock) * L.group_bytes;
    L.total_bytes = L.scale_off + 16 * L.n_pad;
    return L;
}

// byte offset of byte b of channel n's padded high row / packed low row
__host__ __device__ inline int64_t hi_byte_offset(const WeightLayout& L, int64_t n, int64_t b) {
    return (n / kRowsPerBlock) * L.group_bytes + (b / kRowBytes) * kBlockBytes +
           (n % kRowsPerBlock) * kRowBytes + b % kRowBytes;
}
__host__ __device__ inline int64_t lo_byte_offset(const WeightLayout& L, int64_t n, int64_t b) {
    return (n / kRowsPerBlock) * L.group_bytes + (L.hi_blocks + b / kRowBytes) * kBlockBytes +
           (n % kRowsPerBlock) * kRowBytes + b % kRowBytes;
}

}  // namespace resq
