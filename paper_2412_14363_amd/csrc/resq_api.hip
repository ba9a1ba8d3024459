// C ABI of the library: argument checks on the host, then kernel launches on
// the caller's stream.  See include/resq.h for the contract of every entry.
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

#include <atomic>

#include "resq.h"
#include "resq_decode.hip.h"
#include "resq_eig.hip.h"
#include "resq_gemm.hip.h"
#include "resq_gemm_m64.hip.h"
#include "resq_basis.hip.h"
#include "resq_hadamard.hip.h"
#include "resq_headproj.hip.h"
#include "resq_layout.h"
#include "resq_quantize.hip.h"

using namespace resq;

namespace {

constexpr int64_t kMaxK = 1 << 20;
constexpr int64_t kMaxLoWidth = 1 << 20;  // 1680 * (K - r) < 2^31 (widened low sums)
constexpr int64_t kMaxHiWidth = 132104;  // 128 * 127 * r < 2^31 (stored asymmetric codes reach -128)

inline bool aligned(const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

inline int shape_ok(int64_t rows, int64_t K, int64_t r) {
    if (rows < 1 || K < 1 || K > kMaxK || r < 0 || r > K) return 0;
    if ((K - r) % 2 != 0) return 0;
    if (rows > 0x7FFFFFFF) return 0;
    return 1;
}

inline int launch_status() { return hipGetLastError() == hipSuccess ? RESQ_OK : RESQ_ERR_HIP; }

// One-shot timing request of resq_time_next_kernel(): the next main kernel this
// thread launches is bracketed by the two events (exact kernel start and end).
thread_local hipEvent_t g_time_start = nullptr, g_time_stop = nullptr;

template <typename... KArgs, typename... Args>
inline void launch(void (*kernel)(KArgs...), dim3 grid, dim3 block, size_t lds, hipStream_t st, Args... args) {
    hipEvent_t e0 = g_time_start, e1 = g_time_stop;
    g_time_start = g_time_stop = nullptr;
    hipExtLaunchKernelGGL(kernel, grid, block, lds, st, e0, e1, 0, args...);
}

// ---- built-in scratch area of resq_sym_eig_static -------------------------------------------
// Largest order it serves, and the bytes that order needs (the layout of
// resq_sym_eig_workspace_bytes: matrix and transposed vectors in fp64, the round's rotations
// and pairs, the per-sweep counters).
constexpr int64_t kEigStaticMaxOrder = 512;
constexpr size_t kEigStaticBytes = 2 * (size_t)kEigStaticMaxOrder * kEigStaticMaxOrder * sizeof(double) +
                                   (size_t)kEigStaticMaxOrder * sizeof(double) + 256 +
                                   (size_t)kEigStaticMaxOrder * sizeof(int) + 256 + kEigMaxSweeps * sizeof(int) + 256;
static __device__ __align__(256) unsigned char g_eig_scratch[kEigStaticBytes];

// The array's name is a host-side stand-in; its device address differs per GPU and is looked
// up once per device, with that device current, and kept.
constexpr int kMaxDevices = 64;
std::atomic<void*> g_eig_scratch_addr[kMaxDevices];

void* eig_scratch_on_current_device() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    void* ptr = g_eig_scratch_addr[dev].load(std::memory_order_acquire);
    if (ptr) return ptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(g_eig_scratch)) != hipSuccess || !ptr) return nullptr;
    g_eig_scratch_addr[dev].store(ptr, std::memory_order_release);   // every thread finds the same address
    return ptr;
}

}  // namespace

extern "C" {

const char* resq_status_string(int status) {
    switch (status) {
        case RESQ_OK: return "RESQ_OK";
        case RESQ_ERR_NULL: return "RESQ_ERR_NULL: a required pointer is null";
        case RESQ_ERR_SHAPE: return "RESQ_ERR_SHAPE: invalid sizes, group width or leading dimension";
        case RESQ_ERR_ALIGN: return "RESQ_ERR_ALIGN: pointer or leading dimension misaligned";
        case RESQ_ERR_BUFFER: return "RESQ_ERR_BUFFER: packed weight buffer, workspace or built-in scratch area too small";
        case RESQ_ERR_HIP: return "RESQ_ERR_HIP: the HIP runtime refused the launch";
        default: return "unknown resq status";
    }
}

int resq_time_next_kernel(void* start_event, void* stop_event) {
    if (!start_event || !stop_event) return RESQ_ERR_NULL;
    g_time_start = static_cast<hipEvent_t>(start_event);
    g_time_stop = static_cast<hipEvent_t>(stop_event);
    return RESQ_OK;
}

int64_t resq_act_hi_ld(int64_t K, int64_t r) {
    if (K < 1 || r < 0 || r > K || (K - r) % 2 != 0) return -1;
    return round_up(r, kHiPad);
}

int64_t resq_act_lo_ld(int64_t K, int64_t r) {
    if (K < 1 || r < 0 || r > K || (K - r) % 2 != 0) return -1;
    return round_up(K - r, kLoPad) / 2;
}

size_t resq_packed_weight_bytes(int64_t N, int64_t K, int64_t r) {
    if (!shape_ok(N, K, r)) return 0;
    return (size_t)make_weight_layout(N, K, r).total_bytes;
}

int64_t resq_hadamard_block(int64_t width) {
    if (width < 1) return 0;
    int64_t b = width & (-width);
    return b > 8192 ? 8192 : b;
}

// shared by the four activation quantizer entry points: rot.log2b == 0 means no
// rotation, c_hi == c_lo == null the symmetric quantizer
static int quantize_act_impl(const void* x, int64_t ldx, int64_t M, int64_t K, int64_t r,
                             int8_t* q_hi, uint8_t* q_lo, float* s_hi, float* s_lo,
                             int32_t* lo_sum, const RotateArgs& rot, bool asym, float* c_hi,
                             float* c_lo, void* stream) {
    if (!shape_ok(M, K, r) || ldx < K) return RESQ_ERR_SHAPE;
    if (!x) return RESQ_ERR_NULL;
    if (r > 0 && (!q_hi || !s_hi || (asym && !c_hi))) return RESQ_ERR_NULL;
    if (K - r > 0 && (!q_lo || !s_lo || !lo_sum || (asym && !c_lo))) return RESQ_ERR_NULL;
    if (!aligned(x, 2) || !aligned(q_hi, 16) || !aligned(q_lo, 16) || !aligned(s_hi, 4) ||
        !aligned(s_lo, 4) || !aligned(lo_sum, 4) || !aligned(c_hi, 4) || !aligned(c_lo, 4))
        return RESQ_ERR_ALIGN;
    const int64_t ld_hi = round_up(r, kHiPad), ld_lo = round_up(K - r, kLoPad) / 2;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const uint16_t* xp = static_cast<const uint16_t*>(x);
    const dim3 block(kQuantThreads), grid((unsigned)M);
    const bool vec = aligned(x, 16) && ldx % 8 == 0 && K % 8 == 0 && r % 8 == 0 && K <= 16384;
    const bool rotate = rot.log2b > 0;
#define RESQ_QA_ARGS xp, ldx, (int)K, (int)r, q_hi, ld_hi, q_lo, ld_lo, s_hi, s_lo, lo_sum
    // blocks of 256: the first five butterfly stages on the matrix cores
    if (rot.log2b == 8 && aligned(x, 16) && ldx % 8 == 0 && r <= 4096 && K - r <= 13 * 2048) {
#define RESQ_LAUNCH_H256(HI, LO)                                                                    \
    do {                                                                                            \
        if (asym)                                                                                   \
            launch(hadamard256_quantize_kernel<HI, LO, true>, grid, block, 0, st, RESQ_QA_ARGS, rot, c_hi, c_lo);  \
        else                                                                                        \
            launch(hadamard256_quantize_kernel<HI, LO, false>, grid, block, 0, st, RESQ_QA_ARGS, rot, c_hi, c_lo); \
    } while (0)
        if (r <= 2048 && K - r <= 2 * 2048) RESQ_LAUNCH_H256(1, 2);
        else if (r <= 2048 && K - r <= 7 * 2048) RESQ_LAUNCH_H256(1, 7);
        else RESQ_LAUNCH_H256(2, 13);
#undef RESQ_LAUNCH_H256
        return launch_status();
    }
    if (rotate && !vec) return RESQ_ERR_ALIGN;
#define RESQ_LAUNCH_QA(ITERS)                                                                       \
    do {                                                                                            \
        if (rotate && asym)                                                                         \
            launch(quantize_act_vec_kernel<ITERS, true, true>, grid, block, 0, st, RESQ_QA_ARGS, rot, c_hi, c_lo);   \
        else if (rotate)                                                                            \
            launch(quantize_act_vec_kernel<ITERS, true, false>, grid, block, 0, st, RESQ_QA_ARGS, rot, c_hi, c_lo);  \
        else if (asym)                                                                              \
            launch(quantize_act_vec_kernel<ITERS, false, true>, grid, block, 0, st, RESQ_QA_ARGS, rot, c_hi, c_lo);  \
        else                                                                                        \
            launch(quantize_act_vec_kernel<ITERS, false, false>, grid, block, 0, st, RESQ_QA_ARGS, rot, c_hi, c_lo); \
    } while (0)
    if (vec && K <= 512 && !rotate) {
        // short rows (an attention head of a K/V cache entry): 16, 32 or 64 lanes per row
#define RESQ_LAUNCH_SHORT(G)                                                                       \
    do {                                                                                           \
        const dim3 grid_s((unsigned)((M + kQuantThreads / G - 1) / (kQuantThreads / G)));          \
        if (asym)                                                                                  \
            launch(quantize_act_short_kernel<true, G>, grid_s, block, 0, st, xp, ldx, M, (int)K,   \
                   (int)r, q_hi, ld_hi, q_lo, ld_lo, s_hi, s_lo, lo_sum, c_hi, c_lo);              \
        else                                                                                       \
            launch(quantize_act_short_kernel<false, G>, grid_s, block, 0, st, xp, ldx, M, (int)K,  \
                   (int)r, q_hi, ld_hi, q_lo, ld_lo, s_hi, s_lo, lo_sum, c_hi, c_lo);              \
    } while (0)
        if (K <= 128) RESQ_LAUNCH_SHORT(16);
        else if (K <= 256) RESQ_LAUNCH_SHORT(32);
        else RESQ_LAUNCH_SHORT(64);
#undef RESQ_LAUNCH_SHORT
    } else if (vec) {
        if (K <= 2048) RESQ_LAUNCH_QA(1);
        else if (K <= 4096) RESQ_LAUNCH_QA(2);
        else if (K <= 8192) RESQ_LAUNCH_QA(4);
        else RESQ_LAUNCH_QA(8);
    } else if (asym) {
        launch(quantize_act_generic_kernel<true>, grid, block, 0, st, RESQ_QA_ARGS, c_hi, c_lo);
    } else {
        launch(quantize_act_generic_kernel<false>, grid, block, 0, st, RESQ_QA_ARGS, c_hi, c_lo);
    }
#undef RESQ_LAUNCH_QA
#undef RESQ_QA_ARGS
    return launch_status();
}

// checks the block of a fused rotation and fills rot; block == 0 selects the default
static int make_rotate_args(int64_t K, int64_t r, int64_t block, void* x_rot, int64_t ld_rot,
                            RotateArgs& rot) {
    const int64_t width = K - r;
    if (width < 1) return RESQ_ERR_SHAPE;
    if (block == 0) block = resq_hadamard_block(width);
    if (block < 8 || block > 512 || (block & (block - 1)) != 0 || width % block != 0 || r % block != 0)
        return RESQ_ERR_SHAPE;
    if (x_rot && ld_rot < K) return RESQ_ERR_SHAPE;
    if (x_rot && (!aligned(x_rot, 16) || ld_rot % 8 != 0)) return RESQ_ERR_ALIGN;
    rot.log2b = 0;
    while ((int64_t(1) << rot.log2b) < block) ++rot.log2b;
    rot.scale = 1.0f / sqrtf((float)block);
    rot.x_rot = static_cast<uint16_t*>(x_rot);
    rot.ld_rot = ld_rot;
    return RESQ_OK;
}

int resq_quantize_act(const void* x, int64_t ldx, int64_t M, int64_t K, int64_t r, int8_t* q_hi,
                      uint8_t* q_lo, float* s_hi, float* s_lo, int32_t* lo_sum, void* stream) {
    RotateArgs rot{0, 1.0f, nullptr, 0};
    return quantize_act_impl(x, ldx, M, K, r, q_hi, q_lo, s_hi, s_lo, lo_sum, rot, false, nullptr,
                             nullptr, stream);
}

int resq_hadamard_quantize_act(const void* x, int64_t ldx, int64_t M, int64_t K, int64_t r,
                               int64_t block, int8_t* q_hi, uint8_t* q_lo, float* s_hi,
                               float* s_lo, int32_t* lo_sum, void* x_rot, int64_t ld_rot,
                               void* stream) {
    if (!shape_ok(M, K, r)) return RESQ_ERR_SHAPE;
    RotateArgs rot;
    const int rc = make_rotate_args(K, r, block, x_rot, ld_rot, rot);
    if (rc != RESQ_OK) return rc;
    return quantize_act_impl(x, ldx, M, K, r, q_hi, q_lo, s_hi, s_lo, lo_sum, rot, false, nullptr,
                             nullptr, stream);
}

int resq_hadamard_quantize_act_asym(const void* x, int64_t ldx, int64_t M, int64_t K, int64_t r,
                                    int64_t block, int8_t* q_hi, uint8_t* q_lo, float* s_hi,
                                    float* s_lo, float* c_hi, float* c_lo, int32_t* lo_sum,
                                    void* x_rot, int64_t ld_rot, void* stream) {
    if (!shape_ok(M, K, r)) return RESQ_ERR_SHAPE;
    RotateArgs rot;
    const int rc = make_rotate_args(K, r, block, x_rot, ld_rot, rot);
    if (rc != RESQ_OK) return rc;
    return quantize_act_impl(x, ldx, M, K, r, q_hi, q_lo, s_hi, s_lo, lo_sum, rot, true, c_hi, c_lo,
                             stream);
}

int resq_quantize_act_asym(const void* x, int64_t ldx, int64_t M, int64_t K, int64_t r,
                           int64_t hadamard_block, int8_t* q_hi, uint8_t* q_lo, float* s_hi,
                           float* s_lo, float* c_hi, float* c_lo, int32_t* lo_sum, void* stream) {
    if (!shape_ok(M, K, r)) return RESQ_ERR_SHAPE;
    RotateArgs rot{0, 1.0f, nullptr, 0};
    if (hadamard_block != 0) {
        const int rc = make_rotate_args(K, r, hadamard_block < 0 ? 0 : hadamard_block, nullptr, 0, rot);
        if (rc != RESQ_OK) return rc;
    }
    return quantize_act_impl(x, ldx, M, K, r, q_hi, q_lo, s_hi, s_lo, lo_sum, rot, true, c_hi, c_lo,
                             stream);
}

static bool kv_cache_shape_ok(int64_t rows, int64_t d_head, int64_t r) {
    return rows >= 0 && rows <= 0x7FFFFFFF && d_head >= 8 && d_head <= 512 && d_head % 8 == 0 && r >= 0 &&
           r <= d_head && r % 8 == 0;
}

size_t resq_kv_cache_row_bytes(int64_t d_head, int64_t r) {
    if (!kv_cache_shape_ok(0, d_head, r)) return 0;
    return (size_t)(r + (d_head - r) / 2 + 16);
}

int resq_quantize_kv_cache(const void* x, int64_t ldx, int64_t rows, int64_t d_head, int64_t r, void* cache,
                           int64_t row_bytes, void* stream) {
    if (!kv_cache_shape_ok(rows, d_head, r) || ldx < d_head) return RESQ_ERR_SHAPE;
    if (row_bytes < (int64_t)resq_kv_cache_row_bytes(d_head, r)) return RESQ_ERR_BUFFER;
    if (rows == 0) return RESQ_OK;
    if (!x || !cache) return RESQ_ERR_NULL;
    if (!aligned(x, 16) || ldx % 8 != 0 || !aligned(cache, 4) || row_bytes % 4 != 0) return RESQ_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const uint16_t* xp = static_cast<const uint16_t*>(x);
    uint8_t* cp = static_cast<uint8_t*>(cache);
#define RESQ_LAUNCH_KV(G)                                                                          \
    launch(quantize_kv_cache_kernel<G>, dim3((unsigned)((rows + kQuantThreads / G - 1) / (kQuantThreads / G))), \
           dim3(kQuantThreads), 0, st, xp, ldx, rows, (int)d_head, (int)r, cp, row_bytes)
    if (d_head <= 128) RESQ_LAUNCH_KV(16);
    else if (d_head <= 256) RESQ_LAUNCH_KV(32);
    else RESQ_LAUNCH_KV(64);
#undef RESQ_LAUNCH_KV
    return launch_status();
}

int resq_dequantize_kv_cache(const void* cache, int64_t row_bytes, int64_t rows, int64_t d_head, int64_t r,
                             void* x, int64_t ldx, void* stream) {
    if (!kv_cache_shape_ok(rows, d_head, r) || ldx < d_head) return RESQ_ERR_SHAPE;
    if (row_bytes < (int64_t)resq_kv_cache_row_bytes(d_head, r)) return RESQ_ERR_BUFFER;
    if (rows == 0) return RESQ_OK;
    if (!x || !cache) return RESQ_ERR_NULL;
    if (!aligned(x, 16) || ldx % 8 != 0 || !aligned(cache, 4) || row_bytes % 4 != 0) return RESQ_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const uint8_t* cp = static_cast<const uint8_t*>(cache);
    uint16_t* xp = static_cast<uint16_t*>(x);
#define RESQ_LAUNCH_KV(G)                                                                          \
    launch(dequantize_kv_cache_kernel<G>, dim3((unsigned)((rows + kQuantThreads / G - 1) / (kQuantThreads / G))), \
           dim3(kQuantThreads), 0, st, cp, row_bytes, rows, (int)d_head, (int)r, xp, ldx)
    if (d_head <= 128) RESQ_LAUNCH_KV(16);
    else if (d_head <= 256) RESQ_LAUNCH_KV(32);
    else RESQ_LAUNCH_KV(64);
#undef RESQ_LAUNCH_KV
    return launch_status();
}

int resq_pack_weights(const void* w, int64_t ldw, int64_t N, int64_t K, int64_t r, void* packed,
                      size_t packed_bytes, void* stream) {
    if (!shape_ok(N, K, r) || ldw < K) return RESQ_ERR_SHAPE;
    if (K - r > kMaxLoWidth || r > kMaxHiWidth) return RESQ_ERR_SHAPE;
    if (!w || !packed) return RESQ_ERR_NULL;
    if (!aligned(w, 2) || !aligned(packed, 256)) return RESQ_ERR_ALIGN;
    const WeightLayout L = make_weight_layout(N, K, r);
    if (packed_bytes < (size_t)L.total_bytes) return RESQ_ERR_BUFFER;
    hipLaunchKernelGGL(pack_weights_kernel, dim3((unsigned)L.n_pad), dim3(kQuantThreads), 0,
                       static_cast<hipStream_t>(stream), static_cast<const uint16_t*>(w), ldw, L,
                       static_cast<uint8_t*>(packed));
    return launch_status();
}

int resq_unpack_weights(const void* packed, int64_t N, int64_t K, int64_t r, int8_t* w_hi,
                        int8_t* w_lo, uint16_t* sw_hi, uint16_t* sw_lo, void* stream) {
    if (!shape_ok(N, K, r)) return RESQ_ERR_SHAPE;
    if (!packed) return RESQ_ERR_NULL;
    if (r > 0 && (!w_hi || !sw_hi)) return RESQ_ERR_NULL;
    if (K - r > 0 && (!w_lo || !sw_lo)) return RESQ_ERR_NULL;
    if (!aligned(packed, 256) || !aligned(sw_hi, 2) || !aligned(sw_lo, 2)) return RESQ_ERR_ALIGN;
    const WeightLayout L = make_weight_layout(N, K, r);
    hipLaunchKernelGGL(unpack_weights_kernel, dim3((unsigned)N), dim3(kQuantThreads), 0,
                       static_cast<hipStream_t>(stream), static_cast<const uint8_t*>(packed), L,
                       w_hi, w_lo, sw_hi, sw_lo);
    return launch_status();
}

// Which kernel resq_gemm_mixed runs for a shape, and with how many token groups per
// workgroup (TG) and runs per channel group (SK).
//   kernel 0: M <= 16 and code rows of at most 140 KiB in all: the weights stream once,
//             activation operands straight from the code rows (beyond that size the chunked
//             kernel reads them once per workgroup instead of once per wavefront); SK = runs
//             per group (layers with at most 1024 groups are cut until more than half of the
//             chip's 2048 wavefronts have a run, or a run would get shorter than 4 blocks).
//   kernel 1: a few tens of tokens, and up to 1024 of them where the tiled kernel would
//             leave most of the chip idle (few tiles, each walking the whole reduction axis
//             alone): the same single pass over the weights, activation codes chunked
//             through LDS, in slices of 16 TG tokens (each slice streams the weights for
//             itself, out of the last-level cache after the first).  TG and SK are the pair
//             with the lowest estimate from the measured costs of the kernel (constants
//             below), never less than one pass over the weights at 6 TB/s.
//   kernel 2: the tiled kernel on 128 x 128 tiles; a round of 512 tiles (two per compute
//             unit) costs 10 us + 0.5 us per block by the same measure.
//   kernel 3: the tiled kernel on 64 x 128 tiles, where those are at most 512 (one round);
//             SK = 2: eight wavefronts per tile in two rings (at most 256 tiles), else 1.
struct GemmPlan {
    int kernel, tg, sk;
};
// runs per channel group of the weight-streaming kernel for at most 16 tokens
static int decode_runs(const WeightLayout& L) {
    const int blocks = (int)(L.hi_blocks + L.lo_blocks);
    const int64_t groups = (L.N + 15) / 16;
    int sk = 1;
    while (sk < 8 && groups * sk <= 1024 && blocks / (2 * sk) >= 4) sk *= 2;
    return sk;
}
static GemmPlan plan_gemm(int64_t M, const WeightLayout& L) {
    const int blocks = (int)(L.hi_blocks + L.lo_blocks);
    const int64_t groups = (L.N + 15) / 16;
    const int64_t lds_row = L.kh_pad + L.kl_pad / 2 + kDecodeRowPad;
    if (M <= kDecodeMaxM && M * lds_row <= 140 * 1024) {
        const int sk = decode_runs(L);
        // From ten tokens on, a load of one block's codes straight from their rows touches so
        // many cache lines (one per token) that the chunked kernel, which brings the codes
        // through LDS, is faster on a wide layer too large for the caches (measured on 132 MB
        // of weights: 24.1 / 24.9 -> 22.6 us at M = 12 / 16, equal at M = 9; on a 38 MB layer
        // the plain kernel stays ahead at every M)
        const bool chunked = M >= 10 && sk == 1 && L.total_bytes >= (int64_t)64 << 20;
        if (!chunked) return {0, 1, sk};
    }
    int tg = 0, sk = 0;
    double stream_us = 0.0;
    if (M <= 16 * kStreamMaxM) {
        // Estimate per (token groups, runs): 1.9 us + rounds of 256 workgroups x (a fixed part + a
        // cost per 1 KiB block of a run), never less than one pass over the weights at 6 TB/s.
        // The constants are a least-squares fit to a sweep of all pairs over seven layer shapes and
        // M = 24..512 (on which this choice is the measured best or within 1 % of it).
        static const double kFixed[3][4] = {{1.46, 1.88, 0.31, 3.0}, {3.23, 4.72, 0.0, 0.0}, {4.62, 0.0, 0.0, 0.0}};
        static const double kPerBlock[3][4] = {{0.139, 0.146, 0.250, 0.45}, {0.170, 0.194, 0.0, 0.0}, {0.257, 0.0, 0.0, 0.0}};
        const double pass_us = (double)L.total_bytes / 6.0e6;
        for (int ti = 0; ti < 3; ++ti) {
            const int cand_tg = 1 << ti;
            const int64_t slices = (M + cand_tg * 16 - 1) / (cand_tg * 16);
            // pairs (2, 4) and (4, 2) were the measured best nowhere in that sweep: not built
            for (int si = 0; cand_tg == 1 ? si <= 3 : (cand_tg << si) <= 4; ++si) {
                const int cand_sk = 1 << si;
                // runs of at least two chunks, at most 2048 of them
                if (cand_sk > 1 && (groups * cand_sk > 2048 || blocks / cand_sk < 2 * kChunkBlocks)) break;
                const int64_t sets = (groups * cand_sk + 7) / 8;
                const int64_t wgs = (sets < 256 ? sets : 256) * slices;
                const int64_t rounds = ((wgs + 255) / 256) * ((sets + 255) / 256);
                double us = 1.9 + (double)rounds * (kFixed[ti][si] + kPerBlock[ti][si] * (double)(blocks / cand_sk));
                if (us < pass_us) us = pass_us;
                if (tg == 0 || us < stream_us) {
                    stream_us = us;
                    tg = cand_tg;
                    sk = cand_sk;
                }
            }
        }
    }
    // The tiled kernels: 64-token tiles where they fill at most one round of two workgroups per
    // compute unit (measured against 128-token tiles on the seven shapes of that sweep: 8 to 30 %
    // faster up to 384 such tiles, equal within 2 % up to 512, 10 to 25 % slower above); at most
    // one per compute unit: with both rings (a further 5 to 14 %)
    const int64_t tiles64 = ((M + kBM64 - 1) / kBM64) * ((L.N + kBN - 1) / kBN);
    const bool narrow = tiles64 <= 512;
    const int rings = narrow ? (tiles64 <= 256 ? 2 : 1) : 0;
    bool streaming = M <= kStreamMaxM;  // (measured: the streaming kernel is ahead or equal there on every shape)
    if (!streaming && tg != 0) {
        if (narrow) {
            // Fits to the sweep (within 10 %).  One ring: a workgroup alone on its compute unit
            // walks a stage in 0.21 us and slows down as more compute units stream; past 256 tiles
            // two workgroups share one.  Two rings: 0.14 us per stage.
            double tiled_us;
            if (rings == 2)
                tiled_us = 5.8 + 0.1435 * blocks + (0.5 + 0.08 * blocks) * (double)tiles64 / 256.0;
            else
                tiled_us = 6.9 + 0.258 * blocks + 0.18 * blocks * (double)(tiles64 - 256) / 256.0;
            // (the streaming estimate is up to 14 % low at four token groups)
            streaming = stream_us * (tg == 4 ? 1.12 : 1.0) < tiled_us;
        } else {
            // 512 tiles run at a time, two per compute unit
            const int64_t tiles = ((M + kBM - 1) / kBM) * ((L.N + kBN - 1) / kBN);
            const double tiled_us = (double)((tiles + 511) / 512) * (10.0 + 0.5 * (double)blocks);
            streaming = stream_us < 0.9 * tiled_us;
        }
    }
    if (streaming) return {1, tg, sk};
    return {narrow ? 3 : 2, 0, rings};
}

// arguments of the weight-streaming kernels; the code pointers are null when the kernel
// quantizes x itself
static DecodeArgs make_decode_args(const int8_t* q_hi, const uint8_t* q_lo, const float* s_hi,
                                   const float* s_lo, const float* c_hi, const float* c_lo,
                                   const int32_t* lo_sum, int64_t M, const void* packed,
                                   const WeightLayout& L, void* y, int64_t ldy, int32_t* dbg_acc_hi,
                                   int32_t* dbg_acc_lo, bool swiglu, int64_t lds_row) {
    DecodeArgs d;
    d.q_hi = reinterpret_cast<const uint8_t*>(q_hi);
    d.q_lo = q_lo;
    d.ld_hi = L.kh_pad;
    d.ld_lo = L.kl_pad / 2;
    d.s_hi = s_hi;
    d.s_lo = s_lo;
    d.lo_sum = lo_sum;
    d.c_hi = c_hi;
    d.c_lo = c_lo;
    d.packed = static_cast<const uint8_t*>(packed);
    d.L = L;
    d.M = (int)M;
    d.y = static_cast<uint16_t*>(y);
    d.ldy = ldy;
    d.dbg_hi = dbg_acc_hi;
    d.dbg_lo = dbg_acc_lo;
    d.swiglu = swiglu ? 1 : 0;
    d.groups = (int)((L.N + 15) / 16);
    d.lds_row = (int)lds_row;
    d.x = nullptr;
    d.ldx = 0;
    d.fuse_rows = 1;
    return d;
}

// The weight-streaming kernels for at most 16 tokens whose code rows fit LDS.  fused: the
// kernels quantize d.x themselves instead of reading codes.
static int launch_decode(const DecodeArgs& d, bool dbg, bool fused, hipStream_t st) {
    const WeightLayout& L = d.L;
    // the code rows go through LDS only when the kernel makes them itself
    const int sk = decode_runs(L);
    // the code rows go through LDS only when the kernel makes them itself
    int lds_bytes = fused ? ((d.M * d.lds_row + 15) & ~15) : 0;
    const int extra = fused ? kFusedScratchFloats * 4 : 0;
    const dim3 blk(kDecodeThreads);
#define RESQ_LAUNCH_DECODE(KERNEL, GRID)                                                           \
    do {                                                                                           \
        auto kernel = KERNEL;                                                                      \
        if (lds_bytes > 64 * 1024 &&                                                               \
            hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),                             \
                                hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes) != hipSuccess) \
            return RESQ_ERR_HIP;                                                                   \
        launch(kernel, GRID, blk, lds_bytes, st, d);                                               \
    } while (0)
    if (sk > 1) {
        lds_bytes += (kDecodeThreads / 64) * 2 * 64 * 16 + extra;   // the partial sums
        const int sets = (d.groups * sk + 7) / 8;
        const dim3 grid((unsigned)(sets < 256 ? sets : 256));
#define RESQ_LAUNCH_SPLITK(SK)                                                                     \
    do {                                                                                           \
        if (fused) RESQ_LAUNCH_DECODE((gemm_decode_splitk_kernel<false, SK, kActQuantize>), grid);  \
        else if (dbg) RESQ_LAUNCH_DECODE((gemm_decode_splitk_kernel<true, SK, kActDirect>), grid);  \
        else RESQ_LAUNCH_DECODE((gemm_decode_splitk_kernel<false, SK, kActDirect>), grid);          \
    } while (0)
        if (sk == 2) RESQ_LAUNCH_SPLITK(2);
        else if (sk == 4) RESQ_LAUNCH_SPLITK(4);
        else RESQ_LAUNCH_SPLITK(8);
#undef RESQ_LAUNCH_SPLITK
        return launch_status();
    }
    lds_bytes += extra;
    // one workgroup per compute unit (256 of them), fewer when there is less work
    const dim3 grid((unsigned)(d.groups < 256 ? d.groups : 256));
    if (fused) RESQ_LAUNCH_DECODE((gemm_decode_kernel<false, kActQuantize>), grid);
    else if (dbg) RESQ_LAUNCH_DECODE((gemm_decode_kernel<true, kActDirect>), grid);
    else RESQ_LAUNCH_DECODE((gemm_decode_kernel<false, kActDirect>), grid);
#undef RESQ_LAUNCH_DECODE
    return launch_status();
}

// shared by resq_gemm_mixed (asym false, c_hi = c_lo = null) and resq_gemm_mixed_asym
static int gemm_mixed_impl(const int8_t* q_hi, const uint8_t* q_lo, const float* s_hi,
                           const float* s_lo, bool asym, const float* c_hi, const float* c_lo,
                           const int32_t* lo_sum, int64_t M, const void* packed, int64_t N,
                           int64_t K, int64_t r, void* y, int64_t ldy, int32_t* dbg_acc_hi,
                           int32_t* dbg_acc_lo, void* stream, bool swiglu = false) {
    if (!shape_ok(N, K, r) || M < 1 || M > 0x7FFFFFFF) return RESQ_ERR_SHAPE;
    if (swiglu ? (N % 2 != 0 || ldy < N / 2) : (ldy < N)) return RESQ_ERR_SHAPE;
    if (K - r > kMaxLoWidth || r > kMaxHiWidth) return RESQ_ERR_SHAPE;
    if (!packed || !y) return RESQ_ERR_NULL;
    if (r > 0 && (!q_hi || !s_hi || (asym && !c_hi))) return RESQ_ERR_NULL;
    if (K - r > 0 && (!q_lo || !s_lo || !lo_sum || (asym && !c_lo))) return RESQ_ERR_NULL;
    if (!aligned(lo_sum, 4) || !aligned(c_hi, 4) || !aligned(c_lo, 4)) return RESQ_ERR_ALIGN;
    // an empty group's pointer is never read; null both when the codes are symmetric
    if (!asym || r == 0) c_hi = nullptr;
    if (!asym || K - r == 0) c_lo = nullptr;
    if (!aligned(q_hi, 16) || !aligned(q_lo, 16) || !aligned(packed, 256) || !aligned(y, 2) ||
        !aligned(s_hi, 4) || !aligned(s_lo, 4) || !aligned(dbg_acc_hi, 4) ||
        !aligned(dbg_acc_lo, 4))
        return RESQ_ERR_ALIGN;

    const WeightLayout L = make_weight_layout(N, K, r);
    hipStream_t st = static_cast<hipStream_t>(stream);
    const bool dbg = dbg_acc_hi || dbg_acc_lo;

    const GemmPlan plan = plan_gemm(M, L);
    if (plan.kernel == 0) {
        const int64_t lds_row = L.kh_pad + L.kl_pad / 2 + kDecodeRowPad;
        const DecodeArgs d = make_decode_args(q_hi, q_lo, s_hi, s_lo, c_hi, c_lo, lo_sum, M, packed, L, y, ldy,
                                              dbg_acc_hi, dbg_acc_lo, swiglu, lds_row);
        return launch_decode(d, dbg, false, st);
    }
    if (plan.kernel == 1) {
        const int tg = plan.tg, sk = plan.sk;
        const DecodeArgs d = make_decode_args(q_hi, q_lo, s_hi, s_lo, c_hi, c_lo, lo_sum, M, packed, L, y, ldy,
                                              dbg_acc_hi, dbg_acc_lo, swiglu, 0);
        const int slices = (int)((M + tg * 16 - 1) / (tg * 16));  // of tg * 16 tokens
        const int sets = (d.groups * sk + 7) / 8;
        const dim3 grid((unsigned)(sets < 256 ? sets : 256), (unsigned)slices), blk(kDecodeThreads);
        const int lds_bytes = 2 * sk * tg * kChunkBlocks * kBlockBytes;
        // one slice over a layer that no cache holds: nobody reads the weights again (measured:
        // 132 MB layers 4 to 10 % faster with the hint, a 38 MB layer 3 to 9 % slower)
        const bool nt = !dbg && slices == 1 && L.total_bytes >= (int64_t)64 << 20;
#define RESQ_LAUNCH_STREAM(TG, SK)                                                                 \
    do {                                                                                           \
        auto kernel = dbg ? gemm_stream_kernel<true, TG, SK>                                       \
                          : (nt ? gemm_stream_kernel<false, TG, SK, true> : gemm_stream_kernel<false, TG, SK>); \
        if (lds_bytes > 64 * 1024 &&                                                               \
            hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),                             \
                                hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes) != hipSuccess) \
            return RESQ_ERR_HIP;                                                                   \
        launch(kernel, grid, blk, lds_bytes, st, d);                                               \
    } while (0)
        switch (tg * 16 + sk) {
            case 1 * 16 + 1: RESQ_LAUNCH_STREAM(1, 1); break;
            case 1 * 16 + 2: RESQ_LAUNCH_STREAM(1, 2); break;
            case 1 * 16 + 4: RESQ_LAUNCH_STREAM(1, 4); break;
            case 1 * 16 + 8: RESQ_LAUNCH_STREAM(1, 8); break;
            case 2 * 16 + 1: RESQ_LAUNCH_STREAM(2, 1); break;
            case 2 * 16 + 2: RESQ_LAUNCH_STREAM(2, 2); break;
            default: RESQ_LAUNCH_STREAM(4, 1); break;
        }
#undef RESQ_LAUNCH_STREAM
        return launch_status();
    }

    GemmArgs a;
    a.q_hi = reinterpret_cast<const uint8_t*>(q_hi);
    a.q_lo = q_lo;
    a.L = L;
    a.ld_hi = a.L.kh_pad;
    a.ld_lo = a.L.kl_pad / 2;
    a.s_hi = s_hi;
    a.s_lo = s_lo;
    a.lo_sum = lo_sum;
    a.c_hi = c_hi;
    a.c_lo = c_lo;
    a.packed = static_cast<const uint8_t*>(packed);
    a.M = M;
    a.y = static_cast<uint16_t*>(y);
    a.ldy = ldy;
    a.dbg_hi = dbg_acc_hi;
    a.dbg_lo = dbg_acc_lo;
    a.swiglu = swiglu ? 1 : 0;
    a.stages_hi = (int)a.L.hi_blocks;  // one stage = one 64-byte block per row
    a.stages_lo = (int)a.L.lo_blocks;
    const bool narrow = plan.kernel == 3;  // 64-token tiles
    a.tiles_m = narrow ? (int)((M + kBM64 - 1) / kBM64) : (int)((M + kBM - 1) / kBM);
    a.tiles_n = (int)(a.L.n_pad / kBN);
    const int64_t tiles = (int64_t)a.tiles_m * a.tiles_n;
    if (tiles > 0x7FFFFFFF) return RESQ_ERR_SHAPE;

    // static LDS (68.5 or 76.5 KiB): two workgroups per compute unit
    if (narrow) {
        if (plan.sk == 2) {  // both rings
            if (dbg) launch(gemm_mixed_m64_kernel<true, 2>, dim3((unsigned)tiles), dim3(2 * kGemmThreads), 0, st, a);
            else launch(gemm_mixed_m64_kernel<false, 2>, dim3((unsigned)tiles), dim3(2 * kGemmThreads), 0, st, a);
        } else {
            if (dbg) launch(gemm_mixed_m64_kernel<true, 1>, dim3((unsigned)tiles), dim3(kGemmThreads), 0, st, a);
            else launch(gemm_mixed_m64_kernel<false, 1>, dim3((unsigned)tiles), dim3(kGemmThreads), 0, st, a);
        }
    } else {
        if (dbg) launch(gemm_mixed_kernel<true>, dim3((unsigned)tiles), dim3(kGemmThreads), 0, st, a);
        else launch(gemm_mixed_kernel<false>, dim3((unsigned)tiles), dim3(kGemmThreads), 0, st, a);
    }
    return launch_status();
}

int resq_gemm_mixed(const int8_t* q_hi, const uint8_t* q_lo, const float* s_hi, const float* s_lo,
                    const int32_t* lo_sum, int64_t M, const void* packed, int64_t N, int64_t K,
                    int64_t r, void* y, int64_t ldy, int32_t* dbg_acc_hi, int32_t* dbg_acc_lo,
                    void* stream) {
    return gemm_mixed_impl(q_hi, q_lo, s_hi, s_lo, false, nullptr, nullptr, lo_sum, M, packed, N, K,
                           r, y, ldy, dbg_acc_hi, dbg_acc_lo, stream);
}

int resq_quantize_gemm_mixed(const void* x, int64_t ldx, int64_t M, const void* packed, int64_t N,
                             int64_t K, int64_t r, void* y, int64_t ldy, void* stream) {
    if (!shape_ok(N, K, r) || M < 1 || ldx < K || ldy < N) return RESQ_ERR_SHAPE;
    if (K - r > kMaxLoWidth || r > kMaxHiWidth) return RESQ_ERR_SHAPE;
    if (!x || !packed || !y) return RESQ_ERR_NULL;
    if (!aligned(x, 16) || ldx % 8 != 0 || K % 8 != 0 || r % 8 != 0 || !aligned(packed, 256) || !aligned(y, 2))
        return RESQ_ERR_ALIGN;
    const WeightLayout L = make_weight_layout(N, K, r);
    const int64_t lds_row = L.kh_pad + L.kl_pad / 2 + kDecodeRowPad;
    if (M > kDecodeMaxM || M * lds_row > 140 * 1024) return RESQ_ERR_SHAPE;
    DecodeArgs d = make_decode_args(nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, M, packed, L, y,
                                    ldy, nullptr, nullptr, false, lds_row);
    d.x = static_cast<const uint16_t*>(x);
    d.ldx = ldx;
    // rows quantized at a time, each by 512 / R threads holding at most kFusedUnits 16-byte units
    const int64_t nunits = K / 8;
    if (nunits > (int64_t)kFusedUnits * kDecodeThreads) return RESQ_ERR_SHAPE;
    int R = 1;
    while (R < 8 && R < M && nunits * (2 * R) <= (int64_t)kFusedUnits * kDecodeThreads) R *= 2;
    d.fuse_rows = R;
    return launch_decode(d, false, true, static_cast<hipStream_t>(stream));
}

int resq_gemm_mixed_plan(int64_t M, int64_t N, int64_t K, int64_t r, int* kernel, int* token_groups,
                         int* runs) {
    if (!shape_ok(N, K, r) || M < 1 || M > 0x7FFFFFFF) return RESQ_ERR_SHAPE;
    if (K - r > kMaxLoWidth || r > kMaxHiWidth) return RESQ_ERR_SHAPE;
    if (!kernel || !token_groups || !runs) return RESQ_ERR_NULL;
    const GemmPlan plan = plan_gemm(M, make_weight_layout(N, K, r));
    *kernel = plan.kernel;
    *token_groups = plan.tg;
    *runs = plan.sk;
    return RESQ_OK;
}

int resq_gemm_mixed_swiglu(const int8_t* q_hi, const uint8_t* q_lo, const float* s_hi,
                           const float* s_lo, const int32_t* lo_sum, int64_t M, const void* packed,
                           int64_t N2, int64_t K, int64_t r, void* y, int64_t ldy, void* stream) {
    return gemm_mixed_impl(q_hi, q_lo, s_hi, s_lo, false, nullptr, nullptr, lo_sum, M, packed, N2, K,
                           r, y, ldy, nullptr, nullptr, stream, true);
}

int resq_gemm_mixed_asym(const int8_t* q_hi, const uint8_t* q_lo, const float* s_hi,
                         const float* s_lo, const float* c_hi, const float* c_lo,
                         const int32_t* lo_sum, int64_t M, const void* packed, int64_t N, int64_t K,
                         int64_t r, void* y, int64_t ldy, int32_t* dbg_acc_hi, int32_t* dbg_acc_lo,
                         void* stream) {
    return gemm_mixed_impl(q_hi, q_lo, s_hi, s_lo, true, c_hi, c_lo, lo_sum, M, packed, N, K, r, y,
                           ldy, dbg_acc_hi, dbg_acc_lo, stream);
}

int resq_online_hadamard(const void* x, void* y, int64_t ld, int64_t M, int64_t K,
                         int64_t col_begin, int64_t col_end, int64_t block, void* stream) {
    if (M < 1 || K < 1 || K > kMaxK || ld < K || col_begin < 0 || col_end > K ||
        col_begin >= col_end)
        return RESQ_ERR_SHAPE;
    if (!x || !y) return RESQ_ERR_NULL;
    const int64_t width = col_end - col_begin;
    if (block == 0) block = resq_hadamard_block(width);
    if (block < 1 || block > 8192 || (block & (block - 1)) != 0 || width % block != 0)
        return RESQ_ERR_SHAPE;
    if (!aligned(x, 16) || !aligned(y, 16) || ld % 8 != 0 || col_begin % 8 != 0 || width % 8 != 0)
        return RESQ_ERR_ALIGN;

    HadArgs a;
    a.x = static_cast<const uint16_t*>(x);
    a.y = static_cast<uint16_t*>(y);
    a.ld = ld;
    a.M = M;
    a.K = (int)K;
    a.c0 = (int)col_begin;
    a.c1 = (int)col_end;
    int lg = 0;
    while ((int64_t(1) << lg) < block) ++lg;
    a.log2b = lg;
    a.scale = 1.0f / sqrtf((float)block);
    const int I = block <= 512 ? 1 : (int)(block / 512);
    const int64_t span = 512 * (int64_t)I;
    a.spans_per_row = (int)((width + span - 1) / span);
    const int64_t items = M * a.spans_per_row;
    const int64_t blocks = (items + kHadThreads / 64 - 1) / (kHadThreads / 64);
    if (blocks > 0x7FFFFFFF || M > 0x7FFFFFFF) return RESQ_ERR_SHAPE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (x != y && (col_begin > 0 || col_end < K))
        hipLaunchKernelGGL(hadamard_copy_rest_kernel, dim3((unsigned)M), dim3(kHadThreads), 0, st, a);
    const dim3 grid((unsigned)blocks), blk(kHadThreads);
    switch (I) {
        case 1: launch(hadamard_kernel<1>, grid, blk, 0, st, a); break;
        case 2: launch(hadamard_kernel<2>, grid, blk, 0, st, a); break;
        case 4: launch(hadamard_kernel<4>, grid, blk, 0, st, a); break;
        case 8: launch(hadamard_kernel<8>, grid, blk, 0, st, a); break;
        default: launch(hadamard_kernel<16>, grid, blk, 0, st, a); break;
    }
    return launch_status();
}

int resq_project_heads(const void* x, int64_t ldx, int64_t rows, int64_t d_head, const void* packed,
                       void* y, int64_t ldy, void* stream) {
    if (rows < 0 || rows > 0x7FFFFFFF || (d_head != 64 && d_head != 128) || ldx < d_head || ldy < d_head)
        return RESQ_ERR_SHAPE;
    if (rows == 0) return RESQ_OK;
    if (!x || !packed || !y) return RESQ_ERR_NULL;
    if (!aligned(x, 16) || ldx % 8 != 0 || !aligned(packed, 256) || !aligned(y, 2)) return RESQ_ERR_ALIGN;
    HeadProjArgs a;
    a.x = static_cast<const uint16_t*>(x);
    a.ldx = ldx;
    a.rows = rows;
    a.packed = static_cast<const uint8_t*>(packed);
    a.L = make_weight_layout(d_head, d_head, d_head);
    a.y = static_cast<uint16_t*>(y);
    a.ldy = ldy;
    const int store_bytes = (int)d_head / 8;  // d_head / 16 consecutive channels per lane
    a.vec_store = aligned(y, store_bytes) && (ldy * 2) % store_bytes == 0;
    const int64_t tiles = (rows + 15) / 16;
    const int64_t wgs = (tiles + kHeadProjThreads / 64 - 1) / (kHeadProjThreads / 64);
    const dim3 grid((unsigned)(wgs < 768 ? wgs : 768)), blk(kHeadProjThreads);  // three per compute unit
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (d_head == 128) launch(head_project_kernel<128>, grid, blk, 0, st, a);
    else launch(head_project_kernel<64>, grid, blk, 0, st, a);
    return launch_status();
}

int resq_gram_accumulate(const void* x, int64_t ldx, int64_t T, int64_t K, float* c, int64_t ldc,
                         void* stream) {
    if (T < 0 || K < 1 || K > kMaxK || ldx < K || ldc < K) return RESQ_ERR_SHAPE;
    if (T == 0) return RESQ_OK;
    if (!x || !c) return RESQ_ERR_NULL;
    if (!aligned(x, 16) || !aligned(c, 4) || ldx % 8 != 0 || K % 8 != 0) return RESQ_ERR_ALIGN;
    BasisGemmArgs g;
    g.a = x; g.b = x; g.c = c;
    g.lda = ldx; g.ldb = ldx; g.ldc = ldc;
    g.I = K; g.J = K; g.T = T;
    g.accumulate = 1;
    // slices of the token axis (their sums meet by atomic adds) until the chip is full
    const int64_t tiles = ((K + kBasisTile - 1) / kBasisTile) * ((K + kBasisTile - 1) / kBasisTile);
    int64_t slices = 1;
    while (tiles * slices < 512 && T / (2 * slices) >= 512) slices *= 2;
    g.t_per_slice = round_up((T + slices - 1) / slices, kBasisChunk);
    slices = (T + g.t_per_slice - 1) / g.t_per_slice;
    const dim3 grid((unsigned)((K + kBasisTile - 1) / kBasisTile), (unsigned)((K + kBasisTile - 1) / kBasisTile),
                    (unsigned)slices);
    launch(basis_gemm_kernel<true, true, true, false>, grid, dim3(kBasisThreads), 0,
           static_cast<hipStream_t>(stream), g);
    return launch_status();
}

int resq_project_rows(const void* a, int a_is_bf16, int64_t lda, int64_t rows, int64_t K, const float* u,
                      int64_t ldu, int64_t J, void* out, int out_is_bf16, int64_t ldo, void* stream) {
    if (rows < 0 || rows > 0x7FFFFFFF || K < 1 || K > kMaxK || J < 1 || J > kMaxK || lda < K || ldu < J || ldo < J)
        return RESQ_ERR_SHAPE;
    if (rows == 0) return RESQ_OK;
    if (!a || !u || !out) return RESQ_ERR_NULL;
    if (!aligned(a, 16) || !aligned(u, 16) || !aligned(out, out_is_bf16 ? 2 : 4) || lda % 8 != 0 ||
        ldu % 8 != 0 || J % 8 != 0)
        return RESQ_ERR_ALIGN;
    BasisGemmArgs g;
    g.a = a; g.b = u; g.c = out;
    g.lda = lda; g.ldb = ldu; g.ldc = ldo;
    g.I = rows; g.J = J; g.T = K;
    g.accumulate = 0;
    g.t_per_slice = round_up(K, kBasisChunk);
    const dim3 grid((unsigned)((J + kBasisTile - 1) / kBasisTile), (unsigned)((rows + kBasisTile - 1) / kBasisTile), 1);
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (a_is_bf16) {
        if (out_is_bf16) launch(basis_gemm_kernel<false, true, false, true>, grid, dim3(kBasisThreads), 0, st, g);
        else launch(basis_gemm_kernel<false, true, false, false>, grid, dim3(kBasisThreads), 0, st, g);
    } else {
        if (out_is_bf16) launch(basis_gemm_kernel<false, false, false, true>, grid, dim3(kBasisThreads), 0, st, g);
        else launch(basis_gemm_kernel<false, false, false, false>, grid, dim3(kBasisThreads), 0, st, g);
    }
    return launch_status();
}

size_t resq_sym_eig_workspace_bytes(int64_t K) {
    if (K < 2 || K % 2 != 0 || K > kEigMaxOrder) return 0;
    const size_t nn = (size_t)K * (size_t)K * sizeof(double);
    return 2 * round_up((int64_t)nn, 256) + round_up(K * (int64_t)sizeof(double), 256) +
           round_up(K * (int64_t)sizeof(int), 256) + round_up(kEigMaxSweeps * (int64_t)sizeof(int), 256);
}

// the Jacobi iteration on a workspace that holds resq_sym_eig_workspace_bytes(K) bytes
static int sym_eig_on_workspace(const float* c, int64_t ldc, int64_t K, int sweeps, float* eigvals, float* p,
                                int64_t ldp, void* workspace, void* stream) {
    const int n = (int)K;
    const size_t nn = (size_t)round_up((int64_t)((size_t)n * n * sizeof(double)), 256);
    uint8_t* w = static_cast<uint8_t*>(workspace);
    EigPlan e;
    e.n = n;
    e.a = reinterpret_cast<double*>(w);
    e.vt = reinterpret_cast<double*>(w + nn);
    e.cs = reinterpret_cast<double*>(w + 2 * nn);
    e.pq = reinterpret_cast<int*>(w + 2 * nn + round_up(K * (int64_t)sizeof(double), 256));
    e.nrot = reinterpret_cast<int*>(w + 2 * nn + round_up(K * (int64_t)sizeof(double), 256) +
                                    round_up(K * (int64_t)sizeof(int), 256));
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int lds_bytes = 2 * n * (int)sizeof(double);
    if (lds_bytes > 64 * 1024 &&
        hipFuncSetAttribute(reinterpret_cast<const void*>(eig_round_kernel),
                            hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes) != hipSuccess)
        return RESQ_ERR_HIP;
    const int64_t elems = (int64_t)n * n;
    hipLaunchKernelGGL(eig_init_kernel, dim3((unsigned)((elems + 255) / 256)), dim3(256), 0, st, c, ldc, e);  // >= 256 threads
    const dim3 rot_grid((unsigned)((n / 2 + 255) / 256));
    for (int sweep = 0; sweep < sweeps; ++sweep) {
        for (int round = 0; round < n - 1; ++round) {
            hipLaunchKernelGGL(eig_rotations_kernel, rot_grid, dim3(256), 0, st, e, sweep, round);
            hipLaunchKernelGGL(eig_round_kernel, dim3((unsigned)(n / 2)), dim3(kEigThreads), lds_bytes, st, e, sweep);
        }
    }
    launch(eig_finish_kernel, dim3((unsigned)n), dim3(kEigThreads), 0, st, e, eigvals, p, ldp);
    return launch_status();
}

int resq_sym_eig(const float* c, int64_t ldc, int64_t K, int sweeps, float* eigvals, float* p, int64_t ldp,
                 void* workspace, size_t workspace_bytes, void* stream) {
    if (K < 2 || K % 2 != 0 || K > kEigMaxOrder || ldc < K || ldp < K || sweeps < 1 || sweeps > kEigMaxSweeps)
        return RESQ_ERR_SHAPE;
    if (!c || !eigvals || !p || !workspace) return RESQ_ERR_NULL;
    if (!aligned(c, 4) || !aligned(eigvals, 4) || !aligned(p, 4) || !aligned(workspace, 256)) return RESQ_ERR_ALIGN;
    if (workspace_bytes < resq_sym_eig_workspace_bytes(K)) return RESQ_ERR_BUFFER;
    return sym_eig_on_workspace(c, ldc, K, sweeps, eigvals, p, ldp, workspace, stream);
}

int resq_sym_eig_static(const float* c, int64_t ldc, int64_t K, int sweeps, float* eigvals, float* p,
                        int64_t ldp, void* stream) {
    if (K < 2 || K % 2 != 0 || K > kEigMaxOrder || ldc < K || ldp < K || sweeps < 1 || sweeps > kEigMaxSweeps)
        return RESQ_ERR_SHAPE;
    if (K > kEigStaticMaxOrder || resq_sym_eig_workspace_bytes(K) > kEigStaticBytes)
        return RESQ_ERR_BUFFER;   // beyond the built-in scratch area
    if (!c || !eigvals || !p) return RESQ_ERR_NULL;
    if (!aligned(c, 4) || !aligned(eigvals, 4) || !aligned(p, 4)) return RESQ_ERR_ALIGN;
    void* scratch = eig_scratch_on_current_device();
    if (!scratch) return RESQ_ERR_HIP;
    return sym_eig_on_workspace(c, ldc, K, sweeps, eigvals, p, ldp, scratch, stream);
}

}  // extern "C"
