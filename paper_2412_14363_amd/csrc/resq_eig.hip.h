// Symmetric eigendecomposition for the PCA step of the basis construction
// (Section 4.2: P = eigenvectors of the activations' covariance matrix; the r
// of largest eigenvalue span the high-precision subspace): cyclic Jacobi in
// fp64 with the round-robin ("tournament") ordering, n / 2 disjoint rotations
// per round, n - 1 rounds per sweep.
//
// A round applies J = product of its plane rotations as A <- J^T A J, V <- V J.
// Everything is done as ROW operations on contiguous rows: with A symmetric,
//   A2 = (J^T A)^T = A J      and      A3 = (J^T A2)^T = J^T A J,
// so the same kernel (rotate pairs of rows, write the result transposed into the
// other buffer) runs twice per round; the eigenvectors are kept transposed
// (Vt <- J^T Vt, in place).  In the tournament ordering 16 consecutive pairs have
// 16 consecutive p and 16 consecutive q (mod n - 1), so the transposed writes are
// contiguous runs as well.  Offline step, bound by HBM: 6 n^2 fp64 words move per
// round (the matrix read and written twice, the vectors once).  Rotations of
// elements already negligible are skipped, and once a whole sweep has skipped
// all of them the remaining kernels return at once.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace resq {

constexpr int kEigThreads = 256;
constexpr int kEigPairs = 16;   // pairs per workgroup of the transposing kernel
constexpr int kEigCols = 64;    // columns per workgroup of the transposing kernel

struct EigPlan {
    int n;            // matrix order, even
    double* a[2];     // ping-pong copies of the matrix, [n][n]
    double* vt;       // eigenvectors as rows, [n][n]
    int* pq;          // [n / 2][2]: the round's pairs, p < q
    double* cs;       // [n / 2][2]: cosine and sine of each pair's rotation
    int* nrot;        // [kEigMaxSweeps]: rotations that each sweep still had to make
};

constexpr int kEigMaxSweeps = 64;
// an off-diagonal element below this fraction of sqrt(a_pp a_qq) is left alone: fp32
// outputs cannot tell, and a sweep that finds nothing larger ends the iteration
constexpr double kEigSkip = 1.0 / (1ull << 40);

// a sweep after one that rotated nothing has nothing to do (the host enqueues a fixed
// number of sweeps, so that the call never waits for the device)
__device__ __forceinline__ bool eig_converged(const EigPlan& e, int sweep) {
    return sweep > 0 && e.nrot[sweep - 1] == 0;
}

// pair k of round s: (n - 1, s) for k = 0, else ((s + k) mod (n - 1), (s - k) mod (n - 1))
__device__ __forceinline__ void eig_pair(int n, int s, int k, int& p, int& q) {
    const int m = n - 1;
    int a = k == 0 ? m : (s + k) % m;
    int b = k == 0 ? s : (s - k + m) % m;
    p = a < b ? a : b;
    q = a < b ? b : a;
}

__global__ void eig_init_kernel(const float* __restrict__ c, int64_t ldc, EigPlan e) {
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t nn = (int64_t)e.n * e.n;
    if (idx < kEigMaxSweeps) e.nrot[idx] = 0;   // the grid has at least that many threads
    if (idx >= nn) return;
    const int i = (int)(idx / e.n), j = (int)(idx % e.n);
    // the symmetric part, so that rounding differences between c[i][j] and c[j][i] do not matter
    e.a[0][idx] = 0.5 * ((double)c[(int64_t)i * ldc + j] + (double)c[(int64_t)j * ldc + i]);
    e.vt[idx] = i == j ? 1.0 : 0.0;
}

// rotation that annihilates a[p][q] (the smaller of the two angles)
__global__ void eig_rotations_kernel(EigPlan e, int sweep, int round) {
    const int k = blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= e.n / 2 || eig_converged(e, sweep)) return;
    int p, q;
    eig_pair(e.n, round, k, p, q);
    const double* a = e.a[0];
    const double app = a[(int64_t)p * e.n + p], aqq = a[(int64_t)q * e.n + q], apq = a[(int64_t)p * e.n + q];
    double c = 1.0, s = 0.0;
    if (fabs(apq) > kEigSkip * sqrt(fabs(app * aqq))) {
        atomicAdd(&e.nrot[sweep], 1);
        const double tau = (aqq - app) / (2.0 * apq);
        const double t = (tau >= 0.0 ? 1.0 : -1.0) / (fabs(tau) + sqrt(1.0 + tau * tau));
        c = 1.0 / sqrt(1.0 + t * t);
        s = t * c;
    }
    e.pq[2 * k] = p;
    e.pq[2 * k + 1] = q;
    e.cs[2 * k] = c;
    e.cs[2 * k + 1] = s;
}

// dst = (J^T src)^T: row p' = c row p - s row q, row q' = s row p + c row q, written as columns
__global__ __launch_bounds__(kEigThreads) void eig_rotate_transpose_kernel(EigPlan e, int sweep, int from) {
    __shared__ double tile[kEigCols][2 * kEigPairs + 1];
    if (eig_converged(e, sweep)) return;
    const double* __restrict__ src = e.a[from];
    double* __restrict__ dst = e.a[from ^ 1];
    const int n = e.n;
    const int t = threadIdx.x;
    const int k0 = blockIdx.y * kEigPairs, j0 = blockIdx.x * kEigCols;
    {
        const int kl = t >> 4, cg = (t & 15) * 4;   // pair of the workgroup, first of 4 columns
        const int k = k0 + kl;
        if (k < n / 2) {
            const int p = e.pq[2 * k], q = e.pq[2 * k + 1];
            const double c = e.cs[2 * k], s = e.cs[2 * k + 1];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int j = j0 + cg + u;
                if (j < n) {
                    const double ap = src[(int64_t)p * n + j], aq = src[(int64_t)q * n + j];
                    tile[cg + u][2 * kl] = c * ap - s * aq;
                    tile[cg + u][2 * kl + 1] = s * ap + c * aq;
                }
            }
        }
    }
    __syncthreads();
    {
        // thread -> column j0 + t / 4, pairs (t % 4) * 4 .. + 4: consecutive threads write
        // consecutive p (and consecutive q) of one destination row
        const int col = t >> 2, j = j0 + col;
        if (j < n) {
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int kl = (t & 3) * 4 + u, k = k0 + kl;
                if (k < n / 2) {
                    dst[(int64_t)j * n + e.pq[2 * k]] = tile[col][2 * kl];
                    dst[(int64_t)j * n + e.pq[2 * k + 1]] = tile[col][2 * kl + 1];
                }
            }
        }
    }
}

// Vt <- J^T Vt, in place
__global__ __launch_bounds__(kEigThreads) void eig_rotate_rows_kernel(EigPlan e, int sweep) {
    if (eig_converged(e, sweep)) return;
    const int k = blockIdx.y;
    const int j = blockIdx.x * kEigThreads + threadIdx.x;
    if (j >= e.n) return;
    const int p = e.pq[2 * k], q = e.pq[2 * k + 1];
    const double c = e.cs[2 * k], s = e.cs[2 * k + 1];
    double* rp = e.vt + (int64_t)p * e.n;
    double* rq = e.vt + (int64_t)q * e.n;
    const double vp = rp[j], vq = rq[j];
    rp[j] = c * vp - s * vq;
    rq[j] = s * vp + c * vq;
}

// eigenvalue i = a[i][i]; its position in decreasing order (ties by index); column
// rank[i] of P = row i of Vt
__global__ __launch_bounds__(kEigThreads) void eig_finish_kernel(EigPlan e, float* __restrict__ eigvals,
                                                                 float* __restrict__ p, int64_t ldp) {
    const int i = blockIdx.x;
    const int n = e.n;
    const double* a = e.a[0];
    const double li = a[(int64_t)i * n + i];
    __shared__ int count[kEigThreads];
    int c = 0;
    for (int j = threadIdx.x; j < n; j += kEigThreads) {
        const double lj = a[(int64_t)j * n + j];
        c += (lj > li || (lj == li && j < i)) ? 1 : 0;
    }
    count[threadIdx.x] = c;
    __syncthreads();
    for (int w = kEigThreads / 2; w > 0; w >>= 1) {
        if (threadIdx.x < w) count[threadIdx.x] += count[threadIdx.x + w];
        __syncthreads();
    }
    const int rank = count[0];
    if (threadIdx.x == 0) eigvals[rank] = (float)li;
    for (int j = threadIdx.x; j < n; j += kEigThreads) p[(int64_t)j * ldp + rank] = (float)e.vt[(int64_t)i * n + j];
}

}  // namespace resq
