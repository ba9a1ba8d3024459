// Symmetric eigendecomposition for the PCA step of the basis construction
// (Section 4.2: P = eigenvectors of the activations' covariance matrix; the r
// of largest eigenvalue span the high-precision subspace): cyclic Jacobi in
// fp64 with the round-robin ("tournament") ordering, n / 2 disjoint rotations
// per round, n - 1 rounds per sweep.
//
// A round applies J = product of its plane rotations as A <- J^T A J, V <- V J,
// in one pass over the matrix: the workgroup of pair (p, q) owns rows p and q.
// J^T A mixes exactly those two rows, element by element; (J^T A) J then mixes,
// inside each row, the elements of every pair of the round, so the two rotated
// rows sit in LDS (16 n bytes) while all n / 2 column rotations are applied to
// them, and go back in place.  The eigenvectors are kept transposed, so that
// their update Vt <- J^T Vt is the same two-row operation.  Every access to
// memory is a contiguous row.  Offline step, bound by HBM: 4 n^2 fp64 words move
// per round (matrix and vectors, read and written once).  Rotations of elements
// already negligible are skipped, and once a whole sweep has skipped all of them
// the remaining kernels return at once.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace resq {

constexpr int kEigThreads = 256;
constexpr int kEigMaxOrder = 8192;  // two fp64 rows in LDS: 128 KiB

struct EigPlan {
    int n;            // matrix order, even
    double* a;        // the matrix, [n][n], symmetric between rounds
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
    e.a[idx] = 0.5 * ((double)c[(int64_t)i * ldc + j] + (double)c[(int64_t)j * ldc + i]);
    e.vt[idx] = i == j ? 1.0 : 0.0;
}

// rotation that annihilates a[p][q] (the smaller of the two angles)
__global__ void eig_rotations_kernel(EigPlan e, int sweep, int round) {
    const int k = blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= e.n / 2 || eig_converged(e, sweep)) return;
    int p, q;
    eig_pair(e.n, round, k, p, q);
    const double* a = e.a;
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

// one round for pair blockIdx.x: rows p, q of A <- J^T A J, rows p, q of Vt <- J^T Vt
__global__ __launch_bounds__(kEigThreads) void eig_round_kernel(EigPlan e, int sweep) {
    extern __shared__ __attribute__((aligned(16))) double rows[];  // [2][n]
    if (eig_converged(e, sweep)) return;
    const int n = e.n, t = threadIdx.x, k = blockIdx.x;
    const int p = e.pq[2 * k], q = e.pq[2 * k + 1];
    const double c = e.cs[2 * k], s = e.cs[2 * k + 1];
    double* ap = e.a + (int64_t)p * n;
    double* aq = e.a + (int64_t)q * n;
    double* rp = rows;
    double* rq = rows + n;
    for (int j = t; j < n; j += kEigThreads) {
        const double x = ap[j], y = aq[j];
        rp[j] = c * x - s * y;
        rq[j] = s * x + c * y;
    }
    {
        double* vp = e.vt + (int64_t)p * n;
        double* vq = e.vt + (int64_t)q * n;
        for (int j = t; j < n; j += kEigThreads) {
            const double x = vp[j], y = vq[j];
            vp[j] = c * x - s * y;
            vq[j] = s * x + c * y;
        }
    }
    __syncthreads();
    // the column rotations of every pair of the round, on both rows (the pairs are disjoint)
    for (int kk = t; kk < n / 2; kk += kEigThreads) {
        const int p2 = e.pq[2 * kk], q2 = e.pq[2 * kk + 1];
        const double c2 = e.cs[2 * kk], s2 = e.cs[2 * kk + 1];
        const double x0 = rp[p2], y0 = rp[q2], x1 = rq[p2], y1 = rq[q2];
        rp[p2] = c2 * x0 - s2 * y0;
        rp[q2] = s2 * x0 + c2 * y0;
        rq[p2] = c2 * x1 - s2 * y1;
        rq[q2] = s2 * x1 + c2 * y1;
    }
    __syncthreads();
    for (int j = t; j < n; j += kEigThreads) {
        ap[j] = rp[j];
        aq[j] = rq[j];
    }
}

// eigenvalue i = a[i][i]; its position in decreasing order (ties by index); column
// rank[i] of P = row i of Vt
__global__ __launch_bounds__(kEigThreads) void eig_finish_kernel(EigPlan e, float* __restrict__ eigvals,
                                                                 float* __restrict__ p, int64_t ldp) {
    const int i = blockIdx.x;
    const int n = e.n;
    const double* a = e.a;
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
        if ((int)threadIdx.x < w) count[threadIdx.x] += count[threadIdx.x + w];
        __syncthreads();
    }
    const int rank = count[0];
    if (threadIdx.x == 0) eigvals[rank] = (float)li;
    for (int j = threadIdx.x; j < n; j += kEigThreads) p[(int64_t)j * ldp + rank] = (float)e.vt[(int64_t)i * n + j];
}

}  // namespace resq
