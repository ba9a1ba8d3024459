"""CPU oracle of the offline basis construction (Section 4.2): plain numpy, fp64.

TEST INFRASTRUCTURE ONLY: imported by the tests and the benchmark's cpu_baseline
leg, never by the product path.

The steps, in the paper's order:
  1. the covariance (Gram) matrix of the calibration activations, sum_t x_t x_t^T;
  2. its eigenvectors P (PCA).  Section 4.2 shows that the quantization error
     bound of Theorem 4.2 is lowest when the high-precision subspace P_h is
     spanned by the eigenvectors of the r LARGEST eigenvalues;
  3. U = P blockdiag(R) with random orthogonal R inside each group (the
     equation that defines U in Section 4.2; Lemma 4.1 for why R);
  4. activations and weights are expressed in that basis: X U and W U
     (Section 4.1, Eq. 4: Q(X U) Q(U^T W)); the weights are folded offline
     (Section 4.3).
The symmetric eigensolver is LAPACK's, through numpy: a library primitive as one
step.  Column convention of this library: the high group comes FIRST (columns
[0, r)), so eigenvectors are ordered by DECREASING eigenvalue; the paper orders
them increasingly and keeps the last r, which is the same split with the column
order reversed (a fixed permutation absorbed into U).
"""
from __future__ import annotations

import numpy as np


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    b = np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << 16
    return b.view(np.float32).astype(np.float64)


def f64_to_bf16_bits(v: np.ndarray) -> np.ndarray:
    """Round to nearest even, from the fp32 rounding of v (values here are far from
    fp32's limits; double rounding through fp32 is what a device that accumulates in
    fp32 and stores bf16 does as well)."""
    u = np.ascontiguousarray(v, dtype=np.float64).astype(np.float32).view(np.uint32).astype(np.uint64)
    rounded = u + 0x7FFF + ((u >> 16) & 1)
    return (rounded >> 16).astype(np.uint16)


def gram(x: np.ndarray) -> np.ndarray:
    """sum over tokens of x_t x_t^T for x [T, K] (the covariance matrix of Section 4.2,
    unnormalized and uncentred as there; scaling does not change eigenvectors)."""
    x = np.asarray(x, np.float64)
    return x.T @ x


def pca_basis(c: np.ndarray):
    """Eigenvalues (decreasing) and eigenvectors (columns, same order) of the symmetric c."""
    lam, vec = np.linalg.eigh(np.asarray(c, np.float64))   # ascending
    order = np.argsort(-lam, kind="stable")
    return lam[order], vec[:, order]


def compose_basis(p: np.ndarray, r_h: np.ndarray, r_l: np.ndarray) -> np.ndarray:
    """U = [P_h R_h, P_l R_l] with P_h the first r = R_h.shape[0] columns of P."""
    p = np.asarray(p, np.float64)
    r = r_h.shape[0]
    assert r_l.shape[0] == p.shape[1] - r
    return np.concatenate([p[:, :r] @ np.asarray(r_h, np.float64),
                           p[:, r:] @ np.asarray(r_l, np.float64)], axis=1)


def project(a: np.ndarray, u: np.ndarray) -> np.ndarray:
    """Rows of a expressed in the basis u: a @ u (activations X U; weights W U, whose
    transpose is the U^T W of Eq. 4 for W stored as [out_features, in_features])."""
    return np.asarray(a, np.float64) @ np.asarray(u, np.float64)
