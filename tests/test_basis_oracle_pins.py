"""Pins of the basis-construction oracle (Section 4.2) to what the mathematics fixes.

None compares the oracle with itself: planted spectra whose eigenvectors are
known by construction, hand-computed 2 x 2 cases, orthogonality and invariance
identities, the variational (Ky Fan) characterisation of the top-r subspace, and
the paper's own claim that the projection lowers the quantization error.
"""
import numpy as np
import pytest
import torch

from oracle import resq_basis_oracle as bo
from paper_2412_14363_amd import workloads as wl


def planted(seed, T, K, sigmas):
    """x = z diag(sigma) Q^T with z having exactly orthonormal columns: the Gram matrix is
    exactly Q diag(sigma^2) Q^T, eigenvectors = columns of Q."""
    q = wl.random_orthogonal(K, seed).double().numpy()
    g = torch.Generator().manual_seed(seed + 100)
    z = np.linalg.qr(torch.randn(T, K, generator=g, dtype=torch.float64).numpy())[0]
    return (z * np.asarray(sigmas)) @ q.T, q


def test_gram_hand_case_and_orientation():
    # [T=3, K=2]: the Gram matrix is K x K (features), not T x T: a transposed operand fails
    x = np.array([[1.0, 2.0], [3.0, 4.0], [5.0, 6.0]])
    assert np.array_equal(bo.gram(x), np.array([[35.0, 44.0], [44.0, 56.0]]))


def test_pca_two_by_two_closed_form():
    # [[2, 1], [1, 2]]: eigenvalues 3 and 1, eigenvectors (1, 1)/sqrt2 and (1, -1)/sqrt2;
    # decreasing order, columns (not rows) are the vectors
    lam, p = bo.pca_basis(np.array([[2.0, 1.0], [1.0, 2.0]]))
    assert np.allclose(lam, [3.0, 1.0])
    assert np.allclose(np.abs(p[:, 0]), [2 ** -0.5, 2 ** -0.5]) and p[0, 0] * p[1, 0] > 0
    assert np.allclose(np.abs(p[:, 1]), [2 ** -0.5, 2 ** -0.5]) and p[0, 1] * p[1, 1] < 0


def test_pca_recovers_planted_basis_in_decreasing_order():
    K = 24
    sig = np.linspace(5.0, 0.5, K) * np.where(np.arange(K) % 2 == 0, 1.0, 1.07)  # distinct, shuffled below
    perm = np.random.default_rng(3).permutation(K)
    x, q = planted(1, 200, K, sig[perm])
    lam, p = bo.pca_basis(bo.gram(x))
    order = np.argsort(-sig[perm])
    assert np.allclose(lam, np.sort(sig ** 2)[::-1], rtol=1e-6)      # Q comes from an fp32 QR
    # each eigenvector equals the planted column up to sign
    dots = np.abs(np.sum(p * q[:, order], axis=0))
    assert np.allclose(dots, 1.0, atol=1e-5)


def test_projected_coordinates_are_uncorrelated_with_decreasing_variance():
    # PCA: (XP)^T (XP) = diag(lambda), largest first (Section 4.2: the projected
    # coefficients are sorted by variance)
    x = np.random.default_rng(5).standard_normal((300, 16)) * np.linspace(1, 4, 16)
    lam, p = bo.pca_basis(bo.gram(x))
    c = bo.gram(bo.project(x, p))
    assert np.allclose(c, np.diag(lam), atol=1e-8 * lam[0])
    assert np.all(np.diff(lam) <= 0)


def test_top_r_subspace_maximizes_captured_energy():
    # Section 4.2: ||X P_h||_F is largest for the eigenvectors of the r largest
    # eigenvalues (Ky Fan): no other orthonormal r-frame captures more
    rng = np.random.default_rng(7)
    x = rng.standard_normal((400, 32)) * np.concatenate([np.full(4, 10.0), np.ones(28)])
    x = x @ wl.random_orthogonal(32, 9).double().numpy()
    lam, p = bo.pca_basis(bo.gram(x))
    r = 4
    best = np.linalg.norm(bo.project(x, p[:, :r])) ** 2
    assert np.isclose(best, lam[:r].sum(), rtol=1e-10)
    for s in range(20):
        f = wl.random_orthogonal(32, 100 + s).double().numpy()[:, :r]
        assert np.linalg.norm(x @ f) ** 2 <= best * (1 + 1e-12)
    # and the LAST r columns (the mistake of keeping the smallest eigenvalues) capture least
    assert np.linalg.norm(bo.project(x, p[:, -r:])) ** 2 < 0.1 * best


def test_compose_basis_is_orthogonal_and_keeps_the_split():
    K, r = 20, 6
    x, _ = planted(11, 100, K, np.linspace(3, 1, K))
    _, p = bo.pca_basis(bo.gram(x))
    r_h = wl.random_orthogonal(r, 1).double().numpy()
    r_l = wl.random_orthogonal(K - r, 2).double().numpy()
    u = bo.compose_basis(p, r_h, r_l)
    assert np.allclose(u.T @ u, np.eye(K), atol=1e-6)
    # U_h spans the span of P_h (U_h U_h^T = P_h P_h^T), U_l that of P_l
    assert np.allclose(u[:, :r] @ u[:, :r].T, p[:, :r] @ p[:, :r].T, atol=1e-6)
    assert np.allclose(u[:, r:] @ u[:, r:].T, p[:, r:] @ p[:, r:].T, atol=1e-6)
    # and it is not P itself: the rotation inside the groups was applied
    assert not np.allclose(u, p, atol=1e-3)


def test_layer_output_is_invariant_without_quantization():
    # Section 4.1: (X U)(W U)^T = X W^T for orthogonal U
    rng = np.random.default_rng(13)
    x, w = rng.standard_normal((9, 12)), rng.standard_normal((7, 12))
    _, p = bo.pca_basis(bo.gram(rng.standard_normal((50, 12))))
    u = bo.compose_basis(p, wl.random_orthogonal(3, 1).double().numpy(), wl.random_orthogonal(9, 2).double().numpy())
    assert np.allclose(bo.project(x, u) @ bo.project(w, u).T, x @ w.T, atol=1e-6)   # R comes from an fp32 QR


def test_bf16_rounding_helpers():
    v = np.array([1.0, -2.5, 3.140625, 1.00390625, 1.01171875, 0.0, 65280.0])
    t = torch.tensor(v, dtype=torch.float64).to(torch.bfloat16)
    assert np.array_equal(bo.f64_to_bf16_bits(v), wl.bf16_bits(t))
    assert np.array_equal(bo.bf16_bits_to_f64(wl.bf16_bits(t)), t.double().numpy())


def test_projection_raises_layer_snr_on_outlier_activations(oracle):
    # the point of Sections 4.1-4.2: with the PCA + rotation basis, keeping r = K/8
    # coefficients in 8 bits gives a higher output SNR than quantizing the raw activations
    # the same way (whose outlier channels are not where the 8-bit group is)
    K, N, T, r = 128, 96, 256, 16
    g = torch.Generator().manual_seed(21)
    x = torch.randn(T, K, generator=g)
    cols = torch.randperm(K, generator=g)[:6]
    x[:, cols] *= 20.0                                     # outlier channels anywhere
    x = x.to(torch.bfloat16)
    w = (torch.randn(N, K, generator=g) * 0.02).to(torch.bfloat16)
    xd, wd = x.double().numpy(), w.double().numpy()
    ref = xd @ wd.T
    raw = oracle.snr_db(ref, oracle.linear(wl.bf16_bits(x), wl.bf16_bits(w), r).y)
    _, p = bo.pca_basis(bo.gram(xd))
    u = bo.compose_basis(p, wl.random_orthogonal(r, 1).double().numpy(),
                         wl.random_orthogonal(K - r, 2).double().numpy())
    xr = bo.f64_to_bf16_bits(bo.project(xd, u))
    wr = bo.f64_to_bf16_bits(bo.project(wd, u))
    rot = oracle.snr_db(ref, oracle.linear(xr, wr, r).y)
    assert rot > raw + 6.0, (raw, rot)
