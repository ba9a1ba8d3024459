"""GPU parity of the offline basis construction (Section 4.2) against its oracle, through the C ABI.

Floating point: the Gram matrix and the projections accumulate exact bf16/fp32 products in
fp32, so they are compared with the fp64 oracle at a tolerance derived from the length of the
sum; eigenvalues are unique and compared directly; eigenvectors are unique only up to sign
and, inside clusters, up to a rotation, so what is compared is the projector onto the top-r
subspace (unique when the r-th gap is open) and the rest is checked for validity (orthonormal,
small residual).
"""
import numpy as np
import pytest
import torch

from oracle import resq_basis_oracle as bo
from paper_2412_14363_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def rq():
    from paper_2412_14363_amd import binding
    binding.lib()
    return binding


def calib(seed, T, K, outliers=6):
    g = torch.Generator().manual_seed(seed)
    x = torch.randn(T, K, generator=g)
    cols = torch.randperm(K, generator=g)[:outliers]
    x[:, cols] *= 20.0
    return x.to(torch.bfloat16)


@pytest.mark.parametrize("T,K", [(300, 128), (1000, 256), (77, 8), (4096, 520), (5000, 64), (16, 1024)])
def test_gram_accumulate(rq, T, K):
    x = calib(T + K, T, K)
    ref = bo.gram(x.double().numpy())
    c = rq.resq_gram_accumulate(x.cuda())
    torch.cuda.synchronize()
    got = c.double().cpu().numpy()
    # fp32 accumulation of T exact products: error <= T * 2^-24 * sum |x_i x_j|, far below this
    bound = 4 * T * 2.0 ** -24 * (np.abs(x.double().numpy()).T @ np.abs(x.double().numpy())) + 1e-30
    assert np.all(np.abs(got - ref) <= bound)
    # accumulates: a second call with other tokens adds
    x2 = calib(T + K + 1, 130, K)
    rq.resq_gram_accumulate(x2.cuda(), c)
    torch.cuda.synchronize()
    ref2 = ref + bo.gram(x2.double().numpy())
    assert np.allclose(c.double().cpu().numpy(), ref2, rtol=1e-4, atol=1e-4 * np.abs(ref2).max())


def test_gram_strided_rows_and_untouched_padding(rq):
    T, K = 200, 72
    buf = torch.randn(T, K + 24).to(torch.bfloat16)
    cbuf = torch.full((K, K + 8), 7.0, dtype=torch.float32, device="cuda")
    cbuf[:, :K] = 0
    rq.resq_gram_accumulate(buf.cuda()[:, :K], cbuf[:, :K])
    torch.cuda.synchronize()
    assert torch.all(cbuf[:, K:] == 7.0)
    assert np.allclose(cbuf[:, :K].double().cpu().numpy(), bo.gram(buf[:, :K].double().numpy()), rtol=1e-4, atol=1e-3)


@pytest.mark.parametrize("rows,K,J,a_dtype,out_dtype", [
    (300, 128, 128, torch.bfloat16, torch.bfloat16), (130, 256, 64, torch.float32, torch.float32),
    (7, 72, 8, torch.bfloat16, torch.float32), (257, 1000, 264, torch.float32, torch.bfloat16),
    (1, 16, 16, torch.float32, torch.float32),
])
def test_project_rows(rq, rows, K, J, a_dtype, out_dtype):
    g = torch.Generator().manual_seed(rows + K + J)
    a = torch.randn(rows, K, generator=g).to(a_dtype)
    u = torch.randn(K, J, generator=g) / K ** 0.5
    ref = bo.project(a.double().numpy(), u.double().numpy())
    out = rq.resq_project_rows(a.cuda(), u.cuda(), out_dtype=out_dtype)
    torch.cuda.synchronize()
    got = out.double().cpu().numpy()
    mag = np.abs(a.double().numpy()) @ np.abs(u.double().numpy())
    if out_dtype == torch.bfloat16:
        # fp32 result rounded once more to bf16
        assert np.all(np.abs(got - ref) <= 2.0 ** -8 * np.abs(ref) + 4 * K * 2.0 ** -24 * mag)
    else:
        assert np.all(np.abs(got - ref) <= 4 * K * 2.0 ** -24 * mag + 1e-30)


def test_project_rows_on_column_blocks(rq):
    # U_h = P_h R_h written into the first r columns of U: sub-blocks in and out
    K, r = 64, 16
    p = wl.random_orthogonal(K, 3).contiguous().cuda()
    r_h = wl.random_orthogonal(r, 4).contiguous().cuda()
    u = torch.zeros(K, K, device="cuda")
    rq.resq_project_rows(p[:, :r], r_h, out=u[:, :r])
    torch.cuda.synchronize()
    assert torch.all(u[:, r:] == 0)
    assert np.allclose(u[:, :r].double().cpu().numpy(),
                       p[:, :r].double().cpu().numpy() @ r_h.double().cpu().numpy(), atol=1e-6)


@pytest.mark.parametrize("K,r", [(8, 2), (64, 8), (128, 16), (256, 32),
                                 (1024, 128),      # a hidden-size basis of a small model
                                 (4608, 576)])     # two rows of this order need more than 64 KiB of LDS
def test_sym_eig_against_oracle(rq, K, r):
    # planted spectrum with an open gap after the r-th eigenvalue
    sig = np.concatenate([np.linspace(30.0, 20.0, r), np.linspace(4.0, 0.5, K - r)])
    q = wl.random_orthogonal(K, K).double().numpy()
    c = (q * sig ** 2) @ q.T
    c32 = torch.tensor(c, dtype=torch.float32)
    lam_ref, p_ref = bo.pca_basis(c32.double().numpy())
    lam, p = rq.resq_sym_eig(c32.cuda(), sweeps=10 if K <= 256 else 14)
    torch.cuda.synchronize()
    lam, p = lam.double().cpu().numpy(), p.double().cpu().numpy()
    scale = lam_ref[0]
    assert np.all(np.diff(lam) <= 0)
    assert np.allclose(lam, lam_ref, atol=1e-6 * scale)          # fp32 outputs of an fp64 iteration
    assert np.allclose(p.T @ p, np.eye(K), atol=1e-5)             # orthonormal columns
    # eigenpairs of the input; the fp32 rounding of the K entries of a vector adds up in c @ p
    assert np.abs(c32.double().numpy() @ p - p * lam).max() <= (1e-5 if K <= 256 else 4e-5) * scale
    # the high-precision subspace is the oracle's
    assert np.allclose(p[:, :r] @ p[:, :r].T, p_ref[:, :r] @ p_ref[:, :r].T, atol=1e-4)


def test_sym_eig_repeated_eigenvalues_and_diagonal_input(rq):
    # a matrix that is already diagonal with a repeated value: sorted, vectors a permutation
    d = np.array([3.0, 1.0, 3.0, 2.0, 0.0, 5.0, 1.0, 4.0])
    lam, p = rq.resq_sym_eig(torch.tensor(np.diag(d), dtype=torch.float32).cuda(), sweeps=3)
    torch.cuda.synchronize()
    assert np.array_equal(lam.cpu().numpy(), np.sort(d)[::-1].astype(np.float32))
    pp = p.double().cpu().numpy()
    assert np.allclose(pp.T @ pp, np.eye(8), atol=1e-12) and np.allclose(np.abs(pp).sum(0), 1.0)


def test_basis_end_to_end_raises_layer_snr(rq):
    # the whole offline path on the GPU (Gram matrix, PCA, U = P blockdiag(R), X U, W U), then
    # the layer on the projected operands: the output SNR against the unprojected fp64 product
    # must equal what the oracle's basis gives, and beat quantizing the raw operands
    from oracle import resq_oracle as oracle
    oracle.build()
    K, N, T, r = 128, 96, 512, 16
    x = calib(5, T, K)
    g = torch.Generator().manual_seed(6)
    w = (torch.randn(N, K, generator=g) * 0.02).to(torch.bfloat16)
    r_h, r_l = wl.random_orthogonal(r, 1).contiguous(), wl.random_orthogonal(K - r, 2).contiguous()
    xd, wd = x.cuda(), w.cuda()
    c = rq.resq_gram_accumulate(xd)
    lam, p = rq.resq_sym_eig(c, sweeps=10)
    u = torch.empty(K, K, device="cuda")
    rq.resq_project_rows(p[:, :r], r_h.cuda(), out=u[:, :r])
    rq.resq_project_rows(p[:, r:], r_l.cuda(), out=u[:, r:])
    xr = rq.resq_project_rows(xd, u)
    wr = rq.resq_project_rows(wd, u)
    y = rq.resq_gemm_mixed(rq.resq_quantize_act(xr, r), rq.resq_pack_weights(wr, r), N)
    torch.cuda.synchronize()
    un = u.double().cpu().numpy()
    assert np.allclose(un.T @ un, np.eye(K), atol=1e-5)
    ref = x.double().numpy() @ w.double().numpy().T
    snr_gpu = oracle.snr_db(ref, y.float().cpu().numpy())
    # the oracle's own path
    _, p_o = bo.pca_basis(bo.gram(x.double().numpy()))
    u_o = bo.compose_basis(p_o, r_h.double().numpy(), r_l.double().numpy())
    xo = bo.f64_to_bf16_bits(bo.project(x.double().numpy(), u_o))
    wo = bo.f64_to_bf16_bits(bo.project(w.double().numpy(), u_o))
    snr_cpu = oracle.snr_db(ref, oracle.linear(xo, wo, r).y)
    snr_raw = oracle.snr_db(ref, oracle.linear(wl.bf16_bits(x), wl.bf16_bits(w), r).y)
    # eigenvector signs differ, so codes differ: the SNRs agree statistically, not bitwise
    assert abs(snr_gpu - snr_cpu) < 1.0, (snr_gpu, snr_cpu)
    assert snr_gpu > snr_raw + 6.0, (snr_gpu, snr_raw)
    # the span of the high group is the oracle's
    ph = p[:, :r].double().cpu().numpy()
    assert np.allclose(ph @ ph.T, p_o[:, :r] @ p_o[:, :r].T, atol=1e-3)
