"""The entry point that allocates nothing (resq_sym_eig_static: the Jacobi eigensolver on the
library's built-in scratch area) against the entry point it is a variant of (resq_sym_eig with
a caller-provided workspace), through the C ABI: same kernels, same arguments, so eigenvalues
and eigenvectors must agree bit for bit, on two calls in a row of which the second is smaller
(it reuses the scratch area that the first left dirty)."""
import numpy as np
import pytest
import torch

from paper_2412_14363_amd import workloads as wl

pytestmark = pytest.mark.gpu


def planted(K, r, seed):
    sig = np.concatenate([np.linspace(30.0, 20.0, r), np.linspace(4.0, 0.5, K - r)])
    q = wl.random_orthogonal(K, seed).double().numpy()
    return torch.tensor((q * sig ** 2) @ q.T, dtype=torch.float32)


def test_sym_eig_static_matches_sym_eig_on_two_calls_in_a_row():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU; there is no CPU fallback")
    from paper_2412_14363_amd import binding as rq
    L = rq.lib()
    st = torch.cuda.current_stream().cuda_stream
    for K, r, sweeps in ((256, 32, 10), (64, 8, 9)):          # the second call is the smaller one
        c = planted(K, r, K + 1).cuda()
        lam = torch.full((K,), -1.0, dtype=torch.float32, device="cuda")
        p = torch.full((K, K + 8), -1.0, dtype=torch.float32, device="cuda")   # ldp > K: padding stays
        rc = L.resq_sym_eig_static(c.data_ptr(), c.stride(0), K, sweeps, lam.data_ptr(), p.data_ptr(),
                                   p.stride(0), st)
        assert rc == 0, rq.STATUS_NAMES.get(rc, rc)
        lam_ref, p_ref = rq.resq_sym_eig(c, sweeps=sweeps)      # caller-provided workspace
        torch.cuda.synchronize()
        assert torch.equal(lam, lam_ref), f"K = {K}: eigenvalues differ"
        assert torch.equal(p[:, :K], p_ref), f"K = {K}: eigenvectors differ"
        assert torch.all(p[:, K:] == -1.0), "wrote past K columns"
        # and they are eigenpairs of the input (the bar of the eigensolver's own parity test)
        pn, ln, cn = p[:, :K].double().cpu().numpy(), lam.double().cpu().numpy(), c.double().cpu().numpy()
        assert np.all(np.diff(ln) <= 0)
        assert np.allclose(pn.T @ pn, np.eye(K), atol=1e-5)
        assert np.abs(cn @ pn - pn * ln).max() <= 1e-5 * ln[0]


def test_sym_eig_static_python_binding_and_size_limit():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU; there is no CPU fallback")
    from paper_2412_14363_amd import binding as rq
    K = 128
    c = planted(K, 16, 3).cuda()
    lam = torch.empty(K, dtype=torch.float32, device="cuda")
    p = torch.empty((K, K), dtype=torch.float32, device="cuda")
    rq.resq_sym_eig_static(c, lam, p, sweeps=10)
    lam_ref, p_ref = rq.resq_sym_eig(c, sweeps=10)
    torch.cuda.synchronize()
    assert torch.equal(lam, lam_ref) and torch.equal(p, p_ref)
    big = torch.eye(514, dtype=torch.float32, device="cuda")
    with pytest.raises(rq.ResqError, match="RESQ_ERR_BUFFER"):
        rq.resq_sym_eig_static(big, torch.empty(514, device="cuda"), torch.empty((514, 514), device="cuda"))
