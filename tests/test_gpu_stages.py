"""Stage hooks on the GPU: the Householder stage (Sec. 3.1) and the shifted QR
stage (Sec. 3.2) are pinned separately so that a failure can be localised."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def _to_dev(x):
    import torch
    return torch.from_numpy(np.ascontiguousarray(x)).to("cuda:0")


@pytest.mark.parametrize("n", [3, 4, 8, 13, 16, 24, 32, 48, 64])
def test_tridiag_stage(n):
    import torch
    from oracle import jacobi
    from paper_2207_04228_amd import binding
    print(f"[tridiag] n={n}", flush=True)
    rng = np.random.default_rng(300 + n)
    A = rng.standard_normal((19, n, n))
    A = (0.5 * (A + A.transpose(0, 2, 1))).astype(np.float32)
    d, e, P = binding.bed_tridiag(_to_dev(A))
    torch.cuda.synchronize()
    d, e, P = d.cpu().numpy().astype(np.float64), e.cpu().numpy().astype(np.float64), P.cpu().numpy().astype(np.float64)
    assert np.all(e[:, n - 1] == 0)
    T = np.zeros((19, n, n))
    idx = np.arange(n)
    T[:, idx, idx] = d
    T[:, idx[1:], idx[:-1]] = e[:, :n - 1]
    T[:, idx[:-1], idx[1:]] = e[:, :n - 1]
    A64 = A.astype(np.float64)
    I = np.eye(n)[None]
    orth = np.sqrt(((P.transpose(0, 2, 1) @ P - I) ** 2).sum(axis=(1, 2)))
    assert orth.max() <= 1e-5 * n
    rec = P @ T @ P.transpose(0, 2, 1) - A64
    rel = np.sqrt((rec ** 2).sum(axis=(1, 2))) / np.sqrt((A64 ** 2).sum(axis=(1, 2)))
    assert rel.max() <= 1e-5 * n
    # first row/column of P are those of the identity (column 0 is reduced first)
    assert np.allclose(P[:, 0, 0], 1.0) and np.allclose(P[:, 0, 1:], 0.0) and np.allclose(P[:, 1:, 0], 0.0)
    # similarity: same spectrum
    lam_A, _ = jacobi.syevd(A)
    lam_T, _ = jacobi.syevd(T)
    assert np.abs(lam_A - lam_T).max() <= 1e-5 * np.abs(lam_A).max()
    # implicit-Q uniqueness (Sec. 3.2.5): |d|, |e| agree with a library Hessenberg reduction
    import scipy.linalg
    H = scipy.linalg.hessenberg(A64[0])
    assert np.allclose(np.diag(H), d[0], atol=2e-5 * np.abs(lam_A).max())
    assert np.allclose(np.abs(np.diag(H, -1)), np.abs(e[0, :n - 1]), atol=2e-5 * np.abs(lam_A).max())


@pytest.mark.parametrize("n", [2, 5, 8, 16, 31, 32, 64])
def test_qr_stage_on_toeplitz_closed_form(n):
    import torch
    from paper_2207_04228_amd import binding
    print(f"[qr-stage] toeplitz n={n}", flush=True)
    d = np.full((3, n), 2.0, dtype=np.float32)
    e = np.full((3, n), -1.0, dtype=np.float32)
    ev, V, info, rot = binding.bed_tridiag_qr(_to_dev(d), _to_dev(e))
    torch.cuda.synchronize()
    k = np.arange(1, n + 1)
    expect = 2.0 - 2.0 * np.cos(k * np.pi / (n + 1))
    assert np.abs(ev.cpu().numpy() - expect[None]).max() <= 1e-5 * 4.0
    S = np.sin(np.outer(k, k) * np.pi / (n + 1)) * np.sqrt(2.0 / (n + 1))
    Vn = V.cpu().numpy().astype(np.float64)
    dots = np.abs(np.einsum("bij,ij->bj", Vn, S))
    gaps = np.minimum(np.diff(expect, prepend=-np.inf), np.diff(expect, append=np.inf))
    assert np.all(1.0 - dots[:, gaps > 5e-3 * 4.0] < 1e-5)
    assert np.all(info.cpu().numpy() == 0)


@pytest.mark.parametrize("n", [4, 16, 32, 64])
def test_qr_stage_random_tridiagonal_vs_library(n):
    import scipy.linalg
    import torch
    from paper_2207_04228_amd import binding
    print(f"[qr-stage] random n={n}", flush=True)
    rng = np.random.default_rng(500 + n)
    d = rng.standard_normal((11, n)).astype(np.float32)
    e = rng.standard_normal((11, n)).astype(np.float32)
    ev, V, info, rot = binding.bed_tridiag_qr(_to_dev(d), _to_dev(e))
    torch.cuda.synchronize()
    ev = ev.cpu().numpy()
    for b in range(11):
        ref = scipy.linalg.eigh_tridiagonal(d[b].astype(np.float64), e[b, :n - 1].astype(np.float64),
                                            eigvals_only=True)
        assert np.abs(ev[b] - ref).max() <= 1e-5 * np.abs(ref).max()
    Vn = V.cpu().numpy().astype(np.float64)
    G = Vn.transpose(0, 2, 1) @ Vn - np.eye(n)
    assert np.sqrt((G * G).sum(axis=(1, 2))).max() <= 1e-5 * n
