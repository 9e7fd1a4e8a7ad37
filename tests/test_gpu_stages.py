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


def _explicit_double_shift_step(d, e):
    """One outer iteration written out with explicit QR factorisations in float64
    (Sec. 3.2.1 and Eq. (15)): both shifts are the eigenvalues of the trailing 2x2 block of
    T_k, the one closer to the last diagonal entry first; T_{k+1/2} = R Q + mu_1 I from
    T_k - mu_1 I = Q R, then the same with mu_2 on T_{k+1/2}."""
    n = d.size
    T = np.diag(d) + np.diag(e[:n - 1], 1) + np.diag(e[:n - 1], -1)
    a, b, c = T[n - 2, n - 2], T[n - 2, n - 1], T[n - 1, n - 1]
    mus = np.linalg.eigvalsh(np.array([[a, b], [b, c]]))
    mu1, mu2 = (mus[0], mus[1]) if abs(mus[0] - c) <= abs(mus[1] - c) else (mus[1], mus[0])
    Qtot = np.eye(n)
    for mu in (mu1, mu2):
        Q, R = np.linalg.qr(T - mu * np.eye(n))
        T = R @ Q + mu * np.eye(n)
        Qtot = Qtot @ Q
    return T, Qtot


@pytest.mark.parametrize("n", [3, 5, 8, 16, 24, 32, 33, 48, 64])
def test_one_iteration_is_two_explicit_qr_steps_with_the_shifts_of_the_same_matrix(n):
    import torch
    from paper_2207_04228_amd import binding
    print(f"[qr-stage] one double-shift iteration, n={n}", flush=True)
    rng = np.random.default_rng(600 + n)
    batch = 6
    d = rng.uniform(-1.0, 1.0, size=(batch, n)).astype(np.float32)
    e = rng.uniform(0.2, 1.0, size=(batch, n)).astype(np.float32) * rng.choice([-1.0, 1.0], size=(batch, n)).astype(np.float32)
    d1, e1, Q, rot = binding.bed_tridiag_qr_sweeps(_to_dev(d), _to_dev(e), 2)
    torch.cuda.synchronize()
    d1, e1, Q = d1.cpu().numpy().astype(np.float64), e1.cpu().numpy().astype(np.float64), Q.cpu().numpy().astype(np.float64)
    assert (rot.cpu().numpy() == 2 * (n - 1)).all()              # two sweeps over the whole matrix
    for b in range(batch):
        T_ref, Q_ref = _explicit_double_shift_step(d[b].astype(np.float64), e[b].astype(np.float64))
        scale = np.abs(T_ref).max()
        # (the trailing entries after a sweep with a shift close to an eigenvalue are
        # ill-conditioned functions of the shift; a float32 shift moves them by ~1e-5.
        # A different shift strategy, e.g. a second shift taken from T_{k+1/2}, moves them by
        # 1e-2 and more.)
        errs = (np.abs(d1[b] - np.diag(T_ref)).max() / scale,
                np.abs(np.abs(e1[b, :n - 1]) - np.abs(np.diag(T_ref, -1))).max() / scale,
                np.abs(np.abs(Q[b].T @ Q_ref) - np.eye(n)).max())
        print(f"[qr-stage] n={n} b={b}: d {errs[0]:.1e} e {errs[1]:.1e} Q {errs[2]:.1e}", flush=True)
        assert errs[0] <= 3e-4 and errs[1] <= 3e-4
        # the rotations: Q = Q_1 Q_2 up to the signs of its columns, and T_out = Q^T T Q
        assert errs[2] <= 2e-3
        T0 = np.diag(d[b].astype(np.float64)) + np.diag(e[b, :n - 1].astype(np.float64), 1) + np.diag(e[b, :n - 1].astype(np.float64), -1)
        T1 = np.diag(d1[b]) + np.diag(e1[b, :n - 1], 1) + np.diag(e1[b, :n - 1], -1)
        assert np.abs(Q[b].T @ T0 @ Q[b] - T1).max() <= 2e-5 * scale * np.sqrt(n)
