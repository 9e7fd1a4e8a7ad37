"""64 < n <= 128: the four-wavefront kernel against the CPU oracle, to the same bar as
the smaller sizes (eigenvalues 1e-5 ||A||_2, residual and orthogonality 1e-5 n, subspace
angle 1e-3 for gapped clusters)."""
import numpy as np
import pytest

from test_gpu_parity import _check, _solve_gpu

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("n", [65, 72, 96, 100, 127, 128])
def test_wishart(n):
    from paper_2207_04228_amd import workloads
    _check(workloads.covariance(6, n, 4 * n, 1e-4, 4100 + n), f"wishart n={n}")


@pytest.mark.parametrize("n", [80, 128])
def test_clustered_spectrum(n):
    from paper_2207_04228_amd import workloads
    lam = workloads.clustered_spectrum(4, n, 555 + n)
    _check(workloads.from_spectrum(lam, seed=556 + n), f"clustered n={n}")


def test_degenerate_inputs():
    n = 96
    rng = np.random.default_rng(9)
    mats = [np.zeros((n, n)), np.eye(n), np.diag(rng.standard_normal(n))]
    blk = np.zeros((n, n))
    for s, e in ((0, 30), (30, 31), (31, 96)):
        X = rng.standard_normal((e - s, e - s))
        blk[s:e, s:e] = X + X.T
    mats.append(blk)
    T = np.diag(2.0 * np.ones(n)) - np.diag(np.ones(n - 1), 1) - np.diag(np.ones(n - 1), -1)
    mats.append(T)                                         # already tridiagonal (Toeplitz closed form)
    x = rng.standard_normal(n)
    mats.append(np.outer(x, x) + 0.5 * np.eye(n))          # rank one plus a multiple of the identity
    mats.append(-(np.outer(x, x) + 0.5 * np.eye(n)))       # negative definite
    A = np.stack(mats).astype(np.float32)
    _check(A, "degenerate n=96")
    lam, _ = _solve_gpu(A)
    k = np.arange(1, n + 1)
    assert np.abs(lam[4] - (2 - 2 * np.cos(k * np.pi / (n + 1)))).max() <= 1e-5 * 4


def test_scaling_and_lower_triangle():
    from paper_2207_04228_amd import workloads
    A = workloads.covariance(3, 100, 400, 1e-4, 777)
    for s in (1e-20, 1e18):
        _check((A.astype(np.float64) * s).astype(np.float32), f"scaled by {s:g}")
    B = A.copy()
    iu = np.triu_indices(100, 1)
    B[:, iu[0], iu[1]] = 1e6                               # the upper triangle is never read
    l1, V1 = _solve_gpu(A)
    l2, V2 = _solve_gpu(B)
    assert np.array_equal(l1, l2) and np.array_equal(V1, V2)


def test_eigenvalues_only_info_and_nan():
    import torch
    from paper_2207_04228_amd import binding, workloads
    A = workloads.covariance(5, 128, 512, 1e-4, 778)
    lam_full, _ = _solve_gpu(A)
    lam_only, none = _solve_gpu(A, want_vectors=False)
    assert none is None
    assert np.abs(lam_full - lam_only).max() <= 1e-5 * np.abs(lam_full).max()
    lam, V, info, rot = _solve_gpu(A, info=True)
    assert (info == 0).all() and (rot > 128).all() and (rot < 40 * 128 * 128).all()
    Bad = A.copy()
    Bad[1, 5, 3] = np.nan
    Bad[3, 90, 90] = np.inf
    lam, V, info, rot = _solve_gpu(Bad, info=True)
    assert info[1] > 0 and info[3] > 0 and info[0] == 0 and info[2] == 0 and info[4] == 0
    assert np.isfinite(lam[[0, 2, 4]]).all() and np.isfinite(V[[0, 2, 4]]).all()


def test_stage_hooks():
    import scipy.linalg
    import torch
    from oracle import jacobi
    from paper_2207_04228_amd import binding, workloads
    A32 = workloads.covariance(3, 90, 360, 1e-4, 779)
    At = torch.from_numpy(A32).to("cuda:0")
    d, e, P = binding.bed_tridiag(At)
    torch.cuda.synchronize()
    d, e, P = d.cpu().numpy().astype(np.float64), e.cpu().numpy().astype(np.float64), P.cpu().numpy().astype(np.float64)
    n = 90
    for b in range(3):
        T = np.diag(d[b]) + np.diag(e[b, :-1], 1) + np.diag(e[b, :-1], -1)
        A = A32[b].astype(np.float64)
        assert np.linalg.norm(P[b].T @ P[b] - np.eye(n)) <= 1e-5 * n
        assert np.linalg.norm(P[b] @ T @ P[b].T - A) / np.linalg.norm(A) <= 1e-5 * n
        # implicit-Q uniqueness (Sec. 3.2.5): d, |e| agree with a library Hessenberg reduction
        H = scipy.linalg.hessenberg(A)
        scale = np.abs(np.linalg.eigvalsh(A)).max()
        dd = np.abs(np.diag(H) - d[b]).max() / scale
        de = np.abs(np.abs(np.diag(H, -1)) - np.abs(e[b, :-1])).max() / scale
        print(f"[tridiag-stage] n={n} b={b}: d {dd:.2e} e {de:.2e}", flush=True)
        # (the entries of T are ill-conditioned functions of A at this size; the decomposition
        # itself is held to the 1e-5 n bar above)
        assert dd <= 1e-3 and de <= 1e-3
    dt = torch.from_numpy(d.astype(np.float32)).to("cuda:0")
    et = torch.from_numpy(e.astype(np.float32)).to("cuda:0")
    ev, Q, info, rot = binding.bed_tridiag_qr(dt, et)
    torch.cuda.synchronize()
    lam_o, _ = jacobi.syevd(A32)
    assert (info.cpu().numpy() == 0).all()
    assert np.abs(ev.cpu().numpy() - lam_o).max() <= 2e-5 * np.abs(lam_o).max()
    Q = Q.cpu().numpy().astype(np.float64)
    assert np.linalg.norm(Q[0].T @ Q[0] - np.eye(n)) <= 1e-5 * n


@pytest.mark.parametrize("fn", [0, 1])
def test_spectral_function(fn):
    from test_gpu_spd_fn import _check as check_fn
    from paper_2207_04228_amd import workloads
    check_fn(workloads.covariance(4, 100, 400, 1e-3, 780), fn, 1e-6, "wishart n=100")
    check_fn(workloads.covariance(3, 128, 300, 1e-2, 781), fn, 1e-6, "wishart n=128")


def test_gradients():
    from test_gpu_backward import _check_ed, _check_fn
    from paper_2207_04228_amd import workloads
    for n in (65, 100, 128):
        A = workloads.covariance(5, n, 4 * n, 1e-3, 782 + n)
        _check_ed(A, 0, f"wishart n={n}", gap_floor=1e-5, seed=n)
        _check_ed(A, 1, f"wishart n={n}", degree=9, seed=n)
        _check_fn(A, 0, 1e-6, f"wishart n={n}", seed=n)
        _check_fn(A, 1, 1e-6, f"wishart n={n}", seed=n)
    lam = workloads.clustered_spectrum(3, 96, 901)
    _check_ed(workloads.from_spectrum(lam, seed=902), 1, "clustered n=96", degree=9, seed=3)
