"""Pins for oracle/lockstep.py (the paper's own fixed-budget iteration in float64): each
building block against a library routine or a closed form, the whole against the exact
spectrum within the bound its dropped off-diagonals allow, and planted mistakes that the
pins must catch.  CPU only."""
import numpy as np
import pytest
import scipy.linalg

from oracle import lockstep
from paper_2207_04228_amd import workloads


def _sym(rng, n):
    A = rng.standard_normal((n, n))
    return (A + A.T) / 2


def _tri(d, e):
    return np.diag(d) + np.diag(e, 1) + np.diag(e, -1)


@pytest.mark.parametrize("n", [3, 4, 7, 16, 33])
def test_householder_matches_definition_and_library(n):
    """Sec. 3.1: A = P T P^T with P orthogonal, P e_1 = e_1, T tridiagonal; by the
    uniqueness of the reduction (Sec. 3.2.5) |d|, |e| equal the library's Hessenberg form."""
    A = _sym(np.random.default_rng(n), n)
    d, e, P = lockstep.householder_tridiagonalize(A)
    T = _tri(d, e)
    assert np.abs(P @ T @ P.T - A).max() <= 1e-13 * n
    assert np.abs(P.T @ P - np.eye(n)).max() <= 1e-14 * n
    assert np.abs(P[:, 0] - np.eye(n)[:, 0]).max() == 0.0
    H = scipy.linalg.hessenberg(A)
    assert np.abs(np.diag(H) - d).max() <= 1e-12
    assert np.abs(np.abs(np.diag(H, -1)) - np.abs(e)).max() <= 1e-12


def test_householder_skips_reduced_columns():
    A = np.diag([3.0, 1.0, 2.0, 5.0])
    A[1, 0] = A[0, 1] = 0.5
    d, e, P = lockstep.householder_tridiagonalize(A)
    assert np.array_equal(P, np.eye(4)) and np.array_equal(d, np.diag(A)) and e[0] == 0.5


@pytest.mark.parametrize("abd", [(2.0, 1.0, 3.0), (3.0, -0.5, 2.0), (1.0, 0.0, 4.0), (5.0, 2.0, 5.0), (-1.0, 1e-9, -1.5)])
def test_wilkinson_pair_is_the_2x2_spectrum(abd):
    """App. A.3: both shifts are the eigenvalues of the block, the first the closer to d."""
    a, b, d = abd
    mu1, mu2 = lockstep.wilkinson_pair(a, b, d)
    ref = np.linalg.eigvalsh(np.array([[a, b], [b, d]]))
    assert np.allclose(sorted((mu1, mu2)), ref, rtol=0, atol=1e-14 * max(1, abs(a), abs(d)))
    assert abs(mu1 - d) <= abs(mu2 - d)
    if a == d:
        assert mu1 < mu2


@pytest.mark.parametrize("n,m", [(5, 5), (8, 8), (8, 5), (12, 2)])
def test_qr_step_is_rq_plus_shift(n, m):
    """Sec. 3.2.1: T - mu I = QR, T' = RQ + mu I, here against numpy's Householder QR
    (signs of the off-diagonals are free); the rest of T is untouched; T' = Q^T T Q."""
    rng = np.random.default_rng(10 * n + m)
    T = _tri(rng.standard_normal(n), rng.standard_normal(n - 1))
    mu = 0.37
    T2, Q = lockstep.qr_step(T, m, mu)
    q, r = np.linalg.qr(T[:m, :m] - mu * np.eye(m))
    ref = r @ q + mu * np.eye(m)
    assert np.abs(np.diag(T2[:m, :m]) - np.diag(ref)).max() <= 1e-13
    assert np.abs(np.abs(np.diag(T2[:m, :m], -1)) - np.abs(np.diag(ref, -1))).max() <= 1e-13
    assert np.abs(Q.T @ T[:m, :m] @ Q - T2[:m, :m]).max() <= 1e-13
    assert np.abs(Q.T @ Q - np.eye(m)).max() <= 1e-14
    assert np.array_equal(T2[m:, :], T[m:, :]) and np.array_equal(T2[:, m:], T[:, m:])
    # the rotations are Givens rotations of adjacent rows: Q is upper Hessenberg
    assert np.abs(np.tril(Q, -2)).max() == 0.0


def test_qr_step_with_exact_eigenvalue_deflates_last_row():
    """A shift equal to an eigenvalue makes the last sub-diagonal vanish (the property
    Sec. 3.2.2 builds on)."""
    rng = np.random.default_rng(3)
    T = _tri(rng.standard_normal(6), rng.standard_normal(5))
    lam = np.linalg.eigvalsh(T)[2]
    T2, _ = lockstep.qr_step(T, 6, lam)
    assert abs(T2[5, 4]) <= 1e-12 and abs(T2[5, 5] - lam) <= 1e-12


@pytest.mark.parametrize("n", [4, 8, 16, 32])
@pytest.mark.parametrize("uniform", [True, False])
@pytest.mark.parametrize("each_step", [True, False])
def test_result_within_the_bound_of_what_was_dropped(n, uniform, each_step):
    """Whatever the budget, diag(T) differs from the exact spectrum by at most the 2-norm
    of the off-diagonal part that is ignored: entries dropped by the shrinking (each at
    most eps) and whatever is left at the end (Weyl; ||E||_2 <= 2 max|e|), and A V = V T
    holds for the similarity that was actually applied."""
    A = (workloads.config1()[:6] if n == 4 else workloads.config3(n, batch=6)).astype(np.float64)
    r = lockstep.syevd_lockstep(A, 1e-5, None, uniform, each_step)
    exact = np.linalg.eigvalsh(A)
    bound = 2.0 * np.abs(r.offdiag).max(axis=1) + 1e-12
    assert np.all(np.abs(r.evals - exact).max(axis=1) <= bound)
    for b in range(len(A)):
        V = r.evecs[b]
        assert np.abs(V.T @ V - np.eye(n)).max() <= 1e-13 * n
        # trace is kept by every similarity step
        assert abs(r.evals[b].sum() - np.trace(A[b])) <= 1e-12 * n
    if uniform:
        assert len(set(r.reductions.tolist())) == 1


@pytest.mark.parametrize("n", [4, 8, 16])
def test_ample_budget_converges_to_the_eigendecomposition(n):
    """With a tight threshold, the test after each step and a generous budget the
    procedure is a complete solver: library spectrum to 1e-10, small residual."""
    A = (workloads.config1()[:8] if n == 4 else workloads.config3(n, batch=8)).astype(np.float64)
    r = lockstep.syevd_lockstep(A, 1e-13, 6 * n, uniform=False, test_each_step=True)
    exact = np.linalg.eigvalsh(A)
    assert np.abs(r.evals - exact).max() <= 1e-10
    assert np.all(r.reductions == n - 1)
    for b in range(len(A)):
        res = np.linalg.norm(A[b] @ r.evecs[b] - r.evecs[b] * r.evals[b]) / np.linalg.norm(A[b])
        assert res <= 1e-10


def test_reduction_times_in_the_range_the_paper_reports():
    """App. C.4 reports reduction times mainly between n/3 and 3n/4 for the budget of n
    iterations; the per-iteration test reproduces that range on covariance-like input
    (mean over the batch; both the batch-uniform and the per-matrix rule)."""
    for n in (16, 24, 32):
        A = workloads.config3(n, batch=16).astype(np.float64)
        for uniform in (True, False):
            r = lockstep.syevd_lockstep(A, 1e-5, None, uniform, False)
            assert n / 3 - 1 <= r.reductions.mean() <= 3 * n / 4, (n, uniform, r.reductions)


# ---- planted mistakes: each must trip one of the pins above --------------------------------

def test_mutation_transposed_rotation_is_caught(monkeypatch):
    def bad_qr_step(T, m, mu, pivots=None):
        M = T[:m, :m] - mu * np.eye(m)
        Q = np.eye(m)
        for k in range(m - 1):
            x1, x2 = M[k, k], M[k + 1, k]
            r = np.hypot(x1, x2)
            c, s = x1 / r, x2 / r
            Gt = np.eye(m)
            Gt[k, k], Gt[k, k + 1], Gt[k + 1, k], Gt[k + 1, k + 1] = c, -s, s, c     # transposed
            M = Gt @ M
            Q = Q @ Gt.T
        out = T.copy()
        out[:m, :m] = M @ Q + mu * np.eye(m)
        return out, Q
    monkeypatch.setattr(lockstep, "qr_step", bad_qr_step)
    with pytest.raises(AssertionError):
        test_qr_step_is_rq_plus_shift(5, 5)


def test_mutation_shift_not_restored_is_caught(monkeypatch):
    good = lockstep.qr_step

    def bad_qr_step(T, m, mu, pivots=None):
        out, Q = good(T, m, mu)
        out[:m, :m] -= mu * np.eye(m)
        return out, Q
    monkeypatch.setattr(lockstep, "qr_step", bad_qr_step)
    with pytest.raises(AssertionError):
        test_result_within_the_bound_of_what_was_dropped(8, False, True)


def test_mutation_swapped_shift_order_is_caught(monkeypatch):
    good = lockstep.wilkinson_pair
    monkeypatch.setattr(lockstep, "wilkinson_pair", lambda a, b, d: good(a, b, d)[::-1])
    with pytest.raises(AssertionError):
        test_wilkinson_pair_is_the_2x2_spectrum((2.0, 1.0, 3.0))


def test_mutation_reflector_without_factor_two_is_caught(monkeypatch):
    def bad(A):
        T = np.array(A, dtype=np.float64)
        n = T.shape[0]
        P = np.eye(n)
        for J in range(n - 2):
            x = T[J + 1:, J]
            sigma = np.linalg.norm(x) * (1.0 if x[0] >= 0.0 else -1.0)
            u = np.zeros(n)
            u[J + 1:] = x
            u[J + 1] += sigma
            H = np.eye(n) - np.outer(u, u) / (u @ u)
            T = H @ T @ H
            P = P @ H
        return np.diag(T).copy(), np.diag(T, -1).copy(), P
    monkeypatch.setattr(lockstep, "householder_tridiagonalize", bad)
    with pytest.raises(AssertionError):
        test_householder_matches_definition_and_library(7)


# ---- what the fixed budget delivers (recorded behaviour of the procedure, not a pin) -------

def test_fixed_budget_accuracy_by_reading():
    """App. B's budget (n iterations, eps 1e-5) on covariance-like 32x32 input: with a
    window shared by the whole batch the spectrum is still O(1e-2) off when the budget
    ends, under either placement of the test; with a window per matrix and the test after
    each step every row deflates and the error is at the level of eps.  This is why the
    GPU path deflates per matrix and runs until convergence."""
    n = 32
    A = workloads.config3(n, batch=16).astype(np.float64)
    exact = np.linalg.eigvalsh(A)
    scale = np.abs(exact).max()
    err = {}
    for uniform in (True, False):
        for each_step in (False, True):
            r = lockstep.syevd_lockstep(A, 1e-5, None, uniform, each_step)
            err[uniform, each_step] = np.abs(r.evals - exact).max() / scale
    assert err[True, False] > 1e-3 and err[True, True] > 1e-3
    assert err[False, True] <= 1e-5
