"""Pins for the backward oracle (float64): finite differences of the forward
oracles, textbook closed forms, and the series identity of the Taylor coupling."""
import numpy as np
import pytest

from oracle import backward, jacobi, spectral
from paper_2207_04228_amd import workloads


def _sym(rng, n):
    E = rng.standard_normal((n, n))
    return 0.5 * (E + E.T)


def _eig_signed(A, Vref=None):
    lam, V = jacobi.syevd(A[None])
    lam, V = lam[0], V[0]
    if Vref is not None:                       # same sign choice as the reference decomposition
        V = V * np.sign(np.sum(V * Vref, axis=0))[None, :]
    return lam, V


@pytest.mark.parametrize("n", [2, 3, 5, 8])
def test_eigendecomposition_gradient_matches_finite_differences(n):
    rng = np.random.default_rng(100 + n)
    lam0 = np.sort(rng.uniform(0.5, 1.0, n)) + np.arange(n)          # gaps >= 0.5
    A = workloads.from_spectrum(lam0[None], seed=7 + n)[0].astype(np.float64)
    lam, V = _eig_signed(A)
    w = rng.standard_normal(n)
    W = rng.standard_normal((n, n))
    loss = lambda l, v: float(w @ l + np.sum(W * v))
    gA = backward.syevd_backward(lam[None], V[None], w[None], W[None], backward.MODE_EXACT, 0.0)[0]
    assert np.allclose(gA, gA.T, atol=1e-12)
    h = 1e-6
    for trial in range(4):
        E = _sym(rng, n)
        lp, Vp = _eig_signed(A + h * E, V)
        lm, Vm = _eig_signed(A - h * E, V)
        fd = (loss(lp, Vp) - loss(lm, Vm)) / (2 * h)
        assert abs(fd - np.sum(gA * E)) <= 1e-6 * (1 + abs(fd)), (trial, fd, np.sum(gA * E))


def test_textbook_gradients_of_trace_and_frobenius_norm():
    A = workloads.config3(8, batch=5).astype(np.float64)
    lam, V = jacobi.syevd(A)
    n = 8
    gA = backward.syevd_backward(lam, V, np.ones_like(lam), None)
    assert np.allclose(gA, np.eye(n)[None], atol=1e-12)              # d tr(A) / dA = I
    gA = backward.syevd_backward(lam, V, 2 * lam, None)
    assert np.allclose(gA, 2 * A, atol=1e-12)                        # d ||A||_F^2 / dA = 2A
    # a loss that depends on V only through V V^T = I has zero gradient: g_V = V S, S symmetric
    S = np.random.default_rng(1).standard_normal((5, n, n))
    S = S + np.swapaxes(S, 1, 2)
    gA = backward.syevd_backward(lam, V, None, V @ S)
    assert np.abs(gA).max() <= 1e-10


def test_gap_floor_removes_only_the_close_pairs():
    lam = np.array([[1.0, 1.0 + 1e-7, 2.0, 4.0]])
    K = backward.coupling_exact(lam, 1e-3)
    assert K[0, 0, 1] == 0 and K[0, 1, 0] == 0
    assert K[0, 0, 2] == pytest.approx(1.0) and K[0, 2, 0] == pytest.approx(-1.0)
    assert K[0, 2, 3] == pytest.approx(0.5) and np.all(np.diagonal(K[0]) == 0)
    assert np.allclose(K, -np.swapaxes(K, 1, 2))


@pytest.mark.parametrize("degree", [0, 1, 9, 30])
def test_taylor_coupling_is_the_truncated_geometric_series(degree):
    """sum_{k<=D} r^k = (1 - r^(D+1)) / (1 - r): the truncated coupling equals the exact one
    times (1 - r^(D+1)), r = smaller/larger eigenvalue; for equal eigenvalues it is (D+1)/lambda."""
    rng = np.random.default_rng(2)
    lam = np.sort(rng.uniform(0.1, 3.0, (6, 7)), axis=1)
    K = backward.coupling_taylor(lam, degree)
    Kx = backward.coupling_exact(lam, 0.0)
    a, b = lam[:, :, None], lam[:, None, :]
    r = np.minimum(a, b) / np.maximum(a, b)
    off = ~np.eye(7, dtype=bool)
    assert np.allclose(K[:, off], (Kx * (1 - r ** (degree + 1)))[:, off], rtol=1e-10)
    assert np.allclose(K, -np.swapaxes(K, 1, 2))
    # equal eigenvalues: finite, (D+1)/lambda in magnitude, and still antisymmetric
    lam2 = np.array([[0.7, 0.7, 0.7, 1.9]])
    K2 = backward.coupling_taylor(lam2, degree)
    assert K2[0, 0, 1] == pytest.approx((degree + 1) / 0.7) and K2[0, 1, 2] == pytest.approx((degree + 1) / 0.7)
    assert np.array_equal(K2, -np.swapaxes(K2, 1, 2))


def test_taylor_gradient_converges_to_the_exact_one():
    A = workloads.config4(batch=3, n=16)
    lam, V = jacobi.syevd(A)
    rng = np.random.default_rng(3)
    gV = rng.standard_normal(V.shape)
    exact = backward.syevd_backward(lam, V, None, gV, backward.MODE_EXACT, 0.0)
    errs = [np.abs(backward.syevd_backward(lam, V, None, gV, backward.MODE_TAYLOR, degree=d) - exact).max()
            for d in (9, 100, 2000)]
    assert errs[0] > errs[1] > errs[2] and errs[2] <= 1e-6 * np.abs(exact).max()


@pytest.mark.parametrize("fn", [spectral.FN_SQRT, spectral.FN_INV_SQRT])
@pytest.mark.parametrize("n", [2, 4, 7])
def test_spectral_function_gradient_matches_finite_differences(fn, n):
    rng = np.random.default_rng(200 + n)
    A = workloads.covariance(1, n, 3 * n, 0.05, 300 + n)[0].astype(np.float64)
    G = rng.standard_normal((n, n))
    lam, V = jacobi.syevd(A[None])
    gA = backward.spd_fn_backward(lam, V, G[None], fn, 1e-9)[0]
    assert np.allclose(gA, gA.T, atol=1e-12)
    h = 1e-6
    for trial in range(4):
        E = _sym(rng, n)
        Fp = spectral.spd_fn((A + h * E)[None], fn, 1e-9)[0]
        Fm = spectral.spd_fn((A - h * E)[None], fn, 1e-9)[0]
        fd = np.sum(G * (Fp - Fm)) / (2 * h)
        assert abs(fd - np.sum(gA * E)) <= 1e-6 * (1 + abs(fd)), (trial, fd, np.sum(gA * E))


def test_square_root_gradient_solves_the_sylvester_equation():
    """F = A^(1/2): F dF + dF F = dA, so the adjoint X = g_A satisfies F X + X F = sym(G)."""
    A = workloads.config3(16, batch=4).astype(np.float64)
    lam, V = jacobi.syevd(A)
    F = spectral.spd_fn(A, spectral.FN_SQRT, 0.0)
    G = np.random.default_rng(4).standard_normal(A.shape)
    X = backward.spd_fn_backward(lam, V, G, backward.FN_SQRT, 0.0)
    assert np.allclose(F @ X + X @ F, 0.5 * (G + np.swapaxes(G, 1, 2)), atol=1e-11)


def test_clamped_eigenvalues_carry_no_gradient_of_their_own():
    Q = workloads.haar_orthogonal(1, 4, np.random.default_rng(5))[0]
    lam = np.array([1e-4, 2e-4, 0.5, 2.0])
    V = Q
    G = np.random.default_rng(6).standard_normal((4, 4))
    gA = backward.spd_fn_backward(lam[None], V[None], G[None], backward.FN_INV_SQRT, 1e-2)[0]
    M = V.T @ gA @ V
    assert np.abs(M[:2, :2]).max() <= 1e-12          # both clamped: the function is constant on that block
    # finite differences through the clamped forward function
    A = (V * lam) @ V.T
    rng = np.random.default_rng(8)
    h = 1e-7
    for _ in range(3):
        E = _sym(rng, 4)
        Fp = spectral.spd_fn((A + h * E)[None], spectral.FN_INV_SQRT, 1e-2)[0]
        Fm = spectral.spd_fn((A - h * E)[None], spectral.FN_INV_SQRT, 1e-2)[0]
        fd = np.sum(G * (Fp - Fm)) / (2 * h)
        assert abs(fd - np.sum(gA * E)) <= 1e-5 * (1 + abs(fd))


_MUTATIONS = {
    "coupling with the opposite sign": ("d = lam[..., None, :] - lam[..., :, None]\n    dd",
                                        "d = lam[..., :, None] - lam[..., None, :]\n    dd"),
    "symmetrisation dropped": ("M = 0.5 * (M + np.swapaxes(M, -1, -2))", "M = M"),
    "g_V^T V instead of V^T g_V": ("C = np.swapaxes(V, -1, -2) @ np.asarray(g_V, dtype=np.float64)",
                                   "C = np.swapaxes(np.asarray(g_V, dtype=np.float64), -1, -2) @ V"),
    "derivative on the diagonal dropped": ("return np.where(same, 0.5 * (fp[..., :, None] + fp[..., None, :]), Phi)",
                                           "return Phi"),
    "series one term short": ("for k in range(degree + 1):", "for k in range(degree):"),
    "wrong sign of the inverse square root's derivative": ("fp = -0.5 * a ** -1.5", "fp = 0.5 * a ** -1.5"),
    "clamped eigenvalues keep their derivative": ("fp = np.where(clamped, 0.0, fp)", "fp = fp"),
}


@pytest.mark.parametrize("name", sorted(_MUTATIONS))
def test_pins_catch_planted_mistakes(name):
    """Each planted mistake in a copy of the oracle must fail at least one pin above."""
    import os
    import types
    src = open(os.path.join(os.path.dirname(backward.__file__), "backward.py")).read()
    old, new = _MUTATIONS[name]
    assert src.count(old) == 1
    mutant = types.ModuleType("backward_mutant")
    mutant.__dict__["__name__"] = "oracle.backward_mutant"
    exec(compile(src.replace(old, new).replace("from __future__ import annotations", ""), "backward_mutant", "exec"),
         mutant.__dict__)
    pins = [lambda: test_eigendecomposition_gradient_matches_finite_differences(5),
            test_textbook_gradients_of_trace_and_frobenius_norm,
            lambda: test_taylor_coupling_is_the_truncated_geometric_series(9),
            lambda: test_spectral_function_gradient_matches_finite_differences(spectral.FN_INV_SQRT, 4),
            lambda: test_spectral_function_gradient_matches_finite_differences(spectral.FN_SQRT, 4),
            test_square_root_gradient_solves_the_sylvester_equation,
            test_clamped_eigenvalues_carry_no_gradient_of_their_own]
    g = globals()
    original = g["backward"]
    g["backward"] = mutant
    try:
        caught = 0
        for pin in pins:
            try:
                pin()
            except AssertionError:
                caught += 1
        assert caught >= 1, f"no pin notices: {name}"
    finally:
        g["backward"] = original
