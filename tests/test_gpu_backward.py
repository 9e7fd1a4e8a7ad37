"""Parity of the gradient kernels (bed_syevd_backward, bed_spd_fn_backward) with the
float64 backward oracle, element by element.  Both sides receive the same float32
eigenvalues and eigenvectors (those the GPU eigensolver wrote) and the same float32
upstream gradients, so the only difference is float32 arithmetic.

Tolerance, from the arithmetic (u = 2^-24, |.| elementwise).  A product accumulates n terms
in sequence; its rounding error is at most n u |X||Y| and, the roundings being independent,
about sqrt(n) u |X||Y| in practice.  C = V^T g_V carries dC ~ |V|^T |g_V|, the coupling
scales it elementwise, M = sym(K o C) + diag(g_lambda) adds a few u |M| of its own, and the
two outer products with the (nearly) orthogonal V add about 2 ||M||_F each way.  The bar is
four times the sqrt(n) estimate,

  max|g_A - g_A^oracle| <= 4 sqrt(n) u ( || |K| o (|V|^T |g_V|) ||_F + 2 ||M||_F ) + 4 u ||M||_F,

evaluated in float64 by the test; it is below the worst-case bound (n in place of 4 sqrt(n),
and a further sqrt(n) on the second term) for n >= 16 and tight enough to notice a loss of
precision in the products, not only a wrong formula.  For the spectral function
C = V^T sym(G) V is two products: the first term doubles, with |V|^T |G| |V| and the divided
differences Phi in place of K.
Where the gap floor decides whether a pair is dropped, the oracle takes the decision on the
float32 difference, as the kernel does.
"""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

U = 2.0 ** -24


def _forward(A32):
    import torch
    from paper_2207_04228_amd import binding
    At = torch.from_numpy(A32).to("cuda:0")
    lam, V = binding.bed_syevd(At)
    torch.cuda.synchronize()
    return lam, V


def _check_ed(A32, mode, name, gap_floor=0.0, degree=9, with_lam=True, with_V=True, seed=0):
    import torch
    from oracle import backward
    from paper_2207_04228_amd import binding
    print(f"[backward] {name} mode={mode} shape={A32.shape}", flush=True)
    batch, n, _ = A32.shape
    rng = np.random.default_rng(seed)
    g_lam = rng.standard_normal((batch, n)).astype(np.float32) if with_lam else None
    g_V = rng.standard_normal((batch, n, n)).astype(np.float32) if with_V else None
    lam, V = _forward(A32)
    to = lambda x: None if x is None else torch.from_numpy(x).to("cuda:0")
    gA = binding.bed_syevd_backward(lam, V, to(g_lam), to(g_V), mode=mode, degree=degree, gap_floor=gap_floor)
    torch.cuda.synchronize()
    gA = gA.cpu().numpy().astype(np.float64)
    lam64, V64 = lam.cpu().numpy().astype(np.float64), V.cpu().numpy().astype(np.float64)
    ref = backward.syevd_backward(lam64, V64, g_lam, g_V, mode, gap_floor, degree, decide_in_float32=True)
    K = (backward.coupling_exact(lam64, gap_floor, True) if mode == backward.MODE_EXACT
         else backward.coupling_taylor(lam64, degree))
    Vt = np.swapaxes(V64, 1, 2)
    M = np.zeros_like(V64)
    T1 = np.zeros(batch)
    if with_V:
        g64 = g_V.astype(np.float64)
        M = K * (Vt @ g64)
        M = 0.5 * (M + np.swapaxes(M, 1, 2))
        T1 = np.linalg.norm(np.abs(K) * (np.abs(Vt) @ np.abs(g64)), axis=(1, 2))
    if with_lam:
        M = M + g_lam.astype(np.float64)[:, :, None] * np.eye(n)
    T2 = np.linalg.norm(M, axis=(1, 2))
    err = np.abs(gA - ref).max(axis=(1, 2))
    tol = 4 * np.sqrt(n) * U * (T1 + 2 * T2) + 4 * U * T2
    if mode == backward.MODE_TAYLOR:
        tol = tol + (degree + 2) * U * T2          # the series is summed in float32, one rounding per term
    w = int(np.argmax(err / np.maximum(tol, 1e-300)))
    print(f"[backward] {name}: max err {err.max():.2e}, worst err/tol {err[w] / max(tol[w], 1e-300):.3f} "
          f"(max|K| up to {np.abs(K).max():.2e})", flush=True)
    assert np.isfinite(gA).all()
    assert (err <= tol).all()
    return gA, ref


@pytest.mark.parametrize("mode", [0, 1])
def test_headline_sizes(mode):
    from paper_2207_04228_amd import workloads
    for n, A32 in workloads.headline_points():
        _check_ed(A32, mode, f"headline n={n}", gap_floor=1e-4, seed=n)


@pytest.mark.parametrize("mode", [0, 1])
def test_clustered_and_medium(mode):
    from paper_2207_04228_amd import workloads
    _check_ed(workloads.config1(), mode, "config1", gap_floor=1e-4, seed=1)
    _check_ed(workloads.config4(batch=256), mode, "config4", gap_floor=1e-6, seed=4)
    for n in (48, 64):
        # repeated and nearly repeated eigenvalues: close pairs are dropped (exact) or bounded (series)
        _check_ed(workloads.config5(n, batch=32), mode, f"config5 n={n}", gap_floor=1e-3, seed=n)


@pytest.mark.parametrize("n", [1, 2, 3, 5, 7, 13, 24, 31, 32, 33, 40, 47, 63, 64])
def test_ragged_n(n):
    from paper_2207_04228_amd import workloads
    A = workloads.covariance(19, n, 2 * n + 3, 0.05, 1991 + n)
    _check_ed(A, 0, f"ragged n={n}", gap_floor=1e-5, seed=n)
    _check_ed(A, 1, f"ragged n={n}", degree=9, seed=n)


def test_single_inputs_and_degrees():
    from paper_2207_04228_amd import workloads
    A = workloads.config3(16, batch=33)
    gA, _ = _check_ed(A, 0, "eigenvalue gradient only", with_V=False, seed=5)
    _check_ed(A, 0, "eigenvector gradient only", gap_floor=1e-5, with_lam=False, seed=6)
    for degree in (0, 1, 20, 64):
        _check_ed(A, 1, f"series of degree {degree}", degree=degree, seed=7)
    # d tr(A) / dA = I: g_lambda = 1, no g_V
    import torch
    from paper_2207_04228_amd import binding
    lam, V = _forward(A)
    ones = torch.ones_like(lam)
    gI = binding.bed_syevd_backward(lam, V, ones, None, mode=0)
    torch.cuda.synchronize()
    assert np.abs(gI.cpu().numpy() - np.eye(16)[None]).max() <= 1e-5


def _check_fn(A32, fn, floor, name, seed=0):
    import torch
    from oracle import backward
    from paper_2207_04228_amd import binding
    print(f"[backward] spd_fn {name} fn={fn} floor={floor} shape={A32.shape}", flush=True)
    batch, n, _ = A32.shape
    G = np.random.default_rng(seed).standard_normal((batch, n, n)).astype(np.float32)
    lam, V = _forward(A32)
    gA = binding.bed_spd_fn_backward(lam, V, torch.from_numpy(G).to("cuda:0"), fn, floor)
    torch.cuda.synchronize()
    gA = gA.cpu().numpy().astype(np.float64)
    lam64, V64 = lam.cpu().numpy().astype(np.float64), V.cpu().numpy().astype(np.float64)
    ref = backward.spd_fn_backward(lam64, V64, G, fn, floor)
    Phi = backward.divided_differences(lam64, fn, floor)
    Vt = np.swapaxes(V64, 1, 2)
    Gs = 0.5 * (G.astype(np.float64) + np.swapaxes(G.astype(np.float64), 1, 2))
    T1 = 2 * np.linalg.norm(np.abs(Phi) * (np.abs(Vt) @ np.abs(Gs) @ np.abs(V64)), axis=(1, 2))
    T2 = np.linalg.norm(Phi * (Vt @ Gs @ V64), axis=(1, 2))
    err = np.abs(gA - ref).max(axis=(1, 2))
    tol = 4 * np.sqrt(n) * U * (T1 + 2 * T2) + 4 * U * T2
    w = int(np.argmax(err / tol))
    print(f"[backward] spd_fn {name}: max err {err.max():.2e}, worst err/tol {err[w] / tol[w]:.3f}", flush=True)
    assert np.isfinite(gA).all()
    assert (err <= tol).all()
    assert np.abs(gA - np.swapaxes(gA, 1, 2)).max() <= 2 * tol.max()


@pytest.mark.parametrize("fn", [0, 1])
def test_spectral_function_gradient(fn):
    from paper_2207_04228_amd import workloads
    for n, A32 in workloads.headline_points():
        _check_fn(A32, fn, 1e-6, f"headline n={n}", seed=n)
    _check_fn(workloads.config4(batch=256), fn, 1e-6, "config4", seed=44)
    for n in (48, 64):
        _check_fn(workloads.config5(n, batch=32), fn, 1e-6, f"config5 n={n}", seed=n)
    for n in (1, 2, 3, 7, 17, 33, 63):
        _check_fn(workloads.covariance(11, n, 2 * n + 3, 0.05, 2991 + n), fn, 1e-6, f"ragged n={n}", seed=n)


def test_spectral_function_gradient_with_clamped_eigenvalues():
    from paper_2207_04228_amd import workloads
    lam = np.tile(np.array([-0.5, -1e-4, 1e-5, 1e-3, 0.02, 0.3, 1.0, 2.0]), (40, 1))
    A = workloads.from_spectrum(lam, seed=78)
    _check_fn(A, 1, 1e-2, "indefinite input, inverse square root floored at 1e-2", seed=3)
    _check_fn(A, 0, 1e-2, "indefinite input, square root floored at 1e-2", seed=4)


def test_whitening_chain_against_finite_differences_of_the_forward_oracle():
    """End to end: loss = <G, A^(-1/2)>; gradient from the GPU (bed_syevd + bed_spd_fn_backward)
    against central differences of the float64 forward oracle."""
    import torch
    from oracle import spectral
    from paper_2207_04228_amd import binding, workloads
    A32 = workloads.config3(8, batch=4)
    rng = np.random.default_rng(12)
    G = rng.standard_normal(A32.shape).astype(np.float32)
    lam, V = _forward(A32)
    gA = binding.bed_spd_fn_backward(lam, V, torch.from_numpy(G).to("cuda:0"), 1, 1e-6)
    torch.cuda.synchronize()
    gA = gA.cpu().numpy().astype(np.float64)
    A = A32.astype(np.float64)
    h = 1e-5
    for trial in range(3):
        E = rng.standard_normal(A.shape)
        E = 0.5 * (E + np.swapaxes(E, 1, 2))
        fd = np.sum(G * (spectral.spd_fn(A + h * E, 1, 1e-6) - spectral.spd_fn(A - h * E, 1, 1e-6)), axis=(1, 2)) / (2 * h)
        an = np.sum(gA * E, axis=(1, 2))
        assert np.all(np.abs(fd - an) <= 2e-4 * (1 + np.abs(fd))), (fd, an)


def test_batch_edges_and_argument_errors():
    import torch
    from paper_2207_04228_amd import binding, workloads
    A = workloads.config3(8, batch=3)
    lam, V = _forward(A)
    g = torch.ones_like(V)
    one = binding.bed_syevd_backward(lam[:1].contiguous(), V[:1].contiguous(), None, g[:1].contiguous())
    allb = binding.bed_syevd_backward(lam, V, None, g)
    torch.cuda.synchronize()
    assert torch.equal(one[0], allb[0])
    e = torch.empty((0, 8), device="cuda:0"), torch.empty((0, 8, 8), device="cuda:0")
    out = binding.bed_syevd_backward(e[0], e[1], e[0], None)
    assert out.shape == (0, 8, 8)
    with pytest.raises(binding.BedError):
        binding.bed_syevd_backward(lam, V, None, None)                       # nothing to propagate
    with pytest.raises(binding.BedError):
        binding.bed_syevd_backward(lam, V, None, g, mode=1, degree=65)
    with pytest.raises(binding.BedError):
        binding.bed_syevd_backward(lam, V, None, g, mode=0, gap_floor=-1.0)
    with pytest.raises(binding.BedError):
        binding.bed_syevd_backward(lam, V, None, g, grad_A=V)                # output aliases an input
    with pytest.raises(binding.BedError):
        binding.bed_spd_fn_backward(lam, V, g, 1, 0.0)                       # inverse square root needs floor > 0
