"""Parity of bed_spd_fn (V f(max(Lambda, floor)) V^T in one launch) with the
float64 spectral oracle.

Tolerance.  The kernel applies f to the spectrum of A + E, where E is the
backward error of the float32 eigendecomposition, ||E|| <= r ||A||_2 with
r = 1e-6 n (ten times tighter than the residual bar of the eigensolver itself,
about five times what is observed).  For a symmetric
matrix function ||f(A+E) - f(A)|| <= L ||E|| with L the largest |f'| on the
(floored) spectrum, so relative to ||f(A)||_2:

  sqrt       L = 1/(2 sqrt(lmin)),  ||f(A)|| = sqrt(lmax)   -> r * sqrt(cond)/2,
             and never more than sqrt(r) because |sqrt a - sqrt b| <= sqrt|a-b|
  inv sqrt   L = 1/(2 lmin^1.5),    ||f(A)|| = lmin^-0.5    -> r * cond/2

with lmin the floored smallest eigenvalue and cond = lmax / lmin; the bar is
r * (1 + that factor), evaluated in float64 per matrix.
"""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

R = 1e-6


def _gpu(A32, fn, floor, want_evals=True):
    import torch
    from paper_2207_04228_amd import binding
    At = torch.from_numpy(A32).to("cuda:0")
    out, ev, info = binding.bed_spd_fn(At, fn, floor, want_evals=want_evals)
    torch.cuda.synchronize()
    assert torch.equal(At.cpu(), torch.from_numpy(A32)), "input was modified"
    return out.cpu().numpy().astype(np.float64), None if ev is None else ev.cpu().numpy(), info.cpu().numpy()


def _check(A32, fn, floor, name):
    from oracle import jacobi, spectral
    print(f"[spd_fn] {name} fn={fn} floor={floor} shape={A32.shape}", flush=True)
    n = A32.shape[-1]
    lam, _ = jacobi.syevd(A32)
    F_ref = spectral.spd_fn(A32, fn, floor)
    F, ev, info = _gpu(A32, fn, floor)
    assert (info == 0).all()
    assert np.isfinite(F).all()
    lmax = np.abs(lam).max(axis=1)
    lmin = np.maximum(lam.min(axis=1), floor)
    r = R * n
    if fn == spectral.FN_SQRT:
        with np.errstate(divide="ignore"):
            factor = np.minimum(0.5 * np.sqrt(lmax / lmin), 1.0 / np.sqrt(r))
    else:
        factor = 0.5 * lmax / lmin
    tol = r * (1.0 + factor)
    norm = np.linalg.norm(F_ref, ord=2, axis=(1, 2))
    err = np.abs(F - F_ref).max(axis=(1, 2)) / norm
    sym = np.abs(F - np.swapaxes(F, 1, 2)).max(axis=(1, 2)) / norm
    worst = int(np.argmax(err / tol))
    print(f"[spd_fn] {name}: max err/norm {err.max():.2e} (tol there {tol[np.argmax(err)]:.2e}), "
          f"worst err/tol {err[worst] / tol[worst]:.3f}, asym {sym.max():.2e}", flush=True)
    assert (err <= tol).all()
    assert (sym <= 2 * tol).all()
    assert np.abs(ev - lam).max() <= 1e-5 * lmax.max()
    assert np.all(np.diff(ev, axis=1) >= 0)
    return F


@pytest.mark.parametrize("fn", [0, 1])
def test_headline_sizes(fn):
    from paper_2207_04228_amd import workloads
    for n, A32 in workloads.headline_points():
        _check(A32, fn, 1e-6, f"headline n={n}")


@pytest.mark.parametrize("fn", [0, 1])
def test_clustered_and_medium(fn):
    from paper_2207_04228_amd import workloads
    _check(workloads.config1(), fn, 1e-6, "config1")
    _check(workloads.config4(batch=256), fn, 1e-6, "config4")
    for n in (48, 64):
        A = workloads.config5(n, batch=32)
        _check(A, fn, 1e-2, f"config5 n={n} (power-law spectrum, floored at 1e-2)")
        _check(A, 0, 0.0, f"config5 n={n} sqrt unfloored")


@pytest.mark.parametrize("n", [1, 2, 3, 5, 7, 13, 24, 31, 33, 47, 63])
def test_ragged_n(n):
    from paper_2207_04228_amd import workloads
    A = workloads.covariance(37, n, 2 * n + 3, 0.05, 991 + n)
    _check(A, 0, 0.0, f"ragged n={n}")
    _check(A, 1, 1e-6, f"ragged n={n}")


def test_defining_identities_at_headline_size():
    """(A^1/2)^2 = A and A^-1/2 A A^-1/2 = I, checked against the input itself (no oracle)."""
    from oracle.acceptance import mirror_lower
    from paper_2207_04228_amd import workloads
    for n, A32 in workloads.headline_points():
        A = mirror_lower(A32)
        S, _, _ = _gpu(A32, 0, 0.0)
        W, _, _ = _gpu(A32, 1, 1e-12)
        lam = np.linalg.eigvalsh(A)
        cond = lam[:, -1] / lam[:, 0]
        scale = np.linalg.norm(A, ord=2, axis=(1, 2))
        e1 = np.abs(S @ S - A).max(axis=(1, 2)) / scale
        e2 = np.abs(W @ A @ W - np.eye(n)).max(axis=(1, 2))
        print(f"[spd_fn] identities n={n}: sqrt^2 {e1.max():.2e}  whitening {e2.max():.2e} "
              f"(cond up to {cond.max():.1f})", flush=True)
        assert (e1 <= 2 * R * n).all()
        assert (e2 <= 2 * R * n * cond).all()


def test_floor_on_indefinite_and_singular_input():
    from paper_2207_04228_amd import workloads
    rng = np.random.default_rng(5)
    lam = np.tile(np.array([-0.5, -1e-4, 0.0, 1e-7, 1e-3, 0.3, 1.0, 2.0]), (64, 1))
    A = workloads.from_spectrum(lam, seed=77)
    _check(A, 1, 1e-2, "indefinite, inverse sqrt floored at 1e-2")
    _check(A, 0, 1e-2, "indefinite, sqrt floored at 1e-2")
    Z = np.zeros((3, 6, 6), dtype=np.float32)
    F, ev, info = _gpu(Z, 1, 0.25)
    assert np.allclose(F, 2.0 * np.eye(6)[None], atol=1e-6) and (ev == 0).all() and (info == 0).all()
    D = np.stack([np.diag(rng.uniform(0.5, 4.0, 5)) for _ in range(4)]).astype(np.float32)
    F, _, _ = _gpu(D, 0, 0.0)
    assert np.allclose(F, np.sqrt(D.astype(np.float64)), atol=1e-6)


def test_without_eigenvalue_output_and_batch_edges():
    import torch
    from paper_2207_04228_amd import binding, workloads
    A32 = workloads.config3(16, batch=70)
    F1, _, _ = _gpu(A32, 1, 1e-6, want_evals=False)
    F2, _, _ = _gpu(A32, 1, 1e-6, want_evals=True)
    assert np.array_equal(F1, F2)
    one, _, _ = _gpu(A32[:1].copy(), 1, 1e-6)
    assert np.array_equal(one[0], F1[0])
    empty = torch.empty((0, 16, 16), dtype=torch.float32, device="cuda:0")
    out, _, info = binding.bed_spd_fn(empty, 0, 0.0)
    assert out.shape == (0, 16, 16) and info.numel() == 0
    with pytest.raises(binding.BedError):
        binding.bed_spd_fn(torch.from_numpy(A32).to("cuda:0"), 1, 0.0)       # inverse sqrt needs floor > 0
    with pytest.raises(binding.BedError):
        binding.bed_spd_fn(torch.from_numpy(A32).to("cuda:0"), 2, 1.0)       # unknown function


def test_large_batch_small_n():
    from paper_2207_04228_amd import workloads
    _check(workloads.config2(20000), 1, 1e-6, "config2 batch 20000 (n=4)")


@pytest.mark.parametrize("fn", [0, 1])
def test_where_the_packed_and_lane_kernels_are_dispatched(fn):
    """The fused spectral function at the batch sizes that go to four matrices per wavefront
    (n <= 16 from batch 2560, 16 < n <= 32 from batch 4096) and to one matrix per lane (n <= 4 from batch 20480, n <= 8 from batch
    32768), ragged last wavefronts included; 65536 matrices of 4 x 4 are the shape of App. B.3."""
    from paper_2207_04228_amd import binding, workloads
    cases = [("packed_kernel<16>", workloads.config4()),
             ("packed_kernel<12>", workloads.covariance(2560 + 3, 12, 48, 1e-4, 61)),
             ("packed_kernel<8>", workloads.config3(8, batch=4096 + 1)),
             ("packed_kernel<4>", workloads.config2(4096)),
             ("packed_rows_kernel<32>", workloads.config3(32, batch=4096 + 5)),
             ("packed_rows_kernel<24>", workloads.covariance(4096 + 2, 21, 84, 1e-4, 65)),
             ("packed_rows_kernel<20>", workloads.covariance(4096, 17, 68, 1e-4, 66)),
             ("lane_kernel<4>", workloads.config2(65536)),
             ("lane_kernel<4>", workloads.covariance(20480 + 64 + 13, 3, 16, 1e-3, 62)),
             ("lane_kernel<8>", workloads.config3(8, batch=32768 + 7)),
             ("lane_kernel<8>", workloads.covariance(32768 + 64, 6, 24, 1e-4, 63))]
    for variant, A in cases:
        assert binding.bed_kernel_variant(A.shape[0], A.shape[-1]) == variant
        _check(A, fn, 1e-6, f"{variant} batch {A.shape[0]} n={A.shape[-1]}")


def test_floor_and_degenerate_rows_in_the_packed_and_lane_kernels():
    """Zero, diagonal and indefinite matrices inside large batches: the floor acts per matrix."""
    from paper_2207_04228_amd import workloads
    for batch, n in ((4096, 8), (32768, 8), (20480, 4), (4096, 24)):
        A = workloads.covariance(batch, n, 4 * n, 1e-4, 64 + n).copy()
        A[5] = 0.0
        A[6] = np.diag(np.linspace(0.5, 4.0, n)).astype(np.float32)
        A[7] = -A[7]
        F, ev, info = _gpu(A, 1, 0.25)
        assert (info == 0).all()
        assert np.allclose(F[5], 2.0 * np.eye(n), atol=1e-6) and (ev[5] == 0).all()
        assert np.allclose(F[6], np.diag(1.0 / np.sqrt(np.maximum(np.linspace(0.5, 4.0, n), 0.25))), atol=1e-6)
        assert np.allclose(F[7], 2.0 * np.eye(n), atol=1e-5)        # every eigenvalue negative: all floored
