"""bed_syevd_lockstep (the paper's fixed-budget procedure, Sec. 3.2.3 / App. B) against
oracle/lockstep.py, which writes the same procedure out in float64 with dense matrices.

The iteration is not contractive once rows wait for the rest of the batch (rotations computed
from rounding-level numbers), so float32 and float64 runs can only be compared value by value
over the first iterations; over the whole budget the checks are the identities that hold for
any run of the procedure (similarity, orthogonality, trace, the Weyl bound of what is left)
and a loose comparison of the reduction counts."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def _inputs(n, batch):
    from paper_2207_04228_amd import workloads
    if n <= 4:
        return workloads.covariance(batch, n, 16, 1e-3, 4100 + n)
    return workloads.covariance(batch, n, 4 * n, 1e-4, 4100 + n)


def _run(A, eps, iterations, uniform):
    import torch
    from paper_2207_04228_amd import binding
    ev, V, off, red = binding.bed_syevd_lockstep(torch.from_numpy(A).to("cuda:0"), eps, iterations, uniform)
    torch.cuda.synchronize()
    return (ev.cpu().numpy().astype(np.float64), V.cpu().numpy().astype(np.float64),
            off.cpu().numpy().astype(np.float64), red.cpu().numpy())


def _identities(A, ev, V, off, n):
    A64 = A.astype(np.float64)
    A64 = np.tril(A64) + np.swapaxes(np.tril(A64, -1), 1, 2)
    fro = np.linalg.norm(A64, axis=(1, 2))
    orth = np.linalg.norm(np.swapaxes(V, 1, 2) @ V - np.eye(n), axis=(1, 2))
    assert orth.max() <= 1e-5 * n
    # A V - V diag(evals) = V (T - diag T): its norm is that of the sub-diagonal that is left
    res = np.linalg.norm(A64 @ V - V * ev[:, None, :], axis=(1, 2))
    left = np.sqrt(2.0 * (off ** 2).sum(axis=1))
    assert np.all(np.abs(res - left) <= 1e-5 * n * fro), np.abs(res - left).max()
    assert np.all(np.abs(ev.sum(axis=1) - np.trace(A64, axis1=1, axis2=2)) <= 1e-5 * n * fro)
    exact = np.linalg.eigvalsh(A64)
    assert np.all(np.abs(ev - exact).max(axis=1) <= 2.0 * off.max(axis=1) + 1e-5 * np.abs(exact).max(axis=1))
    assert np.all(off[:, n - 1] == 0.0)


@pytest.mark.parametrize("uniform", [True, False])
@pytest.mark.parametrize("n", [2, 3, 4, 8, 16, 32, 48, 64])
def test_first_iterations_match_the_oracle(n, uniform):
    """Value by value over the first iterations, for the runs in which every rotation of the
    float64 procedure was computed from a vector of length >= 1e-2 ||A||_2.  A rotation from a
    shorter vector amplifies rounding errors by its inverse length (from two rounding-level
    numbers, as in the second step on a converged 2x2 window, it is arbitrary), so such runs
    have no float32 value to compare and are left to the identities."""
    from oracle import lockstep
    batch = 8
    A = _inputs(n, batch)
    A64 = A.astype(np.float64)
    compared = 0
    for iterations in (0, 1, 2, 3):
        ev, V, off, red = _run(A, 1e-5, iterations, uniform)
        ref = lockstep.syevd_lockstep(A64, 1e-5, iterations, uniform, False)
        scale = np.abs(ref.evals).max(axis=1)
        sound = ref.min_pivot >= 1e-2 * scale
        # a rotation from a vector of length r turns an error delta of its inputs into an angle
        # error delta / r, which moves entries of size ||T|| by ||T|| delta / r; with a few
        # float32 roundings (u = 2^-24) of ||T|| per earlier rotation and up to 2n rotations per
        # iteration: 20 n u ||T||^2 / r_min, and never below the 3e-4 ||T|| of the one-iteration
        # pin of the per-matrix solver
        tol = np.maximum(3e-4, 20.0 * n * 2.0 ** -24 * scale / np.maximum(ref.min_pivot, 1e-300)) * scale
        if uniform and not sound.all():
            sound[:] = False             # a shared window passes one matrix's arbitrariness on to all
        err_ev = np.abs(ev - ref.evals).max(axis=1)
        err_off = np.abs(off[:, :n - 1] - np.abs(ref.offdiag)).max(axis=1, initial=0.0)
        assert np.all(err_ev[sound] <= tol[sound]), (n, iterations, err_ev, sound)
        assert np.all(err_off[sound] <= tol[sound]), (n, iterations, err_off, sound)
        # the shrink decisions are compared where the oracle's were not close calls (|e| within a
        # factor 1.4 of epsilon)
        last = np.array(ref.last_e) if iterations else np.zeros((0, batch))
        active = np.array(ref.window) >= 2 if iterations else np.zeros((0, batch), dtype=bool)
        close = (active & (last > 0) & (np.abs(np.log10(np.maximum(last, 1e-300) / 1e-5)) < 0.15)).any(axis=0)
        sure = (sound & ~close) if not uniform else (sound & ~close.any())
        assert np.array_equal(red[sure], ref.reductions[sure]), (n, iterations, red, ref.reductions)
        compared += int(sound.sum())
        _identities(A, ev, V, off, n)
    print(f"[lockstep] n={n} uniform={uniform}: {compared} of {4 * batch} (matrix, budget) pairs compared by value", flush=True)
    assert compared >= batch          # the reduction alone (budget 0) is always comparable


@pytest.mark.parametrize("uniform", [True, False])
@pytest.mark.parametrize("n", [4, 16, 32, 64])
def test_whole_budget(n, uniform):
    """App. B's budget (n iterations, eps 1e-5): identities, and reduction counts near the
    oracle's (App. C.4 reports n/3 .. 3n/4)."""
    from oracle import lockstep
    batch = 16
    A = _inputs(n, batch)
    ev, V, off, red = _run(A, 1e-5, n, uniform)
    _identities(A, ev, V, off, n)
    ref = lockstep.syevd_lockstep(A.astype(np.float64), 1e-5, n, uniform, False)
    print(f"[lockstep] n={n} uniform={uniform}: rows dropped, GPU mean {red.mean():.1f} (min {red.min()}, max {red.max()}), "
          f"oracle mean {ref.reductions.mean():.1f}; largest sub-diagonal left {off.max():.2e}", flush=True)
    if uniform:
        assert len(set(red.tolist())) == 1
    assert abs(red.mean() - ref.reductions.mean()) <= max(2.0, 0.25 * n)


@pytest.mark.parametrize("n", [4, 16, 32, 64])
def test_per_matrix_rule_with_ample_budget_converges(n):
    from oracle import jacobi
    batch = 16
    A = _inputs(n, batch)
    ev, V, off, red = _run(A, 1e-5, 4 * n, False)
    _identities(A, ev, V, off, n)
    lam, _ = jacobi.syevd(A)
    assert np.all(red == n - 1)
    assert np.abs(ev - lam).max() <= 3e-5 * np.abs(lam).max()


def test_eigenvalues_only_and_batch_edges():
    import torch
    from paper_2207_04228_amd import binding
    A = _inputs(16, 5)
    At = torch.from_numpy(A).to("cuda:0")
    ev, V, off, red = binding.bed_syevd_lockstep(At, 1e-5, 16, True)
    ev2, V2, off2, red2 = binding.bed_syevd_lockstep(At, 1e-5, 16, True, want_vectors=False)
    torch.cuda.synchronize()
    assert V2 is None
    assert torch.equal(ev, ev2) and torch.equal(off, off2) and torch.equal(red, red2)
    one = binding.bed_syevd_lockstep(torch.full((3, 1, 1), 2.5, device="cuda:0"), 1e-5, 4, True)
    torch.cuda.synchronize()
    assert torch.all(one[0] == 2.5) and torch.all(one[1] == 1.0) and torch.all(one[3] == 0)
    empty = binding.bed_syevd_lockstep(torch.empty((0, 8, 8), device="cuda:0"), 1e-5, 8, True)
    assert empty[0].shape == (0, 8)
