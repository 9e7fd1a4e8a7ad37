"""Heavily repeated eigenvalues.  Inside a cluster the recurrence leaves the off-diagonals at
the rounding level of the diagonal; with a deflation tolerance of 2^-23 such windows could
hover around the tolerance until the sweep cap (0.2 % of these matrices did not converge).
Every matrix must converge (info = 0, no runaway rotation counts) and meet the parity bar."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def _spectra(rng, batch, n):
    return [np.round(rng.uniform(0, 3, (batch, n))),                              # integers 0 .. 3
            2.0 * np.ones((batch, n)) + (rng.uniform(0, 1, (batch, n)) < 0.2),    # mostly 2, some 3
            np.round(rng.uniform(0, 2, (batch, n))) * 1024.0,                     # the same, scaled
            np.where(rng.uniform(0, 1, (batch, n)) < 0.5, 1.0, 1.0 + 1e-6)]       # two values 1e-6 apart


@pytest.mark.parametrize("n", [4, 8, 16, 32, 64, 96, 128])
def test_repeated_eigenvalues_converge(n):
    import torch
    from oracle import jacobi
    from oracle.acceptance import evaluate
    from paper_2207_04228_amd import binding, workloads
    worst_rot = 0.0
    relaxed, matrices = 0, 0   # off-diagonals deflated only by the fallback test (upper half of info)
    for seed in (1, 2, 6, 10):                       # seeds that used to stall are among them
        rng = np.random.default_rng(7000 + 100 * n + seed)
        batch = 48 if n <= 64 else 16
        for kind, lam in enumerate(_spectra(rng, batch, n)):
            A = workloads.from_spectrum(lam, seed=seed * 7 + kind)
            ev, V, info, rot = binding.bed_syevd_info(torch.from_numpy(A).to("cuda:0"))
            torch.cuda.synchronize()
            assert int((info & 0xFFFF).max()) == 0, (n, seed, kind)
            relaxed += int((info >> 16).sum())
            matrices += int((info >> 16 > 0).sum())
            worst_rot = max(worst_rot, int(rot.max()) / (n * n))
            lam_o, V_o = jacobi.syevd(A)
            acc = evaluate(A, ev.cpu().numpy(), V.cpu().numpy(), lam_o, V_o)
            assert acc.passes(), (n, seed, kind, acc.worst())
    print(f"[repeated] n={n}: max rotations / n^2 = {worst_rot:.2f}; fallback deflations: "
          f"{relaxed} in {matrices} matrices", flush=True)
    assert worst_rot <= 4.0


def test_lane_kernel_with_repeated_eigenvalues():
    import torch
    from oracle import jacobi
    from oracle.acceptance import evaluate
    from paper_2207_04228_amd import binding, workloads
    for n in (4, 8):
        rng = np.random.default_rng(7100 + n)
        batch = 12288 + 17
        lam = np.round(rng.uniform(0, 2, (batch, n))) + 1.0
        A = workloads.from_spectrum(lam, seed=n)
        ev, V, info, rot = binding.bed_syevd_info(torch.from_numpy(A).to("cuda:0"), family=binding.BED_FAMILY_LANE)
        torch.cuda.synchronize()
        assert int((info & 0xFFFF).max()) == 0 and int(rot.max()) <= 6 * n * n
        print(f"[repeated] lane kernel n={n}: fallback deflations: {int((info >> 16).sum())}",
              flush=True)
        lam_o, V_o = jacobi.syevd(A)
        assert evaluate(A, ev.cpu().numpy(), V.cpu().numpy(), lam_o, V_o).passes()
