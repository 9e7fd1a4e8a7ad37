"""Parity on matrices whose structure stresses deflation, scaling and clustering (graded and
paired spectra, scales 1e-30 and 1e+30, Wilkinson and glued Wilkinson matrices, rank-deficient,
sparse, arrow, nearly scalar, Hilbert ...), in every size class of the kernels."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("n", [2, 3, 5, 8, 13, 16, 21, 32, 33, 47, 64, 65, 96, 128])
def test_structured_matrices(n):
    import torch
    from oracle import jacobi
    from oracle.acceptance import evaluate
    from paper_2207_04228_amd import binding, workloads
    batch = 16 if n <= 64 else 4
    worst = {"eval_err": 0.0, "residual": 0.0, "orth": 0.0}
    relaxed = 0       # off-diagonals deflated only by the fallback test (upper half of info)
    for name, A in workloads.structured_cases(n, batch, seed=900 + n):
        ev, V, info, rot = binding.bed_syevd_info(torch.from_numpy(A).to("cuda:0"))
        torch.cuda.synchronize()
        assert int((info & 0xFFFF).max()) == 0, (n, name)
        relaxed += int((info >> 16).sum())
        assert int(rot.max()) <= 4 * n * n + 8, (n, name, int(rot.max()))
        lam_o, V_o = jacobi.syevd(A)
        acc = evaluate(A, ev.cpu().numpy(), V.cpu().numpy(), lam_o, V_o)
        w = acc.worst()
        assert acc.passes(), (n, name, w)
        for k in worst:
            worst[k] = max(worst[k], w[k])
    print(f"[structured] n={n}: eval {worst['eval_err']:.2e} res {worst['residual']:.2e} orth {worst['orth']:.2e}; "
          f"fallback deflations: {relaxed}", flush=True)


@pytest.mark.parametrize("batch,family", [(2, 0), (8192, 1), (8192, 2), (8192, 3)])
def test_fixed_point_of_the_double_shift(batch, family):
    """diag(1, 0, 1) with unit off-diagonals is mapped onto itself (up to signs) by a pair of
    sweeps shifted with the two eigenvalues of its trailing block, in exact arithmetic for
    ever; the solver has to leave it after a few iterations, in every kernel family that serves
    n = 3 (one wavefront per matrix, four matrices per wavefront, one matrix per lane)."""
    import torch
    from paper_2207_04228_amd import binding, workloads
    W = workloads.wilkinson_tridiagonal(3).astype(np.float32)
    A = np.stack([W * np.float32(s) for s in (1.0, -1.0, 0.125, 3.0)] * (batch // 4 + 1))[:batch]
    ev, V, info, rot = binding.bed_syevd_info(torch.from_numpy(np.ascontiguousarray(A)).to("cuda:0"), family=family)
    torch.cuda.synchronize()
    assert int(info.max()) == 0
    assert int(rot.max()) <= 44, int(rot.max())
    exact = np.array([-1.0, 1.0, 2.0])
    scale = np.array([1.0, -1.0, 0.125, 3.0] * (batch // 4 + 1))[:batch]
    ref = np.sort(exact[None, :] * scale[:, None], axis=1)
    assert np.abs(ev.cpu().numpy() - ref).max() <= 1e-5 * 6.0
