"""Every size n = 1 .. 128 (all instantiations and both sides of every dispatch boundary)
with five kinds of spectra each, held to the parity bar against the oracle."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("first", [1, 33, 65, 97])
def test_every_n(first):
    import torch
    from oracle import jacobi
    from oracle.acceptance import evaluate
    from paper_2207_04228_amd import binding, workloads
    worst = dict(eval_err=0.0, residual=0.0, orth=0.0, angle=0.0)
    relaxed = []      # (n, kind, count): off-diagonals deflated only by the fallback test (upper half of info)
    for n in range(first, first + 32):
        rng = np.random.default_rng(5000 + n)
        batch = 12 if n <= 64 else 5
        mats = [workloads.covariance(batch, n, max(2, n // 2), 0.0, 10 + n),                      # rank deficient
                workloads.covariance(batch, n, 4 * n, 1e-4, 20 + n),
                workloads.from_spectrum(rng.uniform(-2, 2, (batch, n)), seed=30 + n),             # indefinite
                workloads.from_spectrum(np.round(rng.uniform(0, 3, (batch, n))), seed=40 + n),    # heavy multiplicities
                workloads.from_spectrum(10.0 ** rng.uniform(-7, 0, (batch, n)), seed=50 + n)]     # graded
        for kind, A in enumerate(mats):
            ev, V, info, rot = binding.bed_syevd_info(torch.from_numpy(A).to("cuda:0"))
            torch.cuda.synchronize()
            lam_o, V_o = jacobi.syevd(A)
            acc = evaluate(A, ev.cpu().numpy(), V.cpu().numpy(), lam_o, V_o)
            w = acc.worst()
            assert acc.passes() and int((info & 0xFFFF).max()) == 0, (n, kind, w)
            if int((info >> 16).sum()):
                relaxed.append((n, kind, int((info >> 16).sum())))
            for key in worst:
                worst[key] = max(worst[key], w[key] / (n if key in ("residual", "orth") else 1))
    print(f"[every n] {first}..{first + 31}: worst eval {worst['eval_err']:.2e}, residual/n {worst['residual']:.2e}, "
          f"orth/n {worst['orth']:.2e}, angle {worst['angle']:.2e}; "
          f"fallback deflations (n, kind, count): {relaxed}", flush=True)
    # the fallback is for spectra graded over many orders of magnitude (kind 4) and rank-deficient input (kind 0)
    assert all(kind in (0, 4) for _, kind, _ in relaxed), relaxed
