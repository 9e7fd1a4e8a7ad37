"""Seeded sweep over random sizes, batches and spectra (all size classes of the dispatch,
ragged n and ragged batches), every matrix held to the parity bar against the oracle."""
import numpy as np
import pytest

from test_gpu_parity import _check

pytestmark = pytest.mark.gpu


def _draw(seed):
    from paper_2207_04228_amd import workloads
    rng = np.random.default_rng(9000 + seed)
    n = int(rng.choice([rng.integers(1, 9), rng.integers(9, 33), rng.integers(33, 65), rng.integers(65, 129)]))
    batch = int(rng.integers(1, 40 if n > 64 else 90))
    kind = int(rng.integers(0, 5))
    if kind == 0:
        A = workloads.covariance(batch, n, int(rng.integers(n, 5 * n + 2)), 1e-4, 100 + seed)
        name = "wishart"
    elif kind == 1:
        lam = rng.uniform(-3.0, 3.0, size=(batch, n))                       # indefinite
        A = workloads.from_spectrum(lam, seed=200 + seed)
        name = "indefinite"
    elif kind == 2:
        lam = np.sort(rng.choice(rng.uniform(0.5, 2.0, size=3), size=(batch, n)), axis=1)   # three distinct values
        A = workloads.from_spectrum(lam, seed=300 + seed)
        name = "three eigenvalues"
    elif kind == 3:
        lam = 10.0 ** rng.uniform(-6.0, 0.0, size=(batch, n))               # condition number up to 1e6
        A = workloads.from_spectrum(lam, seed=400 + seed)
        name = "graded"
    else:
        X = rng.standard_normal((batch, n, n))
        A = (X + np.swapaxes(X, 1, 2)).astype(np.float32) * np.float32(10.0 ** rng.integers(-12, 12))
        name = "gaussian symmetric, scaled"
    return A, f"{name} n={n} batch={batch}"


@pytest.mark.parametrize("seed", range(24))
def test_random_case(seed):
    A, name = _draw(seed)
    _check(A, f"seed {seed}: {name}")
