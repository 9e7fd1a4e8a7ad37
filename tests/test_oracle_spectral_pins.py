"""Pins for the spectral-function oracle (float64): things other than itself."""
import math

import numpy as np
import pytest
import scipy.linalg

from oracle import spectral
from oracle.acceptance import mirror_lower
from paper_2207_04228_amd import workloads


def test_two_by_two_closed_form_square_root():
    """For a 2x2 SPD matrix, sqrt(A) = (A + s I) / t with s = sqrt(det A), t = sqrt(tr A + 2 s)."""
    rng = np.random.default_rng(1)
    for _ in range(10):
        X = rng.standard_normal((3, 2))
        A = X.T @ X + 0.1 * np.eye(2)
        s = math.sqrt(np.linalg.det(A))
        t = math.sqrt(np.trace(A) + 2 * s)
        expect = (A + s * np.eye(2)) / t
        got = spectral.spd_fn(A[None], spectral.FN_SQRT, 0.0)[0]
        assert np.allclose(got, expect, atol=1e-13)
        inv = spectral.spd_fn(A[None], spectral.FN_INV_SQRT, 1e-300)[0]
        assert np.allclose(inv, np.linalg.inv(expect), atol=1e-12)


def test_diagonal_input_is_elementwise():
    d = np.array([4.0, 0.25, 9.0, 1.0, 16.0])
    got = spectral.spd_fn(np.diag(d)[None], spectral.FN_SQRT, 0.0)[0]
    assert np.allclose(got, np.diag(np.sqrt(d)), atol=1e-15)
    got = spectral.spd_fn(np.diag(d)[None], spectral.FN_INV_SQRT, 1e-12)[0]
    assert np.allclose(got, np.diag(1 / np.sqrt(d)), atol=1e-15)


@pytest.mark.parametrize("name,A", [("config1", workloads.config1()), ("config3_n16", workloads.config3(16, batch=12)),
                                    ("config4", workloads.config4(batch=12)), ("config5_n48", workloads.config5(48, batch=3))],
                         ids=lambda x: x if isinstance(x, str) else "")
def test_defining_identities(name, A):
    A64 = mirror_lower(A)
    n = A.shape[-1]
    S = spectral.spd_fn(A, spectral.FN_SQRT, 0.0)
    W = spectral.spd_fn(A, spectral.FN_INV_SQRT, 1e-300)
    I = np.eye(n)[None]
    scale = np.abs(A64).max()
    assert np.allclose(S @ S, A64, atol=1e-12 * scale)                    # (A^1/2)^2 = A
    assert np.abs(W @ A64 @ W - I).max() <= 1e-10                         # A^-1/2 A A^-1/2 = I
    assert np.allclose(S, np.swapaxes(S, 1, 2), atol=1e-14 * scale)       # symmetric
    assert np.abs(S @ A64 - A64 @ S).max() <= 1e-12 * scale ** 1.5        # commutes with A
    assert np.abs(S @ W - I).max() <= 1e-10                               # inverse of each other


def test_matches_library_sqrtm():
    A = workloads.config3(8, batch=4).astype(np.float64)
    S = spectral.spd_fn(A, spectral.FN_SQRT, 0.0)
    for b in range(4):
        ref = scipy.linalg.sqrtm(A[b]).real
        assert np.allclose(S[b], ref, atol=1e-12)


def test_floor_clamps_small_and_negative_eigenvalues():
    Q = workloads.haar_orthogonal(1, 4, np.random.default_rng(3))[0]
    lam = np.array([-1e-3, 1e-9, 0.5, 2.0])
    A = (Q * lam) @ Q.T
    A = 0.5 * (A + A.T)
    got = spectral.spd_fn(A[None], spectral.FN_INV_SQRT, 1e-2)[0]
    expect = (Q * (1 / np.sqrt(np.maximum(lam, 1e-2)))) @ Q.T
    assert np.allclose(got, expect, atol=1e-9)
