"""Pins for the CPU oracle (float64 cyclic Jacobi).

The oracle is pinned to things other than itself: closed forms, the
definition, constructions with a known answer, invariants, a library routine
on special cases and brute force on tiny inputs.  Each test names what a
mistake in the oracle (dropped term, wrong sign/index, transposed operand,
wrong ordering) would break.
"""
import math
import os

import numpy as np
import pytest

from oracle import jacobi
from oracle.acceptance import evaluate, mirror_lower, clusters
from paper_2207_04228_amd import workloads

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _sym(rng, batch, n, scale=1.0):
    A = rng.standard_normal((batch, n, n)) * scale
    return 0.5 * (A + A.transpose(0, 2, 1))


# --- P1: 2x2 closed form (same algebra as App. A.1 / A.3 of the paper) -------

@pytest.mark.parametrize("a,b,d", [
    (2.0, 1.0, -1.0), (1.0, 0.0, 3.0), (3.0, 0.0, 1.0), (1.5, 0.25, 1.5),
    (1.0, 1e-9, 1.0 + 1e-9), (-4.0, 2.5, 7.0), (0.0, 1.0, 0.0), (1e6, 3.0, -2e-3),
])
def test_p1_two_by_two_closed_form(a, b, d):
    A = np.array([[[a, b], [b, d]]], dtype=np.float64)
    lam, V = jacobi.syevd(A)
    mid, rad = 0.5 * (a + d), math.hypot(0.5 * (a - d), b)
    expect = np.array([mid - rad, mid + rad])
    scale = max(abs(expect).max(), 1e-300)
    assert np.allclose(lam[0], expect, rtol=0, atol=4e-16 * scale)
    # eigenvector for lam: proportional to (b, lam - a) (or (lam - d, b))
    for j in range(2):
        v = V[0][:, j]
        w = np.array([b, lam[0][j] - a])
        if np.linalg.norm(w) < 1e-8 * scale:
            w = np.array([lam[0][j] - d, b])
        if np.linalg.norm(w) == 0:      # a == d, b == 0: any basis is valid
            continue
        w = w / np.linalg.norm(w)
        assert abs(abs(v @ w) - 1.0) < 1e-7
    assert np.allclose(V[0].T @ V[0], np.eye(2), atol=1e-15)


def test_p1_rotated_block_entries_match_appendix_formula():
    """App. A.1: R^T X R with R = [[c, s], [-s, c]] has off-diagonal
    x2 (c^2 - s^2) + (x1 - x3) c s.  The oracle's V for a 2x2 must zero it."""
    x1, x2, x3 = 0.7, -1.3, 2.1
    lam, V = jacobi.syevd(np.array([[[x1, x2], [x2, x3]]]))
    # write V as [[c, s], [-s, c]] up to column signs
    c, s = V[0][0, 0], V[0][0, 1]
    if V[0][1, 1] * c < 0:  # fix orientation to a proper rotation
        c, s = V[0][0, 0], -V[0][0, 1]
    off = x2 * (c * c - s * s) + (x1 - x3) * c * s
    # one of the two sign conventions annihilates the off-diagonal
    off2 = x2 * (c * c - s * s) - (x1 - x3) * c * s
    assert min(abs(off), abs(off2)) < 1e-14


# --- P2: diagonal input -------------------------------------------------------

def test_p2_diagonal_input_sorted_exactly_with_permutation_vectors():
    diag = np.array([3.0, -1.0, 2.0, 2.0, -7.5, 0.0, 2.0])
    A = np.diag(diag)[None]
    lam, V = jacobi.syevd(A)
    assert np.array_equal(lam[0], np.sort(diag))
    # V is a signed permutation and maps each eigenvalue to a matching entry
    assert np.array_equal(np.abs(V[0]).sum(axis=0), np.ones(7))
    assert np.array_equal(np.abs(V[0]).sum(axis=1), np.ones(7))
    for j in range(7):
        i = int(np.argmax(np.abs(V[0][:, j])))
        assert diag[i] == lam[0][j]


# --- P3: block-diagonal input -------------------------------------------------

def test_p3_block_diagonal_union_of_block_spectra():
    rng = np.random.default_rng(3)
    B1 = _sym(rng, 1, 2)[0] + 10.0 * np.eye(2)     # spectrum near 10
    B2 = _sym(rng, 1, 3)[0] - 10.0 * np.eye(3)     # spectrum near -10
    A = np.zeros((5, 5))
    A[:2, :2] = B1
    A[2:, 2:] = B2
    lam, V = jacobi.syevd(A[None])
    # block spectra from the 2x2 closed form and numpy's cubic roots
    a, b, d = B1[0, 0], B1[0, 1], B1[1, 1]
    l1 = np.array([0.5 * (a + d) - math.hypot(0.5 * (a - d), b),
                   0.5 * (a + d) + math.hypot(0.5 * (a - d), b)])
    l2 = np.sort(np.roots(np.poly(B2)).real)
    expect = np.sort(np.concatenate([l1, l2]))
    assert np.allclose(lam[0], expect, atol=1e-12)
    # eigenvectors are supported on their own block (spectra are disjoint)
    for j in range(5):
        v = V[0][:, j]
        top, bot = np.linalg.norm(v[:2]), np.linalg.norm(v[2:])
        assert min(top, bot) < 1e-14 and abs(max(top, bot) - 1.0) < 1e-14
        assert (lam[0][j] > 0) == (top > bot)


# --- P4: A = Q diag(lam) Q^T with known lam -----------------------------------

@pytest.mark.parametrize("n", [4, 16, 33, 64])
def test_p4_known_spectrum_recovered_in_double(n):
    rng = np.random.default_rng(40 + n)
    lam = np.sort(rng.uniform(-3.0, 5.0, size=(6, n)), axis=1)
    Q = workloads.haar_orthogonal(6, n, rng)
    A = (Q * lam[:, None, :]) @ Q.transpose(0, 2, 1)
    A = 0.5 * (A + A.transpose(0, 2, 1))
    got, V = jacobi.syevd(A)          # float64 input path
    assert np.max(np.abs(got - lam)) <= n * 2e-15 * 5.0
    # vectors: gaps are O(1/n), compare up to sign
    dots = np.abs(np.einsum("bij,bij->bj", V, Q))
    gaps = np.minimum(np.diff(lam, axis=1, prepend=-np.inf), np.diff(lam, axis=1, append=np.inf))
    assert np.all(1.0 - dots[gaps > 1e-3] < 1e-9)


def test_p4_config4_spectrum_after_fp32_rounding():
    A32, Q, A64, lam = workloads.config4(batch=32, return_parts=True)
    got, _ = jacobi.syevd(A32)
    expect = np.sort(lam, axis=1)
    # rounding A to fp32 perturbs eigenvalues by at most ||dA||_2 <= n * 2^-24 * max|a|
    assert np.max(np.abs(got - expect)) <= 16 * 2.0 ** -24


def test_p4_config5_clusters_after_fp32_rounding():
    A32, Q, A64, lam = workloads.config5(48, batch=8, return_parts=True)
    got, _ = jacobi.syevd(A32)
    expect = np.sort(lam, axis=1)
    assert np.max(np.abs(got - expect)) <= 48 * 2.0 ** -24 * 10.0
    got64, _ = jacobi.syevd(A64)
    assert np.max(np.abs(got64 - expect)) <= 48 * 4e-16 * 10.0


# --- P5: invariants on every kind of test matrix ------------------------------

def _all_workloads_small():
    yield "config1", workloads.config1()
    yield "config2", workloads.config2(256)
    for n in workloads.CONFIG3_DIMS:
        yield f"config3_n{n}", workloads.config3(n, batch=24)
    yield "config4", workloads.config4(batch=48)
    for n in workloads.CONFIG5_DIMS:
        yield f"config5_n{n}", workloads.config5(n, batch=6)
    rng = np.random.default_rng(5)
    yield "indefinite", _sym(rng, 16, 13).astype(np.float32)


@pytest.mark.parametrize("name,A", list(_all_workloads_small()), ids=lambda x: x if isinstance(x, str) else "")
def test_p5_invariants(name, A):
    lam, V = jacobi.syevd(A)
    A64 = mirror_lower(A)
    n = A.shape[-1]
    tr = np.trace(A64, axis1=1, axis2=2)
    fro2 = np.sum(A64 * A64, axis=(1, 2))
    scale = np.sqrt(fro2)
    assert np.all(np.abs(lam.sum(axis=1) - tr) <= 1e-13 * n * scale)
    assert np.all(np.abs((lam * lam).sum(axis=1) - fro2) <= 1e-13 * n * fro2)
    acc = evaluate(A, lam, V, lam, V)
    assert np.all(acc.residual <= 1e-13 * n)
    assert np.all(acc.orth <= 1e-14 * n)
    assert np.all(np.diff(lam, axis=1) >= 0)


# --- P6: tridiagonal Toeplitz closed form -------------------------------------

@pytest.mark.parametrize("n", [2, 3, 5, 8, 16, 31, 48, 64])
def test_p6_toeplitz_tridiagonal_closed_form(n):
    A = 2.0 * np.eye(n) - np.eye(n, k=1) - np.eye(n, k=-1)
    lam, V = jacobi.syevd(A[None])
    k = np.arange(1, n + 1)
    expect = 2.0 - 2.0 * np.cos(k * np.pi / (n + 1))
    assert np.allclose(lam[0], expect, atol=5e-15 * n)
    j = np.arange(1, n + 1)
    S = np.sin(np.outer(j, k) * np.pi / (n + 1)) * math.sqrt(2.0 / (n + 1))
    dots = np.abs(np.einsum("ij,ij->j", V[0], S))
    assert np.all(1.0 - dots < 1e-10)


with open(os.path.join(GOLDEN, "toeplitz_n4_eigenvalues.txt")) as _f:
    _TOEPLITZ4 = [float(x) for x in _f.read().split("#")[0].split()]


def test_p6_golden_toeplitz_n4_values():
    """tests/golden/toeplitz_n4_eigenvalues.txt holds (3 -/+ sqrt5)/2 and
    (5 -/+ sqrt5)/2, typed from the closed form, not computed by any code here."""
    A = 2.0 * np.eye(4) - np.eye(4, k=1) - np.eye(4, k=-1)
    lam, _ = jacobi.syevd(A[None])
    assert np.allclose(lam[0], _TOEPLITZ4, atol=1e-14)


# --- P7: rank-one plus multiple of identity (repeated eigenvalues) ------------

@pytest.mark.parametrize("n,alpha", [(4, 0.0), (9, 0.5), (32, -2.0), (64, 1e-3)])
def test_p7_rank_one_plus_identity(n, alpha):
    rng = np.random.default_rng(70 + n)
    x = rng.standard_normal(n)
    A = np.outer(x, x) + alpha * np.eye(n)
    lam, V = jacobi.syevd(A[None])
    top = alpha + x @ x
    assert np.allclose(lam[0][:-1], alpha, atol=1e-13 * abs(top))
    assert abs(lam[0][-1] - top) <= 1e-13 * abs(top)
    assert abs(abs(V[0][:, -1] @ x) / np.linalg.norm(x) - 1.0) < 1e-12
    assert np.allclose(V[0].T @ V[0], np.eye(n), atol=1e-13)


# --- P8: library cross-check ---------------------------------------------------

@pytest.mark.parametrize("n", [1, 2, 3, 7, 16, 24, 32, 48, 64])
def test_p8_matches_lapack_eigh(n):
    rng = np.random.default_rng(80 + n)
    A = _sym(rng, 10, n)
    lam, V = jacobi.syevd(A)
    ref_l, ref_v = np.linalg.eigh(A)
    scale = np.max(np.abs(ref_l), axis=1, keepdims=True)
    assert np.all(np.abs(lam - ref_l) <= 1e-12 * scale)
    acc = evaluate(A, lam, V, ref_l, ref_v, gap_rel=1e-3)
    assert np.all(acc.angle <= 1e-9)


def test_p8_float32_entry_point_equals_float64_entry_point():
    rng = np.random.default_rng(81)
    A32 = _sym(rng, 7, 12).astype(np.float32)
    l32, v32 = jacobi.syevd(A32)
    l64, v64 = jacobi.syevd(A32.astype(np.float64))
    assert np.array_equal(l32, l64) and np.array_equal(v32, v64)


def test_lower_triangle_is_the_one_that_is_read():
    rng = np.random.default_rng(82)
    A = _sym(rng, 3, 6)
    B = A.copy()
    B[:, np.triu_indices(6, 1)[0], np.triu_indices(6, 1)[1]] = 123.0  # garbage above the diagonal
    la, _ = jacobi.syevd(A)
    lb, _ = jacobi.syevd(B)
    assert np.array_equal(la, lb)


# --- P9: brute force on tiny inputs (characteristic polynomial) ---------------

def test_p9_three_by_three_trigonometric_roots():
    rng = np.random.default_rng(9)
    for _ in range(20):
        A = _sym(rng, 1, 3)[0]
        # det(lam I - A) = 0 via the trigonometric solution of the depressed cubic
        q = np.trace(A) / 3.0
        B = A - q * np.eye(3)
        p = math.sqrt(np.sum(B * B) / 6.0)
        r = np.linalg.det(B / p) / 2.0
        phi = math.acos(min(1.0, max(-1.0, r))) / 3.0
        e3 = q + 2 * p * math.cos(phi)
        e1 = q + 2 * p * math.cos(phi + 2 * math.pi / 3)
        e2 = 3 * q - e1 - e3
        lam, _ = jacobi.syevd(A[None])
        assert np.allclose(lam[0], [e1, e2, e3], atol=1e-12)


def test_p9_one_by_one():
    lam, V = jacobi.syevd(np.array([[[-3.25]]]))
    assert lam[0, 0] == -3.25 and abs(V[0, 0, 0]) == 1.0


# --- P10: covariance under permutation, scaling and shift ---------------------

def test_p10_permutation_scaling_shift():
    rng = np.random.default_rng(10)
    n = 11
    A = _sym(rng, 4, n)
    lam, _ = jacobi.syevd(A)
    perm = rng.permutation(n)
    lp, _ = jacobi.syevd(A[:, perm][:, :, perm])
    assert np.allclose(lp, lam, atol=1e-13 * np.abs(lam).max())
    ls, _ = jacobi.syevd(-2.5 * A)
    assert np.allclose(ls, np.sort(-2.5 * lam, axis=1), atol=1e-13 * np.abs(lam).max() * 2.5)
    lsh, _ = jacobi.syevd(A + 4.0 * np.eye(n)[None])
    assert np.allclose(lsh, lam + 4.0, atol=1e-13 * (np.abs(lam).max() + 4.0))


# --- the acceptance metrics themselves ----------------------------------------

def test_acceptance_detects_planted_mistakes():
    """Plant mistakes in a copy of the oracle's output and check that each
    acceptance metric reacts to the one it is meant to catch."""
    A = workloads.config3(8, batch=4)
    lam, V = jacobi.syevd(A)
    ok = evaluate(A, lam, V, lam, V)
    assert ok.passes()
    bad = lam.copy(); bad[:, 3] += 1e-4 * np.abs(lam).max()
    assert not evaluate(A, bad, V, lam, V).passes()
    Vt = V.transpose(0, 2, 1).copy()                      # rows instead of columns
    assert not evaluate(A, lam, Vt, lam, V).passes()
    Vs = V.copy(); Vs[:, :, [0, 1]] = Vs[:, :, [1, 0]]     # two columns swapped
    assert not evaluate(A, lam, Vs, lam, V).passes()
    Vn = V.copy(); Vn[:, :, 2] *= 1.001                    # a column not normalised
    assert not evaluate(A, lam, Vn, lam, V).passes()
    Vneg = V * np.where(np.arange(8) % 2 == 0, 1.0, -1.0)  # sign flips are allowed
    assert evaluate(A, lam, Vneg, lam, V).passes()


def test_cluster_splitting():
    lam = np.array([0.0, 1e-7, 1.0, 1.0 + 1e-7, 1.0 + 2e-7, 5.0])
    assert clusters(lam, 1e-3) == [(0, 2), (2, 5), (5, 6)]


def test_workload_generators_are_deterministic_and_symmetric():
    a = workloads.config3(16, batch=8)
    b = workloads.config3(16, batch=8)
    assert a.dtype == np.float32 and np.array_equal(a, b)
    assert np.array_equal(a, a.transpose(0, 2, 1))
    c5 = workloads.config5(48, batch=2)
    assert c5.shape == (2, 48, 48)
    lam = workloads.clustered_spectrum(3, 48, 1)
    s = np.sort(lam, axis=1)
    # multiplicity four and a 1e-6-relative pair are present in every row
    assert np.all(np.sum(np.diff(s, axis=1) == 0.0, axis=1) == 3)
    rel = np.diff(s, axis=1) / s[:, 1:]
    assert np.all(np.sum((rel > 0) & (rel < 2e-6), axis=1) >= 1)


def test_structured_cases_are_symmetric_finite_and_known():
    """The structured inputs of the GPU parity tests, and two of them against their closed
    forms through the oracle: all-ones has the spectrum {0 (n-1 times), n}; the Wilkinson matrix
    W_n^+ is symmetric about its anti-diagonal, so its spectrum is that of J W J."""
    for n in (3, 8, 21):
        cases = dict(workloads.structured_cases(n, 4, seed=900 + n))
        again = dict(workloads.structured_cases(n, 4, seed=900 + n))
        for name, A in cases.items():
            assert A.dtype == np.float32 and A.shape[1:] == (n, n), name
            assert np.isfinite(A).all() and np.array_equal(A, A.transpose(0, 2, 1)), name
            assert np.array_equal(A, again[name]), name
        lam, _ = jacobi.syevd(cases["all ones"])
        assert np.abs(lam[:, :-1]).max() <= 1e-12 * n and np.abs(lam[:, -1] - n).max() <= 1e-12 * n
        W = cases["wilkinson"][0].astype(np.float64)
        assert np.array_equal(W, W[::-1, ::-1])
        assert abs(np.trace(W) - jacobi.syevd(cases["wilkinson"])[0][0].sum()) <= 1e-12 * n


# --- mutation check: the pins above reject plausible mistakes ------------------

def _battery(solve) -> bool:
    """A compact subset of the pins (P1 closed form, P5 invariants, P6 closed
    form, ordering) applied to an arbitrary solver callable."""
    try:
        a, b, d = 2.0, 1.0, -1.0
        lam, V = solve(np.array([[[a, b], [b, d]]]))
        mid, rad = 0.5 * (a + d), math.hypot(0.5 * (a - d), b)
        if not np.allclose(lam[0], [mid - rad, mid + rad], atol=1e-14):
            return False
        n = 9
        A = 2.0 * np.eye(n) - np.eye(n, k=1) - np.eye(n, k=-1)
        lam, V = solve(A[None])
        k = np.arange(1, n + 1)
        if not np.allclose(lam[0], 2.0 - 2.0 * np.cos(k * np.pi / (n + 1)), atol=1e-13):
            return False
        S = np.sin(np.outer(k, k) * np.pi / (n + 1)) * math.sqrt(2.0 / (n + 1))
        if np.any(1.0 - np.abs(np.einsum("ij,ij->j", V[0], S)) > 1e-10):
            return False
        rng = np.random.default_rng(77)
        A = _sym(rng, 3, 7)
        lam, V = solve(A)
        acc = evaluate(A, lam, V, lam, V)
        if np.any(acc.residual > 1e-12) or np.any(acc.orth > 1e-12):
            return False
        if np.any(np.diff(lam, axis=1) < 0):
            return False
        return True
    except Exception:
        return False


_MUTANTS = [
    ("V[r * n + q] = s * vrp + c * vrq;", "V[r * n + q] = -s * vrp + c * vrq;"),
    ("W[p * n + p] = app - t * apq;", "W[p * n + p] = app + t * apq;"),
    ("theta = (aqq - app) / (2.0 * apq);", "theta = (app - aqq) / (2.0 * apq);"),
    ("W[r * n + p] = c * arp - s * arq;", "W[r * n + p] = c * arp + s * arq;"),
    ("W[perm[j] * n + perm[j]] > kv", "W[perm[j] * n + perm[j]] < kv"),
    ("W[r * n + i] = V[r * n + perm[i]];", "W[r * n + i] = V[perm[i] * n + r];"),
    ("c = 1.0 / sqrt(t * t + 1.0);", "c = 1.0 / sqrt(t * t + 2.0);"),
]


def test_pins_reject_mutated_oracles(tmp_path):
    import ctypes
    import subprocess
    src = open(os.path.join(os.path.dirname(jacobi.__file__), "jacobi.c")).read()

    def make_solver(text, tag):
        c = tmp_path / f"m{tag}.c"
        so = tmp_path / f"m{tag}.so"
        c.write_text(text)
        subprocess.run(["gcc", "-O1", "-fPIC", "-shared", "-std=c99", "-o", str(so), str(c), "-lm"], check=True)
        lib = ctypes.CDLL(str(so))
        dp = ctypes.POINTER(ctypes.c_double)
        lib.oracle_syevd_f64_in64.argtypes = [dp, ctypes.c_int, ctypes.c_int, dp, dp, ctypes.c_void_p, ctypes.c_int]

        def solve(A):
            A = np.ascontiguousarray(A, dtype=np.float64)
            b, n, _ = A.shape
            lam = np.empty((b, n)); V = np.empty((b, n, n))
            lib.oracle_syevd_f64_in64(A.ctypes.data_as(dp), b, n, lam.ctypes.data_as(dp),
                                      V.ctypes.data_as(dp), None, 1)
            return lam, V
        return solve

    assert _battery(make_solver(src, "orig"))
    assert _battery(lambda A: jacobi.syevd(np.asarray(A, dtype=np.float64)))
    for i, (old, new) in enumerate(_MUTANTS):
        assert src.count(old) == 1, old
        assert not _battery(make_solver(src.replace(old, new), str(i))), f"mutant {i} survived: {new}"
