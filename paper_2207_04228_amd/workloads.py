"""Seeded synthetic input generators (shared by tests, bench and the oracle's
callers).  This module holds none of the solver's arithmetic: it only draws
random symmetric matrices with the shapes and spectra of the paper's
workloads -- grouped feature covariances (Sec. 2.1, App. B.1, B.3: mini-batches
of 4x4 ... 32x32 SPD matrices) and the "randomly generated matrices" of the
numerical test (Sec. 4.1, App. B "Implementation Details").

Every generator builds in float64, symmetrises, casts to float32 once and
returns that float32 array; the same array is handed to the GPU library and
(widened) to the CPU oracle.
"""
from __future__ import annotations

import numpy as np

BASE_SEED = 20220704


def _seed(config: int, index: int = 0) -> int:
    return BASE_SEED + 1000 * config + index


def _finish(A64: np.ndarray) -> np.ndarray:
    A64 = 0.5 * (A64 + np.swapaxes(A64, -1, -2))
    return np.ascontiguousarray(A64.astype(np.float32))


def covariance(batch: int, n: int, m: int, ridge: float, seed: int) -> np.ndarray:
    """A = X^T X / m + ridge * I with X in R^{m x n} i.i.d. N(0,1)."""
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((batch, m, n))
    A = np.swapaxes(X, 1, 2) @ X / float(m) + ridge * np.eye(n)[None]
    return _finish(A)


def haar_orthogonal(batch: int, n: int, rng: np.random.Generator) -> np.ndarray:
    """Haar-distributed orthogonal matrices: QR of a Gaussian matrix with the
    columns of Q multiplied by sign(diag R)."""
    G = rng.standard_normal((batch, n, n))
    Q, R = np.linalg.qr(G)
    sgn = np.sign(np.diagonal(R, axis1=1, axis2=2))
    sgn = np.where(sgn == 0, 1.0, sgn)
    return Q * sgn[:, None, :]


def from_spectrum(lam: np.ndarray, seed: int, return_parts: bool = False):
    """A_b = Q_b diag(lam_b) Q_b^T, Q_b Haar.  lam: [batch, n] float64."""
    rng = np.random.default_rng(seed)
    batch, n = lam.shape
    Q = haar_orthogonal(batch, n, rng)
    A = (Q * lam[:, None, :]) @ np.swapaxes(Q, 1, 2)
    A32 = _finish(A)
    if return_parts:
        return A32, Q, 0.5 * (A + np.swapaxes(A, 1, 2))
    return A32


def power_law_spectrum(batch: int, n: int) -> np.ndarray:
    """lam_i = i^-2, i = 1..n (condition number n^2)."""
    i = np.arange(1, n + 1, dtype=np.float64)
    return np.tile(i ** -2.0, (batch, 1))


def clustered_spectrum(batch: int, n: int, seed: int) -> np.ndarray:
    """lam ~ U(0.1, 10) i.i.d.; then entries 0..3 are set to one common value
    (multiplicity 4) and entry 5 to entry 4 * (1 + 1e-6) (a pair separated by
    1e-6 relative); finally each row is shuffled."""
    rng = np.random.default_rng(seed)
    lam = rng.uniform(0.1, 10.0, size=(batch, n))
    lam[:, 1:4] = lam[:, 0:1]
    lam[:, 5] = lam[:, 4] * (1.0 + 1e-6)
    for b in range(batch):
        rng.shuffle(lam[b])
    return lam


# ---------------------------------------------------------------------------
# The five named configurations.
# ---------------------------------------------------------------------------

def config1() -> np.ndarray:
    """batch 64, n 4: A = X^T X / 16 + 1e-3 I, X in R^{16x4}."""
    return covariance(64, 4, 16, 1e-3, _seed(1))


CONFIG2_BATCHES = (256, 512, 4096, 65536)


def config2(batch: int) -> np.ndarray:
    """n 4: A = X^T X / 64 + 1e-3 I, X in R^{64x4}; batch in CONFIG2_BATCHES."""
    idx = CONFIG2_BATCHES.index(batch) if batch in CONFIG2_BATCHES else 99
    return covariance(batch, 4, 64, 1e-3, _seed(2, idx))


CONFIG3_DIMS = (8, 16, 24, 32)


def config3(n: int, batch: int = 512) -> np.ndarray:
    """batch 512: A = X^T X / (4n) + 1e-4 I, X in R^{4n x n}; n in CONFIG3_DIMS."""
    idx = CONFIG3_DIMS.index(n) if n in CONFIG3_DIMS else 99
    return covariance(batch, n, 4 * n, 1e-4, _seed(3, idx))


def config4(batch: int = 4096, n: int = 16, return_parts: bool = False):
    """batch 4096, n 16: Haar Q, lam_i = i^-2."""
    lam = power_law_spectrum(batch, n)
    out = from_spectrum(lam, _seed(4), return_parts=return_parts)
    if return_parts:
        return out + (lam,)
    return out


CONFIG5_DIMS = (48, 64)


def config5(n: int, batch: int = 256, return_parts: bool = False):
    """batch 256, n in {48, 64}: Haar Q, clustered spectrum."""
    idx = CONFIG5_DIMS.index(n) if n in CONFIG5_DIMS else 99
    lam = clustered_spectrum(batch, n, _seed(5, idx))
    out = from_spectrum(lam, _seed(5, idx) + 500, return_parts=return_parts)
    if return_parts:
        return out + (lam,)
    return out


def headline_points():
    """The four (n, A) points of the headline metric: batch 512, n = 4/8/16/32."""
    return [(4, config2(512)), (8, config3(8)), (16, config3(16)), (32, config3(32))]


def wilkinson_tridiagonal(n: int) -> np.ndarray:
    """W_n^+: diagonal |i - (n-1)/2|, off-diagonals 1 (its large eigenvalues come in pairs
    that agree to many digits)."""
    return (np.diag(np.abs(np.arange(n) - (n - 1) / 2.0)) + np.diag(np.ones(n - 1), 1)
            + np.diag(np.ones(n - 1), -1))


def glued_wilkinson(n: int, blocks: int = 4, glue: float = 1e-6) -> np.ndarray:
    """Wilkinson blocks coupled by a tiny off-diagonal entry: clusters of eigenvalues whose
    vectors are spread over several blocks."""
    G = np.zeros((n, n))
    k = max(2, n // blocks)
    for j in range(0, n, k):
        kk = min(k, n - j)
        G[j:j + kk, j:j + kk] = wilkinson_tridiagonal(kk)
        if j > 0:
            G[j, j - 1] = G[j - 1, j] = glue
    return G


def structured_cases(n: int, batch: int, seed: int):
    """[(name, A float32 [b][n][n])]: matrices with structure that stresses deflation,
    scaling and clustering rather than the covariance-like bulk of the configs: graded and
    +- paired spectra, extreme scales, Wilkinson and glued Wilkinson matrices (plain and
    hidden by a random orthogonal similarity), rank one, identity, zero, sparse, arrow,
    near-identity, rank two, Hilbert and Kac-Murdock-Szego matrices."""
    rng = np.random.default_rng(seed)
    idx = np.arange(n)
    out = []

    def add(name, A):
        out.append((name, np.ascontiguousarray(A, dtype=np.float32)))

    lam = np.logspace(-10, 0, n)[None, :].repeat(batch, 0) * rng.uniform(0.5, 1, (batch, n))
    add("graded", from_spectrum(lam, seed=seed + 1))
    lam = np.concatenate([-np.arange(1, n // 2 + 1), np.arange(1, n - n // 2 + 1)])[None, :].repeat(batch, 0)
    add("plus-minus pairs", from_spectrum(lam.astype(np.float64), seed=seed + 2))
    A = from_spectrum(rng.uniform(0.1, 1, (batch, n)), seed=seed + 3)
    add("scale 1e-30", A * np.float32(1e-30))
    add("scale 1e+30", A * np.float32(1e30))
    add("wilkinson", wilkinson_tridiagonal(n)[None].repeat(2, 0))
    if n >= 8:
        G = glued_wilkinson(n)
        add("glued wilkinson", G[None].repeat(2, 0))
        Q = haar_orthogonal(2, n, rng)
        add("glued wilkinson, rotated", Q @ G @ np.swapaxes(Q, 1, 2))
    add("all ones", np.ones((2, n, n)))
    add("identity", np.eye(n)[None].repeat(2, 0))
    add("zero", np.zeros((2, n, n)))
    S = rng.standard_normal((batch, n, n)) * (rng.uniform(0, 1, (batch, n, n)) < 0.1)
    add("sparse", (S + np.swapaxes(S, 1, 2)) / 2)
    Ar = np.zeros((batch, n, n))
    Ar[:, idx, idx] = rng.uniform(0, 1, (batch, n))
    Ar[:, 0, :] = Ar[:, :, 0] = rng.standard_normal((batch, n))
    add("arrow", Ar)
    P = rng.standard_normal((batch, n, n)) * 1e-7
    add("near identity", np.eye(n)[None] * 3 + (P + np.swapaxes(P, 1, 2)) / 2)
    X = rng.standard_normal((batch, n, 2))
    add("rank two", X @ np.swapaxes(X, 1, 2))
    add("hilbert", (1.0 / (idx[:, None] + idx[None, :] + 1.0))[None].repeat(2, 0))
    add("kac-murdock-szego", np.exp(-3.0 * np.abs(idx[:, None] - idx[None, :]))[None].repeat(2, 0))
    return out
