"""TEST ORACLE -- gradients through the eigendecomposition, float64.

Written from the first-order perturbation theory of A = V diag(lambda) V^T
(the decomposition defined in Sec. 3.1 Eq. (1) of the paper); the paper itself
only names the technique it uses for the backward pass (App. B: a Taylor
polynomial of degree 9 in place of 1/(lambda_i - lambda_j), App. B.1).

  d lambda_j = v_j^T dA v_j
  d v_j      = sum_{i != j} v_i (v_i^T dA v_j) / (lambda_j - lambda_i)

so for a loss L(lambda, V) with upstream gradients g_lam, g_V

  g_A = V ( diag(g_lam) + sym( K o (V^T g_V) ) ) V^T,   K_ij = 1 / (lambda_j - lambda_i), K_ii = 0

and for F = V f(Lambda) V^T with upstream gradient G (Daleckii-Krein)

  g_A = V ( Phi o (V^T sym(G) V) ) V^T,   Phi_ij = (f(l_i) - f(l_j)) / (l_i - l_j),  Phi_ii = f'(l_i).

Plain einsum/matmul steps, no blocking.  Test infrastructure only; shares
nothing with the GPU path.
"""
from __future__ import annotations

import numpy as np

MODE_EXACT = 0    # K_ij = 1/(l_j - l_i) where |l_j - l_i| >= gap_floor, else 0
MODE_TAYLOR = 1   # K_ij replaced by its truncated geometric series (degree D)
FN_SQRT = 0
FN_INV_SQRT = 1


def coupling_exact(lam: np.ndarray, gap_floor: float, decide_in_float32: bool = False) -> np.ndarray:
    """K [.., n, n] with K_ij = 1/(lam_j - lam_i) for |lam_j - lam_i| >= gap_floor (and i != j), else 0.
    With decide_in_float32 the comparison against gap_floor is taken on the float32 difference,
    the precision in which the GPU takes the same decision."""
    d = lam[..., None, :] - lam[..., :, None]
    dd = (lam.astype(np.float32)[..., None, :] - lam.astype(np.float32)[..., :, None]) if decide_in_float32 else d
    n = lam.shape[-1]
    keep = (np.abs(dd) >= gap_floor) & ~np.eye(n, dtype=bool) & (d != 0)
    K = np.zeros_like(d)
    K[keep] = 1.0 / d[keep]
    return K


def coupling_taylor(lam: np.ndarray, degree: int) -> np.ndarray:
    """K_ij for the pair (a, b) = (lam_i, lam_j): with b the larger in magnitude,
    1/(b - a) = (1/b) / (1 - a/b) is replaced by (1/b) sum_{k=0}^{degree} (a/b)^k;
    otherwise by -(1/a) sum_k (b/a)^k.  Finite for equal eigenvalues; for equal magnitudes
    the one with the larger index counts as the larger (the eigenvalues are sorted), so
    that K stays antisymmetric like the exact coupling."""
    n = lam.shape[-1]
    a = np.broadcast_to(lam[..., :, None], lam.shape + (n,))
    b = np.broadcast_to(lam[..., None, :], lam.shape + (n,))
    later = np.arange(n)[None, :] > np.arange(n)[:, None]            # j > i
    big_b = (np.abs(b) > np.abs(a)) | ((np.abs(b) == np.abs(a)) & later)
    num = np.where(big_b, a, b)
    den = np.where(big_b, b, a)
    K = np.zeros(a.shape)
    ok = den != 0
    rho = np.zeros(a.shape)
    rho[ok] = num[ok] / den[ok]
    s = np.zeros(a.shape)
    for k in range(degree + 1):
        s = s + rho ** k
    K[ok] = s[ok] / den[ok]
    K = np.where(big_b, K, -K)
    K[..., np.arange(n), np.arange(n)] = 0.0
    return K


def syevd_backward(lam, V, g_lam, g_V, mode=MODE_EXACT, gap_floor=0.0, degree=9, decide_in_float32=False):
    """g_A [batch, n, n] (symmetric) from g_lam [batch, n] and g_V [batch, n, n] (either may be None)."""
    lam = np.asarray(lam, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    n = lam.shape[-1]
    M = np.zeros(V.shape)
    if g_V is not None:
        C = np.swapaxes(V, -1, -2) @ np.asarray(g_V, dtype=np.float64)
        K = coupling_exact(lam, gap_floor, decide_in_float32) if mode == MODE_EXACT else coupling_taylor(lam, degree)
        M = K * C
        M = 0.5 * (M + np.swapaxes(M, -1, -2))
    if g_lam is not None:
        M = M + np.asarray(g_lam, dtype=np.float64)[..., :, None] * np.eye(n)
    return V @ M @ np.swapaxes(V, -1, -2)


def divided_differences(lam: np.ndarray, fn: int, floor: float) -> np.ndarray:
    """Phi_ij = (f~(l_i) - f~(l_j)) / (l_i - l_j) with f~(x) = f(max(x, floor)); where the two
    eigenvalues coincide (and on the diagonal) the derivative of f~."""
    a = np.maximum(lam, floor)
    clamped = lam < floor
    if fn == FN_SQRT:
        f = np.sqrt(a)
        with np.errstate(divide="ignore"):
            fp = 0.5 / np.sqrt(a)
    elif fn == FN_INV_SQRT:
        f = 1.0 / np.sqrt(a)
        fp = -0.5 * a ** -1.5
    else:
        raise ValueError("unknown fn")
    fp = np.where(clamped, 0.0, fp)                      # the clamped function is constant below the floor
    dl = lam[..., :, None] - lam[..., None, :]
    df = f[..., :, None] - f[..., None, :]
    same = dl == 0
    Phi = np.where(same, 0.0, df / np.where(same, 1.0, dl))
    # equal eigenvalues (and the diagonal): the derivative
    return np.where(same, 0.5 * (fp[..., :, None] + fp[..., None, :]), Phi)


def spd_fn_backward(lam, V, G, fn, floor):
    """Gradient of <G, V f(max(Lambda, floor)) V^T> with respect to A (symmetric)."""
    lam = np.asarray(lam, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    G = np.asarray(G, dtype=np.float64)
    Phi = divided_differences(lam, fn, floor)
    C = np.swapaxes(V, -1, -2) @ (0.5 * (G + np.swapaxes(G, -1, -2))) @ V
    return V @ (Phi * C) @ np.swapaxes(V, -1, -2)
