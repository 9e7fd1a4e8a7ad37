"""TEST ORACLE -- the paper's own iteration, step by step, in float64 with dense
matrices: Householder tridiagonalisation (Sec. 3.1), then a fixed number of outer
iterations, each made of two shifted QR steps by Givens rotations whose shifts are the
two eigenvalues of the trailing 2x2 block of the matrix the iteration starts from
(Sec. 3.2.1, 3.2.2, App. A.3), with the progressive shrinking of Sec. 3.2.3: after an
iteration the last row and column are dropped when the last sub-diagonal entry is at
most epsilon in magnitude (absolute test, that one entry only, at most one row per
iteration).  App. B fixes epsilon = 1e-5 and n outer iterations.

`uniform=True` is the reading a batched tensor forces: the window has one size for the
whole mini-batch, so a row is dropped only when EVERY matrix of the batch passes the
test.  `uniform=False` applies the same rule to each matrix on its own.

Unlike the Jacobi oracle this one does not compute "the" eigendecomposition but what
the paper's procedure returns after its fixed budget: diag(T) and P*Q_1*Q_2*..., with
whatever off-diagonal mass is left.  Everything is written as the definition (explicit
reflector matrices, explicit rotation matrices, T - mu*I = QR, T' = RQ + mu*I); nothing
is shared with the GPU path, which uses an O(n) recurrence.  Test infrastructure only.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np


def householder_tridiagonalize(A: np.ndarray):
    """Sec. 3.1: T = H_{n-2} ... H_1 A H_1 ... H_{n-2}, P = H_1 ... H_{n-2}, with
    H = I - 2 u u^T / |u|^2 and u the part of column J below the diagonal plus
    sign(x_0)|x| on its first entry (sign(0) = +1); columns are reduced first to last,
    a zero column is skipped.  Returns d (n), e (n-1), P (n x n) with A = P T P^T."""
    T = np.array(A, dtype=np.float64)
    n = T.shape[0]
    T = np.tril(T) + np.tril(T, -1).T           # the lower triangle is the matrix
    P = np.eye(n)
    for J in range(n - 2):
        x = T[J + 1:, J]
        if not np.any(x[1:] != 0.0):
            continue
        sigma = np.linalg.norm(x) * (1.0 if x[0] >= 0.0 else -1.0)
        u = np.zeros(n)
        u[J + 1:] = x
        u[J + 1] += sigma
        H = np.eye(n) - 2.0 * np.outer(u, u) / (u @ u)
        T = H @ T @ H
        P = P @ H
    return np.diag(T).copy(), np.diag(T, -1).copy(), P


def wilkinson_pair(a: float, b: float, d: float):
    """App. A.3: the two eigenvalues of [[a, b], [b, d]]; the first one returned is the
    one closer to d (the lower one when both are equally close)."""
    mean = 0.5 * (a + d)
    rad = np.hypot(0.5 * (a - d), b)
    lo, hi = mean - rad, mean + rad
    if abs(hi - d) < abs(lo - d):
        return hi, lo
    return lo, hi


def qr_step(T: np.ndarray, m: int, mu: float, pivots: list | None = None):
    """Sec. 3.2.1 with the shift of Sec. 3.2.2 on the leading m x m block:
    T - mu I = Q R by m-1 Givens rotations (rotation k annihilates entry (k+1, k)),
    then T' = R Q + mu I.  Returns the updated full matrix and Q (m x m).  If `pivots` is a
    list, the length r of the vector each rotation is computed from is appended to it (a
    rotation from a tiny vector is determined by rounding errors; bookkeeping for tests)."""
    M = T[:m, :m] - mu * np.eye(m)
    Q = np.eye(m)
    for k in range(m - 1):
        x1, x2 = M[k, k], M[k + 1, k]
        r = np.hypot(x1, x2)
        if pivots is not None:
            pivots.append(r)
        c, s = (1.0, 0.0) if r == 0.0 else (x1 / r, x2 / r)
        Gt = np.eye(m)                          # G^T [x1; x2] = [r; 0]
        Gt[k, k], Gt[k, k + 1], Gt[k + 1, k], Gt[k + 1, k + 1] = c, s, -s, c
        M = Gt @ M
        Q = Q @ Gt.T
    out = T.copy()
    step = M @ Q + mu * np.eye(m)
    # RQ of a symmetric tridiagonal matrix is symmetric tridiagonal; what rounding
    # leaves outside the band (1e-16) is dropped so that T stays in that form
    band = np.diag(np.diag(step)) + np.diag(np.diag(step, -1), -1) + np.diag(np.diag(step, -1), 1)
    out[:m, :m] = band
    return out, Q


@dataclass
class LockstepResult:
    evals: np.ndarray                 # [batch][n] ascending
    evecs: np.ndarray                 # [batch][n][n], columns in the order of evals
    reductions: np.ndarray            # [batch] rows dropped (all equal when uniform)
    offdiag: np.ndarray               # [batch][n-1] sub-diagonal left at the end (dropped entries as they were when dropped)
    window: list = field(default_factory=list)     # window size at the start of each iteration: [iterations][batch]
    last_e: list = field(default_factory=list)     # |last sub-diagonal of the window| after each iteration: [iterations][batch]
    min_pivot: np.ndarray = None      # [batch] shortest vector any rotation of the run was computed from


def tridiag_qr_lockstep(d: np.ndarray, e: np.ndarray, eps: float = 1e-5, iterations: int | None = None,
                        uniform: bool = True, test_each_step: bool = False, V0: np.ndarray | None = None,
                        sort: bool = True) -> LockstepResult:
    """App. B: `iterations` (default n) outer iterations on a batch of tridiagonal
    matrices (d [batch][n], e [batch][n-1]), each two QR steps shifted by the eigenvalue
    of the trailing 2x2 block of the window closer to its last diagonal entry, then by
    the other one, both taken from the matrix the iteration starts from.  The window
    shrinks by one when |last sub-diagonal| <= eps (for every matrix of the batch if
    `uniform`); the test runs after each outer iteration, or after each of its two QR
    steps if `test_each_step` (Sec. 3.2.3 places the test after an iteration and App. C.4
    counts reductions per QR iteration; whether that means the pair of steps or each
    single step is open, so both are available).  V0 (default identity)
    is multiplied by the rotations from the right."""
    d = np.asarray(d, dtype=np.float64)
    e = np.asarray(e, dtype=np.float64)
    batch, n = d.shape
    iterations = n if iterations is None else iterations
    T = [np.diag(d[b]) + np.diag(e[b, :n - 1], -1) + np.diag(e[b, :n - 1], 1) for b in range(batch)]
    V = [np.eye(n) if V0 is None else np.array(V0[b], dtype=np.float64) for b in range(batch)]
    m = np.full(batch, n, dtype=np.int64)
    res = LockstepResult(None, None, None, None)
    pivots = [[] for _ in range(batch)]
    for _ in range(iterations):
        res.window.append(m.copy())
        shifts = [wilkinson_pair(T[b][m[b] - 2, m[b] - 2], T[b][m[b] - 1, m[b] - 2], T[b][m[b] - 1, m[b] - 1])
                  if m[b] >= 2 else (0.0, 0.0) for b in range(batch)]
        for half in range(2):
            last = np.zeros(batch)
            for b in range(batch):
                mb = int(m[b])
                if mb < 2:
                    continue
                T[b], Q = qr_step(T[b], mb, shifts[b][half], pivots[b])
                V[b][:, :mb] = V[b][:, :mb] @ Q
                last[b] = abs(T[b][mb - 1, mb - 2])
            if half == 1:
                res.last_e.append(last)
            if half == 1 or test_each_step:
                ok = (last <= eps) & (m >= 2)
                if uniform:
                    if np.all(ok | (m < 2)) and np.any(m >= 2):
                        m = np.where(m >= 2, m - 1, m)
                else:
                    m = np.where(ok, m - 1, m)
    lam = np.stack([np.diag(T[b]) for b in range(batch)])
    Vs = np.stack(V)
    if sort:
        order = np.argsort(lam, axis=1, kind="stable")
        lam = np.take_along_axis(lam, order, axis=1)
        Vs = np.take_along_axis(Vs, order[:, None, :], axis=2)
    res.evals, res.evecs = lam, Vs
    res.reductions = n - m
    res.min_pivot = np.array([min(pv) if pv else np.inf for pv in pivots])
    res.offdiag = np.stack([np.diag(T[b], -1) for b in range(batch)]) if n > 1 else np.zeros((batch, 0))
    return res


def syevd_lockstep(A: np.ndarray, eps: float = 1e-5, iterations: int | None = None,
                   uniform: bool = True, test_each_step: bool = False) -> LockstepResult:
    """The whole procedure on a batch of symmetric matrices [batch][n][n]."""
    A = np.asarray(A, dtype=np.float64)
    batch, n, _ = A.shape
    d = np.zeros((batch, n))
    e = np.zeros((batch, max(n - 1, 0)))
    P = np.zeros((batch, n, n))
    for b in range(batch):
        d[b], e[b], P[b] = householder_tridiagonalize(A[b])
    return tridiag_qr_lockstep(d, e, eps, iterations, uniform, test_each_step, V0=P)
