"""TEST INFRASTRUCTURE -- acceptance metrics for an eigendecomposition.

Given the input batch, a candidate (evals, evecs) and the oracle's (evals,
evecs), compute in float64 the four quantities the parity bar is stated in:

  (i)   eigenvalue error   max_i |l_i - l_i^oracle| / ||A||_2
  (ii)  residual           ||A V - V L||_F / ||A||_F
  (iii) orthogonality      ||V^T V - I||_F
  (iv)  eigenvector angle  for every eigenvalue cluster that is separated from
        the rest of the spectrum by at least ``gap_rel * ||A||_2``:
        ||(I - Vo Vo^T) Vc||_2, the sine of the largest principal angle
        between the candidate's and the oracle's invariant subspace (for a
        cluster of size one this is the sign-free angle between the vectors).

These follow the definition A = V L V^T (Sec. 3.1 Eq. (1) and the closing
equation of Sec. 3.2.1 of the paper); nothing here depends on how either side
computed its result.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

GAP_REL_DEFAULT = 5e-3


def mirror_lower(A: np.ndarray) -> np.ndarray:
    """float64 copy of A with the lower triangle mirrored to the upper."""
    A = np.asarray(A, dtype=np.float64)
    L = np.tril(A)
    return L + np.swapaxes(np.tril(A, -1), -1, -2)


@dataclass
class Acceptance:
    eval_err: np.ndarray      # [batch]   (i)
    residual: np.ndarray      # [batch]   (ii)
    orth: np.ndarray          # [batch]   (iii)
    angle: np.ndarray         # [batch]   (iv) max over gapped clusters (0 if none)
    n_gapped_clusters: np.ndarray  # [batch]
    n: int

    def worst(self):
        return dict(eval_err=float(np.max(self.eval_err, initial=0.0)),
                    residual=float(np.max(self.residual, initial=0.0)),
                    orth=float(np.max(self.orth, initial=0.0)),
                    angle=float(np.max(self.angle, initial=0.0)))

    def passes(self, eval_tol=1e-5, res_tol=1e-5, orth_tol=1e-5, angle_tol=1e-3):
        n = self.n
        w = self.worst()
        return (np.isfinite(list(w.values())).all()
                and w["eval_err"] <= eval_tol
                and w["residual"] <= res_tol * n
                and w["orth"] <= orth_tol * n
                and w["angle"] <= angle_tol)


def clusters(lam: np.ndarray, thresh: float):
    """Split ascending eigenvalues into maximal runs whose internal gaps are
    < thresh.  Returns a list of (start, stop) index pairs."""
    n = lam.shape[0]
    out = []
    s = 0
    for i in range(1, n):
        if lam[i] - lam[i - 1] >= thresh:
            out.append((s, i))
            s = i
    out.append((s, n))
    return out


def evaluate(A, evals, evecs, evals_ref, evecs_ref, gap_rel: float = GAP_REL_DEFAULT) -> Acceptance:
    A64 = mirror_lower(A)
    if A64.ndim == 2:
        A64 = A64[None]
    L = np.asarray(evals, dtype=np.float64).reshape(A64.shape[0], -1)
    V = np.asarray(evecs, dtype=np.float64).reshape(A64.shape)
    Lr = np.asarray(evals_ref, dtype=np.float64).reshape(L.shape)
    Vr = np.asarray(evecs_ref, dtype=np.float64).reshape(A64.shape)
    batch, n, _ = A64.shape

    norm2 = np.max(np.abs(Lr), axis=1)
    normF = np.sqrt(np.sum(A64 * A64, axis=(1, 2)))
    safe2 = np.where(norm2 > 0, norm2, 1.0)
    safeF = np.where(normF > 0, normF, 1.0)

    eval_err = np.max(np.abs(L - Lr), axis=1) / safe2
    R = A64 @ V - V * L[:, None, :]
    residual = np.sqrt(np.sum(R * R, axis=(1, 2))) / safeF
    G = np.swapaxes(V, 1, 2) @ V - np.eye(n)[None]
    orth = np.sqrt(np.sum(G * G, axis=(1, 2)))

    angle = np.zeros(batch)
    ncl = np.zeros(batch, dtype=np.int64)
    for b in range(batch):
        thresh = gap_rel * safe2[b]
        worst = 0.0
        cnt = 0
        for (s, e) in clusters(Lr[b], thresh):
            # a cluster counts when it is separated on both sides (always true
            # by construction of `clusters`) and is not the whole spectrum
            if e - s == n and n > 1:
                continue
            Vo = Vr[b][:, s:e]
            Vc = V[b][:, s:e]
            D = Vc - Vo @ (Vo.T @ Vc)
            sv = np.linalg.norm(D, 2) if np.isfinite(D).all() else np.inf
            worst = max(worst, float(sv))
            cnt += 1
        angle[b] = worst
        ncl[b] = cnt
    return Acceptance(eval_err, residual, orth, angle, ncl, n)
