"""TEST ORACLE -- spectral functions of symmetric positive (semi-)definite
matrices, float64: F(A) = V f(max(Lambda, floor)) V^T, which is the definition
the paper's applications use (Sec. 4.2 / App. B.1: whitening with A^(-1/2);
Sec. 4.3 / App. B.2: covariance pooling with A^(1/2); Sec. 4.4 / App. B.3:
whitening and colouring).  The eigendecomposition comes from the float64
Jacobi oracle; nothing here is shared with the GPU path.  Test infrastructure
only.
"""
from __future__ import annotations

import numpy as np

from . import jacobi

FN_SQRT = 0
FN_INV_SQRT = 1


def spd_fn(A: np.ndarray, fn: int, floor: float) -> np.ndarray:
    lam, V = jacobi.syevd(A)
    lam = np.maximum(lam, floor)
    if fn == FN_SQRT:
        g = np.sqrt(lam)
    elif fn == FN_INV_SQRT:
        g = 1.0 / np.sqrt(lam)
    else:
        raise ValueError("unknown fn")
    return (V * g[:, None, :]) @ np.swapaxes(V, 1, 2)
