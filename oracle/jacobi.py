"""TEST ORACLE binding -- not part of the product path.

ctypes wrapper around ``oracle/jacobi.c`` (double-precision cyclic Jacobi, the
plain definition of the result stated in Sec. 3.1 Eq. (1) / end of Sec. 3.2.1
of the paper: A = V diag(lambda) V^T).  Only tests, the smoke check and the
benchmark's cpu_baseline leg may import this module.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "jacobi.c")
_LIB = os.path.join(_HERE, "liboracle_jacobi.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile jacobi.c with gcc (OpenMP) into liboracle_jacobi.so."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c99",
               "-ffp-contract=off", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        dp = ctypes.POINTER(ctypes.c_double)
        fp = ctypes.POINTER(ctypes.c_float)
        ip = ctypes.POINTER(ctypes.c_int)
        lib.oracle_syevd_f64.argtypes = [fp, ctypes.c_int, ctypes.c_int, dp, dp, ip, ctypes.c_int]
        lib.oracle_syevd_f64.restype = ctypes.c_int
        lib.oracle_syevd_f64_in64.argtypes = [dp, ctypes.c_int, ctypes.c_int, dp, dp, ip, ctypes.c_int]
        lib.oracle_syevd_f64_in64.restype = ctypes.c_int
        lib.oracle_max_threads.argtypes = []
        lib.oracle_max_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def max_threads() -> int:
    return int(_load().oracle_max_threads())


def syevd(A: np.ndarray, threads: int = 0, return_sweeps: bool = False):
    """Eigendecomposition of a batch of symmetric matrices, in float64.

    A: [batch, n, n] float32 (the exact array handed to the GPU) or float64.
    Returns (evals [batch, n] ascending, evecs [batch, n, n] columns =
    eigenvectors), both float64; optionally the Jacobi sweep counts and the
    thread count used.
    """
    lib = _load()
    A = np.asarray(A)
    if A.ndim == 2:
        A = A[None]
    if A.ndim != 3 or A.shape[1] != A.shape[2]:
        raise ValueError("A must be [batch, n, n]")
    batch, n, _ = A.shape
    evals = np.empty((batch, n), dtype=np.float64)
    evecs = np.empty((batch, n, n), dtype=np.float64)
    sweeps = np.zeros((batch,), dtype=np.int32)
    dp = ctypes.POINTER(ctypes.c_double)
    ip = ctypes.POINTER(ctypes.c_int)
    if A.dtype == np.float32:
        Ac = np.ascontiguousarray(A)
        used = lib.oracle_syevd_f64(Ac.ctypes.data_as(ctypes.POINTER(ctypes.c_float)),
                                    batch, n, evals.ctypes.data_as(dp),
                                    evecs.ctypes.data_as(dp), sweeps.ctypes.data_as(ip),
                                    int(threads))
    else:
        Ac = np.ascontiguousarray(A, dtype=np.float64)
        used = lib.oracle_syevd_f64_in64(Ac.ctypes.data_as(dp), batch, n,
                                         evals.ctypes.data_as(dp), evecs.ctypes.data_as(dp),
                                         sweeps.ctypes.data_as(ip), int(threads))
    if used < 0:
        raise ValueError("oracle_syevd_f64: bad arguments")
    if return_sweeps:
        return evals, evecs, sweeps, used
    return evals, evecs
