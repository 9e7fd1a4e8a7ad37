"""ctypes binding over libbed.so -- argument marshalling only.

Every function takes torch CUDA tensors (used purely as device buffers),
passes their raw pointers and the current HIP stream to the C ABI declared in
``include/bed.h`` and raises ``BedError`` on a negative status.  There is no
CPU fallback: if the library is missing, loading fails loudly.
"""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libbed.so")
_lib = None

BED_MAX_N = 128
# fields of the per-matrix info word (include/bed.h)
BED_INFO_COUNT_MASK = 0xFFFF
BED_INFO_RELAXED_SHIFT = 16


class BedError(RuntimeError):
    def __init__(self, status: int, what: str):
        super().__init__(f"{what}: {bed_status_string(status)} ({status})")
        self.status = status


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """dlopen libbed.so (built in-tree by ``paper_2207_04228_amd.build``)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise FileNotFoundError(
                f"{_LIB_PATH} not found: build it with "
                "`python -m paper_2207_04228_amd.build` (needs hipcc)")
        lib = ctypes.CDLL(_LIB_PATH)
        vp, ci = ctypes.c_void_p, ctypes.c_int
        lib.bed_syevd.argtypes = [vp, ci, ci, vp, vp, vp]
        lib.bed_syevd.restype = ci
        lib.bed_syevd_info.argtypes = [vp, ci, ci, vp, vp, vp, vp, vp]
        lib.bed_syevd_info.restype = ci
        lib.bed_syevd_family.argtypes = [vp, ci, ci, vp, vp, vp, vp, ci, vp]
        lib.bed_syevd_family.restype = ci
        lib.bed_syevd_tol.argtypes = [vp, ci, ci, vp, vp, vp, vp, ctypes.c_float, ci, vp]
        lib.bed_syevd_tol.restype = ci
        lib.bed_tridiag.argtypes = [vp, ci, ci, vp, vp, vp, vp]
        lib.bed_tridiag.restype = ci
        lib.bed_tridiag_qr.argtypes = [vp, vp, ci, ci, vp, vp, vp, vp, vp]
        lib.bed_tridiag_qr.restype = ci
        lib.bed_tridiag_qr_sweeps.argtypes = [vp, vp, ci, ci, ci, vp, vp, vp, vp, vp]
        lib.bed_tridiag_qr_sweeps.restype = ci
        lib.bed_spd_fn.argtypes = [vp, ci, ci, ci, ctypes.c_float, vp, vp, vp, vp]
        lib.bed_spd_fn.restype = ci
        lib.bed_syevd_backward.argtypes = [vp, vp, vp, vp, ci, ci, ci, ci, ctypes.c_float, vp, vp]
        lib.bed_syevd_backward.restype = ci
        lib.bed_spd_fn_backward.argtypes = [vp, vp, vp, ci, ci, ci, ctypes.c_float, vp, vp]
        lib.bed_spd_fn_backward.restype = ci
        lib.bed_syevd_lockstep_workspace.argtypes = [ci, ci, ci]
        lib.bed_syevd_lockstep_workspace.restype = ctypes.c_size_t
        lib.bed_syevd_lockstep.argtypes = [vp, ci, ci, ctypes.c_float, ci, ci, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
        lib.bed_syevd_lockstep.restype = ci
        lib.bed_syevd_lockstep_static_capacity.argtypes = []
        lib.bed_syevd_lockstep_static_capacity.restype = ctypes.c_size_t
        lib.bed_syevd_lockstep_static.argtypes = [vp, ci, ci, ctypes.c_float, ci, ci, vp, vp, vp, vp, vp]
        lib.bed_syevd_lockstep_static.restype = ci
        lib.bed_ceiling_fma.argtypes = [vp, ci, ci, ci, ci, vp]
        lib.bed_ceiling_fma.restype = ci
        lib.bed_ceiling_copy.argtypes = [vp, vp, ctypes.c_size_t, ci, vp]
        lib.bed_ceiling_copy.restype = ci
        lib.bed_timing_begin.argtypes = [ci]
        lib.bed_timing_begin.restype = ci
        lib.bed_timing_arm.argtypes = [ci]
        lib.bed_timing_arm.restype = ci
        lib.bed_timing_end.argtypes = [vp, ci, vp]
        lib.bed_timing_end.restype = ci
        lib.bed_kernel_variant.argtypes = [ci, ci, ci]
        lib.bed_kernel_variant.restype = ctypes.c_char_p
        lib.bed_status_string.argtypes = [ci]
        lib.bed_status_string.restype = ctypes.c_char_p
        lib.bed_version.argtypes = []
        lib.bed_version.restype = ci
        _lib = lib
    return _lib


def bed_kernel_variant(batch: int, n: int, want_vectors: bool = True) -> str:
    """Name of the kernel bed_syevd launches for this batch and n."""
    r = load_library().bed_kernel_variant(int(batch), int(n), 1 if want_vectors else 0)
    if r is None:
        raise ValueError("batch or n out of range")
    return r.decode()


def bed_ceiling_fma(out, blocks, threads, chains, iters, *, stream=None):
    """Measurement aid: `chains` independent chains of `iters` plain FMAs per lane.
    Returns the flops of the launch."""
    import torch
    _check_dev(out, "out", torch.float32, (int(blocks) * int(threads),))
    st = load_library().bed_ceiling_fma(_ptr(out), int(blocks), int(threads), int(chains), int(iters), _stream(stream))
    if st != 0:
        raise BedError(st, "bed_ceiling_fma")
    return 2.0 * blocks * threads * chains * iters


def bed_ceiling_copy(src, dst, blocks, *, stream=None):
    """Measurement aid: plain device copy src -> dst.  Returns the bytes moved (read + write)."""
    import torch
    _check_dev(src, "src", torch.float32)
    _check_dev(dst, "dst", torch.float32, tuple(src.shape), src)
    st = load_library().bed_ceiling_copy(_ptr(src), _ptr(dst), src.numel(), int(blocks), _stream(stream))
    if st != 0:
        raise BedError(st, "bed_ceiling_copy")
    return 8.0 * src.numel()


def bed_timing_begin(capacity: int) -> None:
    """Measurement aid: prepares per-launch timing of up to `capacity` of this thread's launches."""
    st = load_library().bed_timing_begin(int(capacity))
    if st != 0:
        raise BedError(st, "bed_timing_begin")


def bed_timing_arm(on: bool) -> None:
    """Measurement aid: from now on this thread's launches are (on) / are not (off) timed."""
    st = load_library().bed_timing_arm(1 if on else 0)
    if st != 0:
        raise BedError(st, "bed_timing_arm")


def bed_timing_end(max_count: int):
    """Measurement aid: waits for the timed kernels and returns their durations in microseconds
    (numpy float32, launch order; at most max_count of them) and the number of timed launches."""
    import numpy as np
    us = np.zeros((max(int(max_count), 1),), dtype=np.float32)
    count = ctypes.c_int(0)
    st = load_library().bed_timing_end(us.ctypes.data_as(ctypes.c_void_p), int(max_count), ctypes.byref(count))
    if st != 0:
        raise BedError(st, "bed_timing_end")
    return us[:min(count.value, int(max_count))].copy(), count.value


def bed_version() -> int:
    return int(load_library().bed_version())


def bed_status_string(status: int) -> str:
    return load_library().bed_status_string(int(status)).decode()


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    import torch
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _check_dev(t, name, dtype, shape=None, like=None):
    """A buffer handed to the C ABI: a contiguous CUDA tensor of the given dtype and, where the
    caller supplied it, of exactly the shape (and on the device) the library will write.  The C
    side sees raw pointers only, so a smaller, strided or differently typed buffer would become
    an out-of-bounds device access."""
    import torch
    if not isinstance(t, torch.Tensor):
        raise TypeError(f"{name} must be a torch.Tensor")
    if t.dtype != dtype:
        raise TypeError(f"{name} must be {dtype}, got {t.dtype}")
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name} must have shape {tuple(shape)}, got {tuple(t.shape)}")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    if not t.is_cuda:
        raise TypeError(f"{name} must be a CUDA tensor")
    if like is not None and t.device != like.device:
        raise ValueError(f"{name} is on {t.device}, expected {like.device}")


def _square_batch(A, name="A"):
    if A.dim() != 3 or A.shape[1] != A.shape[2]:
        raise ValueError(f"{name} must be [batch, n, n]")
    return int(A.shape[0]), int(A.shape[1])


def bed_syevd(A, evals=None, evecs=None, *, want_vectors=True, stream=None):
    """Eigendecomposition of A [batch, n, n] (float32, CUDA, symmetric; the
    lower triangle is read).  Returns (evals [batch, n] ascending,
    evecs [batch, n, n] with eigenvectors as columns, or None)."""
    import torch
    _check_dev(A, "A", torch.float32)
    batch, n = _square_batch(A)
    if evals is None:
        evals = torch.empty((batch, n), dtype=torch.float32, device=A.device)
    if evecs is None and want_vectors:
        evecs = torch.empty((batch, n, n), dtype=torch.float32, device=A.device)
    if not want_vectors:
        evecs = None
    _check_dev(evals, "evals", torch.float32, (batch, n), A)
    if evecs is not None:
        _check_dev(evecs, "evecs", torch.float32, (batch, n, n), A)
    st = load_library().bed_syevd(_ptr(A), batch, n, _ptr(evals), _ptr(evecs), _stream(stream))
    if st != 0:
        raise BedError(st, "bed_syevd")
    return evals, evecs


BED_FAMILY_AUTO, BED_FAMILY_WAVE, BED_FAMILY_PACKED, BED_FAMILY_LANE, BED_FAMILY_BLOCK, BED_FAMILY_PAIR, BED_FAMILY_PACKED_ROWS = range(7)


def bed_syevd_info(A, evals=None, evecs=None, *, want_vectors=True, stream=None, family=BED_FAMILY_AUTO):
    """bed_syevd plus (info int32 [batch], rotations int32-view of uint32 [batch]); `family`
    forces one kernel family (bed_syevd_family)."""
    import torch
    _check_dev(A, "A", torch.float32)
    batch, n = _square_batch(A)
    if evals is None:
        evals = torch.empty((batch, n), dtype=torch.float32, device=A.device)
    if evecs is None and want_vectors:
        evecs = torch.empty((batch, n, n), dtype=torch.float32, device=A.device)
    if not want_vectors:
        evecs = None
    _check_dev(evals, "evals", torch.float32, (batch, n), A)
    if evecs is not None:
        _check_dev(evecs, "evecs", torch.float32, (batch, n, n), A)
    info = torch.empty((batch,), dtype=torch.int32, device=A.device)
    rot = torch.empty((batch,), dtype=torch.int32, device=A.device)
    st = load_library().bed_syevd_family(_ptr(A), batch, n, _ptr(evals), _ptr(evecs),
                                         _ptr(info), _ptr(rot), int(family), _stream(stream))
    if st != 0:
        raise BedError(st, "bed_syevd_info")
    return evals, evecs, info, rot


def bed_syevd_tol(A, epsilon_abs=0.0, sweep_cap=0, *, want_vectors=True, stream=None):
    """bed_syevd_info with the paper's absolute deflation threshold (epsilon_abs > 0; App. B: 1e-5; an entry
    is negligible if it passes that or the library's relative test) and / or a cap on the number of sweeps.  Returns (evals, evecs or None, info, rotations)."""
    import torch
    _check_dev(A, "A", torch.float32)
    batch, n = _square_batch(A)
    evals = torch.empty((batch, n), dtype=torch.float32, device=A.device)
    evecs = torch.empty((batch, n, n), dtype=torch.float32, device=A.device) if want_vectors else None
    info = torch.empty((batch,), dtype=torch.int32, device=A.device)
    rot = torch.empty((batch,), dtype=torch.int32, device=A.device)
    st = load_library().bed_syevd_tol(_ptr(A), batch, n, _ptr(evals), _ptr(evecs), _ptr(info), _ptr(rot),
                                      float(epsilon_abs), int(sweep_cap), _stream(stream))
    if st != 0:
        raise BedError(st, "bed_syevd_tol")
    return evals, evecs, info, rot


def bed_tridiag(A, *, want_P=True, stream=None):
    """Householder tridiagonalisation.  Returns (d [batch,n], e [batch,n], P or None)."""
    import torch
    _check_dev(A, "A", torch.float32)
    batch, n = _square_batch(A)
    d = torch.empty((batch, n), dtype=torch.float32, device=A.device)
    e = torch.empty((batch, n), dtype=torch.float32, device=A.device)
    P = torch.empty((batch, n, n), dtype=torch.float32, device=A.device) if want_P else None
    st = load_library().bed_tridiag(_ptr(A), batch, n, _ptr(d), _ptr(e), _ptr(P), _stream(stream))
    if st != 0:
        raise BedError(st, "bed_tridiag")
    return d, e, P


def bed_tridiag_qr(d, e, *, want_vectors=True, stream=None):
    """Shifted QR iterations on tridiagonal (d, e).  Returns (evals, evecs, info, rotations)."""
    import torch
    _check_dev(d, "d", torch.float32)
    _check_dev(e, "e", torch.float32)
    if d.dim() != 2:
        raise ValueError("d must be [batch, n]")
    batch, n = d.shape
    _check_dev(e, "e", torch.float32, (batch, n), d)
    evals = torch.empty((batch, n), dtype=torch.float32, device=d.device)
    evecs = torch.empty((batch, n, n), dtype=torch.float32, device=d.device) if want_vectors else None
    info = torch.empty((batch,), dtype=torch.int32, device=d.device)
    rot = torch.empty((batch,), dtype=torch.int32, device=d.device)
    st = load_library().bed_tridiag_qr(_ptr(d), _ptr(e), batch, n, _ptr(evals), _ptr(evecs),
                                       _ptr(info), _ptr(rot), _stream(stream))
    if st != 0:
        raise BedError(st, "bed_tridiag_qr")
    return evals, evecs, info, rot


def bed_tridiag_qr_sweeps(d, e, sweeps, *, stream=None):
    """At most `sweeps` shifted QR sweeps on tridiagonal (d, e).  Returns (d_out, e_out, Q, rotations)."""
    import torch
    _check_dev(d, "d", torch.float32)
    _check_dev(e, "e", torch.float32)
    if d.dim() != 2:
        raise ValueError("d must be [batch, n]")
    batch, n = d.shape
    _check_dev(e, "e", torch.float32, (batch, n), d)
    d_out = torch.empty_like(d)
    e_out = torch.empty_like(e)
    Q = torch.empty((batch, n, n), dtype=torch.float32, device=d.device)
    rot = torch.empty((batch,), dtype=torch.int32, device=d.device)
    st = load_library().bed_tridiag_qr_sweeps(_ptr(d), _ptr(e), batch, n, int(sweeps), _ptr(d_out), _ptr(e_out),
                                              _ptr(Q), _ptr(rot), _stream(stream))
    if st != 0:
        raise BedError(st, "bed_tridiag_qr_sweeps")
    return d_out, e_out, Q, rot


def bed_syevd_lockstep(A, epsilon=1e-5, iterations=None, uniform=True, *, want_vectors=True, workspace=None,
                       stream=None):
    """The paper's fixed-budget procedure (n outer iterations by default, absolute threshold on the
    last sub-diagonal entry, window shared by the batch if `uniform`).
    Returns (evals, evecs or None, offdiag [batch, n], reductions int32 [batch])."""
    import torch
    _check_dev(A, "A", torch.float32)
    batch, n = _square_batch(A)
    iterations = n if iterations is None else int(iterations)
    lib = load_library()
    need = int(lib.bed_syevd_lockstep_workspace(batch, n, iterations))
    if workspace is None:
        workspace = torch.empty((max(need, 4) // 4,), dtype=torch.int32, device=A.device)
    _check_dev(workspace, "workspace", torch.int32, None, A)     # its size is checked by the library
    evals = torch.empty((batch, n), dtype=torch.float32, device=A.device)
    evecs = torch.empty((batch, n, n), dtype=torch.float32, device=A.device) if want_vectors else None
    offdiag = torch.empty((batch, n), dtype=torch.float32, device=A.device)
    red = torch.empty((batch,), dtype=torch.int32, device=A.device)
    st = lib.bed_syevd_lockstep(_ptr(A), batch, n, float(epsilon), iterations, 1 if uniform else 0, _ptr(evals),
                                _ptr(evecs), _ptr(offdiag), _ptr(red), _ptr(workspace),
                                workspace.numel() * workspace.element_size(), _stream(stream))
    if st != 0:
        raise BedError(st, "bed_syevd_lockstep")
    return evals, evecs, offdiag, red


def bed_syevd_lockstep_static(A, epsilon=1e-5, iterations=None, uniform=True, *, evals=None, evecs=None,
                              offdiag=None, reductions=None, want_vectors=True, stream=None):
    """bed_syevd_lockstep on the library's built-in scratch memory.  With all four output buffers
    supplied, neither this wrapper nor the library allocates anything.
    Returns (evals, evecs or None, offdiag [batch, n], reductions int32 [batch])."""
    import torch
    _check_dev(A, "A", torch.float32)
    batch, n = _square_batch(A)
    iterations = n if iterations is None else int(iterations)
    if evals is None:
        evals = torch.empty((batch, n), dtype=torch.float32, device=A.device)
    if evecs is None and want_vectors:
        evecs = torch.empty((batch, n, n), dtype=torch.float32, device=A.device)
    if not want_vectors:
        evecs = None
    if offdiag is None:
        offdiag = torch.empty((batch, n), dtype=torch.float32, device=A.device)
    if reductions is None:
        reductions = torch.empty((batch,), dtype=torch.int32, device=A.device)
    _check_dev(evals, "evals", torch.float32, (batch, n), A)
    if evecs is not None:
        _check_dev(evecs, "evecs", torch.float32, (batch, n, n), A)
    _check_dev(offdiag, "offdiag", torch.float32, (batch, n), A)
    _check_dev(reductions, "reductions", torch.int32, (batch,), A)
    st = load_library().bed_syevd_lockstep_static(_ptr(A), batch, n, float(epsilon), iterations, 1 if uniform else 0,
                                                  _ptr(evals), _ptr(evecs), _ptr(offdiag), _ptr(reductions),
                                                  _stream(stream))
    if st != 0:
        raise BedError(st, "bed_syevd_lockstep_static")
    return evals, evecs, offdiag, reductions


def bed_syevd_lockstep_static_capacity() -> int:
    return int(load_library().bed_syevd_lockstep_static_capacity())


BED_FN_SQRT = 0
BED_FN_INV_SQRT = 1


def bed_spd_fn(A, fn, floor, out=None, *, want_evals=False, stream=None):
    """out_b = V_b f(max(Lambda_b, floor)) V_b^T for fn in {BED_FN_SQRT, BED_FN_INV_SQRT}.
    Returns (out [batch, n, n], evals or None, info int32 [batch])."""
    import torch
    _check_dev(A, "A", torch.float32)
    batch, n = _square_batch(A)
    if out is None:
        out = torch.empty((batch, n, n), dtype=torch.float32, device=A.device)
    _check_dev(out, "out", torch.float32, (batch, n, n), A)
    evals = torch.empty((batch, n), dtype=torch.float32, device=A.device) if want_evals else None
    info = torch.empty((batch,), dtype=torch.int32, device=A.device)
    st = load_library().bed_spd_fn(_ptr(A), batch, n, int(fn), float(floor), _ptr(out), _ptr(evals),
                                   _ptr(info), _stream(stream))
    if st != 0:
        raise BedError(st, "bed_spd_fn")
    return out, evals, info


BED_GRAD_EXACT = 0
BED_GRAD_TAYLOR = 1


def bed_syevd_backward(evals, evecs, grad_evals=None, grad_evecs=None, *, mode=BED_GRAD_TAYLOR, degree=9,
                       gap_floor=0.0, grad_A=None, stream=None):
    """grad_A = V (diag(grad_evals) + sym(K o (V^T grad_evecs))) V^T, the gradient with respect to A."""
    import torch
    _check_dev(evals, "evals", torch.float32)
    _check_dev(evecs, "evecs", torch.float32)
    batch, n = _square_batch(evecs, "evecs")
    _check_dev(evals, "evals", torch.float32, (batch, n), evecs)
    for t, name, shape in ((grad_evals, "grad_evals", (batch, n)), (grad_evecs, "grad_evecs", (batch, n, n))):
        if t is not None:
            _check_dev(t, name, torch.float32, shape, evecs)
    if grad_A is None:
        grad_A = torch.empty((batch, n, n), dtype=torch.float32, device=evecs.device)
    _check_dev(grad_A, "grad_A", torch.float32, (batch, n, n), evecs)
    st = load_library().bed_syevd_backward(_ptr(evals), _ptr(evecs), _ptr(grad_evals), _ptr(grad_evecs), batch, n,
                                           int(mode), int(degree), float(gap_floor), _ptr(grad_A), _stream(stream))
    if st != 0:
        raise BedError(st, "bed_syevd_backward")
    return grad_A


def bed_spd_fn_backward(evals, evecs, grad_out, fn, floor, *, grad_A=None, stream=None):
    """Gradient of <grad_out, V f(max(Lambda, floor)) V^T> with respect to A."""
    import torch
    _check_dev(evals, "evals", torch.float32)
    _check_dev(evecs, "evecs", torch.float32)
    _check_dev(grad_out, "grad_out", torch.float32)
    batch, n = _square_batch(evecs, "evecs")
    _check_dev(evals, "evals", torch.float32, (batch, n), evecs)
    _check_dev(grad_out, "grad_out", torch.float32, (batch, n, n), evecs)
    if grad_A is None:
        grad_A = torch.empty((batch, n, n), dtype=torch.float32, device=evecs.device)
    _check_dev(grad_A, "grad_A", torch.float32, (batch, n, n), evecs)
    st = load_library().bed_spd_fn_backward(_ptr(evals), _ptr(evecs), _ptr(grad_out), batch, n, int(fn),
                                            float(floor), _ptr(grad_A), _stream(stream))
    if st != 0:
        raise BedError(st, "bed_spd_fn_backward")
    return grad_A
