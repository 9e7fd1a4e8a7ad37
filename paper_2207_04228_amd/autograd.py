"""torch.autograd glue over the C ABI: the forward and backward passes are the library's
kernels (bed_syevd / bed_spd_fn and bed_syevd_backward / bed_spd_fn_backward); this module only
saves tensors and routes gradients.  The paper uses the decomposition as a differentiable layer
(Sec. 2: gradients by the truncated series of degree 9; Sec. 4.2-4.4: whitening, covariance
pooling, colouring)."""
from __future__ import annotations

from . import binding


def _functions():
    import torch

    class Syevd(torch.autograd.Function):
        @staticmethod
        def forward(ctx, A, degree):
            evals, evecs = binding.bed_syevd(A.contiguous())
            ctx.save_for_backward(evals, evecs)
            ctx.degree = degree
            return evals, evecs

        @staticmethod
        def backward(ctx, g_evals, g_evecs):
            evals, evecs = ctx.saved_tensors
            g_evals = None if g_evals is None else g_evals.contiguous()
            g_evecs = None if g_evecs is None else g_evecs.contiguous()
            if g_evals is None and g_evecs is None:
                return None, None
            return binding.bed_syevd_backward(evals, evecs, g_evals, g_evecs, mode=binding.BED_GRAD_TAYLOR,
                                              degree=ctx.degree), None

    class SpdFn(torch.autograd.Function):
        @staticmethod
        def forward(ctx, A, fn, floor):
            A = A.contiguous()
            out, _, _ = binding.bed_spd_fn(A, fn, floor)
            ctx.save_for_backward(A)
            ctx.fn, ctx.floor = fn, floor
            return out

        @staticmethod
        def backward(ctx, g_out):
            (A,) = ctx.saved_tensors
            # the fused forward keeps V on chip; the backward needs it, so it is recomputed
            evals, evecs = binding.bed_syevd(A)
            return binding.bed_spd_fn_backward(evals, evecs, g_out.contiguous(), ctx.fn, ctx.floor), None, None

    return Syevd, SpdFn


_cache = None


def _get():
    global _cache
    if _cache is None:
        _cache = _functions()
    return _cache


def eigh(A, degree: int = 9):
    """Differentiable (evals ascending, evecs as columns) of symmetric A [batch, n, n]; the
    gradient uses the truncated series of the given degree for the eigenvalue coupling."""
    return _get()[0].apply(A, degree)


def spd_sqrt(A, floor: float = 0.0):
    """Differentiable A^(1/2) with eigenvalues raised to `floor`."""
    return _get()[1].apply(A, binding.BED_FN_SQRT, float(floor))


def spd_inv_sqrt(A, floor: float = 1e-6):
    """Differentiable A^(-1/2) with eigenvalues raised to `floor` (> 0)."""
    return _get()[1].apply(A, binding.BED_FN_INV_SQRT, float(floor))
