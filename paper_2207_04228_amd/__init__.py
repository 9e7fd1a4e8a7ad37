"""bed -- batched symmetric eigendecomposition for MI355X (gfx950).

Python binding over the C-ABI library ``libbed.so`` (see ``include/bed.h``).
The library is loaded lazily on first use; importing this package never
touches the GPU.
"""
from .binding import (  # noqa: F401
    BED_FAMILY_AUTO,
    BED_FAMILY_BLOCK,
    BED_FAMILY_LANE,
    BED_FAMILY_PACKED,
    BED_FAMILY_PAIR,
    BED_FAMILY_PACKED_ROWS,
    BED_FAMILY_WAVE,
    BED_FN_INV_SQRT,
    BED_GRAD_EXACT,
    BED_GRAD_TAYLOR,
    BED_FN_SQRT,
    BedError,
    bed_ceiling_copy,
    bed_timing_begin,
    bed_timing_arm,
    bed_timing_end,
    bed_ceiling_fma,
    bed_kernel_variant,
    bed_spd_fn,
    bed_spd_fn_backward,
    bed_syevd_backward,
    bed_syevd,
    bed_syevd_info,
    bed_syevd_lockstep,
    bed_syevd_tol,
    bed_syevd_lockstep_static,
    bed_syevd_lockstep_static_capacity,
    bed_tridiag,
    bed_tridiag_qr,
    bed_tridiag_qr_sweeps,
    bed_version,
    bed_status_string,
    library_path,
    load_library,
)
from . import autograd  # noqa: F401,E402  (torch is imported on first use only)
