"""CPU-side checks of the C-ABI library: it loads, exports every symbol that
include/bed.h declares, and rejects bad arguments on the host without
touching a GPU."""
import ctypes
import os
import re

import pytest

from paper_2207_04228_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.library_path()):
        from paper_2207_04228_amd import build
        build.build()
    return binding.load_library()


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "bed.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(bed_[a-z_0-9]+)\s*\(", text)))


def test_header_symbols_are_exported(lib):
    names = _declared_symbols()
    assert {"bed_syevd", "bed_syevd_info", "bed_syevd_family", "bed_syevd_tol", "bed_tridiag", "bed_tridiag_qr", "bed_tridiag_qr_sweeps", "bed_spd_fn", "bed_syevd_backward", "bed_spd_fn_backward", "bed_syevd_lockstep", "bed_syevd_lockstep_workspace",
            "bed_status_string", "bed_version"} <= set(names)
    for name in names:
        assert hasattr(lib, name), name


def test_timing_calls_without_a_timer_are_refused(lib):
    """The per-launch timing aid keeps its state per thread; nothing here touches a GPU."""
    assert lib.bed_timing_begin(0) == -7
    assert lib.bed_timing_begin(-3) == -7
    assert lib.bed_timing_begin((1 << 20) + 1) == -7
    assert lib.bed_timing_arm(1) == -7                          # no bed_timing_begin before it
    cnt = ctypes.c_int(-1)
    assert lib.bed_timing_end(None, 0, ctypes.byref(cnt)) == -7
    assert cnt.value == -1


def test_version_and_status_strings(lib):
    assert binding.bed_version() == 500
    assert binding.bed_status_string(0) == "BED_OK"
    for code in (-1, -2, -3, -4, -5, -6, -7, -8):
        assert binding.bed_status_string(code).startswith("BED_ERR_")
    assert "UNKNOWN" in binding.bed_status_string(-99)


def test_argument_validation_is_host_side(lib):
    p = lambda x: ctypes.c_void_p(x)
    A, L, V = p(0x10000), p(0x20000), p(0x30000)
    assert lib.bed_syevd(None, 1, 4, L, V, None) == -1          # NULL A
    assert lib.bed_syevd(A, 1, 4, None, V, None) == -1          # NULL evals
    assert lib.bed_syevd(A, -1, 4, L, V, None) == -2            # batch < 0
    assert lib.bed_syevd(A, 1, 0, L, V, None) == -3             # n < 1
    assert lib.bed_syevd(A, 1, 129, L, V, None) == -3           # n > 128
    assert lib.bed_syevd(p(0x10002), 1, 4, L, V, None) == -4    # misaligned
    assert lib.bed_syevd(A, 1, 4, L, p(0x10010), None) == -6    # evecs overlaps A
    assert lib.bed_syevd(A, 0, 4, L, V, None) == 0              # batch 0: no-op
    assert lib.bed_tridiag(A, 1, 4, None, L, V, None) == -1
    assert lib.bed_tridiag(A, 0, 4, L, V, None, None) == 0
    assert lib.bed_tridiag_qr(A, None, 1, 4, L, V, None, None, None) == -1
    assert lib.bed_tridiag_qr(A, L, 0, 4, V, None, None, None, None) == 0
    assert lib.bed_syevd_info(A, 1, 4, L, V, p(0x40001), None, None) == -4
    # the lock-step procedure on built-in scratch memory: argument errors first, then the capacity
    f = ctypes.c_float
    assert lib.bed_syevd_lockstep_static(None, 1, 4, f(1e-5), 4, 1, L, V, None, None, None) == -1
    assert lib.bed_syevd_lockstep_static(A, 1, 65, f(1e-5), 4, 1, L, V, None, None, None) == -3
    assert lib.bed_syevd_lockstep_static(A, 1, 4, f(1e-5), -1, 1, L, V, None, None, None) == -7
    assert lib.bed_syevd_lockstep_static(A, 1, 4, f(1e-5), 4, 2, L, V, None, None, None) == -7
    assert lib.bed_syevd_lockstep_static(A, 0, 4, f(1e-5), 4, 1, L, V, None, None, None) == 0
    assert lib.bed_syevd_lockstep_static(p(0x10000000), 4096, 64, f(1e-5), 64, 1, p(0x20000000), None, None, None,
                                         None) == -8
    assert lib.bed_syevd_lockstep_static_capacity() == 1 << 20
    # measurement aids
    assert lib.bed_ceiling_fma(None, 1, 64, 1, 64, None) == -1
    assert lib.bed_ceiling_fma(A, 1, 65, 1, 64, None) == -7
    assert lib.bed_ceiling_fma(A, 1, 64, 2, 64, None) == -7
    assert lib.bed_ceiling_fma(A, 1, 64, 1, 100, None) == -7
    assert lib.bed_ceiling_copy(A, None, 4, 1, None) == -1
    assert lib.bed_ceiling_copy(p(0x10004), L, 4, 1, None) == -4
    assert lib.bed_ceiling_copy(A, L, 6, 1, None) == -7
    assert binding.bed_kernel_variant(512, 32) == "wave_kernel<32>"
    assert binding.bed_kernel_variant(65536, 4) == "lane_kernel<4>"
    assert binding.bed_kernel_variant(4096, 16) == "packed_kernel<16>"
    assert binding.bed_kernel_variant(4096, 4) == "packed_kernel<4>"
    assert binding.bed_kernel_variant(2048, 16) == "wave_kernel<16>"
    assert binding.bed_kernel_variant(4095, 17) == "wave_kernel<20>"
    assert binding.bed_kernel_variant(4096, 17) == "packed_rows_kernel<20>"
    assert binding.bed_kernel_variant(4096, 32) == "packed_rows_kernel<32>"
    assert binding.bed_kernel_variant(4096, 33) == "wave_kernel<40>"
    assert binding.bed_kernel_variant(256, 100) == "block_kernel"
    assert binding.bed_kernel_variant(256, 64) == "pair_kernel<64>"
    assert binding.bed_kernel_variant(256, 64, want_vectors=False) == "wave_kernel<64>"
    assert binding.bed_kernel_variant(513, 64) == "wave_kernel<64>"
    assert binding.bed_kernel_variant(256, 33) == "pair_kernel<40>"
    assert lib.bed_kernel_variant(1, 129, 1) is None
    f = ctypes.c_float
    assert lib.bed_spd_fn(None, 1, 4, 0, f(0.0), V, None, None, None) == -1        # NULL A
    assert lib.bed_spd_fn(A, 1, 4, 0, f(0.0), None, None, None, None) == -1        # NULL out
    assert lib.bed_spd_fn(A, 1, 4, 2, f(1.0), V, None, None, None) == -7           # unknown function
    assert lib.bed_spd_fn(A, 1, 4, 1, f(0.0), V, None, None, None) == -7           # inverse sqrt, floor 0
    assert lib.bed_spd_fn(A, 1, 4, 0, f(-1.0), V, None, None, None) == -7          # negative floor
    assert lib.bed_spd_fn(A, 1, 4, 0, f(float("nan")), V, None, None, None) == -7  # NaN floor
    assert lib.bed_spd_fn(A, 1, 4, 0, f(float("inf")), V, None, None, None) == -7  # infinite floor
    assert lib.bed_spd_fn(A, 1, 129, 0, f(0.0), V, None, None, None) == -3
    assert lib.bed_spd_fn(A, 1, 4, 0, f(0.0), p(0x10020), None, None, None) == -6  # out overlaps A
    assert lib.bed_spd_fn(A, 0, 4, 0, f(0.0), V, None, None, None) == 0
    O = p(0x50000)
    D2, E2 = p(0x60000), p(0x70000)
    assert lib.bed_tridiag_qr_sweeps(A, L, 1, 4, 0, D2, E2, V, None, None) == -7      # sweeps < 1
    assert lib.bed_tridiag_qr_sweeps(A, L, 1, 65, 2, D2, E2, V, None, None) == -3     # hook limited to n <= 64
    assert lib.bed_tridiag_qr_sweeps(A, L, 1, 4, 2, D2, E2, None, None, None) == -1
    assert lib.bed_tridiag_qr_sweeps(A, L, 1, 4, 2, A, E2, V, None, None) == -6
    assert lib.bed_tridiag_qr_sweeps(A, L, 0, 4, 2, D2, E2, V, None, None) == 0
    assert lib.bed_syevd_backward(L, V, None, None, 1, 4, 0, 9, f(0.0), O, None) == -1      # no gradient given
    assert lib.bed_syevd_backward(None, V, L, None, 1, 4, 0, 9, f(0.0), O, None) == -1
    assert lib.bed_syevd_backward(L, V, L, None, 1, 4, 2, 9, f(0.0), O, None) == -7         # unknown mode
    assert lib.bed_syevd_backward(L, V, L, None, 1, 4, 1, 65, f(0.0), O, None) == -7        # degree out of range
    assert lib.bed_syevd_backward(L, V, L, None, 1, 4, 0, 9, f(float("nan")), O, None) == -7
    assert lib.bed_syevd_backward(L, V, L, None, 1, 4, 0, 9, f(0.0), V, None) == -6         # output aliases evecs
    assert lib.bed_syevd_backward(L, V, L, None, 1, 129, 0, 9, f(0.0), O, None) == -3
    assert lib.bed_spd_fn_backward(L, V, A, 1, 129, 0, f(0.0), O, None) == -3
    assert lib.bed_syevd_backward(L, V, L, None, 0, 4, 0, 9, f(0.0), O, None) == 0
    assert lib.bed_spd_fn_backward(L, V, None, 1, 4, 0, f(0.0), O, None) == -1
    assert lib.bed_spd_fn_backward(L, V, A, 1, 4, 1, f(0.0), O, None) == -7                 # inverse sqrt, floor 0
    assert lib.bed_spd_fn_backward(L, V, A, 1, 4, 3, f(1.0), O, None) == -7
    assert lib.bed_spd_fn_backward(L, V, A, 1, 4, 0, f(0.0), A, None) == -6
    assert lib.bed_spd_fn_backward(L, V, A, 0, 4, 0, f(0.0), O, None) == 0
    # the fixed-budget procedure: workspace size and argument checks (nothing is launched)
    sz = ctypes.c_size_t
    need = lib.bed_syevd_lockstep_workspace(8, 16, 16)
    assert need >= 4 * (2 * 8 * 16 + 16 + 8) and need % 256 == 0
    assert lib.bed_syevd_lockstep_workspace(8, 65, 16) == 0
    W = p(0x800000)
    assert lib.bed_syevd_lockstep(A, 8, 65, f(1e-5), 16, 1, L, V, None, None, W, sz(1 << 20), None) == -3
    assert lib.bed_syevd_lockstep(A, 8, 16, f(1e-5), -1, 1, L, V, None, None, W, sz(need), None) == -7
    assert lib.bed_syevd_lockstep(A, 8, 16, f(1e-5), 16, 2, L, V, None, None, W, sz(need), None) == -7
    assert lib.bed_syevd_lockstep(A, 8, 16, f(float("nan")), 16, 1, L, V, None, None, W, sz(need), None) == -7
    assert lib.bed_syevd_lockstep(A, 8, 16, f(1e-5), 16, 1, L, V, None, None, None, sz(need), None) == -1
    assert lib.bed_syevd_lockstep(A, 8, 16, f(1e-5), 16, 1, L, V, None, None, W, sz(need - 256), None) == -7
    assert lib.bed_syevd_lockstep(A, 8, 16, f(1e-5), 16, 1, L, L, None, None, W, sz(need), None) == -6
    assert lib.bed_syevd_lockstep(A, 8, 16, f(1e-5), 16, 1, L, V, None, None, p(0x30000), sz(need), None) == -6
    assert lib.bed_syevd_lockstep(A, 0, 16, f(1e-5), 16, 1, L, V, None, None, W, sz(need), None) == 0


def test_binding_rejects_cpu_tensors():
    import torch
    with pytest.raises(TypeError):
        binding.bed_syevd(torch.zeros(2, 4, 4))


def test_binding_rejects_mismatched_buffers_before_any_pointer_is_passed():
    """The C side sees raw pointers only: dtype, shape and contiguity of every buffer are checked
    by the binding, in that order, before the device check (so this runs without a GPU)."""
    import torch
    chk = binding._check_dev
    good = torch.zeros((3, 4, 4), dtype=torch.float32)
    with pytest.raises(TypeError, match="float32"):
        chk(good.double(), "evecs", torch.float32, (3, 4, 4))
    with pytest.raises(ValueError, match="shape"):
        chk(torch.zeros((3, 4, 3)), "evecs", torch.float32, (3, 4, 4))
    with pytest.raises(ValueError, match="shape"):
        chk(torch.zeros((2, 4, 4)), "evecs", torch.float32, (3, 4, 4))
    with pytest.raises(ValueError, match="contiguous"):
        chk(good.transpose(1, 2), "evecs", torch.float32, (3, 4, 4))
    with pytest.raises(TypeError, match="torch.Tensor"):
        chk([1.0], "evecs", torch.float32, (1,))
    with pytest.raises(TypeError, match="CUDA"):       # everything else in order: only the device is wrong
        chk(good, "evecs", torch.float32, (3, 4, 4))
    with pytest.raises(ValueError, match=r"\[batch, n, n\]"):
        binding._square_batch(torch.zeros((3, 4, 5)))
