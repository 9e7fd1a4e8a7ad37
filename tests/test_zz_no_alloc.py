"""bed_syevd_lockstep_static (the lock-step procedure on the library's built-in scratch memory,
for callers that cannot allocate) against bed_syevd_lockstep with a caller-owned workspace:
same kernels, same arithmetic, so the outputs must be bit-identical, on two calls in a row, the
second with a smaller input (the scratch array keeps the first call's contents)."""
import ctypes

import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def _inputs(n, batch, seed):
    from paper_2207_04228_amd import workloads
    return workloads.covariance(batch, n, 4 * n, 1e-4, seed)


def _call_both(A32, eps, iterations, uniform):
    """Both entry points through the C ABI (raw pointers), outputs pre-allocated by the test."""
    import torch
    from paper_2207_04228_amd import binding
    lib = binding.load_library()
    dev = torch.device("cuda:0")
    batch, n, _ = A32.shape
    A = torch.from_numpy(A32).to(dev)
    outs = []
    for static in (False, True):
        ev = torch.full((batch, n), float("nan"), dtype=torch.float32, device=dev)
        V = torch.full((batch, n, n), float("nan"), dtype=torch.float32, device=dev)
        off = torch.full((batch, n), float("nan"), dtype=torch.float32, device=dev)
        red = torch.full((batch,), -7, dtype=torch.int32, device=dev)
        stream = binding._stream(None)
        if static:
            st = lib.bed_syevd_lockstep_static(binding._ptr(A), batch, n, ctypes.c_float(eps), iterations,
                                               1 if uniform else 0, binding._ptr(ev), binding._ptr(V),
                                               binding._ptr(off), binding._ptr(red), stream)
        else:
            need = int(lib.bed_syevd_lockstep_workspace(batch, n, iterations))
            ws = torch.empty((need // 4,), dtype=torch.int32, device=dev)
            st = lib.bed_syevd_lockstep(binding._ptr(A), batch, n, ctypes.c_float(eps), iterations,
                                        1 if uniform else 0, binding._ptr(ev), binding._ptr(V),
                                        binding._ptr(off), binding._ptr(red), binding._ptr(ws),
                                        ctypes.c_size_t(need), stream)
        assert st == 0, binding.bed_status_string(st)
        torch.cuda.synchronize()
        outs.append((ev.cpu().numpy(), V.cpu().numpy(), off.cpu().numpy(), red.cpu().numpy()))
    return outs


@pytest.mark.parametrize("uniform", [True, False])
def test_static_scratch_matches_caller_workspace_twice_in_a_row(uniform):
    # first call: 512 matrices of 32 x 32 with App. B's budget; second call: fewer and smaller
    # matrices and fewer iterations, on scratch memory that still holds the first call's state
    for (n, batch, iterations, seed) in ((32, 512, 32, 11), (16, 100, 9, 12), (4, 3, 4, 13)):
        print(f"[no-alloc] n={n} batch={batch} iterations={iterations} uniform={uniform}", flush=True)
        A = _inputs(n, batch, seed)
        (ev0, V0, off0, red0), (ev1, V1, off1, red1) = _call_both(A, 1e-5, iterations, uniform)
        assert np.isfinite(ev0).all() and np.isfinite(V0).all() and np.isfinite(off0).all()
        assert np.array_equal(ev0, ev1)
        assert np.array_equal(V0, V1)
        assert np.array_equal(off0, off1)
        assert np.array_equal(red0, red1)
        assert (red0 >= 0).all()


def test_static_scratch_rejects_what_does_not_fit_and_bad_arguments():
    import torch
    from paper_2207_04228_amd import binding
    lib = binding.load_library()
    cap = int(lib.bed_syevd_lockstep_static_capacity())
    assert cap == 1 << 20
    dev = torch.device("cuda:0")
    n, batch = 64, 4096                      # 2 * 4096 * 64 * 4 bytes = 2 MiB of state: too large
    assert int(lib.bed_syevd_lockstep_workspace(batch, n, n)) > cap
    A = torch.zeros((batch, n, n), dtype=torch.float32, device=dev)
    ev = torch.zeros((batch, n), dtype=torch.float32, device=dev)
    st = lib.bed_syevd_lockstep_static(binding._ptr(A), batch, n, ctypes.c_float(1e-5), n, 1, binding._ptr(ev),
                                       None, None, None, None)
    assert st == -8 and "scratch" in binding.bed_status_string(st)
    assert lib.bed_syevd_lockstep_static(None, 4, 8, ctypes.c_float(1e-5), 8, 1, binding._ptr(ev), None, None, None,
                                         None) == -1
    assert lib.bed_syevd_lockstep_static(binding._ptr(A), 4, 8, ctypes.c_float(-1.0), 8, 1, binding._ptr(ev), None,
                                         None, None, None) == -7
    assert lib.bed_syevd_lockstep_static(binding._ptr(A), 0, 8, ctypes.c_float(1e-5), 8, 1, binding._ptr(ev), None,
                                         None, None, None) == 0
    torch.cuda.synchronize()


def test_wrapper_with_preallocated_outputs():
    import torch
    from paper_2207_04228_amd import binding
    A32 = _inputs(8, 64, 21)
    dev = torch.device("cuda:0")
    A = torch.from_numpy(A32).to(dev)
    ref = binding.bed_syevd_lockstep(A, 1e-5, 8, False)
    ev = torch.empty((64, 8), dtype=torch.float32, device=dev)
    V = torch.empty((64, 8, 8), dtype=torch.float32, device=dev)
    off = torch.empty((64, 8), dtype=torch.float32, device=dev)
    red = torch.empty((64,), dtype=torch.int32, device=dev)
    got = binding.bed_syevd_lockstep_static(A, 1e-5, 8, False, evals=ev, evecs=V, offdiag=off, reductions=red)
    torch.cuda.synchronize()
    assert got[0] is ev and got[1] is V and got[2] is off and got[3] is red
    for r, g in zip(ref, got):
        assert torch.equal(r, g)
