"""bed_timing_*: per-launch kernel durations from start/stop events attached to the library's
own launches (the figures bench.py's roofline uses)."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def test_timed_launches_are_counted_ordered_and_plausible():
    import torch
    from paper_2207_04228_amd import binding, workloads
    pts = dict(workloads.headline_points())
    A32 = torch.from_numpy(pts[32]).to("cuda:0")
    A8 = torch.from_numpy(pts[8]).to("cuda:0")
    ev32, V32 = torch.empty((512, 32), device="cuda:0"), torch.empty((512, 32, 32), device="cuda:0")
    ev8, V8 = torch.empty((512, 8), device="cuda:0"), torch.empty((512, 8, 8), device="cuda:0")
    for _ in range(3):
        binding.bed_syevd(A32, ev32, V32)
        binding.bed_syevd(A8, ev8, V8)
    torch.cuda.synchronize()
    ref32, ref8 = ev32.clone(), ev8.clone()

    # event-bracketed loop as the yardstick
    stream = torch.cuda.current_stream()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    for _ in range(20):
        binding.bed_syevd(A32, ev32, V32)
    e1.record(stream)
    torch.cuda.synchronize()
    loop_us = e0.elapsed_time(e1) * 1e3 / 20

    binding.bed_timing_begin(12)
    binding.bed_syevd(A8, ev8, V8)                 # not armed yet: untimed
    binding.bed_timing_arm(True)
    for _ in range(5):
        binding.bed_syevd(A32, ev32, V32)
        binding.bed_syevd(A8, ev8, V8)
    binding.bed_timing_arm(False)
    binding.bed_syevd(A32, ev32, V32)              # untimed again
    us, count = binding.bed_timing_end(12)
    torch.cuda.synchronize()
    assert count == 10 and us.shape == (10,)
    t32, t8 = us[0::2], us[1::2]
    print(f"[timing] n=32: {t32}  n=8: {t8}  event loop per launch: {loop_us:.1f} us", flush=True)
    assert np.all(t32 > 0.5 * loop_us) and np.all(t32 < 1.1 * loop_us + 2.0)   # the kernel itself, no launch gap
    assert np.all(t8 > 2.0) and np.all(t8 < 0.5 * t32.min())
    # timed launches compute what untimed ones do
    assert torch.equal(ev32, ref32) and torch.equal(ev8, ref8)


def test_capacity_is_a_limit_not_an_error_and_state_is_cleared():
    import torch
    from paper_2207_04228_amd import binding, workloads
    A = torch.from_numpy(workloads.config3(8, batch=64)).to("cuda:0")
    ev, V = torch.empty((64, 8), device="cuda:0"), torch.empty((64, 8, 8), device="cuda:0")
    binding.bed_timing_begin(3)
    binding.bed_timing_arm(True)
    for _ in range(7):
        binding.bed_syevd(A, ev, V)                # launches 4 .. 7 run untimed
    us, count = binding.bed_timing_end(2)          # fewer slots than timed launches: first two returned
    assert count == 3 and us.shape == (2,) and np.all(us > 0)
    with pytest.raises(binding.BedError):
        binding.bed_timing_arm(True)               # the timer is gone
    binding.bed_syevd(A, ev, V)                    # and launches are plain again
    torch.cuda.synchronize()
