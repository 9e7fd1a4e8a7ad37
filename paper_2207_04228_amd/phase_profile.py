"""Phase-resolved cycle counts of the one-wavefront-per-matrix kernel on the headline workload.

    python -m paper_2207_04228_amd.phase_profile [--n 32] [--build-only]

Builds csrc/profiling/bed_phase_profile.hip (the product's kernel source compiled with
BED_PHASE_CLOCKS) into libbed_phases.so beside libbed.so, runs it on the batch-512 input of the benchmark and
prints, as a markdown table, the shader-clock cycles each phase takes: mean over the wavefronts and
the values of the wavefront that finishes last (which is what the launch lasts).
"""
from __future__ import annotations

import argparse
import ctypes
import os
import subprocess
import sys

from . import build as _build

PHASES = ["load + pre-scale", "tridiagonalisation", "iteration boundary (deflation test, window, shifts, first loads)",
          "fill (two rotations of the first sweep, role set-up)", "steady-state steps", "drain (three closing steps, stores)",
          "sort + store", "outer iterations (count)"]
LIB = os.path.join(_build.HERE, "libbed_phases.so")     # beside libbed.so: ignored by git, travels with the tree


def build_profiling_library() -> str:
    src = os.path.join(_build.CSRC, "profiling", "bed_phase_profile.hip")
    cmd = [_build.HIPCC] + _build.FLAGS + ["-shared", src, "-o", LIB]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(r.stderr[-4000:])
    return LIB


def main(argv=None) -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--n", type=int, default=32, choices=[4, 8, 16, 32, 48, 64],
                    help="4..32: the batch-512 input of the benchmark; 48, 64: config 5 (batch 256, clustered spectrum)")
    ap.add_argument("--family", type=int, default=1, choices=[1, 5],
                    help="1: one wavefront per matrix; 5: two wavefronts per matrix (n = 48, 64)")
    ap.add_argument("--build-only", action="store_true")
    a = ap.parse_args(argv)
    if a.build_only or not os.path.exists(LIB):
        print(build_profiling_library(), file=sys.stderr)
        if a.build_only:
            return 0
    import numpy as np
    import torch
    from . import binding, workloads
    lib = ctypes.CDLL(LIB)
    vp, ci = ctypes.c_void_p, ctypes.c_int
    lib.bed_phase_profile.argtypes = [vp, ci, ci, vp, vp, vp, ci, vp]
    lib.bed_phase_profile.restype = ci
    A32 = workloads.config5(a.n) if a.n >= 48 else dict(workloads.headline_points())[a.n]
    dev = torch.device("cuda:0")
    A = torch.from_numpy(A32).to(dev)
    batch, n = A.shape[0], a.n
    ev = torch.empty((batch, n), dtype=torch.float32, device=dev)
    V = torch.empty((batch, n, n), dtype=torch.float32, device=dev)
    ph = torch.zeros((batch, 8), dtype=torch.int64, device=dev)
    stream = torch.cuda.current_stream()

    def call():
        st = lib.bed_phase_profile(binding._ptr(A), batch, n, binding._ptr(ev), binding._ptr(V), binding._ptr(ph),
                                   a.family, ctypes.c_void_p(stream.cuda_stream))
        assert st == 0, st

    def timed(fn, reps=50):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(reps):
            fn()
        e1.record(stream)
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / reps

    t_instr = timed(call)
    ev2, V2 = torch.empty_like(ev), torch.empty_like(V)
    t_prod = timed(lambda: binding.bed_syevd_info(A, ev2, V2, family=a.family))
    assert torch.equal(ev, ev2) and torch.equal(V, V2), "the profiling build must compute the same result"
    _, _, _, rot = binding.bed_syevd_info(A, ev2, V2, family=a.family)
    p = ph.cpu().numpy().astype(np.float64)
    rot = rot.cpu().numpy().astype(np.float64)
    total = p[:, :7].sum(axis=1)
    last = int(np.argmax(total))
    print(f"n = {n}, batch {batch}, {'one wavefront' if a.family == 1 else 'two wavefronts'} per matrix: product launch {t_prod:.1f} us, instrumented launch {t_instr:.1f} us "
          f"(events around a loop of 50 launches)")
    print(f"rotations per matrix: mean {rot.mean():.0f}, slowest wavefront {rot[last]:.0f}; "
          f"shader clock cycles per wavefront (s_memtime):\n")
    print("| phase | mean cycles | share | slowest wavefront | share |")
    print("|---|---|---|---|---|")
    for i, name in enumerate(PHASES[:7]):
        print(f"| {name} | {p[:, i].mean():.0f} | {100 * p[:, i].mean() / total.mean():.1f} % | {p[last, i]:.0f} | "
              f"{100 * p[last, i] / total[last]:.1f} % |")
    print(f"| total | {total.mean():.0f} | 100 % | {total[last]:.0f} | 100 % |")
    it = p[:, 7]
    steps = rot / 2.0
    print(f"\nouter iterations: mean {it.mean():.1f}, slowest wavefront {it[last]:.0f}; per outer iteration (mean over "
          f"wavefronts): boundary {(p[:, 2] / it).mean():.0f}, fill {(p[:, 3] / it).mean():.0f}, drain "
          f"{(p[:, 5] / it).mean():.0f} cycles; steady state {(p[:, 4].sum() / steps.sum()):.1f} cycles per pair of "
          f"rotations (one of each sweep), counting all rotations as pairs")
    return 0


if __name__ == "__main__":
    sys.exit(main())
