#!/usr/bin/env python3
"""Benchmark of the batched symmetric eigensolver on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

One *step* is one pass of the whole hot path over the headline workload:
four `bed_syevd` calls, batch 512 each, n = 4, 8, 16, 32 (2048 matrices),
inputs already resident in HBM.  The script prints ONE JSON line:

  value        matrices/s over the K timed steps (wall clock, synchronised)
  per_n        per-call figures for each n (HIP events around every call; the
               dominant call, n = 32, is measured inside the timed region, the
               others in a second pass so that their events do not sit in it)
  roofline     the dominant kernel (n = 32): algorithmic flops / mean launch
               duration against the fp32 vector peak
  cpu_baseline the float64 Jacobi oracle on the host cores, same inputs
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_FP32_TFLOPS = 157.3   # 256 CU x 4 SIMD x 16 lanes x 2 (packed) x 2 flop x 2.4 GHz
PEAK_HBM_GBS = 8000.0


def flops_per_matrix(n: int, rotations: float, vectors: bool = True) -> float:
    """Algorithmic flop model: (4/3)n^3 tridiagonalisation + (4/3)n^3 forming P
    + R rotations x (6n for two columns of V + 20 for the tridiagonal)."""
    f = (4.0 / 3.0) * n ** 3 + rotations * 20.0
    if vectors:
        f += (4.0 / 3.0) * n ** 3 + rotations * 6.0 * n
    return f


def bytes_per_matrix(n: int, vectors: bool = True) -> float:
    return 4.0 * (n * n + n + (n * n if vectors else 0))


def main(argv=None) -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the untimed extra measurements (eigenvalues only, spectral function, large batches)")
    ap.add_argument("--workload", default="headline", choices=["headline"])
    ap.add_argument("--only-n", type=int, default=0,
                    help="profiling aid: launch only the batch-512 call of this n, --steps times, and exit")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MIB",
                    help="profiling aid: run a plain device-to-device copy of MIB mebibytes --steps times and exit "
                         "(reference reading for the FETCH_SIZE / WRITE_SIZE counters)")
    a = ap.parse_args(argv)
    if a.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the batch is embarrassingly parallel; "
              "no multi-GPU path exists) -- rerun with --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2207_04228_amd import binding, workloads

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    binding.load_library()   # fail loudly if libbed.so is missing
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    if a.copy_calibration:
        nbytes = a.copy_calibration << 20
        src = torch.empty(nbytes // 4, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        for _ in range(a.steps):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration_bytes": nbytes, "launches": a.steps}))
        return 0

    points = workloads.headline_points()          # [(n, A32)], batch 512 each
    if a.only_n:
        points = [pt for pt in points if pt[0] == a.only_n]
        n, A32 = points[0]
        A = torch.from_numpy(A32).to(dev)
        ev = torch.empty((A.shape[0], n), dtype=torch.float32, device=dev)
        V = torch.empty((A.shape[0], n, n), dtype=torch.float32, device=dev)
        torch.cuda.synchronize()
        for _ in range(a.steps):
            binding.bed_syevd(A, ev, V)
        torch.cuda.synchronize()
        print(json.dumps({"only_n": n, "launches": a.steps, "batch": int(A.shape[0])}))
        return 0
    bufs = []
    for n, A32 in points:
        A = torch.from_numpy(A32).to(dev)
        ev = torch.empty((A.shape[0], n), dtype=torch.float32, device=dev)
        V = torch.empty((A.shape[0], n, n), dtype=torch.float32, device=dev)
        bufs.append((n, A, ev, V))
    stream = torch.cuda.current_stream()

    # rotation counts (for the flop model), outside the timed region
    rot_mean = {}
    rot_max = {}
    for n, A, ev, V in bufs:
        _, _, info, rot = binding.bed_syevd_info(A, ev, V)
        torch.cuda.synchronize()
        assert int(info.max().item()) == 0, "non-converged matrix in the benchmark input"
        rot_mean[n] = float(rot.float().mean().item())
        rot_max[n] = int(rot.max().item())      # a batch-uniform window would run every matrix this long

    def step():
        for n, A, ev, V in bufs:
            binding.bed_syevd(A, ev, V)

    for _ in range(a.warmup):
        step()
    torch.cuda.synchronize()

    # ---- timed region: K steps; HIP events (on the launch stream) around the dominant call ----
    dom_i = len(bufs) - 1                      # n = 32
    starts = [torch.cuda.Event(enable_timing=True) for _ in range(a.steps)]
    stops = [torch.cuda.Event(enable_timing=True) for _ in range(a.steps)]
    for e_ in starts + stops:                  # first use creates the HIP event: keep that out of the timing
        e_.record(stream)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(a.steps):
        for i, (n, A, ev, V) in enumerate(bufs):
            if i == dom_i:
                starts[k].record(stream)
                binding.bed_syevd(A, ev, V)
                stops[k].record(stream)
            else:
                binding.bed_syevd(A, ev, V)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    wall = t1 - t0
    n_mats = sum(int(A.shape[0]) for _, A, _, _ in bufs)
    value = n_mats * a.steps / wall
    dom_durs = np.array([starts[k].elapsed_time(stops[k]) for k in range(a.steps)]) * 1e-3  # s

    # ---- per-n figures: a second, untimed pass with events around every call ----
    ev_a = [[torch.cuda.Event(enable_timing=True) for _ in bufs] for _ in range(a.steps)]
    ev_b = [[torch.cuda.Event(enable_timing=True) for _ in bufs] for _ in range(a.steps)]
    for row in ev_a + ev_b:
        for e_ in row:
            e_.record(stream)
    torch.cuda.synchronize()
    step()                                     # keep the queue non-empty: on an idle queue the first start
    step()                                     # event is processed before the host has submitted its kernel
    for k in range(a.steps):
        for i, (n, A, ev, V) in enumerate(bufs):
            ev_a[k][i].record(stream)
            binding.bed_syevd(A, ev, V)
            ev_b[k][i].record(stream)
    torch.cuda.synchronize()
    per_n = {}
    for i, (n, A, ev, V) in enumerate(bufs):
        durs = np.array([ev_a[k][i].elapsed_time(ev_b[k][i]) for k in range(a.steps)]) * 1e-3  # s
        if i == dom_i:
            durs = dom_durs                    # the dominant kernel: measured inside the timed region
        mean = float(durs.mean())
        B = int(A.shape[0])
        fl = B * flops_per_matrix(n, rot_mean[n])
        by = B * bytes_per_matrix(n)
        per_n[str(n)] = {
            "batch": B,
            "kernel_us_mean": mean * 1e6,
            "kernel_us_median": float(np.median(durs)) * 1e6,
            "matrices_per_s": B / mean,
            "rotations_mean": rot_mean[n],
            "rotations_max": rot_max[n],
            "flops_per_launch": fl,
            "tflops": fl / mean / 1e12,
            "frac_fp32_valu": fl / mean / 1e12 / PEAK_FP32_TFLOPS,
            "gbs": by / mean / 1e9,
            "frac_hbm": by / mean / 1e9 / PEAK_HBM_GBS,
        }

    # ---- back-to-back loop per n without events (launch-throughput view) ----
    for i, (n, A, ev, V) in enumerate(bufs):
        torch.cuda.synchronize()
        ta = time.perf_counter()
        for _ in range(a.steps):
            binding.bed_syevd(A, ev, V)
        torch.cuda.synchronize()
        tb = time.perf_counter()
        per_n[str(n)]["matrices_per_s_back_to_back"] = int(A.shape[0]) * a.steps / (tb - ta)

    # ---- extras (outside the timed region; reported, not part of `value`) ----
    def timed(fn, reps):
        fn()
        torch.cuda.synchronize()
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(reps):
            fn()
        e1.record(stream)
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e-3 / reps

    extras = {"eigenvalues_only_us": {}, "spd_inv_sqrt_us": {}, "syevd_backward_taylor9_us": {},
              "spd_inv_sqrt_backward_us": {}, "large_batch": {}}
    reps = max(10, a.steps // 4)
    for n, A, ev, V in ([] if a.no_extras else bufs):
        F = torch.empty_like(V)
        ev2 = torch.empty_like(ev)
        extras["eigenvalues_only_us"][str(n)] = timed(lambda: binding.bed_syevd(A, ev2, None, want_vectors=False), reps) * 1e6
        extras["spd_inv_sqrt_us"][str(n)] = timed(
            lambda: binding.bed_spd_fn(A, binding.BED_FN_INV_SQRT, 1e-6, out=F), reps) * 1e6
        gl = torch.ones_like(ev)
        gV = torch.ones_like(V)
        extras["syevd_backward_taylor9_us"][str(n)] = timed(
            lambda: binding.bed_syevd_backward(ev, V, gl, gV, mode=binding.BED_GRAD_TAYLOR, degree=9, grad_A=F),
            reps) * 1e6
        extras["spd_inv_sqrt_backward_us"][str(n)] = timed(
            lambda: binding.bed_spd_fn_backward(ev, V, gV, binding.BED_FN_INV_SQRT, 1e-6, grad_A=F), reps) * 1e6
    if not a.no_extras:
        # the four calls of a step recorded once into a HIP graph and replayed
        side = torch.cuda.Stream()
        side.wait_stream(stream)
        with torch.cuda.stream(side):
            step()
        stream.wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
        graph.replay()
        torch.cuda.synchronize()
        tg0 = time.perf_counter()
        for _ in range(a.steps):
            graph.replay()
        torch.cuda.synchronize()
        tg = (time.perf_counter() - tg0) / a.steps
        extras["graph_replay"] = {"ms_per_step": tg * 1e3, "matrices_per_s": n_mats / tg}
        # the four sizes on four streams (independent work; each call fills half of the SIMDs)
        streams = [torch.cuda.Stream() for _ in bufs]
        for st_ in streams:
            st_.wait_stream(stream)
        torch.cuda.synchronize()
        tc0 = time.perf_counter()
        for _ in range(a.steps):
            for st_, (n, A, ev, V) in zip(streams, bufs):
                binding.bed_syevd(A, ev, V, stream=st_)
        torch.cuda.synchronize()
        tcs = (time.perf_counter() - tc0) / a.steps
        extras["four_streams"] = {"ms_per_step": tcs * 1e3, "matrices_per_s": n_mats / tcs}
    if not a.no_extras:
        # the mini-batch shapes of the paper's application tables (Tables 2-4), one call each
        extras["paper_shapes_us"] = {}
        for batch, n in ((16, 4), (8, 8), (4, 16), (768, 32), (768, 36), (256, 4), (128, 8), (64, 16)):
            Ap = torch.from_numpy(workloads.covariance(batch, n, 4 * n, 1e-4, 31 + n)).to(dev)
            evp = torch.empty((batch, n), dtype=torch.float32, device=dev)
            Vp = torch.empty((batch, n, n), dtype=torch.float32, device=dev)
            extras["paper_shapes_us"][f"{batch}x{n}x{n}"] = timed(lambda: binding.bed_syevd(Ap, evp, Vp), 20) * 1e6
    if not a.no_extras:
        # the paper's fixed-budget procedure (n iterations, eps 1e-5) on the same inputs: one
        # launch per iteration; what is left of the sub-diagonal says how far from converged it ends
        extras["lockstep"] = {}
        for n, A, ev, V in bufs:
            ws = torch.empty((1 << 20,), dtype=torch.int32, device=dev)
            for name, uniform in (("uniform", True), ("per_matrix", False)):
                t = timed(lambda: binding.bed_syevd_lockstep(A, 1e-5, n, uniform, workspace=ws), 5)
                _, _, off, red = binding.bed_syevd_lockstep(A, 1e-5, n, uniform, workspace=ws)
                extras["lockstep"][f"n{n}_{name}"] = {
                    "us": t * 1e6, "rows_dropped_mean": float(red.float().mean().item()),
                    "offdiag_left_max": float(off.max().item())}
    for n, batch in (() if a.no_extras else ((4, 65536), (8, 65536), (16, 4096), (32, 4096), (64, 256), (128, 256))):
        A32b = (workloads.config2(batch) if n == 4 else
                workloads.config3(n, batch=batch) if n <= 32 else
                workloads.config5(n, batch=batch) if n == 64 else workloads.covariance(batch, n, 4 * n, 1e-4, 1))
        Ab = torch.from_numpy(A32b).to(dev)
        evb = torch.empty((batch, n), dtype=torch.float32, device=dev)
        Vb = torch.empty((batch, n, n), dtype=torch.float32, device=dev)
        t = timed(lambda: binding.bed_syevd(Ab, evb, Vb), 10)
        _, _, _, rotb = binding.bed_syevd_info(Ab, evb, Vb)
        flb = batch * flops_per_matrix(n, float(rotb.float().mean().item()))
        extras["large_batch"][f"n{n}_b{batch}"] = {
            "kernel_us": t * 1e6, "matrices_per_s": batch / t,
            "gbs": batch * bytes_per_matrix(n) / t / 1e9,
            "tflops": flb / t / 1e12, "frac_fp32_valu": flb / t / 1e12 / PEAK_FP32_TFLOPS}
        del Ab, evb, Vb, A32b

    dom = per_n["32"]
    # HBM bytes per launch of the dominant kernel, from the committed rocprofv3 --pmc summary
    # (FETCH_SIZE + WRITE_SIZE scaled by a plain copy of known size); null if it is absent.
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "wave_kernel_n32_b512_counters.md")
    if os.path.exists(tpath):
        import re
        m = re.search(r"^hbm_bytes_per_launch:\s*([0-9.]+)", open(tpath).read(), flags=re.M)
        if m:
            traffic = float(m.group(1))
    roofline = {
        "kernel": "bed::wave_kernel<32> (n=32, batch 512)",
        "bound": "alu",
        "achieved": dom["tflops"],
        "peak": PEAK_FP32_TFLOPS,
        "unit": "TFLOP/s",
        "frac": dom["frac_fp32_valu"],
        "traffic": traffic,
        "hbm_frac": dom["frac_hbm"],
        "launch_us": dom["kernel_us_mean"],
    }

    cpu_baseline = None
    parity = None
    if not a.no_cpu_baseline:
        from oracle import jacobi
        from oracle.acceptance import evaluate
        best = None
        res32 = None
        for rep in range(3):
            tc0 = time.perf_counter()
            used = 0
            for n, A32 in points:
                lam, Vo, _, used = jacobi.syevd(A32, threads=0, return_sweeps=True)
                if n == 32:
                    res32 = (lam, Vo)
            tc1 = time.perf_counter()
            best = (tc1 - tc0) if best is None else min(best, tc1 - tc0)
        # context: the same oracle on one thread, and the host LAPACK (float32 eigh) on the same inputs
        t1a = time.perf_counter()
        for n, A32 in points:
            jacobi.syevd(A32, threads=1)
        t1b = time.perf_counter()
        for n, A32 in points:
            np.linalg.eigh(A32)
        t1c = time.perf_counter()
        cpu_baseline = {
            "single_thread_value": n_mats / (t1b - t1a),
            "lapack_eigh_f32_value": n_mats / (t1c - t1b),
            "value": n_mats / best,
            "unit": "matrices/s",
            "cores": int(used),
            "kind": "oracle",
            "sample": "the full step workload once (4 x 512 matrices, n=4/8/16/32), float64 cyclic Jacobi, "
                      "OpenMP over the batch, best of 3",
        }
        n, A, ev, V = bufs[-1]
        acc = evaluate(points[-1][1], ev.cpu().numpy(), V.cpu().numpy(), res32[0], res32[1])
        parity = {"n32_ok": bool(acc.passes()), **acc.worst()}

    out = {
        "metric": "matrices/sec at batch 512, n=4/8/16/32 fp32; % of fp32 VALU roofline",
        "value": value,
        "unit": "matrices/s",
        "n_gpus": 1,
        "steps": a.steps,
        "warmup": a.warmup,
        "ms_per_step": wall / a.steps * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": "batch 512 x n in {4, 8, 16, 32}: Wishart covariances "
                               "(config 2 at batch 512, config 3 at n = 8, 16, 32); one step = 4 calls = 2048 matrices",
                   "batch": 512, "dims": [4, 8, 16, 32], "eigenvectors": True},
        "per_n": per_n,
        "extras": None if a.no_extras else extras,
        "roofline": roofline,
        "cpu_baseline": cpu_baseline,
        "parity": parity,
    }
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
