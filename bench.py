#!/usr/bin/env python3
"""Benchmark of the batched symmetric eigensolver on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

One *step* is one pass of the whole hot path over the headline workload:
four `bed_syevd` calls, batch 512 each, n = 4, 8, 16, 32 (2048 matrices),
inputs already resident in HBM.  The script prints ONE JSON line:

  value        matrices/s over the K timed steps (wall clock, synchronised)
  per_n        per-call figures for each n (every kernel launched with a start and a stop
               HIP event of its own on the launch stream; the dominant call, n = 32, is
               measured inside the timed region, the others in a second pass)
  roofline     the dominant kernel (n = 32): algorithmic flops / mean launch
               duration against the fp32 vector peak (datasheet, packed), the plain-FMA
               peak, and ceilings measured in this run (plain-FMA kernel, device copy)
  ceilings     those measured ceilings; environment: clocks, ROCm version, device
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
PEAK_FP32_PLAIN_FMA_TFLOPS = 78.6   # the same without packed instructions (v_fma_f32): what this build can reach
PEAK_HBM_GBS = 8000.0


def measure_ceilings(binding, torch, dev, stream):
    """Rates this build reaches on this machine (HIP events on the launch stream, best of 5 launches):
    plain-FMA throughput with the chip full, the FMA rate of 512 single-wavefront workgroups that
    each run ONE dependent chain (the launch shape of the batch-512 calls), and a device copy."""
    def best(fn, reps=5):
        fn()
        torch.cuda.synchronize()
        ts = []
        for _ in range(reps):
            e0 = torch.cuda.Event(enable_timing=True)
            e1 = torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            fn()
            e1.record(stream)
            torch.cuda.synchronize()
            ts.append(e0.elapsed_time(e1) * 1e-3)
        return min(ts)

    out = {}
    blocks, threads, iters = 256 * 16, 256, 4096          # 16 wavefronts per SIMD
    buf = torch.empty((blocks * threads,), dtype=torch.float32, device=dev)
    fl = 2.0 * blocks * threads * 16 * iters
    t = best(lambda: binding.bed_ceiling_fma(buf, blocks, threads, 16, iters))
    out["plain_fma_tflops"] = fl / t / 1e12
    out["plain_fma_command"] = f"bed_ceiling_fma(blocks={blocks}, threads={threads}, chains=16, iters={iters})"
    blocks1, iters1 = 512, 1 << 16                          # one wavefront on every second SIMD, one chain each
    buf1 = torch.empty((blocks1 * 64,), dtype=torch.float32, device=dev)
    t1 = best(lambda: binding.bed_ceiling_fma(buf1, blocks1, 64, 1, iters1))
    out["dependent_chain_512_waves_tflops"] = 2.0 * blocks1 * 64 * iters1 / t1 / 1e12
    out["dependent_chain_ns_per_instruction"] = t1 / iters1 * 1e9
    out["dependent_chain_command"] = f"bed_ceiling_fma(blocks={blocks1}, threads=64, chains=1, iters={iters1})"
    nfl = (256 << 20) // 4                                  # 256 MiB each way
    src = torch.empty((nfl,), dtype=torch.float32, device=dev).normal_()
    dst = torch.empty_like(src)
    tc = best(lambda: binding.bed_ceiling_copy(src, dst, 256 * 32))
    out["copy_gbs"] = 8.0 * nfl / tc / 1e9
    out["copy_command"] = f"bed_ceiling_copy(count={nfl}, blocks={256 * 32})  # 256 MiB read + 256 MiB written"
    del src, dst, buf, buf1
    return out


def environment(torch):
    """Clocks, ROCm version and device as far as an ordinary user can read them."""
    import subprocess
    env = {"torch": torch.__version__, "hip": getattr(torch.version, "hip", None)}
    try:
        env["rocm_version"] = open("/opt/rocm/.info/version").read().strip()
    except OSError:
        env["rocm_version"] = None
    pr = torch.cuda.get_device_properties(0)
    env["device"] = pr.name
    env["gcn_arch"] = getattr(pr, "gcnArchName", None)
    env["compute_units"] = pr.multi_processor_count
    env["max_engine_clock_mhz"] = getattr(pr, "clock_rate", 0) / 1000.0 or None
    env["max_memory_clock_mhz"] = getattr(pr, "memory_clock_rate", 0) / 1000.0 or None
    try:
        r = subprocess.run(["rocm-smi", "--showclocks", "--json"], capture_output=True, text=True, timeout=20)
        env["rocm_smi_clocks"] = json.loads(r.stdout) if r.returncode == 0 and r.stdout.strip() else None
    except Exception:
        env["rocm_smi_clocks"] = None
    return env


def traffic_from_profile():
    """HBM bytes per launch of the dominant kernel from the committed rocprofv3 --pmc summary, but
    only if that summary was taken from exactly the sources this library is built from (it
    records their hash); otherwise None: a counter reading of another kernel is not this one's."""
    import re
    from paper_2207_04228_amd import build
    tpath = os.path.join(ROOT, "profiles", "wave_kernel_n32_b512_counters.md")
    if not os.path.exists(tpath):
        return None, None
    text = open(tpath).read()
    m = re.search(r"^hbm_bytes_per_launch:\s*([0-9.]+)", text, flags=re.M)
    h = re.search(r"^source_hash:\s*([0-9a-f]+)", text, flags=re.M)
    if not m or not h or h.group(1) != build.source_hash():
        return None, "profiles/wave_kernel_n32_b512_counters.md was taken from other sources than this build"
    return float(m.group(1)), "profiles/wave_kernel_n32_b512_counters.md (same source hash as this build)"


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
    ap.add_argument("--only-batch", type=int, default=512,
                    help="with --only-n: the batch size (512: the headline input of that n; 4096 with n = 16: config 4; "
                         "otherwise config 2 / config 3 inputs, tiled beyond 65536)")
    ap.add_argument("--ceilings-only", action="store_true",
                    help="profiling aid: run only the measured-ceiling kernels (plain FMA, dependent chain, copy) and exit")
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

    if a.ceilings_only:
        print(json.dumps(measure_ceilings(binding, torch, dev, torch.cuda.current_stream())))
        return 0

    points = workloads.headline_points()          # [(n, A32)], batch 512 each
    if a.only_n:
        n = a.only_n
        if a.only_batch == 512:
            A32 = dict(points)[n]
        else:
            base = min(a.only_batch, 65536)
            A32 = (workloads.config2(base) if n == 4 else workloads.config4(batch=base) if n == 16 else
                   workloads.config3(n, batch=base))
        A = torch.from_numpy(A32).to(dev)
        if a.only_batch > A.shape[0]:
            A = A.repeat(a.only_batch // A.shape[0], 1, 1).contiguous()
        ev = torch.empty((A.shape[0], n), dtype=torch.float32, device=dev)
        V = torch.empty((A.shape[0], n, n), dtype=torch.float32, device=dev)
        torch.cuda.synchronize()
        for _ in range(a.steps):
            binding.bed_syevd(A, ev, V)
        torch.cuda.synchronize()
        print(json.dumps({"only_n": n, "launches": a.steps, "batch": int(A.shape[0]),
                          "kernel": binding.bed_kernel_variant(int(A.shape[0]), n)}))
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

    # ---- timed region: K steps; the dominant call (n = 32) is launched with a start and a stop
    # event of its own (bed_timing_*: the dispatch's begin and end timestamps on the launch
    # stream, no marker packets between the kernels) ----
    dom_i = len(bufs) - 1                      # n = 32
    binding.bed_timing_begin(a.steps)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(a.steps):
        for i, (n, A, ev, V) in enumerate(bufs):
            if i == dom_i:
                binding.bed_timing_arm(True)
                binding.bed_syevd(A, ev, V)
                binding.bed_timing_arm(False)
            else:
                binding.bed_syevd(A, ev, V)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    wall = t1 - t0
    n_mats = sum(int(A.shape[0]) for _, A, _, _ in bufs)
    value = n_mats * a.steps / wall
    dom_us, timed = binding.bed_timing_end(a.steps)
    assert timed == a.steps, (timed, a.steps)
    dom_durs = dom_us.astype(np.float64) * 1e-6   # s

    # ---- per-n figures: a second, untimed pass with every call timed the same way ----
    binding.bed_timing_begin(a.steps * len(bufs))
    binding.bed_timing_arm(True)
    for k in range(a.steps):
        step()
    torch.cuda.synchronize()
    all_us, timed = binding.bed_timing_end(a.steps * len(bufs))
    assert timed == a.steps * len(bufs), timed
    all_durs = all_us.astype(np.float64).reshape(a.steps, len(bufs)) * 1e-6
    per_n = {}
    for i, (n, A, ev, V) in enumerate(bufs):
        durs = all_durs[:, i]
        if i == dom_i:
            durs = dom_durs                    # the dominant kernel: measured inside the timed region
        mean = float(durs.mean())
        B = int(A.shape[0])
        fl = B * flops_per_matrix(n, rot_mean[n])
        by = B * bytes_per_matrix(n)
        per_n[str(n)] = {
            "batch": B,
            "kernel": binding.bed_kernel_variant(B, n),
            "kernel_us_mean": mean * 1e6,
            "kernel_us_median": float(np.median(durs)) * 1e6,
            "kernel_us_p10": float(np.percentile(durs, 10)) * 1e6,
            "kernel_us_p90": float(np.percentile(durs, 90)) * 1e6,
            "matrices_per_s": B / mean,
            "rotations_mean": rot_mean[n],
            "rotations_max": rot_max[n],
            "flops_per_launch": fl,
            "tflops": fl / mean / 1e12,
            "frac_fp32_valu": fl / mean / 1e12 / PEAK_FP32_TFLOPS,
            "frac_plain_fma": fl / mean / 1e12 / PEAK_FP32_PLAIN_FMA_TFLOPS,
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
        """Seconds per call: best of three event-bracketed loops of `reps` calls (the first loop
        after host-side work runs while the clocks are still ramping up, up to 15 % slow)."""
        fn()
        torch.cuda.synchronize()
        best = float("inf")
        for _ in range(3):
            e0 = torch.cuda.Event(enable_timing=True)
            e1 = torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            for _ in range(reps):
                fn()
            e1.record(stream)
            torch.cuda.synchronize()
            best = min(best, e0.elapsed_time(e1) * 1e-3 / reps)
        return best

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
    # Saturated batches.  n = 16 at batch 4096 is config 4 (Haar Q, lambda_i = i^-2); the sweeps of
    # n = 4 and n = 8 go up to 2^20 matrices (config 2 / config 3 inputs, tiled beyond 65536) so that
    # the rate with every SIMD holding several wavefronts is on record.
    big = ((4, 4096), (4, 65536), (4, 1 << 18), (4, 1 << 20), (8, 4096), (8, 65536), (8, 1 << 18), (8, 1 << 20),
           (16, 4096), (16, 65536), (32, 4096), (32, 16384), (48, 256), (64, 256), (128, 256))
    for n, batch in (() if a.no_extras else big):
        base = min(batch, 65536)
        A32b = (workloads.config2(base) if n == 4 else
                workloads.config4(batch=base) if n == 16 else
                workloads.config3(n, batch=base) if n <= 32 else
                workloads.config5(n, batch=base) if n in (48, 64) else workloads.covariance(base, n, 4 * n, 1e-4, 1))
        Ab = torch.from_numpy(A32b).to(dev)
        if batch > base:
            Ab = Ab.repeat(batch // base, 1, 1).contiguous()
        evb = torch.empty((batch, n), dtype=torch.float32, device=dev)
        Vb = torch.empty((batch, n, n), dtype=torch.float32, device=dev)
        t = timed(lambda: binding.bed_syevd(Ab, evb, Vb), 10)
        t_ev = timed(lambda: binding.bed_syevd(Ab, evb, None, want_vectors=False), 10)
        t_fn = timed(lambda: binding.bed_spd_fn(Ab, binding.BED_FN_INV_SQRT, 1e-6, out=Vb), 10)
        _, _, _, rotb = binding.bed_syevd_info(Ab, evb, Vb)
        flb = batch * flops_per_matrix(n, float(rotb.float().mean().item()))
        extras["large_batch"][f"n{n}_b{batch}"] = {
            "kernel": binding.bed_kernel_variant(batch, n),
            "kernel_us": t * 1e6, "matrices_per_s": batch / t,
            "eigenvalues_only_us": t_ev * 1e6,
            "spd_inv_sqrt_us": t_fn * 1e6,
            "gbs": batch * bytes_per_matrix(n) / t / 1e9,
            "frac_hbm": batch * bytes_per_matrix(n) / t / 1e9 / PEAK_HBM_GBS,
            "tflops": flb / t / 1e12, "frac_fp32_valu": flb / t / 1e12 / PEAK_FP32_TFLOPS}
        del Ab, evb, Vb, A32b

    dom = per_n["32"]
    ceilings = measure_ceilings(binding, torch, dev, stream)
    traffic, traffic_source = traffic_from_profile()
    roofline = {
        "kernel": "bed::wave_kernel<32, true, 0> (n=32, batch 512)",
        "bound": "alu",
        "achieved": dom["tflops"],
        "peak": PEAK_FP32_TFLOPS,
        "unit": "TFLOP/s",
        "frac": dom["frac_fp32_valu"],
        "peak_plain_fma": PEAK_FP32_PLAIN_FMA_TFLOPS,
        "frac_vs_plain_fma": dom["tflops"] / PEAK_FP32_PLAIN_FMA_TFLOPS,
        "peak_measured": ceilings["plain_fma_tflops"],
        "frac_vs_measured": dom["tflops"] / ceilings["plain_fma_tflops"],
        "launch_shape_ceiling": ceilings["dependent_chain_512_waves_tflops"],
        "frac_vs_launch_shape_ceiling": dom["tflops"] / ceilings["dependent_chain_512_waves_tflops"],
        "traffic": traffic,
        "traffic_source": traffic_source,
        "hbm_frac": dom["frac_hbm"],
        "hbm_peak_measured_gbs": ceilings["copy_gbs"],
        "hbm_frac_vs_measured": dom["gbs"] / ceilings["copy_gbs"],
        "launch_us": dom["kernel_us_mean"],
        "launch_us_p10": dom["kernel_us_p10"],
        "launch_us_p90": dom["kernel_us_p90"],
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
        "ceilings": ceilings,
        "environment": environment(torch),
        "cpu_baseline": cpu_baseline,
        "parity": parity,
    }
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
