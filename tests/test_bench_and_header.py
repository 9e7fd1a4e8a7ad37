"""Host-side checks of the benchmark's contract and of the public header (no GPU needed)."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_work_model_matches_its_definition():
    """bytes = 8 n^2 + 4 n (A read once, V and lambda written once); flops = (8/3) n^3 + R (6 n + 20)."""
    sys.path.insert(0, ROOT)
    import bench
    for n, bytes_expected in ((4, 144), (8, 544), (16, 2112), (24, 4704), (32, 8320), (48, 18624), (64, 33024)):
        assert bench.bytes_per_matrix(n) == bytes_expected
        R = n * n
        assert abs(bench.flops_per_matrix(n, R) - ((8.0 / 3.0) * n ** 3 + R * (6 * n + 20))) < 1e-6
        # eigenvalues only: no P, no rotation of V
        assert abs(bench.flops_per_matrix(n, R, vectors=False) - ((4.0 / 3.0) * n ** 3 + 20 * R)) < 1e-6
    assert abs(bench.flops_per_matrix(32, 32 * 32) - 304e3) < 2e3        # the nominal 304 k flops of a 32 x 32 matrix
    assert bench.PEAK_FP32_TFLOPS == 157.3 and bench.PEAK_HBM_GBS == 8000.0
    assert bench.PEAK_FP32_PLAIN_FMA_TFLOPS == 78.6      # v_fma_f32 only: what a build without packed fp32 can reach


def test_traffic_is_reported_only_for_the_profiled_sources(tmp_path, monkeypatch):
    """roofline.traffic comes from the committed counter summary only while that summary's
    source hash equals the hash of the sources the library is built from."""
    sys.path.insert(0, ROOT)
    import bench
    from paper_2207_04228_amd import build
    prof = tmp_path / "profiles"
    prof.mkdir()
    f = prof / "wave_kernel_n32_b512_counters.md"
    monkeypatch.setattr(bench, "ROOT", str(tmp_path))
    f.write_text(f"source_hash: {build.source_hash()}\nhbm_bytes_per_launch: 4879718\n")
    assert bench.traffic_from_profile()[0] == 4879718.0
    f.write_text("source_hash: 0123456789abcdef\nhbm_bytes_per_launch: 4879718\n")
    assert bench.traffic_from_profile()[0] is None
    f.write_text("hbm_bytes_per_launch: 4879718\n")
    assert bench.traffic_from_profile()[0] is None


def test_public_header_is_plain_c(tmp_path):
    src = tmp_path / "use_bed.c"
    src.write_text('#include "bed.h"\n'
                   "int use(const float* A, float* w, float* V) {\n"
                   "    int a = bed_syevd(A, 1, 4, w, V, (void*)0);\n"
                   "    int b = bed_spd_fn(A, 1, 4, BED_FN_INV_SQRT, 1e-6f, V, w, (int*)0, (void*)0);\n"
                   "    int c = bed_syevd_backward(w, V, w, V, 1, 4, BED_GRAD_TAYLOR, 9, 0.f, V, (void*)0);\n"
                   "    return a + b + c + BED_MAX_N + bed_version();\n"
                   "}\n")
    r = subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-pedantic", "-fsyntax-only",
                        "-I", os.path.join(ROOT, "include"), str(src)], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
