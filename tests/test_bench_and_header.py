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
