"""Every kernel family against the oracle at batch sizes on both sides of the automatic dispatch
(bed_syevd_family), ragged last wavefronts included, with and without eigenvectors."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def _solve(A32, family, want_vectors=True):
    import torch
    from paper_2207_04228_amd import binding
    At = torch.from_numpy(np.ascontiguousarray(A32)).to("cuda:0")
    ev, V, info, rot = binding.bed_syevd_info(At, want_vectors=want_vectors, family=family)
    torch.cuda.synchronize()
    return (ev.cpu().numpy(), None if V is None else V.cpu().numpy(), info.cpu().numpy(),
            rot.cpu().numpy().astype(np.int64))


def _check(A32, family, name, allow_fallback=False):
    from oracle import jacobi
    from oracle.acceptance import evaluate
    print(f"[family] {name} shape={A32.shape}", flush=True)
    lam_o, V_o = jacobi.syevd(A32)
    lam_g, V_g, info, rot = _solve(A32, family)
    assert np.isfinite(lam_g).all() and np.isfinite(V_g).all()
    assert np.all(np.diff(lam_g, axis=1) >= 0)
    assert np.all((info & 0xFFFF) == 0)
    if not allow_fallback:
        assert np.all(info == 0)
    acc = evaluate(A32, lam_g, V_g, lam_o, V_o)
    w = acc.worst()
    print(f"[family] {name}: eval {w['eval_err']:.2e} res {w['residual']:.2e} orth {w['orth']:.2e} "
          f"angle {w['angle']:.2e} rot mean {rot.mean():.1f}", flush=True)
    assert acc.passes(), w
    lam_e, V_e, info_e, rot_e = _solve(A32, family, want_vectors=False)
    assert V_e is None and np.all(info_e == info)
    norm2 = np.maximum(np.abs(lam_o).max(axis=1, keepdims=True), 1e-300)
    assert (np.abs(lam_e - lam_o) / norm2).max() <= 1e-5
    return lam_g, V_g, rot


PACKED = 2
LANE = 3
WAVE = 1
PACKED_ROWS = 6


@pytest.mark.parametrize("n", list(range(1, 33)))
def test_packed_kernel_every_n(n):
    """Four (n <= 16) or two (n <= 32) matrices per wavefront, every n it serves; batches that
    leave groups of the last wavefront empty; indefinite input."""
    rng = np.random.default_rng(8100 + n)
    for batch in (1, 2, 3, 4, 37, 258):
        A = rng.standard_normal((batch, n, n))
        A = (0.5 * (A + A.transpose(0, 2, 1))).astype(np.float32)
        _check(A, PACKED, f"packed_n{n}_b{batch}")


def test_packed_kernel_on_the_configs():
    from paper_2207_04228_amd import workloads
    _check(workloads.config1(), PACKED, "packed_config1")
    _check(workloads.config2(4096), PACKED, "packed_config2_b4096")
    _check(workloads.config3(8), PACKED, "packed_config3_n8")
    _check(workloads.config3(16), PACKED, "packed_config3_n16")
    _check(workloads.config4(), PACKED, "packed_config4")
    _check(workloads.config3(24), PACKED, "packed_config3_n24")
    _check(workloads.config3(32), PACKED, "packed_config3_n32")
    _check(workloads.config3(32, batch=4099), PACKED, "packed_n32_b4099")


def test_packed_kernel_mixed_convergence_in_one_wavefront():
    """Rows of one wavefront that finish at very different times: a diagonal matrix, a zero matrix,
    the identity, a dense one and matrices with repeated eigenvalues side by side."""
    from paper_2207_04228_amd import workloads
    n = 12
    rng = np.random.default_rng(8200)
    dense = rng.standard_normal((8, n, n))
    dense = 0.5 * (dense + dense.transpose(0, 2, 1))
    rep = workloads.from_spectrum(np.round(rng.uniform(0, 2, (8, n))), seed=5).astype(np.float64)
    mats = [np.diag(np.arange(n, 0, -1.0)), np.zeros((n, n)), np.eye(n), dense[0], rep[0], dense[1], np.eye(n) * -3,
            rep[1], 2.0 * np.eye(n) - np.eye(n, k=1) - np.eye(n, k=-1), dense[2], rep[2], np.zeros((n, n)), dense[3]]
    A = np.stack(mats).astype(np.float32)
    lam, V, rot = _check(A, PACKED, "packed_mixed")
    assert np.array_equal(lam[0], np.arange(1, n + 1, dtype=np.float32))
    assert np.array_equal(lam[1], np.zeros(n, dtype=np.float32))
    assert np.array_equal(lam[2], np.ones(n, dtype=np.float32))
    assert rot[1] == 0 and rot[2] == 0


def test_packed_kernel_nan_is_confined_to_its_row():
    from paper_2207_04228_amd import workloads
    A = workloads.config3(16, batch=10).copy()
    A[5, 3, 1] = np.nan
    A[6, 0, 0] = np.inf
    lam, V, info, rot = _solve(A, PACKED)
    good = [0, 1, 2, 3, 4, 7, 8, 9]
    assert np.isfinite(lam[good]).all() and np.isfinite(V[good]).all() and np.all(info[good] == 0)
    assert info[5] > 0 and info[6] > 0 and not np.isfinite(lam[5]).all()


def test_packed_kernel_structured_and_repeated():
    from paper_2207_04228_amd import workloads
    for n in (5, 8, 13, 16, 21, 32):
        for name, A in workloads.structured_cases(n, 16, seed=900 + n):
            _check(A, PACKED, f"packed_structured_n{n}_{name}", allow_fallback=True)
        rng = np.random.default_rng(8300 + n)
        for kind, lam in enumerate((np.round(rng.uniform(0, 3, (48, n))),
                                    np.where(rng.uniform(0, 1, (48, n)) < 0.5, 1.0, 1.0 + 1e-6))):
            _check(workloads.from_spectrum(lam, seed=kind + n), PACKED, f"packed_repeated_n{n}_{kind}")


@pytest.mark.parametrize("n", list(range(1, 33)))
def test_packed_rows_kernel_every_n(n):
    """Four matrices per wavefront with two rows per lane, every n it accepts (it is dispatched for
    16 < n <= 32); batches that leave groups of the last wavefront empty; indefinite input."""
    rng = np.random.default_rng(8600 + n)
    for batch in (1, 2, 3, 4, 5, 37, 258):
        A = rng.standard_normal((batch, n, n))
        A = (0.5 * (A + A.transpose(0, 2, 1))).astype(np.float32)
        _check(A, PACKED_ROWS, f"packed_rows_n{n}_b{batch}")


def test_packed_rows_kernel_on_the_configs_and_where_it_is_dispatched():
    from paper_2207_04228_amd import binding, workloads
    _check(workloads.config3(24), PACKED_ROWS, "packed_rows_config3_n24")
    _check(workloads.config3(32), PACKED_ROWS, "packed_rows_config3_n32")
    for n in (20, 24, 28, 32):
        assert binding.bed_kernel_variant(4096, n) == f"packed_rows_kernel<{n}>"
        assert binding.bed_kernel_variant(4096, n, False) == f"packed_rows_kernel<{n}>"
        assert binding.bed_kernel_variant(4095, n) == f"wave_kernel<{n}>"
        assert binding.bed_kernel_variant(3072, n, False) == f"packed_rows_kernel<{n}>"
        assert binding.bed_kernel_variant(3071, n, False) == f"wave_kernel<{n}>"
    assert binding.bed_kernel_variant(4096, 17) == "packed_rows_kernel<20>"
    assert binding.bed_kernel_variant(4096, 16) == "packed_kernel<16>"
    # through the automatic dispatch, ragged last wavefront
    A = workloads.config3(32, batch=4099)
    _check(A, 0, "auto_n32_b4099")
    _check(workloads.config3(21, batch=4097), 0, "auto_n21_b4097")


def test_packed_rows_kernel_mixed_convergence_nan_and_structure():
    from paper_2207_04228_amd import workloads
    n = 28
    rng = np.random.default_rng(8700)
    dense = rng.standard_normal((8, n, n))
    dense = 0.5 * (dense + dense.transpose(0, 2, 1))
    rep = workloads.from_spectrum(np.round(rng.uniform(0, 2, (8, n))), seed=6).astype(np.float64)
    mats = [np.diag(np.arange(n, 0, -1.0)), np.zeros((n, n)), np.eye(n), dense[0], rep[0], dense[1], np.eye(n) * -3,
            rep[1], 2.0 * np.eye(n) - np.eye(n, k=1) - np.eye(n, k=-1), dense[2], rep[2], np.zeros((n, n)), dense[3]]
    A = np.stack(mats).astype(np.float32)
    lam, V, rot = _check(A, PACKED_ROWS, "packed_rows_mixed")
    assert np.array_equal(lam[0], np.arange(1, n + 1, dtype=np.float32))
    assert np.array_equal(lam[1], np.zeros(n, dtype=np.float32))
    assert np.array_equal(lam[2], np.ones(n, dtype=np.float32))
    assert rot[1] == 0 and rot[2] == 0
    B = workloads.config3(24, batch=10).copy()
    B[5, 20, 1] = np.nan
    B[6, 0, 0] = np.inf
    lam, V, info, rot = _solve(B, PACKED_ROWS)
    good = [0, 1, 2, 3, 4, 7, 8, 9]
    assert np.isfinite(lam[good]).all() and np.isfinite(V[good]).all() and np.all(info[good] == 0)
    assert info[5] > 0 and info[6] > 0 and not np.isfinite(lam[5]).all()
    for m in (21, 32):
        for name, S in workloads.structured_cases(m, 16, seed=950 + m):
            _check(S, PACKED_ROWS, f"packed_rows_structured_n{m}_{name}", allow_fallback=True)
        r2 = np.random.default_rng(8800 + m)
        for kind, sp in enumerate((np.round(r2.uniform(0, 3, (48, m))),
                                   np.where(r2.uniform(0, 1, (48, m)) < 0.5, 1.0, 1.0 + 1e-6))):
            _check(workloads.from_spectrum(sp, seed=kind + m), PACKED_ROWS, f"packed_rows_repeated_n{m}_{kind}")


@pytest.mark.parametrize("n,batch", [(4, 64), (4, 1000), (8, 130), (6, 513)])
def test_lane_kernel_at_small_batches(n, batch):
    rng = np.random.default_rng(8400 + n)
    A = rng.standard_normal((batch, n, n))
    A = (0.5 * (A + A.transpose(0, 2, 1))).astype(np.float32)
    _check(A, LANE, f"lane_n{n}_b{batch}")


@pytest.mark.parametrize("n,batch", [(4, 8192), (8, 16384), (16, 4096)])
def test_wave_kernel_at_large_batches(n, batch):
    from paper_2207_04228_amd import workloads
    A = workloads.config2(batch) if n == 4 else (workloads.config3(8, batch=batch) if n == 8 else workloads.config4())
    _check(A, WAVE, f"wave_n{n}_b{batch}")


def test_family_argument_checks():
    import torch
    from paper_2207_04228_amd import binding
    A = torch.zeros((4, 33, 33), dtype=torch.float32, device="cuda:0")
    for fam in (PACKED, LANE, 4, PACKED_ROWS):
        with pytest.raises(binding.BedError) as e:
            binding.bed_syevd_info(A, family=fam)
        assert e.value.status == -3
    with pytest.raises(binding.BedError) as e:
        binding.bed_syevd_info(A, family=9)
    assert e.value.status == -7


PAIR = 5


@pytest.mark.parametrize("n", [33, 36, 40, 41, 47, 48, 49, 56, 57, 63, 64])
def test_pair_kernel_every_size_class(n):
    """Two wavefronts per matrix (32 < n <= 64): odd and even batch sizes (a workgroup holds two
    matrices), indefinite input."""
    rng = np.random.default_rng(8500 + n)
    for batch in (1, 2, 5, 64):
        A = rng.standard_normal((batch, n, n))
        A = (0.5 * (A + A.transpose(0, 2, 1))).astype(np.float32)
        print(f"[family] pair n={n} batch={batch}", flush=True)
        from oracle import jacobi
        from oracle.acceptance import evaluate
        lam_o, V_o = jacobi.syevd(A)
        lam_g, V_g, info, rot = _solve(A, PAIR)
        assert np.all(info == 0)
        assert evaluate(A, lam_g, V_g, lam_o, V_o).passes()
        lam_w, V_w, info_w, rot_w = _solve(A, WAVE)
        assert np.array_equal(rot, rot_w)            # same shifts, same deflation decisions


def test_pair_kernel_on_config5_and_structured_input():
    from oracle import jacobi
    from oracle.acceptance import evaluate
    from paper_2207_04228_amd import binding, workloads
    for n in (48, 64):
        A = workloads.config5(n)
        assert binding.bed_kernel_variant(A.shape[0], n) == f"pair_kernel<{n}>"
        lam_o, V_o = jacobi.syevd(A)
        lam_g, V_g, info, rot = _solve(A, 0)
        acc = evaluate(A, lam_g, V_g, lam_o, V_o)
        print(f"[family] pair config5 n={n}: {acc.worst()}", flush=True)
        assert np.all(info == 0) and acc.passes()
    for n in (33, 47, 64):
        for name, A in workloads.structured_cases(n, 7, seed=900 + n):
            lam_o, V_o = jacobi.syevd(A)
            lam_g, V_g, info, rot = _solve(A, PAIR)
            assert np.all((info & 0xFFFF) == 0), (n, name)
            assert evaluate(A, lam_g, V_g, lam_o, V_o).passes(), (n, name)


def test_pair_kernel_nan_and_argument_checks():
    import torch
    from paper_2207_04228_amd import binding, workloads
    A = workloads.config5(48, batch=5).copy()
    A[2, 7, 3] = np.nan
    lam, V, info, rot = _solve(A, PAIR)
    good = [0, 1, 3, 4]
    assert np.isfinite(lam[good]).all() and np.isfinite(V[good]).all() and np.all(info[good] == 0)
    assert info[2] > 0 and not np.isfinite(lam[2]).all()
    At = torch.from_numpy(A).to("cuda:0")
    with pytest.raises(binding.BedError) as e:
        binding.bed_syevd_info(At, want_vectors=False, family=PAIR)      # the pair kernels always form eigenvectors
    assert e.value.status == -1
    with pytest.raises(binding.BedError) as e:
        binding.bed_syevd_info(At[:, :32, :32].contiguous(), family=PAIR)
    assert e.value.status == -3
