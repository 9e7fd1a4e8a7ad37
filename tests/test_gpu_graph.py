"""The entry points enqueue one kernel and nothing else (no allocation, no memset, no
synchronisation), so a caller can record them into a HIP graph.  A graph holding the four
calls of the headline step, a spectral-function call and a gradient call is replayed
several times, with eager work and synchronisations between the replays, and every replay
is compared with the eager results."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def test_graph_replays_match_eager_results():
    import torch
    from paper_2207_04228_amd import binding, workloads
    dev = torch.device("cuda:0")
    pts = [(n, torch.from_numpy(A).to(dev)) for n, A in workloads.headline_points()]
    eager = []
    for n, A in pts:
        ev, V = binding.bed_syevd(A)
        eager.append((ev.clone(), V.clone()))
    n32, A32 = pts[-1]
    F_eager, _, _ = binding.bed_spd_fn(A32, binding.BED_FN_INV_SQRT, 1e-6)
    G = torch.randn_like(A32)
    gA_eager = binding.bed_spd_fn_backward(eager[-1][0], eager[-1][1], G, binding.BED_FN_INV_SQRT, 1e-6)
    torch.cuda.synchronize()

    outs = [(torch.empty_like(ev), torch.empty_like(V)) for ev, V in eager]
    F = torch.empty_like(A32)
    info = torch.empty((A32.shape[0],), dtype=torch.int32, device=dev)
    gA = torch.empty_like(A32)
    lib = binding.load_library()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                     # warm-up on the capture stream's side
        for (n, A), (ev, V) in zip(pts, outs):
            binding.bed_syevd(A, ev, V)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        for (n, A), (ev, V) in zip(pts, outs):
            binding.bed_syevd(A, ev, V)
        st = lib.bed_spd_fn(binding._ptr(A32), A32.shape[0], n32, binding.BED_FN_INV_SQRT, 1e-6,
                            binding._ptr(F), None, binding._ptr(info), binding._stream(None))
        assert st == 0
        binding.bed_spd_fn_backward(outs[-1][0], outs[-1][1], G, binding.BED_FN_INV_SQRT, 1e-6, grad_A=gA)
    for replay in range(4):
        for ev, V in outs:
            ev.zero_()
            V.zero_()
        F.zero_()
        gA.zero_()
        scratch = torch.randn(1 << 16, device=dev).sum()      # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for (ev, V), (ev0, V0) in zip(outs, eager):
            assert torch.equal(ev, ev0) and torch.equal(V, V0), f"replay {replay}"
        assert torch.equal(F, F_eager), f"replay {replay}"
        assert torch.equal(gA, gA_eager), f"replay {replay}"
        assert int(info.max()) == 0 and np.isfinite(float(scratch))
