"""gemm_f16f32_noalloc (the entry point for callers that cannot allocate: K-slice partials in
a fixed per-GPU array) against gemm_f16f32, through the C ABI, bit for bit: two calls in a row,
the second on a smaller input, so that what the first left in the array must not leak into
the second; then the refusal of a forced configuration that needs more than the array holds."""
import numpy as np
import pytest

import gemm_inputs as gi

pytestmark = pytest.mark.gpu


def test_noalloc_matches_the_allocating_entry_point_twice_in_a_row():
    import torch
    import paper_2003_06324_amd as g
    stream = torch.cuda.current_stream().cuda_stream
    # (shape, forced configuration): automatic selection on a deep-K shape (K-sliced), then a
    # smaller product with forced slices, then an unsliced one (needs no scratch at all)
    cases = [((1024, 768, 16384), None), ((192, 160, 1536), "t64x64:s8"), ((300, 260, 200), None)]
    for dist in ("normal", "int"):
        for (M, N, K), force in cases:
            A, B = gi.make_problem(1200 + M, M, N, K, dist, "f16")
            dA = torch.from_numpy(gi.store(A, gi.COL_MAJOR).view(np.int16)).cuda()
            dB = torch.from_numpy(gi.store(B, gi.ROW_MAJOR).view(np.int16)).cuda()
            want = torch.full((M * N,), float("nan"), dtype=torch.float32, device="cuda")
            got = torch.full((M * N,), float("nan"), dtype=torch.float32, device="cuda")
            g.force_config(force)
            try:
                g.gemm_f16f32(M, N, K, dA, gi.COL_MAJOR, 0, dB, gi.ROW_MAJOR, 0, want, gi.ROW_MAJOR, 0, stream)
                cfg_want = g.last_config()
                g.gemm_f16f32_noalloc(M, N, K, dA, gi.COL_MAJOR, 0, dB, gi.ROW_MAJOR, 0, got, gi.ROW_MAJOR, 0, stream)
                cfg_got = g.last_config()
            finally:
                g.force_config(None)
            torch.cuda.synchronize()
            assert cfg_got.replace(" static-scratch", "") == cfg_want, (cfg_got, cfg_want)
            if (M, N, K) != (300, 260, 200):
                assert "static-scratch" in cfg_got and " s1" not in cfg_got, cfg_got
            w, c = want.cpu().numpy(), got.cpu().numpy()
            assert np.all(np.isfinite(c))
            assert np.array_equal(w.view(np.uint32), c.view(np.uint32)), ((M, N, K), dist, cfg_got)


def test_noalloc_refuses_what_does_not_fit_and_never_picks_it():
    import torch
    import paper_2003_06324_amd as g
    stream = torch.cuda.current_stream().cuda_stream
    M, N, K = 2048, 2304, 2048           # 32 slices of partials = 604 MB, beyond the 64 MiB array
    assert 32 * M * N * 4 > g.NOALLOC_SCRATCH_BYTES
    dA = torch.zeros(M * K, dtype=torch.int16, device="cuda")
    dB = torch.zeros(K * N, dtype=torch.int16, device="cuda")
    dC = torch.full((M * N,), float("nan"), dtype=torch.float32, device="cuda")
    g.force_config("t128x128:s32")
    try:
        rc = g.gemm_f16f32_noalloc(M, N, K, dA, 0, 0, dB, 0, 0, dC, 0, 0, stream, check=False)
    finally:
        g.force_config(None)
    assert rc == -4 and "workspace" in g.status_string(rc)
    torch.cuda.synchronize()
    assert bool(torch.isnan(dC).all()), "a refused call must not enqueue anything"
    # the automatic selection stays within the array
    g.gemm_f16f32_noalloc(M, N, K, dA, 0, 0, dB, 0, 0, dC, 0, 0, stream)
    torch.cuda.synchronize()
    assert bool((dC == 0).all())


def test_noalloc_k_sliced_call_under_graph_capture(oracle):
    # The use the entry point is for: a K-sliced product recorded into a HIP graph (the allocating
    # entry point may call hipMalloc there).  The graph is replayed several times with eager work
    # and synchronisation in between, inputs changed in place, every replay checked against the
    # oracle bit for bit (integer-valued operands).
    import torch
    import paper_2003_06324_amd as g
    M, N, K = 192, 160, 1536
    A0, B0 = gi.make_problem(1300, M, N, K, "int", "f16")
    dA = torch.from_numpy(gi.store(A0, gi.ROW_MAJOR).view(np.int16)).cuda()
    dB = torch.from_numpy(gi.store(B0, gi.COL_MAJOR).view(np.int16)).cuda()
    dC = torch.full((M * N,), float("nan"), dtype=torch.float32, device="cuda")
    g.force_config("t64x64:s6")
    try:
        graph = torch.cuda.CUDAGraph()
        torch.cuda.synchronize()
        with torch.cuda.graph(graph):
            s = torch.cuda.current_stream().cuda_stream
            g.gemm_f16f32_noalloc(M, N, K, dA, gi.ROW_MAJOR, 0, dB, gi.COL_MAJOR, 0, dC, gi.ROW_MAJOR, 0, s)
            assert "s6 static-scratch" in g.last_config()
    finally:
        g.force_config(None)
    for rep in range(4):
        A, B = gi.make_problem(1301 + rep, M, N, K, "int", "f16")
        dA.copy_(torch.from_numpy(gi.store(A, gi.ROW_MAJOR).view(np.int16)))
        dB.copy_(torch.from_numpy(gi.store(B, gi.COL_MAJOR).view(np.int16)))
        dC.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        want = oracle.gemm(M, N, K, A, gi.ROW_MAJOR, B, gi.ROW_MAJOR, "f16").astype(np.float32)
        assert np.array_equal(dC.cpu().numpy().reshape(M, N), want), rep
