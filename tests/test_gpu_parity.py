"""Parity of the HIP path (through the C ABI) with the CPU oracle, element by element,
on seeded inputs.  Floating-point bar: max|C-Cref| / (K max|A| max|B|) <= 1e-6 (f32),
<= 2e-4 (f16 operands, f32 accumulation); integer-valued inputs must match bit for bit."""
import itertools

import numpy as np
import pytest

import gemm_inputs as gi
from gpu_util import ran_tile, all_tiles, check, run_gpu

pytestmark = pytest.mark.gpu

LAYS = (gi.ROW_MAJOR, gi.COL_MAJOR)
LAYOUT_PAIRS = list(itertools.product(LAYS, repeat=2))
TILES = all_tiles()   # every configuration the library has, the K-split-across-waves ones included

# several tiles of every configuration plus ragged tails in every dimension
SHAPES = [(256, 256, 256), (300, 200, 100), (129, 257, 65), (513, 383, 130), (64, 72, 520),
          (1, 1, 1), (7, 5, 3), (33, 1, 77), (1, 300, 64)]


def ref_of(oracle, A, B, dtype):
    M, K = A.shape
    return oracle.gemm(M, B.shape[1], K, A, gi.ROW_MAJOR, B, gi.ROW_MAJOR, dtype)


@pytest.mark.parametrize("dtype", ["f16", "f32"])
@pytest.mark.parametrize("shape", SHAPES)
def test_random_all_layouts(oracle, dtype, shape):
    M, N, K = shape
    A, B = gi.make_problem(100 + M + N + K, M, N, K, "uniform", dtype)
    ref = ref_of(oracle, A, B, dtype)
    for la, lb in LAYOUT_PAIRS:
        C = run_gpu(dtype, A, B, la, lb)
        check(C, ref, A, B, dtype, "%s %s la=%d lb=%d" % (dtype, shape, la, lb))


@pytest.mark.parametrize("dtype", ["f16", "f32"])
@pytest.mark.parametrize("tile", TILES)
def test_integer_bit_exact_every_tile(oracle, dtype, tile):
    # entries in {-4..4}: every partial sum is an exact integer below 2^24, so any
    # summation order gives the same binary32 result and equality must be exact
    for (M, N, K) in [(300, 260, 200), (257, 129, 67), (512, 512, 192)]:
        A, B = gi.make_problem(7 + M, M, N, K, "int", dtype)
        ref = ref_of(oracle, A, B, dtype).astype(np.float32)
        for la, lb in LAYOUT_PAIRS:
            for splits in (1, 3):
                C, cfg = run_gpu(dtype, A, B, la, lb, force="%s:s%d" % (tile, splits), return_config=True)
                assert ran_tile(tile, cfg)
                assert np.array_equal(C, ref), (dtype, tile, M, N, K, la, lb, splits, cfg)


@pytest.mark.parametrize("dtype", ["f16", "f32"])
def test_k_loop_lengths(oracle, dtype):
    # every K-loop trip count from a lone partial slab up to 18 slabs and a tail, on aligned
    # and unaligned leading dimensions: prologue only, the run-time-slot tiles, one, two and
    # three groups of the loop that is unrolled over the five-slot ring, each with and
    # without leftover tiles and a ragged tail (bk = K-slab of the kernels)
    bk = 64 if dtype == "f16" else 32
    ks = [1, 2, 7, 8, bk - 1, bk, bk + 1, bk + 8, 2 * bk, 3 * bk + 8, 4 * bk, 4 * bk + 1, 5 * bk,
          6 * bk + 16, 7 * bk, 8 * bk, 8 * bk + 8, 9 * bk, 10 * bk, 11 * bk + 1, 12 * bk, 13 * bk + 8,
          14 * bk, 17 * bk, 18 * bk + 24]
    for K in ks:
        A, B = gi.make_problem(900 + K, 136, 72, K, "int", dtype)
        ref = ref_of(oracle, A, B, dtype).astype(np.float32)
        for la, lb in LAYOUT_PAIRS:
            for tile in TILES:
                C = run_gpu(dtype, A, B, la, lb, force=tile)
                assert np.array_equal(C, ref), (dtype, K, la, lb, tile)


@pytest.mark.parametrize("dtype", ["f16", "f32"])
def test_unaligned_edges_and_last_k_row(oracle, dtype):
    # Operands whose rows are not 16-byte aligned take the register-staged loop.  M or N not a
    # multiple of the 16-byte granule makes granules of an M/N-contiguous operand straddle the
    # matrix edge; K a multiple of the slab puts the operand's last k-row into a full slab
    # (which such tiles must leave to the guarded loop); tiny leading dimensions and K slices
    # on top.  Padding is NaN, so a value read from outside the matrix would show.
    bk = 64 if dtype == "f16" else 32
    shapes = [(300, 260, 4 * bk), (300, 260, 2 * bk), (77, 9, 3 * bk), (5, 7, 2 * bk), (12, 20, bk),
              (264, 300, 9 * bk), (130, 67, 9 * bk + 5), (3, 2, 5 * bk)]
    for (M, N, K) in shapes:
        A, B = gi.make_problem(400 + M + K, M, N, K, "int", dtype)
        ref = ref_of(oracle, A, B, dtype).astype(np.float32)
        for la, lb in LAYOUT_PAIRS:
            for tile in TILES:
                for splits, pads in ((1, (0, 0, 0)), (2, (0, 0, 0)), (1, (1, 3, 0)), (1, (2, 0, 1))):
                    C, cfg = run_gpu(dtype, A, B, la, lb, pads=pads, force="%s:s%d" % (tile, splits),
                                     return_config=True)
                    assert np.array_equal(C, ref), (dtype, M, N, K, la, lb, tile, splits, pads, cfg)


@pytest.mark.parametrize("dtype", ["f16", "f32"])
def test_leading_dimension_beyond_32_bit_tile_offsets(oracle, dtype):
    # 256 rows of such an operand span 2 GiB or more, so tile-local byte offsets do not fit
    # 32 bits: neither the direct loads nor the register-staged loop may be used
    ld = (1 << 31) // 256 // (2 if dtype == "f16" else 4)
    M, N, K = 3, 70, 200
    A, B = gi.make_problem(55, M, N, K, "int", dtype)
    ref = ref_of(oracle, A, B, dtype).astype(np.float32)
    for extra in (0, 8, 3):
        C, cfg = run_gpu(dtype, A, B, gi.ROW_MAJOR, gi.ROW_MAJOR, pads=(ld + extra - K, 0, 0), return_config=True)
        assert "general" in cfg and np.array_equal(C, ref), (dtype, extra, cfg)
        C, cfg = run_gpu(dtype, B.T.copy(), A.T.copy(), gi.COL_MAJOR, gi.COL_MAJOR, pads=(0, ld + extra - K, 0),
                         return_config=True)
        assert "general" in cfg and np.array_equal(C, ref.T), (dtype, extra, cfg)


@pytest.mark.parametrize("dtype", ["f16", "f32"])
def test_column_major_c_padding_and_offsets(oracle, dtype):
    A, B = gi.make_problem(31, 200, 168, 144, "int", dtype)
    ref = ref_of(oracle, A, B, dtype).astype(np.float32)
    epc = 8 if dtype == "f16" else 4
    for la, lb, lc in itertools.product(LAYS, repeat=3):
        # aligned padding keeps the direct-load kernels, odd padding / offsets force the guarded ones
        for pads, offs in (((epc, 2 * epc, 3), (0, 0, 0)), ((1, 3, 5), (0, 0, 0)), ((0, 0, 0), (1, 3, 1)),
                           ((epc, epc, 0), (epc, 2 * epc, 2))):
            C, cfg = run_gpu(dtype, A, B, la, lb, lc, pads=pads, offsets=offs, return_config=True)
            assert np.array_equal(C, ref), (dtype, la, lb, lc, pads, offs, cfg)


@pytest.mark.parametrize("dtype", ["f16", "f32"])
def test_split_k_matches_oracle(oracle, dtype):
    A, B = gi.make_problem(77, 192, 160, 1100, "uniform", dtype)
    ref = ref_of(oracle, A, B, dtype)
    for la, lb in LAYOUT_PAIRS:
        for splits in (2, 5, 16):
            C, cfg = run_gpu(dtype, A, B, la, lb, force="t64x64:s%d" % splits, return_config=True)
            used = int(cfg.rsplit(" s", 1)[1])   # slices actually used (empty slices are dropped)
            assert 1 < used <= splits, cfg
            check(C, ref, A, B, dtype, cfg)


@pytest.mark.parametrize("dtype", ["f16", "f32"])
def test_degenerate_sizes(dtype):
    import torch
    import paper_2003_06324_amd as g
    fn = g.gemm_f32 if dtype == "f32" else g.gemm_f16f32
    npdt = np.float32 if dtype == "f32" else np.float16
    # K == 0: C is the empty sum
    C = run_gpu(dtype, np.zeros((5, 0), npdt), np.zeros((0, 9), npdt), 0, 0)
    assert np.array_equal(C, np.zeros((5, 9), np.float32))
    C = run_gpu(dtype, np.zeros((5, 0), npdt), np.zeros((0, 9), npdt), 1, 0, gi.COL_MAJOR, pads=(0, 0, 2))
    assert np.array_equal(C, np.zeros((5, 9), np.float32))
    # M == 0 or N == 0: nothing happens, no error
    x = torch.ones(64, dtype=torch.float32, device="cuda")
    assert fn(0, 4, 4, None, 0, 0, x, 0, 0, None, 0, 0) == 0
    assert fn(4, 0, 4, x, 0, 0, None, 0, 0, None, 0, 0) == 0
    # invalid arguments are rejected with a status, nothing is launched
    assert fn(-1, 4, 4, x, 0, 0, x, 0, 0, x, 0, 0, check=False) == -1
    assert fn(4, 4, 4, x, 0, 3, x, 0, 0, x, 0, 0, check=False) == -1   # lda < K
    assert fn(4, 4, 4, x, 2, 0, x, 0, 0, x, 0, 0, check=False) == -1   # bad layout
    assert fn(4, 4, 4, None, 0, 0, x, 0, 0, x, 0, 0, check=False) == -1  # null A
    assert g.force_config("t1x1", check=False) == -3
    torch.cuda.synchronize()


def test_run_to_run_bit_identical():
    # same launch twice: a race in the double buffer would show as differing bits
    A, B = gi.make_problem(5, 640, 512, 1024, "normal", "f16")
    for la, lb in LAYOUT_PAIRS:
        first = run_gpu("f16", A, B, la, lb)
        for _ in range(3):
            assert np.array_equal(run_gpu("f16", A, B, la, lb), first)


def test_inf_and_nan_only_where_the_inputs_put_them(oracle):
    A, B = gi.make_problem(9, 130, 140, 70, "uniform", "f16")
    A = A.copy()
    A[3, 5] = np.inf
    A[100, 69] = np.nan
    ref = ref_of(oracle, A, B, "f16")
    for la, lb in LAYOUT_PAIRS:
        C = run_gpu("f16", A, B, la, lb)
        assert np.array_equal(np.isnan(C), np.isnan(ref))
        assert np.array_equal(np.isinf(C), np.isinf(ref))
        ok = np.isfinite(ref)
        assert np.max(np.abs(C[ok] - ref[ok])) <= 2e-4 * 70


def test_user_streams_workspace_growth_and_shutdown(oracle):
    # Work is enqueued on the caller's stream (no priorities, plain torch streams) and ordered with
    # what that stream already holds; the K-slice workspace grows on demand, survives being grown
    # while earlier launches are still queued, and is rebuilt after gemm_shutdown().
    import torch
    import paper_2003_06324_amd as g
    A, B = gi.make_problem(91, 192, 160, 1536, "int", "f16")
    ref = ref_of(oracle, A, B, "f16").astype(np.float32)
    dA = torch.from_numpy(gi.store(A, gi.ROW_MAJOR).view(np.int16)).cuda()
    dB = torch.from_numpy(gi.store(B, gi.COL_MAJOR).view(np.int16)).cuda()
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    outs = []
    for rep, splits in enumerate((2, 8, 3, 16)):           # workspace 2, 8, 3, 16 slices: grows twice
        s = streams[rep % 2]
        with torch.cuda.stream(s):
            dC = torch.full((192 * 160,), float("nan"), dtype=torch.float32, device="cuda")   # ordered before the GEMM
            g.force_config("t64x64:s%d" % splits)
            g.gemm_f16f32(192, 160, 1536, dA, gi.ROW_MAJOR, 0, dB, gi.COL_MAJOR, 0, dC, gi.ROW_MAJOR, 0, s.cuda_stream)
            doubled = dC * 2.0                                                                # ordered after it
        s.synchronize()   # one stream at a time may use the workspace (include/gemm.h)
        outs.append((dC, doubled))
    g.force_config(None)
    for dC, doubled in outs:
        assert np.array_equal(dC.cpu().numpy().reshape(192, 160), ref)
        assert np.array_equal(doubled.cpu().numpy().reshape(192, 160), 2 * ref)
    assert g.shutdown() == 0 and g.shutdown() == 0
    C = run_gpu("f16", A, B, gi.ROW_MAJOR, gi.COL_MAJOR, force="t64x64:s4")
    assert np.array_equal(C, ref)


def test_graph_capture_and_replay(oracle):
    # Launches without K-slices allocate nothing, so a HIP graph can capture them.  The graph is
    # replayed several times with eager work and synchronisation in between, and every replay is
    # compared with the oracle (inputs change between replays, in place).
    import torch
    import paper_2003_06324_amd as g
    M, N, K = 384, 320, 704
    A0, B0 = gi.make_problem(101, M, N, K, "int", "f16")
    dA = torch.from_numpy(gi.store(A0, gi.ROW_MAJOR).view(np.int16)).cuda()
    dB = torch.from_numpy(gi.store(B0, gi.COL_MAJOR).view(np.int16)).cuda()
    dC = torch.full((M * N,), float("nan"), dtype=torch.float32, device="cuda")
    dC16 = torch.full((M * N,), float("nan"), dtype=torch.float16, device="cuda")
    g.force_config("t128x128:s1")
    try:
        graph = torch.cuda.CUDAGraph()
        torch.cuda.synchronize()
        with torch.cuda.graph(graph):
            s = torch.cuda.current_stream().cuda_stream
            g.gemm_f16f32(M, N, K, dA, gi.ROW_MAJOR, 0, dB, gi.COL_MAJOR, 0, dC, gi.ROW_MAJOR, 0, s)
            g.gemm_f16f16(M, N, K, dA, gi.ROW_MAJOR, 0, dB, gi.COL_MAJOR, 0, dC16, gi.ROW_MAJOR, 0, s)
    finally:
        g.force_config(None)
    for rep in range(4):
        A, B = gi.make_problem(200 + rep, M, N, K, "int", "f16")
        dA.copy_(torch.from_numpy(gi.store(A, gi.ROW_MAJOR).view(np.int16)))
        dB.copy_(torch.from_numpy(gi.store(B, gi.COL_MAJOR).view(np.int16)))
        dC.fill_(float("nan"))
        dC16.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        exact = ref_of(oracle, A, B, "f16")
        assert np.array_equal(dC.cpu().numpy().reshape(M, N), exact.astype(np.float32)), rep
        assert np.array_equal(dC16.cpu().numpy().reshape(M, N).view(np.uint16), oracle.round_to_half(exact).view(np.uint16)), rep
