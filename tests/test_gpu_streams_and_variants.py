"""Behaviour around the kernels: K-sliced calls issued concurrently on several streams, a stale
runtime error left by the caller, the fully synchronised ("safe") variant of every tile, and
the two ways C is stored (staged through LDS in whole rows, or straight from registers)."""
import ctypes
import itertools

import numpy as np
import pytest

import gemm_inputs as gi
from gpu_util import ran_tile, run_gpu

pytestmark = pytest.mark.gpu

LAYS = (gi.ROW_MAJOR, gi.COL_MAJOR)
LAYOUT_PAIRS = list(itertools.product(LAYS, repeat=2))


def ref_of(oracle, A, B, dtype):
    M, K = A.shape
    return oracle.gemm(M, B.shape[1], K, A, gi.ROW_MAJOR, B, gi.ROW_MAJOR, dtype)


def test_k_sliced_calls_on_two_streams_without_host_sync(oracle):
    # Both streams run K-sliced products of different shapes, interleaved, with no host
    # synchronisation in between: each (device, stream) pair has its own workspace, so the
    # partial sums of one call can never land in the other's.  The larger product is issued
    # first on each stream so that the second call of a stream finds a workspace big enough,
    # the third round grows it again while the earlier launches are still queued.
    import torch
    import paper_2003_06324_amd as g
    shapes = [(512, 384, 4096, 8), (192, 160, 1536, 4), (640, 512, 2048, 16)]
    problems = []
    for i, (M, N, K, s) in enumerate(shapes):
        A, B = gi.make_problem(700 + i, M, N, K, "int", "f16")
        problems.append((M, N, K, s, ref_of(oracle, A, B, "f16").astype(np.float32),
                         torch.from_numpy(gi.store(A, gi.ROW_MAJOR).view(np.int16)).cuda(),
                         torch.from_numpy(gi.store(B, gi.COL_MAJOR).view(np.int16)).cuda()))
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    outs = []
    try:
        for rep in range(3):
            for si, s in enumerate(streams):
                for pi in range(len(problems)):
                    M, N, K, slices, ref, dA, dB = problems[(pi + si + rep) % len(problems)]
                    with torch.cuda.stream(s):
                        dC = torch.full((M * N,), float("nan"), dtype=torch.float32, device="cuda")
                        g.force_config("t64x64:s%d" % slices)
                        g.gemm_f16f32(M, N, K, dA, gi.ROW_MAJOR, 0, dB, gi.COL_MAJOR, 0, dC, gi.ROW_MAJOR, 0, s.cuda_stream)
                        assert " s%d" % slices in g.last_config()
                    outs.append((dC, ref, M, N))
    finally:
        g.force_config(None)
    torch.cuda.synchronize()
    for dC, ref, M, N in outs:
        assert np.array_equal(dC.cpu().numpy().reshape(M, N), ref)


def _hip_runtime():
    """The HIP runtime this process already uses (the one torch loaded), by its mapped path."""
    for line in open("/proc/self/maps"):
        if "libamdhip64" in line:
            return ctypes.CDLL(line.split()[-1])
    raise RuntimeError("no HIP runtime mapped")


def test_stale_runtime_error_of_the_caller_is_not_reported(oracle):
    # An earlier failing runtime call of the caller (here: selecting a device that does not exist)
    # leaves its error pending in the thread; the library must report its own launches only,
    # also on the K-sliced path where a misread status would skip the reduce pass.
    import torch
    import paper_2003_06324_amd as g
    M, N, K = 192, 160, 1536
    A, B = gi.make_problem(41, M, N, K, "int", "f16")
    ref = ref_of(oracle, A, B, "f16").astype(np.float32)
    dA = torch.from_numpy(gi.store(A, gi.ROW_MAJOR).view(np.int16)).cuda()
    dB = torch.from_numpy(gi.store(B, gi.COL_MAJOR).view(np.int16)).cuda()
    stream = torch.cuda.current_stream().cuda_stream
    hip = _hip_runtime()
    try:
        for force in ("t64x64:s1", "t64x64:s4"):
            dC = torch.full((M * N,), float("nan"), dtype=torch.float32, device="cuda")
            g.force_config(force)
            torch.cuda.synchronize()
            assert hip.hipSetDevice(ctypes.c_int(4096)) != 0   # fails, error stays pending
            rc = g.gemm_f16f32(M, N, K, dA, gi.ROW_MAJOR, 0, dB, gi.COL_MAJOR, 0, dC, gi.ROW_MAJOR, 0, stream, check=False)
            hip.hipGetLastError()                               # cleared before torch looks at it
            assert rc == 0, (force, rc)
            torch.cuda.synchronize()
            assert np.array_equal(dC.cpu().numpy().reshape(M, N), ref), force
    finally:
        hip.hipGetLastError()
        g.force_config(None)


@pytest.mark.parametrize("dtype", ["f16", "f32"])
def test_safe_variant_bit_exact_every_tile(oracle, dtype):
    # the same kernels with every hand-over of an LDS buffer fully synchronised
    import paper_2003_06324_amd as g
    bk = 64 if dtype == "f16" else 32
    for (M, N, K) in [(300, 260, 9 * bk), (257, 129, 3 * bk + 5)]:
        A, B = gi.make_problem(17 + M, M, N, K, "int", dtype)
        ref = ref_of(oracle, A, B, dtype).astype(np.float32)
        for tile in g.config_names():
            for la, lb in LAYOUT_PAIRS:
                for pads in ((0, 0, 0), (1, 3, 0)):   # direct-load and register-staged pipelines
                    C, cfg = run_gpu(dtype, A, B, la, lb, pads=pads, force="%s:s1:safe" % tile, return_config=True)
                    assert "safe" in cfg and ran_tile(tile, cfg)
                    assert np.array_equal(C, ref), (dtype, tile, M, N, K, la, lb, pads, cfg)
    # and on data where the order of the additions shows: identical bits with and without
    A, B = gi.make_problem(18, 512, 384, 1024, "normal", dtype)
    for tile in g.config_names():
        plain = run_gpu(dtype, A, B, gi.ROW_MAJOR, gi.COL_MAJOR, force=tile)
        safe = run_gpu(dtype, A, B, gi.ROW_MAJOR, gi.COL_MAJOR, force=tile + ":safe")
        assert np.array_equal(plain, safe), (dtype, tile)


@pytest.mark.parametrize("dtype,out", [("f16", "f32"), ("f16", "f16"), ("f32", "f32"), ("bf16", "f32")])
def test_staged_and_direct_stores_agree(oracle, dtype, out):
    # Interior tiles of a C whose rows start on 16-byte boundaries are staged through LDS and
    # written 16 bytes per lane; ":direct" keeps the register-to-memory stores for the same tiles.
    # Both must give the oracle's bits on integer data, with padded C rows, offset bases that are
    # still 16-byte aligned, column-major C (operands swapped) and K slices.
    import paper_2003_06324_amd as g
    A, B = gi.make_problem(23, 600, 520, 200, "int", dtype)
    if dtype == "bf16":
        exact = oracle.gemm(600, 520, 200, gi.bfloat16_bits(A), 0, gi.bfloat16_bits(B), 0, "bf16")
    else:
        exact = oracle.gemm(600, 520, 200, A, 0, B, 0, dtype)
    want = exact.astype(np.float32) if out == "f32" else oracle.round_to_half(exact)
    step = 4 if out == "f32" else 8   # elements per 16 bytes of C
    for tile in g.config_names():
        for lc in LAYS:
            for pads, offs in (((0, 0, 0), (0, 0, 0)), ((0, 0, step), (0, 0, 2 * step)), ((0, 0, 3), (0, 0, 0))):
                for slices in (1, 2):
                    for how in ("", ":direct", ":staged"):
                        C, cfg = run_gpu(dtype, A, B, gi.ROW_MAJOR, gi.COL_MAJOR, lc, pads=pads, offsets=offs,
                                         force="%s:s%d%s" % (tile, slices, how), return_config=True, out=out)
                        assert np.array_equal(C.view(np.uint16 if out == "f16" else np.uint32),
                                              want.view(np.uint16 if out == "f16" else np.uint32)), (cfg, lc, pads, offs, how)


@pytest.mark.parametrize("dtype,out", [("f16", "f32"), ("f16", "f16"), ("f32", "f32"), ("bf16", "f32")])
def test_k_split_across_the_waves_of_a_workgroup(oracle, dtype, out):
    # The "k" configurations give each of the four waves the whole tile and one k-group of every
    # slab, and sum the four partial tiles in LDS.  K is a multiple of the slab and the operands
    # are 16-byte aligned here, so this kernel (not its two-dimensional stand-in) must run:
    # every slab count from 1 to 7 and a long one, ragged M and N, all layouts, K-slices across
    # workgroups on top, padded and column-major C, the fully synchronised variant.
    import paper_2003_06324_amd as g
    bk = 32 if dtype == "f32" else 64
    ktiles = [t for t in g.config_names() if t[0] == "k"]
    assert ktiles
    for tile in ktiles:
        for slabs in (1, 2, 3, 4, 5, 6, 7, 23):
            K = slabs * bk
            for (M, N) in ((136, 72), (64, 64), (200, 328)) if slabs in (1, 4, 23) else ((136, 72),):
                A, B = gi.make_problem(51 + K + M, M, N, K, "int", dtype)
                if dtype == "bf16":
                    exact = oracle.gemm(M, N, K, gi.bfloat16_bits(A), 0, gi.bfloat16_bits(B), 0, "bf16")
                else:
                    exact = oracle.gemm(M, N, K, A, 0, B, 0, dtype)
                want = exact.astype(np.float32) if out == "f32" else oracle.round_to_half(exact)
                bits = np.uint16 if out == "f16" else np.uint32
                for la, lb in LAYOUT_PAIRS:
                    for force, lc, pads in ((tile, gi.ROW_MAJOR, (0, 0, 0)), (tile + ":s2", gi.ROW_MAJOR, (0, 0, 0)),
                                            (tile + ":safe", gi.COL_MAJOR, (0, 0, 3)), (tile, gi.ROW_MAJOR, (8, 8, 8))):
                        C, cfg = run_gpu(dtype, A, B, la, lb, lc, pads=pads, force=force, return_config=True, out=out)
                        # M or N not a multiple of the 16-byte granule makes an M/N-contiguous operand
                        # unaligned (granules straddle the edge): then the stand-in tile runs
                        served = (la == gi.ROW_MAJOR or M % (16 // A.itemsize if dtype != "bf16" else 8) == 0) and \
                                 (lb == gi.COL_MAJOR or N % (16 // B.itemsize if dtype != "bf16" else 8) == 0)
                        assert (tile in cfg.split()) == served, (cfg, M, N, K, la, lb)
                        assert np.array_equal(C.view(bits), want.view(bits)), (cfg, M, N, K, la, lb, lc, pads)
    # random data: the bar of the other kernels
    from gpu_util import check
    if out == "f32":
        A, B = gi.make_problem(52, 320, 192, 20 * bk, "normal", dtype)
        if dtype == "bf16":
            ref = oracle.gemm(320, 192, 20 * bk, gi.bfloat16_bits(A), 0, gi.bfloat16_bits(B), 0, "bf16")
        else:
            ref = oracle.gemm(320, 192, 20 * bk, A, 0, B, 0, dtype)
        for tile in ktiles:
            for la, lb in LAYOUT_PAIRS:
                C, cfg = run_gpu(dtype, A, B, la, lb, force=tile, return_config=True)
                assert tile in cfg.split()
                check(C, ref, A, B, dtype, cfg)


@pytest.mark.parametrize("dtype", ["f16", "f32", "bf16"])
def test_direct_loads_on_four_byte_aligned_operands(oracle, dtype):
    # Bases and leading dimensions that are multiples of 4 bytes but not of 16 run the direct
    # global->LDS loads (the configuration string says "aligned4"): every tile, all layouts, base
    # offsets and row paddings of 4, 8 and 12 bytes, K slices, a ragged K tail.  The same inputs
    # through the register-staged kernels (":regload") must give the same bits.
    import paper_2003_06324_amd as g
    esz = 4 if dtype == "f32" else 2
    for (M, N, K) in [(264, 136, 200), (512, 384, 324)]:
        A, B = gi.make_problem(71 + M, M, N, K, "int", dtype)
        if dtype == "bf16":
            ref = oracle.gemm(M, N, K, gi.bfloat16_bits(A), 0, gi.bfloat16_bits(B), 0, "bf16").astype(np.float32)
        else:
            ref = ref_of(oracle, A, B, dtype).astype(np.float32)
        for tile in g.config_names():
            for la, lb in LAYOUT_PAIRS:
                for off_bytes, pad_bytes in ((4, 0), (8, 8), (12, 4), (0, 12)):
                    offs = (off_bytes // esz, off_bytes // esz, 0)
                    pads = (pad_bytes // esz, pad_bytes // esz, 0)
                    for how in ("", ":s2", ":regload"):
                        C, cfg = run_gpu(dtype, A, B, la, lb, pads=pads, offsets=offs, force=tile + how, return_config=True)
                        assert ("general" if how == ":regload" else "aligned4") in cfg.split(), cfg
                        assert np.array_equal(C, ref), (dtype, M, N, K, la, lb, offs, pads, cfg)


def test_register_staged_kernels_forced_on_aligned_operands(oracle):
    # ":regload" keeps the register-staged pipeline reachable for operands the direct loads serve
    import paper_2003_06324_amd as g
    for dtype in ("f16", "f32"):
        bk = 32 if dtype == "f32" else 64
        A, B = gi.make_problem(73, 300, 264, 7 * bk + 8, "int", dtype)
        ref = ref_of(oracle, A, B, dtype).astype(np.float32)
        for tile in g.config_names():
            for la, lb in LAYOUT_PAIRS:
                C, cfg = run_gpu(dtype, A, B, la, lb, force=tile + ":regload", return_config=True)
                assert "general" in cfg.split(), cfg
                assert np.array_equal(C, ref), (dtype, tile, la, lb, cfg)


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_two_byte_aligned_operands(oracle, dtype):
    # 16-bit operands whose bases or leading dimensions are odd element counts are only 2-byte
    # aligned and run the register-staged kernels (16-byte loads at element alignment).  Odd leading
    # dimensions move the misalignment from row to row, odd base offsets shift every row; edge tiles
    # re-read rows; every tile, layout pair, K slices and a K tail.
    import paper_2003_06324_amd as g
    for (M, N, K) in [(264, 136, 200), (77, 300, 3 * 64 + 5), (513, 129, 2 * 64), (1, 9, 64), (130, 2, 4 * 64)]:
        A, B = gi.make_problem(81 + M, M, N, K, "int", dtype)
        if dtype == "bf16":
            ref = oracle.gemm(M, N, K, gi.bfloat16_bits(A), 0, gi.bfloat16_bits(B), 0, "bf16").astype(np.float32)
        else:
            ref = ref_of(oracle, A, B, dtype).astype(np.float32)
        for tile in g.config_names():
            for la, lb in LAYOUT_PAIRS:
                for pads, offs in (((1, 1, 0), (0, 0, 0)), ((0, 0, 0), (1, 3, 0)), ((3, 5, 0), (1, 1, 0)), ((1, 0, 0), (0, 1, 0))):
                    for how in ("", ":s2"):
                        C, cfg = run_gpu(dtype, A, B, la, lb, pads=pads, offsets=offs, force=tile + how, return_config=True)
                        lda = (K if la == gi.ROW_MAJOR else M) + pads[0]
                        ldb = (N if lb == gi.ROW_MAJOR else K) + pads[1]
                        two_byte = any(x % 2 for x in (lda, ldb, offs[0], offs[1]))   # odd element counts
                        assert ("general" in cfg.split()) == two_byte, (cfg, lda, ldb, offs)
                        assert np.array_equal(C, ref), (dtype, M, N, K, la, lb, pads, offs, cfg)


@pytest.mark.parametrize("entry", ["f16", "f16f16", "bf16", "f32", "noalloc"])
def test_k_slices_with_every_residue_of_n(oracle, entry):
    # Rows of the K-slice workspace are padded to a multiple of 32 floats, so N need not be a multiple
    # of 4 for the partials and the reduce pass to use 16-byte accesses; the last piece of a row is then
    # stored element by element, and C itself may have rows that are not 16-byte aligned.  Every N mod 4
    # (and N below one piece), forced slice counts on a square and a rectangular tile, C with and without
    # row padding and base offset, and the automatic choice on a deep K (which slices it).
    import torch
    import paper_2003_06324_amd as g
    dtype = {"f16f16": "f16", "noalloc": "f16"}.get(entry, entry)
    for N in (1, 3, 30, 33, 61, 62, 63, 64, 130):
        M, K = 70, 64 * 64 + 8     # deep enough for the automatic choice to cut K as well
        A, B = gi.make_problem(700 + N, M, N, K, "int", dtype)
        if dtype == "bf16":
            exact = oracle.gemm(M, N, K, gi.bfloat16_bits(A), 0, gi.bfloat16_bits(B), 0, "bf16")
        else:
            exact = ref_of(oracle, A, B, dtype)
        for force in ("t64x64:s3", "t128x64:s4", "t64x128:s2", None):
            for pads, offs in (((0, 0, 0), (0, 0, 0)), ((0, 0, 3), (0, 0, 1)), ((8, 8, 4), (0, 0, 4))):
                if entry == "noalloc":
                    if pads != (0, 0, 0):
                        continue
                    dA, dB = (torch.from_numpy(np.ascontiguousarray(x).view(np.int16)).cuda() for x in (A, B))
                    dC = torch.full((M * N,), float("nan"), dtype=torch.float32, device="cuda")
                    g.force_config(force)
                    try:
                        g.gemm_f16f32_noalloc(M, N, K, dA, gi.ROW_MAJOR, 0, dB, gi.ROW_MAJOR, 0, dC, gi.ROW_MAJOR, 0,
                                              torch.cuda.current_stream().cuda_stream)
                        cfg = g.last_config()
                    finally:
                        g.force_config(None)
                    torch.cuda.synchronize()
                    C = dC.cpu().numpy().reshape(M, N)
                    assert "static-scratch" in cfg, cfg
                else:
                    C, cfg = run_gpu(dtype, A, B, gi.ROW_MAJOR, gi.COL_MAJOR, pads=pads, offsets=offs, force=force,
                                     return_config=True, out="f16" if entry == "f16f16" else "f32")
                assert int(cfg.split()[4][1:]) > 1, cfg    # K really was cut into slices
                if entry == "f16f16":
                    assert np.array_equal(C.view(np.uint16), oracle.round_to_half(exact).view(np.uint16)), (N, force, pads, cfg)
                else:
                    assert np.array_equal(C, exact.astype(np.float32)), (entry, N, force, pads, offs, cfg)
