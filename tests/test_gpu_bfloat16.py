"""Parity of the bfloat16-operand entry point (gemm_bf16f32) with the CPU oracle: the kernels
are the binary16 ones with the other matrix instruction, so the cases are the ones that
separate the two (values outside the binary16 range, bit-exact integer sums through every
tile, layout, K-slice count and load path) plus the random-data bar of the binary16 tests."""
import itertools

import numpy as np
import pytest

import gemm_inputs as gi
from gpu_util import ran_tile, all_tiles, check, run_gpu

pytestmark = pytest.mark.gpu

LAYS = (gi.ROW_MAJOR, gi.COL_MAJOR)
LAYOUT_PAIRS = list(itertools.product(LAYS, repeat=2))
TILES = all_tiles()   # every configuration the library has, the K-split-across-waves ones included


def reference(oracle, A, B):
    M, K = A.shape
    return oracle.gemm(M, B.shape[1], K, gi.bfloat16_bits(A), gi.ROW_MAJOR, gi.bfloat16_bits(B), gi.ROW_MAJOR, "bf16")


@pytest.mark.parametrize("shape", [(256, 256, 256), (300, 200, 100), (129, 257, 65), (513, 383, 130), (64, 72, 520),
                                   (1, 1, 1), (7, 5, 3), (1, 300, 64), (640, 512, 1100)])
def test_random_all_layouts(oracle, shape):
    M, N, K = shape
    for dist in ("uniform", "normal"):
        A, B = gi.make_problem(300 + M + N + K, M, N, K, dist, "bf16")
        ref = reference(oracle, A, B)
        for la, lb in LAYOUT_PAIRS:
            C, cfg = run_gpu("bf16", A, B, la, lb, return_config=True)
            assert cfg.startswith("bf16 ")
            check(C, ref, A, B, "bf16", "%s %s la=%d lb=%d" % (shape, dist, la, lb))


@pytest.mark.parametrize("tile", TILES)
def test_integer_inputs_bit_exact_every_tile(oracle, tile):
    for (M, N, K) in [(300, 260, 200), (257, 129, 67), (512, 512, 1024)]:
        A, B = gi.make_problem(23 + M, M, N, K, "int", "bf16")
        ref = reference(oracle, A, B)
        assert np.array_equal(ref, A.astype(np.int64) @ B.astype(np.int64))
        for la, lb in LAYOUT_PAIRS:
            for splits in (1, 3):
                C, cfg = run_gpu("bf16", A, B, la, lb, force="%s:s%d" % (tile, splits), return_config=True)
                assert ran_tile(tile, cfg) and cfg.startswith("bf16 ")
                assert np.array_equal(C.astype(np.float64), ref), (tile, M, N, K, la, lb, splits, cfg)


def test_unaligned_bases_padding_and_column_major_c(oracle):
    A, B = gi.make_problem(41, 200, 168, 144, "int", "bf16")
    ref = reference(oracle, A, B)
    for la, lb, lc in itertools.product(LAYS, repeat=3):
        for pads, offs in (((8, 16, 3), (0, 0, 0)), ((1, 3, 5), (0, 0, 0)), ((0, 0, 0), (1, 3, 1)),
                           ((8, 8, 0), (8, 16, 2))):
            C, cfg = run_gpu("bf16", A, B, la, lb, lc, pads=pads, offsets=offs, return_config=True)
            assert np.array_equal(C.astype(np.float64), ref), (la, lb, lc, pads, offs, cfg)


def test_values_outside_the_binary16_range(oracle):
    # powers of two from 2^-40 to 2^40 in A against their inverses in B: every product is a
    # small integer, every operand is far outside what binary16 holds, so a kernel that read
    # the patterns as binary16 (or the binary16 instruction) cannot produce these sums
    M, N, K = 96, 80, 164
    rng = np.random.default_rng(5)
    e = rng.integers(-40, 41, size=K)
    A = (rng.integers(-3, 4, size=(M, K)) * 2.0 ** e[None, :]).astype(np.float32)
    B = (rng.integers(-3, 4, size=(K, N)) * 2.0 ** -e[:, None]).astype(np.float32)
    assert np.array_equal(gi.round_to_bfloat16(A), A) and np.array_equal(gi.round_to_bfloat16(B), B)
    ref = reference(oracle, A, B)
    assert np.max(np.abs(ref)) > 50
    for la, lb in LAYOUT_PAIRS:
        for force in (None, "t256x256", "t64x64:s2"):
            C = run_gpu("bf16", A, B, la, lb, force=force)
            assert np.array_equal(C.astype(np.float64), ref), (la, lb, force)
    # seven fraction bits: 1 + 2^-7 is a bfloat16 number, its square 1 + 2^-6 + 2^-14 is exact in binary32
    A1 = np.full((33, 8), 1.0 + 2.0 ** -7, np.float32)
    C = run_gpu("bf16", A1, np.ascontiguousarray(A1.T), 0, 0)
    assert np.array_equal(C, np.full((33, 33), 8 * (1.0 + 2.0 ** -6 + 2.0 ** -14), np.float32))


def test_degenerate_sizes(oracle):
    A = np.zeros((5, 0), np.float32)
    B = np.zeros((0, 7), np.float32)
    C = run_gpu("bf16", A, B, 0, 0)
    assert C.shape == (5, 7) and np.array_equal(C, np.zeros((5, 7), np.float32))
    C = run_gpu("bf16", np.zeros((0, 4), np.float32), np.zeros((4, 3), np.float32), 0, 1)
    assert C.shape == (0, 3)


def test_headline_size_sampled(oracle):
    # the 8192^3 NT launch of the benchmark with bfloat16 patterns: sampled entries, one by one
    import torch
    import paper_2003_06324_amd as g
    S = 8192
    A, B = gi.make_problem(3100, S, S, S, "normal", "bf16")
    bA, bB = gi.bfloat16_bits(A), gi.bfloat16_bits(np.ascontiguousarray(B.T))
    dA, dB = torch.from_numpy(bA.view(np.int16)).cuda(), torch.from_numpy(bB.view(np.int16)).cuda()
    dC = torch.empty(S * S, dtype=torch.float32, device="cuda")
    g.gemm_bf16f32(S, S, S, dA, 0, 0, dB, 1, 0, dC, 0, 0, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    assert g.last_config() == "bf16 t256x256 NT aligned s1"
    rng = np.random.default_rng(1)
    rows = np.concatenate([rng.integers(0, S, 2000), [0, S - 1, 255, 256, S - 1]])
    cols = np.concatenate([rng.integers(0, S, 2000), [0, S - 1, 256, 255, 0]])
    want = oracle.gemm_at(S, S, S, bA.reshape(-1), 0, 0, bB.reshape(-1), 1, 0, rows, cols, "bf16")
    got = dC.cpu().numpy().reshape(S, S)[rows, cols].astype(np.float64)
    scale = S * np.sqrt(np.mean(A.astype(np.float64) ** 2)) * np.sqrt(np.mean(B.astype(np.float64) ** 2))
    assert np.max(np.abs(got - want)) / scale <= 8 * 2.0 ** -24
