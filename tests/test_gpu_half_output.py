"""Parity of the binary16-output entry point (gemm_f16f16) with the CPU oracle.

The oracle gives the exact sum in float64 and its single rounding to binary16; the GPU
rounds its binary32 accumulator.  Where the binary32 sum is exact (integer-valued inputs)
the two must agree bit for bit; otherwise the result may sit one binary16 step away from
the oracle's when the accumulation error carries the sum across a rounding boundary, so the
bar is: half a binary16 step at the value, plus the binary32 accumulation bound of the
binary32-output tests (8 * 2^-24 * K * rms|A| * rms|B|)."""
import itertools

import numpy as np
import pytest

import gemm_inputs as gi
from gpu_util import ran_tile, all_tiles, TIGHT, run_gpu

pytestmark = pytest.mark.gpu

LAYS = (gi.ROW_MAJOR, gi.COL_MAJOR)
LAYOUT_PAIRS = list(itertools.product(LAYS, repeat=2))
TILES = all_tiles()   # every configuration the library has, the K-split-across-waves ones included


def half_step(x):
    """Spacing of binary16 numbers at magnitude x (float64 array)."""
    x = np.maximum(np.abs(x), 2.0 ** -14)
    return np.maximum(2.0 ** (np.floor(np.log2(x)) - 10), 2.0 ** -24)


def check_half(C, ref, A, B, what=""):
    K = A.shape[1]
    a64, b64 = A.astype(np.float64), B.astype(np.float64)
    acc = TIGHT["f16"] * K * np.sqrt(np.mean(a64 ** 2)) * np.sqrt(np.mean(b64 ** 2))
    bound = 0.5 * half_step(np.abs(ref) + acc) + acc
    err = np.abs(C.astype(np.float64) - ref)
    assert np.all(np.isfinite(C.astype(np.float64))), what
    worst = float(np.max(err / bound)) if err.size else 0.0
    assert worst <= 1.0, "%s: error is %.3f of the bound" % (what, worst)


@pytest.mark.parametrize("shape", [(256, 256, 256), (300, 200, 100), (129, 257, 65), (513, 383, 130), (64, 72, 520),
                                   (1, 1, 1), (7, 5, 3), (1, 300, 64)])
def test_random_all_layouts(oracle, shape):
    M, N, K = shape
    A, B = gi.make_problem(200 + M + N + K, M, N, K, "uniform", "f16")
    ref = oracle.gemm(M, N, K, A, gi.ROW_MAJOR, B, gi.ROW_MAJOR, "f16")
    for la, lb in LAYOUT_PAIRS:
        C = run_gpu("f16", A, B, la, lb, out="f16")
        check_half(C, ref, A, B, "%s la=%d lb=%d" % (shape, la, lb))


@pytest.mark.parametrize("tile", TILES)
def test_integer_inputs_bit_exact_every_tile(oracle, tile):
    # entries in {-4..4}: the binary32 sum is the exact integer, so the stored binary16 must be
    # the oracle's rounding of that integer, bit for bit (sums beyond 2048 are really rounded)
    for (M, N, K) in [(300, 260, 200), (257, 129, 67), (512, 512, 1024)]:
        A, B = gi.make_problem(17 + M, M, N, K, "int", "f16")
        exact = oracle.gemm(M, N, K, A, gi.ROW_MAJOR, B, gi.ROW_MAJOR, "f16")
        ref = oracle.round_to_half(exact)
        for la, lb in LAYOUT_PAIRS:
            for splits in (1, 3):
                C, cfg = run_gpu("f16", A, B, la, lb, force="%s:s%d" % (tile, splits), return_config=True, out="f16")
                assert ran_tile(tile, cfg) and "f16f16" in cfg
                assert np.array_equal(C.view(np.uint16), ref.view(np.uint16)), (tile, M, N, K, la, lb, splits, cfg)


def test_column_major_c_padding_and_offsets(oracle):
    A, B = gi.make_problem(31, 200, 168, 144, "int", "f16")
    ref = oracle.round_to_half(oracle.gemm(200, 168, 144, A, gi.ROW_MAJOR, B, gi.ROW_MAJOR, "f16"))
    for la, lb, lc in itertools.product(LAYS, repeat=3):
        for pads, offs in (((8, 16, 3), (0, 0, 0)), ((1, 3, 5), (0, 0, 0)), ((0, 0, 0), (1, 3, 1)),
                           ((8, 8, 0), (8, 16, 2))):
            C, cfg = run_gpu("f16", A, B, la, lb, lc, pads=pads, offsets=offs, return_config=True, out="f16")
            assert np.array_equal(C.view(np.uint16), ref.view(np.uint16)), (la, lb, lc, pads, offs, cfg)


def test_overflow_zero_k_and_rounding_to_even(oracle):
    # 2048 * 32 = 65536 is beyond the binary16 range: infinity; 2049 is halfway between
    # 2048 and 2050: the even neighbour 2048; the empty sum is +0
    A = np.zeros((4, 32), np.float16)
    B = np.zeros((32, 3), np.float16)
    A[0, :] = 64.0
    B[:, 0] = 32.0          # 32 terms of 2048
    A[1, :2] = [2048.0, 1.0]
    B[:2, 1] = [1.0, 1.0]   # 2049
    A[2, :2] = [-2048.0, -3.0]
    B[:2, 2] = [1.0, 1.0]   # -2051 -> -2052
    exact = oracle.gemm(4, 3, 32, A, gi.ROW_MAJOR, B, gi.ROW_MAJOR, "f16")
    ref = oracle.round_to_half(exact)
    assert np.isinf(ref[0, 0]) and ref[1, 1] == 2048.0 and ref[2, 2] == -2052.0
    for la, lb in LAYOUT_PAIRS:
        C = run_gpu("f16", A, B, la, lb, out="f16")
        assert np.array_equal(C.view(np.uint16), ref.view(np.uint16)), (la, lb)
    C = run_gpu("f16", np.zeros((5, 0), np.float16), np.zeros((0, 9), np.float16), 0, 0, out="f16")
    assert np.array_equal(C.view(np.uint16), np.zeros((5, 9), np.uint16))


def test_full_size_sampled(oracle):
    # the benchmark's shape and data, A row-major, B column-major, on sampled entries
    import torch
    import paper_2003_06324_amd as g
    S = 8192
    A, B = gi.make_problem(3000, S, S, S, "normal", "f16")
    dA = torch.from_numpy(A.view(np.int16)).cuda()
    dB = torch.from_numpy(np.ascontiguousarray(B.T).view(np.int16)).cuda()
    dC = torch.empty(S * S, dtype=torch.float16, device="cuda")
    g.gemm_f16f16(S, S, S, dA, gi.ROW_MAJOR, 0, dB, gi.COL_MAJOR, 0, dC, gi.ROW_MAJOR, 0,
                  torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    assert "t256x256" in g.last_config()
    C = dC.cpu().numpy().reshape(S, S)
    rng = np.random.default_rng(1)
    rows = np.concatenate([rng.integers(0, S, 2000), [0, S - 1, 255, 256]])
    cols = np.concatenate([rng.integers(0, S, 2000), [0, S - 1, 256, 255]])
    ref = oracle.gemm_at(S, S, S, A, gi.ROW_MAJOR, 0, gi.store(B, gi.COL_MAJOR), gi.COL_MAJOR, 0, rows, cols, "f16")
    got = C[rows, cols]
    K = S
    acc = TIGHT["f16"] * K * 1.0
    bound = 0.5 * half_step(np.abs(ref) + acc) + acc
    assert np.all(np.abs(got.astype(np.float64) - ref) <= bound)
