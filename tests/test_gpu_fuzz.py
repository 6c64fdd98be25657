"""Seeded random sweep over shapes, layouts, leading dimensions, base offsets, tile
configurations, K-slice counts and result types: integer-valued operands, so the result of
every kernel variant must equal the oracle's bit for bit."""
import numpy as np
import pytest

import gemm_inputs as gi
from gpu_util import all_tiles, run_gpu

pytestmark = pytest.mark.gpu

TILES = all_tiles()   # every configuration the library has, the K-split-across-waves ones included


def draw_case(rng):
    dtype = "f16" if rng.random() < 0.65 else "f32"
    bk = 64 if dtype == "f16" else 32
    kind = rng.integers(0, 4)
    if kind == 0:      # small and ragged
        M, N, K = (int(rng.integers(1, 140)) for _ in range(3))
    elif kind == 1:    # several tiles, K around multiples of the slab
        M, N = int(rng.integers(1, 700)), int(rng.integers(1, 700))
        K = max(1, int(rng.integers(1, 24)) * bk + int(rng.choice([0, 0, 1, -1, 8, 17])))
    elif kind == 2:    # granule-aligned sizes (direct-load kernels unless padding says otherwise)
        M, N = 8 * int(rng.integers(1, 80)), 8 * int(rng.integers(1, 80))
        K = 8 * int(rng.integers(1, 200))
    else:              # skinny
        M, N = int(rng.integers(1, 40)), int(rng.integers(200, 900))
        if rng.random() < 0.5:
            M, N = N, M
        K = int(rng.integers(1, 1500))
    la, lb, lc = (int(rng.integers(0, 2)) for _ in range(3))
    epc = 8 if dtype == "f16" else 4
    # paddings and base offsets in elements: multiples of the 16-byte granule, of 4 bytes (direct loads on rows
    # that straddle cache lines) and odd counts (2-byte aligned binary16: register-staged loads)
    pads = tuple(int(rng.choice([0, 0, epc, 2 * epc, 1, 3, 5, 2, 4, 6])) for _ in range(3))
    offs = tuple(int(rng.choice([0, 0, 0, epc, 1, 2, 4, 6])) for _ in range(3))
    force = None
    if rng.random() < 0.7:
        force = "%s:s%d" % (rng.choice(TILES), int(rng.choice([1, 1, 1, 2, 3, 4, 7])))
        # variants of the same kernels: fully synchronised hand-overs, either store path, register-staged loads
        for suffix, prob in ((":safe", 0.15), (str(rng.choice([":direct", ":staged"])), 0.3), (":regload", 0.15)):
            if rng.random() < prob:
                force += suffix
    out = "f16" if (dtype == "f16" and rng.random() < 0.3) else "f32"
    return dtype, M, N, K, la, lb, lc, pads, offs, force, out


@pytest.mark.parametrize("chunk", range(8))
def test_random_cases_bit_exact(oracle, chunk):
    rng = np.random.default_rng(20240 + chunk)
    for case in range(30):
        dtype, M, N, K, la, lb, lc, pads, offs, force, out = draw_case(rng)
        A, B = gi.make_problem(int(rng.integers(1, 1 << 30)), M, N, K, "int", dtype)
        exact = oracle.gemm(M, N, K, A, gi.ROW_MAJOR, B, gi.ROW_MAJOR, dtype)
        what = (chunk, case, dtype, M, N, K, la, lb, lc, pads, offs, force, out)
        C, cfg = run_gpu(dtype, A, B, la, lb, lc, pads=pads, offsets=offs, force=force, return_config=True, out=out)
        if out == "f16":
            want = oracle.round_to_half(exact)
            assert np.array_equal(C.view(np.uint16), want.view(np.uint16)), (what, cfg)
        else:
            assert np.array_equal(C, exact.astype(np.float32)), (what, cfg)


@pytest.mark.parametrize("chunk", range(3))
def test_random_cases_bit_exact_bfloat16(oracle, chunk):
    # the 16-bit draws of the same generator, as bfloat16 patterns through gemm_bf16f32
    rng = np.random.default_rng(30240 + chunk)
    done = 0
    while done < 25:
        dtype, M, N, K, la, lb, lc, pads, offs, force, _ = draw_case(rng)
        seed = int(rng.integers(1, 1 << 30))
        if dtype != "f16":
            continue
        done += 1
        A, B = gi.make_problem(seed, M, N, K, "int", "bf16")
        exact = oracle.gemm(M, N, K, gi.bfloat16_bits(A), gi.ROW_MAJOR, gi.bfloat16_bits(B), gi.ROW_MAJOR, "bf16")
        what = (chunk, done, M, N, K, la, lb, lc, pads, offs, force)
        C, cfg = run_gpu("bf16", A, B, la, lb, lc, pads=pads, offsets=offs, force=force, return_config=True)
        assert cfg.startswith("bf16 ")
        assert np.array_equal(C, exact.astype(np.float32)), (what, cfg)
