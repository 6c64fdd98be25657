"""Pins of the oracle's bfloat16 leg (CPU only): the widening against the format's definition
and against binary32 (a bfloat16 is the binary32 number with the same upper half), and the
product against exact integer arithmetic and against the separately pinned binary32 leg."""
import itertools
import math
import os
from fractions import Fraction

import numpy as np
import pytest

import gemm_inputs as gi

LAYS = (gi.ROW_MAJOR, gi.COL_MAJOR)
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def run(oracle, A, B, la, lb, lc=gi.ROW_MAJOR, pad=(0, 0, 0), dtype="bf16"):
    """Oracle on logical float32 matrices (holding bfloat16 values when dtype is bf16)."""
    M, K = A.shape
    N = B.shape[1]
    lda = (K if la == gi.ROW_MAJOR else M) + pad[0]
    ldb = (N if lb == gi.ROW_MAJOR else K) + pad[1]
    ldc = (N if lc == gi.ROW_MAJOR else M) + pad[2]
    bufA, bufB = gi.store(A, la, lda), gi.store(B, lb, ldb)
    if dtype == "bf16":
        C, ldc = oracle.gemm_bf16_raw(M, N, K, gi.bfloat16_bits(bufA), la, lda, gi.bfloat16_bits(bufB), lb, ldb, lc, ldc)
    else:
        C, ldc = oracle.gemm_f32_raw(M, N, K, bufA, la, lda, bufB, lb, ldb, lc, ldc)
    return np.array(gi.load(C, M, N, lc, ldc))


def test_widening_hand_constants(oracle):
    n = 0
    for line in open(os.path.join(GOLDEN, "bfloat16_constants.txt")):
        line = line.split("#")[0].strip()
        if not line:
            continue
        bits, value = line.split()
        want = float.fromhex(value) if "0x" in value else float(value)
        got = oracle.bfloat16_bits_to_double(int(bits, 16))
        assert got == want and math.copysign(1.0, got) == math.copysign(1.0, want), (bits, got, want)
        n += 1
    assert n >= 12


def test_widening_all_patterns_against_binary32(oracle):
    bits = np.arange(65536, dtype=np.uint32)
    with np.errstate(invalid="ignore"):  # signalling NaN patterns
        want = (bits << 16).astype(np.uint32).view(np.float32).astype(np.float64)
    got = np.array([oracle.bfloat16_bits_to_double(int(b)) for b in bits])
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], want[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(want[~nan]))
    # exactly the patterns with all exponent bits set and a non-zero fraction are NaN
    assert np.array_equal(nan, ((bits >> 7) & 0xFF == 0xFF) & (bits & 0x7F != 0))


def test_generator_rounding_to_nearest_even():
    # 1 + 2^-8 is halfway between 1 (even pattern 3f80) and 1 + 2^-7 (3f81); 1 + 3*2^-8 is
    # halfway between 3f81 and 3f82 (even); anything past a midpoint goes up
    x = np.array([1.0, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -20, 257.0, 259.0, -0.3], np.float32)
    bits = gi.bfloat16_bits(gi.round_to_bfloat16(x))
    assert [hex(b) for b in bits] == ["0x3f80", "0x3f80", "0x3f82", "0x3f81", "0x4380", "0x4382", "0xbe9a"]
    with pytest.raises(ValueError):
        gi.bfloat16_bits(np.array([1.0 + 2.0 ** -8], np.float32))


def test_brute_force_tiny_all_layouts(oracle):
    rng = np.random.default_rng(12)
    for M, N, K in itertools.product((1, 2, 3, 5), repeat=3):
        A = rng.integers(-7, 8, size=(M, K))
        B = rng.integers(-7, 8, size=(K, N))
        want = np.array([[int(sum(Fraction(int(A[i, k])) * int(B[k, j]) for k in range(K))) for j in range(N)]
                         for i in range(M)], dtype=np.float64)
        for la, lb, lc in itertools.product(LAYS, repeat=3):
            for pad in ((0, 0, 0), (3, 1, 2)):
                got = run(oracle, A.astype(np.float32), B.astype(np.float32), la, lb, lc, pad)
                assert np.array_equal(got, want), (M, N, K, la, lb, lc, pad)


def test_equals_binary32_leg_on_the_same_values(oracle):
    # a bfloat16 number is a binary32 number: both legs widen to the same float64 values and
    # must give identical sums; a wrong field width or bias in the widening shows here
    A, B = gi.make_problem(91, 37, 29, 150, "normal", "bf16")
    for la, lb in itertools.product(LAYS, repeat=2):
        assert np.array_equal(run(oracle, A, B, la, lb), run(oracle, A, B, la, lb, dtype="f32"))
    # values far from 1 in both directions (exponent handling)
    scale = np.float32(2.0) ** np.arange(-60, 60, 4, dtype=np.float32)
    A2 = gi.round_to_bfloat16(np.outer(np.arange(1, 6, dtype=np.float32), scale))
    B2 = gi.round_to_bfloat16(np.outer(1.0 / scale, np.arange(1, 4, dtype=np.float32)))
    assert np.array_equal(run(oracle, A2, B2, 0, 0), run(oracle, A2, B2, 0, 0, dtype="f32"))
    assert np.all(run(oracle, A2, B2, 0, 0) != 0)


def test_small_integers_closed_forms_and_transpose(oracle):
    A, B = gi.make_problem(9, 41, 23, 200, "int", "bf16")
    want = A.astype(np.int64) @ B.astype(np.int64)
    for la, lb in itertools.product(LAYS, repeat=2):
        assert np.array_equal(run(oracle, A, B, la, lb), want.astype(np.float64))
    ones = run(oracle, np.ones((6, 300), np.float32), np.ones((300, 7), np.float32), 0, 1)
    assert np.array_equal(ones, np.full((6, 7), 300.0))
    A, B = gi.make_problem(22, 13, 17, 29, "normal", "bf16")
    C = run(oracle, A, B, gi.ROW_MAJOR, gi.COL_MAJOR)
    Ct = run(oracle, np.ascontiguousarray(B.T), np.ascontiguousarray(A.T), gi.COL_MAJOR, gi.ROW_MAJOR)
    assert np.array_equal(C.T, Ct)
    # identity operand returns the other one
    X = gi.make_problem(5, 19, 19, 19, "normal", "bf16")[0]
    assert np.array_equal(run(oracle, np.eye(19, dtype=np.float32), X, 1, 0), X.astype(np.float64))


def test_sampled_entries_and_degenerate_sizes(oracle):
    A, B = gi.make_problem(14, 33, 27, 70, "uniform", "bf16")
    full = run(oracle, A, B, 0, 1)
    rows = [0, 32, 5, 17, 32]
    cols = [0, 26, 11, 3, 0]
    got = oracle.gemm_at(33, 27, 70, gi.bfloat16_bits(gi.store(A, 0)), 0, 0, gi.bfloat16_bits(gi.store(B, 1)), 1, 0,
                         rows, cols, "bf16")
    assert np.array_equal(got, full[rows, cols])
    z = np.zeros(0, np.uint16)
    C, _ = oracle.gemm_bf16_raw(3, 2, 0, z, 0, 0, z, 0, 0)
    assert np.array_equal(C, np.zeros(6))
    C, _ = oracle.gemm_bf16_raw(0, 4, 5, z, 0, 0, np.zeros(20, np.uint16), 0, 0)
    assert C.size == 0
    with pytest.raises(ValueError):
        oracle.gemm_bf16_raw(2, 2, 2, np.zeros(4, np.uint16), 0, 1, np.zeros(4, np.uint16), 0, 0)
