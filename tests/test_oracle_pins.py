"""Pins for the CPU oracle: it is checked against things other than itself.

Each test states what a mistake in the oracle would have to look like to slip
past it.  None of these needs a GPU.
"""
import itertools
import os
from fractions import Fraction

import numpy as np
import pytest

import gemm_inputs as gi

LAYS = (gi.ROW_MAJOR, gi.COL_MAJOR)
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def brute(A, B):
    """Literal definition in exact rational arithmetic (Python ints / Fractions)."""
    M, K = len(A), (len(A[0]) if A else 0)
    N = len(B[0]) if B else 0
    return [[sum(Fraction(A[i][k]) * Fraction(B[k][j]) for k in range(K)) for j in range(N)]
            for i in range(M)]


def run(oracle, A, B, la, lb, lc=gi.ROW_MAJOR, dtype="f32", pad=(0, 0, 0)):
    """Oracle on logical numpy matrices with explicit layouts and ld padding."""
    M, K = A.shape
    N = B.shape[1]
    lda = (K if la == gi.ROW_MAJOR else M) + pad[0]
    ldb = (N if lb == gi.ROW_MAJOR else K) + pad[1]
    ldc = (N if lc == gi.ROW_MAJOR else M) + pad[2]
    fn = oracle.gemm_f32_raw if dtype == "f32" else oracle.gemm_f16_raw
    C, ldc = fn(M, N, K, gi.store(A, la, lda), la, lda, gi.store(B, lb, ldb), lb, ldb, lc, ldc)
    return np.array(gi.load(C, M, N, lc, ldc))


@pytest.mark.parametrize("dtype", ["f32", "f16"])
def test_brute_force_tiny_all_layouts(oracle, dtype):
    # wrong index, transposed operand, wrong ld use: all change some entry of a
    # non-square, non-symmetric integer product
    rng = np.random.default_rng(11)
    npdt = np.float32 if dtype == "f32" else np.float16
    for M, N, K in itertools.product((1, 2, 3, 5), repeat=3):
        A = rng.integers(-7, 8, size=(M, K))
        B = rng.integers(-7, 8, size=(K, N))
        want = np.array([[int(v) for v in row] for row in brute(A.tolist(), B.tolist())], dtype=np.float64)
        for la, lb, lc in itertools.product(LAYS, repeat=3):
            for pad in ((0, 0, 0), (3, 1, 2)):
                got = run(oracle, A.astype(npdt), B.astype(npdt), la, lb, lc, dtype, pad)
                assert np.array_equal(got, want), (M, N, K, la, lb, lc, pad)


def test_hand_worked_example(oracle):
    rows = [l.split() for l in open(os.path.join(GOLDEN, "matmul_hand_example.txt"))
            if l.strip() and not l.startswith("#")]
    vals = [[float(x) for x in r] for r in rows]
    A, B, C = np.array(vals[0:2], np.float32), np.array(vals[2:5], np.float32), np.array(vals[5:7])
    for la, lb in itertools.product(LAYS, repeat=2):
        assert np.array_equal(run(oracle, A, B, la, lb), C)
        assert np.array_equal(run(oracle, A.astype(np.float16), B.astype(np.float16), la, lb, dtype="f16"), C)


def test_exact_rational_non_integer(oracle):
    # dyadic fractions: products and sums exact in float64, so equality with the
    # rational brute force is exact; catches a dropped or doubled term
    rng = np.random.default_rng(5)
    A = (rng.integers(-64, 65, size=(4, 7)) / 32.0).astype(np.float32)
    B = (rng.integers(-64, 65, size=(7, 3)) / 16.0).astype(np.float32)
    want = np.array([[float(v) for v in row] for row in brute(A.tolist(), B.tolist())])
    for la, lb in itertools.product(LAYS, repeat=2):
        assert np.array_equal(run(oracle, A, B, la, lb), want)
        assert np.array_equal(run(oracle, A.astype(np.float16), B.astype(np.float16), la, lb, dtype="f16"), want)


@pytest.mark.parametrize("dtype", ["f32", "f16"])
def test_identity_and_permutation(oracle, dtype):
    rng = np.random.default_rng(3)
    M, K, N = 9, 9, 6
    X = gi.logical_matrix(rng, K, N, "uniform", dtype)
    Y = gi.logical_matrix(rng, M, K, "uniform", dtype)
    I = np.eye(K, dtype=X.dtype)
    perm = rng.permutation(K)
    P = I[:, perm]  # (Y @ P)[:, j] = Y[:, perm[j]]
    Q = I[perm, :]  # (Q @ X)[i, :] = X[perm[i], :]
    for la, lb in itertools.product(LAYS, repeat=2):
        assert np.array_equal(run(oracle, I, X, la, lb, dtype=dtype), X.astype(np.float64))
        assert np.array_equal(run(oracle, Y, I, la, lb, dtype=dtype), Y.astype(np.float64))
        assert np.array_equal(run(oracle, Y, P, la, lb, dtype=dtype), Y.astype(np.float64)[:, perm])
        assert np.array_equal(run(oracle, Q, X, la, lb, dtype=dtype), X.astype(np.float64)[perm, :])


@pytest.mark.parametrize("dtype", ["f32", "f16"])
def test_transpose_invariant(oracle, dtype):
    # (A B)^T == B^T A^T, exact: each entry adds the same products in the same k order
    A, B = gi.make_problem(21, 13, 17, 29, "normal", dtype)
    C = run(oracle, A, B, gi.ROW_MAJOR, gi.COL_MAJOR, dtype=dtype)
    Ct = run(oracle, np.ascontiguousarray(B.T), np.ascontiguousarray(A.T), gi.COL_MAJOR, gi.ROW_MAJOR, dtype=dtype)
    assert np.array_equal(C.T, Ct)


@pytest.mark.parametrize("dtype", ["f32", "f16"])
def test_small_integer_inputs_match_int64(oracle, dtype):
    # entries in {-4..4}: every partial sum is an exact integer in float64
    A, B = gi.make_problem(8, 67, 45, 300, "int", dtype)
    want = A.astype(np.int64) @ B.astype(np.int64)
    for la, lb in itertools.product(LAYS, repeat=2):
        got = run(oracle, A, B, la, lb, dtype=dtype)
        assert np.array_equal(got, want.astype(np.float64))
        assert np.array_equal(got.astype(np.float32).astype(np.int64), want)


@pytest.mark.parametrize("dtype", ["f32", "f16"])
def test_closed_forms(oracle, dtype):
    npdt = np.float32 if dtype == "f32" else np.float16
    M, N, K = 20, 33, 77
    ones = run(oracle, np.ones((M, K), npdt), np.ones((K, N), npdt), 0, 1, dtype=dtype)
    assert np.array_equal(ones, np.full((M, N), float(K)))
    A = np.tile((np.arange(M) % 8)[:, None], (1, K)).astype(npdt)
    B = np.tile((np.arange(N) % 8)[None, :], (K, 1)).astype(npdt)
    want = K * np.outer(np.arange(M) % 8, np.arange(N) % 8).astype(np.float64)
    assert np.array_equal(run(oracle, A, B, 1, 0, dtype=dtype), want)
    # one-hot rows of A pick rows of B
    rng = np.random.default_rng(2)
    X = gi.logical_matrix(rng, K, N, "normal", dtype)
    sel = rng.integers(0, K, size=M)
    H = np.zeros((M, K), npdt)
    H[np.arange(M), sel] = 1
    assert np.array_equal(run(oracle, H, X, 0, 0, dtype=dtype), X.astype(np.float64)[sel])


def test_ascending_k_single_accumulator(oracle):
    # float64 running sum in ascending k: (2^60 + 1) - 2^60 == 0, while any order
    # that adds the two big terms first, or a pairwise tree, gives 1
    A = np.array([[2.0 ** 60, 1.0, -(2.0 ** 60)]], np.float32)
    B = np.ones((3, 1), np.float32)
    assert run(oracle, A, B, 0, 0)[0, 0] == 0.0
    A2 = np.array([[2.0 ** 60, -(2.0 ** 60), 1.0]], np.float32)
    assert run(oracle, A2, B, 0, 0)[0, 0] == 1.0
    got = oracle.gemm_at(1, 1, 3, A.reshape(-1), 0, 0, B.reshape(-1), 0, 0, [0], [0], "f32")
    assert got[0] == 0.0


@pytest.mark.parametrize("dtype", ["f32", "f16"])
def test_numpy_float64_cross_check(oracle, dtype):
    # library matmul on float64 copies: differs from the oracle only in
    # summation order, bounded by K * 2^-52 * sum|a||b|
    A, B = gi.make_problem(77, 96, 80, 513, "normal", dtype)
    got = run(oracle, A, B, 0, 1, dtype=dtype)
    A64, B64 = A.astype(np.float64), B.astype(np.float64)
    bound = 513 * 2.0 ** -52 * (np.abs(A64) @ np.abs(B64))
    assert np.all(np.abs(got - A64 @ B64) <= bound)


def test_half_decode_all_bit_patterns(oracle):
    bits = np.arange(65536, dtype=np.uint16)
    want = bits.view(np.float16).astype(np.float64)
    got = np.array([oracle.half_bits_to_double(int(b)) for b in bits])
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], want[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(want[~nan]))


def test_half_rounding_hand_constants(oracle):
    path = os.path.join(os.path.dirname(__file__), "golden", "binary16_rounding_constants.txt")
    n = 0
    for line in open(path):
        fields = line.split("#")[0].split()
        if not fields:
            continue
        value = float.fromhex(fields[0]) if "p" in fields[0] else float(fields[0])
        assert oracle.double_to_half_bits(value) == int(fields[1], 16), fields
        n += 1
    assert n >= 20


def test_half_rounding_round_trip_and_ties(oracle):
    bits = np.arange(65536, dtype=np.uint16)
    vals = bits.view(np.float16).astype(np.float64)
    finite = np.isfinite(vals)
    # every binary16 value encodes back to its own pattern (infinities included)
    back = oracle.round_to_half(vals[~np.isnan(vals)]).view(np.uint16)
    assert np.array_equal(back, bits[~np.isnan(vals)])
    assert np.all(np.isnan(oracle.round_to_half(vals[np.isnan(vals)]).astype(np.float64)))
    # the exact midpoint of two neighbours goes to the one with the even pattern; a hair to
    # either side goes to the nearer one (positive finite patterns h, h+1)
    h = np.arange(0, 0x7BFF, dtype=np.uint16)
    lo, hi = vals[h], vals[h + 1]
    assert np.all(finite[h] & finite[h + 1])
    mid = (lo + hi) / 2          # exact in float64: 11 + 1 significant bits
    even = np.where(h % 2 == 0, h, h + 1)
    assert np.array_equal(oracle.round_to_half(mid).view(np.uint16), even)
    assert np.array_equal(oracle.round_to_half(-mid).view(np.uint16), even | 0x8000)
    eps = (hi - lo) * 2.0 ** -20
    assert np.array_equal(oracle.round_to_half(mid - eps).view(np.uint16), h)
    assert np.array_equal(oracle.round_to_half(mid + eps).view(np.uint16), h + 1)


def test_half_rounding_matches_numpy_conversion(oracle):
    # numpy's float64 -> float16 cast is an independent implementation of the same rounding
    rng = np.random.default_rng(42)
    x = rng.standard_normal(200000) * np.exp(rng.uniform(-20.0, 11.0, 200000))
    with np.errstate(over="ignore"):
        want = x.astype(np.float16).view(np.uint16)
    assert np.array_equal(oracle.round_to_half(x).view(np.uint16), want)


def test_half_subnormals_and_extremes_in_product(oracle):
    # smallest subnormal times largest normal; exact in float64
    A = np.array([[0x0001, 0x7BFF, 0x8001]], np.uint16).view(np.float16)
    B = np.array([[0x7BFF], [0x0001], [0x0400]], np.uint16).view(np.float16)
    want = 2.0 ** -24 * 65504.0 * 2 - 2.0 ** -24 * 2.0 ** -14
    assert run(oracle, A, B, 0, 0, dtype="f16")[0, 0] == want


@pytest.mark.parametrize("dtype", ["f32", "f16"])
def test_sampled_entries_match_brute_force_and_full(oracle, dtype):
    A, B = gi.make_problem(4, 23, 31, 40, "int", dtype)
    rows = np.array([0, 22, 5, 5, 17])
    cols = np.array([30, 0, 7, 8, 17])
    want = (A.astype(np.int64) @ B.astype(np.int64))[rows, cols].astype(np.float64)
    for la, lb in itertools.product(LAYS, repeat=2):
        got = oracle.gemm_at(23, 31, 40, gi.store(A, la), la, 0, gi.store(B, lb), lb, 0, rows, cols, dtype)
        assert np.array_equal(got, want)
    A, B = gi.make_problem(6, 23, 31, 40, "normal", dtype)
    full = run(oracle, A, B, 1, 0, dtype=dtype)
    got = oracle.gemm_at(23, 31, 40, gi.store(A, 1), 1, 0, gi.store(B, 0), 0, 0, rows, cols, dtype)
    assert np.array_equal(got, full[rows, cols])


def test_degenerate_sizes(oracle):
    z = np.zeros(0, np.float32)
    C, _ = oracle.gemm_f32_raw(3, 4, 0, z, 0, 0, z, 0, 0)
    assert np.array_equal(C, np.zeros(12))  # empty sum
    C, _ = oracle.gemm_f32_raw(0, 4, 5, z, 0, 0, np.ones(20, np.float32), 0, 0)
    assert C.size == 0
    C, _ = oracle.gemm_f32_raw(3, 0, 5, np.ones(15, np.float32), 0, 0, z, 0, 0)
    assert C.size == 0


def test_ld_padding_is_never_read(oracle):
    # gemm_inputs.store fills ld padding with NaN: a read of it poisons C
    A, B = gi.make_problem(9, 6, 7, 8, "uniform", "f32")
    for la, lb, lc in itertools.product(LAYS, repeat=3):
        got = run(oracle, A, B, la, lb, lc, pad=(5, 3, 4))
        assert np.all(np.isfinite(got))
        assert np.array_equal(got, run(oracle, A, B, 0, 0))


def test_invalid_arguments(oracle):
    a = np.ones(12, np.float32)
    with pytest.raises(ValueError):
        oracle.gemm_f32_raw(-1, 2, 2, a, 0, 0, a, 0, 0)
    with pytest.raises(ValueError):
        oracle.gemm_f32_raw(2, 2, 3, a, 0, 2, a, 0, 0)   # lda < K
    with pytest.raises(ValueError):
        oracle.gemm_f32_raw(2, 2, 3, a, 2, 0, a, 0, 0)   # bad layout flag
    with pytest.raises(ValueError):
        oracle.gemm_at(2, 2, 3, a, 0, 0, a, 0, 0, [2], [0], "f32")  # row out of range
