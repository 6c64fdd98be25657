"""Special values.  NaN and infinity in A or B reach exactly the entries of C whose sums contain
them (and nothing from padding or neighbouring tiles does); subnormal numbers go through the
matrix instructions unflushed: operands below the normal
range of binary16, bfloat16 and binary32, and binary32 results below 2^-126, equal the oracle's
exact sums (all sums here are exact in binary32, so the comparison is bit for bit)."""
import numpy as np
import pytest

import gemm_inputs as gi
from gpu_util import run_gpu

pytestmark = pytest.mark.gpu


def oracle_c(oracle, A, B, dtype):
    M, K = A.shape
    if dtype == "bf16":
        return oracle.gemm(M, B.shape[1], K, gi.bfloat16_bits(A), 0, gi.bfloat16_bits(B), 0, "bf16")
    return oracle.gemm(M, B.shape[1], K, A, 0, B, 0, dtype)


@pytest.mark.parametrize("case", [
    ("f16", 2.0 ** -24, 1024.0, np.float16),          # smallest binary16 subnormal times a normal number
    ("f16", 3 * 2.0 ** -24, 5 * 2.0 ** -24, np.float16),  # subnormal times subnormal
    ("f32", 2.0 ** -130, 4.0, np.float32),            # binary32 subnormal operand and result
    ("f32", 2.0 ** -70, 2.0 ** -70, np.float32),      # normal operands, subnormal result
    ("bf16", 2.0 ** -130, 2.0 ** 20, np.float32),     # bfloat16 subnormal operand
])
def test_subnormals_are_not_flushed(oracle, case):
    dtype, a, b, npdt = case
    rng = np.random.default_rng(3)
    M, N, K = 70, 66, 96
    A = (rng.integers(1, 4, size=(M, K)) * a).astype(npdt)
    B = (rng.integers(-3, 4, size=(K, N)) * b).astype(npdt)
    ref = oracle_c(oracle, A, B, dtype)
    assert np.any(ref != 0) and np.array_equal(ref.astype(np.float32).astype(np.float64), ref)
    for la, lb in ((0, 0), (0, 1), (1, 0), (1, 1)):
        C = run_gpu(dtype, A, B, la, lb)
        assert np.array_equal(C.astype(np.float64), ref), (case, la, lb)


@pytest.mark.parametrize("dtype", ["f16", "f32", "bf16"])
def test_nan_and_infinity_reach_their_row_and_column_only(oracle, dtype):
    M, N, K = 300, 280, 200
    A, B = gi.make_problem(77, M, N, K, "uniform", dtype)
    A, B = A.copy(), B.copy()
    A[17, 5] = np.nan          # row 17 of C becomes NaN
    A[200, 199] = np.inf       # row 200: +-inf by the sign of B(199, j)
    B[64, 130] = -np.inf       # column 130: -+inf by the sign of A(i, 64)
    B[0, 279] = np.nan         # column 279 becomes NaN
    ref = oracle_c(oracle, A, B, dtype)
    assert np.isnan(ref[17]).all() and np.isnan(ref[:, 279]).all() and np.isinf(ref[200, :130]).all()
    finite = np.isfinite(ref)
    assert finite.sum() == (M - 2) * (N - 2)
    for la, lb in ((0, 0), (0, 1), (1, 0), (1, 1)):
        for force in (None, "t256x256", "t64x64:s3"):
            C = run_gpu(dtype, A, B, la, lb, force=force).astype(np.float64)
            assert np.array_equal(np.isnan(C), np.isnan(ref)), (dtype, la, lb, force)
            assert np.array_equal(np.isinf(C), np.isinf(ref)) and np.array_equal(C[np.isinf(ref)], ref[np.isinf(ref)])
            assert np.max(np.abs(C[finite] - ref[finite])) <= K * 8 * 2.0 ** -24
