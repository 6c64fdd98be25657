"""Subnormal numbers go through the matrix instructions unflushed: operands below the normal
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
