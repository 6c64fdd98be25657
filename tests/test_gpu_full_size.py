"""Parity at the full benchmark sizes, in the launch configuration bench.py times (automatic
tile selection, packed operands, row-major C).  Where the oracle cannot do the whole product in
seconds, sampled entries are compared one by one and, on integer-valued inputs, exact row and
column sums of C (which involve every entry) are checked against int64 arithmetic."""
import numpy as np
import pytest

import gemm_inputs as gi
from gpu_util import TIGHT, TOL, check, run_gpu

pytestmark = pytest.mark.gpu


def sample_positions(M, N, n, seed):
    """Random positions plus tile corners and matrix edges (256-, 128- and 64-tiles)."""
    rng = np.random.default_rng(seed)
    rows = list(rng.integers(0, M, size=n))
    cols = list(rng.integers(0, N, size=n))
    edge_r = sorted({0, M - 1, *[r for t in (64, 128, 256) for r in (t - 1, t, M - t, M - t - 1) if 0 <= r < M]})
    edge_c = sorted({0, N - 1, *[c for t in (64, 128, 256) for c in (t - 1, t, N - t, N - t - 1) if 0 <= c < N]})
    for r in edge_r:
        for c in edge_c:
            rows.append(r)
            cols.append(c)
    return np.array(rows, np.int64), np.array(cols, np.int64)


def check_sampled(oracle, C, A, B, dtype, seed, n=3000):
    M, K = A.shape
    N = B.shape[1]
    rows, cols = sample_positions(M, N, n, seed)
    ref = oracle.gemm_at(M, N, K, gi.store(A, gi.ROW_MAJOR), gi.ROW_MAJOR, 0,
                         gi.store(B, gi.COL_MAJOR), gi.COL_MAJOR, 0, rows, cols, dtype)
    got = C[rows, cols].astype(np.float64)
    assert np.all(np.isfinite(C))
    a64, b64 = np.abs(A.astype(np.float64)), np.abs(B.astype(np.float64))
    diff = np.max(np.abs(got - ref))
    stated = diff / (K * a64.max() * b64.max())
    tight = diff / (K * np.sqrt(np.mean(a64 ** 2)) * np.sqrt(np.mean(b64 ** 2)))
    assert stated <= TOL[dtype], stated
    assert tight <= TIGHT[dtype], tight


def check_integer_sums(C, A, B):
    """Integer-valued operands: every entry of C is an exact integer below 2^24, so row and
    column sums taken in float64 must equal the int64 values A (B 1) and (1^T A) B."""
    Ai, Bi = A.astype(np.int64), B.astype(np.int64)
    C64 = C.astype(np.float64)
    assert np.array_equal(C64.sum(axis=1), (Ai @ Bi.sum(axis=1)).astype(np.float64))
    assert np.array_equal(C64.sum(axis=0), (Ai.sum(axis=0) @ Bi).astype(np.float64))
    # weighted sums catch a pair of swapped entries inside one row or column
    w = (np.arange(C.shape[1]) % 7 + 1).astype(np.int64)
    assert np.array_equal(C64 @ w.astype(np.float64), (Ai @ (Bi @ w)).astype(np.float64))


@pytest.fixture(scope="module")
def f16_8192(request):
    A, B = gi.make_problem(3000, 8192, 8192, 8192, "normal", "f16")
    Ai, Bi = gi.make_problem(3001, 8192, 8192, 8192, "int", "f16")
    return A, B, Ai, Bi


@pytest.mark.parametrize("layout", ["NN", "NT", "TN", "TT"])
def test_f16_8192_all_layouts(oracle, f16_8192, layout):
    A, B, Ai, Bi = f16_8192
    la, lb = gi.LAYOUTS[layout]
    C, cfg = run_gpu("f16", A, B, la, lb, return_config=True)
    assert "aligned" in cfg
    check_sampled(oracle, C, A, B, "f16", seed=31)
    C = run_gpu("f16", Ai, Bi, la, lb)
    check_integer_sums(C, Ai, Bi)
    rows, cols = sample_positions(8192, 8192, 500, 5)
    ref = oracle.gemm_at(8192, 8192, 8192, gi.store(Ai, 0), 0, 0, gi.store(Bi, 0), 0, 0, rows, cols, "f16")
    assert np.array_equal(C[rows, cols].astype(np.float64), ref)


def test_f32_4096_nt(oracle):
    cfg, A, B, _, _ = gi.config_problem("f32_4096_nt")
    C = run_gpu("f32", A, B, gi.ROW_MAJOR, gi.COL_MAJOR)
    check_sampled(oracle, C, A, B, "f32", seed=32)
    Ai, Bi = gi.make_problem(2001, 4096, 4096, 4096, "int", "f32")
    C = run_gpu("f32", Ai, Bi, gi.ROW_MAJOR, gi.COL_MAJOR)
    check_integer_sums(C, Ai, Bi)


def test_f32_256_nn_seed0(oracle):
    cfg, A, B, _, _ = gi.config_problem("f32_256_nn")
    ref = oracle.gemm(256, 256, 256, A, 0, B, 0, "f32")
    check(run_gpu("f32", A, B, 0, 0), ref, A, B, "f32", "f32 256^3")


@pytest.mark.parametrize("name", ["f16_edge_a", "f16_edge_b", "f16_skinny_n", "f16_skinny_m"])
def test_f16_edge_and_skinny_full_compare(oracle, name):
    cfg, A, B, _, _ = gi.config_problem(name)
    la, lb = gi.LAYOUTS[cfg["layout"]]
    ref = oracle.gemm(cfg["M"], cfg["N"], cfg["K"], A, 0, B, 0, "f16")
    C = run_gpu("f16", A, B, la, lb)
    check(C, ref, A, B, "f16", name)
    _, Ai, Bi, _, _ = gi.config_problem(name, dist="int")
    refi = oracle.gemm(cfg["M"], cfg["N"], cfg["K"], Ai, 0, Bi, 0, "f16").astype(np.float32)
    assert np.array_equal(run_gpu("f16", Ai, Bi, la, lb), refi), name


def test_f16_deep_k(oracle):
    cfg, A, B, _, _ = gi.config_problem("f16_deep_k")
    la, lb = gi.LAYOUTS[cfg["layout"]]
    C = run_gpu("f16", A, B, la, lb)
    check_sampled(oracle, C, A, B, "f16", seed=33, n=1500)
    _, Ai, Bi, _, _ = gi.config_problem("f16_deep_k", dist="int")
    C = run_gpu("f16", Ai, Bi, la, lb)
    check_integer_sums(C, Ai, Bi)


# Sizes the paper itself evaluates (Section 5: the 1536 x 1024 x 2048 "NT" case of its first
# experiment, and powers of two from the small (<= 1024) and large (1024..4096) ranges of its
# last one), with the automatic tile selection.
PAPER_SHAPES = [("f16", 1536, 1024, 2048, "NT"), ("f16", 256, 256, 256, "NT"), ("f16", 512, 1024, 256, "TN"),
                ("f16", 1024, 1024, 1024, "NN"), ("f16", 2048, 1024, 4096, "TT"), ("f32", 1024, 512, 2048, "NT"),
                ("f32", 512, 512, 512, "TN")]


@pytest.mark.parametrize("case", PAPER_SHAPES, ids=lambda c: "%s_%dx%dx%d_%s" % c)
def test_paper_sizes(oracle, case):
    dtype, M, N, K, layout = case
    la, lb = gi.LAYOUTS[layout]
    A, B = gi.make_problem(600 + M + N + K, M, N, K, "uniform", dtype)
    ref = oracle.gemm(M, N, K, A, 0, B, 0, dtype)
    check(run_gpu(dtype, A, B, la, lb), ref, A, B, dtype, str(case))
    Ai, Bi = gi.make_problem(601 + M + N + K, M, N, K, "int", dtype)
    refi = oracle.gemm(M, N, K, Ai, 0, Bi, 0, dtype).astype(np.float32)
    assert np.array_equal(run_gpu(dtype, Ai, Bi, la, lb), refi), case


def test_c_beyond_4_gib(oracle):
    # C of 33000 x 33000 binary32 is 4.36 GB: row offsets into C cross 2^32 bytes.  Integer-valued
    # operands, so sampled entries (also in the last rows) must match the oracle exactly.
    import torch
    import paper_2003_06324_amd as g
    M = N = 33000
    K = 64
    A, B = gi.make_problem(61, M, N, K, "int", "f16")
    dA = torch.from_numpy(A.view(np.int16)).cuda()
    dB = torch.from_numpy(np.ascontiguousarray(B.T).view(np.int16)).cuda()
    dC = torch.full((M * N,), float("nan"), dtype=torch.float32, device="cuda")
    g.gemm_f16f32(M, N, K, dA, gi.ROW_MAJOR, 0, dB, gi.COL_MAJOR, 0, dC, gi.ROW_MAJOR, 0,
                  torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    rows, cols = sample_positions(M, N, 4000, 3)
    ref = oracle.gemm_at(M, N, K, gi.store(A, gi.ROW_MAJOR), gi.ROW_MAJOR, 0,
                         gi.store(B, gi.COL_MAJOR), gi.COL_MAJOR, 0, rows, cols, "f16")
    idx = torch.from_numpy(rows * N + cols).cuda()
    got = dC[idx].cpu().numpy()
    assert np.array_equal(got, ref.astype(np.float32))
    # every row and column sum of the whole of C, exact in int64 (sums of |C| stay far below 2^53)
    Ai, Bi = A.astype(np.int64), B.astype(np.int64)
    C2 = dC.view(M, N)
    assert np.array_equal(C2.sum(dim=1, dtype=torch.float64).cpu().numpy(), (Ai @ Bi.sum(axis=1)).astype(np.float64))
    assert np.array_equal(C2.sum(dim=0, dtype=torch.float64).cpu().numpy(), (Ai.sum(axis=0) @ Bi).astype(np.float64))


def test_operand_beyond_4_gib(oracle):
    # A of 66000 x 32768 binary16 is 4.33 GB: tile origins in A lie beyond 2^32 bytes
    # (a formula instead of the seeded generator keeps the host side to a few seconds)
    import torch
    import paper_2003_06324_amd as g
    M, N, K = 66000, 72, 32768
    i = np.arange(M, dtype=np.int32)[:, None]
    k = np.arange(K, dtype=np.int32)[None, :]
    A = (((i * 7 + k * 3) % 9) - 4).astype(np.float16)
    B = ((np.arange(K)[:, None] * 5 + np.arange(N)[None, :] * 11) % 7 - 3).astype(np.float16)
    dA = torch.from_numpy(A.view(np.int16)).cuda()
    dB = torch.from_numpy(np.ascontiguousarray(B.T).view(np.int16)).cuda()
    rows, cols = sample_positions(M, N, 1500, 4)
    ref = oracle.gemm_at(M, N, K, A.reshape(-1), gi.ROW_MAJOR, 0, gi.store(B, gi.COL_MAJOR), gi.COL_MAJOR, 0,
                         rows, cols, "f16").astype(np.float32)
    stream = torch.cuda.current_stream().cuda_stream
    for force in (None, "t256x256:s1", "t64x64:s2"):
        dC = torch.full((M * N,), float("nan"), dtype=torch.float32, device="cuda")
        g.force_config(force)
        try:
            g.gemm_f16f32(M, N, K, dA, gi.ROW_MAJOR, 0, dB, gi.COL_MAJOR, 0, dC, gi.ROW_MAJOR, 0, stream)
            cfg = g.last_config()
        finally:
            g.force_config(None)
        torch.cuda.synchronize()
        C = dC.cpu().numpy().reshape(M, N)
        assert np.array_equal(C[rows, cols], ref), cfg
        # exact column sums of the whole of C in int64
        col_sums = A.sum(axis=0, dtype=np.float64).astype(np.int64) @ B.astype(np.int64)   # |sums| < 2^53: exact
        assert np.array_equal(C.sum(axis=0, dtype=np.float64), col_sums.astype(np.float64)), cfg


# ---------------------------------------------------------------------------
# Every element at full size: one complete oracle product per case (tens of seconds on the
# GPU machine's cores), compared with all of C at both bars.
# ---------------------------------------------------------------------------
def test_f16_8192_every_element_all_layouts(oracle, f16_8192):
    A, B, _, _ = f16_8192
    ref = oracle.gemm(8192, 8192, 8192, A, gi.ROW_MAJOR, B, gi.ROW_MAJOR, "f16")
    for layout in ("NN", "NT", "TN", "TT"):
        la, lb = gi.LAYOUTS[layout]
        C = run_gpu("f16", A, B, la, lb)
        check(C, ref, A, B, "f16", "f16 8192^3 %s, every element" % layout)


def test_f32_4096_nt_every_element(oracle):
    cfg, A, B, _, _ = gi.config_problem("f32_4096_nt")
    ref = oracle.gemm(4096, 4096, 4096, A, gi.ROW_MAJOR, B, gi.ROW_MAJOR, "f32")
    check(run_gpu("f32", A, B, gi.ROW_MAJOR, gi.COL_MAJOR), ref, A, B, "f32", "f32 4096^3 NT, every element")


def test_f16_deep_k_every_element(oracle):
    cfg, A, B, _, _ = gi.config_problem("f16_deep_k")
    la, lb = gi.LAYOUTS[cfg["layout"]]
    ref = oracle.gemm(cfg["M"], cfg["N"], cfg["K"], A, gi.ROW_MAJOR, B, gi.ROW_MAJOR, "f16")
    check(run_gpu("f16", A, B, la, lb), ref, A, B, "f16", "f16 1024x1024x65536, every element")
