"""Per-size tuning by measurement (gemm_tune): the paper's exhaustive search per input size (Section 5.3),
run on the device; the recorded pick replaces the cost model's for calls of the same class."""
import numpy as np
import pytest

import gemm_inputs as gi
from gpu_util import to_device

pytestmark = pytest.mark.gpu


def _problem(oracle, dtype, M, N, K, seed):
    A, B = gi.make_problem(seed, M, N, K, "int", dtype)
    exact = oracle.gemm(M, N, K, A, gi.ROW_MAJOR, B, gi.ROW_MAJOR, dtype).astype(np.float32)
    return A, B, exact


@pytest.mark.parametrize("dtype,kind_name", [("f16", "KIND_F16F32"), ("f32", "KIND_F32")])
def test_tune_records_the_measured_pick_and_calls_use_it(oracle, dtype, kind_name, tmp_path):
    import torch
    import paper_2003_06324_amd as g
    kind = getattr(g, kind_name)
    call = g.gemm_f16f32 if dtype == "f16" else g.gemm_f32
    elem = 2 if dtype == "f16" else 4
    stream = torch.cuda.current_stream().cuda_stream
    M, N, K = 520, 264, 1024
    A, B, exact = _problem(oracle, dtype, M, N, K, 4100)
    dA, dB = to_device(gi.store(A, gi.ROW_MAJOR, K)), to_device(gi.store(B, gi.COL_MAJOR, K))
    dC = torch.full((M * N,), float("nan"), dtype=torch.float32, device="cuda")
    g.force_config(None)
    g.tune_clear()
    try:
        pick = g.tune(kind, M, N, K, dA, gi.ROW_MAJOR, 0, dB, gi.COL_MAJOR, 0, dC, gi.ROW_MAJOR, 0, stream)
        torch.cuda.synchronize()
        tile, slices = pick.split(":s")
        assert tile in g.config_names() and 1 <= int(slices) <= 32
        assert np.array_equal(dC.cpu().numpy().reshape(M, N), exact)        # C holds the product afterwards
        # the class of this call now answers with the measured pick, and a plain call runs it
        assert g.query_config(elem, M, N, K, 16, gi.ROW_MAJOR, gi.COL_MAJOR) == pick
        dC.fill_(float("nan"))
        call(M, N, K, dA, gi.ROW_MAJOR, 0, dB, gi.COL_MAJOR, 0, dC, gi.ROW_MAJOR, 0, stream)
        cfg = g.last_config().split()
        assert cfg[1] == tile and cfg[4] == "s" + slices, (cfg, pick)
        torch.cuda.synchronize()
        assert np.array_equal(dC.cpu().numpy().reshape(M, N), exact)
        # it is looked up before the cost model: a distorted model does not change it, forgetting it does
        g.cost_model_scale(g.COST_SLAB, 1000.0)
        assert g.query_config(elem, M, N, K, 16, gi.ROW_MAJOR, gi.COL_MAJOR) == pick
        assert g.query_config(elem, M, N, K, 16, gi.COL_MAJOR, gi.COL_MAJOR) != pick      # another class: the model's answer
        g.tune_clear()
        assert g.query_config(elem, M, N, K, 16, gi.ROW_MAJOR, gi.COL_MAJOR) != pick
        g.cost_model_scale(-1)
        # saved and loaded again, the pick serves the next process's calls
        pick = g.tune(kind, M, N, K, dA, gi.ROW_MAJOR, 0, dB, gi.COL_MAJOR, 0, dC, gi.ROW_MAJOR, 0, stream)
        g.tune_save(tmp_path / "picks.txt")
        g.tune_clear()
        g.tune_load(tmp_path / "picks.txt")
        call(M, N, K, dA, gi.ROW_MAJOR, 0, dB, gi.COL_MAJOR, 0, dC, gi.ROW_MAJOR, 0, stream)
        cfg = g.last_config().split()
        assert cfg[1] + ":" + cfg[4] == pick, (cfg, pick)
        # a forced configuration overrides a recorded pick
        pick = g.tune(kind, M, N, K, dA, gi.ROW_MAJOR, 0, dB, gi.COL_MAJOR, 0, dC, gi.ROW_MAJOR, 0, stream, max_candidates=3)
        g.force_config("t128x128:s2")
        assert g.query_config(elem, M, N, K, 16, gi.ROW_MAJOR, gi.COL_MAJOR) == "t128x128:s2"
    finally:
        g.force_config(None)
        g.cost_model_scale(-1)
        g.tune_clear()


def test_tune_other_entry_points_layouts_and_degenerate_calls(oracle):
    import torch
    import paper_2003_06324_amd as g
    stream = torch.cuda.current_stream().cuda_stream
    g.force_config(None)
    g.tune_clear()
    try:
        # binary16 result, column-major C, operands offset by one element (2-byte aligned class), ragged sizes
        M, N, K = 203, 77, 645
        A, B, _ = _problem(oracle, "f16", M, N, K, 4200)
        exact = oracle.gemm(M, N, K, A, gi.ROW_MAJOR, B, gi.ROW_MAJOR, "f16")
        bufA = np.concatenate([np.full(1, np.nan, A.dtype), gi.store(A, gi.COL_MAJOR, M)])
        dA, dB = to_device(bufA), to_device(gi.store(B, gi.ROW_MAJOR, N))
        dC = torch.full((M * N,), float("nan"), dtype=torch.float16, device="cuda")
        pick = g.tune(g.KIND_F16F16, M, N, K, dA.data_ptr() + 2, gi.COL_MAJOR, 0, dB, gi.ROW_MAJOR, 0, dC, gi.COL_MAJOR, 0,
                      stream, max_candidates=8)
        torch.cuda.synchronize()
        assert pick.split(":s")[0] in g.config_names()
        got = np.array(gi.load(dC.cpu().numpy(), M, N, gi.COL_MAJOR, M))
        assert np.array_equal(got.view(np.uint16), oracle.round_to_half(exact).view(np.uint16))
        # bfloat16 operands
        A, B = gi.make_problem(4300, 96, 160, 512, "int", "bf16")
        exact = oracle.gemm(96, 160, 512, gi.bfloat16_bits(A), 0, gi.bfloat16_bits(B), 0, "bf16").astype(np.float32)
        dA = to_device(gi.bfloat16_bits(gi.store(A, gi.ROW_MAJOR, 512)).view(np.int16))
        dB = to_device(gi.bfloat16_bits(gi.store(B, gi.ROW_MAJOR, 160)).view(np.int16))
        dC = torch.full((96 * 160,), float("nan"), dtype=torch.float32, device="cuda")
        pick = g.tune(g.KIND_BF16F32, 96, 160, 512, dA, gi.ROW_MAJOR, 0, dB, gi.ROW_MAJOR, 0, dC, gi.ROW_MAJOR, 0, stream)
        torch.cuda.synchronize()
        assert np.array_equal(dC.cpu().numpy().reshape(96, 160), exact)
        # nothing to multiply: nothing recorded; K == 0 zero-fills as the entry point does
        assert g.tune(g.KIND_F32, 0, 5, 7, None, 0, 0, dB, 0, 0, None, 0, 0, stream) == "none"
        dZ = torch.full((6,), float("nan"), dtype=torch.float32, device="cuda")
        assert g.tune(g.KIND_F32, 2, 3, 0, None, 0, 0, None, 0, 0, dZ, 0, 0, stream) == "none"
        torch.cuda.synchronize()
        assert np.array_equal(dZ.cpu().numpy(), np.zeros(6, np.float32))
        # errors are the entry point's
        assert g.tune(g.KIND_F32, 2, 2, 2, None, 0, 0, dB, 0, 0, dC, 0, 0, stream, check=False)[0] == -1
        assert g.tune(9, 2, 2, 2, dA, 0, 0, dB, 0, 0, dC, 0, 0, stream, check=False)[0] == -1
        assert g.tune(g.KIND_F32, 2, 2, 2, dA, 0, 0, dB, 0, 0, dC, 0, 0, stream, max_candidates=-1, check=False)[0] == -1
    finally:
        g.tune_clear()
