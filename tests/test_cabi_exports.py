"""The C-ABI library loads and exports every symbol include/gemm.h declares (no GPU needed)."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "gemm.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(gemm_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    from paper_2003_06324_amd import gemm
    lib = gemm.load_library()
    names = declared_functions()
    assert set(gemm.EXPORTS) == set(names), (gemm.EXPORTS, names)
    for name in names:
        assert isinstance(getattr(lib, name), ctypes._CFuncPtr)


def test_host_only_entry_points():
    import paper_2003_06324_amd as g
    assert g.status_string(0) == "ok"
    assert "invalid" in g.status_string(-1)
    names = g.config_names()
    assert names and all(n.startswith("t") for n in names)
    for n in names:
        assert g.force_config(n) == 0
        assert g.force_config(n + ":s4") == 0
    assert g.force_config("nope", check=False) == -3
    assert g.force_config("t64x64:x2", check=False) == -3
    assert g.force_config(None) == 0
    # argument validation happens before any device work
    assert g.gemm_f32(-1, 1, 1, 16, 0, 0, 16, 0, 0, 16, 0, 0, check=False) == -1
    assert g.gemm_f16f32(2, 2, 2, 16, 0, 1, 16, 0, 0, 16, 0, 0, check=False) == -1
    assert g.gemm_f16f32(2, 2, 2, 16, 0, 0, 16, 3, 0, 16, 0, 0, check=False) == -1
    assert g.gemm_f32(2, 2, 2, None, 0, 0, 16, 0, 0, 16, 0, 0, check=False) == -1
    assert g.gemm_f32(2 ** 31, 1, 1, 16, 0, 0, 16, 0, 0, 16, 0, 0, check=False) == -3
    assert g.gemm_f32(0, 0, 5, None, 0, 0, None, 0, 0, None, 0, 0) == 0
