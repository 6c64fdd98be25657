"""MI355X-native dense GEMM (C = A*B): thin Python binding of the C-ABI library.

Everything is computed by the HIP kernels in csrc/; this package only loads
libgemm_mi355x.so and marshals arguments.  There is no CPU fallback: if the
library cannot be loaded, calls raise.
"""
from .gemm import (COL_MAJOR, COST_FIXED, COST_HBM, COST_L2, COST_SLAB, ROW_MAJOR, GemmError, config_names, cost_model_scale, force_config, gemm_bf16f32,
                   gemm_f16f16, gemm_f16f32, gemm_f16f32_noalloc, gemm_f32, NOALLOC_SCRATCH_BYTES, last_config, library_path, query_config, set_phase_trace, load_library, shutdown, status_string,
                   tune, tune_clear, tune_save, tune_load, load_tuned_table, TUNED_TABLE, KIND_F32, KIND_F16F32, KIND_F16F16, KIND_BF16F32)

__all__ = ["ROW_MAJOR", "COL_MAJOR", "GemmError", "gemm_f32", "gemm_f16f32", "gemm_f16f16", "gemm_bf16f32", "gemm_f16f32_noalloc", "NOALLOC_SCRATCH_BYTES", "force_config",
           "config_names", "query_config", "set_phase_trace", "cost_model_scale", "COST_SLAB", "COST_HBM", "COST_L2", "COST_FIXED", "last_config", "status_string", "shutdown", "load_library",
           "library_path", "tune", "tune_clear", "tune_save", "tune_load", "load_tuned_table", "TUNED_TABLE", "KIND_F32", "KIND_F16F32", "KIND_F16F16", "KIND_BF16F32"]
