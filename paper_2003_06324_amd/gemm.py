"""ctypes binding of include/gemm.h.  Argument marshalling only.

The functions take raw device addresses (ints), or any object exposing
``data_ptr()`` (a torch tensor) -- torch is used by callers purely to own
device memory and streams.  Names and argument order follow the C header.
"""
import ctypes
import os

ROW_MAJOR = 0
COL_MAJOR = 1

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libgemm_mi355x.so")
_lib = None

EXPORTS = ("gemm_f32", "gemm_f16f32", "gemm_f16f16", "gemm_bf16f32", "gemm_f16f32_noalloc", "gemm_cost_model_scale", "gemm_set_phase_trace", "gemm_force_config", "gemm_query_config", "gemm_query_config_layouts", "gemm_tune", "gemm_tune_clear", "gemm_tune_save", "gemm_tune_load", "gemm_num_configs", "gemm_config_name",
           "gemm_last_config", "gemm_status_string", "gemm_shutdown")


class GemmError(RuntimeError):
    def __init__(self, status, text):
        super().__init__("gemm call failed: %s (status %d)" % (text, status))
        self.status = status


def library_path():
    return _LIB_PATH


def load_library():
    """Load libgemm_mi355x.so (building it first only if no built library exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        from . import build as _build
        _build.build()
    # One HIP runtime per process: PyTorch ships its own libamdhip64 under the same soname
    # as the system one.  Importing torch first makes this library bind to the runtime
    # that owns the caller's tensors and streams, whatever the import order.
    try:
        import torch  # noqa: F401
    except ImportError:
        pass
    lib = ctypes.CDLL(_LIB_PATH)
    i64, i32, p = ctypes.c_int64, ctypes.c_int, ctypes.c_void_p
    sig = [i64, i64, i64, p, i32, i64, p, i32, i64, p, i32, i64, p]
    for name in ("gemm_f32", "gemm_f16f32", "gemm_f16f16", "gemm_bf16f32", "gemm_f16f32_noalloc"):
        fn = getattr(lib, name)
        fn.argtypes = sig
        fn.restype = i32
    lib.gemm_force_config.argtypes = [ctypes.c_char_p]
    lib.gemm_force_config.restype = i32
    lib.gemm_set_phase_trace.argtypes = [p, i64]
    lib.gemm_set_phase_trace.restype = i32
    lib.gemm_cost_model_scale.argtypes = [i32, ctypes.c_double]
    lib.gemm_cost_model_scale.restype = i32
    lib.gemm_query_config.argtypes = [i32, i64, i64, i64, i32, ctypes.c_char_p, i32]
    lib.gemm_query_config.restype = i32
    lib.gemm_query_config_layouts.argtypes = [i32, i64, i64, i64, i32, i32, i32, ctypes.c_char_p, i32]
    lib.gemm_query_config_layouts.restype = i32
    lib.gemm_tune.argtypes = [i32, i64, i64, i64, ctypes.c_void_p, i32, i64, ctypes.c_void_p, i32, i64, ctypes.c_void_p, i32, i64,
                              ctypes.c_void_p, i32, ctypes.c_char_p, i32]
    lib.gemm_tune.restype = i32
    lib.gemm_tune_clear.argtypes = []
    lib.gemm_tune_clear.restype = i32
    lib.gemm_tune_save.argtypes = [ctypes.c_char_p]
    lib.gemm_tune_save.restype = i32
    lib.gemm_tune_load.argtypes = [ctypes.c_char_p]
    lib.gemm_tune_load.restype = i32
    lib.gemm_num_configs.argtypes = []
    lib.gemm_num_configs.restype = i32
    lib.gemm_config_name.argtypes = [i32]
    lib.gemm_config_name.restype = ctypes.c_char_p
    lib.gemm_last_config.argtypes = []
    lib.gemm_last_config.restype = ctypes.c_char_p
    lib.gemm_status_string.argtypes = [i32]
    lib.gemm_status_string.restype = ctypes.c_char_p
    lib.gemm_shutdown.argtypes = []
    lib.gemm_shutdown.restype = i32
    _lib = lib
    return lib


def _ptr(x):
    if x is None:
        return None
    if hasattr(x, "data_ptr"):
        return x.data_ptr() or None
    return int(x) or None


def status_string(status):
    return load_library().gemm_status_string(int(status)).decode()


def _check(status):
    if status != 0:
        raise GemmError(status, status_string(status))
    return status


def gemm_f32(M, N, K, A, layoutA, lda, B, layoutB, ldb, C, layoutC, ldc, stream=None, check=True):
    """C = A*B, binary32. A, B, C: device addresses or tensors; stream: hipStream_t as int."""
    rc = load_library().gemm_f32(M, N, K, _ptr(A), layoutA, lda, _ptr(B), layoutB, ldb,
                                 _ptr(C), layoutC, ldc, stream or None)
    return _check(rc) if check else rc


def gemm_f16f32(M, N, K, A, layoutA, lda, B, layoutB, ldb, C, layoutC, ldc, stream=None, check=True):
    """C = A*B, binary16 operands, binary32 accumulation and result."""
    rc = load_library().gemm_f16f32(M, N, K, _ptr(A), layoutA, lda, _ptr(B), layoutB, ldb,
                                    _ptr(C), layoutC, ldc, stream or None)
    return _check(rc) if check else rc


def gemm_f16f16(M, N, K, A, layoutA, lda, B, layoutB, ldb, C, layoutC, ldc, stream=None, check=True):
    """C = A*B, binary16 operands, binary32 accumulation, C rounded to binary16 (16-bit patterns)."""
    rc = load_library().gemm_f16f16(M, N, K, _ptr(A), layoutA, lda, _ptr(B), layoutB, ldb,
                                    _ptr(C), layoutC, ldc, stream or None)
    return _check(rc) if check else rc


def gemm_bf16f32(M, N, K, A, layoutA, lda, B, layoutB, ldb, C, layoutC, ldc, stream=None, check=True):
    """C = A*B, bfloat16 operands (16-bit patterns), binary32 accumulation and result."""
    rc = load_library().gemm_bf16f32(M, N, K, _ptr(A), layoutA, lda, _ptr(B), layoutB, ldb,
                                     _ptr(C), layoutC, ldc, stream or None)
    return _check(rc) if check else rc


def gemm_f16f32_noalloc(M, N, K, A, layoutA, lda, B, layoutB, ldb, C, layoutC, ldc, stream=None, check=True):
    """gemm_f16f32 that never allocates: K-slice partials go to the library's fixed per-GPU array."""
    rc = load_library().gemm_f16f32_noalloc(M, N, K, _ptr(A), layoutA, lda, _ptr(B), layoutB, ldb,
                                            _ptr(C), layoutC, ldc, stream or None)
    return _check(rc) if check else rc


NOALLOC_SCRATCH_BYTES = 64 << 20
COST_SLAB, COST_HBM, COST_L2, COST_FIXED = 0, 1, 2, 3


def cost_model_scale(term, factor=1.0, check=True):
    """Multiply one term of the selection's cost model by factor; term < 0 resets all terms."""
    rc = load_library().gemm_cost_model_scale(int(term), float(factor))
    return _check(rc) if check else rc


def set_phase_trace(buffer=None, workgroups=0):
    """Device buffer of 8 * workgroups uint64 that the kernels fill with per-workgroup phase
    timestamps (see include/gemm.h); None switches the trace off."""
    return _check(load_library().gemm_set_phase_trace(_ptr(buffer), int(workgroups)))


KIND_F32, KIND_F16F32, KIND_F16F16, KIND_BF16F32 = 0, 1, 2, 3


def tune(kind, M, N, K, A, layoutA, lda, B, layoutB, ldb, C, layoutC, ldc, stream=None, max_candidates=0, check=True):
    """Times the candidate configurations for this call (kind: KIND_*, the other arguments as that entry point's),
    records the fastest for later calls of the same class and returns it as "<tile>:s<slices>".  Blocks the host.
    With check=False returns (status, text)."""
    buf = ctypes.create_string_buffer(64)
    rc = load_library().gemm_tune(kind, M, N, K, _ptr(A), layoutA, lda, _ptr(B), layoutB, ldb, _ptr(C), layoutC, ldc,
                                  stream or None, max_candidates, buf, 64)
    if check:
        _check(rc)
        return buf.value.decode()
    return rc, buf.value.decode()


def tune_clear():
    return _check(load_library().gemm_tune_clear())


def tune_save(path, check=True):
    """Writes the picks gemm_tune has recorded to a text file."""
    rc = load_library().gemm_tune_save(str(path).encode())
    return _check(rc) if check else rc


TUNED_TABLE = os.path.join(os.path.dirname(os.path.abspath(__file__)), "tuned_mi355x.txt")


def load_tuned_table():
    """Loads the picks measured on an MI355X over the paper's size ranges (M, N, K powers of two from 256 to 4096,
    16-byte aligned operands; written by tune_paper_ranges.py).  Not loaded by default: the cost model answers unless
    the caller asks for the measured table."""
    return tune_load(TUNED_TABLE)


def tune_load(path, check=True):
    """Adds the picks of a file written by tune_save to the table."""
    rc = load_library().gemm_tune_load(str(path).encode())
    return _check(rc) if check else rc


def query_config(elem_bytes, M, N, K, aligned=True, layout_a=None, layout_b=None):
    """The "<tile>:s<splits>" the selection picks for this shape (host only, nothing is launched).
    aligned: True / False, or the common alignment of bases and leading dimensions in bytes.
    layout_a, layout_b: ROW_MAJOR / COL_MAJOR of A (M x K) and B (K x N); both row-major if not given."""
    buf = ctypes.create_string_buffer(64)
    lib = load_library()
    if layout_a is None and layout_b is None:
        _check(lib.gemm_query_config(elem_bytes, M, N, K, int(aligned), buf, 64))
    else:
        _check(lib.gemm_query_config_layouts(elem_bytes, M, N, K, int(aligned), ROW_MAJOR if layout_a is None else layout_a,
                                             ROW_MAJOR if layout_b is None else layout_b, buf, 64))
    return buf.value.decode()


def force_config(name=None, check=True):
    rc = load_library().gemm_force_config(name.encode() if name else None)
    return _check(rc) if check else rc


def config_names():
    lib = load_library()
    return [lib.gemm_config_name(i).decode() for i in range(lib.gemm_num_configs())]


def last_config():
    return load_library().gemm_last_config().decode()


def shutdown():
    return _check(load_library().gemm_shutdown())
