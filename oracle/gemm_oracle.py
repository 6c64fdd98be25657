"""ctypes front end of the CPU oracle in gemm_oracle.c.

TEST INFRASTRUCTURE ONLY: the tests, the smoke check and the benchmark's
CPU-baseline leg use it; the product never does.  It shares nothing with the
GPU path.

The oracle evaluates the paper's MatMul specification (Section 3.1): for an
M x K matrix A and a K x N matrix B, C(i,j) = sum_k A(i,k) * B(k,j), products
added in ascending k into one float64 accumulator, C overwritten (Section 3.2,
"Epilog": the accumulator starts at zero).  All arithmetic is in the C file;
this module only compiles it with gcc, marshals numpy arrays and returns
float64 results.

Matrices are passed as 1-D or 2-D numpy buffers plus a layout flag
(0 = row-major, 1 = column-major) and a leading dimension; element (r,c) of a
row-major matrix is buffer[r*ld + c], of a column-major one buffer[r + c*ld].
"""
import ctypes
import os
import subprocess

import numpy as np

ROW_MAJOR = 0
COL_MAJOR = 1

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gemm_oracle.c")
_LIB = os.path.join(_HERE, "libgemm_oracle.so")
_lib = None


def build(force=False):
    """Compile gemm_oracle.c into libgemm_oracle.so next to it (gcc, OpenMP)."""
    if not force and os.path.exists(_LIB) and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC):
        return _LIB
    tmp = _LIB + ".tmp%d" % os.getpid()
    cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared",
           "-ffp-contract=off", "-fno-fast-math", "-o", tmp, _SRC, "-lm"]
    subprocess.run(cmd, check=True)
    os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        i64, p, i32 = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int
        full = [i64, i64, i64, p, i32, i64, p, i32, i64, p, i32, i64]
        samp = [i64, i64, i64, p, i32, i64, p, i32, i64, i64, p, p, p]
        for name, sig in (("oracle_gemm_f32", full), ("oracle_gemm_f16", full), ("oracle_gemm_bf16", full),
                          ("oracle_gemm_f32_at", samp), ("oracle_gemm_f16_at", samp),
                          ("oracle_gemm_bf16_at", samp)):
            fn = getattr(lib, name)
            fn.argtypes = sig
            fn.restype = i32
        lib.oracle_half_bits_to_double.argtypes = [ctypes.c_uint16]
        lib.oracle_half_bits_to_double.restype = ctypes.c_double
        lib.oracle_bfloat16_bits_to_double.argtypes = [ctypes.c_uint16]
        lib.oracle_bfloat16_bits_to_double.restype = ctypes.c_double
        lib.oracle_num_threads.restype = i32
        lib.oracle_double_to_half_bits.argtypes = [ctypes.c_double]
        lib.oracle_double_to_half_bits.restype = ctypes.c_uint16
        lib.oracle_round_to_half.argtypes = [i64, p, p]
        lib.oracle_round_to_half.restype = i32
        _lib = lib
    return _lib


def num_threads():
    return int(_load().oracle_num_threads())


def half_bits_to_double(bits):
    return float(_load().oracle_half_bits_to_double(int(bits) & 0xFFFF))


def bfloat16_bits_to_double(bits):
    return float(_load().oracle_bfloat16_bits_to_double(int(bits) & 0xFFFF))


def double_to_half_bits(value):
    """Binary16 pattern of one float64, rounded to nearest even."""
    return int(_load().oracle_double_to_half_bits(float(value)))


def round_to_half(values):
    """Binary16 (numpy float16 array, same shape) of a float64 array, each element rounded once
    to nearest even: what the binary16-output entry point stores for an exact sum."""
    v = np.ascontiguousarray(values, dtype=np.float64)
    out = np.zeros(max(v.size, 1), dtype=np.uint16)
    if _load().oracle_round_to_half(v.size, v.ctypes.data, out.ctypes.data) != 0:
        raise ValueError("oracle_round_to_half rejected its arguments")
    return out[:v.size].view(np.float16).reshape(v.shape)


def _packed_ld(layout, rows, cols):
    return cols if layout == ROW_MAJOR else rows


def _min_len(layout, ld, rows, cols):
    if rows == 0 or cols == 0:
        return 0
    return (rows - 1) * ld + cols if layout == ROW_MAJOR else (cols - 1) * ld + rows


def _operand(buf, dtype, layout, ld, rows, cols):
    buf = np.ascontiguousarray(buf).reshape(-1)
    if buf.dtype == np.float16 and dtype == np.uint16:
        buf = buf.view(np.uint16)
    if buf.dtype != dtype:
        raise TypeError("expected %s buffer, got %s" % (np.dtype(dtype), buf.dtype))
    if ld == 0:
        ld = _packed_ld(layout, rows, cols)
    if ld >= _packed_ld(layout, rows, cols) and buf.size < _min_len(layout, ld, rows, cols):
        raise ValueError("buffer too small for the stated shape")
    return buf, ld


def _gemm(fn_name, dtype, M, N, K, A, layoutA, lda, B, layoutB, ldb, layoutC, ldc):
    lib = _load()
    A, lda = _operand(A, dtype, layoutA, lda, M, K)
    B, ldb = _operand(B, dtype, layoutB, ldb, K, N)
    if ldc == 0:
        ldc = _packed_ld(layoutC, M, N)
    n_out = max(_min_len(layoutC, ldc, M, N), 0) if ldc >= _packed_ld(layoutC, M, N) else 0
    C = np.full(max(n_out, 1), np.nan, dtype=np.float64)
    rc = getattr(lib, fn_name)(M, N, K, A.ctypes.data, layoutA, lda, B.ctypes.data, layoutB, ldb,
                               C.ctypes.data, layoutC, ldc)
    if rc != 0:
        raise ValueError("%s rejected its arguments (rc=%d)" % (fn_name, rc))
    return C[:n_out], ldc


def gemm_f32_raw(M, N, K, A, layoutA, lda, B, layoutB, ldb, layoutC=ROW_MAJOR, ldc=0):
    """Float32 operands; returns (flat float64 C buffer in layoutC with ldc, ldc)."""
    return _gemm("oracle_gemm_f32", np.float32, M, N, K, A, layoutA, lda, B, layoutB, ldb, layoutC, ldc)


def gemm_f16_raw(M, N, K, A, layoutA, lda, B, layoutB, ldb, layoutC=ROW_MAJOR, ldc=0):
    """Binary16 operands (uint16 bit patterns or float16 arrays); float64 result."""
    return _gemm("oracle_gemm_f16", np.uint16, M, N, K, A, layoutA, lda, B, layoutB, ldb, layoutC, ldc)


def gemm_bf16_raw(M, N, K, A, layoutA, lda, B, layoutB, ldb, layoutC=ROW_MAJOR, ldc=0):
    """bfloat16 operands (uint16 bit patterns); float64 result."""
    return _gemm("oracle_gemm_bf16", np.uint16, M, N, K, A, layoutA, lda, B, layoutB, ldb, layoutC, ldc)


def gemm(M, N, K, A, layoutA, B, layoutB, dtype):
    """Packed operands -> logical M x N float64 array. dtype is 'f32', 'f16' or 'bf16'
    (bf16: uint16 bit patterns)."""
    fn = {"f32": gemm_f32_raw, "f16": gemm_f16_raw, "bf16": gemm_bf16_raw}[dtype]
    C, _ = fn(M, N, K, A, layoutA, 0, B, layoutB, 0, ROW_MAJOR, 0)
    return C.reshape(M, N)


def gemm_at(M, N, K, A, layoutA, lda, B, layoutB, ldb, rows, cols, dtype):
    """Same definition evaluated only at positions (rows[t], cols[t]); float64 vector."""
    lib = _load()
    npdt = np.float32 if dtype == "f32" else np.uint16
    A, lda = _operand(A, npdt, layoutA, lda, M, K)
    B, ldb = _operand(B, npdt, layoutB, ldb, K, N)
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    cols = np.ascontiguousarray(cols, dtype=np.int64)
    out = np.full(max(rows.size, 1), np.nan, dtype=np.float64)
    fn = {"f32": lib.oracle_gemm_f32_at, "f16": lib.oracle_gemm_f16_at, "bf16": lib.oracle_gemm_bf16_at}[dtype]
    rc = fn(M, N, K, A.ctypes.data, layoutA, lda, B.ctypes.data, layoutB, ldb,
            rows.size, rows.ctypes.data, cols.ctypes.data, out.ctypes.data)
    if rc != 0:
        raise ValueError("oracle sample call rejected its arguments (rc=%d)" % rc)
    return out[:rows.size]
