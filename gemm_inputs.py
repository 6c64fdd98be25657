"""Seeded synthetic inputs for dense GEMM tests and benchmarks.

Holds no GEMM arithmetic: it only draws random matrices and lays them out in
memory.  Both the CPU oracle's tests and the GPU library's tests take their
operands from here, so the two sides see the same bits.

The paper's workload is random dense matrices of a given size (Section 5
evaluates square and rectangular sizes up to 4096 with half and single
precision); the recipes below follow that: i.i.d. uniform[-1,1] or standard
normal entries drawn as float32 from numpy's PCG64 generator in logical
row-major order, rounded to binary16 or bfloat16 (round to nearest even) for
the 16-bit cases, then stored row- or column-major per operand.  Because
values are drawn in logical order, the four storage combinations of one
(seed, shape) hold the same logical matrices.
"""
import numpy as np

ROW_MAJOR = 0
COL_MAJOR = 1


def logical_matrix(rng, rows, cols, dist, dtype):
    """rows x cols logical matrix. dist: 'uniform' [-1,1], 'normal' N(0,1), 'int' {-4..4}."""
    if dist == "uniform":
        x = rng.uniform(-1.0, 1.0, size=(rows, cols)).astype(np.float32)
    elif dist == "normal":
        x = rng.standard_normal(size=(rows, cols), dtype=np.float32)
    elif dist == "int":
        x = rng.integers(-4, 5, size=(rows, cols)).astype(np.float32)
    else:
        raise ValueError(dist)
    if dtype == "f16":
        return x.astype(np.float16)
    if dtype == "f32":
        return x
    if dtype == "bf16":
        return round_to_bfloat16(x)
    raise ValueError(dtype)


def round_to_bfloat16(x):
    """float32 array -> float32 array whose values are bfloat16 numbers (the nearest one,
    ties to the even pattern).  numpy has no bfloat16 type, so logical bfloat16 matrices are
    kept as such float32 arrays and turned into 16-bit patterns by bfloat16_bits()."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    r = (u + 0x7FFF + ((u >> 16) & 1)) >> 16
    return (r << 16).astype(np.uint32).view(np.float32).reshape(np.shape(x))


def bfloat16_bits(x):
    """uint16 patterns (the upper halves) of a float32 array holding bfloat16 values."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    if np.any(u[~np.isnan(x.reshape(u.shape))] & 0xFFFF):
        raise ValueError("not a bfloat16 value")
    return (u >> 16).astype(np.uint16).reshape(np.shape(x))


def store(x, layout, ld=0):
    """Flat buffer holding logical matrix x in the given layout and leading dimension.

    ld == 0 means packed.  Padding elements (ld larger than packed) are filled
    with NaN so that any read of them shows up in a result.
    """
    rows, cols = x.shape
    if layout == ROW_MAJOR:
        major, minor, src = rows, cols, x
    else:
        major, minor, src = cols, rows, x.T
    if ld == 0:
        ld = minor
    if ld < minor:
        raise ValueError("ld below packed minimum")
    if major == 0 or minor == 0:
        return np.zeros(0, dtype=x.dtype)
    buf = np.full((major, ld), np.nan, dtype=x.dtype)
    buf[:, :minor] = src
    return buf.reshape(-1)[: (major - 1) * ld + minor].copy()


def load(buf, rows, cols, layout, ld=0):
    """Inverse of store: logical rows x cols view of a flat buffer."""
    if layout == ROW_MAJOR:
        major, minor = rows, cols
    else:
        major, minor = cols, rows
    if ld == 0:
        ld = minor
    if major == 0 or minor == 0:
        return np.zeros((rows, cols), dtype=buf.dtype)
    full = np.zeros(major * ld, dtype=buf.dtype)
    full[: buf.size] = buf
    m = full.reshape(major, ld)[:, :minor]
    return m if layout == ROW_MAJOR else m.T


def make_problem(seed, M, N, K, dist, dtype):
    """Logical A (M x K) and B (K x N) for one seeded case."""
    rng = np.random.default_rng(seed)
    A = logical_matrix(rng, M, K, dist, dtype)
    B = logical_matrix(rng, K, N, dist, dtype)
    return A, B


# The benchmark configurations, restated concretely.  Layout letters follow the
# row-major-centric convention of the configuration list: N = row-major
# operand, T = column-major operand.
LAYOUTS = {"NN": (ROW_MAJOR, ROW_MAJOR), "NT": (ROW_MAJOR, COL_MAJOR),
           "TN": (COL_MAJOR, ROW_MAJOR), "TT": (COL_MAJOR, COL_MAJOR)}

CONFIGS = {
    "f32_256_nn":      dict(dtype="f32", M=256, N=256, K=256, layout="NN", dist="uniform", seed=0),
    "f32_4096_nt":     dict(dtype="f32", M=4096, N=4096, K=4096, layout="NT", dist="uniform", seed=2000),
    "f16_8192_nn":     dict(dtype="f16", M=8192, N=8192, K=8192, layout="NN", dist="normal", seed=3000),
    "f16_8192_nt":     dict(dtype="f16", M=8192, N=8192, K=8192, layout="NT", dist="normal", seed=3000),
    "f16_8192_tn":     dict(dtype="f16", M=8192, N=8192, K=8192, layout="TN", dist="normal", seed=3000),
    "f16_8192_tt":     dict(dtype="f16", M=8192, N=8192, K=8192, layout="TT", dist="normal", seed=3000),
    "f16_edge_a":      dict(dtype="f16", M=1000, N=1500, K=2000, layout="NN", dist="uniform", seed=4001),
    "f16_edge_b":      dict(dtype="f16", M=4097, N=3073, K=1025, layout="NN", dist="uniform", seed=4002),
    "f16_skinny_n":    dict(dtype="f16", M=8192, N=128, K=8192, layout="TN", dist="normal", seed=5001),
    "f16_skinny_m":    dict(dtype="f16", M=128, N=8192, K=8192, layout="TN", dist="normal", seed=5002),
    "f16_deep_k":      dict(dtype="f16", M=1024, N=1024, K=65536, layout="TN", dist="normal", seed=5003),
}


def config_problem(name, dist=None):
    """(cfg, A_logical, B_logical, A_buffer, B_buffer) for a named configuration."""
    cfg = dict(CONFIGS[name])
    if dist is not None:
        cfg["dist"] = dist
    A, B = make_problem(cfg["seed"], cfg["M"], cfg["N"], cfg["K"], cfg["dist"], cfg["dtype"])
    la, lb = LAYOUTS[cfg["layout"]]
    return cfg, A, B, store(A, la), store(B, lb)
