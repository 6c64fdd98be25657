"""Helpers for the GPU parity tests: move seeded operands to the device, call the
C-ABI library through its Python binding, bring C back as a logical matrix."""
import numpy as np

import gemm_inputs as gi

# max|C-Cref| / (K max|A| max|B|), the stated bar; bfloat16 operands take the binary16 one: the
# products are exact in binary32 in both cases and the accumulation is the same
TOL = {"f32": 1e-6, "f16": 2e-4, "bf16": 2e-4}
# Stricter internal bar, max|C-Cref| / (K rms|A| rms|B|) <= 8 * 2^-24: binary32 accumulation
# of K terms of size ~rms^2 drifts by about 2^-24 * K * rms^2 / sqrt(2) (random walk of the
# per-add roundings, each ~2^-24 of a partial sum ~sqrt(k) rms^2); 8 leaves room for the
# maximum over all entries.  One dropped or doubled term costs ~rms^2, i.e. 1/K >> the bar.
TIGHT = {"f32": 8 * 2.0 ** -24, "f16": 8 * 2.0 ** -24, "bf16": 8 * 2.0 ** -24}


def all_tiles():
    """Names of all kernel configurations of the built library (host call, no GPU needed)."""
    import paper_2003_06324_amd as g
    return g.config_names()


def ran_tile(tile, cfg):
    """The configuration string names the forced tile; a K-split-across-waves configuration
    ("k64x64") hands operands it does not serve (not 16-byte aligned, K not a multiple of the
    slab) to the two-dimensional tile of the same size ("t64x64")."""
    return tile in cfg.split() or (tile[0] == "k" and "t" + tile[1:] in cfg.split())


def to_device(buf):
    import torch
    if buf.dtype == np.float16:
        buf = buf.view(np.int16)
    if buf.size == 0:
        return torch.empty(0, dtype=torch.from_numpy(buf).dtype, device="cuda")
    return torch.from_numpy(np.ascontiguousarray(buf)).cuda()


def run_gpu(dtype, A, B, la, lb, lc=gi.ROW_MAJOR, pads=(0, 0, 0), offsets=(0, 0, 0), force=None,
            return_config=False, out="f32"):
    """HIP path on logical matrices A (M x K), B (K x N); returns logical float32 C
    (out="f16": the binary16-output entry point, returns a float16 array).  dtype "bf16": A and
    B are float32 arrays holding bfloat16 values, handed over as their 16-bit patterns.

    pads: extra leading-dimension elements per operand (padding is NaN-filled and, for C,
    checked to be untouched).  offsets: element offsets of each base pointer inside its
    allocation (to exercise unaligned bases)."""
    import torch
    import paper_2003_06324_amd as g
    M, K = A.shape
    N = B.shape[1]
    lda = (K if la == gi.ROW_MAJOR else M) + pads[0]
    ldb = (N if lb == gi.ROW_MAJOR else K) + pads[1]
    ldc = (N if lc == gi.ROW_MAJOR else M) + pads[2]
    esz = 4 if dtype == "f32" else 2
    bufA = np.concatenate([np.full(offsets[0], np.nan, A.dtype), gi.store(A, la, lda)])
    bufB = np.concatenate([np.full(offsets[1], np.nan, B.dtype), gi.store(B, lb, ldb)])
    if dtype == "bf16":
        bufA, bufB = gi.bfloat16_bits(bufA).view(np.int16), gi.bfloat16_bits(bufB).view(np.int16)
    dA, dB = to_device(bufA), to_device(bufB)
    c_major = M if lc == gi.ROW_MAJOR else N
    c_minor = N if lc == gi.ROW_MAJOR else M
    c_len = ((c_major - 1) * ldc + c_minor) if (M > 0 and N > 0) else 0
    c_np, c_torch, c_esz = (np.float32, torch.float32, 4) if out == "f32" else (np.float16, torch.float16, 2)
    dC = torch.full((offsets[2] + c_len + 8,), float("nan"), dtype=c_torch, device="cuda")
    fn = {"f32": g.gemm_f32, "bf16": g.gemm_bf16f32, "f16": g.gemm_f16f32 if out == "f32" else g.gemm_f16f16}[dtype]
    stream = torch.cuda.current_stream().cuda_stream
    g.force_config(force)
    try:
        fn(M, N, K, dA.data_ptr() + offsets[0] * esz, la, lda, dB.data_ptr() + offsets[1] * esz, lb, ldb,
           dC.data_ptr() + offsets[2] * c_esz, lc, ldc, stream)
        cfg = g.last_config()
    finally:
        g.force_config(None)
    torch.cuda.synchronize()
    host = dC.cpu().numpy()
    assert np.all(np.isnan(host[:offsets[2]])) and np.all(np.isnan(host[offsets[2] + c_len:])), \
        "wrote outside C"
    body = host[offsets[2]:offsets[2] + c_len]
    if c_len and pads[2]:
        full = np.full(c_major * ldc, np.nan, c_np)
        full[:c_len] = body
        assert np.all(np.isnan(full.reshape(c_major, ldc)[:, c_minor:].reshape(-1)[:-pads[2]])), \
            "wrote into the ld padding of C"
    C = np.array(gi.load(body, M, N, lc, ldc))
    return (C, cfg) if return_config else C


def errors(C, ref, A, B):
    """(stated metric, tight metric) of a result against the float64 reference."""
    K = A.shape[1]
    if C.size == 0 or K == 0:
        return 0.0, 0.0
    diff = np.max(np.abs(C.astype(np.float64) - ref))
    a64, b64 = np.abs(A.astype(np.float64)), np.abs(B.astype(np.float64))
    amax, bmax = a64.max(), b64.max()
    arms, brms = np.sqrt(np.mean(a64 ** 2)), np.sqrt(np.mean(b64 ** 2))
    stated = diff / (K * amax * bmax) if amax * bmax > 0 else diff
    tight = diff / (K * arms * brms) if arms * brms > 0 else diff
    return float(stated), float(tight)


def check(C, ref, A, B, dtype, what=""):
    assert np.all(np.isfinite(C)), "non-finite output " + what
    stated, tight = errors(C, ref, A, B)
    assert stated <= TOL[dtype], "%s: stated error %.3e > %.1e" % (what, stated, TOL[dtype])
    assert tight <= TIGHT[dtype], "%s: tight error %.3e > %.1e" % (what, tight, TIGHT[dtype])
    return stated, tight
