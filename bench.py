"""Benchmark of the GEMM hot path on one MI355X.

A step is one pass over the headline workload: the FP16-in / FP32-accumulate
8192^3 product in all four operand layouts (NN, NT, TN, TT; N = row-major
operand, T = column-major operand), i.e. four library calls.  Inputs are
seeded synthetic matrices already resident in HBM.  Prints one JSON line.

Beside the headline it carries, outside the timed step: `configs`, one row per benchmark
configuration (kernel chosen, median / minimum microseconds per launch from HIP events, TFLOP/s,
the MFMA and HBM floors and the fraction of the binding one); `counters`, the rocprofv3 figures of
the dominant headline launch read from profiles/counters.json (MfmaUtil, LDS bank-conflict ratio,
HBM bytes, turned into GB/s with the launch time measured here); the zero-data, binary16-output
and bfloat16 context runs; and the CPU oracle's rate on a bounded sample.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_TFLOPS = {"f16": 2516.6, "f32": 157.3}   # MI355X dense MFMA peaks: 256 CU x 2.4 GHz x 4096 / 256 flop/clk/CU


def device_operands(A, B, layout):
    """Device buffers of logical torch matrices A (M x K), B (K x N) in the given layouts."""
    import gemm_inputs as gi
    la, lb = gi.LAYOUTS[layout]
    dA = A.contiguous() if la == gi.ROW_MAJOR else A.t().contiguous()
    dB = B.contiguous() if lb == gi.ROW_MAJOR else B.t().contiguous()
    return dA, la, dB, lb


def time_calls(fn, calls, steps, warmup):
    """Run `calls` (list of argument tuples) per step; returns (wall seconds for `steps`
    steps, per-call mean milliseconds from HIP events recorded on the launch stream).
    The clocks cannot be locked here, so median and minimum are kept beside the mean."""
    import torch
    stream = torch.cuda.current_stream()
    for _ in range(warmup):
        for args in calls:
            fn(*args, stream.cuda_stream)
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(len(calls) + 1)] for _ in range(steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(steps):
        events[s][0].record(stream)
        for i, args in enumerate(calls):
            fn(*args, stream.cuda_stream)
            events[s][i + 1].record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    samples = [sorted(events[s][i].elapsed_time(events[s][i + 1]) for s in range(steps)) for i in range(len(calls))]
    per_call = [sum(x) / steps for x in samples]
    time_calls.spread = [(x[len(x) // 2], x[0]) for x in samples]   # (median, min) per call of the last run
    return wall, per_call


def config_rows(per_layout, S, skip_big):
    """One row per benchmark configuration.  The four headline launches are taken from the timed
    step; the others are timed here, each on its own seeded operands (generated on the host
    exactly as the parity tests generate them); median and minimum over batches of back-to-back launches."""
    import numpy as np
    import torch
    import gemm_inputs as gi
    import paper_2003_06324_amd as g
    rows = []
    stream = torch.cuda.current_stream()
    for name, cfg in gi.CONFIGS.items():
        M, N, K, lay, dt = cfg["M"], cfg["N"], cfg["K"], cfg["layout"], cfg["dtype"]
        esz = 4 if dt == "f32" else 2
        flop = 2.0 * M * N * K
        algo = (M * K + K * N) * esz + M * N * 4
        mfma_us = flop / (PEAK_TFLOPS[dt] * 1e12) * 1e6
        hbm_us = algo / 8e12 * 1e6
        if name.startswith("f16_8192_") and S == 8192:
            pl = per_layout[lay]
            med, mn, kernel = pl["ms_median"] * 1e3, pl["ms_min"] * 1e3, pl["kernel"]
        else:
            if skip_big and M * K + K * N > (1 << 27):
                continue
            _, A_np, B_np, bufA, bufB = gi.config_problem(name)
            if dt == "f16":
                bufA, bufB = bufA.view(np.int16), bufB.view(np.int16)
            dA, dB = torch.from_numpy(bufA).cuda(), torch.from_numpy(bufB).cuda()
            C = torch.empty(M * N, dtype=torch.float32, device="cuda")
            la, lb = gi.LAYOUTS[lay]
            fn = g.gemm_f32 if dt == "f32" else g.gemm_f16f32
            # raw addresses: for the few-microsecond shapes the binding's per-call work would otherwise show
            call = (M, N, K, dA.data_ptr(), la, 0, dB.data_ptr(), lb, 0, C.data_ptr(), gi.ROW_MAJOR, 0)
            # back-to-back launches between two events, as the tuning sweep times them (an event after
            # every launch would add a few microseconds of its own to the small shapes); seven batches
            iters = 20 if flop > 5e10 else 100
            for _ in range(20):
                fn(*call, stream.cuda_stream)
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(8)]
            ev[0].record(stream)   # no host wait after the warm-up: the part would drop its clock in the gap
            for b in range(7):
                for _ in range(iters):
                    fn(*call, stream.cuda_stream)
                ev[b + 1].record(stream)
            torch.cuda.synchronize()
            us = sorted(ev[b].elapsed_time(ev[b + 1]) * 1e3 / iters for b in range(7))
            med, mn, kernel = us[len(us) // 2], us[0], g.last_config()
            del dA, dB, C
        floor = max(mfma_us, hbm_us)
        rows.append({"config": name, "shape": [M, N, K], "layout": lay, "dtype": dt, "kernel": kernel,
                     "us_median": round(med, 2), "us_min": round(mn, 2), "tflops": round(flop / med / 1e6, 1),
                     "floor_mfma_us": round(mfma_us, 2), "floor_hbm_us": round(hbm_us, 2),
                     "bound": "mfma" if mfma_us >= hbm_us else "hbm", "frac_of_floor": round(floor / med, 4)})
    return rows


def cpu_baseline(A_np, B_np, gpu_rows, target_seconds=15.0):
    """Oracle timed on the host cores on the first rows of the NT case; also returns the
    largest deviation of the GPU result on those rows (stated metric)."""
    import numpy as np
    import gemm_inputs as gi
    from oracle import gemm_oracle
    M, K = A_np.shape
    N = B_np.shape[1]
    Bt = gi.store(B_np, gi.COL_MAJOR)
    gemm_oracle.build()

    def run(rows):
        t0 = time.perf_counter()
        out, _ = gemm_oracle.gemm_f16_raw(rows, N, K, gi.store(A_np[:rows], gi.ROW_MAJOR), 0, 0, Bt, 1, 0)
        return time.perf_counter() - t0, out

    # time = fixed operand-widening cost + rows * per-row cost: two probes give both
    t_a, _ = run(16)
    t_b, _ = run(80)
    per_row = max((t_b - t_a) / 64.0, 1e-9)
    fixed = max(t_a - 16 * per_row, 0.0)
    rows = int(max(64, min(M, (target_seconds - fixed) / per_row)))
    secs, ref = run(rows)
    ref = ref.reshape(rows, N)
    got = gpu_rows(rows)
    err = float(np.max(np.abs(got - ref)) / (K * float(np.abs(A_np).max()) * float(np.abs(B_np).max())))
    return {"value": 2.0 * rows * N * K / secs / 1e12, "unit": "TFLOP/s", "cores": gemm_oracle.num_threads(),
            "kind": "oracle", "seconds": round(secs, 2),
            "sample": "first %d of %d rows of C of the NT case (%d x %d x %d), float64 triple loop" % (rows, M, rows, N, K)}, err


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--size", type=int, default=8192, help="M = N = K of the headline workload")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-configs", action="store_true", help="skip the per-configuration rows (they launch other kernels)")
    ap.add_argument("--no-context", action="store_true",
                    help="skip the zero-data and binary16-output context runs (they launch the headline kernels "
                         "on other data, which would mix into per-kernel averages of a profiler)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        sys.exit("bench.py: this build is single-GPU (a GEMM tile needs no exchange; see DESIGN.md); run with --gpus 1")

    import numpy as np
    import torch
    import gemm_inputs as gi
    import paper_2003_06324_amd as g

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    g.load_library()
    torch.cuda.set_device(0)
    S = args.size
    # --- headline workload: FP16 in, FP32 accumulate, S^3, four layouts, N(0,1) entries, seed 3000
    A_np, B_np = gi.make_problem(3000, S, S, S, "normal", "f16")
    A = torch.from_numpy(A_np.view(np.int16)).cuda()
    B = torch.from_numpy(B_np.view(np.int16)).cuda()
    names = ["NN", "NT", "TN", "TT"]
    keep, calls, outs = [], [], {}
    for name in names:
        dA, la, dB, lb = device_operands(A, B, name)
        C = torch.empty(S * S, dtype=torch.float32, device="cuda")
        keep.append((dA, dB, C))
        outs[name] = C
        calls.append((S, S, S, dA, la, 0, dB, lb, 0, C, gi.ROW_MAJOR, 0))
    wall, per_call = time_calls(g.gemm_f16f32, calls, args.steps, args.warmup)
    spread = time_calls.spread
    configs = {}
    for name, c in zip(names, calls):
        g.gemm_f16f32(*c, torch.cuda.current_stream().cuda_stream)
        configs[name] = g.last_config()
    torch.cuda.synchronize()
    flop = 2.0 * S * S * S
    ms_per_step = wall * 1e3 / args.steps
    value = 4 * flop / (ms_per_step * 1e-3) / 1e12
    per_layout = {n: {"ms": round(ms, 4), "ms_median": round(md, 4), "ms_min": round(mn, 4),
                      "tflops": round(flop / ms / 1e9, 1), "kernel": configs[n]}
                  for n, ms, (md, mn) in zip(names, per_call, spread)}
    # dominant kernel = the layout that takes the largest share of the step
    dom = max(names, key=lambda n: per_layout[n]["ms"])
    achieved = flop / per_layout[dom]["ms"] / 1e9
    traffic, counters = None, None
    cpath = os.path.join(ROOT, "profiles", "counters.json")
    if os.path.exists(cpath):
        try:
            c = json.load(open(cpath)).get("f16_%d_%s" % (S, dom))
            if c:
                traffic = c["hbm_bytes"]
                counters = {"case": "f16_%d_%s" % (S, dom), "mfma_util": c["mfma_util"],
                            "lds_bank_conflict_ratio": c["lds_bank_conflict_ratio"],
                            "hbm_bytes_per_launch": c["hbm_bytes"], "algorithmic_bytes_per_launch": c["algorithmic_bytes"],
                            "hbm_gbps": round(c["hbm_bytes"] / (per_layout[dom]["ms"] * 1e-3) / 1e9, 1),
                            "source": "profiles/counters.json <- profiles/benchmark_configs_pmc_counters.txt (rocprofv3 --pmc, "
                                      "separate runs); GB/s uses the launch time measured in this run"}
        except Exception:
            traffic, counters = None, None
    roofline = {"bound": "mfma", "achieved": round(achieved, 1), "peak": PEAK_TFLOPS["f16"], "unit": "TFLOP/s",
                "frac": round(achieved / PEAK_TFLOPS["f16"], 4), "traffic": traffic,
                "kernel": per_layout[dom]["kernel"], "flop_per_launch": flop,
                "avg_launch_ms": per_layout[dom]["ms"]}

    zero_data = fp16_out = bf16 = None
    if not args.no_context:
        # --- context, not part of the timed step: the same four launches on all-zero operands.  With
        # N(0,1) data the part lowers its clock to stay inside its power limit; zeros do not toggle the
        # matrix cores' inputs, so this is the rate of the same kernels at (nearly) the full clock.
        Z = torch.zeros(S * S, dtype=torch.int16, device="cuda")
        CZ = torch.empty(S * S, dtype=torch.float32, device="cuda")  # the headline results stay untouched
        zcalls = [c[:3] + (Z, c[4], 0, Z, c[7], 0, CZ) + c[10:] for c in calls]
        zwall, _ = time_calls(g.gemm_f16f32, zcalls, max(5, args.steps // 5), max(2, args.warmup // 5))
        z_tflops = 4 * flop / (zwall / max(5, args.steps // 5)) / 1e12
        zero_data = {"workload": "same four launches, all-zero operands (no data-dependent clock throttling)",
                     "tflops": round(z_tflops, 1), "frac_of_peak": round(z_tflops / PEAK_TFLOPS["f16"], 4)}
        del Z, CZ

        # --- context: the binary16-output entry point on the NT case (the operand and result types of
        # the paper's own tensor-core kernels and of the half-precision routine it is measured against)
        C16 = torch.empty(S * S, dtype=torch.float16, device="cuda")
        nt = calls[names.index("NT")]
        _, pc16 = time_calls(g.gemm_f16f16, [nt[:9] + (C16,) + nt[10:]], max(5, args.steps // 2), max(2, args.warmup // 2))
        fp16_out = {"workload": "f16f16_%dx%dx%d_NT (binary16 C)" % (S, S, S), "ms": round(pc16[0], 4),
                    "tflops": round(flop / pc16[0] / 1e9, 1), "kernel": g.last_config()}
        del C16

        # --- context: the bfloat16 sibling on the same NT launch (same kernels, other MFMA instruction);
        # N(0,1) entries rounded to bfloat16
        Ab = torch.from_numpy(gi.bfloat16_bits(gi.round_to_bfloat16(A_np.astype(np.float32))).view(np.int16)).cuda()
        Bb = torch.from_numpy(gi.bfloat16_bits(gi.round_to_bfloat16(B_np.astype(np.float32))).view(np.int16)).cuda()
        dAb, _, dBb, _ = device_operands(Ab, Bb, "NT")
        Cb = torch.empty(S * S, dtype=torch.float32, device="cuda")  # the headline results stay untouched
        _, pcb = time_calls(g.gemm_bf16f32, [nt[:3] + (dAb, nt[4], 0, dBb, nt[7], 0, Cb) + nt[10:]],
                            max(5, args.steps // 2), max(2, args.warmup // 2))
        bf16 = {"workload": "bf16f32_%dx%dx%d_NT" % (S, S, S), "ms": round(pcb[0], 4),
                "tflops": round(flop / pcb[0] / 1e9, 1), "kernel": g.last_config()}
        del Ab, Bb, dAb, dBb, Cb

    # --- secondary workload (not part of the timed step): FP32 4096^3, A row-major, B column-major
    A32_np, B32_np = gi.make_problem(2000, 4096, 4096, 4096, "uniform", "f32")
    A32 = torch.from_numpy(A32_np).cuda()
    B32 = torch.from_numpy(B32_np).cuda()
    dA, la, dB, lb = device_operands(A32, B32, "NT")
    C32 = torch.empty(4096 * 4096, dtype=torch.float32, device="cuda")
    _, pc = time_calls(g.gemm_f32, [(4096, 4096, 4096, dA, la, 0, dB, lb, 0, C32, gi.ROW_MAJOR, 0)],
                       max(5, args.steps), max(2, args.warmup))
    f32_tflops = 2.0 * 4096 ** 3 / pc[0] / 1e9
    fp32 = {"workload": "f32_4096x4096x4096_NT", "ms": round(pc[0], 4), "tflops": round(f32_tflops, 1),
            "frac_of_peak": round(f32_tflops / PEAK_TFLOPS["f32"], 4), "peak": PEAK_TFLOPS["f32"],
            "kernel": g.last_config()}

    out = {
        "metric": "GEMM TFLOP/s (FP16-in/FP32-acc, %d^3, mean over NN/NT/TN/TT) at 1 GPU" % S,
        "value": round(value, 1), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16", "data": "synthetic",
        "config": {"workload": "f16f32_%dx%dx%d_NN+NT+TN+TT" % (S, S, S), "gemms_per_step": 4,
                   "entries": "N(0,1) rounded to binary16, seed 3000", "C": "binary32 row-major"},
        "pct_of_peak": round(100.0 * value / PEAK_TFLOPS["f16"], 2),
        "per_layout": per_layout, "roofline": roofline, "fp32": fp32,
    }
    if counters is not None:
        out["counters"] = counters
    if not args.no_configs:
        out["configs"] = config_rows(per_layout, S, skip_big=False)
    if zero_data is not None:
        out["zero_data"], out["fp16_out"], out["bf16"] = zero_data, fp16_out, bf16
    if not args.no_cpu_baseline:
        def gpu_rows(rows):
            return outs["NT"][: rows * S].cpu().numpy().reshape(rows, S)
        base, err = cpu_baseline(A_np, B_np, gpu_rows)
        out["cpu_baseline"] = base
        out["parity_on_sample"] = {"max_err_over_K_maxA_maxB": err, "tolerance": 2e-4, "ok": bool(err <= 2e-4)}
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
