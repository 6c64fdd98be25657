"""Collects the rocprofv3 evidence kept under profiles/ and writes the summaries.

Run from the repository root on an MI355X machine:

    python3 -m paper_2003_06324_amd.collect_profiles --raw gpurun_out/prof --out gpurun_out/profiles

It runs, each as its own rocprofv3 process with its own time limit (one counter set per run, no
trace domain mixed with counters):

  * `rocprofv3 --kernel-trace --stats -- python3 bench.py --no-context --no-cpu-baseline`
  * per benchmark configuration three counter passes over
    `python3 -m paper_2003_06324_amd.profile_workload ...`: FETCH_SIZE, WRITE_SIZE (both with a
    1 GiB copy kernel whose readings calibrate the two counters) and the SQ set (LDS bank
    conflicts, LDS index-active cycles, MFMA busy cycles, GRBM_GUI_ACTIVE);

and writes into --out: `bench_f16_8192_kernel_trace.txt`, `benchmark_configs_pmc_counters.txt` and
`counters.json` (what bench.py reports as `roofline.traffic` and in its `counters` block).
The raw rocprofv3 output stays under --raw.  This module never touches the GPU itself.
"""
import argparse
import collections
import csv
import glob
import json
import os
import re
import subprocess
import sys

# name, profile_workload arguments, algorithmic bytes (each operand read once, C written once)
CASES = [
    ("f16_8192_NT", "--dtype f16 --size 8192 --layout NT --dist normal", (2 * 8192 * 8192) * 2 + 8192 * 8192 * 4),
    ("f16_8192_NN", "--dtype f16 --size 8192 --layout NN --dist normal", (2 * 8192 * 8192) * 2 + 8192 * 8192 * 4),
    ("f16_8192_TN", "--dtype f16 --size 8192 --layout TN --dist normal", (2 * 8192 * 8192) * 2 + 8192 * 8192 * 4),
    ("f16_8192_TT", "--dtype f16 --size 8192 --layout TT --dist normal", (2 * 8192 * 8192) * 2 + 8192 * 8192 * 4),
    ("f32_4096_NT", "--dtype f32 --size 4096 --layout NT --dist uniform", (2 * 4096 * 4096) * 4 + 4096 * 4096 * 4),
    ("f16_8192x128x8192_TN", "--dtype f16 --size 8192 128 8192 --layout TN --dist normal",
     (8192 * 8192 + 8192 * 128) * 2 + 8192 * 128 * 4),
    ("f16_128x8192x8192_TN", "--dtype f16 --size 128 8192 8192 --layout TN --dist normal",
     (128 * 8192 + 8192 * 8192) * 2 + 128 * 8192 * 4),
    ("f16_1024x1024x65536_TN", "--dtype f16 --size 1024 1024 65536 --layout TN --dist normal",
     (2 * 1024 * 65536) * 2 + 1024 * 1024 * 4),
    ("f16_4097x3073x1025_NN", "--dtype f16 --size 4097 3073 1025 --layout NN --dist uniform",
     (4097 * 1025 + 1025 * 3073) * 2 + 4097 * 3073 * 4),
    ("f16_1000x1500x2000_NN", "--dtype f16 --size 1000 1500 2000 --layout NN --dist uniform",
     (1000 * 2000 + 2000 * 1500) * 2 + 1000 * 1500 * 4),
]
SQ = "SQ_LDS_BANK_CONFLICT SQ_LDS_IDX_ACTIVE SQ_VALU_MFMA_BUSY_CYCLES SQ_BUSY_CU_CYCLES GRBM_GUI_ACTIVE"
ITERS = 12
SKIP = 2     # dispatches left out of the averages (cold caches, clock ramp); the copy kernel runs 3 times


def run(cmd, log, limit):
    print("+", cmd, flush=True)
    with open(log, "w") as f:
        rc = subprocess.run(cmd, shell=True, stdout=f, stderr=subprocess.STDOUT, timeout=limit).returncode
    if rc != 0:
        sys.exit("failed (%d): %s -- see %s" % (rc, cmd, log))


def collect(raw):
    os.makedirs(raw, exist_ok=True)
    run("rocprofv3 --kernel-trace --stats --output-format csv -d %s/bench_trace -o bench -- python3 bench.py --no-context "
        "--no-cpu-baseline" % raw, "%s/bench_trace.log" % raw, 600)
    for name, args, _ in CASES:
        wl = "python3 -m paper_2003_06324_amd.profile_workload %s --iters %d" % (args, ITERS)
        run("rocprofv3 --pmc FETCH_SIZE --output-format csv -d %s/fetch_%s -o p -- %s --copy-mib 1024" % (raw, name, wl),
            "%s/fetch_%s.log" % (raw, name), 180)
        run("rocprofv3 --pmc WRITE_SIZE --output-format csv -d %s/write_%s -o p -- %s --copy-mib 1024" % (raw, name, wl),
            "%s/write_%s.log" % (raw, name), 180)
        run("rocprofv3 --pmc %s --output-format csv -d %s/sq_%s -o p -- %s" % (SQ, raw, name, wl),
            "%s/sq_%s.log" % (raw, name), 180)


def find(raw, sub, suffix):
    hits = glob.glob(os.path.join(raw, sub, "**", "*" + suffix), recursive=True)
    if not hits:
        sys.exit("no %s under %s/%s" % (suffix, raw, sub))
    return hits[0]


def short(name):
    """Readable kernel name (the profiler leaves names with a _Float16 argument mangled)."""
    m = re.search(r"gemm_(tile|ksplit)_kernel<([^>]*)>", name)
    if m:
        return "gemm_%s_kernel<%s>" % (m.group(1), m.group(2).replace("_Float16", "f16").replace(" ", ""))
    m = re.search(r"gemm_(tile|ksplit)_kernelI(DF16_|DF16b|f)((?:L[ib]\d+E)+)E", name)
    if m:
        elem = {"DF16_": "f16", "DF16b": "bf16", "f": "float"}[m.group(2)]
        # Lb0E / Lb1E are booleans, Li<n>E integers
        args = [("true" if v == "1" else "false") if k == "b" else v for k, v in re.findall(r"L([ib])(\d+)E", m.group(3))]
        return "gemm_%s_kernel<%s>" % (m.group(1), ",".join([elem] + args))
    return name[:90]


def counters(raw, sub, pattern):
    """Mean per dispatch of every counter over the dispatches whose kernel name contains pattern."""
    acc = collections.defaultdict(list)
    for r in csv.DictReader(open(find(raw, sub, "counter_collection.csv"))):
        if pattern in r["Kernel_Name"]:
            acc[r["Counter_Name"]].append(float(r["Counter_Value"]))
    return {k: sum(v[SKIP:]) / len(v[SKIP:]) for k, v in acc.items()}


def summed(raw, sub, patterns):
    """Per launch of the library call: the gemm kernel plus, with K slices, its reduce pass."""
    total = collections.defaultdict(float)
    for pat in patterns:
        acc = collections.defaultdict(list)
        for r in csv.DictReader(open(find(raw, sub, "counter_collection.csv"))):
            if pat in r["Kernel_Name"]:
                acc[r["Counter_Name"]].append(float(r["Counter_Value"]))
        for k, v in acc.items():
            total[k] += sum(v[SKIP:]) / len(v[SKIP:])
    return total


def summarise(raw, out):
    os.makedirs(out, exist_ok=True)
    # ---- kernel trace of bench.py
    rows = list(csv.DictReader(open(find(raw, "bench_trace", "kernel_stats.csv"))))
    line = [l for l in open("%s/bench_trace.log" % raw) if l.startswith('{"metric"')][-1].strip()
    txt = ["rocprofv3 kernel-trace summary of bench.py (headline step = f16 8192^3 in NN, NT, TN, TT; then the other benchmark",
           "configurations and the binary32 4096^3 product)",
           "command: rocprofv3 --kernel-trace --stats --output-format csv -d <raw>/bench_trace -o bench -- python3 bench.py --no-context --no-cpu-baseline",
           "(run and summarised by: python3 -m paper_2003_06324_amd.collect_profiles)", "",
           "%-92s %6s %12s %8s" % ("kernel", "calls", "avg_us", "pct")]
    for r in rows:
        txt.append("%-92s %6d %12.1f %8.4g" % (short(r["Name"]), int(r["Calls"]), float(r["AverageNs"]) / 1e3,
                                               float(r["Percentage"])))
    txt += ["", "Template arguments: element type, BM, BN, waves in M, waves in N, A K-contiguous, B K-contiguous, direct-load path.",
            "Per-kernel averages include the warm-up steps.  --no-context leaves out bench.py's zero-data, binary16-output and",
            "bfloat16 runs, which launch the headline kernels on other data and would mix into these averages.",
            "bench.py's JSON line of this same run:", line, ""]
    open(os.path.join(out, "bench_f16_8192_kernel_trace.txt"), "w").write("\n".join(txt))
    # ---- counters
    first = CASES[0][0]
    cf = counters(raw, "fetch_" + first, "copyBuffer")["FETCH_SIZE"]   # mean of the third copy (SKIP = 2)
    cw = counters(raw, "write_" + first, "copyBuffer")["WRITE_SIZE"]
    ff, wf = 1048576.0 / cf, 1048576.0 / cw   # the copy moves 1 GiB = 1048576 KiB each way
    table, js = [], {}
    for name, _, algo in CASES:
        kernels = ["gemm_tile_kernel", "gemm_ksplit_kernel", "splitk_reduce_kernel"]
        f = summed(raw, "fetch_" + name, kernels)["FETCH_SIZE"]
        w = summed(raw, "write_" + name, kernels)["WRITE_SIZE"]
        sq = counters(raw, "sq_" + name, "gemm_")
        util = sq["SQ_VALU_MFMA_BUSY_CYCLES"] / (sq["GRBM_GUI_ACTIVE"] / 8 * 1024)
        conflict = sq["SQ_LDS_BANK_CONFLICT"] / max(sq["SQ_LDS_IDX_ACTIVE"], 1.0)
        fb, wb = f * ff * 1024, w * wf * 1024
        table.append("%-24s %11.0f %11.0f %9.1f %9.1f %9.1f %6.2f %13.0f %15.0f %9.3f %10.0f" % (
            name, f, w, fb / 1e6, wb / 1e6, algo / 1e6, (fb + wb) / algo, sq["SQ_LDS_BANK_CONFLICT"], sq["SQ_LDS_IDX_ACTIVE"],
            util, sq["GRBM_GUI_ACTIVE"] / 8))
        js[name] = {"hbm_fetch_bytes": int(fb), "hbm_write_bytes": int(wb), "hbm_bytes": int(fb + wb), "algorithmic_bytes": algo,
                    "mfma_util": round(util, 4), "lds_bank_conflict_ratio": round(conflict, 6),
                    "cycles_per_xcd": int(sq["GRBM_GUI_ACTIVE"] / 8)}
    js["_source"] = ("profiles/benchmark_configs_pmc_counters.txt (python3 -m paper_2003_06324_amd.collect_profiles): FETCH_SIZE x "
                     "%.3f + WRITE_SIZE x %.3f KiB per library call; mfma_util = SQ_VALU_MFMA_BUSY_CYCLES / (GRBM_GUI_ACTIVE / 8 x 1024)"
                     % (ff, wf))
    json.dump(js, open(os.path.join(out, "counters.json"), "w"), indent=1)
    txt = ["HBM traffic and SQ counters per library call, rocprofv3 --pmc, one counter set per run (the K-sliced shapes include their",
           "reduce pass in the traffic columns; MfmaUtil and LDS counters are those of the gemm kernel)",
           "run and summarised by: python3 -m paper_2003_06324_amd.collect_profiles; per case it runs",
           "  rocprofv3 --pmc FETCH_SIZE --output-format csv -d <raw>/fetch_<case> -o p -- python3 -m paper_2003_06324_amd.profile_workload <case args> --iters 12 --copy-mib 1024",
           "  rocprofv3 --pmc WRITE_SIZE --output-format csv -d <raw>/write_<case> -o p -- (same)",
           "  rocprofv3 --pmc %s --output-format csv -d <raw>/sq_<case> -o p -- python3 -m paper_2003_06324_amd.profile_workload <case args> --iters 12" % SQ,
           "case args:"] + ["  %-24s %s" % (n, a) for n, a, _ in CASES] + [
           "",
           "calibration: the copy kernel of the same run (1024 MiB read + 1024 MiB written) reads FETCH_SIZE = %.0f -> factor %.3f," % (cf, ff),
           "  WRITE_SIZE = %.0f -> factor %.3f (both counters are in KiB)" % (cw, wf), "",
           "%-24s %11s %11s %9s %9s %9s %6s %13s %15s %9s %10s" % ("case", "FETCH_SIZE", "WRITE_SIZE", "fetch_MB", "write_MB", "algo_MB",
                                                                  "x algo", "LDS_CONFLICT", "LDS_IDX_ACTIVE", "MfmaUtil", "cyc/XCD")] + table + [
           "",
           "MfmaUtil = SQ_VALU_MFMA_BUSY_CYCLES / (GRBM_GUI_ACTIVE / 8 XCDs x 1024 SIMDs): the share of the launch's cycles, at whatever",
           "clock the part ran, in which a SIMD's matrix core was busy.  Counter runs serialise kernels and are slower than untraced",
           "runs: use them for ratios, not for durations.", ""]
    open(os.path.join(out, "benchmark_configs_pmc_counters.txt"), "w").write("\n".join(txt))
    print("\n".join(txt))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--raw", default="gpurun_out/prof")
    ap.add_argument("--out", default="gpurun_out/profiles")
    ap.add_argument("--summarise-only", action="store_true", help="the raw rocprofv3 output is already there")
    args = ap.parse_args()
    if not args.summarise_only:
        collect(args.raw)
    summarise(args.raw, args.out)


if __name__ == "__main__":
    main()
