"""Small driver for rocprofv3 runs: launches one GEMM configuration a few times and,
optionally, a plain device-to-device copy of known size whose FETCH_SIZE / WRITE_SIZE
readings calibrate the HBM-traffic counters.

    python3 -m paper_2003_06324_amd.profile_workload --dtype f16 --size 8192 --layout NT --iters 5 --copy-mib 1024

With --sustain SECONDS it instead keeps the launches going for that long while a thread samples
`amd-smi metric -p -c` (socket power, per-XCD clocks) and prints rate, power, clock and energy
per launch: the part holds a power limit by lowering its clock, which is what bounds the
random-data figures.

    python3 -m paper_2003_06324_amd.profile_workload --size 8192 --layout NT --dist normal --sustain 4

With --phases it switches on the library's per-workgroup phase trace (gemm_set_phase_trace), runs
the launch a few times and prints, from the last launch, how long the workgroups spend in each
phase of a tile (start-up, K loop, hand-over of shared memory, stores) and how long a CU waits
between two workgroups: where the time that is not matrix-core time goes.

    python3 -m paper_2003_06324_amd.profile_workload --size 8192 --layout NT --dist normal --phases
"""
import argparse
import os
import sys

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--dtype", choices=["f16", "f32"], default="f16")
    ap.add_argument("--size", type=int, nargs="+", default=[8192], help="M N K, or one value for a cube")
    ap.add_argument("--layout", choices=["NN", "NT", "TN", "TT"], default="NT")
    ap.add_argument("--dist", choices=["normal", "uniform", "zeros"], default="normal")
    ap.add_argument("--iters", type=int, default=5)
    ap.add_argument("--copy-mib", type=int, default=0, help="also run a copy kernel of this many MiB")
    ap.add_argument("--force", default=None, help="tile configuration override, e.g. t256x256")
    ap.add_argument("--sustain", type=float, default=0.0, help="seconds of back-to-back launches with power sampling")
    ap.add_argument("--phases", action="store_true", help="per-workgroup phase trace of the last launch")
    args = ap.parse_args()

    import torch
    import gemm_inputs as gi
    import paper_2003_06324_amd as g

    M, N, K = (args.size * 3)[:3] if len(args.size) == 1 else args.size
    tdt = torch.float16 if args.dtype == "f16" else torch.float32
    gen = torch.Generator(device="cuda").manual_seed(0)

    def draw(n):
        if args.dist == "zeros":
            return torch.zeros(n, dtype=tdt, device="cuda")
        x = torch.empty(n, dtype=torch.float32, device="cuda")
        x.normal_(generator=gen) if args.dist == "normal" else x.uniform_(-1, 1, generator=gen)
        return x.to(tdt)

    A, B = draw(M * K), draw(K * N)
    C = torch.empty(M * N, dtype=torch.float32, device="cuda")
    la, lb = gi.LAYOUTS[args.layout]
    fn = g.gemm_f16f32 if args.dtype == "f16" else g.gemm_f32
    stream = torch.cuda.current_stream().cuda_stream
    g.force_config(args.force)
    if args.sustain > 0:
        sustain(lambda: fn(M, N, K, A, la, 0, B, lb, 0, C, gi.ROW_MAJOR, 0, stream), args.sustain,
                2.0 * M * N * K, "%s %dx%dx%d %s %s" % (args.dtype, M, N, K, args.layout, args.dist))
        print("gemm:", g.last_config())
        return
    if args.phases:
        phases(lambda: fn(M, N, K, A, la, 0, B, lb, 0, C, gi.ROW_MAJOR, 0, stream), max(args.iters, 20),
               "%s %dx%dx%d %s %s" % (args.dtype, M, N, K, args.layout, args.dist))
        return
    for _ in range(args.iters):
        fn(M, N, K, A, la, 0, B, lb, 0, C, gi.ROW_MAJOR, 0, stream)
    torch.cuda.synchronize()
    print("gemm:", g.last_config(), "x", args.iters)
    if args.copy_mib:
        n = args.copy_mib * (1 << 20) // 4
        src = torch.ones(n, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print("copy: %d MiB read + %d MiB written, x3" % (args.copy_mib, args.copy_mib))


def phases(launch, iters, what):
    """Phase table of the last of `iters` launches from the library's per-workgroup trace."""
    import numpy as np
    import torch
    import paper_2003_06324_amd as g
    cap = 1 << 16
    buf = torch.zeros(cap * 8, dtype=torch.int64, device="cuda")
    torch.cuda.synchronize()
    g.set_phase_trace(buf, cap)
    try:
        for _ in range(iters):
            launch()
        torch.cuda.synchronize()
    finally:
        g.set_phase_trace(None)
    rec = buf.cpu().numpy().reshape(cap, 8)
    rec = rec[rec[:, 0] != 0]
    ts = (rec[:, :6] - rec[:, 0].min()) * 0.01          # microseconds (100 MHz clock)
    print("%s [%s]: %d workgroups, span of the launch %.1f us" % (what, g.last_config(), len(rec), ts[:, 5].max()))
    have_first = bool((rec[:, 1] != 0).all())     # only the direct-load kernels record it
    spans = ([("start -> first operands landed", 0, 1), ("K loop", 1, 2)] if have_first
             else [("start -> K loop done", 0, 2)])
    spans += [("shared memory handed to the epilogue", 2, 3), ("stores issued", 3, 4), ("stores complete", 4, 5)]
    for name, i0, i1 in spans:
        d = ts[:, i1] - ts[:, i0]
        print("  %-38s mean %7.2f us   p10 %7.2f   p50 %7.2f   p90 %7.2f   max %7.2f" % (
            name, d.mean(), np.percentile(d, 10), np.percentile(d, 50), np.percentile(d, 90), d.max()))
    hw, xcc = rec[:, 7] & 0xFFFFFFFF, rec[:, 7] >> 32
    cu = ((xcc & 0xF) << 12) | (((hw >> 13) & 7) << 8) | (((hw >> 12) & 1) << 4) | ((hw >> 8) & 0xF)
    gaps, per_cu = [], []
    for c in np.unique(cu):
        idx = np.where(cu == c)[0]
        idx = idx[np.argsort(ts[idx, 0])]
        per_cu.append(len(idx))
        gaps += [ts[b, 0] - ts[a, 5] for a, b in zip(idx[:-1], idx[1:])]
    print("  %d CUs used, %d..%d workgroups each" % (len(per_cu), min(per_cu), max(per_cu)))
    if gaps and np.median(gaps) < 0:
        # a CU runs more than one workgroup of this tile at a time: there is no gap to measure, and
        # the phases of one workgroup include the time it waits for the matrix cores the other uses
        print("  workgroups overlap on a CU (next one starts %.1f us before the previous ends, median)" % -np.median(gaps))
    elif gaps:
        gaps = np.array(gaps)
        print("  %-38s mean %7.2f us   p50 %7.2f   p90 %7.2f   max %7.2f" % (
            "CU idle between two workgroups", gaps.mean(), np.percentile(gaps, 50), np.percentile(gaps, 90), gaps.max()))
    total = ts[:, 5] - ts[:, 0]
    loop = ts[:, 2] - ts[:, 1 if have_first else 0]
    print("  per workgroup: %.2f us in all, %.2f us (%.1f %%) outside the K loop" % (
        total.mean(), (total - loop).mean(), 100.0 * (total - loop).mean() / total.mean()))


def sustain(launch, seconds, flop, what):
    import json
    import subprocess
    import threading
    import time
    import torch
    samples, stop = [], []

    def sampler():
        while not stop:
            try:
                out = subprocess.run(["amd-smi", "metric", "-p", "-c", "--json"], capture_output=True, text=True,
                                     timeout=10).stdout
                gpu = json.loads(out)["gpu_data"][0]
                clocks = [v["clk"]["value"] for k, v in gpu["clock"].items() if k.startswith("gfx_")]
                samples.append((float(gpu["power"]["socket_power"]["value"]), sum(clocks) / len(clocks)))
            except Exception:
                pass
            time.sleep(0.3)

    th = threading.Thread(target=sampler)
    th.start()
    for _ in range(10):
        launch()
    torch.cuda.synchronize()
    t0, n = time.time(), 0
    while time.time() - t0 < seconds:
        for _ in range(50):
            launch()
        torch.cuda.synchronize()
        n += 50
    dt = time.time() - t0
    stop.append(1)
    th.join()
    steady = samples[len(samples) // 3:] or samples
    line = "%s: %.1f TFLOP/s, %.1f us per launch" % (what, flop * n / dt / 1e12, dt / n * 1e6)
    if steady:
        watts = sum(s[0] for s in steady) / len(steady)
        mhz = sum(s[1] for s in steady) / len(steady)
        line += ", socket power %.0f W, mean XCD clock %.0f MHz, %.0f mJ per launch (%d samples)" % (
            watts, mhz, watts * dt / n * 1e3, len(steady))
    else:
        line += ", no power samples (amd-smi not usable here)"
    print(line, flush=True)


if __name__ == "__main__":
    main()
