"""Per-size tuning over the paper's size ranges (Section 5.3: small sizes up to 1024, large sizes 1024..4096,
powers of two), by the library's own search (gemm_tune): for every M, N, K in {256, 512, 1024, 2048, 4096}, every
layout pair and both operand types, lets gemm_tune time every configuration, then times the cost model's pick and
the recorded pick alternately in one pass, and writes the table of recorded picks.

    python3 -m paper_2003_06324_amd.tune_paper_ranges [--out picks.txt] [--sizes 256,512,...]
    python3 -m paper_2003_06324_amd.tune_paper_ranges --shapes-file paper_2003_06324_amd/tune_shapes/validation.txt --out /tmp/picks.txt
        (the same comparison on a list of shapes, lines "f16|f32 M N K NN|NT|TN|TT [byte offset of the operand bases]")

Prints one line per shape and a summary (time of the model's pick over time of the tuned pick).  The table it
writes is what paper_2003_06324_amd/tuned_mi355x.txt holds; load it with gemm.tune_load() (the library does not
load it by itself: the cost model is the default, this is the measured alternative for these sizes).
"""
import itertools
import os
import sys

import numpy as np

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))


def main():
    import torch
    import gemm_inputs as gi
    import paper_2003_06324_amd as g

    args = sys.argv[1:]
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "tuned_mi355x.txt")
    sizes = [256, 512, 1024, 2048, 4096]
    if "--out" in args:
        out = args[args.index("--out") + 1]
    if "--sizes" in args:
        sizes = [int(x) for x in args[args.index("--sizes") + 1].split(",")]
    listed = None
    if "--shapes-file" in args:
        listed = []
        for line in open(args[args.index("--shapes-file") + 1]):
            f = line.split()
            if f and not f[0].startswith("#"):
                listed.append((f[0], int(f[1]), int(f[2]), int(f[3]), f[4], int(f[5]) if len(f) > 5 else 0))
    stream = torch.cuda.current_stream().cuda_stream

    def timed(fn, configs, iters):
        """Microseconds per call under each forced configuration of `configs`, in one pass: 30 launches of the automatic
        choice, then per configuration 3 untimed and `iters` timed launches between two events, everything enqueued back
        to back and one wait at the end (the part lowers its clock within microseconds of idling; a wait between
        configurations would time the next one on a rising clock)."""
        g.force_config(None)
        for _ in range(30):
            fn()
        pairs = []
        for cfg in configs:
            g.force_config(cfg)
            for _ in range(3):
                fn()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(iters):
                fn()
            e1.record()
            pairs.append((e0, e1))
        g.force_config(None)
        torch.cuda.synchronize()
        return [e0.elapsed_time(e1) / iters * 1e3 for e0, e1 in pairs]

    g.force_config(None)
    g.tune_clear()
    ratios = {"f16": [], "f32": []}
    changed = 0
    if listed is None:
        listed = [(dt, M, N, K, lay, 0) for dt in ("f16", "f32") for M, N, K in itertools.product(sizes, repeat=3)
                  for lay in ("NN", "NT", "TN", "TT")]
    for dt, tdt, kind, call in (("f16", torch.float16, g.KIND_F16F32, g.gemm_f16f32), ("f32", torch.float32, g.KIND_F32, g.gemm_f32)):
        mine = [sh for sh in listed if sh[0] == dt]
        if not mine:
            continue
        # one pair of operand buffers of the largest size serves every shape (packed leading dimensions)
        big_a = max(sh[1] * sh[3] for sh in mine) + 16
        big_b = max(sh[3] * sh[2] for sh in mine) + 16
        A0, B0 = torch.randn(big_a, device="cuda", dtype=tdt), torch.randn(big_b, device="cuda", dtype=tdt)
        C = torch.empty(max(sh[1] * sh[2] for sh in mine), device="cuda", dtype=torch.float32)
        for _, M, N, K, lay, off in mine:
            iters = 20 if 2.0 * M * N * K > 5e10 else 100
            A, B = A0.data_ptr() + off, B0.data_ptr() + off
            if True:
                la, lb = gi.LAYOUTS[lay]
                fn = lambda: call(M, N, K, A, la, 0, B, lb, 0, C, gi.ROW_MAJOR, 0, stream)
                fn()
                model = g.last_config().split()
                model = model[1] + ":" + model[4]
                pick = g.tune(kind, M, N, K, A, la, 0, B, lb, 0, C, gi.ROW_MAJOR, 0, stream)
                # both picks forced alternately in one pass, the better take of each
                takes = timed(fn, [model, pick, model, pick], iters)
                t_model, t_tuned = min(takes[0::2]), min(takes[1::2])
                if pick == model:
                    t_model = t_tuned = min(t_model, t_tuned)
                else:
                    changed += 1
                ratios[dt].append(t_model / t_tuned)
                print("%s %dx%dx%d %s%s: model %s %.1f us | tuned %s %.1f us | model/tuned %.2f" % (
                    dt, M, N, K, lay, " +%dB" % off if off else "", model, t_model, pick, t_tuned, t_model / t_tuned), flush=True)
    g.tune_save(out)
    for dt, r in ratios.items():
        if not r:
            continue
        r = np.array(r)
        print("%s: %d shapes, model/tuned geometric mean %.3f, median %.2f, 90th percentile %.2f, worst %.2f" % (
            dt, len(r), float(np.exp(np.log(r).mean())), float(np.median(r)), float(np.quantile(r, 0.9)), float(r.max())))
    print("%d of %d picks differ from the model's; table written to %s" % (changed, sum(len(r) for r in ratios.values()), out))
    g.tune_clear()


if __name__ == "__main__":
    main()
