"""Fits the constants of the selection's cost model (estimate_cost in csrc/gemm_api.hip) to sweeps.

The per-size tuning of the paper's Section 5.3 is an exhaustive search per input size; this
library replaces the search at call time by a cost model whose constants come from such searches
done once: `tune_sweep.py --all` times every configuration at 1..32 K slices on a list of shapes,
and this script fits the model to those logs.

    python3 -m paper_2003_06324_amd.tune_sweep --all --shapes-file paper_2003_06324_amd/tune_shapes/fit_a.txt > a.log
    ... (fit_b.txt, fit_c.txt, paper_ranges.txt, and the built-in shapes: tune_sweep --all > tuned.log)
    python3 -m paper_2003_06324_amd.fit_cost_model --tuned tuned.log --paper paper.log a.log b.log c.log

Two steps per operand class (binary16 / binary32 x aligned / 4-byte aligned / 2-byte aligned):
least squares on log(predicted / measured) over all configurations of all shapes, then a random
search that lowers the time lost by the model's pick against the best measured configuration
(geometric mean and worst case over the random shapes and, as a group of its own, over the paper's
power-of-two sizes; more weight on the built-in shapes, which are the benchmark configurations,
and on the same picks with each of the four run-time scale factors of the model at 0.88 and 1.12).
A microsecond is added to both times of a ratio: the few-microsecond shapes time +-20 % from run to run.  The script prints the table rows and constants
to carry into gemm_api.hip by hand; tune_shapes/validation.txt is never passed to it.

This file mirrors the model's formula; tests/test_cabi_exports.py checks the library's picks, not
this mirror.  Needs numpy and scipy; runs on the CPU.
"""
import math
import re
import sys

import numpy as np
from scipy.optimize import least_squares

NUM_CU = 256
# name: (BM, BN, workgroups per CU, slabs in flight on the register-staged path)
TILES = {"t256x256": (256, 256, 1, 1), "t128x128": (128, 128, 2, 3), "t64x64": (64, 64, 4, 4), "t256x256w8": (256, 256, 1, 1),
         "t256x128": (256, 128, 1, 1), "t128x256": (128, 256, 1, 1), "t64x128": (64, 128, 2, 3), "t128x64": (128, 64, 2, 3),
         "k64x64": (64, 64, 4, 1)}
NAMES = list(TILES)
PATH_OF_CLASS = {"aligned": 0, "aligned4": 3, "general": 2}
K_CONTIG = {"NN": 1, "NT": 2, "TN": 0, "TT": 1}     # how many of A, B have K as their contiguous dimension
GLOBALS = dict(fixed=2.7, lat=0.85, hbm_cap=4.8e6, l2=22e6, red_fixed=1.5, red_rate=3.8e6, red_slice=0.087,
               foot_factor=0.29, foot_lo=2.2e5, foot_hi=1.5e7)
GLOBAL_NAMES = list(GLOBALS)
# starting points: (alone, full, fixed) per 64-k binary16 slab, (alone, full) per 32-k binary32 slab
START16 = {"t256x256": (1.1, 1.1, 5.0), "t128x128": (0.5, 0.85, 1.5), "t64x64": (0.28, 0.72, 1.2), "t256x256w8": (1.15, 1.15, 3.4),
           "t256x128": (0.8, 0.8, 3.0), "t128x256": (0.73, 0.73, 3.1), "t64x128": (0.36, 0.59, 1.4), "t128x64": (0.37, 0.6, 1.3),
           "k64x64": (0.29, 0.71, 2.3)}
START32 = {"t256x256": (7.5, 7.5), "t128x128": (1.9, 3.3), "t64x64": (0.48, 1.7), "t256x256w8": (7.0, 7.0), "t256x128": (3.6, 3.6),
           "t128x256": (3.4, 3.4), "t64x128": (0.89, 1.7), "t128x64": (0.97, 1.65), "k64x64": (0.55, 1.8)}
PERTURBED = [tuple(f if i == j else 1.0 for i in range(4)) for j in range(4) for f in (0.88, 1.12)]


def cdiv(a, b):
    return -(-a // b)


def load(path):
    """One dict per shape of a `tune_sweep --all` log."""
    lines = open(path).read().split("\n")
    out = []
    for i, line in enumerate(lines):
        if not line.startswith("   all:"):
            continue
        meas = {}
        for item in line.split()[1:]:
            name, us = item.split("=")
            tile, slices = name.split(":s")
            meas[(tile, int(slices))] = float(us)
        m = re.match(r"(f16|f32) (\d+)x(\d+)x(\d+) (\w\w)( \+\d+B)?: auto [\d.]+ us \[\w+ \w+ \w+ (\w+) s", lines[i + 1])
        dt, M, N, K, lay, _, cls = m.groups()
        M, N, K = int(M), int(N), int(K)
        path = PATH_OF_CLASS[cls]
        slab_k = 32 if dt == "f32" else 64
        if path != 0 or K % slab_k:   # the launch path substitutes t64x64 there: not a measurement of k64x64
            meas = {k: v for k, v in meas.items() if k[0] != "k64x64"}
        out.append(dict(dt=dt, M=M, N=N, K=K, lay=lay, path=path, meas=meas, KT=cdiv(K, slab_k), best=min(meas.values())))
    return out


def cost(tile, alone, full, fixed, hbm_eff, G, sh, splits, esz, mult=1.0, floor_lat=0.0, tail=0.0, lay=(1, 1, 1), sc=(1, 1, 1, 1)):
    """The formula of estimate_cost; sc = the four run-time scale factors (slab, HBM, L2, fixed)."""
    M, N, K, KT = sh["M"], sh["N"], sh["K"], sh["KT"]
    BM, BN, occ, depth = TILES[tile]
    tiles = cdiv(M, BM) * cdiv(N, BN)
    per = cdiv(KT, splits)
    S = cdiv(KT, per)
    W = tiles * S
    slots = NUM_CU * occ
    rounds = cdiv(W, slots)
    share = min(cdiv(W, NUM_CU), occ)
    slab = alone + ((full - alone) * (share - 1) / (occ - 1) if occ > 1 else 0.0)
    slab *= mult * lay[K_CONTIG[sh["lay"]]]
    foot = (M * K + K * N) * esz      # operands that stay in the L2s are served faster
    if foot <= G["foot_lo"]:
        slab *= G["foot_factor"]
    elif foot < G["foot_hi"]:
        slab *= math.exp(math.log(G["foot_factor"]) * (math.log(G["foot_hi"]) - math.log(foot)) /
                         (math.log(G["foot_hi"]) - math.log(G["foot_lo"])))
    if floor_lat:
        slab = max(slab, floor_lat / (share * depth))
    slab *= sc[0]
    t_mfma = rounds * (per * slab + fixed)
    if K % (128 // esz):
        t_mfma += tail * slab
    unique = (M * K + K * N) * esz + M * N * 4
    resident = min(W, slots)
    hbm = min(G["hbm_cap"], resident * 1.5 * (BM + BN) * 128 / G["lat"]) * hbm_eff * sc[1]
    t_l2 = W * per * (BM + BN) * 128 / (G["l2"] * sc[2])
    c = G["fixed"] * sc[3] + max(t_mfma, unique / hbm, t_l2)
    if S > 1:
        c += (G["red_fixed"] + G["red_slice"] * S) * sc[3] + M * N * 4 * (S + 1) / (G["red_rate"] * sc[1])
    return c


def points(shapes):
    """(shape, tile, slices, microseconds, weight): configurations far from the best weigh less."""
    return [(sh, t, s, v, 1.0 if v < 1.5 * sh["best"] else 0.3)
            for sh in shapes for (t, s), v in sh["meas"].items() if not (s > sh["KT"] and s > 1)]


def regret(shapes, cf):
    """Measured time of the model's pick over the best measured time, per shape (a microsecond added to both)."""
    out = []
    for sh in shapes:
        best = None
        for t in NAMES:
            if not any(k[0] == t for k in sh["meas"]):
                continue
            for s in (1, 2, 4, 8, 16, 32):
                if s > 1 and s > sh["KT"]:
                    break
                c = cf(sh, t, s)
                if best is None or c < best[0]:
                    best = (c, t, s)
        _, t, s = best
        KT, meas = sh["KT"], sh["meas"]
        us = meas.get((t, s))
        if us is None:   # beyond the slab count: the forced count that gives the same non-empty slices
            us = min(v for (t_, s_), v in meas.items() if t_ == t and cdiv(KT, cdiv(KT, s_)) == cdiv(KT, cdiv(KT, s)))
        out.append((us + 1.0) / (sh["best"] + 1.0))
    return out


def summary(r):
    r = np.array(r)
    return "n %d geomean %.3f p90 %.2f max %.2f" % (len(r), math.exp(np.log(r).mean()), np.quantile(r, .9), r.max()) if len(r) else "n 0"


def objective(groups, tuned, cf):
    j = 0.0
    for shapes in groups:
        if shapes:
            r = np.log(regret(shapes, cf))
            j += r.mean() + 0.15 * r.max()
    if tuned:
        u = np.log(regret(tuned, cf))
        j += 4.0 * u.mean() + 3.0 * u.max()
        for sc in PERTURBED:
            j += 0.5 * np.log(regret(tuned, lambda sh, t, s: cf(sh, t, s, sc))).max()
    return j


def refine(x, make_cf, groups, tuned, iters, seed=0, sigma=0.05):
    rng = np.random.default_rng(seed)
    best = objective(groups, tuned, make_cf(x))
    for _ in range(iters):
        y = x.copy()
        k = rng.choice(len(x), size=rng.integers(1, 4), replace=False)
        y[k] += rng.normal(0, sigma, size=len(k))
        j = objective(groups, tuned, make_cf(y))
        if j < best:
            best, x = j, y
    return x


def select(dt, path, shapes):
    return [sh for sh in shapes if sh["dt"] == dt and sh["path"] == path]


def fit_stage(x0, make_cf, rand, paper, tuned, iters, spread, label):
    pts = points(rand + paper + tuned)

    def residuals(x):
        cf = make_cf(x)
        return np.array([w * math.log(cf(sh, t, s) / v) for sh, t, s, v, w in pts])

    x = least_squares(residuals, x0, bounds=(x0 - spread, x0 + spread), max_nfev=80).x
    for stage in ("least squares", "refined"):
        if stage == "refined":
            x = refine(x, make_cf, [rand, paper], tuned, iters)
        print("%s, %s (rms %.3f): pick/best on random shapes %s | paper's sizes %s | built-in shapes %s" % (
            label, stage, residuals(x).std(), summary(regret(rand, make_cf(x))),
            summary(regret(paper, make_cf(x))) if paper else "-", summary(regret(tuned, make_cf(x))) if tuned else "-"), flush=True)
    return x


def main():
    args = sys.argv[1:]
    iters = 1500
    tuned = []
    paper = []
    if "--iters" in args:
        i = args.index("--iters")
        iters = int(args[i + 1])
        del args[i:i + 2]
    if "--tuned" in args:
        i = args.index("--tuned")
        tuned = load(args[i + 1])
        del args[i:i + 2]
    if "--paper" in args:
        i = args.index("--paper")
        paper = load(args[i + 1])
        del args[i:i + 2]
    if not args:
        sys.exit(__doc__)
    rand = [sh for path in args for sh in load(path)]
    NG = len(GLOBAL_NAMES)

    # binary16, aligned: slab times, fixed part and HBM efficiency per tile, the global terms, the ragged-K tail
    def unpack16(x):
        T = {}
        for i, t in enumerate(NAMES):
            a, f, fx, he = np.exp(x[4 * i:4 * i + 4])
            T[t] = (a, max(a, f) if TILES[t][2] > 1 else a, fx, he)
        G = {k: math.exp(v) for k, v in zip(GLOBAL_NAMES, x[36:36 + NG])}
        return T, G, math.exp(x[36 + NG])

    def make16(x):
        T, G, tail = unpack16(x)
        return lambda sh, t, s, sc=(1, 1, 1, 1): cost(t, *T[t], G, sh, s, 2, tail=tail, sc=sc)

    x0 = []
    for t in NAMES:
        x0 += [math.log(v) for v in START16[t]] + [0.0]
    x0 = np.array(x0 + [math.log(GLOBALS[k]) for k in GLOBAL_NAMES] + [math.log(2.5)])
    T16, G, tail16 = unpack16(fit_stage(x0, make16, select("f16", 0, rand), select("f16", 0, paper), select("f16", 0, tuned), iters,
                                        5.0, "f16 aligned"))

    # binary32, aligned: slab times and tail only (fixed part, HBM efficiency and globals as fitted above)
    def unpack32(x):
        T = {}
        for i, t in enumerate(NAMES):
            a, f = np.exp(x[2 * i:2 * i + 2])
            T[t] = (a, max(a, f) if TILES[t][2] > 1 else a, T16[t][2], T16[t][3])
        return T, math.exp(x[18])

    def make32(x):
        T, tail = unpack32(x)
        return lambda sh, t, s, sc=(1, 1, 1, 1): cost(t, *T[t], G, sh, s, 4, tail=tail, sc=sc)

    x0 = []
    for t in NAMES:
        x0 += [math.log(v) for v in START32[t]]
    x0 = np.array(x0 + [math.log(1.5)])
    T32, tail32 = unpack32(fit_stage(x0, make32, select("f32", 0, rand), select("f32", 0, paper), select("f32", 0, tuned), iters,
                                     5.0, "f32 aligned"))

    # misaligned classes: a slab-time multiplier per tile, a factor per number of K-contiguous operands, the tail
    tiles = [t for t in NAMES if t != "k64x64"]
    classes = {}
    for dt, path, T, esz, m0, floor_lat, tail0 in (("f16", 3, T16, 2, 1.15, 0.0, 2.4), ("f32", 3, T32, 4, 1.0, 0.0, 1.5),
                                                   ("f16", 2, T16, 2, 1.7, 1.2, 3.6)):
        def unpack(x):
            return ({t: math.exp(x[i]) for i, t in enumerate(tiles)}, (math.exp(x[8]), 1.0, math.exp(x[9])), math.exp(x[10]))

        def make(x, T=T, esz=esz, floor_lat=floor_lat):
            m, lay, tail = unpack(x)
            return lambda sh, t, s, sc=(1, 1, 1, 1): cost(t, *T[t], G, sh, s, esz, m[t], floor_lat, tail, lay, sc)

        x0 = np.array([math.log(m0)] * 8 + [0.0, 0.0, math.log(tail0)])
        classes[dt, path] = unpack(fit_stage(x0, make, select(dt, path, rand), [], select(dt, path, tuned), iters, 3.0,
                                             "%s path %d" % (dt, path)))

    print("\nglobal terms:", {k: float("%.3g" % v) for k, v in G.items()}, "ragged-K tail f16 %.3g f32 %.3g" % (tail16, tail32))
    print("tile: f16_alone, f16_full, f32_alone, f32_full, fixed, hbm_eff, f16_a4, f32_a4, f16_a2")
    for t in NAMES:
        a4 = classes["f16", 3][0].get(t, classes["f16", 3][0]["t64x64"])
        b4 = classes["f32", 3][0].get(t, classes["f32", 3][0]["t64x64"])
        a2 = classes["f16", 2][0].get(t, classes["f16", 2][0]["t64x64"])
        print("  %-11s" % t + ", ".join("%.3g" % v for v in (T16[t][0], T16[t][1], T32[t][0], T32[t][1], T16[t][2], T16[t][3], a4, b4, a2)))
    for (dt, path), (_, lay, tail) in classes.items():
        print("%s path %d: factor by K-contiguous operands (0, 1, 2) %s, ragged-K tail %.3g" % (
            dt, path, ["%.3g" % v for v in lay], tail))


if __name__ == "__main__":
    main()
