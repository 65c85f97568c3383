#!/usr/bin/env python3
"""Fault-injection campaign on the GPU path: detection, false-alarm and correction rates.

Runs many trials of one workload through the C ABI (encode once, then per trial: plant
0-2 faults, multiply, verify, correct, read the report, restore the operands) and compares
the located errors with the planted ones.  No oracle is involved: the ground truth is the
fault list itself.  Prints one JSON object.

    python -m paper_2508_04355_amd.campaign --workload cfg3 --trials 10000

Pairs of faults in one column of A (one row of B) are beyond the code (that line carries two
parity symbols, Section III); they are counted in classes of their own, where "corrected_exactly"
means the expected outcome, UNCORRECTABLE.

Fault classes follow the paper's scenarios (Section VI: a = A, b = B, c = C, d = A+C,
e = B+C, f = C+C) plus the pairs it does not test (A+A, B+B, A+B) and the fault-free case.
"""
import argparse
import collections
import json
import math
import sys

import numpy as np
import torch

from . import configs, gecc, inputs

MA, MB, MC = inputs.MAT_A, inputs.MAT_B, inputs.MAT_C
CLASS_NAME = {(): "none", (MA,): "a:A", (MB,): "b:B", (MC,): "c:C", (MA, MC): "d:A+C", (MB, MC): "e:B+C",
              (MC, MC): "f:C+C", (MA, MA): "A+A", (MB, MB): "B+B", (MA, MB): "A+B"}


def run(workload: str, trials: int, seed_cfg: int = 30, progress=None):
    w = configs.ALL[workload]
    if w.batch != 1:
        raise ValueError("campaign runs single-product workloads")
    dev = "cuda:0"
    n, k, m = w.n, w.k, w.m
    rng = inputs.rng_for(seed_cfg, 0)
    A, B = inputs.operands(rng, n, k, m, w.law_a, w.law_b, w.dtype)
    tdt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
    hA = A.T.copy() if w.trans_a else A
    hB = B.T.copy() if w.trans_b else B
    dA = torch.from_numpy(hA).to(tdt).to(dev)[None]
    dB = torch.from_numpy(hB).to(tdt).to(dev)[None]
    ctx = gecc.Context(n, k, m, gecc.BF16 if w.dtype == "bf16" else gecc.F32, w.tau,
                       trans_a=w.trans_a, trans_b=w.trans_b)
    A_par, B_par, C_par = ctx.alloc_parities()
    rep = ctx.alloc_report()
    Cd = ctx.alloc_c()
    ctx.encode_a(dA, A_par)
    ctx.encode_b(dB, B_par)
    Aclean, Bclean = dA.clone(), dB.clone()

    stats = collections.defaultdict(lambda: collections.Counter())
    by_decade = collections.defaultdict(lambda: collections.Counter())
    failures = []                                       # the first trials that were not corrected exactly
    for t in range(trials):
        frng = inputs.rng_for(seed_cfg, 1 + t)
        count = int(frng.integers(0, 3))
        faults = inputs.draw_faults(frng, n, k, m, count, w.offset_law)
        cf, want, touched = [], [], []
        for f in faults:
            if f.matrix == MC:
                cf.append((0, f.row, f.col, f.offset))
                want.append((MC, f.row, f.col))
                continue
            T, tr = (dA, w.trans_a) if f.matrix == MA else (dB, w.trans_b)
            i, j = (f.col, f.row) if tr else (f.row, f.col)
            old = T[0, i, j].item()
            T[0, i, j] += f.offset                      # rounds to the storage type
            if T[0, i, j].item() != old:                # a fault that survives the rounding
                want.append((f.matrix, f.row, f.col))
            touched.append((T, i, j, old))
        cls = CLASS_NAME[tuple(sorted(f.matrix for f in faults))]
        if len(want) == 2 and want[0][0] == want[1][0] != MC and \
                want[0][2 if want[0][0] == MA else 1] == want[1][2 if want[0][0] == MA else 1]:
            # two wrong symbols in one column of A (one row of B): that line carries two parity
            # symbols (Section III), so the pair is beyond the code and has to be recomputed
            cls += " (one line)"
        fl, nf = gecc.make_faults(cf, dev)
        ctx.multiply(dA, A_par, dB, B_par, Cd, C_par, fl, nf)
        ctx.verify(Cd, C_par, rep, fused=True)
        ctx.correct(dA, A_par, dB, B_par, Cd, C_par, rep)
        r = ctx.report_to_host(rep)[0]
        got = [(e[0], e[1], e[2]) for e in r.errors()]
        detected = r.status != gecc.CLEAN
        exact = r.status == gecc.CORRECTED and got == sorted(want)
        if cls.endswith("(one line)"):
            exact = r.status == gecc.UNCORRECTABLE
        st = stats[cls]
        st["trials"] += 1
        st["detected"] += int(detected)
        st["corrected_exactly"] += int(exact)
        st["uncorrectable"] += int(r.status == gecc.UNCORRECTABLE)
        st["miscorrected"] += int(r.status == gecc.CORRECTED and got != sorted(want))
        if want:
            dec = int(math.floor(math.log10(min(abs(f.offset) for f in faults))))
            bd = by_decade["1e%d" % dec]
            bd["trials"] += 1
            bd["detected"] += int(detected)
            bd["corrected_exactly"] += int(exact)
        if want and not exact and len(failures) < 32:
            failures.append({"trial": t, "class": cls, "status": int(r.status), "n_total": int(r.n_total),
                             "faults": [[int(f.matrix), int(f.row), int(f.col), float(f.offset)] for f in faults],
                             "located": [[int(e[0]), int(e[1]), int(e[2]), float(e[3])] for e in r.errors()]})
        if touched and (not exact or r.status != gecc.CORRECTED):   # the attempt may have patched elsewhere
            dA.copy_(Aclean)
            dB.copy_(Bclean)
        for (T, i, j, old) in touched:                  # restore the planted symbols
            T[0, i, j] = old
        if progress and (t + 1) % progress == 0:
            print("trial %d / %d" % (t + 1, trials), file=sys.stderr, flush=True)

    out = {"workload": w.name, "trials": trials,
           "thresholds": [w.tau.r1, w.tau.r2, w.tau.q1, w.tau.q2],
           "by_class": {c: dict(v) for c, v in sorted(stats.items())},
           "by_smallest_offset_decade": {d: dict(v) for d, v in sorted(by_decade.items())},
           "failures": failures}
    none = stats.get("none")
    if none:
        out["false_alarm_rate"] = none["detected"] / max(1, none["trials"])
    faulty = [v for c, v in stats.items() if c != "none"]
    if faulty:
        out["detection_rate"] = sum(v["detected"] for v in faulty) / sum(v["trials"] for v in faulty)
        out["exact_correction_rate"] = sum(v["corrected_exactly"] for v in faulty) / sum(v["trials"] for v in faulty)
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="cfg3")
    ap.add_argument("--trials", type=int, default=10000)
    ap.add_argument("--progress", type=int, default=1000)
    args = ap.parse_args()
    print(json.dumps(run(args.workload, args.trials, progress=args.progress)))


if __name__ == "__main__":
    main()
