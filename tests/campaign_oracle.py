#!/usr/bin/env python3
"""Fault campaign on one operand pair, every trial decided twice: by the HIP path (through the
binding of the C ABI) and by the CPU oracle (oracle/incremental.py, the oracle evaluated as
changes of the clean C-bar).  Test infrastructure: lives under tests/ because it imports the oracle.

Per trial: 0, 1 or 2 faults uniform over the data symbols of A, B and C (the workload's offset
law); operand faults are written into the device operands after the parities were formed, faults
of C go into the product kernel's fault list; multiply -> verify -> correct -> report; the same
faults go to the oracle.  Compared: status and located positions bit for bit, magnitudes and the
whole corrected C within tolerance, the operands after correction.

A trial is *margin-safe* when the oracle reaches the same status and positions with all four
thresholds halved and doubled: then no decision of it hangs on a syndrome that rounding noise
(the GPU forms syndromes from fp32 sums, the oracle in fp64; clean syndromes stay below a quarter
of the thresholds) could move across a threshold.  Parity is demanded on every margin-safe trial;
the others are counted and listed.

    python tests/campaign_oracle.py --workload cfg3 --trials 10000     # prints one JSON object
"""
import argparse
import collections
import json
import math
import os
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

from oracle import grid_code as oc                      # noqa: E402
from oracle.incremental import IncrementalOracle        # noqa: E402
from paper_2508_04355_amd import configs, gecc, inputs  # noqa: E402

MA, MB, MC = inputs.MAT_A, inputs.MAT_B, inputs.MAT_C
CLASS_NAME = {(): "none", (MA,): "a:A", (MB,): "b:B", (MC,): "c:C", (MA, MC): "d:A+C", (MB, MC): "e:B+C",
              (MC, MC): "f:C+C", (MA, MA): "A+A", (MB, MB): "B+B", (MA, MB): "A+B"}
STATUS = {0: "clean", 1: "corrected", 2: "uncorrectable", 3: "detected"}


def _scaled(tau, f):
    return oc.Thresholds(tau.r1 * f, tau.r2 * f, tau.q1 * f, tau.q2 * f, tau.op, tau.rep, tau.rel)


def run(workload: str, trials: int, seed_cfg: int = 30, progress=None, tol_c=1e-5):
    w = configs.ALL[workload]
    assert w.batch == 1
    dev = "cuda:0"
    n, k, m = w.n, w.k, w.m
    rng = inputs.rng_for(seed_cfg, 0)
    A, B = inputs.operands(rng, n, k, m, w.law_a, w.law_b, w.dtype)
    tau = oc.Thresholds(w.tau.r1, w.tau.r2, w.tau.q1, w.tau.q2, w.tau.op, w.tau.rep, w.tau.rel)
    t0 = time.perf_counter()
    inc = IncrementalOracle(A, B, tau)
    t_setup = time.perf_counter() - t0

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
    Cref = torch.from_numpy(np.ascontiguousarray(inc.C)).to(dev)       # the oracle's clean data block, fp64
    scale = inc.scale

    stats = collections.defaultdict(collections.Counter)
    by_decade = collections.defaultdict(collections.Counter)
    mismatches, unsafe = [], []
    worst_c = worst_left = worst_c_no_operand_fault = 0.0
    t_oracle = t_gpu = 0.0
    for t in range(trials):
        frng = inputs.rng_for(seed_cfg, 1 + t)
        count = int(frng.integers(0, 3))
        faults = inputs.draw_faults(frng, n, k, m, count, w.offset_law)
        a_f, b_f, c_f = [], [], []
        for f in faults:
            if f.matrix == MC:
                c_f.append((f.row, f.col, f.offset))
                continue
            M = A if f.matrix == MA else B
            old = float(M[f.row, f.col])
            new = float(inputs.store(np.array([old + f.offset]), w.dtype)[0])
            if new != old:                              # a fault that survives the storage rounding
                (a_f if f.matrix == MA else b_f).append((f.row, f.col, new))
        cls = CLASS_NAME[tuple(sorted(f.matrix for f in faults))]

        # ---- the oracle, at the stated thresholds and at half and twice them -------------------
        t1 = time.perf_counter()
        res = inc.trial(a_f, b_f, c_f)
        key = (res.status, [e[:3] for e in res.errors])
        safe = all((r.status, [e[:3] for e in r.errors]) == key
                   for r in (inc.trial(a_f, b_f, c_f, _scaled(tau, 0.5)), inc.trial(a_f, b_f, c_f, _scaled(tau, 2.0))))
        t_oracle += time.perf_counter() - t1

        # ---- the HIP path ------------------------------------------------------------------------
        t1 = time.perf_counter()
        for (i, l, v) in a_f:
            if w.trans_a: dA[0, l, i] = v
            else: dA[0, i, l] = v
        for (l, j, v) in b_f:
            if w.trans_b: dB[0, j, l] = v
            else: dB[0, l, j] = v
        fl, nf = gecc.make_faults([(0,) + c for c in c_f], dev)
        ctx.multiply(dA, A_par, dB, B_par, Cd, C_par, fl, nf)
        ctx.verify(Cd, C_par, rep, fused=True)
        ctx.correct(dA, A_par, dB, B_par, Cd, C_par, rep)
        r = ctx.report_to_host(rep)[0]
        got = r.errors()
        why = None if r.status == res.status else "status"
        if why is None and res.status != oc.UNCORRECTABLE:
            if r.n_total != len(res.errors) or [e[:3] for e in got] != [e[:3] for e in res.errors[:gecc.MAX_ERR]]:
                why = "positions"
            # corrected C: tol_c of the largest symbol; a line repaired after an operand fault keeps the
            # rounding of the corrupted terms f = e b_lj (or a_il e) that sat in its fp32 running sums,
            # bounded like the decoder's own allowance for such lines by tau_rep sqrt(k) max|f|
            fmax = max([abs(v - A[i, l]) * float(np.max(np.abs(B[l, :]))) for (i, l, v) in a_f] +
                       [abs(v - B[l, j]) * float(np.max(np.abs(A[:, l]))) for (l, j, v) in b_f] + [0.0])
            tol = min(w.tol_c, tol_c + w.tau.rep * math.sqrt(k) * fmax / scale)
            # (a magnitude read from a syndrome that crosses a repaired line carries that rounding too)
            for x, y in zip(got, res.errors):
                if why is None and abs(x[3] - y[3]) > 10 * tol_c * scale + 2e-6 * abs(y[3]) + w.tau.rep * math.sqrt(k) * fmax:
                    why = "magnitude"
            err_c = float((Cd[0, :, :m].double() - Cref).abs().max()) / scale
            worst_c = max(worst_c, err_c)
            if not fmax:
                worst_c_no_operand_fault = max(worst_c_no_operand_fault, err_c)
            if why is None and not err_c <= tol:
                why = "C"
            ops_ok = bool(torch.equal(dA, Aclean) and torch.equal(dB, Bclean))
            if res.status == oc.CORRECTED and res.operands_restored:
                if why is None and not ops_ok:
                    why = "operands"
                worst_left = max(worst_left, res.left_in_cbar / scale)
            if not ops_ok:
                dA.copy_(Aclean); dB.copy_(Bclean)
        else:
            dA.copy_(Aclean); dB.copy_(Bclean)
        same = why is None
        t_gpu += time.perf_counter() - t1

        st = stats[cls]
        st["trials"] += 1
        st["oracle_" + STATUS[res.status]] += 1
        st["gpu_" + STATUS[r.status]] += 1
        st["margin_safe"] += int(safe)
        st["agree"] += int(same)
        st["agree_margin_safe"] += int(same and safe)
        want = sorted([(MA, i, l) for (i, l, v) in a_f] + [(MB, l, j) for (l, j, v) in b_f] + [(MC, i, j) for (i, j, e) in c_f])
        st["oracle_exact"] += int(res.status == (oc.CORRECTED if want else oc.CLEAN) and [e[:3] for e in res.errors] == want)
        if faults:
            dec = int(math.floor(math.log10(min(abs(f.offset) for f in faults))))
            bd = by_decade["1e%d" % dec]
            bd["trials"] += 1
            bd["detected_gpu"] += int(r.status != gecc.CLEAN)
            bd["detected_oracle"] += int(res.status != oc.CLEAN)
            bd["agree"] += int(same)
        if not same:
            rec = {"trial": t, "class": cls, "margin_safe": bool(safe), "differs_in": why,
                   "faults": [[int(f.matrix), int(f.row), int(f.col), float(f.offset)] for f in faults],
                   "oracle": [int(res.status)] + [[int(e[0]), int(e[1]), int(e[2]), float(e[3])] for e in res.errors[:8]],
                   "gpu": [int(r.status)] + [[int(e[0]), int(e[1]), int(e[2]), float(e[3])] for e in got]}
            (mismatches if safe else unsafe).append(rec)
        if progress and (t + 1) % progress == 0:
            print("trial %d / %d" % (t + 1, trials), file=sys.stderr, flush=True)

    none = stats.get("none", collections.Counter())
    faulty = [v for c, v in stats.items() if c != "none"]
    n_faulty = max(1, sum(v["trials"] for v in faulty))
    return {"workload": w.name, "trials": trials, "thresholds": [w.tau.r1, w.tau.r2, w.tau.q1, w.tau.q2],
            "by_class": {c: dict(v) for c, v in sorted(stats.items())},
            "by_smallest_offset_decade": {d: dict(v) for d, v in sorted(by_decade.items())},
            "trials_without_faults": none["trials"],
            "false_alarms_gpu": none["trials"] - none["gpu_clean"],
            "false_alarms_oracle": none["trials"] - none["oracle_clean"],
            "detection_rate_gpu": sum(v["trials"] - v["gpu_clean"] for v in faulty) / n_faulty,
            "detection_rate_oracle": sum(v["trials"] - v["oracle_clean"] for v in faulty) / n_faulty,
            "agree": sum(v["agree"] for v in stats.values()),
            "margin_safe": sum(v["margin_safe"] for v in stats.values()),
            "mismatches_on_margin_safe_trials": mismatches, "mismatches_on_other_trials": unsafe[:32],
            "n_mismatches_on_other_trials": len(unsafe),
            "worst_corrected_C_error": worst_c, "worst_corrected_C_error_without_operand_faults": worst_c_no_operand_fault, "oracle_worst_left_in_cbar": worst_left,
            "seconds": {"oracle_setup": round(t_setup, 2), "oracle_trials_x3": round(t_oracle, 2), "gpu_trials": round(t_gpu, 2)}}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="cfg3")
    ap.add_argument("--trials", type=int, default=10000)
    ap.add_argument("--progress", type=int, default=1000)
    args = ap.parse_args()
    print(json.dumps(run(args.workload, args.trials, progress=args.progress)))


if __name__ == "__main__":
    main()
