#!/usr/bin/env python3
"""Benchmark of the protected GEMM hot path on one MI355X.

A "step" is one pass of the whole path over one batch of synthetic input that is already
resident in HBM: encode A, encode B, encoded product (data block on the MFMA units with the
fused partial-syndrome epilogue + the parity blocks), syndromes/thresholds, and the
(device-gated) correction stage.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg4-fwd]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_TFLOPS = {"bf16": 2500.0, "f32": 157.3}     # MI355X dense MFMA peaks
HBM_PEAK_GBS = 8000.0

# Memory traffic of the product kernel per launch (bytes), from rocprofv3 --pmc FETCH_SIZE and
# WRITE_SIZE runs, each scaled by what the same counter reads for a 1 GiB copy (the factors are in
# the files); profiles/bench_<workload>_hbm_traffic.txt.  Workloads not listed: not measured.
TRAFFIC_BYTES = {"cfg4-fwd": 3.051e9 + 1.003e9, "cfg4-dgrad": 6.478e9 + 6.418e8, "cfg4-wgrad": 9.478e9 + 5.606e8}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=40)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="cfg4-fwd")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--block", type=int, nargs=2, default=None, metavar=("BLOCK_N", "BLOCK_M"),
                    help="also time the blocked grid code with these block sizes (multiples of 128 dividing n, m)")
    ap.add_argument("--panels", type=int, default=0,
                    help="also time the per-k-panel path (gecc_protected_gemm_panels) with this many panels")
    ap.add_argument("--traffic-ref", action="store_true",
                    help="also run one 1 GiB device copy (untimed): the known-size kernel that "
                         "FETCH_SIZE / WRITE_SIZE counter runs are scaled by")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (--gpus 1); the path shards without "
              "communication, no multi-GPU figure is produced.", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2508_04355_amd import configs, gecc, inputs

    w = configs.ALL[args.workload]
    dev = "cuda:0"
    torch.cuda.set_device(0)
    n, k, m, batch = w.n, w.k, w.m, w.batch

    # ---- synthetic inputs (seeded), moved to HBM before any timing --------------------------
    rng = inputs.rng_for(40, 0)
    tdt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
    As, Bs = [], []
    for b in range(batch):
        A, B = inputs.operands(rng, n, k, m, w.law_a, w.law_b, w.dtype)
        As.append(A.T.copy() if w.trans_a else A)
        Bs.append(B.T.copy() if w.trans_b else B)
    hA, hB = np.stack(As), np.stack(Bs)
    dA = torch.from_numpy(hA).to(tdt).to(dev)
    dB = torch.from_numpy(hB).to(tdt).to(dev)
    ctx = gecc.Context(n, k, m, gecc.BF16 if w.dtype == "bf16" else gecc.F32, w.tau, batch=batch,
                       trans_a=w.trans_a, trans_b=w.trans_b)
    A_par, B_par, C_par = ctx.alloc_parities()
    rep = ctx.alloc_report()
    Cd = ctx.alloc_c()

    if args.traffic_ref:
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    def step():
        ctx.protected_gemm(dA, dB, Cd, A_par, B_par, C_par, rep)

    # the same product kernel without parity work, the denominator of the overhead: timed before
    # and after the protected steps and averaged, because the clock the chip settles at drifts
    # over the first hundred milliseconds of load
    def time_plain():
        for _ in range(args.warmup):
            ctx.plain_gemm(dA, dB, Cd)
        torch.cuda.synchronize()
        t = time.perf_counter()
        for _ in range(args.steps):
            ctx.plain_gemm(dA, dB, Cd)
        torch.cuda.synchronize()
        return (time.perf_counter() - t) * 1e3 / args.steps

    ms_plain_before = time_plain()
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    ctx.timing_enable(args.steps, (gecc.K_PRODUCT,))
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    gemm_ms = [ms for (_, ms) in ctx.timing_read(args.steps)]
    ctx.timing_enable(0)
    ms_step = (t1 - t0) * 1e3 / args.steps
    reports = ctx.report_to_host(rep)
    clean = all(r.status == gecc.CLEAN for r in reports)

    ms_plain = 0.5 * (ms_plain_before + time_plain())

    # ---- per-k-panel verification (optional): the same product one panel of k after the other ----
    panel_out = None
    if args.panels > 1 and batch == 1:
        import ctypes as C
        P = ctx.panel_count(args.panels)
        Cp = ctx.alloc_c()
        C_par_p = torch.empty(P * (2 * n + 2 * m + 4), dtype=torch.float64, device=dev)
        reps_p = torch.zeros(P * C.sizeof(gecc.Report), dtype=torch.uint8, device=dev)

        def pstep():
            ctx.protected_gemm_panels(dA, dB, Cd, Cp, A_par, B_par, C_par_p, reps_p, args.panels)

        for _ in range(args.warmup):
            pstep()
        torch.cuda.synchronize()
        t0p = time.perf_counter()
        for _ in range(args.steps):
            pstep()
        torch.cuda.synchronize()
        ms_p = (time.perf_counter() - t0p) * 1e3 / args.steps
        rp = ctx.reports_to_host(reps_p, P)
        panel_out = {"panels": P, "ms_per_step": round(ms_p, 4), "tflops": round(w.flops / (ms_p * 1e-3) / 1e12, 3),
                     "overhead_pct_vs_plain": round((ms_p / ms_plain - 1.0) * 100.0, 2),
                     "all_clean": all(r.status == gecc.CLEAN for r in rp)}
        del Cp

    # ---- blocked grid code (optional): Section III per block of C, thresholds of one block ---------
    block_out = None
    if args.block and batch == 1:
        nbk, mbk = args.block
        tb = gecc.noise_thresholds(nbk, k, mbk, w.sigma_a, w.sigma_b)
        ctxb = gecc.Context(n, k, m, gecc.BF16 if w.dtype == "bf16" else gecc.F32, tb, trans_a=w.trans_a,
                            trans_b=w.trans_b, block=(nbk, mbk))
        A_pb, B_pb, C_pb = ctxb.alloc_parities()
        rep_b = ctxb.alloc_report()

        def bstep():
            ctxb.protected_gemm(dA, dB, Cd, A_pb, B_pb, C_pb, rep_b)

        for _ in range(args.warmup):
            bstep()
        torch.cuda.synchronize()
        t0b = time.perf_counter()
        for _ in range(args.steps):
            bstep()
        torch.cuda.synchronize()
        ms_b = (time.perf_counter() - t0b) * 1e3 / args.steps
        rb = ctxb.report_to_host(rep_b)
        mxb = np.array([list(r.max_abs_synd) for r in rb]).max(axis=0)
        block_out = {"block": [nbk, mbk], "codewords": ctxb.items, "thresholds": [tb.r1, tb.r2, tb.q1, tb.q2],
                     "max_clean_syndromes": [float(x) for x in mxb],
                     "ms_per_step": round(ms_b, 4), "tflops": round(w.flops / (ms_b * 1e-3) / 1e12, 3),
                     "overhead_pct_vs_plain": round((ms_b / ms_plain - 1.0) * 100.0, 2),
                     "all_clean": all(r.status == gecc.CLEAN for r in rb)}
        del ctxb, A_pb, B_pb, C_pb

    # ---- HBM rooflines of the memory-bound kernels: the same steps once more with an event pair
    # around every launch (not part of `value`: the records cost stream time), then the stand-alone
    # syndrome scan of C, then the same steps on three rotating copies of the operands, so that no
    # scan finds its operand in the 256 MiB memory-side cache -----------------------------------
    s_in = 2 if w.dtype == "bf16" else 4
    ntm, ntn = -(-n // 128), -(-m // 128)
    scan_bytes = {"encode_a": s_in * n * k * batch, "encode_b": s_in * k * m * batch,
                  "parity_r": s_in * n * k * batch, "parity_c": s_in * k * m * batch,
                  "encode_a+parity_r": s_in * n * k * batch, "encode_b+parity_c": s_in * k * m * batch,
                  "threshold": 8 * (ntn * n + ntm * m) * batch, "partials": 4 * n * m * batch}
    scan_kinds = (gecc.K_ENCODE_A, gecc.K_ENCODE_B, gecc.K_PARITY_R, gecc.K_PARITY_C, gecc.K_THRESHOLD,
                  gecc.K_PARTIALS, gecc.K_STAGE2, gecc.K_DECODE, gecc.K_AUDIT_A, gecc.K_AUDIT_B, gecc.K_REPAIR,
                  gecc.K_TILE_A, gecc.K_TILE_B, gecc.K_AUDIT_AB)

    def per_kernel(run, reps):
        ctx.timing_enable(16 * reps, scan_kinds)
        for _ in range(reps):
            run()
        torch.cuda.synchronize()
        rec = ctx.timing_read(16 * reps)
        ctx.timing_enable(0)
        by = {}
        for kind, ms in rec:
            by.setdefault(gecc.K_NAMES[kind], []).append(ms * 1e3)
        return by

    def hbm_table(by):
        out = {}
        for name, us in by.items():
            e = {"launches": len(us), "us": round(float(np.mean(us)), 2)}
            if name in scan_bytes:
                e["bytes"] = scan_bytes[name]
                e["GBs"] = round(scan_bytes[name] / np.mean(us) / 1e3, 1)
                e["frac"] = round(scan_bytes[name] / (np.mean(us) * 1e-6) / (HBM_PEAK_GBS * 1e9), 4)
            out[name] = e
        return out

    reps = max(5, min(args.steps, 20))
    hbm_steady = hbm_table(per_kernel(step, reps))
    rep2 = ctx.alloc_report()
    hbm_steady.update(hbm_table({kk: v for kk, v in per_kernel(lambda: ctx.verify(Cd, C_par, rep2, fused=False), reps).items()
                                 if kk == "partials"}))
    sets = [(dA, dB)] + [(dA.clone(), dB.clone()) for _ in range(2)]
    turn = [0]

    def rotating_step():
        a_, b_ = sets[turn[0] % 3]
        turn[0] += 1
        ctx.protected_gemm(a_, b_, Cd, A_par, B_par, C_par, rep)

    for _ in range(3):
        rotating_step()
    hbm_rotated = {kk: v for kk, v in hbm_table(per_kernel(rotating_step, reps)).items() if kk in scan_bytes}
    del sets

    # ---- the paper's six scenarios (Section VI a-f): correction rate, and the time of one
    # protected product whose correction stage really runs (encode .. correct, median of 5), with
    # the grid code and in single-checksum mode (Table 1 sets the two side by side) -------------
    MA, MB, MC = inputs.MAT_A, inputs.MAT_B, inputs.MAT_C
    scen = {"a": [MA], "b": [MB], "c": [MC], "d": [MA, MC], "e": [MB, MC], "f": [MC, MC]}
    frng = inputs.rng_for(41, 0)
    Aclean, Bclean = dA.clone(), dB.clone()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    plan = {}
    for name, mats in scen.items():
        faults = inputs.draw_faults(frng, n, k, m, len(mats), w.offset_law, mats)
        cf = [(0, f.row, f.col, f.offset) for f in faults if f.matrix == MC]
        plan[name] = (faults, [(f.matrix, f.row, f.col) for f in faults], gecc.make_faults(cf, dev))
    single_tau = gecc.Thresholds(w.tau.r1, w.tau.r2, w.tau.q1, w.tau.q2, w.tau.op, w.tau.rep, w.tau.rel, weighted=False)
    ctx1 = gecc.Context(n, k, m, gecc.BF16 if w.dtype == "bf16" else gecc.F32, single_tau, batch=batch,
                        trans_a=w.trans_a, trans_b=w.trans_b)
    STATUS = {gecc.CLEAN: "clean", gecc.CORRECTED: "corrected", gecc.UNCORRECTABLE: "uncorrectable", gecc.DETECTED: "detected"}

    def run_scenarios(cx):
        times = {name: [] for name in scen}
        good = {name: True for name in scen}
        status = {}
        for rnd in range(6):            # pass 0 untimed: it loads the kernels of the staged calls
            if rnd == 1:                # ... and the chip needs a few products to be back at its steady clock
                for _ in range(args.warmup):
                    cx.plain_gemm(dA, dB, Cd)
            for name in scen:
                faults, want, (fl, nf) = plan[name]
                ev0.record()
                cx.encode_a(dA, A_par)
                cx.encode_b(dB, B_par)
                for f in faults:        # E1/E2 strike after encoding (tiny torch kernels inside the timed span); E3 inside the product
                    if f.matrix != MC:
                        T, tr = (dA, w.trans_a) if f.matrix == MA else (dB, w.trans_b)
                        i, j = (f.col, f.row) if tr else (f.row, f.col)
                        T[0, i, j] += f.offset
                cx.multiply(dA, A_par, dB, B_par, Cd, C_par, fl, nf)
                cx.verify(Cd, C_par, rep, fused=True)
                cx.correct(dA, A_par, dB, B_par, Cd, C_par, rep)
                ev1.record()
                r = cx.report_to_host(rep)[0]
                if rnd > 0:
                    times[name].append(ev0.elapsed_time(ev1))
                got = [(e[0], e[1], e[2]) for e in r.errors()]
                restored = bool(torch.equal(dA, Aclean) and torch.equal(dB, Bclean))
                good[name] = good[name] and r.status == gecc.CORRECTED and got == sorted(want) and restored
                status[name] = STATUS[r.status]
                dA.copy_(Aclean)
                dB.copy_(Bclean)
        return good, {name: round(float(np.median(t)), 4) for name, t in times.items()}, status

    good, scen_ms, _ = run_scenarios(ctx)
    good1, scen_ms1, status1 = run_scenarios(ctx1)
    n_tot, n_ok = len(scen), sum(int(v) for v in good.values())

    flops = w.flops
    value = flops / (ms_step * 1e-3) / 1e12
    plain = flops / (ms_plain * 1e-3) / 1e12
    g_ms = float(np.mean(gemm_ms)) if gemm_ms else None
    achieved = flops / (g_ms * 1e-3) / 1e12 if g_ms else None
    peak = PEAK_TFLOPS[w.dtype]
    out = {
        "metric": "protected_gemm_tflops", "value": round(value, 3), "unit": "TFLOP/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": w.dtype,
        "data": "synthetic",
        "config": {"workload": "%s: A[%dx%d] B[%dx%d] batch %d, %s inputs, fp32 accumulate, "
                               "trans_a=%d trans_b=%d" % (w.name, n, k, k, m, batch, w.dtype, w.trans_a, w.trans_b),
                   "thresholds": [w.tau.r1, w.tau.r2, w.tau.q1, w.tau.q2]},
        "plain_gemm_tflops": round(plain, 3),
        "overhead_pct": round((ms_step / ms_plain - 1.0) * 100.0, 2),
        "all_clean_reported_clean": clean,
        "correction_rate": {"scenarios": "a,b,c,d,e,f (Section VI)", "corrected": n_ok, "trials": n_tot},
        "scenario_ms": scen_ms,
        "scenario_overhead_pct": {kk: round((vv / ms_plain - 1.0) * 100.0, 1) for kk, vv in scen_ms.items()},
        "single_checksum_mode": {"corrected": sum(int(v) for v in good1.values()), "trials": n_tot, "status": status1,
                                 "scenario_ms": scen_ms1,
                                 "scenario_overhead_pct": {kk: round((vv / ms_plain - 1.0) * 100.0, 1) for kk, vv in scen_ms1.items()}},
        "per_k_panel_verification": panel_out,
        "blocked_grid_code": block_out,
        # event pairs recorded per clean step outside the product (the product is one more, two with a k-split tail)
        "launches_per_step_without_product": round(sum(v["launches"] for kk, v in hbm_steady.items() if kk != "partials") / reps, 2),
        "hbm_rooflines": {"peak_GBs": HBM_PEAK_GBS,
                          "steady_loop": hbm_steady,       # as in the timed steps: operands may sit in the memory-side cache
                          "operands_rotated": hbm_rotated},  # three operand sets in turn: every first read comes from HBM
        "roofline": {"bound": "mfma", "kernel": ("gemm_bf16_256" if w.dtype == "bf16" and min(n, m) >= 256 and k % 64 == 0 else "gemm_kernel") + " (data block + fused syndrome partials)",
                     "achieved": round(achieved, 3) if achieved else None, "peak": peak, "unit": "TFLOP/s",
                     "frac": round(achieved / peak, 4) if achieved else None,
                     "kernel_ms": round(g_ms, 4) if g_ms else None,
                     "algorithmic_flops_per_launch": flops,
                     "traffic": TRAFFIC_BYTES.get(w.name)},
    }

    # ---- CPU baseline: the oracle as it stands, on a bounded sample of the same workload -----
    if not args.no_cpu_baseline:
        from oracle import grid_code as oc
        rows = max(1, min(n, int(6e12 / (2.0 * k * m))))       # up to about 6 TFLOP of fp64 work (10-20 s)
        A0 = (hA[0].T if w.trans_a else hA[0])[:rows]
        B0 = hB[0].T if w.trans_b else hB[0]
        tau = oc.Thresholds(w.tau.r1, w.tau.r2, w.tau.q1, w.tau.q2, w.tau.op, w.tau.rep, w.tau.rel)
        t0 = time.perf_counter()
        res = oc.protected_gemm(A0, B0, A0, B0, [], tau)
        dt = time.perf_counter() - t0
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
        except Exception:
            cores = os.cpu_count()
        cpu_model = "unknown"
        try:
            for line in open("/proc/cpuinfo"):
                if line.startswith("model name"):
                    cpu_model = line.split(":", 1)[1].strip()
                    break
        except OSError:
            pass
        out["cpu_baseline"] = {"value": round(2.0 * rows * k * m / dt / 1e12, 4), "unit": "TFLOP/s",
                               "cores": cores, "cpu": cpu_model, "kind": "oracle",
                               "sample": "oracle.protected_gemm (fp64 numpy: encode, product, syndromes, "
                                         "decode) on the first %d of %d rows of A times the full B, "
                                         "batch item 0, no faults, %.1f s" % (rows, n, dt),
                               "status": int(res.status)}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
