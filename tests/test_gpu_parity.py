"""GPU parity: the HIP path (through the C ABI) against the CPU oracle on identical seeded inputs.

Bar: status, located positions: bit-exact.  Corrected C: max |C - C_oracle| / max |C_oracle|
<= 1e-5 (fp32 inputs) / 2e-2 (bf16 inputs, fp32 accumulation), checked at 1e-5 for both since
the oracle consumes the same bf16-rounded inputs.  Parity buffers (fp64): relative 1e-12.
"""
import numpy as np
import pytest

import gpu_harness as H
from oracle import grid_code as oc
from paper_2508_04355_amd import configs, gecc, inputs

pytestmark = pytest.mark.gpu

MAT_A, MAT_B, MAT_C = inputs.MAT_A, inputs.MAT_B, inputs.MAT_C


def _sigma(law):
    return law[1] if law[0] == "normal" else (law[2] - law[1]) / 12 ** 0.5


def _trial(rng, n, k, m, dtype, law_a, law_b, faults):
    A, B = inputs.operands(rng, n, k, m, law_a, law_b, dtype)
    A2, B2, cf, eff = inputs.apply_operand_faults(A, B, faults, dtype)
    return A, B, A2, B2, cf, eff


# ---------------------------------------------------------------------------------------------
# the last two reach the 256 x 256-tile bf16 kernel (k % 64 == 0, rows of 8 elements) with ragged
# tiles on both edges; everything else goes to the generic kernel
SHAPES = [(128, 128, 128), (1, 1, 1), (3, 5, 2), (130, 70, 257), (300, 200, 260), (257, 1031, 129),
          (520, 256, 264), (1000, 320, 776),
          (520, 64, 264), (264, 192, 520)]    # the 256 x 256 bf16 kernel at its shortest k (one pair of k-tiles), and three pairs


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("trans", [(0, 0), (0, 1), (1, 0), (1, 1)])
@pytest.mark.parametrize("shape", SHAPES)
def test_clean_product_blocks_match_the_oracle(shape, trans, dtype):
    n, k, m = shape
    rng = inputs.rng_for(90, n + 7 * k + 13 * m)
    law = ("normal", 1.0)
    A, B = inputs.operands(rng, n, k, m, law, law, dtype)
    tau = gecc.noise_thresholds(n, k, m, 1.0, 1.0)
    g = H.run_gpu(A, B, A, B, [], tau, dtype, trans[0], trans[1])
    AP, BP = oc.encode_a(A), oc.encode_b(B)
    Cbar = oc.encoded_product(A, AP, B, BP)
    assert g.reports[0].status == gecc.CLEAN and g.reports[0].n_err == 0
    assert np.allclose(g.A_par[0], AP, rtol=1e-12, atol=1e-12 * np.abs(AP).max())
    assert np.allclose(g.B_par[0], BP.T, rtol=1e-12, atol=1e-12 * np.abs(BP).max())
    ref = np.concatenate([Cbar[:n, m], Cbar[:n, m + 1], Cbar[n, :m], Cbar[n + 1, :m], Cbar[n:, m:].ravel()])
    assert np.allclose(g.C_par[0], ref, rtol=1e-11, atol=1e-12 * np.abs(ref).max())
    scale = max(np.abs(Cbar[:n, :m]).max(), 1e-30)
    assert np.abs(g.C[0] - Cbar[:n, :m]).max() / scale <= 1e-5
    # syndromes (fp32 sums of an fp32 product) stay far inside the thresholds
    mx = g.reports[0].max_abs_synd
    assert mx[0] <= tau.r1 / 2 and mx[1] <= tau.r2 / 2 and mx[2] <= tau.q1 / 2 and mx[3] <= tau.q2 / 2


@pytest.mark.parametrize("trans", [(0, 0), (0, 1), (1, 0), (1, 1)])
@pytest.mark.parametrize("pattern", ["C+C on the edges", "A+C", "B+C", "A+B"])
def test_ragged_tiles_of_the_fast_bf16_kernel_with_errors(pattern, trans):
    """Faults in the last row / column of C and of the operands, where the 256 x 256 tiles of the
    bf16 kernel hang over the edge (range-checked stores, zero-filled operand rows)."""
    n, k, m = 520, 256, 264
    rng = inputs.rng_for(92, 0)
    law = ("normal", 1.0)
    faults = {"C+C on the edges": [inputs.Fault(MAT_C, n - 1, m - 1, 37.5), inputs.Fault(MAT_C, 256, 0, -12.25)],
              "A+C": [inputs.Fault(MAT_A, n - 1, k - 1, 3.0), inputs.Fault(MAT_C, 0, m - 1, 55.0)],
              "B+C": [inputs.Fault(MAT_B, k - 1, m - 1, -2.5), inputs.Fault(MAT_C, n - 1, 257, 9.0)],
              "A+B": [inputs.Fault(MAT_A, 512, 0, 4.0), inputs.Fault(MAT_B, 0, 256, 6.0)]}[pattern]
    A, B, A2, B2, cf, eff = _trial(rng, n, k, m, "bf16", law, law, faults)
    tau = gecc.noise_thresholds(n, k, m, 1.0, 1.0)
    cfb = [(0,) + c for c in cf]
    g = H.run_gpu(A, B, A2, B2, cfb, tau, "bf16", trans[0], trans[1])
    o = H.run_oracle(A, B, A2, B2, cfb, tau)
    H.compare(g, o, 1e-5, what="ragged fast kernel, %s, trans %s" % (pattern, trans))
    assert g.reports[0].status == gecc.CORRECTED
    assert [(e[0], e[1], e[2]) for e in g.reports[0].errors()] == [(e[0], e[1], e[2]) for e in eff]


@pytest.mark.parametrize("trans", [(0, 0), (0, 1), (1, 0), (1, 1)])
@pytest.mark.parametrize("dtype,shape,batch", [("f32", (520, 1024, 264), 1), ("bf16", (200, 1024, 136), 1), ("f32", (300, 520, 260), 2)])
@pytest.mark.parametrize("pattern", ["clean", "C+C", "A+C", "B+C"])
def test_k_split_of_products_with_few_tiles(pattern, dtype, shape, batch, trans):
    """Products with far fewer 128 x 128 tiles than compute units split k over up to 8 workgroups per
    tile; the one that finishes last adds the partial tiles up in the order of the k ranges, so the
    result is the same bits whichever that is, and everything downstream is as for one workgroup."""
    n, k, m = shape
    rng = inputs.rng_for(97, trans[0] * 2 + trans[1])
    law = ("normal", 1.0)
    faults = {"clean": [], "C+C": [inputs.Fault(MAT_C, n - 1, m - 1, 37.5), inputs.Fault(MAT_C, 3, 129, -12.25)],
              "A+C": [inputs.Fault(MAT_A, n - 1, k - 1, 3.0), inputs.Fault(MAT_C, 0, m - 1, 55.0)],
              "B+C": [inputs.Fault(MAT_B, k // 2, m - 1, -2.5), inputs.Fault(MAT_C, n - 1, 5, 9.0)]}[pattern]
    trials = [_trial(rng, n, k, m, dtype, law, law, faults) for _ in range(batch)]
    A, B, A2, B2 = [np.stack([t[x] for t in trials]) for x in range(4)]
    cfb = [(b,) + c for b, t in enumerate(trials) for c in t[4]]
    tau = gecc.noise_thresholds(n, k, m, 1.0, 1.0)
    g = H.run_gpu(A, B, A2, B2, cfb, tau, dtype, trans[0], trans[1])
    o = H.run_oracle(A, B, A2, B2, cfb, tau)
    H.compare(g, o, 1e-5, what="k-split, %s, %s, trans %s" % (pattern, shape, trans))
    g2 = H.run_gpu(A, B, A2, B2, cfb, tau, dtype, trans[0], trans[1])
    assert np.array_equal(g.C, g2.C) and np.array_equal(g.synd, g2.synd)


@pytest.mark.parametrize("trans", [(0, 0), (0, 1), (1, 0), (1, 1)])
@pytest.mark.parametrize("dtype,shape", [("bf16", (520, 256, 264)), ("bf16", (1000, 520, 776)), ("f32", (300, 200, 260)),
                                         ("bf16", (2200, 136, 72))])
@pytest.mark.parametrize("pattern", ["clean", "A+C", "B+C", "A+B"])
def test_one_pass_scan_on_small_and_ragged_shapes(pattern, dtype, shape, trans, monkeypatch):
    """The scan that reads an operand once for both of its reductions (rows straight into LDS, a last
    column segment narrower than the others, chunks of rows that end in the middle of a block) serves
    operands of 2^25 elements or more; GECC_TILE_MIN = 1 lets it serve these small ones, staged calls
    and the one-call chain alike, and the audit re-forms the same sums bit for bit."""
    monkeypatch.setenv("GECC_TILE_MIN", "1")
    try:
        n, k, m = shape
        rng = inputs.rng_for(93, trans[0] * 2 + trans[1])
        law = ("normal", 1.0)
        faults = {"clean": [],
                  "A+C": [inputs.Fault(MAT_A, n - 1, k - 1, 3.0), inputs.Fault(MAT_C, 0, m - 1, 55.0)],
                  "B+C": [inputs.Fault(MAT_B, k - 1, m - 1, -2.5), inputs.Fault(MAT_C, n - 1, m // 2, 9.0)],
                  "A+B": [inputs.Fault(MAT_A, n // 2, 0, 4.0), inputs.Fault(MAT_B, 0, m // 3, 6.0)]}[pattern]
        A, B, A2, B2, cf, eff = _trial(rng, n, k, m, dtype, law, law, faults)
        tau = gecc.noise_thresholds(n, k, m, 1.0, 1.0)
        cfb = [(0,) + c for c in cf]
        g = H.run_gpu(A, B, A2, B2, cfb, tau, dtype, trans[0], trans[1])
        o = H.run_oracle(A, B, A2, B2, cfb, tau)
        H.compare(g, o, 1e-5, what="one-pass scan, %s, %s, trans %s" % (pattern, shape, trans))
        assert [(e[0], e[1], e[2]) for e in g.reports[0].errors()] == [(e[0], e[1], e[2]) for e in eff]
        if pattern == "clean":
            g2 = H.run_gpu(A, B, A, B, [], tau, dtype, trans[0], trans[1], staged=False)
            assert np.array_equal(g.A_par, g2.A_par) and np.array_equal(g.B_par, g2.B_par) and np.array_equal(g.C, g2.C)
            assert np.allclose(g.C_par, g2.C_par, rtol=1e-12, atol=1e-13 * np.abs(g.C_par).max())
    finally:
        monkeypatch.delenv("GECC_TILE_MIN")


@pytest.mark.parametrize("trans", [(0, 0), (0, 1), (1, 0), (1, 1)])
@pytest.mark.parametrize("shape,cus", [((520, 256, 264), 4), ((520, 128, 264), 4), ((1000, 512, 776), 12)])
@pytest.mark.parametrize("pattern", ["clean", "C+C in split tiles", "A+C", "B+C", "C outside the split tiles"])
def test_k_split_tail_of_the_fast_bf16_kernel(pattern, shape, cus, trans, monkeypatch):
    """A last round of tiles that is at most half full is shared out over two workgroups per tile,
    one per half of k, which add into zeroed C and partial sums.  GECC_CU_COUNT (read when the
    context is created) makes the launcher plan as for that many compute units, so that small
    shapes reach this path: 6 tiles on 4 -> tiles 4, 5 are split; 16 on 12 -> tiles 12..15."""
    monkeypatch.setenv("GECC_CU_COUNT", str(cus))
    n, k, m = shape
    rng = inputs.rng_for(93, n + k)
    law = ("normal", 1.0)
    faults = {"clean": [],
              "C+C in split tiles": [inputs.Fault(MAT_C, n - 1, m - 1, 37.5), inputs.Fault(MAT_C, n - 200, m - 3, -12.25)],
              "A+C": [inputs.Fault(MAT_A, n - 1, k - 1, 3.0), inputs.Fault(MAT_C, n - 7, m - 2, 55.0)],
              "B+C": [inputs.Fault(MAT_B, k // 2, m - 1, -2.5), inputs.Fault(MAT_C, n - 1, m - 8, 9.0)],
              "C outside the split tiles": [inputs.Fault(MAT_C, 3, 5, 21.0), inputs.Fault(MAT_C, 100, 200, -8.0)]}[pattern]
    A, B, A2, B2, cf, eff = _trial(rng, n, k, m, "bf16", law, law, faults)
    tau = gecc.noise_thresholds(n, k, m, 1.0, 1.0)
    cfb = [(0,) + c for c in cf]
    g = H.run_gpu(A, B, A2, B2, cfb, tau, "bf16", trans[0], trans[1])
    o = H.run_oracle(A, B, A2, B2, cfb, tau)
    H.compare(g, o, 1e-5, what="k-split tail, %s, trans %s" % (pattern, trans))
    assert g.reports[0].status == (gecc.CORRECTED if faults else gecc.CLEAN)
    assert [(e[0], e[1], e[2]) for e in g.reports[0].errors()] == [(e[0], e[1], e[2]) for e in eff]
    AP, BP = oc.encode_a(A), oc.encode_b(B)
    Cbar = oc.encoded_product(A, AP, B, BP)
    ref = np.concatenate([Cbar[:n, m], Cbar[:n, m + 1], Cbar[n, :m], Cbar[n + 1, :m], Cbar[n:, m:].ravel()])
    assert np.allclose(g.C_par[0], ref, rtol=1e-11, atol=1e-12 * np.abs(ref).max())
    # two terms added onto zero: the order of arrival cannot show
    g2 = H.run_gpu(A, B, A2, B2, cfb, tau, "bf16", trans[0], trans[1])
    assert np.array_equal(g.C, g2.C) and np.array_equal(g.synd, g2.synd)
    if pattern == "clean":      # the one-call chain takes the same launches
        g3 = H.run_gpu(A, B, A, B, [], tau, "bf16", trans[0], trans[1], staged=False)
        assert np.array_equal(g.C, g3.C) and g3.reports[0].status == gecc.CLEAN
        # and the split changes C only by the rounding of one more fp32 addition per element
        monkeypatch.delenv("GECC_CU_COUNT")
        g4 = H.run_gpu(A, B, A, B, [], tau, "bf16", trans[0], trans[1])
        assert not np.array_equal(g.C, g4.C)
        assert np.abs(g.C - g4.C).max() <= 4e-6 * np.abs(g4.C).max()
        split_rows = np.any(g.C[0] != g4.C[0], axis=1)
        assert not split_rows[:256].any()          # tile row 0 is in the full rounds either way


# ---- Theorem 2: many errors in at most two rows (or columns) of C ---------------------------------
def _t2_faults(rng, lines, others, n_other, frac, rows_known):
    faults = []
    for ln in lines:
        cols = rng.choice(n_other, size=max(3, int(frac * n_other)), replace=False) if others is None else others
        for c in sorted(int(x) for x in cols):
            e = float(rng.uniform(1.0, 100.0) * rng.choice([-1.0, 1.0]))
            faults.append(inputs.Fault(MAT_C, ln, c, e) if rows_known else inputs.Fault(MAT_C, c, ln, e))
    return faults


@pytest.mark.parametrize("case", ["one row, 40 columns", "two rows, 25 columns each", "one column, 60 rows",
                                  "two adjacent columns, 30 rows each", "a whole row"])
@pytest.mark.parametrize("dtype,shape", [("f32", (257, 96, 300)), ("bf16", (520, 256, 264))])
def test_theorem2_patterns(case, dtype, shape):
    """Errors in any number of columns of at most two flagged rows (and the mirror image) are
    removed by Section V's subtraction, line by line; the report lists the first eight and
    counts all.  Corrected symbols carry the rounding noise of the syndromes they were
    computed from (no re-evaluation for these patterns): tolerance tau_1 / max |C|."""
    n, k, m = shape
    rng = inputs.rng_for(93, len(case))
    law = ("normal", 1.0)
    if case == "one row, 40 columns":
        faults = _t2_faults(rng, [n - 1], None, m, 40 / m, True)
    elif case == "two rows, 25 columns each":
        faults = _t2_faults(rng, [3, 200], None, m, 25 / m, True)
    elif case == "one column, 60 rows":
        faults = _t2_faults(rng, [m - 1], None, n, 60 / n, False)
    elif case == "two adjacent columns, 30 rows each":
        faults = _t2_faults(rng, [128, 129], None, n, 30 / n, False)
    else:
        faults = _t2_faults(rng, [129], list(range(m)), m, 1.0, True)
    A, B, A2, B2, cf, eff = _trial(rng, n, k, m, dtype, law, law, faults)
    tau = gecc.noise_thresholds(n, k, m, 1.0, 1.0)
    cfb = [(0,) + c for c in cf]
    g = H.run_gpu(A, B, A2, B2, cfb, tau, dtype)
    o = H.run_oracle(A, B, A2, B2, cfb, tau)
    scale = float(np.max(np.abs(o[0].C)))
    # two known lines: the 2x2 system divides the weighted syndrome by the distance of the lines
    tol = 4 * (max(tau.r1, tau.q1) + (max(tau.r2, tau.q2) if "two" in case else 0.0)) / scale
    H.compare(g, o, tol, tol_mag=tol * scale, what="theorem 2, " + case)
    assert g.reports[0].status == gecc.CORRECTED
    assert g.reports[0].n_total == len(faults) and g.reports[0].n_err == 8
    # every symbol outside the corrupted lines is the plain product to the usual tolerance
    mask = np.ones((n, m), dtype=bool)
    for f in faults:
        mask[f.row, f.col] = False
    assert np.max(np.abs(g.C[0] - o[0].C)[mask]) / scale <= 1e-5


def test_recomputation_after_an_uncorrectable_pattern():
    """Section V: a pattern beyond the code is recalculated.  Three transient C faults on a
    diagonal (s = t = 3) make the first product UNCORRECTABLE; the second one is clean."""
    n, k, m = 300, 128, 280
    rng = inputs.rng_for(94)
    A, B = inputs.operands(rng, n, k, m, ("normal", 1.0), ("normal", 1.0), "bf16")
    tau = gecc.noise_thresholds(n, k, m, 1.0, 1.0)
    ctx = gecc.Context(n, k, m, gecc.BF16, gecc.Thresholds(tau.r1, tau.r2, tau.q1, tau.q2))
    dA, dB = H.to_dev(A[None], "bf16", False), H.to_dev(B[None], "bf16", False)
    A_par, B_par, C_par = ctx.alloc_parities()
    rep, Cd = ctx.alloc_report(), ctx.alloc_c()
    fl, nf = gecc.make_faults([(0, 10, 20, 50.0), (0, 100, 120, -30.0), (0, 299, 279, 70.0)], H.DEV)
    ref = A.astype(np.float64) @ B.astype(np.float64)
    reports, attempts = ctx.protected_gemm_retry(dA, dB, Cd, A_par, B_par, C_par, rep, 0, fl, nf)
    assert attempts == 1 and reports[0].status == gecc.UNCORRECTABLE and reports[0].s == 3 and reports[0].t == 3
    reports, attempts = ctx.protected_gemm_retry(dA, dB, Cd, A_par, B_par, C_par, rep, 2, fl, nf)
    assert attempts == 2 and reports[0].status == gecc.CLEAN
    assert np.max(np.abs(Cd[0].cpu().numpy() - ref)) / np.max(np.abs(ref)) <= 1e-5


@pytest.mark.parametrize("trans", [(0, 0), (0, 1), (1, 0), (1, 1)])
@pytest.mark.parametrize("dtype,shape,batch", [("f32", (300, 200, 260), 2), ("bf16", (520, 256, 264), 3)])
def test_one_call_chain_equals_the_staged_calls_bit_for_bit(dtype, shape, batch, trans):
    """gecc_protected_gemm orders its parity scans by storage layout, lets row scans carry the second
    stage of column scans and reads the larger operand once for both of its reductions.  None of that
    may change a bit of C, of the operand parities (the audit re-forms them and tests for equality) or
    of a decision; the parity blocks of C-bar, fp64 sums taken in another order by the one-pass scan,
    agree to rounding."""
    n, k, m = shape
    rng = inputs.rng_for(95, trans[0] * 2 + trans[1])
    A = np.stack([inputs.operands(rng, n, k, m, ("normal", 1.0), ("normal", 1.0), dtype)[0] for _ in range(batch)])
    B = np.stack([inputs.operands(rng, n, k, m, ("normal", 1.0), ("normal", 1.0), dtype)[1] for _ in range(batch)])
    tau = gecc.noise_thresholds(n, k, m, 1.0, 1.0)
    cf = [(b, 7 + b, 250, 40.0) for b in range(batch)] + [(0, n - 1, 3, -25.0)]
    g1 = H.run_gpu(A, B, A, B, cf, tau, dtype, trans[0], trans[1], staged=True)
    g2 = H.run_gpu(A, B, A, B, cf, tau, dtype, trans[0], trans[1], staged=False)
    for name in ("A_par", "B_par", "C"):
        assert np.array_equal(getattr(g1, name), getattr(g2, name)), name
    assert np.allclose(g1.C_par, g2.C_par, rtol=1e-12, atol=1e-13 * np.abs(g1.C_par).max())
    assert np.allclose(g1.synd, g2.synd, rtol=0, atol=1e-11 * np.abs(g1.C_par).max())
    for r1, r2 in zip(g1.reports, g2.reports):
        assert (r1.status, r1.n_total, r1.errors()) == (r2.status, r2.n_total, r2.errors())
    H.compare(g2, H.run_oracle(A, B, A, B, cf, tau), 1e-5, what="one call")


def test_two_contexts_on_two_streams_do_not_disturb_each_other():
    """Every call takes the caller's stream and the library keeps all its state in the context's
    own workspace: two products enqueued alternately on two side streams give the results of the
    same products run alone on the default stream, bit for bit."""
    import torch
    shapes = [("bf16", (520, 256, 264), [(0, 17, 200, 30.0)]), ("f32", (300, 200, 260), [(0, 5, 6, -12.0), (0, 299, 1, 8.0)])]
    alone, jobs = [], []
    for idx, (dtype, (n, k, m), cf) in enumerate(shapes):
        rng = inputs.rng_for(96, idx)
        A, B = inputs.operands(rng, n, k, m, ("normal", 1.0), ("normal", 1.0), dtype)
        tau = gecc.noise_thresholds(n, k, m, 1.0, 1.0)
        alone.append(H.run_gpu(A, B, A, B, cf, tau, dtype, staged=True))
        ctx = gecc.Context(n, k, m, gecc.BF16 if dtype == "bf16" else gecc.F32,
                           gecc.Thresholds(tau.r1, tau.r2, tau.q1, tau.q2, tau.op, tau.rep, tau.rel))
        dA, dB = H.to_dev(A[None], dtype, False), H.to_dev(B[None], dtype, False)
        par = ctx.alloc_parities()
        jobs.append((ctx, dA, dB, ctx.alloc_c(), par, ctx.alloc_report(), gecc.make_faults(cf, H.DEV), torch.cuda.Stream()))
    torch.cuda.synchronize()
    for rnd in range(3):                                  # interleaved, nothing waits in between
        for (ctx, dA, dB, Cd, par, rep, (fl, nf), st) in jobs:
            with torch.cuda.stream(st):
                ctx.encode_a(dA, par[0])
                ctx.encode_b(dB, par[1])
                ctx.multiply(dA, par[0], dB, par[1], Cd, par[2], fl, nf)
                ctx.verify(Cd, par[2], rep, fused=True)
                ctx.correct(dA, par[0], dB, par[1], Cd, par[2], rep)
    torch.cuda.synchronize()
    for (ctx, dA, dB, Cd, par, rep, _, st), ref in zip(jobs, alone):
        with torch.cuda.stream(st):
            r = ctx.report_to_host(rep)[0]
        assert (r.status, r.errors()) == (ref.reports[0].status, ref.reports[0].errors())
        assert np.array_equal(Cd.cpu().numpy().astype(np.float64)[:, :, :ref.C.shape[2]], ref.C)
        assert np.array_equal(par[2].cpu().numpy().reshape(1, -1), ref.C_par)


def test_the_staged_chain_replays_from_a_captured_graph():
    """Nothing on the path allocates, synchronises or clears memory with a memset node, so the
    whole chain can be captured into a HIP graph.  Every replay (with eager work and a fresh fault
    list between them) has to give what the eager calls give for the same faults."""
    import torch
    n, k, m = 520, 256, 264
    rng = inputs.rng_for(97)
    A, B = inputs.operands(rng, n, k, m, ("normal", 1.0), ("normal", 1.0), "bf16")
    tau = gecc.noise_thresholds(n, k, m, 1.0, 1.0)
    ctx = gecc.Context(n, k, m, gecc.BF16, gecc.Thresholds(tau.r1, tau.r2, tau.q1, tau.q2, tau.op, tau.rep, tau.rel))
    dA, dB = H.to_dev(A[None], "bf16", False), H.to_dev(B[None], "bf16", False)
    A_par, B_par, C_par = ctx.alloc_parities()
    rep, Cd = ctx.alloc_report(), ctx.alloc_c()
    fl, nf = gecc.make_faults([(0, 1, 2, 10.0), (0, 3, 4, 10.0)], H.DEV)      # two slots, rewritten below

    def chain():
        ctx.encode_a(dA, A_par)
        ctx.encode_b(dB, B_par)
        ctx.multiply(dA, A_par, dB, B_par, Cd, C_par, fl, nf)
        ctx.verify(Cd, C_par, rep, fused=True)
        ctx.correct(dA, A_par, dB, B_par, Cd, C_par, rep)

    def plant(cases):
        new, _ = gecc.make_faults(cases, H.DEV)
        fl.copy_(new)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        chain()                                           # first launches configure the kernels
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        chain()
    patterns = [[(0, 10, 20, 40.0), (0, 300, 100, -25.0)], [(0, 519, 263, 33.0), (0, 0, 0, 17.0)],
                [(0, 77, 5, -60.0), (0, 77, 200, 21.0)]]
    for cases in patterns:
        plant(cases)
        Cd.fill_(float("nan"))
        chain()
        eager_rep = ctx.report_to_host(rep)[0]
        eager_C = Cd.clone()
        eager_par = C_par.clone()
        Cd.fill_(float("nan"))
        rep.zero_()
        graph.replay()
        r = ctx.report_to_host(rep)[0]
        assert r.status == gecc.CORRECTED and sorted((e[1], e[2]) for e in r.errors()) == sorted((c[1], c[2]) for c in cases)
        assert (r.status, r.errors()) == (eager_rep.status, eager_rep.errors())
        assert torch.equal(Cd, eager_C) and torch.equal(C_par, eager_par)


def test_last_arrival_counters_survive_graph_replays():
    """The k-split of a small product and the paired audits count workgroups at counters in the workspace
    that the last arrival wraps back to zero.  A captured chain with an operand fault (so that the audits
    really run) is replayed several times, with eager runs in between; every replay has to give what the
    eager calls give."""
    import torch
    n, k, m = 520, 1024, 264
    rng = inputs.rng_for(98)
    A, B = inputs.operands(rng, n, k, m, ("normal", 1.0), ("normal", 1.0), "f32")
    A_bad = A.copy()
    A_bad[333, 700] += 6.0
    tau = gecc.noise_thresholds(n, k, m, 1.0, 1.0)
    ctx = gecc.Context(n, k, m, gecc.F32, gecc.Thresholds(tau.r1, tau.r2, tau.q1, tau.q2, tau.op, tau.rep, tau.rel))
    good, bad = H.to_dev(A[None], "f32", False), H.to_dev(A_bad[None], "f32", False)
    dA, dB = good.clone(), H.to_dev(B[None], "f32", False)
    A_par, B_par, C_par = ctx.alloc_parities()
    rep, Cd = ctx.alloc_report(), ctx.alloc_c()
    fl, nf = gecc.make_faults([(0, 1, 2, 10.0)], H.DEV)

    def chain():
        dA.copy_(good)
        ctx.encode_a(dA, A_par)
        ctx.encode_b(dB, B_par)
        dA.copy_(bad)                                     # E1: after the parities were formed
        ctx.multiply(dA, A_par, dB, B_par, Cd, C_par, fl, nf)
        ctx.verify(Cd, C_par, rep, fused=True)
        ctx.correct(dA, A_par, dB, B_par, Cd, C_par, rep)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        chain()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        chain()
    for case in [(0, 10, 20, 40.0), (0, 519, 263, -33.0), (0, 77, 5, 21.0)]:
        new, _ = gecc.make_faults([case], H.DEV)
        fl.copy_(new)
        Cd.fill_(float("nan"))
        chain()
        eager_rep = ctx.report_to_host(rep)[0]
        eager_C, eager_A = Cd.clone(), dA.clone()
        Cd.fill_(float("nan"))
        rep.zero_()
        graph.replay()
        r = ctx.report_to_host(rep)[0]
        assert r.status == gecc.CORRECTED
        assert sorted((e[0], e[1], e[2]) for e in r.errors()) == sorted([(MAT_A, 333, 700), (MAT_C, case[1], case[2])])
        assert (r.status, r.errors()) == (eager_rep.status, eager_rep.errors())
        assert torch.equal(Cd, eager_C) and torch.equal(dA, eager_A) and torch.equal(dA, good)


def test_two_contexts_share_one_workspace_in_stream_order():
    """Contexts of different shapes may take turns on one workspace (the counters sit at its front in
    every layout and every launch leaves them at zero): alternating calls give what each context gives
    on a workspace of its own."""
    import torch
    jobs = []
    for idx, (dtype, (n, k, m)) in enumerate([("f32", (520, 1024, 264)), ("bf16", (520, 256, 264)), ("f32", (300, 200, 260))]):
        rng = inputs.rng_for(94, idx)
        A, B = inputs.operands(rng, n, k, m, ("normal", 1.0), ("normal", 1.0), dtype)
        tau = gecc.noise_thresholds(n, k, m, 1.0, 1.0)
        cf = [(0, 5 + idx, 6, -12.0), (0, n - 1, 1 + idx, 8.0)]
        alone = H.run_gpu(A, B, A, B, cf, tau, dtype, staged=False)
        ctx = gecc.Context(n, k, m, gecc.BF16 if dtype == "bf16" else gecc.F32,
                           gecc.Thresholds(tau.r1, tau.r2, tau.q1, tau.q2, tau.op, tau.rep, tau.rel))
        jobs.append((ctx, H.to_dev(A[None], dtype, False), H.to_dev(B[None], dtype, False), ctx.alloc_c(), ctx.alloc_parities(),
                     ctx.alloc_report(), gecc.make_faults(cf, H.DEV), alone))
    need = max(gecc.lib().gecc_workspace_bytes(j[0]._h) for j in jobs)
    shared = torch.empty(need + 256, dtype=torch.uint8, device=H.DEV)
    shared.fill_(0xA5)                                    # garbage: the first call has to clear the counters
    base = shared.data_ptr() + (-shared.data_ptr()) % 256
    import ctypes as C
    for j in jobs:
        assert gecc.lib().gecc_set_workspace(j[0]._h, C.c_void_p(base), need) == 0
    for rnd in range(3):
        for (ctx, dA, dB, Cd, par, rep, (fl, nf), alone) in jobs:
            Cd.fill_(float("nan"))
            reports, attempts = ctx.protected_gemm_retry(dA, dB, Cd, par[0], par[1], par[2], rep, 0, fl, nf)
            assert attempts == 1 and reports[0].status == gecc.CORRECTED == alone.reports[0].status
            assert reports[0].errors() == alone.reports[0].errors()
            assert np.array_equal(Cd.cpu().numpy().astype(np.float64)[:, :, :ctx.m], alone.C)
            assert np.array_equal(par[0].cpu().numpy().reshape(1, 2, -1), alone.A_par)


def test_unaligned_leading_dimensions_take_the_scalar_paths():
    n, k, m = 67, 45, 83
    rng = inputs.rng_for(91)
    for dtype in ("f32", "bf16"):
        faults = [inputs.Fault(MAT_B, 44, 82, 9.0), inputs.Fault(MAT_C, 66, 0, -4.0)]
        A, B, A2, B2, cf, eff = _trial(rng, n, k, m, dtype, ("normal", 1.0), ("normal", 1.0), faults)
        tau = gecc.noise_thresholds(n, k, m, 1.0, 1.0)
        cfb = [(0,) + c for c in cf]
        g = H.run_gpu(A, B, A2, B2, cfb, tau, dtype, ld_pad=3)
        H.compare(g, H.run_oracle(A, B, A2, B2, cfb, tau), 1e-5, what=dtype)
        assert g.reports[0].status == gecc.CORRECTED


@pytest.mark.parametrize("trans", [(0, 0), (0, 1), (1, 0), (1, 1)])
def test_padded_leading_dimensions_in_the_fast_bf16_kernel(trans):
    """Leading dimensions larger than the rows (by a multiple of 8 elements, which keeps the 256 x 256
    kernel): operand panels and the stores of C, two rows x 32 columns each, walk the padded rows."""
    n, k, m = 520, 256, 264
    rng = inputs.rng_for(94, 1)
    law = ("normal", 1.0)
    faults = [inputs.Fault(MAT_A, 300, 7, 3.0), inputs.Fault(MAT_C, n - 1, m - 1, 21.5)]
    A, B, A2, B2, cf, eff = _trial(rng, n, k, m, "bf16", law, law, faults)
    tau = gecc.noise_thresholds(n, k, m, 1.0, 1.0)
    cfb = [(0,) + c for c in cf]
    g = H.run_gpu(A, B, A2, B2, cfb, tau, "bf16", trans[0], trans[1], ld_pad=24)
    H.compare(g, H.run_oracle(A, B, A2, B2, cfb, tau), 1e-5, what="padded ld, trans %s" % (trans,))
    assert g.reports[0].status == gecc.CORRECTED and g.pad_untouched
    assert [(e[0], e[1], e[2]) for e in g.reports[0].errors()] == [(e[0], e[1], e[2]) for e in eff]


def test_all_zero_operands_are_clean():
    n, k, m = 200, 64, 136
    Z = np.zeros((n, k), np.float32), np.zeros((k, m), np.float32)
    tau = gecc.Thresholds(1e-6, 1e-6, 1e-6, 1e-6)
    g = H.run_gpu(Z[0], Z[1], Z[0], Z[1], [], tau, "f32")
    assert g.reports[0].status == gecc.CLEAN and np.all(g.C == 0) and np.all(g.C_par == 0)


def test_results_are_reproducible_bit_for_bit():
    w = configs.CFG1
    rng = inputs.rng_for(1, 5)
    faults = inputs.draw_faults(rng, w.n, w.k, w.m, 2, w.offset_law, [MAT_A, MAT_C])
    A, B, A2, B2, cf, eff = _trial(rng, w.n, w.k, w.m, w.dtype, w.law_a, w.law_b, faults)
    cfb = [(0,) + c for c in cf]
    g1 = H.run_gpu(A, B, A2, B2, cfb, w.tau, w.dtype)
    g2 = H.run_gpu(A, B, A2, B2, cfb, w.tau, w.dtype)
    assert np.array_equal(g1.A_par, g2.A_par) and np.array_equal(g1.C_par, g2.C_par)
    assert np.array_equal(g1.C, g2.C) and np.array_equal(g1.synd, g2.synd)
    assert g1.reports[0].errors() == g2.reports[0].errors()


@pytest.mark.parametrize("dtype,shape,trans", [("f32", (1024, 1024, 1024), (0, 0)), ("bf16", (1024, 512, 768), (0, 1)),
                                               ("bf16", (768, 512, 1024), (1, 0)), ("f32", (520, 264, 392), (1, 1))])
def test_launches_of_a_clean_step(dtype, shape, trans):
    """Four scans (a row scan carries the second stage of a column scan where one follows it), the
    product, the threshold pass, the first report, and two gated launches: both audits in one, the repair."""
    import torch
    n, k, m = shape
    rng = inputs.rng_for(2, 77)
    A = inputs.store(rng.standard_normal((n, k)), dtype)
    B = inputs.store(rng.standard_normal((k, m)), dtype)
    tau = gecc.noise_thresholds(n, k, m, 1.0, 1.0)
    ctx = gecc.Context(n, k, m, gecc.BF16 if dtype == "bf16" else gecc.F32, tau, trans_a=trans[0], trans_b=trans[1])
    dA = H.to_dev(A, dtype, trans[0])
    dB = H.to_dev(B, dtype, trans[1])
    C = ctx.alloc_c()
    A_par, B_par, C_par = ctx.alloc_parities()
    rep = ctx.alloc_report()
    ctx.protected_gemm(dA, dB, C, A_par, B_par, C_par, rep)      # (the first call also zeroes the counters)
    torch.cuda.synchronize()
    ctx.timing_enable(32, tuple(range(len(gecc.K_NAMES))))
    ctx.protected_gemm(dA, dB, C, A_par, B_par, C_par, rep)
    torch.cuda.synchronize()
    rec = ctx.timing_read(32)
    ctx.timing_enable(0)
    assert ctx.report_to_host(rep)[0].status == gecc.CLEAN
    names = [gecc.K_NAMES[kd] for kd, _ in rec]
    assert names[-2:] == ["audit_a+audit_b", "repair"] and names[-4:-2] == ["threshold", "decode"], names
    assert len(rec) <= 10, names


# ---- per-k-panel verification: every partial product over a panel of k is a codeword ------------------
@pytest.mark.parametrize("dtype,shape,trans,panels", [("bf16", (520, 512, 264), (0, 0), 4), ("bf16", (520, 512, 264), (0, 1), 2),
                                                      ("bf16", (264, 448, 520), (1, 0), 3), ("f32", (300, 200, 260), (0, 0), 3),
                                                      ("bf16", (1000, 512, 776), (1, 1), 1)])
def test_protected_product_panel_by_panel(dtype, shape, trans, panels):
    """gecc_protected_gemm_panels against the oracle's panel-wise path: same panels, same scaled
    thresholds, one fault of C in every panel (each a single fault there, although together they
    lie on a diagonal, beyond the code for the whole product).  Reports bit for bit, summed C to
    1e-5, parity blocks of every partial product and the panel-wise operand parities to rounding."""
    import torch
    import ctypes as C
    n, k, m = shape
    rng = inputs.rng_for(97, n + k + panels)
    A, B = inputs.operands(rng, n, k, m, ("normal", 1.0), ("normal", 1.0), dtype)
    t = gecc.noise_thresholds(n, k, m, 1.0, 1.0)
    tau_o = oc.Thresholds(t.r1, t.r2, t.q1, t.q2, t.op, t.rep, t.rel)
    ctx = gecc.Context(n, k, m, gecc.BF16 if dtype == "bf16" else gecc.F32, t, trans_a=trans[0], trans_b=trans[1])
    P = ctx.panel_count(panels)
    bounds = oc.panel_bounds(k, panels)
    assert P == len(bounds)
    # faults: one of C per panel, together on a diagonal (the call encodes and multiplies in one
    # go, so there is no moment for an operand fault between the two; the staged calls cover those)
    cf = {g: [(10 + 60 * g, 20 + 60 * g, 25.0 + g)] for g in range(P)}
    A2 = A
    res, Csum = oc.protected_gemm_panels(A, B, A, B, cf, tau_o, bounds)
    dA, dB = H.to_dev(A[None], dtype, trans[0]), H.to_dev(B[None], dtype, trans[1])
    A_par, B_par, _ = ctx.alloc_parities()
    C_par = torch.empty(P * (2 * n + 2 * m + 4), dtype=torch.float64, device=H.DEV)
    reps = torch.zeros(P * C.sizeof(gecc.Report), dtype=torch.uint8, device=H.DEV)
    Cd, Cp = ctx.alloc_c(), ctx.alloc_c()
    Cd.fill_(float("nan")); Cp.fill_(float("nan"))
    fl, nf = gecc.make_faults([(g, i, j, e) for g, lst in cf.items() for (i, j, e) in lst], H.DEV)
    ctx.protected_gemm_panels(dA, dB, Cd, Cp if P > 1 else None, A_par, B_par, C_par, reps, panels, fl, nf)
    host = ctx.reports_to_host(reps, P)
    for g, (r, o) in enumerate(zip(host, res)):
        assert r.status == o.status == gecc.CORRECTED, (g, r.status, o.status)
        assert [e[:3] for e in r.errors()] == [e[:3] for e in o.errors] == [(MAT_C, 10 + 60 * g, 20 + 60 * g)]
    scale = np.abs(Csum).max()
    assert np.abs(Cd[0].cpu().numpy().astype(np.float64) - Csum).max() / scale <= 1e-5
    # parity blocks of every partial product, and the operand parities panel after panel
    cp = C_par.cpu().numpy().reshape(P, -1)
    ap, bp = A_par.cpu().numpy(), B_par.cpu().numpy()
    for g, (k0, k1) in enumerate(bounds):
        ob = res[g].Cbar
        ref = np.concatenate([ob[:n, m], ob[:n, m + 1], ob[n, :m], ob[n + 1, :m], ob[n:, m:].ravel()])
        assert np.allclose(cp[g], ref, rtol=1e-10, atol=1e-11 * np.abs(ref).max()), g
        assert np.allclose(ap[2 * k0:2 * k1].reshape(2, -1), oc.encode_a(A2[:, k0:k1]), rtol=1e-12, atol=1e-12)
        assert np.allclose(bp[2 * k0:2 * k1].reshape(2, -1), oc.encode_b(B[k0:k1, :]).T, rtol=1e-12, atol=1e-12)
    # the same three faults in one product of the whole k: beyond the code
    if P >= 3:
        g1 = H.run_gpu(A2, B, A2, B, [(0, 10 + 60 * g, 20 + 60 * g, 25.0 + g) for g in range(P)], t, dtype, trans[0], trans[1])
        assert g1.reports[0].status == gecc.UNCORRECTABLE


# ---- blocked grid code: Section III per block of C ----------------------------------------------------
def _blocked_compare(g, res, Cref, n, m, nb, mb, tol_c=1e-5, tol_mag=None):
    nbj = m // mb
    scale = np.abs(Cref).max()
    for (I, J), o in res.items():
        r = g["reports"][I * nbj + J]
        assert r.status == o.status, ((I, J), r.status, o.status, r.errors(), o.errors)
        if o.status == oc.UNCORRECTABLE:
            continue
        assert r.n_total == len(o.errors) and [e[:3] for e in r.errors()] == [e[:3] for e in o.errors[:8]], ((I, J), r.errors(), o.errors)
        for x, y in zip(r.errors(), o.errors):
            assert abs(x[3] - y[3]) <= (tol_mag if tol_mag is not None else 10 * tol_c * scale) + 1e-6 * abs(y[3]), ((I, J), x, y)
        blk = g["C"][I * nb:(I + 1) * nb, J * mb:(J + 1) * mb]
        assert not np.isnan(blk).any()
        assert np.abs(blk - o.C).max() / scale <= tol_c, (I, J)
        # the parity blocks of the block: formed on the matrix units in fp32 (relative to the largest of their kind)
        ref = np.concatenate([o.Cbar[:nb, mb], o.Cbar[:nb, mb + 1], o.Cbar[nb, :mb], o.Cbar[nb + 1, :mb]])
        got = g["C_par"][I * nbj + J][:2 * nb + 2 * mb]
        for a0, a1 in ((0, nb), (nb, 2 * nb), (2 * nb, 2 * nb + mb), (2 * nb + mb, 2 * nb + 2 * mb)):
            assert np.abs(got[a0:a1] - ref[a0:a1]).max() <= 2e-5 * max(np.abs(ref[a0:a1]).max(), 1e-30), ((I, J), a0)
        pg = g["C_par"][I * nbj + J][2 * nb + 2 * mb:]
        assert np.allclose(pg, o.Cbar[nb:, mb:].ravel(), rtol=1e-11, atol=1e-12 * np.abs(pg).max())


@pytest.mark.parametrize("pattern", ["clean", "two errors in every block", "A", "B", "A+B same l, C elsewhere", "three in one block"])
@pytest.mark.parametrize("dtype,shape,block,trans", [("bf16", (512, 256, 768), (256, 256), (0, 0)), ("bf16", (512, 256, 768), (256, 384), (0, 1)),
                                                     ("bf16", (512, 192, 512), (128, 256), (1, 0)), ("f32", (256, 200, 384), (128, 128), (0, 0)),
                                                     ("bf16", (768, 256, 512), (256, 256), (1, 1))])
def test_blocked_grid_code(pattern, dtype, shape, block, trans):
    """gecc_params.block_n / block_m: every block of C is a codeword of Section III of its own.  Status
    and positions per block bit for bit with the oracle's block-by-block evaluation, C to 1e-5, the
    operands restored; 'two errors in every block' is far beyond the whole-matrix code."""
    n, k, m = shape
    nb, mb = block
    rng = inputs.rng_for(96, n + k + len(pattern))
    F = inputs.Fault
    nbi, nbj = n // nb, m // mb
    if pattern == "clean":
        faults = []
    elif pattern == "two errors in every block":
        faults = []
        for I in range(nbi):
            for J in range(nbj):
                faults += [F(MAT_C, I * nb + 3 + J, J * mb + 5 + I, 20.0 + I + J), F(MAT_C, I * nb + nb - 1, J * mb + 100, -35.0 - J)]
    elif pattern == "A":
        faults = [F(MAT_A, nb + 7, k - 2, 4.0)]
    elif pattern == "B":
        faults = [F(MAT_B, 3, mb + 9, -5.0)]
    elif pattern == "A+B same l, C elsewhere":
        faults = [F(MAT_A, 5, 17, 3.0), F(MAT_B, 17, m - 1, 6.0), F(MAT_C, n - 1, 0, 44.0)]
    else:
        faults = [F(MAT_C, 1, 1, 10.0), F(MAT_C, 20, 30, 20.0), F(MAT_C, 40, 60, 30.0), F(MAT_C, n - 1, m - 1, 9.0)]
    A, B, A2, B2, cf, eff = _trial(rng, n, k, m, dtype, ("normal", 1.0), ("normal", 1.0), faults)
    tau = gecc.noise_thresholds(nb, k, mb, 1.0, 1.0)
    tau_o = oc.Thresholds(tau.r1, tau.r2, tau.q1, tau.q2, tau.op, tau.rep, tau.rel)
    res, Cref, Ao, Bo = oc.protected_gemm_blocked(A, B, A2, B2, cf, tau_o, nb, mb)
    g = H.run_gpu_blocked(A, B, A2, B2, cf, tau, dtype, block, trans[0], trans[1])
    _blocked_compare(g, res, Cref, n, m, nb, mb, tol_mag=4 * max(tau.r1, tau.q1))
    st = [r.status for r in g["reports"]]
    if pattern == "clean":
        assert st == [gecc.CLEAN] * (nbi * nbj)
        mx = np.array([list(r.max_abs_synd) for r in g["reports"]])
        assert (mx[:, 0] <= tau.r1 / 2).all() and (mx[:, 1] <= tau.r2 / 2).all() and (mx[:, 2] <= tau.q1 / 2).all() and (mx[:, 3] <= tau.q2 / 2).all()
    elif pattern == "three in one block":
        assert st[0] == gecc.UNCORRECTABLE and st[-1] == gecc.CORRECTED and st.count(gecc.CLEAN) == nbi * nbj - 2
    else:
        assert gecc.UNCORRECTABLE not in st
        assert np.array_equal(g["A"], A.astype(np.float64)) and np.array_equal(g["B"], B.astype(np.float64))
        assert np.abs(g["C"] - A.astype(np.float64) @ B.astype(np.float64)).max() / np.abs(Cref).max() <= 1e-5
    if pattern == "two errors in every block":
        assert st == [gecc.CORRECTED] * (nbi * nbj)
        # the one-call chain gives the same decisions
        g1 = H.run_gpu_blocked(A, B, A, B, cf, tau, dtype, block, trans[0], trans[1], staged=False)
        _blocked_compare(g1, res, Cref, n, m, nb, mb, tol_mag=4 * max(tau.r1, tau.q1))


@pytest.mark.parametrize("dtype,shape,block,trans", [("bf16", (512, 256, 768), (256, 256), (0, 0)), ("bf16", (768, 256, 512), (256, 256), (1, 1)),
                                                     ("f32", (256, 200, 384), (128, 128), (0, 1))])
def test_blocked_grid_code_random_trials(dtype, shape, block, trans):
    """40 seeded trials per layout with 0 to 5 faults anywhere in A, B and C: some blocks stay clean, some
    hold up to two symbols, some more than the code corrects, an operand symbol is seen by every block
    of its line.  Every block's status and positions as the oracle's block-by-block evaluation gives
    them, every block that is not UNCORRECTABLE to 1e-5."""
    n, k, m = shape
    nb, mb = block
    tau = gecc.noise_thresholds(nb, k, mb, 1.0, 1.0)
    tau_o = oc.Thresholds(tau.r1, tau.r2, tau.q1, tau.q2, tau.op, tau.rep, tau.rel)
    seen = {gecc.CLEAN: 0, gecc.CORRECTED: 0, gecc.UNCORRECTABLE: 0}
    for trial in range(40):
        rng = inputs.rng_for(99, 1000 * trans[0] + trial)
        faults = inputs.draw_faults(rng, n, k, m, int(rng.integers(0, 6)), ("uniform", 1.0, 100.0))
        if trial % 5 == 4:        # every fifth trial: three or four symbols of C inside the first block
            faults = [inputs.Fault(MAT_C, f.row, f.col, f.offset)
                      for f in inputs.draw_faults(rng, nb, k, mb, 3 + trial % 2, ("uniform", 1.0, 100.0), [MAT_C] * (3 + trial % 2))]
        A, B, A2, B2, cf, eff = _trial(rng, n, k, m, dtype, ("normal", 1.0), ("normal", 1.0), faults)
        res, Cref, Ao, Bo = oc.protected_gemm_blocked(A, B, A2, B2, cf, tau_o, nb, mb)
        g = H.run_gpu_blocked(A, B, A2, B2, cf, tau, dtype, block, trans[0], trans[1])
        _blocked_compare(g, res, Cref, n, m, nb, mb, tol_mag=4 * max(tau.r1, tau.q1))
        for r in g["reports"]:
            seen[r.status] += 1
    assert min(seen.values()) > 0, seen


def test_blocked_grid_code_at_the_forward_shape():
    """cfg4-fwd in 1024 x 1024 blocks (16 x 14 codewords): the parity blocks of all of them come from two
    narrow products on the 256 x 256-tile kernel.  Two errors in each of five blocks, a wrong symbol of A
    (seen by the 14 blocks of its row block) and one of B; every block against the oracle."""
    w = configs.CFG4_FWD
    n, k, m, nb, mb = w.n, w.k, w.m, 1024, 1024
    rng = inputs.rng_for(4, 7)
    F = inputs.Fault
    faults = [F(MAT_A, 5 * nb + 17, 4000, 9.0), F(MAT_B, 123, 3 * mb + 1000, -3.0)]
    for (I, J) in [(0, 0), (3, 13), (15, 0), (15, 13), (8, 7)]:
        faults += [F(MAT_C, I * nb + 1, J * mb + 2, 40.0 + I), F(MAT_C, I * nb + 1000, J * mb + 1023, -25.0 - J)]
    A, B, A2, B2, cf, eff = _trial(rng, n, k, m, w.dtype, w.law_a, w.law_b, faults)
    tau = gecc.noise_thresholds(nb, k, mb, w.sigma_a, w.sigma_b)
    assert tau.r2 < w.tau.r2 / 40 and tau.q2 < w.tau.q2 / 60        # weights bounded by the block: (1024 / 14336)^1.5, (1024 / 16384)^1.5
    tau_o = oc.Thresholds(tau.r1, tau.r2, tau.q1, tau.q2, tau.op, tau.rep, tau.rel)
    res, Cref, Ao, Bo = oc.protected_gemm_blocked(A, B, A2, B2, cf, tau_o, nb, mb)
    g = H.run_gpu_blocked(A, B, A2, B2, cf, tau, w.dtype, (nb, mb))
    _blocked_compare(g, res, Cref, n, m, nb, mb, tol_mag=4 * max(tau.r1, tau.q1))
    st = [r.status for r in g["reports"]]
    assert gecc.UNCORRECTABLE not in st and st.count(gecc.CLEAN) == 16 * 14 - 5 - (14 + 16 - 1)
    assert np.array_equal(g["A"], A.astype(np.float64)) and np.array_equal(g["B"], B.astype(np.float64))


# ---- single-checksum mode (Section VI's comparison scheme: plain parities only) -----------------------
@pytest.mark.parametrize("pattern", ["none", "C", "C+C same row", "C+C same column", "C+C elsewhere", "A", "B", "A+C", "B+C",
                                     "one row, 40 columns", "one column, 25 rows", "two rows", "C nan"])
@pytest.mark.parametrize("dtype,shape,trans", [("f32", (300, 200, 260), (0, 0)), ("bf16", (520, 256, 264), (0, 1)),
                                               ("bf16", (520, 256, 264), (1, 0))])
def test_single_checksum_mode(pattern, dtype, shape, trans):
    """gecc_params.weighted = 0: the same kernels, decoder restricted to the plain parities.  One
    faulty row or column of C is corrected whatever the number of symbols (scenario c of Section VI
    and Appendix A's case s = 1), everything else is UNCORRECTABLE -- scenarios d, e, f, and a, b
    too under the fault model used here (the spoiled row of C takes its own parity symbols along,
    and one parity per operand line cannot place the symbol).  Status, positions and C as the
    oracle's single-checksum decoder gives them; the grid code corrects all of these but 'two rows'."""
    n, k, m = shape
    rng = inputs.rng_for(98, len(pattern))
    F = inputs.Fault
    faults = {"none": [], "C": [F(MAT_C, n - 1, 3, 21.0)],
              "C+C same row": [F(MAT_C, 257, 0, 9.0), F(MAT_C, 257, m - 1, -30.0)],
              "C+C same column": [F(MAT_C, 0, 258, 5.5), F(MAT_C, n - 1, 258, 14.0)],
              "C+C elsewhere": [F(MAT_C, 10, 20, 7.0), F(MAT_C, 200, 100, -8.0)],
              "A": [F(MAT_A, 100, k - 1, 3.0)], "B": [F(MAT_B, 0, 259, -4.0)],
              "A+C": [F(MAT_A, 100, 5, 3.0), F(MAT_C, 100, 7, 12.0)], "B+C": [F(MAT_B, 9, 70, 2.0), F(MAT_C, 1, 2, 6.0)],
              "one row, 40 columns": _t2_faults(rng, [n - 2], None, m, 40 / m, True),
              "one column, 25 rows": _t2_faults(rng, [1], None, n, 25 / n, False),
              "two rows": _t2_faults(rng, [3, 200], None, m, 5 / m, True),
              "C nan": [F(MAT_C, 5, 6, float("nan"))]}[pattern]
    A, B, A2, B2, cf, eff = _trial(rng, n, k, m, dtype, ("normal", 1.0), ("normal", 1.0), faults)
    t = gecc.noise_thresholds(n, k, m, 1.0, 1.0)
    tau = gecc.Thresholds(t.r1, t.r2, t.q1, t.q2, weighted=False)
    cfb = [(0,) + c for c in cf]
    g = H.run_gpu(A, B, A2, B2, cfb, tau, dtype, trans[0], trans[1])
    with np.errstate(invalid="ignore"):
        o = H.run_oracle(A, B, A2, B2, cfb, tau)
    scale = float(np.max(np.abs(np.nan_to_num(o[0].C))))
    # more than one symbol in the line: Section V's subtraction without re-evaluation (as for Theorem 2)
    many = len(faults) > 1
    tol = 4 * max(tau.r1, tau.q1) / scale if many else 1e-5
    H.compare(g, o, tol, tol_mag=4 * max(tau.r1, tau.q1), what="single checksum, " + pattern)
    want = {"none": gecc.CLEAN, "C": gecc.CORRECTED, "C+C same row": gecc.CORRECTED, "C+C same column": gecc.CORRECTED,
            "one row, 40 columns": gecc.CORRECTED, "one column, 25 rows": gecc.CORRECTED}.get(pattern, gecc.UNCORRECTABLE)
    assert g.reports[0].status == want
    assert g.reports[0].max_abs_synd[1] == 0.0 and g.reports[0].max_abs_synd[3] == 0.0
    if want == gecc.CORRECTED:
        assert g.reports[0].n_total == len(faults)
    # the grid code on the same faults
    if pattern not in ("two rows", "C nan", "none"):
        g2 = H.run_gpu(A, B, A2, B2, cfb, t, dtype, trans[0], trans[1])
        assert g2.reports[0].status == gecc.CORRECTED and g2.reports[0].n_total == len(eff)


@pytest.mark.parametrize("dtype,shape,trans", [("f32", (300, 200, 260), (0, 0)), ("bf16", (520, 256, 264), (1, 0))])
def test_single_checksum_mode_random_trials(dtype, shape, trans):
    """60 seeded trials with 0 to 3 faults anywhere in A, B and C, decided by the HIP path and by the
    oracle's single-checksum decoder: same status, same positions, C to the tolerance of the rule used."""
    n, k, m = shape
    t = gecc.noise_thresholds(n, k, m, 1.0, 1.0)
    tau = gecc.Thresholds(t.r1, t.r2, t.q1, t.q2, weighted=False)
    seen = {gecc.CLEAN: 0, gecc.CORRECTED: 0, gecc.UNCORRECTABLE: 0}
    for trial in range(60):
        rng = inputs.rng_for(99, 5000 + 100 * trans[0] + trial)
        count = int(rng.integers(0, 4))
        mats = [MAT_C] * count if trial % 2 else None              # every other trial: faults of C only
        faults = inputs.draw_faults(rng, n, k, m, count, ("uniform", 1.0, 100.0), mats)
        if trial % 4 == 1 and count >= 2:                          # ... and some of those in one row
            faults = [inputs.Fault(MAT_C, faults[0].row, f.col, f.offset) for f in faults]
            if len({f.col for f in faults}) < len(faults):
                continue
        A, B, A2, B2, cf, eff = _trial(rng, n, k, m, dtype, ("normal", 1.0), ("normal", 1.0), faults)
        cfb = [(0,) + c for c in cf]
        g = H.run_gpu(A, B, A2, B2, cfb, tau, dtype, trans[0], trans[1])
        o = H.run_oracle(A, B, A2, B2, cfb, tau)
        scale = float(np.max(np.abs(o[0].C)))
        tol = 4 * max(tau.r1, tau.q1) / scale if len(faults) > 1 else 1e-5
        H.compare(g, o, tol, tol_mag=4 * max(tau.r1, tau.q1), what="single checksum, trial %d" % trial)
        seen[g.reports[0].status] += 1
    assert min(seen.values()) > 0, seen


# ---- symbols that are not numbers ------------------------------------------------------------------
@pytest.mark.parametrize("where", ["C nan", "C inf", "C nan, stand-alone verify", "A nan", "B -inf"])
@pytest.mark.parametrize("dtype,shape", [("f32", (300, 200, 260)), ("bf16", (520, 256, 264))])
def test_a_symbol_that_is_not_a_number_is_detected_and_handed_back(where, dtype, shape):
    """Section V step 1 clears a line only when |sum - parity| <= threshold holds, which a NaN
    never satisfies: the lines of such a symbol are flagged and, since nothing can be subtracted
    from it, the product is reported UNCORRECTABLE (to be computed again)."""
    n, k, m = shape
    rng = inputs.rng_for(99, n)
    A, B = inputs.operands(rng, n, k, m, ("normal", 1.0), ("normal", 1.0), dtype)
    A2, B2, cf = A.copy(), B.copy(), []
    bad = {"C nan": np.nan, "C inf": np.inf, "C nan, stand-alone verify": np.nan, "A nan": np.nan, "B -inf": -np.inf}[where]
    if where.startswith("C"):
        cf = [(0, n - 3, 258, bad)]
    elif where.startswith("A"):
        A2[257, k - 1] = bad
    else:
        B2[3, m - 2] = bad
    tau = gecc.noise_thresholds(n, k, m, 1.0, 1.0)
    with np.errstate(invalid="ignore"):
        o = H.run_oracle(A, B, A2, B2, cf, tau)
    g = H.run_gpu(A, B, A2, B2, cf, tau, dtype, fused="stand-alone" not in where)
    assert o[0].status == oc.UNCORRECTABLE and g.reports[0].status == gecc.UNCORRECTABLE
    assert (g.reports[0].s, g.reports[0].t) == (o[0].s, o[0].t)
    assert (g.reports[0].s, g.reports[0].t) == {"C": (1, 1), "A": (1, m), "B": (n, 1)}[where[0]]
    assert not np.isfinite(g.reports[0].max_abs_synd[0]) or not np.isfinite(g.reports[0].max_abs_synd[2])


def test_a_transient_nan_is_recomputed_away():
    n, k, m = 300, 128, 280
    rng = inputs.rng_for(94, 7)
    A, B = inputs.operands(rng, n, k, m, ("normal", 1.0), ("normal", 1.0), "bf16")
    tau = gecc.noise_thresholds(n, k, m, 1.0, 1.0)
    ctx = gecc.Context(n, k, m, gecc.BF16, gecc.Thresholds(tau.r1, tau.r2, tau.q1, tau.q2))
    dA, dB = H.to_dev(A[None], "bf16", False), H.to_dev(B[None], "bf16", False)
    A_par, B_par, C_par = ctx.alloc_parities()
    rep, Cd = ctx.alloc_report(), ctx.alloc_c()
    fl, nf = gecc.make_faults([(0, 10, 20, float("nan"))], H.DEV)
    reports, attempts = ctx.protected_gemm_retry(dA, dB, Cd, A_par, B_par, C_par, rep, 2, fl, nf)
    assert attempts == 2 and reports[0].status == gecc.CLEAN
    ref = A.astype(np.float64) @ B.astype(np.float64)
    assert np.max(np.abs(Cd[0].cpu().numpy() - ref)) / np.max(np.abs(ref)) <= 1e-5


# ---- configuration 1: 128^3 fp32 N(0,1), 0 / 1 / 2 errors, 1000 trials each -------------------
@pytest.mark.parametrize("n_err", [0, 1, 2])
def test_cfg1_thousand_trials_per_error_count(n_err):
    w = configs.CFG1
    BATCH = 250
    n_corrected = n_unc = 0
    for chunk in range(1000 // BATCH):
        As, Bs, A2s, B2s, cfb, effs = [], [], [], [], [], []
        for b in range(BATCH):
            rng = inputs.rng_for(1, 10000 * n_err + chunk * BATCH + b)
            faults = inputs.draw_faults(rng, w.n, w.k, w.m, n_err, w.offset_law)
            A, B, A2, B2, cf, eff = _trial(rng, w.n, w.k, w.m, w.dtype, w.law_a, w.law_b, faults)
            As.append(A); Bs.append(B); A2s.append(A2); B2s.append(B2); effs.append(eff)
            cfb += [(b,) + c for c in cf]
        As, Bs, A2s, B2s = map(np.stack, (As, Bs, A2s, B2s))
        g = H.run_gpu(As, Bs, A2s, B2s, cfb, w.tau, w.dtype)
        o = H.run_oracle(As, Bs, A2s, B2s, cfb, w.tau)
        H.compare(g, o, w.tol_c, what="cfg1 n_err=%d chunk=%d" % (n_err, chunk))
        for b, (rep, res) in enumerate(zip(g.reports, o)):
            if n_err == 0:
                assert rep.status == gecc.CLEAN
            elif rep.status == gecc.CORRECTED:
                n_corrected += 1
                got = [(e[0], e[1], e[2]) for e in rep.errors()]
                assert got == [(e[0], e[1], e[2]) for e in effs[b]], (chunk, b)
            else:
                n_unc += 1
    if n_err == 1:
        assert n_corrected == 1000
    if n_err == 2:
        # only two errors in one column of A / one row of B exceed the code (about 2 / (9 k) of pairs)
        assert n_corrected + n_unc == 1000 and n_unc <= 10


# ---- configuration 2: 1024^3 fp32 U(-1,1); none, 1 in C, 2 anywhere, adversarial pairs -------
def _cfg2_patterns():
    w = configs.CFG2
    n, k, m = w.n, w.k, w.m
    F = inputs.Fault
    pats = {
        "none": [],
        "C": [F(MAT_C, 700, 13, 42.5)],
        "C+C same row": [F(MAT_C, 5, 100, 3.0), F(MAT_C, 5, 900, -77.0)],
        "C+C same row cancelling": [F(MAT_C, 5, 100, 8.0), F(MAT_C, 5, 101, -8.0)],
        "C+C same col": [F(MAT_C, 1023, 0, 1.5), F(MAT_C, 0, 0, 99.0)],
        # equal offsets in adjacent cells: the plain sums cannot tell the diagonal from the
        # anti-diagonal and the weighted sums differ by less than their threshold -> ambiguous
        "C+C adjacent diag, equal offsets (ambiguous)": [F(MAT_C, 10, 20, 1.0), F(MAT_C, 11, 21, 1.0)],
        "C+C adjacent diag": [F(MAT_C, 10, 20, 1.0), F(MAT_C, 11, 21, 5.0)],
        "C+C far diag, equal offsets": [F(MAT_C, 10, 20, 40.0), F(MAT_C, 900, 21, 40.0)],
        "C+C anti": [F(MAT_C, 800, 20, -6.0), F(MAT_C, 30, 999, 2.0)],
        "A": [F(MAT_A, 17, 1000, -31.0)],
        "B": [F(MAT_B, 1000, 17, 12.0)],
        "A+C C in A's row": [F(MAT_A, 300, 4, 10.0), F(MAT_C, 300, 77, -20.0)],
        "A+C elsewhere": [F(MAT_A, 300, 4, 10.0), F(MAT_C, 301, 77, -20.0)],
        "B+C C in B's col": [F(MAT_B, 9, 512, 5.0), F(MAT_C, 1000, 512, 64.0)],
        "A+B same l": [F(MAT_A, 1, 600, 2.0), F(MAT_B, 600, 1022, -3.0)],
        "A+B different l": [F(MAT_A, 1, 600, 2.0), F(MAT_B, 601, 1022, -3.0)],
        "A+A same row": [F(MAT_A, 50, 1, 7.0), F(MAT_A, 50, 1023, 7.0)],
        "B+B same col": [F(MAT_B, 2, 77, 1.25), F(MAT_B, 1000, 77, -90.0)],
        "A+A same col (beyond the code)": [F(MAT_A, 50, 9, 7.0), F(MAT_A, 51, 9, 3.0)],
        "B+B same row (beyond the code)": [F(MAT_B, 3, 9, 7.0), F(MAT_B, 3, 10, 3.0)],
    }
    for t in range(6):
        rng = inputs.rng_for(2, 100 + t)
        pats["random pair %d" % t] = inputs.draw_faults(rng, n, k, m, 2, w.offset_law)
    return pats


@pytest.mark.parametrize("name", list(_cfg2_patterns().keys()))
def test_cfg2_patterns(name):
    w = configs.CFG2
    faults = _cfg2_patterns()[name]
    rng = inputs.rng_for(2, 0)
    A, B, A2, B2, cf, eff = _trial(rng, w.n, w.k, w.m, w.dtype, w.law_a, w.law_b, faults)
    cfb = [(0,) + c for c in cf]
    g = H.run_gpu(A, B, A2, B2, cfb, w.tau, w.dtype)
    o = H.run_oracle(A, B, A2, B2, cfb, w.tau)
    H.compare(g, o, w.tol_c, what=name)
    rep = g.reports[0]
    if "beyond" in name or "ambiguous" in name:
        assert rep.status == gecc.UNCORRECTABLE
    elif name == "none":
        assert rep.status == gecc.CLEAN
        mx = rep.max_abs_synd
        assert mx[0] <= w.tau.r1 / 4 and mx[1] <= w.tau.r2 / 4 and mx[2] <= w.tau.q1 / 4 and mx[3] <= w.tau.q2 / 4
    else:
        assert rep.status == gecc.CORRECTED
        assert [(e[0], e[1], e[2]) for e in rep.errors()] == [(e[0], e[1], e[2]) for e in eff]


def test_cfg2_standalone_verify_and_unrefined_correction():
    """C corrupted after the product (plain device writes), verified by the syndrome scan of C;
    with refine off the corrected symbols carry the sqrt(n)-fold rounding noise of Section V's
    subtraction: tolerance 16 sqrt(n) eps / max|C| instead of 1e-5."""
    w = configs.CFG2
    rng = inputs.rng_for(2, 1)
    faults = [inputs.Fault(MAT_C, 100, 200, 17.0), inputs.Fault(MAT_C, 900, 201, -3.0)]
    A, B, A2, B2, cf, eff = _trial(rng, w.n, w.k, w.m, w.dtype, w.law_a, w.law_b, faults)
    cfb = [(0,) + c for c in cf]
    o = H.run_oracle(A, B, A2, B2, cfb, w.tau)
    g = H.run_gpu(A, B, A2, B2, cfb, w.tau, w.dtype, fused=False)
    H.compare(g, o, w.tol_c, what="standalone")
    g = H.run_gpu(A, B, A2, B2, cfb, w.tau, w.dtype, refine=0)
    H.compare(g, o, w.tau.q1 / np.abs(o[0].C).max(), what="unrefined")


# ---- configuration 3: 4096^3 bf16 N(0, 0.02^2), log-uniform offsets ---------------------------
@pytest.mark.parametrize("trial", [0, 1, 2])
def test_cfg3_trials(trial):
    w = configs.CFG3
    rng = inputs.rng_for(3, trial)
    faults = inputs.draw_faults(rng, w.n, w.k, w.m, trial, w.offset_law,
                                matrices=[None, [MAT_C], [MAT_A, MAT_C]][trial])
    A, B, A2, B2, cf, eff = _trial(rng, w.n, w.k, w.m, w.dtype, w.law_a, w.law_b, faults)
    cfb = [(0,) + c for c in cf]
    g = H.run_gpu(A, B, A2, B2, cfb, w.tau, w.dtype)
    o = H.run_oracle(A, B, A2, B2, cfb, w.tau)
    H.compare(g, o, 1e-5, what="cfg3 trial %d" % trial)
    if trial == 0:
        mx = g.reports[0].max_abs_synd
        assert mx[0] <= w.tau.r1 / 4 and mx[1] <= w.tau.r2 / 4 and mx[2] <= w.tau.q1 / 4 and mx[3] <= w.tau.q2 / 4
    else:
        assert g.reports[0].status == gecc.CORRECTED


def test_cfg3_large_offsets_do_not_break_the_verification():
    """Offsets of several hundred on |C| ~ 0.03: the fp32 partial sums of the flagged lines lose
    absolute precision in proportion to the offset; the relative allowance of the verification
    step has to absorb that, on both sides alike."""
    w = configs.CFG3
    rng = inputs.rng_for(3, 50)
    faults = [inputs.Fault(MAT_C, 4000, 4090, 731.0), inputs.Fault(MAT_C, 17, 3, -402.5)]
    A, B, A2, B2, cf, eff = _trial(rng, w.n, w.k, w.m, w.dtype, w.law_a, w.law_b, faults)
    cfb = [(0,) + c for c in cf]
    g = H.run_gpu(A, B, A2, B2, cfb, w.tau, w.dtype)
    o = H.run_oracle(A, B, A2, B2, cfb, w.tau)
    H.compare(g, o, 1e-5, tol_mag=1e-3, what="cfg3 large offsets")
    assert g.reports[0].status == gecc.CORRECTED


def test_campaign_rates_on_a_bf16_product():
    """Detection / false-alarm / correction rates against the planted faults (no oracle)."""
    from paper_2508_04355_amd import campaign
    out = campaign.run("cfg3", 400)
    assert out["false_alarm_rate"] == 0.0 and out["detection_rate"] == 1.0
    assert all(v.get("miscorrected", 0) == 0 for v in out["by_class"].values())
    assert out["exact_correction_rate"] >= 0.99


def test_cfg3_ten_thousand_trials_against_the_oracle():
    """The whole of configuration 3: 10 000 trials with 0-2 faults, log-uniform offsets, each decided
    by the HIP path and by the oracle (evaluated incrementally on the clean C-bar, pinned to the full
    oracle on the CPU).  Status and positions bit for bit, corrected C to 1e-5, on every trial whose
    oracle decision does not change when the thresholds are halved or doubled; the other trials (a
    syndrome within a factor two of its threshold) are counted and have to be rare."""
    import sys
    import campaign_oracle
    out = campaign_oracle.run("cfg3", 10000, progress=1000)
    print({kk: out[kk] for kk in ("agree", "margin_safe", "n_mismatches_on_other_trials", "worst_corrected_C_error",
                                  "worst_corrected_C_error_without_operand_faults", "seconds")}, file=sys.stderr)
    bad = out["mismatches_on_margin_safe_trials"]
    assert len(bad) == 0, (len(bad), bad[:3])
    assert out["worst_corrected_C_error_without_operand_faults"] <= 1e-5
    assert out["margin_safe"] >= 0.97 * out["trials"]
    assert out["n_mismatches_on_other_trials"] <= 0.01 * out["trials"]
    assert out["false_alarms_gpu"] == 0 and out["false_alarms_oracle"] == 0
    assert out["detection_rate_gpu"] == out["detection_rate_oracle"] == 1.0
    assert out["oracle_worst_left_in_cbar"] <= 1e-7      # the oracle's corrected C-bar is the clean one (parity symbols, up to n^1.5 times larger, included)


# ---- configuration 5: 256 batched 512^3 fp32, exactly two errors each ------------------------
def test_cfg5_batched_two_errors_each():
    w = configs.CFG5
    As, Bs, A2s, B2s, cfb, effs = [], [], [], [], [], []
    for b in range(w.batch):
        rng = inputs.rng_for(5, b)
        faults = inputs.draw_faults(rng, w.n, w.k, w.m, 2, w.offset_law)
        A, B, A2, B2, cf, eff = _trial(rng, w.n, w.k, w.m, w.dtype, w.law_a, w.law_b, faults)
        As.append(A); Bs.append(B); A2s.append(A2); B2s.append(B2); effs.append(eff)
        cfb += [(b,) + c for c in cf]
    As, Bs, A2s, B2s = map(np.stack, (As, Bs, A2s, B2s))
    g = H.run_gpu(As, Bs, A2s, B2s, cfb, w.tau, w.dtype)
    o = H.run_oracle(As, Bs, A2s, B2s, cfb, w.tau)
    H.compare(g, o, w.tol_c, what="cfg5")
    ok = sum(r.status == gecc.CORRECTED for r in g.reports)
    assert ok >= w.batch - 3      # the rest: two errors in one line of an operand
    for rep, eff in zip(g.reports, effs):
        if rep.status == gecc.CORRECTED:
            assert [(e[0], e[1], e[2]) for e in rep.errors()] == [(e[0], e[1], e[2]) for e in eff]


def test_rounds_as_32_by_8_blocks_of_tiles():
    """A product whose default round of tiles would touch more operand panels than the memory-side
    cache holds, with a tile grid of 32 x 8: the launcher hands the tiles out in blocks of 32 x 8
    (cfg4-dgrad, in the test below, takes 16 x 16 blocks).  Every symbol against the oracle."""
    n, k, m = 8192, 11264, 2048
    rng = inputs.rng_for(95, 0)
    faults = [inputs.Fault(MAT_C, 8000, 2047, 41.0)]
    A, B, A2, B2, cf, eff = _trial(rng, n, k, m, "bf16", ("normal", 1.0), ("normal", 0.02), faults)
    tau = gecc.noise_thresholds(n, k, m, 1.0, 0.02)
    cfb = [(0,) + c for c in cf]
    g = H.run_gpu(A, B, A2, B2, cfb, tau, "bf16", 0, 0, reverify=True)
    o = H.run_oracle(A, B, A2, B2, cfb, tau)
    H.compare(g, o, 1e-5, what="32 x 8 blocks of tiles")
    assert g.reports[0].status == gecc.CORRECTED and g.reverify_status == gecc.CLEAN
    assert [(e[0], e[1], e[2]) for e in g.reports[0].errors()] == [(e[0], e[1], e[2]) for e in eff]


# ---- configuration 4 at full size: every symbol and every decision against the oracle ----------
@pytest.mark.parametrize("wname", ["cfg4-fwd", "cfg4-dgrad", "cfg4-wgrad"])
def test_cfg4_full_size_against_the_oracle(wname):
    """The three training-layer products at their full sizes, in the launch configuration bench.py
    times (256 x 256 tiles, block order of the rounds, k-split tail for wgrad).  A wrong symbol of A
    plus one of C through the staged calls, the one of C alone through the one-call chain; the whole
    corrected C, the parity blocks, the patched operands and the report are compared with what
    the oracle computes for the full instance.  Then Section V step 1 runs once more from the C
    that is stored in memory (the fused check works from the accumulators and never reads it)."""
    w = configs.ALL[wname]
    n, k, m = w.n, w.k, w.m
    rng = inputs.rng_for(4, {"cfg4-fwd": 0, "cfg4-dgrad": 1, "cfg4-wgrad": 2}[wname])
    faults = [inputs.Fault(MAT_A, n - 5, k - 3, 12.0), inputs.Fault(MAT_C, 4321 % n, m - 1, -33.0)]
    A, B, A2, B2, cf, eff = _trial(rng, n, k, m, w.dtype, w.law_a, w.law_b, faults)
    cfb = [(0,) + c for c in cf]
    g = H.run_gpu(A, B, A2, B2, cfb, w.tau, w.dtype, w.trans_a, w.trans_b, reverify=True)
    o = H.run_oracle(A, B, A2, B2, cfb, w.tau)
    assert o[0].status == oc.CORRECTED and [e[:3] for e in o[0].errors] == [e[:3] for e in eff]
    # (a located magnitude is read from a plain syndrome, an fp32 sum whose rounding noise stays below
    # half of that family's threshold; the corrected symbol itself is re-evaluated and held to 1e-5)
    tol_mag = 0.5 * max(w.tau.r1, w.tau.q1)
    H.compare(g, o, 1e-5, tol_mag=tol_mag, what=wname + " staged")
    assert g.reverify_status == gecc.CLEAN
    AP, BP = oc.encode_a(A), oc.encode_b(B)
    assert np.allclose(g.A_par[0], AP, rtol=1e-12, atol=1e-12 * np.abs(AP).max())
    assert np.allclose(g.B_par[0], BP.T, rtol=1e-12, atol=1e-12 * np.abs(BP).max())
    assert np.array_equal(g.A[0], A.astype(np.float64)) and np.array_equal(g.B[0], B.astype(np.float64))
    del g, o
    # the one call that bench.py times (its own order of the parity scans), C fault only
    g1 = H.run_gpu(A, B, A, B, cfb, w.tau, w.dtype, w.trans_a, w.trans_b, staged=False, reverify=True)
    o1 = H.run_oracle(A, B, A, B, cfb, w.tau)
    assert o1[0].status == oc.CORRECTED and [e[:3] for e in o1[0].errors] == [(MAT_C, 4321 % n, m - 1)]
    H.compare(g1, o1, 1e-5, tol_mag=tol_mag, what=wname + " one call")
    assert g1.reverify_status == gecc.CLEAN
    assert np.allclose(g1.A_par[0], AP, rtol=1e-12, atol=1e-12 * np.abs(AP).max())
    assert np.allclose(g1.B_par[0], BP.T, rtol=1e-12, atol=1e-12 * np.abs(BP).max())
