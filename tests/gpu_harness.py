"""Shared driver for the GPU parity tests: runs one protected product through the C ABI
(via the Python binding) and the same inputs through the CPU oracle."""
from dataclasses import dataclass
from typing import List, Optional

import numpy as np
import torch

from oracle import grid_code as oc
from paper_2508_04355_amd import gecc, inputs

DEV = "cuda:0"


def to_dev(x: np.ndarray, dtype: str, trans: bool, ld: Optional[int] = None) -> torch.Tensor:
    """Logical matrix (or batch of matrices) -> device tensor in the storage layout."""
    x = np.ascontiguousarray(np.swapaxes(x, -1, -2) if trans else x)
    if ld is not None and ld != x.shape[-1]:
        pad = np.zeros(x.shape[:-1] + (ld,), dtype=x.dtype)
        pad[..., :x.shape[-1]] = x
        x = pad
    t = torch.from_numpy(x.astype(np.float32))
    if dtype == "bf16":
        t = t.to(torch.bfloat16)
    return t.to(DEV)


def from_dev(t: torch.Tensor, trans: bool, cols: int) -> np.ndarray:
    x = t.float().cpu().numpy().astype(np.float64)[..., :cols]
    return np.swapaxes(x, -1, -2) if trans else x


@dataclass
class GpuResult:
    reports: list
    C: np.ndarray          # (batch, n, m)
    A: np.ndarray          # (batch, n, k) logical, after correction
    B: np.ndarray
    A_par: np.ndarray      # (batch, 2, k)
    B_par: np.ndarray
    C_par: np.ndarray      # (batch, 2n+2m+4)
    synd: np.ndarray
    pad_untouched: bool = True   # the columns of C between m and ldc still hold what they held before
    reverify_status: Optional[int] = None   # gecc_verify(fused=0) on the stored C after correction


def run_gpu(A_enc, B_enc, A_mul, B_mul, c_faults, tau, dtype, trans_a=0, trans_b=0, refine=1,
            fused=True, ld_pad=0, staged=True, reverify=False) -> GpuResult:
    """All array arguments are (batch, rows, cols) or (rows, cols) float32 logical matrices.
    c_faults: [(batch, i, j, e)].  fused=False plants the C faults after the product (plain
    device writes) and verifies with the stand-alone syndrome scan instead."""
    A_enc, B_enc, A_mul, B_mul = [np.asarray(x, dtype=np.float32) for x in (A_enc, B_enc, A_mul, B_mul)]
    if A_enc.ndim == 2:
        A_enc, B_enc, A_mul, B_mul = A_enc[None], B_enc[None], A_mul[None], B_mul[None]
    batch, n, k = A_enc.shape
    m = B_enc.shape[2]
    lda = (n if trans_a else k) + ld_pad
    ldb = (k if trans_b else m) + ld_pad
    ldc = m + ld_pad
    ctx = gecc.Context(n, k, m, gecc.BF16 if dtype == "bf16" else gecc.F32,
                       gecc.Thresholds(tau.r1, tau.r2, tau.q1, tau.q2, tau.op, tau.rep, tau.rel, getattr(tau, 'weighted', True)), batch=batch,
                       trans_a=trans_a, trans_b=trans_b, refine=refine, lda=lda, ldb=ldb, ldc=ldc)
    dA = to_dev(A_enc, dtype, trans_a, lda)
    dB = to_dev(B_enc, dtype, trans_b, ldb)
    A_par, B_par, C_par = ctx.alloc_parities()
    rep = ctx.alloc_report()
    Cd = ctx.alloc_c()
    Cd.fill_(float("nan"))
    if not staged:
        # the one-call chain: everything in one stream-ordered sequence, C faults planted into its
        # product; there is no point between its encode and its product for an operand fault
        assert fused and np.array_equal(A_enc, A_mul) and np.array_equal(B_enc, B_mul)
        fl, nf = gecc.make_faults(c_faults, DEV)
        reports, attempts = ctx.protected_gemm_retry(dA, dB, Cd, A_par, B_par, C_par, rep, 0, fl, nf)
        assert attempts == 1
        return GpuResult(reports=reports, reverify_status=_reverify(ctx, Cd, C_par) if reverify else None,
                         C=Cd.cpu().numpy().astype(np.float64)[:, :, :m], pad_untouched=bool(torch.isnan(Cd[:, :, m:]).all()),
                         A=from_dev(dA, trans_a, n if trans_a else k), B=from_dev(dB, trans_b, k if trans_b else m),
                         A_par=A_par.cpu().numpy().reshape(batch, 2, k), B_par=B_par.cpu().numpy().reshape(batch, 2, k),
                         C_par=C_par.cpu().numpy().reshape(batch, -1), synd=ctx.syndromes_to_host())
    ctx.encode_a(dA, A_par)
    ctx.encode_b(dB, B_par)
    # operand faults strike after the parities were formed (E1/E2)
    dA.copy_(to_dev(A_mul, dtype, trans_a, lda))
    dB.copy_(to_dev(B_mul, dtype, trans_b, ldb))
    if fused:
        fl, nf = gecc.make_faults(c_faults, DEV)
        ctx.multiply(dA, A_par, dB, B_par, Cd, C_par, fl, nf)
        ctx.verify(Cd, C_par, rep, fused=True)
    else:
        ctx.multiply(dA, A_par, dB, B_par, Cd, C_par, None, 0)
        for (b, i, j, e) in c_faults:
            Cd[b, i, j] += e
        ctx.verify(Cd, C_par, rep, fused=False)
    synd = ctx.syndromes_to_host()
    ctx.correct(dA, A_par, dB, B_par, Cd, C_par, rep)
    reports = ctx.report_to_host(rep)
    torch.cuda.synchronize()
    return GpuResult(reports=reports, reverify_status=_reverify(ctx, Cd, C_par) if reverify else None,
                     C=Cd.cpu().numpy().astype(np.float64)[:, :, :m], pad_untouched=bool(torch.isnan(Cd[:, :, m:]).all()),
                     A=from_dev(dA, trans_a, n if trans_a else k), B=from_dev(dB, trans_b, k if trans_b else m),
                     A_par=A_par.cpu().numpy().reshape(batch, 2, k), B_par=B_par.cpu().numpy().reshape(batch, 2, k),
                     C_par=C_par.cpu().numpy().reshape(batch, -1), synd=synd)


def _reverify(ctx, Cd, C_par):
    """Section V step 1 once more, from the C that is stored in memory (the fused path never reads
    it back): status of batch item 0."""
    rep2 = ctx.alloc_report()
    ctx.verify(Cd, C_par, rep2, fused=False)
    return ctx.report_to_host(rep2)[0].status


def run_oracle(A_enc, B_enc, A_mul, B_mul, c_faults, tau) -> List[oc.Result]:
    A_enc, B_enc, A_mul, B_mul = [np.asarray(x, dtype=np.float64) for x in (A_enc, B_enc, A_mul, B_mul)]
    if A_enc.ndim == 2:
        A_enc, B_enc, A_mul, B_mul = A_enc[None], B_enc[None], A_mul[None], B_mul[None]
    out = []
    for b in range(A_enc.shape[0]):
        cf = [(i, j, e) for (bb, i, j, e) in c_faults if bb == b]
        out.append(oc.protected_gemm(A_enc[b], B_enc[b], A_mul[b], B_mul[b], cf,
                                     oc.Thresholds(tau.r1, tau.r2, tau.q1, tau.q2, tau.op, tau.rep, tau.rel, getattr(tau, 'weighted', True))))
    return out


def compare(g: GpuResult, o: List[oc.Result], tol_c: float, tol_mag: float = None, what=""):
    """Bit-exact status / positions / flagged counts; magnitudes and C within tolerance.

    tol_c: max |C_gpu - C_oracle| / max |C_oracle|  (the whole matrix, corrected symbols included).
    """
    for b, (rep, res) in enumerate(zip(g.reports, o)):
        tag = "%s item %d" % (what, b)
        assert rep.status == res.status, (tag, rep.status, res.status, rep.errors(), res.errors)
        if res.status == oc.UNCORRECTABLE:
            continue
        # the report lists the first MAX_ERR located errors and counts all of them
        assert rep.n_total == len(res.errors), (tag, rep.n_total, len(res.errors))
        ge, oe = rep.errors(), res.errors[:gecc.MAX_ERR]
        assert [(x[0], x[1], x[2]) for x in ge] == [(x[0], x[1], x[2]) for x in oe], (tag, ge, oe)
        scale = float(np.max(np.abs(res.C)))
        mt = tol_mag if tol_mag is not None else 10 * tol_c * scale
        for x, y in zip(ge, oe):
            assert abs(x[3] - y[3]) <= mt + 1e-6 * abs(y[3]), (tag, x, y)
        assert not np.isnan(g.C[b]).any(), (tag, "some symbol of C was never written")
        err = float(np.max(np.abs(g.C[b] - res.C))) / scale
        assert err <= tol_c, (tag, "C mismatch", err)
        # the parity blocks of C-bar as the decoder left them (repaired lines included)
        n, m = res.C.shape
        ref = np.concatenate([res.Cbar[:n, m], res.Cbar[:n, m + 1], res.Cbar[n, :m], res.Cbar[n + 1, :m],
                              res.Cbar[n:, m:].ravel()])
        assert np.allclose(g.C_par[b], ref, rtol=1e-10, atol=1e-11 * np.abs(ref).max()), (tag, "parity blocks")
        if res.status == oc.CORRECTED:
            assert np.max(np.abs(g.A[b] - res.A)) <= 1e-6 * max(1.0, np.max(np.abs(res.A))), tag
            assert np.max(np.abs(g.B[b] - res.B)) <= 1e-6 * max(1.0, np.max(np.abs(res.B))), tag


def run_gpu_blocked(A_enc, B_enc, A_mul, B_mul, c_faults, tau, dtype, block, trans_a=0, trans_b=0, staged=True):
    """Blocked grid code (one product, batch 1): block = (block_n, block_m).  c_faults: [(i, j, e)] in
    coordinates of the whole C.  Returns (reports per block in item order, C, A, B, C_par per item, synd)."""
    A_enc, B_enc, A_mul, B_mul = [np.asarray(x, dtype=np.float32)[None] for x in (A_enc, B_enc, A_mul, B_mul)]
    _, n, k = A_enc.shape
    m = B_enc.shape[2]
    ctx = gecc.Context(n, k, m, gecc.BF16 if dtype == "bf16" else gecc.F32,
                       gecc.Thresholds(tau.r1, tau.r2, tau.q1, tau.q2, tau.op, tau.rep, tau.rel), trans_a=trans_a,
                       trans_b=trans_b, block=block)
    dA, dB = to_dev(A_enc, dtype, trans_a), to_dev(B_enc, dtype, trans_b)
    A_par, B_par, C_par = ctx.alloc_parities()
    rep = ctx.alloc_report()
    Cd = ctx.alloc_c()
    Cd.fill_(float("nan"))
    fl, nf = gecc.make_faults([(0, i, j, e) for (i, j, e) in c_faults], DEV)
    if staged:
        ctx.encode_a(dA, A_par)
        ctx.encode_b(dB, B_par)
        dA.copy_(to_dev(A_mul, dtype, trans_a))
        dB.copy_(to_dev(B_mul, dtype, trans_b))
        ctx.multiply(dA, A_par, dB, B_par, Cd, C_par, fl, nf)
        ctx.verify(Cd, C_par, rep, fused=True)
        synd = ctx.syndromes_to_host()
        ctx.correct(dA, A_par, dB, B_par, Cd, C_par, rep)
        reports = ctx.report_to_host(rep)
    else:
        assert np.array_equal(A_enc, A_mul) and np.array_equal(B_enc, B_mul)
        reports, attempts = ctx.protected_gemm_retry(dA, dB, Cd, A_par, B_par, C_par, rep, 0, fl, nf)
        synd = ctx.syndromes_to_host()
    torch.cuda.synchronize()
    items = ctx.items
    return dict(reports=reports, C=Cd.cpu().numpy().astype(np.float64)[0, :, :m],
                A=from_dev(dA, trans_a, n if trans_a else k)[0], B=from_dev(dB, trans_b, k if trans_b else m)[0],
                A_par=A_par.cpu().numpy(), B_par=B_par.cpu().numpy(),
                C_par=C_par.cpu().numpy().reshape(items, -1), synd=synd)
