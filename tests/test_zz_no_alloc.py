"""The allocation-free entry point, gecc_protected_gemm_static, against gecc_protected_gemm.

It runs the same kernels on a scratch array that lives inside the library instead of a workspace
the caller hands over, so every output must equal the existing entry point's bit for bit.  Two
calls in a row share the array; the second one here is the smaller product, so it meets whatever
the first left behind.  This file is collected last on purpose."""
import ctypes as C

import numpy as np
import pytest
import torch

import gpu_harness as H
from paper_2508_04355_amd import gecc, inputs

pytestmark = pytest.mark.gpu


def _params(n, k, m, dtype, tau, batch=1):
    return gecc.Params(n=n, k=k, m=m, batch=batch, dtype=dtype, trans_a=0, trans_b=0, refine=1, lda=k, ldb=m,
                       ldc=m, stride_a=n * k, stride_b=k * m, stride_c=n * m, tau_r1=tau.r1, tau_r2=tau.r2,
                       tau_q1=tau.q1, tau_q2=tau.q2, tau_op=tau.op, tau_rep=tau.rep, tau_rel=tau.rel, weighted=1, block_n=0, block_m=0, reserved=0)


def _both_ways(n, k, m, dtype, seed):
    """One product through gecc_protected_gemm (workspace from torch) and through
    gecc_protected_gemm_static (no workspace at all), raw C ABI; returns both sets of outputs."""
    L = gecc.lib()
    rng = inputs.rng_for(98, seed)
    A, B = inputs.operands(rng, n, k, m, ("normal", 1.0), ("normal", 1.0), dtype)
    tau = gecc.noise_thresholds(n, k, m, 1.0, 1.0)
    dt = gecc.BF16 if dtype == "bf16" else gecc.F32
    st = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    out = []
    for static in (False, True):
        h = C.c_void_p()
        assert L.gecc_create(C.byref(h), C.byref(_params(n, k, m, dt, tau))) == 0
        dA, dB = H.to_dev(A[None], dtype, False), H.to_dev(B[None], dtype, False)
        f64 = dict(dtype=torch.float64, device=H.DEV)
        A_par, B_par = torch.zeros(2 * k, **f64), torch.zeros(2 * k, **f64)
        C_par = torch.zeros(2 * n + 2 * m + 4, **f64)
        Cd = torch.full((n, m), float("nan"), dtype=torch.float32, device=H.DEV)
        rep = torch.zeros(C.sizeof(gecc.Report), dtype=torch.uint8, device=H.DEV)
        ptr = lambda t: C.c_void_p(t.data_ptr())
        if static:
            assert L.gecc_protected_gemm(h, ptr(dA), ptr(dB), ptr(Cd), ptr(A_par), ptr(B_par), ptr(C_par),
                                         ptr(rep), st) == gecc_ERR_WORKSPACE      # it really has no workspace
            rc = L.gecc_protected_gemm_static(h, ptr(dA), ptr(dB), ptr(Cd), ptr(A_par), ptr(B_par), ptr(C_par),
                                              ptr(rep), st)
        else:
            ws = torch.empty(L.gecc_workspace_bytes(h) + 256, dtype=torch.uint8, device=H.DEV)
            off = (-ws.data_ptr()) % 256
            assert L.gecc_set_workspace(h, C.c_void_p(ws.data_ptr() + off), L.gecc_workspace_bytes(h)) == 0
            rc = L.gecc_protected_gemm(h, ptr(dA), ptr(dB), ptr(Cd), ptr(A_par), ptr(B_par), ptr(C_par), ptr(rep), st)
        assert rc == 0, L.gecc_strerror(rc)
        host = (gecc.Report * 1)()
        assert L.gecc_report_to_host(h, ptr(rep), host, 1, st) == 0
        out.append(dict(C=Cd.cpu().numpy(), A_par=A_par.cpu().numpy(), B_par=B_par.cpu().numpy(),
                        C_par=C_par.cpu().numpy(), status=host[0].status, s=host[0].s, t=host[0].t,
                        mx=list(host[0].max_abs_synd)))
        L.gecc_destroy(h)
    return A, B, out


gecc_ERR_WORKSPACE = -2
gecc_ERR_SCRATCH = -5


def test_static_scratch_entry_point_equals_the_workspace_one_on_two_calls_in_a_row():
    # bf16: the 256 x 256-tile kernel with ragged tiles; then a smaller fp32 product (generic kernel)
    for (n, k, m, dtype, seed) in [(1000, 512, 776, "bf16", 0), (300, 200, 260, "f32", 1)]:
        A, B, (ref, got) = _both_ways(n, k, m, dtype, seed)
        assert ref["status"] == gecc.CLEAN and got["status"] == gecc.CLEAN
        for name in ("C", "A_par", "B_par", "C_par"):
            assert np.array_equal(ref[name], got[name]), (name, n, k, m)
        assert (ref["s"], ref["t"], ref["mx"]) == (got["s"], got["t"], got["mx"])
        # and both are the product: element by element against the fp64 definition
        Cref = A.astype(np.float64) @ B.astype(np.float64)
        assert not np.isnan(got["C"]).any()
        assert np.abs(got["C"] - Cref).max() / np.abs(Cref).max() <= 1e-5


def test_static_scratch_entry_point_rejects_what_does_not_fit():
    L = gecc.lib()
    tau = gecc.noise_thresholds(512, 512, 512, 1.0, 1.0)
    h = C.c_void_p()
    assert L.gecc_create(C.byref(h), C.byref(_params(512, 512, 512, gecc.F32, tau, batch=1024))) == 0
    assert L.gecc_workspace_bytes(h) > (48 << 20)
    ok = C.c_void_p(1 << 16)
    assert L.gecc_protected_gemm_static(h, ok, ok, ok, ok, ok, ok, ok, None) == gecc_ERR_SCRATCH
    assert b"GECC_STATIC_SCRATCH_BYTES" in L.gecc_strerror(gecc_ERR_SCRATCH)
    assert L.gecc_protected_gemm_static(h, None, ok, ok, ok, ok, ok, ok, None) == -1
    L.gecc_destroy(h)
