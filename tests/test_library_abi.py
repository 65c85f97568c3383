"""CPU-side checks of the C-ABI library: it loads, exports every symbol the header declares,
validates its arguments, and never needs a GPU for that (no compute call is made here)."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2508_04355_amd", "libgecc.so")


@pytest.fixture(scope="module")
def built():
    if not os.path.exists(LIB):
        from paper_2508_04355_amd import build
        build.build(verbose=False)
    from paper_2508_04355_amd import gecc
    return gecc


def test_every_declared_symbol_is_exported(built):
    header = open(os.path.join(ROOT, "include", "gecc.h")).read()
    declared = set(re.findall(r"\b(gecc_[a-z_]+)\s*\(", header))
    assert {"gecc_encode_a", "gecc_encode_b", "gecc_multiply", "gecc_verify", "gecc_correct",
            "gecc_protected_gemm", "gecc_plain_gemm"} <= declared
    L = C.CDLL(LIB)
    for name in declared:
        assert hasattr(L, name), name
    assert declared == set(built._SYMBOLS)


def test_struct_layouts_match_the_header(built):
    assert C.sizeof(built.Err) == 24
    assert C.sizeof(built.Report) == 16 + 8 * 24 + 32 + 8
    assert C.sizeof(built.Fault) == 16
    assert C.sizeof(built.Params) == 8 * 4 + 6 * 8 + 7 * 8 + 4 * 4


def _params(built, **kw):
    d = dict(n=64, k=32, m=48, batch=1, dtype=built.F32, trans_a=0, trans_b=0, refine=1, lda=32, ldb=48,
             ldc=48, stride_a=64 * 32, stride_b=32 * 48, stride_c=64 * 48, tau_r1=1e-3, tau_r2=1e-3,
             tau_q1=1e-3, tau_q2=1e-3, tau_op=0.0, tau_rep=1e-6, tau_rel=1e-6, weighted=1, block_n=0, block_m=0, reserved=0)
    d.update(kw)
    return built.Params(**d)


def test_create_validates_arguments(built):
    L = built.lib()
    h = C.c_void_p()
    assert L.gecc_create(C.byref(h), C.byref(_params(built))) == 0
    ws = L.gecc_workspace_bytes(h)
    assert ws > 0 and ws % 256 == 0
    assert L.gecc_a_par_len(h) == 64 and L.gecc_b_par_len(h) == 64 and L.gecc_c_par_len(h) == 2 * 64 + 2 * 48 + 4
    # no workspace yet: compute entry points refuse before touching the GPU
    assert L.gecc_encode_a(h, C.c_void_p(16), C.c_void_p(16), None) == -2
    assert L.gecc_set_workspace(h, C.c_void_p(0), ws) == -1
    assert L.gecc_set_workspace(h, C.c_void_p(4096 + 8), ws) == -4
    assert L.gecc_set_workspace(h, C.c_void_p(4096), ws - 1) == -2
    L.gecc_destroy(h)
    for bad in (dict(n=0), dict(k=-1), dict(batch=0), dict(dtype=7), dict(trans_a=2), dict(lda=31),
                dict(ldb=47), dict(ldc=40), dict(tau_q1=-1.0), dict(tau_r2=float("nan")), dict(tau_rep=-1.0), dict(tau_rel=-1.0),
                dict(batch=2, stride_c=10), dict(weighted=2), dict(weighted=-1), dict(block_n=128), dict(block_n=64, block_m=64),
                dict(n=256, m=256, lda=32, ldb=256, ldc=256, block_n=128, block_m=96), dict(n=256, m=256, ldb=256, ldc=256, block_n=128, block_m=128, weighted=0)):
        assert L.gecc_create(C.byref(h), C.byref(_params(built, **bad))) == -1, bad
    assert L.gecc_create(None, C.byref(_params(built))) == -1
    for code in (0, -1, -2, -3, -4, -99):
        assert len(L.gecc_strerror(code)) > 0


def test_workspace_grows_with_the_problem(built):
    """(Shapes of 512 tiles and more: products of fewer tiles than compute units also hold the partial
    tiles of their k-split, at most 16 MiB, whatever the shape.)"""
    L = built.lib()
    sizes = []
    for n in (4096, 8192, 16384):
        h = C.c_void_p()
        assert L.gecc_create(C.byref(h), C.byref(_params(built, n=n, k=n, m=n, lda=n, ldb=n, ldc=n))) == 0
        sizes.append(L.gecc_workspace_bytes(h))
        L.gecc_destroy(h)
    assert sizes[0] < sizes[1] < sizes[2]
    # partial sums stay a small fraction of C (4 n m bytes)
    assert sizes[2] < 0.2 * 4 * 16384 * 16384
    h = C.c_void_p()
    assert L.gecc_create(C.byref(h), C.byref(_params(built, n=1024, k=1024, m=1024, lda=1024, ldb=1024, ldc=1024))) == 0
    assert L.gecc_workspace_bytes(h) < (16 << 20) + 0.3 * 4 * 1024 * 1024
    L.gecc_destroy(h)


def test_noise_thresholds_scale_with_shape(built):
    a = built.noise_thresholds(1024, 1024, 1024, 1.0, 1.0)
    b = built.noise_thresholds(4096, 1024, 1024, 1.0, 1.0)
    assert b.q1 == pytest.approx(2 * a.q1) and b.q2 == pytest.approx(8 * a.q2) and b.r1 == a.r1
    c = built.noise_thresholds(1024, 1024, 1024, 0.5, 1.0)
    assert c.r1 == pytest.approx(0.5 * a.r1)


def test_stated_thresholds_follow_the_noise_model(built):
    from paper_2508_04355_amd import configs
    for w in configs.ALL.values():
        t = built.noise_thresholds(w.n, w.k, w.m, w.sigma_a, w.sigma_b, 16.0)
        for got, want in zip((w.tau.r1, w.tau.r2, w.tau.q1, w.tau.q2), (t.r1, t.r2, t.q1, t.q2)):
            assert got == pytest.approx(want, rel=0.01), w.name


def test_every_compute_entry_point_checks_its_pointers_before_any_gpu_call(built):
    """Null and misaligned pointers come back as error codes (no exceptions, no abort), and they
    do so before the library touches the GPU: this test runs where there is none."""
    L = built.lib()
    h = C.c_void_p()
    assert L.gecc_create(C.byref(h), C.byref(_params(built))) == 0
    ws = L.gecc_workspace_bytes(h)
    assert L.gecc_set_workspace(h, C.c_void_p(1 << 20), ws) == 0      # any aligned address: never dereferenced here
    ok, nul, odd = C.c_void_p(1 << 16), C.c_void_p(0), C.c_void_p((1 << 16) + 2)
    i0 = C.c_int32(0)
    assert L.gecc_encode_a(h, nul, ok, None) == -1 and L.gecc_encode_a(h, ok, nul, None) == -1
    assert L.gecc_encode_a(h, odd, ok, None) == -4 and L.gecc_encode_a(h, ok, odd, None) == -4   # fp32 operand, fp64 parity
    assert L.gecc_encode_b(h, nul, ok, None) == -1 and L.gecc_encode_b(h, ok, odd, None) == -4
    args = [ok] * 6
    for pos in range(6):
        bad = list(args); bad[pos] = nul
        assert L.gecc_multiply(h, *bad, nul, 0, None) == -1, pos
        bad = list(args); bad[pos] = odd
        assert L.gecc_multiply(h, *bad, nul, 0, None) == -4, pos
    assert L.gecc_multiply(h, *args, nul, 1, None) == -1        # faults announced, list missing
    assert L.gecc_multiply(h, *args, ok, -1, None) == -1
    assert L.gecc_verify(h, ok, nul, ok, 1, None) == -1 and L.gecc_verify(h, ok, ok, nul, 1, None) == -1
    assert L.gecc_verify(h, nul, ok, ok, 0, None) == -1         # the stand-alone scan needs C
    for pos in range(7):
        bad = [ok] * 7; bad[pos] = nul
        assert L.gecc_correct(h, *bad, None) == -1, pos
    assert L.gecc_protected_gemm(h, ok, ok, ok, ok, ok, ok, nul, None) == -1
    assert L.gecc_protected_gemm(h, nul, ok, ok, ok, ok, ok, ok, None) == -1
    assert L.gecc_protected_gemm_retry(h, ok, ok, ok, ok, ok, ok, ok, None, 1, nul, 0, None, None) == -1   # no host report
    rep = (built.Report * 1)()
    assert L.gecc_protected_gemm_retry(h, ok, ok, ok, ok, ok, ok, ok, rep, -1, nul, 0, None, None) == -1    # negative retries
    assert L.gecc_plain_gemm(h, nul, ok, ok, None) == -1
    for f in (L.gecc_encode_a, L.gecc_encode_b):
        assert f(None, ok, ok, None) == -1                       # no context
    L.gecc_destroy(h)
