"""Thin binding over the C ABI of libgecc (include/gecc.h): argument marshalling only.

Every step of the path (encode, product, syndromes, decoding, audit) runs in the HIP
kernels of the library.  PyTorch is used for device memory and streams.  There is no CPU
fallback: if the library is missing or fails to load, importing the entry points raises.
"""
import ctypes as C
import math
import os
from dataclasses import dataclass
from typing import List, Optional, Tuple

import torch

F32, BF16 = 0, 1
CLEAN, CORRECTED, UNCORRECTABLE, DETECTED = 0, 1, 2, 3
MAT_A, MAT_B, MAT_C = 0, 1, 2
MAX_ERR, MAX_FAULTS = 8, 1024
# kernel classes of the timing records (include/gecc.h)
(K_ENCODE_A, K_ENCODE_B, K_PARITY_R, K_PARITY_C, K_PRODUCT, K_THRESHOLD, K_DECODE, K_AUDIT_A, K_AUDIT_B,
 K_REPAIR, K_PARTIALS, K_STAGE2, K_TILE_A, K_TILE_B, K_AUDIT_AB) = range(15)
K_NAMES = ["encode_a", "encode_b", "parity_r", "parity_c", "product", "threshold", "decode", "audit_a", "audit_b",
           "repair", "partials", "stage2", "encode_a+parity_r", "encode_b+parity_c", "audit_a+audit_b"]

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libgecc.so")


class Params(C.Structure):
    _fields_ = [("n", C.c_int32), ("k", C.c_int32), ("m", C.c_int32), ("batch", C.c_int32),
                ("dtype", C.c_int32), ("trans_a", C.c_int32), ("trans_b", C.c_int32),
                ("refine", C.c_int32),
                ("lda", C.c_int64), ("ldb", C.c_int64), ("ldc", C.c_int64),
                ("stride_a", C.c_int64), ("stride_b", C.c_int64), ("stride_c", C.c_int64),
                ("tau_r1", C.c_double), ("tau_r2", C.c_double), ("tau_q1", C.c_double),
                ("tau_q2", C.c_double), ("tau_op", C.c_double), ("tau_rep", C.c_double),
                ("tau_rel", C.c_double), ("weighted", C.c_int32), ("block_n", C.c_int32), ("block_m", C.c_int32), ("reserved", C.c_int32)]


class Err(C.Structure):
    _fields_ = [("matrix", C.c_int32), ("row", C.c_int32), ("col", C.c_int32),
                ("reserved", C.c_int32), ("magnitude", C.c_double)]


class Report(C.Structure):
    _fields_ = [("status", C.c_int32), ("s", C.c_int32), ("t", C.c_int32), ("n_err", C.c_int32),
                ("err", Err * MAX_ERR), ("max_abs_synd", C.c_double * 4),
                ("n_total", C.c_int32), ("reserved", C.c_int32)]

    def errors(self) -> List[Tuple[int, int, int, float]]:
        return [(e.matrix, e.row, e.col, e.magnitude) for e in list(self.err)[:self.n_err]]


class Fault(C.Structure):
    _fields_ = [("batch", C.c_int32), ("row", C.c_int32), ("col", C.c_int32), ("offset", C.c_float)]


_lib = None
_SYMBOLS = ["gecc_create", "gecc_destroy", "gecc_workspace_bytes", "gecc_set_workspace",
            "gecc_a_par_len", "gecc_b_par_len", "gecc_c_par_len", "gecc_item_count", "gecc_encode_a", "gecc_encode_b",
            "gecc_multiply", "gecc_verify", "gecc_correct", "gecc_protected_gemm", "gecc_protected_gemm_retry",
            "gecc_protected_gemm_static", "gecc_panel_count", "gecc_protected_gemm_panels",
            "gecc_plain_gemm",
            "gecc_report_to_host", "gecc_syndromes_to_host", "gecc_timing_enable", "gecc_timing_read",
            "gecc_strerror"]


def lib():
    """Loads libgecc.so (built in-tree by paper_2508_04355_amd.build); raises if absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError("libgecc.so is not built: run `python -m paper_2508_04355_amd.build` "
                           "(there is no fallback path)")
    L = C.CDLL(_LIB_PATH)
    vp, i32, sz = C.c_void_p, C.c_int32, C.c_size_t
    L.gecc_create.argtypes = [C.POINTER(vp), C.POINTER(Params)]
    L.gecc_destroy.argtypes = [vp]
    L.gecc_destroy.restype = None
    L.gecc_workspace_bytes.argtypes = [vp]
    L.gecc_workspace_bytes.restype = sz
    L.gecc_set_workspace.argtypes = [vp, vp, sz]
    for f in ("gecc_a_par_len", "gecc_b_par_len", "gecc_c_par_len"):
        getattr(L, f).argtypes = [vp]
        getattr(L, f).restype = sz
    L.gecc_encode_a.argtypes = [vp, vp, vp, vp]
    L.gecc_encode_b.argtypes = [vp, vp, vp, vp]
    L.gecc_multiply.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, i32, vp]
    L.gecc_verify.argtypes = [vp, vp, vp, vp, i32, vp]
    L.gecc_correct.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp]
    L.gecc_protected_gemm.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp]
    L.gecc_protected_gemm_static.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp]
    L.gecc_panel_count.argtypes = [vp, i32]
    L.gecc_panel_count.restype = i32
    L.gecc_item_count.argtypes = [vp]
    L.gecc_item_count.restype = i32
    L.gecc_protected_gemm_panels.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, i32, vp, i32, vp]
    L.gecc_protected_gemm_retry.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, C.POINTER(Report), i32, vp, i32,
                                            C.POINTER(i32), vp]
    L.gecc_plain_gemm.argtypes = [vp, vp, vp, vp, vp]
    L.gecc_report_to_host.argtypes = [vp, vp, C.POINTER(Report), i32, vp]
    L.gecc_syndromes_to_host.argtypes = [vp, vp, vp]
    L.gecc_timing_enable.argtypes = [vp, i32, C.c_uint32]
    L.gecc_timing_read.argtypes = [vp, C.POINTER(C.c_float), C.POINTER(i32), i32, C.POINTER(i32)]
    L.gecc_strerror.argtypes = [C.c_int]
    L.gecc_strerror.restype = C.c_char_p
    for f in _SYMBOLS:
        if f not in ("gecc_destroy", "gecc_workspace_bytes", "gecc_a_par_len", "gecc_b_par_len",
                     "gecc_c_par_len", "gecc_strerror", "gecc_panel_count", "gecc_item_count"):
            getattr(L, f).restype = C.c_int
    _lib = L
    return L


class GeccError(RuntimeError):
    pass


def _check(rc):
    if rc != 0:
        raise GeccError("libgecc: %s (code %d)" % (lib().gecc_strerror(rc).decode(), rc))


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr(t: Optional[torch.Tensor]):
    return C.c_void_p(0 if t is None else t.data_ptr())


@dataclass
class Thresholds:
    r1: float
    r2: float
    q1: float
    q2: float
    op: float = 0.0
    rep: float = 16.0 * 2.0 ** -24     # rounding allowance for repaired lines (fp32 accumulation)
    rel: float = 2.0 ** -20            # relative rounding allowance of a syndrome value (fp32 sums)
    weighted: bool = True              # False: single-checksum mode (plain parities only)


def noise_thresholds(n, k, m, sigma_a, sigma_b, safety=16.0) -> Thresholds:
    """Detection thresholds from a rounding-noise model of the fp32-accumulated product.

    One symbol of C carries rounding noise eps ~ u * sigma_a sigma_b * k / sqrt(6)
    (u = 2^-24; a random walk of k roundings, each proportional to the running sum).
    A plain syndrome over L symbols has noise sqrt(L) eps, a weighted one
    eps * L^1.5 / sqrt(3).  `safety` covers the maximum over the lines of the matrix.
    """
    eps = 2.0 ** -24 * sigma_a * sigma_b * k / math.sqrt(6.0)
    return Thresholds(r1=safety * eps * math.sqrt(m), r2=safety * eps * m ** 1.5 / math.sqrt(3.0),
                      q1=safety * eps * math.sqrt(n), q2=safety * eps * n ** 1.5 / math.sqrt(3.0), op=0.0)


class Context:
    """One protected-product configuration plus its device workspace (a torch uint8 tensor)."""

    def __init__(self, n, k, m, dtype, tau: Thresholds, batch=1, trans_a=0, trans_b=0, refine=1,
                 lda=None, ldb=None, ldc=None, stride_a=None, stride_b=None, stride_c=None,
                 device="cuda:0", block=(0, 0)):
        self.n, self.k, self.m, self.batch, self.dtype = n, k, m, batch, dtype
        self.trans_a, self.trans_b = trans_a, trans_b
        lda = lda if lda is not None else (n if trans_a else k)
        ldb = ldb if ldb is not None else (k if trans_b else m)
        ldc = ldc if ldc is not None else m
        rows_a, rows_b = (k if trans_a else n), (m if trans_b else k)
        self.params = Params(n=n, k=k, m=m, batch=batch, dtype=dtype, trans_a=trans_a, trans_b=trans_b,
                             refine=refine, lda=lda, ldb=ldb, ldc=ldc,
                             stride_a=stride_a if stride_a is not None else rows_a * lda,
                             stride_b=stride_b if stride_b is not None else rows_b * ldb,
                             stride_c=stride_c if stride_c is not None else n * ldc,
                             tau_r1=tau.r1, tau_r2=tau.r2, tau_q1=tau.q1, tau_q2=tau.q2, tau_op=tau.op,
                             tau_rep=tau.rep, tau_rel=tau.rel, weighted=1 if tau.weighted else 0,
                             block_n=block[0], block_m=block[1], reserved=0)
        self._h = C.c_void_p()
        _check(lib().gecc_create(C.byref(self._h), C.byref(self.params)))
        self.device = torch.device(device)
        self.items = lib().gecc_item_count(self._h)
        nbytes = lib().gecc_workspace_bytes(self._h)
        self.workspace = torch.empty(nbytes + 256, dtype=torch.uint8, device=self.device)
        off = (-self.workspace.data_ptr()) % 256
        _check(lib().gecc_set_workspace(self._h, C.c_void_p(self.workspace.data_ptr() + off), nbytes))

    def __del__(self):
        h = getattr(self, "_h", None)
        if h and _lib is not None:
            _lib.gecc_destroy(h)
            self._h = None

    # ---- buffers --------------------------------------------------------------------------
    def alloc_parities(self):
        L = lib()
        f64 = dict(dtype=torch.float64, device=self.device)
        return (torch.empty(self.batch * L.gecc_a_par_len(self._h), **f64),
                torch.empty(self.batch * L.gecc_b_par_len(self._h), **f64),
                torch.empty(self.batch * L.gecc_c_par_len(self._h), **f64))

    def alloc_report(self):
        return torch.zeros(self.items * C.sizeof(Report), dtype=torch.uint8, device=self.device)

    def alloc_c(self):
        return torch.empty((self.batch, self.n, self.params.ldc), dtype=torch.float32, device=self.device)

    # ---- the calls of include/gecc.h ----------------------------------------------------------
    def encode_a(self, A, A_par):
        _check(lib().gecc_encode_a(self._h, _ptr(A), _ptr(A_par), _stream()))

    def encode_b(self, B, B_par):
        _check(lib().gecc_encode_b(self._h, _ptr(B), _ptr(B_par), _stream()))

    def multiply(self, A, A_par, B, B_par, Cmat, C_par, faults: Optional[torch.Tensor] = None, n_faults=0):
        _check(lib().gecc_multiply(self._h, _ptr(A), _ptr(A_par), _ptr(B), _ptr(B_par), _ptr(Cmat),
                                   _ptr(C_par), _ptr(faults), n_faults, _stream()))

    def verify(self, Cmat, C_par, report, fused=True):
        _check(lib().gecc_verify(self._h, _ptr(Cmat), _ptr(C_par), _ptr(report), 1 if fused else 0, _stream()))

    def correct(self, A, A_par, B, B_par, Cmat, C_par, report):
        _check(lib().gecc_correct(self._h, _ptr(A), _ptr(A_par), _ptr(B), _ptr(B_par), _ptr(Cmat),
                                  _ptr(C_par), _ptr(report), _stream()))

    def protected_gemm(self, A, B, Cmat, A_par, B_par, C_par, report):
        _check(lib().gecc_protected_gemm(self._h, _ptr(A), _ptr(B), _ptr(Cmat), _ptr(A_par), _ptr(B_par),
                                         _ptr(C_par), _ptr(report), _stream()))

    def protected_gemm_static(self, A, B, Cmat, A_par, B_par, C_par, report):
        """protected_gemm on the library's static scratch array (no workspace, no allocation)."""
        _check(lib().gecc_protected_gemm_static(self._h, _ptr(A), _ptr(B), _ptr(Cmat), _ptr(A_par),
                                                _ptr(B_par), _ptr(C_par), _ptr(report), _stream()))

    def panel_count(self, panels: int) -> int:
        return lib().gecc_panel_count(self._h, panels)

    def protected_gemm_panels(self, A, B, Cmat, C_partial, A_par, B_par, C_par_panels, reports, panels,
                              faults=None, n_faults=0):
        """The protected product one k-panel at a time (batch 1).  C_par_panels: P x c_par_len doubles,
        reports: P reports (device), with P = panel_count(panels)."""
        _check(lib().gecc_protected_gemm_panels(self._h, _ptr(A), _ptr(B), _ptr(Cmat), _ptr(C_partial), _ptr(A_par),
                                                _ptr(B_par), _ptr(C_par_panels), _ptr(reports), panels,
                                                _ptr(faults), n_faults, _stream()))

    def reports_to_host(self, report, count) -> List[Report]:
        host = (Report * count)()
        _check(lib().gecc_report_to_host(self._h, _ptr(report), host, count, _stream()))
        return list(host)

    def protected_gemm_retry(self, A, B, Cmat, A_par, B_par, C_par, report, max_retries=1, faults=None, n_faults=0):
        """protected_gemm with recomputation on UNCORRECTABLE (waits for the stream after every
        attempt).  Returns (host reports of the last attempt, products computed)."""
        host = (Report * self.items)()
        attempts = C.c_int32(0)
        _check(lib().gecc_protected_gemm_retry(self._h, _ptr(A), _ptr(B), _ptr(Cmat), _ptr(A_par), _ptr(B_par),
                                               _ptr(C_par), _ptr(report), host, max_retries,
                                               _ptr(faults), n_faults,
                                               C.byref(attempts), _stream()))
        return list(host), attempts.value

    def plain_gemm(self, A, B, Cmat):
        _check(lib().gecc_plain_gemm(self._h, _ptr(A), _ptr(B), _ptr(Cmat), _stream()))

    def report_to_host(self, report) -> List[Report]:
        host = (Report * self.items)()
        _check(lib().gecc_report_to_host(self._h, _ptr(report), host, self.items, _stream()))
        return list(host)

    def timing_enable(self, max_records: int, kinds=(K_PRODUCT,)):
        """Record an event pair around the next max_records launches of the given kernel classes."""
        mask = 0
        for kk in kinds:
            mask |= 1 << kk
        _check(lib().gecc_timing_enable(self._h, max_records, mask))

    def timing_read(self, cap: int) -> List[Tuple[int, float]]:
        """[(kernel class, milliseconds)] of the recorded launches, in launch order."""
        ms = (C.c_float * max(cap, 1))()
        kinds = (C.c_int32 * max(cap, 1))()
        cnt = C.c_int32(0)
        _check(lib().gecc_timing_read(self._h, ms, kinds, cap, C.byref(cnt)))
        return [(int(kinds[i]), float(ms[i])) for i in range(cnt.value)]

    def syndromes_to_host(self):
        """(items, 2n+2m) float64 numpy array: r1, r2, q1, q2 of the last verify (blocked mode: n, m
        are the block sizes)."""
        import numpy as np
        bn, bm = self.params.block_n or self.n, self.params.block_m or self.m
        out = np.empty((self.items, 2 * bn + 2 * bm), dtype=np.float64)
        _check(lib().gecc_syndromes_to_host(self._h, C.c_void_p(out.ctypes.data), _stream()))
        return out


def make_faults(entries, device="cuda:0") -> Tuple[Optional[torch.Tensor], int]:
    """entries: [(batch, row, col, offset)] -> device buffer of gecc_fault records."""
    if not entries:
        return None, 0
    arr = (Fault * len(entries))(*[Fault(int(b), int(r), int(c), float(e)) for (b, r, c, e) in entries])
    raw = torch.frombuffer(bytearray(bytes(arr)), dtype=torch.uint8).to(device)
    return raw, len(entries)
