"""Many fault trials on one operand pair, without forming the product again.  TEST INFRASTRUCTURE ONLY.

`grid_code.protected_gemm` evaluates one trial from scratch: encode, (n+2) x k x (m+2) product,
syndromes, decoding.  A campaign of thousands of trials on one pair of operands (4096^3, 10 000
trials) cannot afford the product each time, and does not need it: a fault changes one row of
C-bar (a wrong symbol of A, E1 of Section II-A), one column (a wrong symbol of B, E2) or one symbol
(E3), and the four syndrome families of Section V step 1 are linear in C-bar, so the syndromes of
the faulty product are those of the clean one plus those of the change.  This module keeps the
clean C-bar and its syndromes, applies a trial's faults and every later correction as changes of
rows, columns and symbols (each change also moving the syndromes by its own contribution), takes
the decisions with the *same functions* as the full oracle (`detect`, `d0_correct`,
`known_lines_correct`, `audit_a`, `audit_b`, `LineThresholds` of `grid_code`; the audits are
evaluated on the operand lines a trial touched, all other lines re-encode to their stored
parities bit for bit), and undoes the changes afterwards.

Its order of steps is that of `grid_code.decode`.  It is pinned to it: tests/test_oracle_pins.py
runs every single placement and every pair of placements over A, B and C on tiny sizes, and
random trials with rounding noise on larger ones, through both and demands equal status, equal
positions, magnitudes and corrected C-bar to 1e-9.

The GPU path shares nothing with this file.
"""
from dataclasses import dataclass
from typing import List, Tuple

import numpy as np

from . import grid_code as oc


@dataclass
class TrialResult:
    status: int
    s: int
    t: int
    errors: List[Tuple[int, int, int, float]]     # (matrix, row, col, magnitude), sorted
    max_abs_synd: Tuple[float, float, float, float]
    left_in_cbar: float        # max |C-bar after decoding - clean C-bar| over everything the trial touched
    operands_restored: bool    # A and B after decoding equal the clean operands
    Cbar: np.ndarray = None    # C-bar after decoding (a copy; only when asked for)


class IncrementalOracle:
    def __init__(self, A, B, tau: oc.Thresholds):
        self.A = np.array(A, dtype=np.float64)
        self.B = np.array(B, dtype=np.float64)
        self.n, self.k = self.A.shape
        self.m = self.B.shape[1]
        self.tau = tau
        self.AP = oc.encode_a(self.A)                       # Section III, formed from the clean operands
        self.BP = oc.encode_b(self.B)
        self.clean = oc.encoded_product(self.A, self.AP, self.B, self.BP)   # the clean C-bar, formed once
        self.clean_synd = oc.syndromes(self.clean)          # rounding level
        self.W = self.clean.copy()                          # the C-bar of the trial at hand
        self.wn, self.wm = oc._w(self.n), oc._w(self.m)
        self.scale = float(np.max(np.abs(self.clean[:self.n, :self.m])))

    @property
    def C(self):
        """the clean data block (what a corrected C has to equal)"""
        return self.clean[:self.n, :self.m]

    # ---- changes of C-bar, each moving the four syndrome families by its own contribution ----
    def _add_row(self, i, v):
        """row i of C-bar += v (length m+2: the data part and the row's two parity symbols)"""
        m = self.m
        self._rows.add(i)
        self.W[i, :] += v
        d = v[:m]
        self.q1 += d
        self.q2 += (i + 1.0) * d
        self.r1[i] += d.sum() - v[m]
        self.r2[i] += (self.wm * d).sum() - v[m + 1]

    def _add_col(self, j, v):
        """column j of C-bar += v (length n+2)"""
        n = self.n
        self._cols.add(j)
        self.W[:, j] += v
        d = v[:n]
        self.r1 += d
        self.r2 += (j + 1.0) * d
        self.q1[j] += d.sum() - v[n]
        self.q2[j] += (self.wn * d).sum() - v[n + 1]

    def _add_sym(self, i, j, x):
        self._rows.add(i)
        self.W[i, j] += x
        self.r1[i] += x
        self.r2[i] += (j + 1.0) * x
        self.q1[j] += x
        self.q2[j] += (i + 1.0) * x

    @staticmethod
    def _set_operand(M, journal, i, j, value):
        if (i, j) not in journal:
            journal[(i, j)] = M[i, j]
        M[i, j] = value

    # ---- one trial -----------------------------------------------------------------------------
    def trial(self, a_faults, b_faults, c_faults, tau=None, keep_cbar=False) -> TrialResult:
        """a_faults: [(i, l, value)] symbols of A as the product reads them (stored values, not
        offsets); b_faults: [(l, j, value)]; c_faults: [(i, j, e)] offsets added to data symbols of
        the product.  The parities A_P, B_P are those of the clean operands (E1/E2 strike after
        they were formed).  tau: thresholds of this trial (default: the ones given at set-up)."""
        tau = tau if tau is not None else self.tau
        n, m = self.n, self.m
        A, B, AP, BP = self.A, self.B, self.AP, self.BP
        self._rows, self._cols = set(), set()
        ja, jb = {}, {}              # clean values of the operand symbols a trial writes
        self.r1, self.r2, self.q1, self.q2 = [v.copy() for v in self.clean_synd]
        try:
            # the product of the operands as read:
            # (A + dA)(B-bar + dB) = clean + dA B-bar + A-bar dB + dA dB
            ea = [(i, l, v - A[i, l]) for (i, l, v) in a_faults]
            eb = [(l, j, v - B[l, j]) for (l, j, v) in b_faults]
            for (i, l, e) in ea:
                self._add_row(i, e * np.concatenate([B[l, :], BP[l, :]]))
            for (l, j, e) in eb:
                self._add_col(j, np.concatenate([A[:, l], AP[:, l]]) * e)
            for (i, la, e1) in ea:
                for (lb, j, e2) in eb:
                    if la == lb:
                        self._add_sym(i, j, e1 * e2)
            for (i, l, v) in a_faults:
                self._set_operand(A, ja, i, l, v)
            for (l, j, v) in b_faults:
                self._set_operand(B, jb, l, j, v)
            for (i, j, e) in c_faults:
                assert 0 <= i < n and 0 <= j < m
                self._add_sym(i, j, e)
            status, s0, t0, errs, mx = self._decode(tau, ja, jb)
            rows, cols = sorted(self._rows), sorted(self._cols)
            left = 0.0
            if rows:
                left = max(left, float(np.max(np.abs(self.W[rows, :] - self.clean[rows, :]))))
            if cols:
                left = max(left, float(np.max(np.abs(self.W[:, cols] - self.clean[:, cols]))))
            restored = all(A[i, l] == v for ((i, l), v) in ja.items()) and \
                all(B[l, j] == v for ((l, j), v) in jb.items())
            return TrialResult(status, s0, t0, sorted(errs), mx, left, restored,
                               self.W.copy() if keep_cbar else None)
        finally:
            for i in self._rows:
                self.W[i, :] = self.clean[i, :]
            for j in self._cols:
                self.W[:, j] = self.clean[:, j]
            for (i, l), v in ja.items():
                A[i, l] = v
            for (l, j), v in jb.items():
                B[l, j] = v

    def _audit(self, ja, jb, tau_op):
        """`grid_code.audit_a / audit_b` on the operand lines the trial wrote to (column l of A,
        row l of B); every other line re-encodes to its stored parities bit for bit."""
        A, B, AP, BP = self.A, self.B, self.AP, self.BP
        la = sorted({l for (i, l) in ja})
        lb = sorted({l for (l, j) in jb})
        okA, LA = oc.audit_a(A[:, la], AP[:, la], tau_op) if la else (True, [])
        okB, LB = oc.audit_b(B[lb, :], BP[lb, :], tau_op) if lb else (True, [])
        return okA, [(i, la[x], e) for (i, x, e) in LA], okB, [(lb[x], j, e) for (x, j, e) in LB]

    def _decode(self, tau, ja, jb):
        """The steps of `grid_code.decode`, in its order, on the changed lines."""
        n, m, k = self.n, self.m, self.k
        A, B, AP, BP = self.A, self.B, self.AP, self.BP
        r1, r2, q1, q2 = self.r1, self.r2, self.q1, self.q2
        mx = tuple(float(np.max(np.abs(v))) if v.size else 0.0 for v in (r1, r2, q1, q2))
        Er, Et = oc.detect(r1, r2, q1, q2, tau)
        s0, t0 = len(Er), len(Et)
        if s0 == 0 and t0 == 0:
            return oc.CLEAN, s0, t0, [], mx
        if not oc.all_finite(r1, r2, q1, q2):
            return oc.UNCORRECTABLE, s0, t0, [], mx
        fix = None
        if 1 <= s0 <= 2 and 1 <= t0 <= 2:
            fix = oc.d0_correct(r1, r2, q1, q2, Er, Et, oc.LineThresholds(tau, n, m))
        if fix is not None:
            for (i, j, x) in fix:
                self._add_sym(i, j, -x)
            return oc.CORRECTED, s0, t0, [(oc.MAT_C, i, j, x) for (i, j, x) in fix], mx

        okA, LA, okB, LB = self._audit(ja, jb, tau.op)
        if not (okA and okB) or (len(LA) + len(LB) > oc.MAX_REPORTED):
            return oc.UNCORRECTABLE, s0, t0, [], mx
        errs = []
        c = tau.rep * np.sqrt(k)
        allow = (np.zeros(n), np.zeros(n), np.zeros(m), np.zeros(m))
        for (i, l, e) in LA:
            self._set_operand(A, ja, i, l, A[i, l] - e)
            foot = e * B[l, :]                       # B as the product read it
            self._add_row(i, -e * np.concatenate([B[l, :], BP[l, :]]))
            errs.append((oc.MAT_A, i, l, e))
            allow[0][i] += c * np.sqrt(np.sum(foot ** 2))
            allow[1][i] += c * np.sqrt(np.sum((self.wm * foot) ** 2))
            allow[2][:] += c * np.abs(foot)
            allow[3][:] += c * (i + 1) * np.abs(foot)
        for (l, j, e) in LB:
            self._set_operand(B, jb, l, j, B[l, j] - e)
            foot = A[:, l] * e                       # A already corrected
            self._add_col(j, -np.concatenate([A[:, l], AP[:, l]]) * e)
            errs.append((oc.MAT_B, l, j, e))
            allow[2][j] += c * np.sqrt(np.sum(foot ** 2))
            allow[3][j] += c * np.sqrt(np.sum((self.wn * foot) ** 2))
            allow[0][:] += c * np.abs(foot)
            allow[1][:] += c * (j + 1) * np.abs(foot)
        tau2 = oc.LineThresholds(tau, n, m, allow)
        Er, Et = oc.detect(r1, r2, q1, q2, tau2)
        s, t = len(Er), len(Et)
        if s == 0 and t == 0:
            return oc.CORRECTED, s0, t0, errs, mx
        if not oc.all_finite(r1, r2, q1, q2):
            return oc.UNCORRECTABLE, s0, t0, [], mx
        fix = None
        if 1 <= s <= 2 and 1 <= t <= 2:
            fix = oc.d0_correct(r1, r2, q1, q2, Er, Et, tau2)
        elif 1 <= min(s, t) <= 2:
            fix = oc.known_lines_correct(r1, r2, q1, q2, Er, Et, tau2)
        if fix is not None:
            for (i, j, x) in fix:
                self._add_sym(i, j, -x)
            return oc.CORRECTED, s0, t0, errs + [(oc.MAT_C, i, j, x) for (i, j, x) in fix], mx
        return oc.UNCORRECTABLE, s0, t0, [], mx
