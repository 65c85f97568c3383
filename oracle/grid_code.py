"""CPU fp64 oracle for the grid-code protected matrix product.  TEST INFRASTRUCTURE ONLY.

This module is the slow, plain reference the GPU path is checked against.  It
is imported only by tests, by the smoke check and by the benchmark's CPU
baseline leg; nothing on the product path may call it, and it shares no code
with the HIP library.

Everything is numpy float64.  Indices in this API are 0-based; the paper's
weight for 0-based index i is i+1 (its index sets start at 1, Section II-A).

What follows the paper directly
  * encode_a / encode_b      -- Section III, definitions of A_P, B_P with
                                P_n1 = (1..1), P_n2 = (1..n) (same for m).
  * encoded_product          -- Section III, C-bar = A-bar B-bar and its four
                                blocks C, P_r, P_c, P_g.
  * syndromes / detect       -- Section V step 1, the four threshold tests.
  * d0_correct               -- Section V step 2 (s = 1 rule, 2x2 system for
                                s = 2; stated for s <= t, s > t is its mirror image).
  * single_checksum_correct / decode_single_checksum
                             -- the conventional checksum scheme Section VI compares with
                                (Table 1), as Appendix A uses it: plain parities only.
  * known_lines_correct      -- Theorem 2 and its proof (Appendix B): errors in
                                any number of columns are corrected from the
                                column parities once they are confined to at
                                most two known rows (and the mirror image).
  * global_syndromes         -- Definition 1, constraint (3) (used by the
                                Lemma 3 rank pin only; the decoder of
                                Section V never reads P_g).

Readings taken where the paper is silent or garbled (each is listed again in
the design notes of the repository):
  * the 2x2 right-hand side is "sum minus parity" (Section V prints the
    opposite sign there but subtracts the solution afterwards and Eq. (5)
    uses sum minus parity);
  * the weighted tests compare against the *second* parity symbol
    (the "otherwise" branch of Section V step 1 prints m+1 / n+1 twice);
  * one threshold per syndrome family (tau_r1, tau_r2, tau_q1, tau_q2)
    instead of a single delta, because the weighted sums carry weights up
    to n (or m) and therefore n-times larger rounding noise;
  * operand errors (E1/E2 of Section II-A) hit the data part of A or B
    after the parity rows/columns were formed and before the product reads
    them, so every product term sees the same corrupted symbol;
  * completion D1 (operand audit) -- Section II-A reduces operand errors to
    the errors they cause in C, and Section VI reports 100 % for its scenarios
    a, b, d, e, without a locating rule being given.  Because a corrupted a_il
    also enters row i's own two parity symbols, the row syndromes are blind
    to it; D1 re-forms the operand parities, diffs them with the stored
    ones (each column of A-bar is a two-parity codeword, Section III),
    locates row = weighted/plain ratio, patches the operand and removes the
    rank-one footprint e * b-bar_l from C-bar, then re-runs Section V.
  * every estimate is verified: after the tentative correction all
    syndromes of the flagged rows/columns must fall inside the thresholds
    (propagated through the estimate), otherwise the pattern is handed on.
  * after an operand repair the lines it touched carry extra rounding noise
    in any finite-precision product (the corrupted term e * b_lj sat in the
    running sum of every symbol of that row), so the second pass of Section V
    widens the thresholds of those lines by rep * sqrt(k) * |footprint|
    (root-sum-square over a whole repaired line).  With rep = 0 this is the
    plain second pass.
  * a syndrome is a difference of sums of computed symbols, so in any
    finite-precision product its own rounding error grows with its magnitude
    (Section V closes on the remark that corrected symbols are off by rounding
    only); when an
    estimate is verified, every syndrome y is therefore trusted to
    tau + rel * |y| instead of tau.  Detection itself uses tau alone, and
    rel = 0 gives the plain rule.
  * Theorem 2 presupposes that the rows (columns) of the errors are known; the
    only knowledge the decoder has is Section V step 1, so the at most two
    flagged rows are taken as the known rows when three or more columns are
    flagged (and the other way round).  A row whose own two syndromes vanish
    although it holds errors (the construction of Section IV) is not known;
    then the verification fails and nothing is corrected.  The theorem's
    errors all lie in C-bar, so this decoder runs after the operand audit
    (on what the repair leaves, or on the whole pattern when the operands
    are intact): a wrong symbol of A a few rows from a known row would
    otherwise be taken for a row full of small errors of C.
  * a syndrome or a parity difference that is NaN or infinite counts as outside
    its threshold (Section V step 1 clears a line only when its test holds);
    a pattern with such a value is UNCORRECTABLE: subtracting an estimate
    cannot restore the symbol, the product has to be computed again.
  * the located-error list of a result is complete here; the library's
    report carries the first MAX_REPORTED entries and the total.
  * for s = t = 2 the 2x2 systems are first evaluated under the two sparse
    hypotheses "one error per flagged column" (a column with a single error
    is the s = 1 rule applied to that column); in exact arithmetic this
    equals the 2x2 solution, numerically it avoids dividing a weighted
    syndrome (noise ~ n^1.5) by s2 - s1.

parity pins: see tests/test_oracle_pins.py (exact integer brute force of the
product, block closed forms, zero syndromes, Theorem 1 enumeration, every
single and pair placement over A, B, C on tiny sizes, the counter-example of
Section IV, the rank statement of Lemma 3 built from Eq. (5), reductions to
the single-checksum and weighted-checksum schemes).
"""
from dataclasses import dataclass, field
from typing import List, Optional, Tuple

import numpy as np

CLEAN, CORRECTED, UNCORRECTABLE = 0, 1, 2
MAT_A, MAT_B, MAT_C = 0, 1, 2
MAX_REPORTED = 8          # operand errors one audit accepts; entries the library's report lists


@dataclass
class Thresholds:
    """Detection thresholds, one per syndrome family (Section V, delta)."""
    r1: float
    r2: float
    q1: float
    q2: float
    op: float = 0.0       # operand audit: |parity difference| > op flags a line
    rep: float = 0.0      # relative rounding allowance for lines touched by an operand repair
    rel: float = 0.0      # relative rounding allowance of a syndrome value (verification only)
    weighted: bool = True # False: single-checksum mode, the second parity of every line is ignored


class LineThresholds:
    """Per-line thresholds: the four numbers of `Thresholds` plus per-line allowances."""

    def __init__(self, tau, n, m, allow=None):
        z = np.zeros
        a = allow if allow is not None else (z(n), z(n), z(m), z(m))
        self.r1 = tau.r1 + a[0]
        self.r2 = tau.r2 + a[1]
        self.q1 = tau.q1 + a[2]
        self.q2 = tau.q2 + a[3]
        self.rel = tau.rel

    def trusted_to(self, r1, r2, q1, q2):
        """Uncertainty of each syndrome value: threshold plus rel * |value|."""
        u = LineThresholds.__new__(LineThresholds)
        u.r1 = self.r1 + self.rel * np.abs(r1)
        u.r2 = self.r2 + self.rel * np.abs(r2)
        u.q1 = self.q1 + self.rel * np.abs(q1)
        u.q2 = self.q2 + self.rel * np.abs(q2)
        u.rel = self.rel
        return u


@dataclass
class Result:
    status: int
    s: int                               # flagged rows at first detection
    t: int                               # flagged columns at first detection
    errors: List[Tuple[int, int, int, float]]   # (matrix,row,col,magnitude) sorted
    Cbar: np.ndarray                     # corrected encoded product
    A: np.ndarray                        # (possibly patched) left operand
    B: np.ndarray                        # (possibly patched) right operand
    max_abs_synd: Tuple[float, float, float, float] = (0.0, 0.0, 0.0, 0.0)

    @property
    def C(self):
        n, m = self.Cbar.shape[0] - 2, self.Cbar.shape[1] - 2
        return self.Cbar[:n, :m]


def _w(n):
    """P_n2 of Section III: (1, 2, ..., n)."""
    return np.arange(1, n + 1, dtype=np.float64)


# ---------------------------------------------------------------- Section III
def encode_a(A):
    """A_P (2 x k): row 0 = P_n1 A (column sums), row 1 = P_n2 A (Section III)."""
    A = np.asarray(A, dtype=np.float64)
    n, k = A.shape
    AP = np.empty((2, k), dtype=np.float64)
    AP[0, :] = A.sum(axis=0)
    AP[1, :] = (_w(n)[:, None] * A).sum(axis=0)
    return AP


def encode_b(B):
    """B_P (k x 2): col 0 = B P_m1^T (row sums), col 1 = B P_m2^T (Section III)."""
    B = np.asarray(B, dtype=np.float64)
    k, m = B.shape
    BP = np.empty((k, 2), dtype=np.float64)
    BP[:, 0] = B.sum(axis=1)
    BP[:, 1] = (B * _w(m)[None, :]).sum(axis=1)
    return BP


def encoded_product(A, AP, B, BP):
    """C-bar = [A; A_P] [B  B_P]  ((n+2) x (m+2)), Section III."""
    Abar = np.vstack([np.asarray(A, dtype=np.float64), AP])
    Bbar = np.hstack([np.asarray(B, dtype=np.float64), BP])
    return Abar @ Bbar


def inject_c(Cbar, faults):
    """E3 of Section II-A: add e to data symbol (i, j) of the product."""
    n, m = Cbar.shape[0] - 2, Cbar.shape[1] - 2
    for (i, j, e) in faults:
        assert 0 <= i < n and 0 <= j < m
        Cbar[i, j] += e


# ------------------------------------------------------------------ Section V
def syndromes(Cbar):
    """The four families of Section V step 1, as (sum) - (parity symbol).

    r1_i = sum_j c_ij       - cbar_{i,m+1}      r2_i = sum_j j c_ij - cbar_{i,m+2}
    q1_j = sum_i c_ij       - cbar_{n+1,j}      q2_j = sum_i i c_ij - cbar_{n+2,j}
    (paper's 1-based i, j inside the weights).
    """
    n, m = Cbar.shape[0] - 2, Cbar.shape[1] - 2
    C = Cbar[:n, :m]
    r1 = C.sum(axis=1) - Cbar[:n, m]
    r2 = (C * _w(m)[None, :]).sum(axis=1) - Cbar[:n, m + 1]
    q1 = C.sum(axis=0) - Cbar[n, :m]
    q2 = (_w(n)[:, None] * C).sum(axis=0) - Cbar[n + 1, :m]
    return r1, r2, q1, q2


def global_syndromes(Cbar):
    """Constraint (3) of Definition 1: the four global parity checks."""
    n, m = Cbar.shape[0] - 2, Cbar.shape[1] - 2
    C = Cbar[:n, :m]
    wn, wm = _w(n), _w(m)
    g = np.empty(4)
    g[0] = C.sum() - Cbar[n, m]
    g[1] = (C * wm[None, :]).sum() - Cbar[n, m + 1]
    g[2] = (wn[:, None] * C).sum() - Cbar[n + 1, m]
    g[3] = (wn[:, None] * C * wm[None, :]).sum() - Cbar[n + 1, m + 1]
    return g


def detect(r1, r2, q1, q2, tau):
    """E_r, E_t of Section V step 1 (a line is flagged if either test fails).
    tau: Thresholds (one number per family) or LineThresholds (per-line arrays).

    Section V clears the product when |sum - parity| <= delta holds for every line and
    puts a line into E_r / E_t otherwise.  A line is therefore flagged when its
    syndrome is *not* inside the threshold, which also holds for a syndrome that is
    not a number (a symbol of C that became NaN or infinite)."""
    Er = np.nonzero(~(np.abs(r1) <= tau.r1) | ~(np.abs(r2) <= tau.r2))[0]
    Et = np.nonzero(~(np.abs(q1) <= tau.q1) | ~(np.abs(q2) <= tau.q2))[0]
    return [int(i) for i in Er], [int(j) for j in Et]


def all_finite(*vectors):
    """False when a syndrome (or parity difference) is NaN or infinite: Section V's subtraction
    cannot restore such a symbol, so the pattern is handed back for recomputation."""
    return all(bool(np.all(np.isfinite(v))) for v in vectors)


def _residual_ok(est, r1, r2, q1, q2, Er, Et, tau):
    """All syndromes of the flagged lines must be explained by the estimate.

    est: list of (i, j, x, u): error x at (i, j) known to within +-u.
    """
    for i in Er:
        sx = sum(x for (ii, j, x, u) in est if ii == i)
        su = sum(u for (ii, j, x, u) in est if ii == i)
        wx = sum((j + 1) * x for (ii, j, x, u) in est if ii == i)
        wu = sum((j + 1) * u for (ii, j, x, u) in est if ii == i)
        if abs(r1[i] - sx) > tau.r1[i] + su:
            return False
        if abs(r2[i] - wx) > tau.r2[i] + wu:
            return False
    for j in Et:
        sx = sum(x for (i, jj, x, u) in est if jj == j)
        su = sum(u for (i, jj, x, u) in est if jj == j)
        wx = sum((i + 1) * x for (i, jj, x, u) in est if jj == j)
        wu = sum((i + 1) * u for (i, jj, x, u) in est if jj == j)
        if abs(q1[j] - sx) > tau.q1[j] + su:
            return False
        if abs(q2[j] - wx) > tau.q2[j] + wu:
            return False
    return True


def solve_2x2(w1, w2, y1, y2):
    """Solve [[1, 1], [w1, w2]] (e1, e2)^T = (y1, y2)^T (Section V, s = 2)."""
    e2 = (y2 - w1 * y1) / (w2 - w1)
    e1 = y1 - e2
    return e1, e2


def d0_correct(r1, r2, q1, q2, Er, Et, tau):
    """Section V step 2 for 1 <= s, t <= 2.

    tau: LineThresholds.  Returns the verified list [(i, j, x)] of C errors,
    or None when no estimate explains the syndromes (the caller then tries the
    operand audit).
    """
    s, t = len(Er), len(Et)
    assert 1 <= s <= 2 and 1 <= t <= 2
    tau = tau.trusted_to(r1, r2, q1, q2)      # from here on: how far each syndrome value is trusted

    def accept(est):
        est = [e for e in est if abs(e[2]) > e[3]]       # drop insignificant parts
        if _residual_ok(est, r1, r2, q1, q2, Er, Et, tau):
            return sorted((i, j, x) for (i, j, x, u) in est)
        return None

    if s <= t:
        if s == 1:
            # one faulty row: every flagged column has its error in that row
            return accept([(Er[0], j, q1[j], tau.q1[j]) for j in Et])
        s1, s2 = Er
        t1, t2 = Et
        diag = accept([(s1, t1, q1[t1], tau.q1[t1]), (s2, t2, q1[t2], tau.q1[t2])])
        anti = accept([(s1, t2, q1[t2], tau.q1[t2]), (s2, t1, q1[t1], tau.q1[t1])])
        if diag is not None and anti is not None:
            return None                                  # cannot tell them apart
        if diag is not None:
            return diag
        if anti is not None:
            return anti
        w1, w2 = s1 + 1.0, s2 + 1.0
        est = []
        for j in Et:
            e1, e2 = solve_2x2(w1, w2, q1[j], q2[j])
            u2 = (tau.q2[j] + w1 * tau.q1[j]) / (w2 - w1)
            u1 = tau.q1[j] + u2
            est += [(s1, j, e1, u1), (s2, j, e2, u2)]
        return accept(est)
    # s = 2 > t = 1: mirror image, rows play the role of columns
    return accept([(i, Et[0], r1[i], tau.r1[i]) for i in Er])


def known_lines_correct(r1, r2, q1, q2, Er, Et, tau):
    """Theorem 2 (proof in Appendix B): min(s, t) <= 2 < max(s, t).

    The lines on the short side are the known ones.  With the rows known,
    every flagged column j is decoded on its own from its two column
    syndromes: one known row s1 gives e_{s1,j} = q1_j, two known rows give
    the 2x2 system of Section V; columns known: the mirror image with the row
    syndromes.  The estimates are verified like those of d0_correct.
    Returns [(i, j, x)] or None.
    """
    s, t = len(Er), len(Et)
    assert 1 <= min(s, t) <= 2 < max(s, t)
    tau = tau.trusted_to(r1, r2, q1, q2)
    if s <= 2:
        known, lines, y1, y2, u1_, u2_ = Er, Et, q1, q2, tau.q1, tau.q2
        at = lambda line, kn: (kn, line)
    else:
        known, lines, y1, y2, u1_, u2_ = Et, Er, r1, r2, tau.r1, tau.r2
        at = lambda line, kn: (line, kn)
    est = []
    if len(known) == 1:
        for c in lines:
            i, j = at(c, known[0])
            est.append((i, j, y1[c], u1_[c]))
    else:
        w1, w2 = known[0] + 1.0, known[1] + 1.0
        for c in lines:
            e1, e2 = solve_2x2(w1, w2, y1[c], y2[c])
            ub = (u2_[c] + w1 * u1_[c]) / (w2 - w1)
            ua = u1_[c] + ub
            i, j = at(c, known[0])
            est.append((i, j, e1, ua))
            i, j = at(c, known[1])
            est.append((i, j, e2, ub))
    est = [e for e in est if abs(e[2]) > e[3]]           # drop insignificant parts
    if _residual_ok(est, r1, r2, q1, q2, Er, Et, tau):
        return sorted((i, j, x) for (i, j, x, u) in est)
    return None


# ------------------------------------------------------- completion D1: audit
def audit_a(A, AP, tau_op):
    """Re-form the parity rows of A and compare with the stored ones.

    Each column l of [A; A_P] is a codeword with two parities (Section III):
    a single wrong symbol a_il shows as (u1, u2) = (e, (i+1) e).
    Returns (ok, [(i, l, e)]); ok is False when some column cannot be
    explained by one wrong symbol (two errors in one column exceed the code).
    """
    n, k = A.shape
    cur = encode_a(A)
    u1 = cur[0] - AP[0]
    u2 = cur[1] - AP[1]
    found = []
    if not all_finite(u1, u2):
        return False, []
    for l in np.nonzero((np.abs(u1) > tau_op) | (np.abs(u2) > tau_op))[0]:
        if not abs(u1[l]) > tau_op:
            return False, []
        rho = u2[l] / u1[l]
        w = np.rint(rho)
        if not (abs(rho - w) < 0.25 and 1 <= w <= n):
            return False, []
        found.append((int(w) - 1, int(l), float(u1[l])))
    return True, found


def audit_b(B, BP, tau_op):
    """Mirror of audit_a for the parity columns of B. Returns [(l, j, e)]."""
    k, m = B.shape
    cur = encode_b(B)
    u1 = cur[:, 0] - BP[:, 0]
    u2 = cur[:, 1] - BP[:, 1]
    found = []
    if not all_finite(u1, u2):
        return False, []
    for l in np.nonzero((np.abs(u1) > tau_op) | (np.abs(u2) > tau_op))[0]:
        if not abs(u1[l]) > tau_op:
            return False, []
        rho = u2[l] / u1[l]
        w = np.rint(rho)
        if not (abs(rho - w) < 0.25 and 1 <= w <= m):
            return False, []
        found.append((int(l), int(w) - 1, float(u1[l])))
    return True, found


def decode(Cbar, A, AP, B, BP, tau):
    """Detection, correction and the operand completion, on copies.

    Cbar : (n+2) x (m+2) encoded product as computed (possibly corrupted)
    A, B : operands as the product read them (possibly corrupted)
    AP,BP: parities formed before the corruption
    On UNCORRECTABLE the returned buffers hold whatever the attempt left
    behind; a caller has to compute the product again (Section V step 1, last case).
    """
    Cbar = np.array(Cbar, dtype=np.float64)
    A = np.array(A, dtype=np.float64)
    B = np.array(B, dtype=np.float64)
    n, m = Cbar.shape[0] - 2, Cbar.shape[1] - 2

    r1, r2, q1, q2 = syndromes(Cbar)
    mx = tuple(float(np.max(np.abs(v))) if v.size else 0.0 for v in (r1, r2, q1, q2))
    Er, Et = detect(r1, r2, q1, q2, tau)
    s0, t0 = len(Er), len(Et)

    def done(status, errs):
        return Result(status, s0, t0, sorted(errs), Cbar, A, B, mx)

    if s0 == 0 and t0 == 0:
        return done(CLEAN, [])
    if not all_finite(r1, r2, q1, q2):
        return done(UNCORRECTABLE, [])

    fix = None
    if 1 <= s0 <= 2 and 1 <= t0 <= 2:
        fix = d0_correct(r1, r2, q1, q2, Er, Et, LineThresholds(tau, n, m))
    if fix is not None:
        for (i, j, x) in fix:
            Cbar[i, j] -= x
        return done(CORRECTED, [(MAT_C, i, j, x) for (i, j, x) in fix])

    # D1: operand audit, patch, rank-one repair, then Section V on the rest.  Theorem 2's
    # decoder runs only here, after the audit: it presumes that every error lies in C-bar
    # (Appendix B), and a wrong operand symbol near a known line would otherwise pass for a
    # line full of small errors of C.  With no operand hit the "rest" is the whole pattern.
    okA, LA = audit_a(A, AP, tau.op)
    okB, LB = audit_b(B, BP, tau.op)
    if not (okA and okB) or (len(LA) + len(LB) > MAX_REPORTED):
        return done(UNCORRECTABLE, [])
    errs = []
    k = A.shape[1]
    c = tau.rep * np.sqrt(k)
    allow = (np.zeros(n), np.zeros(n), np.zeros(m), np.zeros(m))
    wn, wm = _w(n), _w(m)
    for (i, l, e) in LA:
        A[i, l] -= e
        foot = e * B[l, :]                       # B as the product read it
        Cbar[i, :] -= e * np.concatenate([B[l, :], BP[l, :]])
        errs.append((MAT_A, i, l, e))
        allow[0][i] += c * np.sqrt(np.sum(foot ** 2))
        allow[1][i] += c * np.sqrt(np.sum((wm * foot) ** 2))
        allow[2][:] += c * np.abs(foot)
        allow[3][:] += c * (i + 1) * np.abs(foot)
    for (l, j, e) in LB:
        B[l, j] -= e
        foot = A[:, l] * e                       # A already corrected
        Cbar[:, j] -= np.concatenate([A[:, l], AP[:, l]]) * e
        errs.append((MAT_B, l, j, e))
        allow[2][j] += c * np.sqrt(np.sum(foot ** 2))
        allow[3][j] += c * np.sqrt(np.sum((wn * foot) ** 2))
        allow[0][:] += c * np.abs(foot)
        allow[1][:] += c * (j + 1) * np.abs(foot)
    tau2 = LineThresholds(tau, n, m, allow)

    r1, r2, q1, q2 = syndromes(Cbar)
    Er, Et = detect(r1, r2, q1, q2, tau2)
    s, t = len(Er), len(Et)
    if s == 0 and t == 0:
        return done(CORRECTED, errs)
    if not all_finite(r1, r2, q1, q2):
        return done(UNCORRECTABLE, [])
    fix = None
    if 1 <= s <= 2 and 1 <= t <= 2:
        fix = d0_correct(r1, r2, q1, q2, Er, Et, tau2)
    elif 1 <= min(s, t) <= 2:
        fix = known_lines_correct(r1, r2, q1, q2, Er, Et, tau2)
    if fix is not None:
        for (i, j, x) in fix:
            Cbar[i, j] -= x
        return done(CORRECTED, errs + [(MAT_C, i, j, x) for (i, j, x) in fix])
    return done(UNCORRECTABLE, [])


# ------------------------------------------ single-checksum mode (the comparison scheme of Section VI)
def single_checksum_correct(r1, q1, Er, Et, tau):
    """Conventional checksum correction: the plain parities alone.

    Appendix A uses exactly this inside the proof of Theorem 1: one erroneous symbol (s = t = 1)
    is corrected by a conventional checksum, and errors that all lie in one row s1 are
    found column by column from the plain column parities, e_{s1,j} = q1_j (mirror image for
    one column).  With one parity per line nothing else is decodable: two faulty rows and two
    faulty columns leave four candidate positions and three independent equations.
    Requires min(s, t) = 1.  tau: LineThresholds.  Verified like d0_correct: the single known
    line's own plain syndrome has to be the sum of what was found in it.
    Returns [(i, j, x)] or None.
    """
    s, t = len(Er), len(Et)
    assert min(s, t) == 1
    if s == 1:
        known, lines, y, u_, z, uz = Er[0], Et, q1, tau.q1 + tau.rel * np.abs(q1), r1, tau.r1 + tau.rel * np.abs(r1)
        at = lambda c: (known, c)
    else:
        known, lines, y, u_, z, uz = Et[0], Er, r1, tau.r1 + tau.rel * np.abs(r1), q1, tau.q1 + tau.rel * np.abs(q1)
        at = lambda c: (c, known)
    est = [(at(c) + (y[c], u_[c])) for c in lines if abs(y[c]) > u_[c]]
    if abs(z[known] - sum(e[2] for e in est)) > uz[known] + sum(e[3] for e in est):
        return None
    return sorted((i, j, x) for (i, j, x, u) in est)


def decode_single_checksum(Cbar, A, AP, B, BP, tau):
    """Detection and correction with the plain parities only (Section VI compares the grid code
    with such a checksum scheme; Table 1: it corrects one faulty line of C and nothing beyond).

    Same order as `decode`: one flagged row and one flagged column are corrected at once;
    otherwise the operands are audited first -- a wrong operand symbol shows in the plain parity
    of its line, but one parity cannot say where in the line it sits, so any hit ends
    UNCORRECTABLE -- and what is left is corrected when it is confined to one row or one column.
    """
    Cbar = np.array(Cbar, dtype=np.float64)
    A = np.array(A, dtype=np.float64)
    B = np.array(B, dtype=np.float64)
    n, m = Cbar.shape[0] - 2, Cbar.shape[1] - 2
    r1, r2, q1, q2 = syndromes(Cbar)
    mx = (float(np.max(np.abs(r1))), 0.0, float(np.max(np.abs(q1))), 0.0)
    inf = np.inf
    lt = LineThresholds(tau, n, m)
    only_plain = Thresholds(tau.r1, inf, tau.q1, inf)
    Er, Et = detect(r1, 0.0 * r1, q1, 0.0 * q1, only_plain)
    s0, t0 = len(Er), len(Et)

    def done(status, errs):
        return Result(status, s0, t0, sorted(errs), Cbar, A, B, mx)

    if s0 == 0 and t0 == 0:
        return done(CLEAN, [])
    if not all_finite(r1, q1):
        return done(UNCORRECTABLE, [])
    fix = None
    if s0 == 1 and t0 == 1:
        fix = single_checksum_correct(r1, q1, Er, Et, lt)
    if fix is None:
        u_a = encode_a(A)[0] - AP[0]
        u_b = encode_b(B)[:, 0] - BP[:, 0]
        if np.any(~(np.abs(u_a) <= tau.op)) or np.any(~(np.abs(u_b) <= tau.op)):
            return done(UNCORRECTABLE, [])
        if min(s0, t0) == 1:
            fix = single_checksum_correct(r1, q1, Er, Et, lt)
    if fix is None:
        return done(UNCORRECTABLE, [])
    for (i, j, x) in fix:
        Cbar[i, j] -= x
    return done(CORRECTED, [(MAT_C, i, j, x) for (i, j, x) in fix])


def protected_gemm(A_enc, B_enc, A_mul, B_mul, c_faults, tau):
    """The whole path: encode -> (operand faults) -> product -> (C faults) -> decode.

    A_enc, B_enc : operands at the time the parities are formed
    A_mul, B_mul : operands as the product reads them (equal to *_enc when no
                   E1/E2 fault is injected)
    c_faults     : [(i, j, e)] added to data symbols of the product (E3)
    """
    AP = encode_a(A_enc)
    BP = encode_b(B_enc)
    Cbar = encoded_product(A_mul, AP, B_mul, BP)
    inject_c(Cbar, c_faults)
    if not tau.weighted:
        return decode_single_checksum(Cbar, A_mul, AP, B_mul, BP, tau)
    return decode(Cbar, A_mul, AP, B_mul, BP, tau)


# ------------------------------------------- per-k-panel verification (linearity of Section III)
def panel_bounds(k, panels, align=64):
    """k cut into `panels` consecutive panels of equal length rounded up to `align` (the last one
    takes what is left; panels past the end of k are empty and dropped): [(k0, k1)]."""
    step = -(-(-(-k // panels)) // align) * align
    return [(g * step, min(k, (g + 1) * step)) for g in range(panels) if g * step < k]


def panel_thresholds(tau, kg, k):
    """Thresholds of a partial product over kg of the k terms: rounding noise of an fp32-accumulated
    sum grows in proportion to the number of terms, and so do the four detection thresholds."""
    f = kg / float(k)
    return Thresholds(tau.r1 * f, tau.r2 * f, tau.q1 * f, tau.q2 * f, tau.op, tau.rep, tau.rel, tau.weighted)


def protected_gemm_panels(A_enc, B_enc, A_mul, B_mul, c_faults_by_panel, tau, bounds):
    """The protected product one k-panel at a time.

    The encoding of Section III is linear in the operands: with the k index cut into panels,
    A-bar B-bar = sum_g A-bar[:, g] B-bar[g, :], and each term is itself an (n+2) x (m+2) matrix
    with the grid structure of Definition 1 -- its parity blocks are the products with the
    panel's slices of A_P and B_P.  So every partial product is encoded, multiplied, verified and
    corrected on its own (a fault is caught in the panel it strikes, before it is summed into
    C), and C is the sum of the corrected partial products.
    c_faults_by_panel: {g: [(i, j, e)]}.  Returns ([Result per panel], C).  Positions of operand
    errors are relative to the panel's slice.
    """
    k = A_enc.shape[1]
    results, C = [], None
    for g, (k0, k1) in enumerate(bounds):
        res = protected_gemm(A_enc[:, k0:k1], B_enc[k0:k1, :], A_mul[:, k0:k1], B_mul[k0:k1, :],
                             c_faults_by_panel.get(g, []), panel_thresholds(tau, k1 - k0, k))
        results.append(res)
        C = res.C.copy() if C is None else C + res.C
    return results, C


# --------------------------------------------------------- blocked grid code (Section III per block)
def protected_gemm_blocked(A_enc, B_enc, A_mul, B_mul, c_faults, tau, nb, mb):
    """The code of Section III applied to every nb x mb block of C on its own.

    Block (I, J) of C is the product of the row block A_I (nb x k) and the column block B_J
    (k x mb), so it is encoded, multiplied and decoded exactly as Section III and V prescribe for
    a product of that size: two parity rows per row block of A (weights 1..nb), two parity
    columns per column block of B (weights 1..mb), parity blocks P_r, P_c, P_g per block of C.
    Up to two errors are corrected *per block* (Theorem 1 holds block by block), the weights of
    the weighted sums stay below the block size, and no syndrome involves more than one block.
    tau: thresholds of one block.  n, m must be multiples of nb, mb.
    Returns ({(I, J): Result} with positions relative to the block, C, A, B): C assembled from the
    corrected blocks; A, B patched where the audit of a row block / column block located wrong
    symbols (a block that needed no audit leaves its operands alone).
    """
    n, k = A_enc.shape
    m = B_enc.shape[1]
    assert n % nb == 0 and m % mb == 0
    A_out = np.array(A_mul, dtype=np.float64)
    B_out = np.array(B_mul, dtype=np.float64)
    C = np.zeros((n, m))
    results = {}
    for I in range(n // nb):
        ri = slice(I * nb, (I + 1) * nb)
        for J in range(m // mb):
            cj = slice(J * mb, (J + 1) * mb)
            cf = [(i - I * nb, j - J * mb, e) for (i, j, e) in c_faults
                  if I * nb <= i < (I + 1) * nb and J * mb <= j < (J + 1) * mb]
            res = protected_gemm(A_enc[ri, :], B_enc[:, cj], A_mul[ri, :], B_mul[:, cj], cf, tau)
            results[(I, J)] = res
            C[ri, cj] = res.C
            for (mt, r, c, e) in res.errors:          # located operand symbols: the same in every block of the line
                if mt == MAT_A:
                    A_out[I * nb + r, c] = res.A[r, c]
                elif mt == MAT_B:
                    B_out[r, J * mb + c] = res.B[r, c]
    return results, C, A_out, B_out
