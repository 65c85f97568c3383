"""Pins of the CPU oracle against what the paper and plain mathematics fix.

None of these tests touches the GPU path.  Each pin is chosen so that a
plausible slip in the oracle (dropped term, wrong sign or index, transposed
operand, off-by-one weight) makes it fail.
"""
import itertools
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import grid_code as oc
from oracle.grid_code import CLEAN, CORRECTED, UNCORRECTABLE, MAT_A, MAT_B, MAT_C, Thresholds

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
TAU0 = Thresholds(1e-9, 1e-9, 1e-9, 1e-9, 0.0)       # exact-integer experiments


def int_mats(seed, n, k, m, lo=1, hi=5):
    rng = np.random.default_rng(seed)
    return (rng.integers(lo, hi + 1, (n, k)).astype(np.float64),
            rng.integers(lo, hi + 1, (k, m)).astype(np.float64))


# ---- pin 1: the data block is the plain definition c_ij = sum_l a_il b_lj (Section II-A),
#      evaluated with Python integers (exact), and the parity blocks follow their
#      closed forms (Section III) evaluated the same way.
@pytest.mark.parametrize("n,k,m", [(3, 4, 5), (5, 2, 3), (1, 1, 1), (6, 7, 2)])
def test_encoded_product_blocks_exact_integers(n, k, m):
    A, B = int_mats(11 + n, n, k, m, -7, 7)
    Cbar = oc.encoded_product(A, oc.encode_a(A), B, oc.encode_b(B))
    Ai = [[int(v) for v in row] for row in A]
    Bi = [[int(v) for v in row] for row in B]
    C = [[sum(Ai[i][l] * Bi[l][j] for l in range(k)) for j in range(m)] for i in range(n)]
    assert Cbar.shape == (n + 2, m + 2)
    for i in range(n):
        for j in range(m):
            assert Cbar[i, j] == C[i][j]
        assert Cbar[i, m] == sum(C[i][j] for j in range(m))                 # P_r col 1
        assert Cbar[i, m + 1] == sum((j + 1) * C[i][j] for j in range(m))   # P_r col 2
    for j in range(m):
        assert Cbar[n, j] == sum(C[i][j] for i in range(n))                 # P_c row 1
        assert Cbar[n + 1, j] == sum((i + 1) * C[i][j] for i in range(n))   # P_c row 2
    assert Cbar[n, m] == sum(C[i][j] for i in range(n) for j in range(m))
    assert Cbar[n, m + 1] == sum((j + 1) * C[i][j] for i in range(n) for j in range(m))
    assert Cbar[n + 1, m] == sum((i + 1) * C[i][j] for i in range(n) for j in range(m))
    assert Cbar[n + 1, m + 1] == sum((i + 1) * (j + 1) * C[i][j] for i in range(n) for j in range(m))


def test_parities_are_not_transposed_or_swapped():
    # asymmetric shapes and a single non-zero entry make any axis/weight slip visible
    A = np.zeros((4, 3)); A[2, 1] = 5.0
    AP = oc.encode_a(A)
    assert AP.shape == (2, 3) and AP[0, 1] == 5.0 and AP[1, 1] == 15.0 and AP[:, [0, 2]].sum() == 0
    B = np.zeros((3, 6)); B[0, 4] = 2.0
    BP = oc.encode_b(B)
    assert BP.shape == (3, 2) and BP[0, 0] == 2.0 and BP[0, 1] == 10.0 and BP[1:, :].sum() == 0


# ---- pin 2: all syndromes (Section V) and all global checks (Definition 1) vanish exactly
def test_zero_syndromes_on_clean_integer_product():
    for seed, (n, k, m) in enumerate([(4, 5, 6), (7, 3, 2), (16, 16, 16)]):
        A, B = int_mats(seed, n, k, m, -9, 9)
        Cbar = oc.encoded_product(A, oc.encode_a(A), B, oc.encode_b(B))
        for v in oc.syndromes(Cbar):
            assert np.all(v == 0)
        assert np.all(oc.global_syndromes(Cbar) == 0)
        res = oc.protected_gemm(A, B, A, B, [], TAU0)
        assert res.status == CLEAN and res.errors == [] and (res.s, res.t) == (0, 0)


def test_syndrome_signs_and_weights():
    # one wrong symbol e at (i, j): r1_i = q1_j = e, r2_i = (j+1) e, q2_j = (i+1) e  (sum - parity)
    n, m = 5, 7
    A, B = int_mats(3, n, 4, m)
    Cbar = oc.encoded_product(A, oc.encode_a(A), B, oc.encode_b(B))
    Cbar[3, 5] += 2.0
    r1, r2, q1, q2 = oc.syndromes(Cbar)
    exp = np.zeros(n); exp[3] = 2.0
    assert np.array_equal(r1, exp) and np.array_equal(r2, exp * 6)
    exp = np.zeros(m); exp[5] = 2.0
    assert np.array_equal(q1, exp) and np.array_equal(q2, exp * 4)


# ---- pin 3: 2x2 closed form of Section V against a generic solver
def test_solve_2x2_matches_linear_solver():
    rng = np.random.default_rng(5)
    for _ in range(50):
        w1, w2 = sorted(rng.choice(np.arange(1, 40), 2, replace=False).astype(float))
        y = rng.standard_normal(2)
        e = np.linalg.solve(np.array([[1.0, 1.0], [w1, w2]]), y)
        assert np.allclose(oc.solve_2x2(w1, w2, y[0], y[1]), e, rtol=1e-10, atol=1e-12)


# ---- pin 4: Theorem 1 -- every pattern inside <= 2 rows x <= 2 columns of C is corrected
def test_theorem1_all_patterns_in_2x2_blocks():
    n, k, m = 4, 3, 4
    A, B = int_mats(21, n, k, m)
    AP, BP = oc.encode_a(A), oc.encode_b(B)
    clean = oc.encoded_product(A, AP, B, BP)
    vals = (0, 1, -1, 3)
    count = 0
    for rows in itertools.combinations(range(n), 2):
        for cols in itertools.combinations(range(m), 2):
            cells = [(i, j) for i in rows for j in cols]
            for mags in itertools.product(vals, repeat=4):
                if not any(mags):
                    continue
                faults = [(i, j, float(e)) for (i, j), e in zip(cells, mags) if e]
                Cbar = clean.copy()
                oc.inject_c(Cbar, faults)
                res = oc.decode(Cbar, A, AP, B, BP, TAU0)
                assert res.status == CORRECTED, (faults,)
                assert np.array_equal(res.Cbar, clean), (faults,)
                assert [(mt, i, j) for (mt, i, j, _) in res.errors] == sorted((MAT_C, i, j) for (i, j, _) in faults)
                assert np.allclose([x for (*_, x) in res.errors], [e for (_, _, e) in sorted(faults)])
                count += 1
    assert count == 36 * (4 ** 4 - 1)


# ---- pin 5: every single placement and every pair over A u B u C (tiny sizes, integers)
def _placements(n, k, m):
    return ([(MAT_A, i, l) for i in range(n) for l in range(k)] +
            [(MAT_B, l, j) for l in range(k) for j in range(m)] +
            [(MAT_C, i, j) for i in range(n) for j in range(m)])


def _run_faults(A, B, AP, BP, placed):
    A2, B2, cf = A.copy(), B.copy(), []
    for (mt, r, c, e) in placed:
        if mt == MAT_A:
            A2[r, c] += e
        elif mt == MAT_B:
            B2[r, c] += e
        else:
            cf.append((r, c, e))
    Cbar = oc.encoded_product(A2, AP, B2, BP)
    oc.inject_c(Cbar, cf)
    return oc.decode(Cbar, A2, AP, B2, BP, TAU0)


@pytest.mark.parametrize("n,k,m", [(3, 3, 3), (4, 2, 3), (3, 4, 5)])
def test_every_single_error_is_located_and_corrected(n, k, m):
    A, B = int_mats(31 + k, n, k, m)
    AP, BP = oc.encode_a(A), oc.encode_b(B)
    clean = oc.encoded_product(A, AP, B, BP)
    for p in _placements(n, k, m):
        for e in (2.0, -7.0):
            res = _run_faults(A, B, AP, BP, [p + (e,)])
            assert res.status == CORRECTED, p
            assert res.errors == [p + (e,)]
            assert np.array_equal(res.Cbar, clean) and np.array_equal(res.A, A) and np.array_equal(res.B, B)


def _beyond_code(p1, p2):
    """Two errors in one column of A, or in one row of B: a two-parity line code has
    distance 3, so such pairs exceed the code (Section III: each column of A-bar and each
    row of B-bar carries exactly two parity symbols)."""
    if p1[0] == p2[0] == MAT_A:
        return p1[2] == p2[2]
    if p1[0] == p2[0] == MAT_B:
        return p1[1] == p2[1]
    return False


@pytest.mark.parametrize("n,k,m,mags", [(3, 3, 3, (1.0, 1.0)), (3, 3, 3, (2.0, -2.0)), (4, 2, 3, (3.0, -5.0)),
                                         (3, 3, 4, (-1.0, 4.0))])
def test_every_pair_of_errors_follows_the_correctability_map(n, k, m, mags):
    A, B = int_mats(41 + n + k + m, n, k, m)
    AP, BP = oc.encode_a(A), oc.encode_b(B)
    clean = oc.encoded_product(A, AP, B, BP)
    n_ok = n_beyond = 0
    for p1, p2 in itertools.combinations(_placements(n, k, m), 2):
        placed = [p1 + (mags[0],), p2 + (mags[1],)]
        res = _run_faults(A, B, AP, BP, placed)
        if _beyond_code(p1, p2):
            n_beyond += 1
            if res.status == CORRECTED:
                # indistinguishable from one error: the decoder "repairs" a codeword at
                # distance 1 -- C-bar is then consistent but the operand is not restored
                assert all(abs(v).max() < 1e-9 for v in oc.syndromes(res.Cbar))
            else:
                assert res.status == UNCORRECTABLE
            continue
        n_ok += 1
        assert res.status == CORRECTED, (p1, p2)
        assert res.errors == sorted(placed), (p1, p2)
        assert np.array_equal(res.Cbar, clean) and np.array_equal(res.A, A) and np.array_equal(res.B, B)
    assert n_ok > 0 and n_beyond > 0


def test_two_errors_in_one_operand_column_hit_the_bound():
    # A(0,l,e) + A(2,l,e) has the same column parities as A(1,l,2e): mis-located by construction;
    # A(0,l,e) + A(1,l,2e) gives a non-integer ratio 5/3: declared uncorrectable.
    n, k, m = 5, 3, 4
    A, B = int_mats(77, n, k, m)
    AP, BP = oc.encode_a(A), oc.encode_b(B)
    res = _run_faults(A, B, AP, BP, [(MAT_A, 0, 1, 1.0), (MAT_A, 2, 1, 1.0)])
    assert res.status == CORRECTED and res.errors == [(MAT_A, 1, 1, 2.0)]
    res = _run_faults(A, B, AP, BP, [(MAT_A, 0, 1, 1.0), (MAT_A, 1, 1, 2.0)])
    assert res.status == UNCORRECTABLE
    res = _run_faults(A, B, AP, BP, [(MAT_B, 1, 0, 1.0), (MAT_B, 1, 1, 2.0)])
    assert res.status == UNCORRECTABLE


# ---- pin 6: operand-error signature (Section II-A: an error in a_il reaches the whole row i)
def test_operand_error_footprint_and_blind_row_syndromes():
    n, k, m = 6, 5, 7
    A, B = int_mats(55, n, k, m)
    AP, BP = oc.encode_a(A), oc.encode_b(B)
    clean = oc.encoded_product(A, AP, B, BP)
    A2 = A.copy(); A2[4, 2] += 3.0
    d = oc.encoded_product(A2, AP, B, BP) - clean
    exp = np.zeros_like(d); exp[4, :] = 3.0 * np.concatenate([B[2], BP[2]])
    assert np.array_equal(d, exp)
    r1, r2, q1, q2 = oc.syndromes(clean + d)
    assert np.all(r1 == 0) and np.all(r2 == 0)
    assert np.array_equal(q1, 3.0 * B[2]) and np.array_equal(q2, 5 * 3.0 * B[2])
    B2 = B.copy(); B2[1, 3] -= 2.0
    d = oc.encoded_product(A, AP, B2, BP) - clean
    exp = np.zeros_like(d); exp[:, 3] = -2.0 * np.concatenate([A[:, 1], AP[:, 1]])
    assert np.array_equal(d, exp)
    r1, r2, q1, q2 = oc.syndromes(clean + d)
    assert np.all(q1 == 0) and np.all(q2 == 0)
    assert np.array_equal(r1, -2.0 * A[:, 1]) and np.array_equal(r2, 4 * -2.0 * A[:, 1])


# ---- pin 7: the counter-example of Section IV (values from the paper, tests/golden)
def _load_counterexample():
    rows = {"e1": [], "e2": []}
    where = {}
    for line in open(os.path.join(GOLDEN, "section4_counterexample.txt")):
        tok = line.split()
        if not tok or tok[0].startswith("#"):
            continue
        if tok[0].endswith("_rows"):
            where[tok[0][:2]] = [int(v) - 1 for v in tok[1:]]
        else:
            rows[tok[0]].append([float(v) for v in tok[1:]])
    return rows, where


def test_section4_counterexample_is_invisible_to_plain_sums_and_ambiguous():
    rows, where = _load_counterexample()
    n = m = 6
    def pattern(name, scale=1.0, at=None):
        E = np.zeros((n + 2, m + 2))
        for r, vals in zip(at or where[name], rows[name]):
            E[r, :len(vals)] = np.array(vals) * scale
        return E
    e1, e2 = pattern("e1"), pattern("e2")
    s1, s2 = oc.syndromes(e1), oc.syndromes(e2)
    # both patterns leave every row syndrome and every plain column sum at zero ...
    for s in (s1, s2):
        assert np.all(s[0] == 0) and np.all(s[1] == 0) and np.all(s[2] == 0)
    # ... and their weighted column syndromes are proportional: the printed e2 is twice the
    # pattern that collides with e1 (e1 moved to rows 3-4); the halved e2 collides exactly.
    assert np.array_equal(s2[3], 2 * s1[3])
    e1_shift = pattern("e1", at=where["e2"])
    assert np.array_equal(e1_shift * 2, e2)
    for a, b in zip(oc.syndromes(e1_shift), s1):
        assert np.array_equal(a, b)
    # the decoder must not "correct" such a pattern
    A, B = int_mats(9, n, 4, m)
    AP, BP = oc.encode_a(A), oc.encode_b(B)
    clean = oc.encoded_product(A, AP, B, BP)
    res = oc.decode(clean + e1, A, AP, B, BP, TAU0)
    assert res.status == UNCORRECTABLE and res.s == 0 and res.t == 3


# ---- pin 8: Lemma 3 / Eq. (5): the 16 constraints on a 3x3 error block have rank 8
def _eval_tokens(expr, env):
    return float(eval(expr, {"__builtins__": {}}, env))


def _oracle_constraint_matrix(n, m, srows, tcols):
    """Column p = response of (row, column, global) checks to a unit error at position p."""
    cols = []
    for i in srows:
        for j in tcols:
            E = np.zeros((n + 2, m + 2)); E[i, j] = 1.0
            r1, r2, q1, q2 = oc.syndromes(E)
            g = oc.global_syndromes(E)
            col = []
            for si in srows:
                col += [r1[si], r2[si]]
            col += [q2[tj] for tj in tcols] + [q1[tj] for tj in tcols]      # printed row order
            col += list(g)
            cols.append(col)
    return np.array(cols).T


@pytest.mark.parametrize("s,t", [((1, 2, 3), (1, 2, 3)), ((2, 5, 9), (1, 4, 6)), ((1, 3, 10), (7, 8, 12))])
def test_lemma3_rank_and_printed_matrix(s, t):
    env = dict(s1=s[0], s2=s[1], s3=s[2], t1=t[0], t2=t[1], t3=t[2])
    printed = []
    for line in open(os.path.join(GOLDEN, "eq5_system.txt")):
        if line.strip() and not line.startswith("#"):
            printed.append([_eval_tokens(tok, env) for tok in line.split()])
    printed = np.array(printed)
    assert printed.shape == (16, 9)
    n, m = 12, 14
    M = _oracle_constraint_matrix(n, m, [v - 1 for v in s], [v - 1 for v in t])
    # Row 15 of the printed matrix (the s-weighted global check) lists s1 s2 s3 three times;
    # with unknowns ordered row-major in (s, t) it has to read s1 s1 s1 s2 s2 s2 s3 s3 s3.
    fixed = printed.copy()
    fixed[14] = np.repeat([float(v) for v in s], 3)
    assert np.array_equal(M, fixed)
    assert np.linalg.matrix_rank(M) == 8
    # null direction = last column of the printed row-reduced matrix (e_p = -c_p e_9)
    last = [_eval_tokens(line, env) for line in open(os.path.join(GOLDEN, "lemma3_reduced_last_column.txt"))
            if line.strip() and not line.startswith("#")]
    null = np.array([-c for c in last] + [1.0])
    assert np.allclose(M @ null, 0, atol=1e-9)
    # consequence (Corollary 4): a 3x3 pattern along the null direction satisfies every
    # check of Definition 1, so it is invisible -- the decoder has to report "clean"
    A, B = int_mats(13, n, 3, m)
    AP, BP = oc.encode_a(A), oc.encode_b(B)
    Cbar = oc.encoded_product(A, AP, B, BP)
    scale = (s[0] - s[1]) * (t[0] - t[1])
    for p, (i, j) in enumerate((i, j) for i in s for j in t):
        Cbar[i - 1, j - 1] += null[p] * scale
    assert np.all(oc.global_syndromes(Cbar) == 0)
    res = oc.decode(Cbar, A, AP, B, BP, TAU0)
    assert res.status == CLEAN and (res.s, res.t) == (0, 0)


# ---- pin 9: reductions to the textbook schemes the paper builds on (Section I)
def test_reduces_to_single_checksum_abft_and_weighted_checksum():
    n, k, m = 8, 5, 9
    A, B = int_mats(99, n, k, m)
    AP, BP = oc.encode_a(A), oc.encode_b(B)
    Cbar = oc.encoded_product(A, AP, B, BP)
    Cbar[6, 2] += 4.0
    r1, r2, q1, q2 = oc.syndromes(Cbar)
    # checksum ABFT: the intersection of the flagged row and column locates the symbol, the
    # plain checksum difference is its error
    assert np.nonzero(r1)[0].tolist() == [6] and np.nonzero(q1)[0].tolist() == [2] and r1[6] == q1[2] == 4.0
    # weighted checksum: ratio of weighted to plain syndrome is the (1-based) position
    assert q2[2] / q1[2] == 7 and r2[6] / r1[6] == 3


# ---- pin 10: rounding remark of Section V -- with real data the corrected symbols agree
#      with an independently computed product up to rounding
def test_real_valued_correction_matches_independent_product():
    rng = np.random.default_rng(2)
    n, k, m = 40, 30, 50
    A, B = rng.standard_normal((n, k)), rng.standard_normal((k, m))
    tau = Thresholds(1e-8, 1e-6, 1e-8, 1e-6)
    ref = np.einsum("il,lj->ij", A, B)
    A2 = A.copy(); A2[7, 3] += 11.5
    res = oc.protected_gemm(A, B, A2, B, [(20, 41, -3.25)], tau)
    assert res.status == CORRECTED
    assert [(e[0], e[1], e[2]) for e in res.errors] == [(MAT_A, 7, 3), (MAT_C, 20, 41)]
    assert np.allclose([e[3] for e in res.errors], [11.5, -3.25], rtol=0, atol=1e-9)
    assert np.max(np.abs(res.C - ref)) < 1e-9 and np.max(np.abs(res.A - A)) < 1e-12


# ---- Theorem 2: any number of errors confined to at most two known rows (columns) ---------------
def _row_known(pattern_row, cols):
    """A row is known to Section V step 1 iff one of its two syndromes is nonzero."""
    e = dict(zip(cols, pattern_row))
    return sum(e.values()) != 0 or sum((j + 1) * x for j, x in e.items()) != 0


@pytest.mark.parametrize("transpose", [False, True])
def test_theorem2_errors_in_one_or_two_known_lines_and_three_or_more_of_the_other_kind(transpose):
    """Every pattern with entries from {0, 1, -2, 3} on one row and 4 columns, from {0, 1, -2} on two rows
    and 3 columns of a 4 x 5
    product (and the mirror image): corrected exactly from the parities of the other direction
    whenever each of the rows is flagged by its own syndromes; never corrected wrongly otherwise."""
    n, k, m = (5, 3, 4) if transpose else (4, 3, 5)
    A, B = int_mats(31, n, k, m)
    AP, BP = oc.encode_a(A), oc.encode_b(B)
    clean = oc.encoded_product(A, AP, B, BP)
    vals = (0, 1, -2, 3)
    nlines, nother = (m, n) if transpose else (n, m)       # known lines are rows unless transposed
    corrected = rejected = 0
    for nk in (1, 2):
        for known in itertools.combinations(range(nlines), nk):
            for others in itertools.combinations(range(nother), 3 if nk == 2 else 4):
                for mags in itertools.product(vals if nk == 1 else vals[:3], repeat=nk * len(others)):
                    M = np.array(mags).reshape(nk, len(others))
                    if not all(M[:, c].any() for c in range(len(others))):
                        continue                            # fewer than 3 lines of the other kind
                    if not all(M[r].any() for r in range(nk)):
                        continue
                    faults = []
                    for r, kn in enumerate(known):
                        for c, ot in enumerate(others):
                            if M[r, c]:
                                faults.append((ot, kn, float(M[r, c])) if transpose else (kn, ot, float(M[r, c])))
                    all_known = all(_row_known(M[r], others) for r in range(nk))
                    Cbar = clean.copy()
                    oc.inject_c(Cbar, faults)
                    res = oc.decode(Cbar, A, AP, B, BP, TAU0)
                    if all_known:
                        assert res.status == CORRECTED, (faults,)
                        assert np.array_equal(res.Cbar, clean), (faults,)
                        assert [(i, j) for (_, i, j, _) in res.errors] == sorted((i, j) for (i, j, _) in faults)
                        assert np.allclose([x for (*_, x) in res.errors], [e for (_, _, e) in sorted(faults)])
                        corrected += 1
                    else:
                        # a row whose sums cancel is invisible to step 1: the rows are not "known"
                        assert res.status != CORRECTED or np.array_equal(res.Cbar, clean), (faults,)
                        rejected += 1
    assert corrected > 5000 and rejected > 0


def test_theorem2_one_known_row_is_the_column_parity_rule():
    """Appendix B, case s = 1: the error in column j of the known row is that column's plain
    syndrome; checked against the injected values on a real-valued product."""
    rng = np.random.default_rng(5)
    n, k, m = 9, 6, 40
    A, B = rng.normal(size=(n, k)), rng.normal(size=(k, m))
    AP, BP = oc.encode_a(A), oc.encode_b(B)
    clean = oc.encoded_product(A, AP, B, BP)
    cols = list(range(3, 33, 2))
    e = rng.uniform(1.0, 5.0, size=len(cols)) * rng.choice([-1.0, 1.0], size=len(cols))
    Cbar = clean.copy()
    oc.inject_c(Cbar, [(4, j, x) for j, x in zip(cols, e)])
    r1, r2, q1, q2 = oc.syndromes(Cbar)
    assert np.allclose(q1[cols], e) and np.allclose(q2[cols], 5 * e)
    res = oc.decode(Cbar, A, AP, B, BP, Thresholds(1e-9, 1e-9, 1e-9, 1e-9))
    assert res.status == CORRECTED and res.s == 1 and res.t == len(cols)
    assert [(i, j) for (_, i, j, _) in res.errors] == [(4, j) for j in cols]
    assert np.allclose(res.Cbar, clean, atol=1e-12)


def test_theorem2_does_not_reach_three_by_three():
    """min(s, t) = 3: outside Theorem 2 (Lemma 3 shows that even known lines do not help)."""
    n, k, m = 6, 3, 6
    A, B = int_mats(33, n, k, m)
    AP, BP = oc.encode_a(A), oc.encode_b(B)
    Cbar = oc.encoded_product(A, AP, B, BP)
    oc.inject_c(Cbar, [(0, 0, 1.0), (1, 1, 2.0), (2, 2, 3.0)])
    assert oc.decode(Cbar, A, AP, B, BP, TAU0).status == UNCORRECTABLE


def test_theorem2_operand_errors_still_go_through_the_audit():
    """An error in A corrupts a whole row of C but leaves that row's own syndromes at zero
    (s = 0): no known row, so the column flags alone must not be decoded by Theorem 2."""
    n, k, m = 5, 4, 7
    A, B = int_mats(34, n, k, m)
    AP, BP = oc.encode_a(A), oc.encode_b(B)
    res = _run_faults(A, B, AP, BP, [(MAT_A, 2, 1, 3.0), (MAT_C, 0, 4, 2.0)])
    assert res.status == CORRECTED
    assert [(mt, i, j) for (mt, i, j, _) in res.errors] == [(MAT_A, 2, 1), (MAT_C, 0, 4)]
    assert res.t >= 3 and res.s == 1


def test_theorem2_runs_after_the_operand_audit():
    """With loose weighted thresholds a wrong symbol of A in row 5 is, seen from the columns,
    the same as errors of C in the flagged row 6 next to it: Theorem 2's decoder alone accepts
    that reading.  The operand parities (Section III: every column of A-bar is a codeword of
    its own) say otherwise, so the decoder has to ask them first."""
    n, k, m = 12, 4, 8
    A, B = int_mats(35, n, k, m)
    B[2, :] = [1, -1, 2, -2, 3, -3, 1, -1]            # row of B with plain and weighted sums near zero
    AP, BP = oc.encode_a(A), oc.encode_b(B)
    tau = Thresholds(0.5, 40.0, 0.5, 40.0, 0.0)
    A2 = A.copy()
    A2[5, 2] += 1.0
    Cbar = oc.encoded_product(A2, AP, B, BP)
    oc.inject_c(Cbar, [(6, 3, 7.0)])
    r1, r2, q1, q2 = oc.syndromes(Cbar)
    Er, Et = oc.detect(r1, r2, q1, q2, tau)
    assert Er == [6] and len(Et) == m
    alone = oc.known_lines_correct(r1, r2, q1, q2, Er, Et, oc.LineThresholds(tau, n, m))
    assert alone is not None and len(alone) == m and all(i == 6 for (i, _, _) in alone)
    res = oc.decode(Cbar, A2, AP, B, BP, tau)
    assert res.status == CORRECTED
    assert res.errors == [(MAT_A, 5, 2, 1.0), (MAT_C, 6, 3, 7.0)]
    assert np.array_equal(res.A, A) and np.array_equal(res.Cbar, oc.encoded_product(A, AP, B, BP))


# ---- pins of the decoder's own readings (thresholded arithmetic; the paper is silent) ----------
def test_equal_offsets_on_a_diagonal_are_ambiguous_below_the_weighted_threshold():
    """Two equal errors x on the diagonal of a 2 x 2 block and the same two on the anti-diagonal
    have identical plain sums; their weighted sums differ by exactly x per line (weights one
    apart, Section V).  Below the weighted threshold the decoder therefore cannot tell them
    apart and must not choose; above it both are corrected."""
    n, k, m = 8, 3, 8
    A, B = int_mats(36, n, k, m)
    AP, BP = oc.encode_a(A), oc.encode_b(B)
    clean = oc.encoded_product(A, AP, B, BP)
    tau = Thresholds(0.5, 5.0, 0.5, 5.0, 0.0)
    for cells in ([(2, 4), (3, 5)], [(2, 5), (3, 4)]):
        Cbar = clean.copy()
        oc.inject_c(Cbar, [(i, j, 2.0) for (i, j) in cells])
        assert oc.decode(Cbar, A, AP, B, BP, tau).status == UNCORRECTABLE
        Cbar = clean.copy()
        oc.inject_c(Cbar, [(i, j, 20.0) for (i, j) in cells])
        res = oc.decode(Cbar, A, AP, B, BP, tau)
        assert res.status == CORRECTED and [(i, j) for (_, i, j, _) in res.errors] == sorted(cells)
        assert np.array_equal(res.Cbar, clean)
    # rows two apart: the weighted sums differ by 2 x, so x = 4 is already enough
    Cbar = clean.copy()
    oc.inject_c(Cbar, [(2, 4, 4.0), (4, 5, 4.0)])
    assert oc.decode(Cbar, A, AP, B, BP, tau).status == CORRECTED


def test_verification_trusts_a_syndrome_relative_to_its_size_detection_does_not():
    """A syndrome that carries a relative error eps (as any finite-precision sum does) puts
    (j+1) x eps into the weighted check of an error x in column j.  With rel = 0 that fails
    the verification as soon as it exceeds the absolute threshold; with rel > eps it passes.
    Detection itself compares with the absolute threshold only."""
    n = m = 64
    i, j, x, eps = 10, 40, 1.0e6, 1.0e-7
    r1, r2, q1, q2 = np.zeros(n), np.zeros(n), np.zeros(m), np.zeros(m)
    r1[i], r2[i] = x, (j + 1) * x * (1 + eps)
    q1[j], q2[j] = x * (1 - eps), (i + 1) * x
    for rel, ok in ((0.0, False), (2.0 ** -20, True)):
        tau = Thresholds(1e-3, 1e-1, 1e-3, 1e-1, 0.0, 0.0, rel)
        fix = oc.d0_correct(r1, r2, q1, q2, [i], [j], oc.LineThresholds(tau, n, m))
        assert (fix is not None) == ok
        if ok:
            assert [(a, b) for (a, b, _) in fix] == [(i, j)] and abs(fix[0][2] - x) <= 2 * eps * x
    # a syndrome of 0.05 in a family whose threshold is 0.1 is not flagged whatever rel is
    r2b = np.zeros(n); r2b[3] = 0.05
    tau = Thresholds(1e-3, 1e-1, 1e-3, 1e-1, 0.0, 0.0, 0.5)
    assert oc.detect(np.zeros(n), r2b, q1 * 0, q2 * 0, tau) == ([], [])


def test_lines_touched_by_an_operand_repair_get_their_allowance_and_only_they():
    """After an operand repair, row i of C-bar still carries the rounding of the corrupted terms
    e b_lj that sat in its sums: noise proportional to |e b_lj|, symbol by symbol.  With
    rep sqrt(k) above that proportion the second pass of Section V ignores it and reports the
    operand error alone; with rep = 0 the same noise is taken for errors of C.  An error of C in an
    untouched line is judged by the plain thresholds either way."""
    n, k, m = 24, 16, 20
    rng = np.random.default_rng(37)
    A, B = rng.standard_normal((n, k)), rng.standard_normal((k, m))
    AP, BP = oc.encode_a(A), oc.encode_b(B)
    i, l, e, rho = 7, 5, 1000.0, 1e-6
    A2 = A.copy(); A2[i, l] += e
    Cbar = oc.encoded_product(A2, AP, B, BP)
    noise = rho * np.abs(e * B[l, :]) * rng.choice([-1.0, 1.0], m)
    Cbar[i, :m] += noise                                   # what a finite-precision product leaves behind
    base = dict(r1=1e-9, r2=1e-9, q1=1e-9, q2=1e-9, op=0.0)
    with_rep = oc.decode(Cbar, A2, AP, B, BP, Thresholds(**base, rep=4 * rho / np.sqrt(k)))
    assert with_rep.status == CORRECTED and [(mt, a, b) for (mt, a, b, _) in with_rep.errors] == [(MAT_A, i, l)]
    assert np.allclose(with_rep.A, A, rtol=0, atol=1e-9)
    without = oc.decode(Cbar, A2, AP, B, BP, Thresholds(**base, rep=0.0))
    assert without.status == UNCORRECTABLE or len(without.errors) > 1
    # the allowance belongs to the repaired row and, in proportion to |e b_lj|, to every column:
    # an error of C in another row that exceeds its column's allowance is still found ...
    Cbar2 = Cbar.copy()
    Cbar2[i + 3, 2] += 1.0
    res = oc.decode(Cbar2, A2, AP, B, BP, Thresholds(**base, rep=4 * rho / np.sqrt(k)))
    assert res.status == CORRECTED
    assert [(mt, a, b) for (mt, a, b, _) in res.errors] == [(MAT_A, i, l), (MAT_C, i + 3, 2)]
    # ... and one below it flags its own row (rows other than i are not widened) but no column:
    # nothing to pair it with, so nothing is corrected
    Cbar3 = Cbar.copy()
    Cbar3[i + 3, 2] += 1e-4
    assert 1e-4 < 4 * rho * abs(e * B[l, 2])
    assert oc.decode(Cbar3, A2, AP, B, BP, Thresholds(**base, rep=4 * rho / np.sqrt(k))).status == UNCORRECTABLE


# ---- pin: the incremental evaluation (oracle/incremental.py) is the full oracle -----------------
def _as_trial(A, B, placed):
    """placements with offsets -> the incremental oracle's arguments (stored values for A, B)"""
    af = [(r, c, A[r, c] + e) for (mt, r, c, e) in placed if mt == MAT_A]
    bf = [(r, c, B[r, c] + e) for (mt, r, c, e) in placed if mt == MAT_B]
    cf = [(r, c, e) for (mt, r, c, e) in placed if mt == MAT_C]
    return af, bf, cf


def _same_outcome(inc_res, full_res, clean_scale, tag):
    assert inc_res.status == full_res.status, tag
    assert (inc_res.s, inc_res.t) == (full_res.s, full_res.t), tag
    assert [e[:3] for e in inc_res.errors] == [e[:3] for e in full_res.errors], tag
    for x, y in zip(inc_res.errors, full_res.errors):
        assert abs(x[3] - y[3]) <= 1e-9 * max(1.0, abs(y[3])), tag
    assert np.allclose(inc_res.max_abs_synd, full_res.max_abs_synd, rtol=1e-9, atol=1e-9 * clean_scale), tag
    if full_res.status != UNCORRECTABLE:
        assert np.max(np.abs(inc_res.Cbar - full_res.Cbar)) <= 1e-9 * clean_scale, tag


@pytest.mark.parametrize("n,k,m,mags", [(3, 3, 3, (1.0, 1.0)), (4, 2, 3, (3.0, -5.0)), (3, 4, 5, (-1.0, 4.0))])
def test_incremental_oracle_equals_the_full_one_on_every_single_and_pair_placement(n, k, m, mags):
    """Linearity of the syndromes (Section V step 1) and of the product in each operand: a trial
    evaluated as changes of rows, columns and symbols of the clean C-bar has to end exactly where
    the from-scratch evaluation ends, for every placement of one and of two faults over A, B, C,
    the pairs beyond the code included."""
    from oracle.incremental import IncrementalOracle
    A, B = int_mats(41 + n + k + m, n, k, m)
    AP, BP = oc.encode_a(A), oc.encode_b(B)
    inc = IncrementalOracle(A, B, TAU0)
    scale = np.abs(inc.clean).max()
    cases = [[p + (mags[0],)] for p in _placements(n, k, m)] + \
            [[p1 + (mags[0],), p2 + (mags[1],)] for p1, p2 in itertools.combinations(_placements(n, k, m), 2)]
    for placed in cases:
        full = _run_faults(A, B, AP, BP, placed)
        got = inc.trial(*_as_trial(A, B, placed), keep_cbar=True)
        _same_outcome(got, full, scale, placed)
        if full.status == CORRECTED and not (len(placed) == 2 and _beyond_code(placed[0], placed[1])):
            assert got.left_in_cbar <= 1e-9 * scale and got.operands_restored
        # a trial leaves nothing behind
        assert np.array_equal(inc.W, inc.clean) and np.array_equal(inc.A, A) and np.array_equal(inc.B, B)
    assert inc.trial([], [], []).status == CLEAN


def test_incremental_oracle_equals_the_full_one_on_real_operands_with_rounding_noise():
    """Real-valued operands, thresholds above the rounding level, second-pass allowances in use,
    0 to 3 faults of any kind, a same-index A+B pair (cross term) and a pattern of Theorem 2."""
    from oracle.incremental import IncrementalOracle
    n, k, m = 40, 24, 36
    rng = np.random.default_rng(2024)
    A, B = rng.standard_normal((n, k)), rng.standard_normal((k, m)) * 0.02
    tau = Thresholds(1e-7, 1e-5, 1e-7, 1e-5, 0.0, rep=1e-9, rel=1e-9)
    inc = IncrementalOracle(A, B, tau)
    scale = np.abs(inc.clean[:n, :m]).max()
    P = _placements(n, k, m)
    cases = []
    for t in range(300):
        cnt = int(rng.integers(0, 4))
        idx = rng.choice(len(P), cnt, replace=False)
        cases.append([P[x] + (float(np.exp(rng.uniform(np.log(1e-3), np.log(1e3))) * rng.choice([-1, 1])),) for x in idx])
    cases.append([(MAT_A, 3, 7, 2.5), (MAT_B, 7, 30, -40.0)])                      # same l: cross term
    cases.append([(MAT_C, 5, j, 1.0 + j) for j in range(0, m, 3)])                 # Theorem 2, one row
    cases.append([(MAT_A, 9, 2, 3.0)] + [(MAT_C, 9, j, 0.5) for j in (1, 4, 8)])   # audit, then the rest in its row
    seen = set()
    for placed in cases:
        A2, B2, cf = A.copy(), B.copy(), []
        for (mt, r, c, e) in placed:
            if mt == MAT_A: A2[r, c] += e
            elif mt == MAT_B: B2[r, c] += e
            else: cf.append((r, c, e))
        full = oc.protected_gemm(A, B, A2, B2, cf, tau)
        af = [(r, c, A2[r, c]) for (mt, r, c, e) in placed if mt == MAT_A]
        bf = [(r, c, B2[r, c]) for (mt, r, c, e) in placed if mt == MAT_B]
        got = inc.trial(af, bf, cf, keep_cbar=True)
        _same_outcome(got, full, scale, placed)
        seen.add(full.status)
    assert seen == {CLEAN, CORRECTED, UNCORRECTABLE}


# ---- pin: the scheme is symmetric under transposition (C^T = B^T A^T swaps the roles of A and B, of
#      rows and columns, of r and q): every B-side branch of the decoder has to mirror its A-side twin
def _mirror(res):
    out = []
    for (mt, r, c, x) in res.errors:
        out.append((MAT_B, c, r, x) if mt == MAT_A else (MAT_A, c, r, x) if mt == MAT_B else (MAT_C, c, r, x))
    return sorted(out)


def test_decoder_is_symmetric_under_transposition():
    n, k, m = 14, 9, 11
    rng = np.random.default_rng(5)
    A, B = rng.standard_normal((n, k)), rng.standard_normal((k, m))
    AP, BP = oc.encode_a(A), oc.encode_b(B)
    tau = Thresholds(r1=1e-8, r2=2e-8, q1=3e-8, q2=4e-8, op=0.0, rep=1e-7, rel=1e-9)
    tau_t = Thresholds(r1=tau.q1, r2=tau.q2, q1=tau.r1, q2=tau.r2, op=0.0, rep=tau.rep, rel=tau.rel)
    P = _placements(n, k, m)
    statuses = set()
    for t in range(400):
        cnt = int(rng.integers(1, 4))
        placed = [P[x] + (float(rng.uniform(1, 50) * rng.choice([-1, 1])),) for x in rng.choice(len(P), cnt, replace=False)]
        A2, B2, cf = A.copy(), B.copy(), []
        for (mt, r, c, e) in placed:
            if mt == MAT_A: A2[r, c] += e
            elif mt == MAT_B: B2[r, c] += e
            else: cf.append((r, c, e))
        Cbar = oc.encoded_product(A2, AP, B2, BP)
        oc.inject_c(Cbar, cf)
        # rounding left behind by a finite-precision product: proportional to the corrupted terms
        for (mt, r, c, e) in placed:
            if mt == MAT_A: Cbar[r, :m] += 1e-8 * np.abs(e * B[c, :]) * rng.choice([-1.0, 1.0], m)
            if mt == MAT_B: Cbar[:n, c] += 1e-8 * np.abs(A[:, r] * e) * rng.choice([-1.0, 1.0], n)
        res = oc.decode(Cbar, A2, AP, B2, BP, tau)
        res_t = oc.decode(Cbar.T, B2.T, BP.T, A2.T, AP.T, tau_t)
        assert res.status == res_t.status, placed
        assert (res.s, res.t) == (res_t.t, res_t.s)
        statuses.add(res.status)
        if res.status == UNCORRECTABLE:
            continue
        mirrored = _mirror(res_t)
        assert [e[:3] for e in mirrored] == [e[:3] for e in res.errors], placed
        # (values agree to the planted noise, not better: with s = t the rule reads the columns, and
        # the columns of the transposed problem are the rows of this one, whose sums hold other noise)
        assert np.allclose([e[3] for e in mirrored], [e[3] for e in res.errors], rtol=1e-6, atol=2e-5)
        assert np.allclose(res.Cbar, res_t.Cbar.T, rtol=0, atol=2e-5)
        assert np.allclose(res.A, res_t.B.T, atol=1e-9) and np.allclose(res.B, res_t.A.T, atol=1e-9)
    assert statuses == {CORRECTED, UNCORRECTABLE}


def test_lines_touched_by_a_repair_of_B_get_their_allowance_and_only_they():
    """Mirror image of the pin for A: after a wrong symbol b_lj is repaired, column j of C-bar keeps
    the rounding of the corrupted terms a_il e; the allowance belongs to that column and, symbol by
    symbol in proportion to |a_il e|, to every row -- and to nothing else."""
    n, k, m = 20, 16, 24
    rng = np.random.default_rng(38)
    A, B = rng.standard_normal((n, k)), rng.standard_normal((k, m))
    AP, BP = oc.encode_a(A), oc.encode_b(B)
    l, j, e, rho = 5, 7, 1000.0, 1e-6
    B2 = B.copy(); B2[l, j] += e
    Cbar = oc.encoded_product(A, AP, B2, BP)
    Cbar[:n, j] += rho * np.abs(A[:, l] * e) * rng.choice([-1.0, 1.0], n)
    base = dict(r1=1e-9, r2=1e-9, q1=1e-9, q2=1e-9, op=0.0)
    with_rep = oc.decode(Cbar, A, AP, B2, BP, Thresholds(**base, rep=4 * rho / np.sqrt(k)))
    assert with_rep.status == CORRECTED and [x[:3] for x in with_rep.errors] == [(MAT_B, l, j)]
    assert np.allclose(with_rep.B, B, rtol=0, atol=1e-9)
    without = oc.decode(Cbar, A, AP, B2, BP, Thresholds(**base, rep=0.0))
    assert without.status == UNCORRECTABLE or len(without.errors) > 1
    # an error of C in another column, above its row's allowance: found beside the operand error
    Cbar2 = Cbar.copy(); Cbar2[2, j + 3] += 1.0
    res = oc.decode(Cbar2, A, AP, B2, BP, Thresholds(**base, rep=4 * rho / np.sqrt(k)))
    assert res.status == CORRECTED and [x[:3] for x in res.errors] == [(MAT_B, l, j), (MAT_C, 2, j + 3)]
    # below it: its own column (not widened) is flagged, no row is: nothing to pair it with
    Cbar3 = Cbar.copy(); Cbar3[2, j + 3] += 1e-4
    assert 1e-4 < 4 * rho * abs(A[2, l] * e)
    assert oc.decode(Cbar3, A, AP, B2, BP, Thresholds(**base, rep=4 * rho / np.sqrt(k))).status == UNCORRECTABLE
    # the allowance of column j itself is the root-sum-square over the column, plain and weighted: a
    # residual in that column just inside it passes, the same residual with half the allowance does not
    foot = A[:, l] * e
    inside = 0.9 * 4 * rho * np.sqrt(np.sum(foot ** 2))
    Cbar4 = oc.encoded_product(A, AP, B2, BP)
    Cbar4[n, j] -= inside                                   # moves q1_j only (a parity symbol of that column)
    ok = oc.decode(Cbar4, A, AP, B2, BP, Thresholds(**base, rep=4 * rho / np.sqrt(k)))
    assert ok.status == CORRECTED and [x[:3] for x in ok.errors] == [(MAT_B, l, j)]
    assert oc.decode(Cbar4, A, AP, B2, BP, Thresholds(**base, rep=2 * rho / np.sqrt(k))).status == UNCORRECTABLE


def test_an_audit_accepts_eight_operand_errors_and_gives_up_at_nine():
    """MAX_REPORTED: eight wrong operand symbols in eight different lines are all repaired; a ninth makes
    the pattern UNCORRECTABLE (the library's report has eight slots)."""
    n, k, m = 12, 12, 12
    A, B = int_mats(99, n, k, m)
    AP, BP = oc.encode_a(A), oc.encode_b(B)
    spots = [(MAT_A, i, i, 3.0 + i) for i in range(5)] + [(MAT_B, l, (l + 2) % m, -2.0 - l) for l in range(5, 9)]
    res = _run_faults(A, B, AP, BP, spots[:8])
    assert res.status == CORRECTED and res.errors == sorted(spots[:8])
    assert np.array_equal(res.A, A) and np.array_equal(res.B, B)
    assert _run_faults(A, B, AP, BP, spots[:9]).status == UNCORRECTABLE
    assert oc.MAX_REPORTED == 8


def test_audit_ratio_tolerance_is_a_quarter_from_both_sides():
    """A line whose weighted/plain ratio misses every integer by 1/4 or more holds more than one wrong
    symbol; within 1/4 it is read as one.  Two errors in one column of A at rows 3 and 4 (1-based)
    with offsets (1-f, f) give the ratio 3 + f exactly."""
    n, k, m = 6, 3, 4
    A, B = int_mats(5, n, k, m)
    AP = oc.encode_a(A)
    for f, want in ((0.2421875, (True, 2)), (0.2578125, (False, None)), (0.7421875, (False, None)), (0.7578125, (True, 3))):
        A2 = A.copy(); A2[2, 1] += 1.0 - f; A2[3, 1] += f       # dyadic fractions: every sum is exact
        ok, found = oc.audit_a(A2, AP, 0.0)
        assert ok == want[0], f
        if ok:
            assert found == [(want[1], 1, 1.0)]
    BP = oc.encode_b(B)
    for f, want in ((0.2421875, (True, 1)), (0.2578125, (False, None)), (0.7578125, (True, 2))):
        B2 = B.copy(); B2[0, 1] += 1.0 - f; B2[0, 2] += f
        ok, found = oc.audit_b(B2, BP, 0.0)
        assert ok == want[0], f
        if ok:
            assert found == [(0, want[1], 1.0)]
    # a ratio that rounds to a row outside 1..n is refused as well
    A2 = A.copy(); A2[0, 0] += 2.0; A2[1, 0] -= 1.0             # ratio (2*1 - 1*2) / 1 = 0
    assert oc.audit_a(A2, AP, 0.0)[0] is False


def test_a_syndrome_equal_to_its_threshold_is_not_flagged():
    """Section V step 1 clears a line whose |sum - parity| is <= delta: equality is inside."""
    z = np.zeros(3)
    tau = Thresholds(0.5, 2.0, 0.25, 4.0)
    r1 = np.array([0.5, -0.5, np.nextafter(0.5, 1.0)])
    assert oc.detect(r1, z, z, z, tau) == ([2], [])
    assert oc.detect(z, np.array([2.0, -np.nextafter(2.0, 3.0), 0.0]), z, z, tau) == ([1], [])
    assert oc.detect(z, z, np.array([0.25, 0.25, -0.25]), np.array([4.0, -4.0, np.nextafter(4.0, 5.0)]), tau) == ([], [2])


def test_a_symbol_that_is_not_a_number_is_detected_and_handed_back():
    """A NaN (or infinite) symbol of C makes its row and column syndromes NaN; `not <= delta` flags
    them, and since no subtraction restores such a symbol the product has to be computed again.  The
    same for an operand symbol (a whole row of C turns NaN)."""
    n, k, m = 6, 4, 5
    A, B = int_mats(3, n, k, m)
    AP, BP = oc.encode_a(A), oc.encode_b(B)
    for bad in (np.nan, np.inf, -np.inf):
        Cbar = oc.encoded_product(A, AP, B, BP)
        Cbar[2, 3] = bad
        r1, r2, q1, q2 = oc.syndromes(Cbar)
        assert oc.detect(r1, r2, q1, q2, TAU0) == ([2], [3])
        res = oc.decode(Cbar, A, AP, B, BP, TAU0)
        assert res.status == UNCORRECTABLE and (res.s, res.t) == (1, 1)
        A2 = A.copy(); A2[1, 2] = bad
        res = oc.protected_gemm(A, B, A2, B, [], TAU0)
        assert res.status == UNCORRECTABLE and res.t == m
    # a NaN that appears only in the second pass (left by a repair) is not waved through either
    A2 = A.copy(); A2[1, 2] += 3.0
    Cbar = oc.encoded_product(A2, AP, B, BP)
    B2 = B.copy(); B2[2, 0] = np.nan        # the repair of row 1 multiplies e by this symbol
    assert oc.decode(Cbar, A2, AP, B2, BP, TAU0).status == UNCORRECTABLE


# ---- single-checksum mode: the conventional checksum scheme Section VI compares with ------------
TAU0_SINGLE = Thresholds(1e-9, 1e-9, 1e-9, 1e-9, 0.0, weighted=False)


def test_single_checksum_corrects_exactly_the_patterns_confined_to_one_line_of_C():
    """With one parity per line, errors of C are decodable iff they all lie in one row or in one
    column (Appendix A: s = t = 1 is the conventional checksum, one faulty row is read column by
    column from the plain column parities).  Every pattern of one to three symbols on a 4 x 4 grid,
    magnitudes 1, 10, 100 (no partial sum cancels)."""
    n, k, m = 4, 3, 4
    A, B = int_mats(7, n, k, m)
    clean = oc.encoded_product(A, oc.encode_a(A), B, oc.encode_b(B))
    cells = [(i, j) for i in range(n) for j in range(m)]
    n_ok = n_not = 0
    for cnt in (1, 2, 3):
        for pos in itertools.combinations(cells, cnt):
            cf = [(i, j, 10.0 ** x) for x, (i, j) in enumerate(pos)]
            one_line = len({i for i, j in pos}) == 1 or len({j for i, j in pos}) == 1
            res = oc.protected_gemm(A, B, A, B, cf, TAU0_SINGLE)
            if one_line:
                n_ok += 1
                assert res.status == CORRECTED and res.errors == sorted((MAT_C, i, j, e) for (i, j, e) in cf), pos
                assert np.array_equal(res.Cbar, clean)
            else:
                n_not += 1
                assert res.status == UNCORRECTABLE, pos
            # the grid code corrects all of these as long as they fit two rows and two columns ...
            if len({i for i, j in pos}) <= 2 and len({j for i, j in pos}) <= 2:
                assert oc.protected_gemm(A, B, A, B, cf, TAU0).status == CORRECTED
    assert n_ok == 16 + 2 * 4 * 6 + 2 * 4 * 4 and n_not > 0


def test_single_checksum_cannot_tell_the_two_diagonals_apart():
    """Textbook fact behind the bound: equal errors on the diagonal and on the anti-diagonal of a
    2 x 2 sub-grid have the same row sums and the same column sums."""
    n, k, m = 5, 3, 6
    A, B = int_mats(8, n, k, m)
    AP, BP = oc.encode_a(A), oc.encode_b(B)
    Cd, Ca = oc.encoded_product(A, AP, B, BP), oc.encoded_product(A, AP, B, BP)
    oc.inject_c(Cd, [(1, 2, 3.0), (3, 4, 3.0)])
    oc.inject_c(Ca, [(1, 4, 3.0), (3, 2, 3.0)])
    sd, sa = oc.syndromes(Cd), oc.syndromes(Ca)
    assert np.array_equal(sd[0], sa[0]) and np.array_equal(sd[2], sa[2])       # plain sums coincide
    assert not np.array_equal(sd[1], sa[1])                                     # the weighted ones do not
    for Cx in (Cd, Ca):
        assert oc.decode_single_checksum(Cx, A, AP, B, BP, TAU0_SINGLE).status == UNCORRECTABLE
        assert oc.decode(Cx, A, AP, B, BP, TAU0).status == CORRECTED


@pytest.mark.parametrize("n,k,m", [(3, 3, 3), (4, 2, 3)])
def test_single_checksum_on_every_single_and_pair_placement(n, k, m):
    """Scenarios of Section VI in single-checksum mode, exhaustively on tiny sizes: one error of C is
    corrected; a wrong operand symbol is detected but cannot be placed (its line carries one parity,
    and the row of C it spoils takes its own parity symbols along); pairs are corrected only when
    both lie in one row or one column of C.  Nothing is ever mis-corrected, nothing goes unseen."""
    A, B = int_mats(41 + n + k + m, n, k, m)
    AP, BP = oc.encode_a(A), oc.encode_b(B)
    clean = oc.encoded_product(A, AP, B, BP)

    def run(placed):
        A2, B2, cf = A.copy(), B.copy(), []
        for (mt, r, c, e) in placed:
            if mt == MAT_A: A2[r, c] += e
            elif mt == MAT_B: B2[r, c] += e
            else: cf.append((r, c, e))
        return oc.protected_gemm(A, B, A2, B2, cf, TAU0_SINGLE)

    P = _placements(n, k, m)
    for p in P:
        res = run([p + (2.0,)])
        if p[0] == MAT_C:
            assert res.status == CORRECTED and res.errors == [p + (2.0,)] and np.array_equal(res.Cbar, clean)
        else:
            assert res.status == UNCORRECTABLE
    seen = set()
    for p1, p2 in itertools.combinations(P, 2):
        res = run([p1 + (3.0,), p2 + (-5.0,)])
        both_c = p1[0] == p2[0] == MAT_C
        if both_c and (p1[1] == p2[1] or p1[2] == p2[2]):
            assert res.status == CORRECTED and res.errors == sorted([p1 + (3.0,), p2 + (-5.0,)])
            assert np.array_equal(res.Cbar, clean)
        else:
            assert res.status == UNCORRECTABLE, (p1, p2)
        seen.add(res.status)
    assert seen == {CORRECTED, UNCORRECTABLE}


def test_single_checksum_verifies_its_estimates_and_ignores_the_weighted_sums():
    n, k, m = 6, 4, 7
    A, B = int_mats(9, n, k, m)
    AP, BP = oc.encode_a(A), oc.encode_b(B)
    Cbar = oc.encoded_product(A, AP, B, BP)
    # a wrong weighted parity symbol alone is invisible in this mode and flags a row of the grid code
    C1 = Cbar.copy(); C1[2, m + 1] += 5.0
    assert oc.decode_single_checksum(C1, A, AP, B, BP, TAU0_SINGLE).status == CLEAN
    assert oc.decode(C1, A, AP, B, BP, TAU0).s == 1
    # one flagged row whose own sum does not add up to what the columns say: refused
    C2 = Cbar.copy(); C2[1, 2] += 4.0; C2[1, 5] -= 1.0; C2[1, m] += 0.5       # row parity symbol off as well
    assert oc.decode_single_checksum(C2, A, AP, B, BP, TAU0_SINGLE).status == UNCORRECTABLE
    # NaN: flagged and handed back
    C3 = Cbar.copy(); C3[0, 0] = np.nan
    res = oc.decode_single_checksum(C3, A, AP, B, BP, TAU0_SINGLE)
    assert res.status == UNCORRECTABLE and (res.s, res.t) == (1, 1)


# ---- per-k-panel verification: the code is linear, every partial product is a codeword -------------
def test_partial_products_over_k_panels_are_codewords_and_add_up():
    """Section III: C-bar = A-bar B-bar is linear in both operands, so with k cut into panels the
    encoded partial products add up to C-bar block by block (exactly, on integers), and each of
    them satisfies all of Definition 1's constraints on its own."""
    n, k, m = 5, 12, 6
    A, B = int_mats(123, n, k, m, -4, 4)
    AP, BP = oc.encode_a(A), oc.encode_b(B)
    full = oc.encoded_product(A, AP, B, BP)
    bounds = oc.panel_bounds(k, 3, align=2)
    assert bounds == [(0, 4), (4, 8), (8, 12)] and oc.panel_bounds(10, 4, align=4) == [(0, 4), (4, 8), (8, 10)]
    total = np.zeros_like(full)
    for (k0, k1) in bounds:
        part = oc.encoded_product(A[:, k0:k1], oc.encode_a(A[:, k0:k1]), B[k0:k1, :], oc.encode_b(B[k0:k1, :]))
        assert np.array_equal(oc.encode_a(A[:, k0:k1]), AP[:, k0:k1]) and np.array_equal(oc.encode_b(B[k0:k1, :]), BP[k0:k1, :])
        assert all(np.all(v == 0) for v in oc.syndromes(part)) and np.all(oc.global_syndromes(part) == 0)
        total += part
    assert np.array_equal(total, full)


def test_a_fault_is_caught_in_the_panel_it_strikes():
    n, k, m = 6, 12, 5
    A, B = int_mats(321, n, k, m)
    bounds = oc.panel_bounds(k, 3, align=2)
    clean = A @ B
    # one fault of C in panel 1's partial product, one wrong symbol of A in panel 2 (column 9 = 1 of its slice)
    A2 = A.copy(); A2[4, 9] += 3.0
    res, C = oc.protected_gemm_panels(A, B, A2, B, {1: [(2, 3, -7.0)]}, TAU0, bounds)
    assert [r.status for r in res] == [CLEAN, CORRECTED, CORRECTED]
    assert res[1].errors == [(MAT_C, 2, 3, -7.0)] and res[2].errors == [(MAT_A, 4, 1, 3.0)]
    assert np.array_equal(C, clean)
    # two faults in two different panels are two single faults: each panel corrects its own, also
    # where the whole product would see a pattern beyond the code (three faults on a diagonal)
    res, C = oc.protected_gemm_panels(A, B, A, B, {0: [(0, 0, 1.0)], 1: [(1, 1, 2.0)], 2: [(2, 2, 4.0)]}, TAU0, bounds)
    assert [r.status for r in res] == [CORRECTED] * 3 and np.array_equal(C, clean)
    assert oc.protected_gemm(A, B, A, B, [(0, 0, 1.0), (1, 1, 2.0), (2, 2, 4.0)], TAU0).status == UNCORRECTABLE
    # thresholds shrink with the panel: a third of the terms, a third of the rounding noise
    t = oc.panel_thresholds(Thresholds(3.0, 6.0, 9.0, 12.0, 0.5, 0.25, 0.125), 4, 12)
    assert (t.r1, t.r2, t.q1, t.q2, t.op, t.rep, t.rel) == (1.0, 2.0, 3.0, 4.0, 0.5, 0.25, 0.125)


# ---- blocked grid code: Section III per nb x mb block of C ------------------------------------------
def test_block_parities_add_up_to_the_parities_of_the_whole_product():
    """Plain block parities of a line add up to the line's plain parity of the whole product, weighted
    ones after shifting the block-local weights (1..mb) to the global ones: sum_J (w_J + J mb s_J)."""
    n, k, m, nb, mb = 6, 5, 8, 3, 4
    A, B = int_mats(55, n, k, m, -5, 5)
    whole = oc.encoded_product(A, oc.encode_a(A), B, oc.encode_b(B))
    pr1, pr2, pc1, pc2 = np.zeros(n), np.zeros(n), np.zeros(m), np.zeros(m)
    for I in range(n // nb):
        for J in range(m // mb):
            AI, BJ = A[I * nb:(I + 1) * nb], B[:, J * mb:(J + 1) * mb]
            blk = oc.encoded_product(AI, oc.encode_a(AI), BJ, oc.encode_b(BJ))
            assert np.array_equal(blk[:nb, :mb], whole[I * nb:(I + 1) * nb, J * mb:(J + 1) * mb])
            assert all(np.all(v == 0) for v in oc.syndromes(blk)) and np.all(oc.global_syndromes(blk) == 0)
            pr1[I * nb:(I + 1) * nb] += blk[:nb, mb]
            pr2[I * nb:(I + 1) * nb] += blk[:nb, mb + 1] + J * mb * blk[:nb, mb]
            pc1[J * mb:(J + 1) * mb] += blk[nb, :mb]
            pc2[J * mb:(J + 1) * mb] += blk[nb + 1, :mb] + I * nb * blk[nb, :mb]
    assert np.array_equal(pr1, whole[:n, m]) and np.array_equal(pr2, whole[:n, m + 1])
    assert np.array_equal(pc1, whole[n, :m]) and np.array_equal(pc2, whole[n + 1, :m])


def test_blocked_code_corrects_two_errors_in_every_block():
    """Theorem 1 block by block: two errors in each of the six blocks (twelve in all, far beyond the
    whole-matrix code) are all located and removed; three errors in general position inside one block
    exceed that block alone."""
    n, k, m, nb, mb = 8, 4, 9, 4, 3
    A, B = int_mats(56, n, k, m)
    clean = A @ B
    cf = []
    for I in range(2):
        for J in range(3):
            cf += [(I * nb + 0, J * mb + 1, 3.0 + I + J), (I * nb + 2, J * mb + 2, -5.0 - J)]
    res, C, A2, B2 = oc.protected_gemm_blocked(A, B, A, B, cf, TAU0, nb, mb)
    assert all(r.status == CORRECTED and len(r.errors) == 2 for r in res.values())
    assert res[(1, 2)].errors == [(MAT_C, 0, 1, 6.0), (MAT_C, 2, 2, -7.0)]        # block-local positions
    assert np.array_equal(C, clean)
    assert oc.protected_gemm(A, B, A, B, cf, TAU0).status == UNCORRECTABLE
    cf3 = [(0, 0, 1.0), (1, 1, 2.0), (2, 2, 4.0), (5, 7, 9.0)]
    res, C, _, _ = oc.protected_gemm_blocked(A, B, A, B, cf3, TAU0, nb, mb)
    assert res[(0, 0)].status == UNCORRECTABLE and res[(1, 2)].status == CORRECTED
    assert sum(r.status == CLEAN for r in res.values()) == 4
    assert np.array_equal(C[nb:], clean[nb:])


def test_blocked_code_traces_an_operand_error_through_every_block_of_its_line():
    """A wrong symbol of A spoils row i of C in every column block; each of those blocks finds it in
    the parity rows of its own row block of A (weights 1..nb: the position comes out block-local),
    repairs its part of the row, and the operand is restored.  The other row blocks stay clean."""
    n, k, m, nb, mb = 8, 4, 9, 4, 3
    A, B = int_mats(57, n, k, m)
    A2 = A.copy(); A2[6, 1] += 5.0
    B2 = B.copy(); B2[3, 4] -= 2.0
    res, C, Ap, Bp = oc.protected_gemm_blocked(A, B, A2, B2, [(1, 8, 7.0)], TAU0, nb, mb)
    assert np.array_equal(C, A @ B) and np.array_equal(Ap, A) and np.array_equal(Bp, B)
    assert [res[(1, J)].errors for J in (0, 2)] == [[(MAT_A, 2, 1, 5.0)]] * 2
    assert res[(1, 1)].errors == [(MAT_A, 2, 1, 5.0), (MAT_B, 3, 1, -2.0)]
    assert res[(0, 1)].errors == [(MAT_B, 3, 1, -2.0)]
    assert res[(0, 2)].errors == [(MAT_C, 1, 2, 7.0)] and res[(0, 0)].status == CLEAN
