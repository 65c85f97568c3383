"""Seeded synthetic inputs and fault placements.

This module holds no arithmetic of the coding scheme: it only draws operand
matrices, rounds them to the storage type, and draws where and by how much a
symbol is overwritten.  Both the CPU oracle's tests and the GPU path's tests
feed on it so that the two see identical inputs.

Workload recipes (shapes, laws, fault magnitudes) follow the benchmark
configurations this repository is measured on; the paper itself states only
one shape (n = m = 1024, k = 4096, Table 1) and six fault scenarios
(Section VI: a = A, b = B, c = C, d = A+C, e = B+C, f = C+C).
"""
from dataclasses import dataclass
from typing import List, Tuple

import numpy as np

SEED_BASE = 0x25080435
MAT_A, MAT_B, MAT_C = 0, 1, 2


def rng_for(cfg: int, trial: int = 0) -> np.random.Generator:
    return np.random.default_rng(SEED_BASE + 1000 * cfg + trial)


# ------------------------------------------------------------ storage rounding
def round_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bfloat16 (ties to even); returns float32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    b = x.view(np.uint32)
    rounded = ((b + (0x7FFF + ((b >> 16) & 1))) & 0xFFFF0000).astype(np.uint32)
    return rounded.view(np.float32)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of values that already are bfloat16-representable."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    return (x.view(np.uint32) >> 16).astype(np.uint16)


def store(x, dtype: str) -> np.ndarray:
    """Round to the storage type ('f32' or 'bf16'); result is float32 holding exact values."""
    x = np.asarray(x, dtype=np.float64).astype(np.float32)
    return round_bf16(x) if dtype == "bf16" else x


# ------------------------------------------------------------------- operands
def operands(rng, n, k, m, law_a, law_b, dtype):
    """law = ('normal', sigma) or ('uniform', lo, hi) or ('int', lo, hi)."""
    def draw(shape, law):
        if law[0] == "normal":
            return rng.standard_normal(shape) * law[1]
        if law[0] == "uniform":
            return rng.uniform(law[1], law[2], shape)
        if law[0] == "int":
            return rng.integers(law[1], law[2] + 1, shape).astype(np.float64)
        raise ValueError(law)
    return store(draw((n, k), law_a), dtype), store(draw((k, m), law_b), dtype)


# --------------------------------------------------------------------- faults
@dataclass
class Fault:
    matrix: int      # MAT_A / MAT_B / MAT_C
    row: int         # 0-based, in the logical (untransposed) matrix
    col: int
    offset: float    # additive offset e


def draw_offset(rng, law):
    """law = ('uniform', lo, hi) magnitude with random sign, or ('loguniform', lo, hi)."""
    if law[0] == "uniform":
        mag = rng.uniform(law[1], law[2])
    elif law[0] == "loguniform":
        mag = float(np.exp(rng.uniform(np.log(law[1]), np.log(law[2]))))
    else:
        raise ValueError(law)
    return float(mag if rng.integers(0, 2) else -mag)


def draw_faults(rng, n, k, m, count, offset_law, matrices=None) -> List[Fault]:
    """`count` distinct data symbols, uniform over A (n*k), B (k*m), C (n*m).

    matrices: optional list fixing the matrix of each fault (e.g. [MAT_A, MAT_C]).
    """
    sizes = (n * k, k * m, n * m)
    cols = (k, m, m)
    seen, out = set(), []
    while len(out) < count:
        if matrices is None:
            f = int(rng.integers(0, sum(sizes)))
            mat = 0 if f < sizes[0] else (1 if f < sizes[0] + sizes[1] else 2)
            f -= (0, sizes[0], sizes[0] + sizes[1])[mat]
        else:
            mat = matrices[len(out)]
            f = int(rng.integers(0, sizes[mat]))
        if (mat, f) in seen:
            continue
        seen.add((mat, f))
        out.append(Fault(mat, f // cols[mat], f % cols[mat], draw_offset(rng, offset_law)))
    return out


def apply_operand_faults(A, B, faults, dtype):
    """Overwrite the hit symbols of A/B: stored value = round_to_storage(old + e).

    Returns (A', B', c_faults, effective) where c_faults = [(i, j, e)] are the
    product faults to be applied by whoever computes the product, and
    `effective` lists the faults that actually changed a stored value, with
    the offset that the storage rounding left ((matrix,row,col,e_effective)).
    """
    A2, B2 = A.copy(), B.copy()
    c_faults, eff = [], []
    for f in faults:
        if f.matrix == MAT_C:
            c_faults.append((f.row, f.col, f.offset))
            eff.append((MAT_C, f.row, f.col, f.offset))
            continue
        M = A2 if f.matrix == MAT_A else B2
        old = float(M[f.row, f.col])
        new = float(store(np.array([old + f.offset]), dtype)[0])
        M[f.row, f.col] = new
        if new != old:
            eff.append((f.matrix, f.row, f.col, new - old))
    return A2, B2, c_faults, sorted(eff)
