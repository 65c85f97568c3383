"""Workload recipes: shapes, input laws, fault laws and the detection thresholds as numbers.

Nothing here is arithmetic of the coding scheme.  The shapes and laws are the benchmark
configurations this repository is measured on (synthetic stand-ins for training GEMMs; the
paper itself quotes one shape, n = m = 1024, k = 4096, in Table 1, with data law, precision
and threshold scale unstated).

Thresholds: the paper uses one delta for the four syndrome families (Section V); here each
family has its own number because the weighted sums carry weights up to n or m.  The numbers
are 16 x the rounding-noise model of gecc.noise_thresholds (tests assert that, and the GPU
tests assert that clean products stay below a quarter of them).
"""
from dataclasses import dataclass
from typing import Tuple

from .gecc import Thresholds


@dataclass(frozen=True)
class Workload:
    name: str
    n: int
    k: int
    m: int
    batch: int
    dtype: str                 # "f32" or "bf16" (inputs); accumulation and C are fp32
    trans_a: int
    trans_b: int
    law_a: Tuple
    law_b: Tuple
    sigma_a: float
    sigma_b: float
    offset_law: Tuple          # additive fault offsets
    tau: Thresholds
    tol_c: float               # max |C - C_oracle| / max |C_oracle| demanded of the corrected C

    @property
    def flops(self):           # useful flops of the data block
        return 2.0 * self.n * self.m * self.k * self.batch


_U = 3.0 ** -0.5   # standard deviation of U(-1, 1)

CFG1 = Workload("cfg1", 128, 128, 128, 1, "f32", 0, 0, ("normal", 1.0), ("normal", 1.0), 1.0, 1.0,
                ("uniform", 1.0, 100.0), Thresholds(5.64e-4, 4.17e-2, 5.64e-4, 4.17e-2), 1e-5)
CFG2 = Workload("cfg2", 1024, 1024, 1024, 1, "f32", 0, 0, ("uniform", -1.0, 1.0), ("uniform", -1.0, 1.0),
                _U, _U, ("uniform", 1.0, 100.0), Thresholds(4.25e-3, 2.51, 4.25e-3, 2.51), 1e-5)
CFG3 = Workload("cfg3", 4096, 4096, 4096, 1, "bf16", 0, 0, ("normal", 0.02), ("normal", 0.02), 0.02, 0.02,
                ("loguniform", 1e-2, 1e3), Thresholds(4.08e-5, 9.65e-2, 4.08e-5, 9.65e-2), 2e-2)
# transformer layer GEMMs: forward X W, dgrad dY W^T (W stored k-major -> trans_b), wgrad X^T dY
CFG4_FWD = Workload("cfg4-fwd", 16384, 4096, 14336, 1, "bf16", 0, 0, ("normal", 1.0), ("normal", 0.02),
                    1.0, 0.02, ("uniform", 1.0, 100.0), Thresholds(3.82e-3, 31.6, 4.08e-3, 38.6), 2e-2)
CFG4_DGRAD = Workload("cfg4-dgrad", 16384, 14336, 4096, 1, "bf16", 0, 1, ("normal", 1.0), ("normal", 0.02),
                      1.0, 0.02, ("uniform", 1.0, 100.0), Thresholds(7.14e-3, 16.9, 1.43e-2, 135.0), 2e-2)
CFG4_WGRAD = Workload("cfg4-wgrad", 4096, 16384, 14336, 1, "bf16", 1, 0, ("normal", 1.0), ("normal", 1.0),
                      1.0, 1.0, ("uniform", 1.0, 100.0), Thresholds(0.764, 6.32e3, 0.408, 965.0), 2e-2)
CFG5 = Workload("cfg5", 512, 512, 512, 256, "f32", 0, 0, ("uniform", -1.0, 1.0), ("uniform", -1.0, 1.0),
                _U, _U, ("uniform", 1.0, 100.0), Thresholds(1.50e-3, 0.444, 1.50e-3, 0.444), 1e-5)

ALL = {w.name: w for w in (CFG1, CFG2, CFG3, CFG4_FWD, CFG4_DGRAD, CFG4_WGRAD, CFG5)}
