"""The seeded input generators: reproducible, correctly rounded, faults placed as documented."""
import numpy as np
import torch

from paper_2508_04355_amd import inputs


def test_bf16_rounding_matches_round_to_nearest_even():
    x = np.random.default_rng(0).standard_normal(200000).astype(np.float32) * 3
    x[:4] = [1.0 + 2 ** -8, 1.0 + 3 * 2 ** -8, -0.0, 65280.0]          # two exact ties, zero, large
    r = inputs.round_bf16(x)
    t = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(r, t)
    assert r[0] == 1.0 and r[1] == 1.0 + 2 ** -6                        # ties go to the even mantissa
    bits = inputs.bf16_bits(r)
    assert np.array_equal((bits.astype(np.uint32) << 16).view(np.float32), r)


def test_operands_are_seeded_and_in_the_storage_type():
    a1, b1 = inputs.operands(inputs.rng_for(3, 7), 64, 32, 48, ("normal", 0.02), ("uniform", -1, 1), "bf16")
    a2, b2 = inputs.operands(inputs.rng_for(3, 7), 64, 32, 48, ("normal", 0.02), ("uniform", -1, 1), "bf16")
    a3, _ = inputs.operands(inputs.rng_for(3, 8), 64, 32, 48, ("normal", 0.02), ("uniform", -1, 1), "bf16")
    assert np.array_equal(a1, a2) and np.array_equal(b1, b2) and not np.array_equal(a1, a3)
    assert a1.shape == (64, 32) and b1.shape == (32, 48) and a1.dtype == np.float32
    assert np.array_equal(inputs.round_bf16(a1), a1) and np.array_equal(inputs.round_bf16(b1), b1)
    assert abs(a1.std() - 0.02) < 0.002 and np.abs(b1).max() <= 1.0
    ai, _ = inputs.operands(inputs.rng_for(0), 8, 8, 8, ("int", -3, 3), ("int", 1, 5), "f32")
    assert np.array_equal(ai, np.rint(ai)) and ai.min() >= -3 and ai.max() <= 3


def test_faults_are_distinct_uniform_and_respect_the_fixed_matrices():
    rng = inputs.rng_for(9)
    n, k, m = 5, 4, 3
    seen = set()
    for _ in range(300):
        fs = inputs.draw_faults(rng, n, k, m, 2, ("uniform", 1.0, 100.0))
        pos = [(f.matrix, f.row, f.col) for f in fs]
        assert len(set(pos)) == 2
        for f in fs:
            lim = {inputs.MAT_A: (n, k), inputs.MAT_B: (k, m), inputs.MAT_C: (n, m)}[f.matrix]
            assert 0 <= f.row < lim[0] and 0 <= f.col < lim[1] and 1.0 <= abs(f.offset) <= 100.0
            seen.add((f.matrix, f.row, f.col))
    assert len(seen) == n * k + k * m + n * m          # every data symbol gets hit sooner or later
    fs = inputs.draw_faults(rng, n, k, m, 2, ("loguniform", 1e-2, 1e3), [inputs.MAT_B, inputs.MAT_C])
    assert [f.matrix for f in fs] == [inputs.MAT_B, inputs.MAT_C] and all(1e-2 <= abs(f.offset) <= 1e3 for f in fs)


def test_operand_faults_store_the_rounded_value_and_report_the_effective_offset():
    A = inputs.store(np.full((2, 2), 0.02), "bf16")
    B = inputs.store(np.ones((2, 2)), "bf16")
    faults = [inputs.Fault(inputs.MAT_A, 1, 0, 1.0), inputs.Fault(inputs.MAT_B, 0, 1, 1e-6),
              inputs.Fault(inputs.MAT_C, 1, 1, -3.5)]
    A2, B2, cf, eff = inputs.apply_operand_faults(A, B, faults, "bf16")
    assert A2[1, 0] == inputs.round_bf16(np.array([A[1, 0] + 1.0], np.float32))[0]
    assert np.array_equal(B2, B)                        # 1e-6 does not survive bf16 storage next to 1.0
    assert cf == [(1, 1, -3.5)]
    assert eff == [(inputs.MAT_A, 1, 0, float(A2[1, 0]) - float(A[1, 0])), (inputs.MAT_C, 1, 1, -3.5)]
    assert A[1, 0] == inputs.store(np.array([0.02]), "bf16")[0]   # inputs untouched
