"""Pins for the GEMM oracle and the bf16 helpers."""
import numpy as np

from oracle.gemm import gemm_nt
from workloads import gemm_inputs


def test_against_triple_loop_and_identity():
    rng = np.random.default_rng(0)
    a = rng.integers(-4, 5, size=(5, 7)).astype(np.float64)
    b = rng.integers(-4, 5, size=(3, 7)).astype(np.float64)
    want = [[sum(a[i][k] * b[j][k] for k in range(7)) for j in range(3)] for i in range(5)]
    assert np.array_equal(gemm_nt(a, b), np.array(want))
    assert np.array_equal(gemm_nt(a, np.eye(7)), a)            # B = I (as [N, K]) returns A


def test_bf16_rounding_ties_to_even():
    # 1 + 2^-8 lies halfway between bf16 neighbours 1 and 1 + 2^-7: ties go to the even mantissa (1.0)
    x = np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -20, -2.5, 0.0], dtype=np.float32)
    r = gemm_inputs.bf16_round(x)
    assert r.tolist() == [1.0, 1.0 + 2.0 ** -6, 1.0 + 2.0 ** -7, -2.5, 0.0]
    assert np.array_equal(gemm_inputs.bits_to_f32(gemm_inputs.bf16_bits(r)), r)
