"""Pins for step (v) of the scheme in the oracle: C <- alpha D + beta C, and transposed operands."""
from fractions import Fraction

import numpy as np

import oracle
from paper_2409_13313_amd import inputs


def test_alpha_one_beta_zero_is_the_plain_product_and_old_c_is_not_read():
    A, B = inputs.phi_pair(9, 40, 7, 1.0, seed=41)
    D = oracle.dgemm(A, B, 8)
    C = np.full((9, 7), np.nan)
    assert np.array_equal(oracle.gemm_ex(False, False, 1.0, A, B, 0.0, C, 8), D)


def test_three_rounded_operations_per_element():
    A, B = inputs.phi_pair(5, 33, 6, 0.5, seed=42)
    rng = np.random.Generator(np.random.PCG64(43))
    C = rng.standard_normal((5, 6))
    alpha, beta = 1.0 / 3.0, -0.7
    D = oracle.dgemm(A, B, 9)
    got = oracle.gemm_ex(False, False, alpha, A, B, beta, C, 9)
    for i in range(5):
        for j in range(6):
            t1 = float(Fraction(alpha) * Fraction(float(D[i, j])))      # Fraction -> float rounds correctly
            t2 = float(Fraction(beta) * Fraction(float(C[i, j])))
            assert got[i, j] == float(Fraction(t1) + Fraction(t2))


def test_power_of_two_scalars_are_exact_and_alpha_zero_scales_c():
    A, B = inputs.phi_pair(6, 20, 4, 2.0, seed=44)
    C = np.random.Generator(np.random.PCG64(45)).standard_normal((6, 4))
    D = oracle.dgemm(A, B, 7)
    assert np.array_equal(oracle.gemm_ex(False, False, 4.0, A, B, 0.0, C, 7), 4.0 * D)
    assert np.array_equal(oracle.gemm_ex(False, False, 0.0, A, B, 0.5, C, 7), 0.0 * D + 0.5 * C)
    assert np.array_equal(oracle.gemm_ex(False, False, -2.0, A, B, 1.0, C, 7), -2.0 * D + C)


def test_transposed_operands_are_the_product_of_the_transposes():
    A, B = inputs.phi_pair(8, 30, 5, 1.0, seed=46)
    D = oracle.dgemm(A, B, 8)
    Z = np.zeros((8, 5))
    At, Bt = np.ascontiguousarray(A.T), np.ascontiguousarray(B.T)
    assert np.array_equal(oracle.gemm_ex(True, False, 1.0, At, B, 0.0, Z, 8), D)
    assert np.array_equal(oracle.gemm_ex(False, True, 1.0, A, Bt, 0.0, Z, 8), D)
    assert np.array_equal(oracle.gemm_ex(True, True, 1.0, At, Bt, 0.0, Z, 8), D)
