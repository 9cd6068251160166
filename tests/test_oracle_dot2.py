"""Pins for the compensated (Dot2) reference: exact rational dot products."""
from fractions import Fraction

import numpy as np

import oracle

U = Fraction(1, 2 ** 53)


def exact_dot(a, b):
    return sum(Fraction(float(x)) * Fraction(float(y)) for x, y in zip(a, b))


def test_dot2_is_twice_working_precision_on_ill_conditioned_dots():
    rng = np.random.Generator(np.random.PCG64(31))
    n = 200
    for trial in range(6):
        a = rng.standard_normal(n) * 2.0 ** rng.integers(-20, 20, n)
        b = rng.standard_normal(n) * 2.0 ** rng.integers(-20, 20, n)
        # force heavy cancellation: second half undoes the first half up to a small remainder
        a[n // 2:] = a[: n // 2]
        b[n // 2:] = -b[: n // 2] * (1 + 2.0 ** -30)
        ex = exact_dot(a, b)
        hi, lo = oracle.dot2_gemm(a[None, :], b[:, None])
        got = Fraction(float(hi[0, 0])) + Fraction(float(lo[0, 0]))
        mag = sum(abs(Fraction(float(x)) * Fraction(float(y))) for x, y in zip(a, b))
        # Ogita-Rump-Oishi: |res - exact| <= u|exact| + gamma_n^2 * sum|a_i b_i|; hi+lo drops the first term
        gamma = (n * U) / (1 - n * U)
        assert abs(got - ex) <= 2 * gamma * gamma * mag + U * U * abs(ex)
        plain = Fraction(float(np.dot(a, b)))
        assert abs(got - ex) < abs(plain - ex) or plain == ex
        assert abs(float(lo[0, 0])) <= abs(float(hi[0, 0])) * 2.0 ** -52 or hi[0, 0] == 0


def test_dot2_exact_on_integer_data_and_layout():
    rng = np.random.Generator(np.random.PCG64(32))
    A = rng.integers(-1000, 1000, size=(5, 33)).astype(np.float64)
    B = rng.integers(-1000, 1000, size=(33, 4)).astype(np.float64)
    hi, lo = oracle.dot2_gemm(A, B)
    assert np.array_equal(hi, (A.astype(np.int64) @ B.astype(np.int64)).astype(np.float64))
    assert not lo.any()
