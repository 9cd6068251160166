"""Pins for the oracle's scale exponents and INT8 slice extraction.

The slices are pinned by the DEFINITION they must satisfy, checked in exact
rational arithmetic on the oracle's outputs only: slice s is the integer
nearest to (remainder / grid_s), ties to even, which is unique.  A dropped
rounding, a wrong grid exponent, a wrong sign or an off-by-one in the scale all
break one of the inequalities below.
"""
from fractions import Fraction

import numpy as np
import pytest

import oracle
from paper_2409_13313_amd import inputs


def two(e):
    return Fraction(2) ** e


def check_exponents(X, e):
    """2^(e-1) < max|row| <= 2^e  (i.e. e = ceil(log2 max)); zero row -> 0."""
    for i in range(X.shape[0]):
        mx = max(Fraction(abs(float(v))) for v in X[i])
        if mx == 0:
            assert e[i] == 0
        else:
            assert two(int(e[i]) - 1) < mx <= two(int(e[i]))


def check_slices(X, S, e, beta, ties_expected=False):
    """S[s-1][i][j] is RNE(remainder / grid_s), grid_s = 2^(e_i + 1 - s beta)."""
    k = S.shape[0]
    saw_tie = False
    for i in range(X.shape[0]):
        for j in range(X.shape[1]):
            rem = Fraction(float(X[i, j]))
            for s in range(1, k + 1):
                grid = two(int(e[i]) + 1 - s * beta)
                q = int(S[s - 1, i, j])
                assert abs(q) <= 2 ** (beta - 1)                  # tighter than the paper's I_{beta+1}
                rem_new = rem - q * grid
                assert abs(rem_new) <= grid / 2                   # nearest
                if abs(rem_new) == grid / 2:                      # tie -> even
                    assert q % 2 == 0
                    saw_tie = True
                rem = rem_new
            # the bound on V_k of Section 5.1: |V_k| <= 2^(-beta k + 1) * ufp(row max); 2^e <= 2 ufp
            assert abs(rem) <= two(int(e[i]) - k * beta)
    if ties_expected:
        assert saw_tie


CASES = [(0.5, 7, 9), (2.0, 7, 12), (4.0, 7, 14), (1.0, 6, 10), (1.0, 3, 20), (0.5, 1, 8)]


@pytest.mark.parametrize("phi,beta,k", CASES)
def test_split_rows_is_nearest_even_on_each_grid(phi, beta, k):
    A, _ = inputs.phi_pair(7, 33, 1, phi, seed=11)
    S, e = oracle.split_rows(A, k, beta)
    check_exponents(A, e)
    check_slices(A, S, e, beta)


@pytest.mark.parametrize("phi,beta,k", CASES)
def test_split_cols_is_split_rows_of_transpose(phi, beta, k):
    _, B = inputs.phi_pair(1, 29, 6, phi, seed=12)
    S, e = oracle.split_cols(B, k, beta)
    check_exponents(B.T, e)
    check_slices(np.ascontiguousarray(B.T), np.ascontiguousarray(S.transpose(0, 2, 1)), e, beta)
    St, et = oracle.split_rows(np.ascontiguousarray(B.T), k, beta)
    assert np.array_equal(et, e)
    assert np.array_equal(St.transpose(0, 2, 1), S)


def special_matrix():
    rows = [
        [1.0, -0.7, 0.3, 1.2345 * 2.0 ** -10, 0.0, 2.5 / 64, 3.5 / 64, -2.5 / 64],   # power-of-two max, ties
        [0.0] * 8,                                                                     # zero row
        [3.0, -3.0, 1.5, 0.75, 2.0 ** -60, -2.0 ** -61, 1e-300, 2.9999999999999996],
        [2.0 ** -1070, -2.0 ** -1074, 3 * 2.0 ** -1074, 0.0, 2.0 ** -1072, 0, 0, 0],   # subnormal row
        [2.0 ** 900, -1.0, 2.0 ** 899 + 2.0 ** 860, 5e269, -2.0 ** 900, 1e-5, 0, 7.0],
        [-5.0, 4.999999999999999, 0.5 + 2.0 ** -53, 0.5 - 2.0 ** -54, 1 / 3, -2 / 3, 0.1, 6.5],
        [2.0 ** -7 * 1.5, 2.0 ** -7 * 0.5, 2.0 ** -14 * 0.5, 2.0 ** -14 * 1.5, 1.0, 0, 0, 0],  # ties on grids 1 and 2
    ]
    return np.array(rows, dtype=np.float64)


@pytest.mark.parametrize("beta,k", [(7, 9), (7, 16), (5, 12), (2, 20)])
def test_split_special_values(beta, k):
    X = special_matrix()
    S, e = oracle.split_rows(X, k, beta)
    check_exponents(X, e)
    check_slices(X, S, e, beta, ties_expected=(beta == 7))
    assert e[0] == 0 and S[0, 0, 0] == 2 ** (beta - 1)        # a power-of-two maximum gives q_1 = 2^(beta-1)
    assert not S[:, 1, :].any()


def test_row_of_five_hand_checked_digits():
    # 1.0 with scale 2^0 and beta = 7: only q_1 = 64.  0.0: all zero.
    # 2.5/64 is a tie on grid 1/64 -> q_1 = 2 (even), remainder +1/128 = 64 * 2^-13 -> q_2 = 64.
    # 3.5/64 -> q_1 = 4, remainder -1/128 -> q_2 = -64.
    X = np.array([[1.0, 0.0, 2.5 / 64, 3.5 / 64]])
    S, e = oracle.split_rows(X, 3, 7)
    assert e[0] == 0
    assert S[:, 0, 0].tolist() == [64, 0, 0]
    assert S[:, 0, 1].tolist() == [0, 0, 0]
    assert S[:, 0, 2].tolist() == [2, 64, 0]
    assert S[:, 0, 3].tolist() == [4, -64, 0]


@pytest.mark.parametrize("phi", [0.0, 0.5, 2.0, 4.0])
@pytest.mark.parametrize("beta,k", [(7, 12), (6, 10), (4, 20)])
def test_integer_form_equals_floating_point_recipe_of_algorithm_8(phi, beta, k):
    A, B = inputs.phi_pair(37, 129, 41, phi, seed=3)
    S0, e0 = oracle.split_rows(A, k, beta, form="int")
    S1, e1 = oracle.split_rows(A, k, beta, form="sigma")
    assert np.array_equal(e0, e1) and np.array_equal(S0, S1)
    T0, _ = oracle.split_cols(B, k, beta, form="int")
    T1, _ = oracle.split_cols(B, k, beta, form="sigma")
    assert np.array_equal(T0, T1)


def test_two_forms_agree_on_special_values_in_fp_range():
    X = special_matrix()[[0, 1, 2, 5, 6]]     # rows whose sigma stays finite and whose entries are normal
    for beta, k in [(7, 9), (7, 16), (3, 20)]:
        S0, _ = oracle.split_rows(X, k, beta, form="int")
        S1, _ = oracle.split_rows(X, k, beta, form="sigma")
        assert np.array_equal(S0, S1)


def test_slices_reconstruct_bit_exactly_once_k_covers_the_mantissa():
    # the expansion of A of Section 2: A = diag(2^eA) sum_s 2^(1 - s beta) A''_s + V_k.  Entries within
    # one binade of the row maximum have all 53 bits above 2^(eA - 54), so
    # k * beta - 1 >= 54 (k = 8, beta = 7) leaves V_k = 0 and in-order FP64
    # summation of the slices returns a_ij bit for bit.
    rng = np.random.Generator(np.random.PCG64(5))
    A = (1.0 + rng.random((16, 64))) * np.where(rng.random((16, 64)) < 0.5, -1.0, 1.0)
    A *= 2.0 ** rng.integers(-30, 30, size=(16, 1))
    k, beta = 8, 7
    S, e = oracle.split_rows(A, k, beta)
    R = np.zeros_like(A)
    for s in range(1, k + 1):
        R = R + np.ldexp(S[s - 1].astype(np.float64), (e[:, None] + 1 - s * beta).astype(np.int32))
    assert np.array_equal(R, A)
    # with one slice fewer the residual is not zero everywhere, and it obeys the bound on V_k of Section 5.1
    S7 = S[:7]
    R7 = sum(np.ldexp(S7[s - 1].astype(np.float64), (e[:, None] + 1 - s * beta).astype(np.int32)) for s in range(1, 8))
    V = A - R7
    assert V.any()
    assert (np.abs(V) <= np.ldexp(1.0, (e[:, None] - 7 * beta).astype(np.int32))).all()
