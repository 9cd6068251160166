"""Pins for the oracle's round-to-nearest split with one scale per slice (Algorithm 5) and for the
product built on it (ozIMMU_RN: Algorithm 5 slices, one FP64 addition per slice pair)."""
from fractions import Fraction

import numpy as np
import pytest

import oracle
from paper_2409_13313_amd import inputs


def two(e):
    return Fraction(2) ** e


def rne(x: Fraction) -> int:
    """Nearest integer, ties to even, in exact rationals."""
    f = x.numerator // x.denominator
    d = x - f
    if d > Fraction(1, 2) or (d == Fraction(1, 2) and f % 2 == 1):
        f += 1
    return f


def ceil_log2(x: Fraction) -> int:
    e = 0
    while two(e) < x:
        e += 1
    while two(e - 1) >= x:
        e -= 1
    return e


def alg5_exact(vec, beta, k):
    """Algorithm 5 on one vector in exact rationals: (slices[k][len], exponents[k])."""
    rem = [Fraction(float(v)) for v in vec]
    S, E = [], []
    for _ in range(k):
        mx = max(abs(v) for v in rem)
        e = ceil_log2(mx) if mx > 0 else 0
        mu = two(e + 1 - beta)
        q = [rne(v / mu) for v in rem]
        rem = [v - qi * mu for v, qi in zip(rem, q)]
        S.append(q)
        E.append(e)
    return S, E, rem


@pytest.mark.parametrize("phi,beta,k,seed", [(0.5, 7, 9, 71), (2.0, 7, 12, 72), (4.0, 6, 10, 73), (1.0, 3, 20, 74)])
def test_per_slice_split_matches_exact_rational_walk(phi, beta, k, seed):
    A, _ = inputs.phi_pair(6, 9, 1, phi, seed=seed)
    A[0, 3] = 0.0
    A[1, :] = 0.0                         # all-zero vector: exponent 0, slices 0
    A[2, :] = 0.0
    A[2, 4] = -0.7                        # a single non-zero: every slice re-normalises to it
    A[3, 0] = 2.0 ** 5                    # power-of-two maximum: q_1 = 2^(beta-1)
    A[3, 1:] *= 2.0 ** 4 / np.abs(A[3, 1:]).max()
    S, E = oracle.split_per_slice(A, k, beta, by_col=False)
    for i in range(A.shape[0]):
        Sx, Ex, rem = alg5_exact(A[i], beta, k)
        assert [int(e) for e in E[:, i]] == Ex
        assert [[int(q) for q in S[s, i]] for s in range(k)] == Sx
    assert S[0, 3, 0] == 2 ** (beta - 1)
    assert not S[:, 1, :].any() and not E[:, 1].any()


def test_worked_vector_single_element_renormalises_every_slice():
    # -0.7 alone, beta = 7: e_1 = 0, q_1 = RNE(-0.7 * 64) = -45, remainder 0.003125 = 0.8 * 2^-8;
    # e_2 = -8, q_2 = RNE(0.8 * 64) = 51, remainder 0.2 * 2^-14 = 0.8 * 2^-16; e_3 = -16, q_3 = 51; ...
    # (Algorithm 8 with the one scale 2^0 gives -45, 26, -51, -26, ... instead.)
    S, E = oracle.split_per_slice(np.array([[-0.7]]), 4, 7, by_col=False)
    assert [int(q) for q in S[:, 0, 0]] == [-45, 51, 51, 51]
    assert [int(e) for e in E[:, 0]] == [0, -8, -16, -24]
    S8, e8 = oracle.split_rows(np.array([[-0.7]]), 4, 7)
    assert [int(q) for q in S8[:, 0, 0]] == [-45, 26, -51, -26] and e8[0] == 0


@pytest.mark.parametrize("by_col", [False, True])
@pytest.mark.parametrize("beta,k", [(7, 10), (5, 14), (2, 20)])
def test_per_slice_split_two_forms_invariants_and_reconstruction(by_col, beta, k):
    A, B = inputs.phi_pair(7, 40, 5, 2.0, seed=75)
    X = B if by_col else A
    S, E = oracle.split_per_slice(X, k, beta, by_col=by_col, form="int")
    S2, E2 = oracle.split_per_slice(X, k, beta, by_col=by_col, form="sigma")
    assert np.array_equal(S, S2) and np.array_equal(E, E2)      # scaling + rint == the printed (a+sigma)-sigma recipe
    assert np.abs(S.astype(np.int32)).max() <= 2 ** (beta - 1)
    spent = ~np.abs(S[1:]).any(axis=1 if by_col else 2)         # nothing left of the vector: exponent 0 by convention
    assert ((E[1:] <= E[:-1] - beta) | (spent & (E[1:] == 0))).all()   # |remainder| <= mu'(s)/2 = 2^(e_s - beta)
    # reconstruction in exact rationals; the remainder after slice k is at most half the last grid
    Ev = E[:, None, :] if by_col else E[:, :, None]
    total = np.zeros(X.shape, dtype=object)
    for s in range(k):
        for idx in np.ndindex(*X.shape):
            e = int(np.broadcast_to(Ev[s], X.shape)[idx])
            total[idx] += int(S[s][idx]) * two(e + 1 - beta)
    for idx in np.ndindex(*X.shape):
        e_last = int(np.broadcast_to(Ev[k - 1], X.shape)[idx])
        assert abs(Fraction(float(X[idx])) - total[idx]) <= two(e_last - beta)
    if beta * k >= 60:
        # enough bits for every entry within a few binades of its vector's maximum: exact
        near = np.abs(X) >= np.abs(X).max(axis=0 if by_col else 1, keepdims=True) * 2.0 ** -6
        assert all(Fraction(float(X[idx])) == total[idx] for idx in np.ndindex(*X.shape) if near[idx])


def test_per_slice_split_of_columns_is_the_transpose():
    _, B = inputs.phi_pair(1, 23, 5, 1.0, seed=76)
    S, E = oracle.split_per_slice(B, 7, 7, by_col=True)
    St, Et = oracle.split_per_slice(np.ascontiguousarray(B.T), 7, 7, by_col=False)
    assert np.array_equal(E, Et) and np.array_equal(S, St.transpose(0, 2, 1))


def test_first_slice_is_algorithm_8s_first_slice():
    A, _ = inputs.phi_pair(9, 50, 1, 1.0, seed=77)
    S5, E5 = oracle.split_per_slice(A, 3, 7, by_col=False)
    S8, e8 = oracle.split_rows(A, 3, 7)
    assert np.array_equal(E5[0], e8) and np.array_equal(S5[0], S8[0])


def test_long_random_vectors_reduce_to_the_shared_scale_split():
    # With many entries per vector the largest remainder after slice s almost surely lies in
    # (2^(e_s-beta-1), 2^(e_s-beta)], so e_(s+1) = e_s - beta: Algorithm 5 then IS Algorithm 8, and
    # ozIMMU_RN is the round-to-nearest split with one addition per slice pair, bit for bit.
    A, B = inputs.phi_pair(12, 600, 10, 0.5, seed=78)
    k, beta = 6, 7
    S5, E5 = oracle.split_per_slice(A, k, beta, by_col=False)
    S8, e8 = oracle.split_rows(A, k, beta)
    assert np.array_equal(E5, e8[None, :] - beta * np.arange(k)[:, None])
    assert np.array_equal(S5, S8)
    D5 = oracle.dgemm_per_slice(A, B, k)
    D8 = oracle.dgemm_variant(A, B, k, "rn", "per_pair")
    assert np.array_equal(D5, D8)


def walk_per_slice(A, B, k):
    """ozIMMU_RN re-walked in exact rationals from the oracle's slices: one correctly rounded FP64
    addition per slice pair, g = s + t ascending, s ascending."""
    m, n = A.shape
    p = B.shape[1]
    beta, _ = oracle.params(n)
    SA, EA = oracle.split_per_slice(A, k, beta, by_col=False)
    SB, EB = oracle.split_per_slice(B, k, beta, by_col=True)
    D = np.zeros((m, p))
    count = 0
    for g in range(2, k + 2):
        for s in range(1, g):
            t = g - s
            C = SA[s - 1].astype(np.int64) @ SB[t - 1].astype(np.int64)
            for i in range(m):
                for j in range(p):
                    term = int(C[i, j]) * two(int(EA[s - 1, i]) + int(EB[t - 1, j]) + 2 - 2 * beta)
                    D[i, j] = float(Fraction(float(D[i, j])) + term)     # Fraction -> float rounds to nearest even
            count += 1
    return D, count


@pytest.mark.parametrize("m,n,p,k,phi,seed", [(5, 3, 4, 5, 2.0, 79), (4, 17, 6, 8, 4.0, 80), (3, 1, 3, 3, 1.0, 81)])
def test_dgemm_per_slice_matches_exact_walk_on_short_vectors(m, n, p, k, phi, seed):
    # short vectors: the per-slice scales differ from the shared-scale ones, so this exercises them
    A, B = inputs.phi_pair(m, n, p, phi, seed=seed)
    D, w = oracle.dgemm_per_slice(A, B, k, return_addends=True)
    Dw, count = walk_per_slice(A, B, k)
    assert w == count == k * (k + 1) // 2
    assert np.array_equal(D, Dw)
    if n > 1:
        assert not np.array_equal(D, oracle.dgemm_variant(A, B, k, "rn", "per_pair"))


def test_dgemm_per_slice_one_slice_equals_shared_scale_method():
    A, B = inputs.phi_pair(6, 20, 7, 1.0, seed=82)
    assert np.array_equal(oracle.dgemm_per_slice(A, B, 1), oracle.dgemm(A, B, 1))


def test_dgemm_per_slice_exact_on_small_integers_and_accurate_on_random_input():
    A, B = inputs.small_int_pair(9, 33, 8, 64, seed=83)
    assert np.array_equal(oracle.dgemm_per_slice(A, B, 1), A @ B)
    A, B = inputs.phi_pair(24, 200, 24, 2.0, seed=84)
    hi, lo = oracle.dot2_gemm(A, B)
    absab = np.abs(A) @ np.abs(B)
    errs = [float((np.abs((oracle.dgemm_per_slice(A, B, k) - hi) - lo) / absab).max()) for k in (4, 6, 8, 10)]
    assert errs[0] > errs[1] > errs[2] and errs[3] < 1e-15
    # the same k with the shared-scale split is never much better: per-slice scales only tighten the grids
    errs_h = [float((np.abs((oracle.dgemm_variant(A, B, k, "rn", "per_pair") - hi) - lo) / absab).max())
              for k in (4, 6, 8)]
    assert all(e5 <= 1.01 * e8 for e5, e8 in zip(errs, errs_h))
