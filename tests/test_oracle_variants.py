"""Pins for the comparison variants in the oracle: bit-mask slices (Algorithm 3), one FP64 addition
per slice pair (Algorithm 4), and the wider INT32 chunks that round-to-nearest slices allow."""
from fractions import Fraction

import numpy as np
import pytest

import oracle
from paper_2409_13313_amd import inputs

U = 2.0 ** -53


def two(e):
    return Fraction(2) ** e


@pytest.mark.parametrize("phi,beta,k", [(0.5, 7, 9), (2.0, 7, 12), (4.0, 6, 10), (1.0, 3, 20)])
def test_bitmask_slices_are_truncated_digits_of_the_magnitude(phi, beta, k):
    A, _ = inputs.phi_pair(6, 31, 1, phi, seed=61)
    A[0, 3] = 0.0
    A[1, :] = 0.0
    A[2, 0] = 2.0 ** 5            # power-of-two maximum
    A[2, 1:] *= 2.0 ** 5 / (np.abs(A[2, 1:]).max() * 1.5)
    S, e = oracle.split_rows(A, k, beta, form="bitmask")
    for i in range(A.shape[0]):
        mx = max(Fraction(abs(float(v))) for v in A[i])
        if mx == 0:
            assert e[i] == 0 and not S[:, i, :].any()
            continue
        assert two(int(e[i])) <= mx < two(int(e[i]) + 1)                  # floor(log2 max), Algorithm 3, its scale
        for j in range(A.shape[1]):
            a = Fraction(float(A[i, j]))
            sign = 1 if a >= 0 else -1
            rem = abs(a)
            for s in range(1, k + 1):
                grid = two(int(e[i]) + 1 - s * beta)
                q = int(S[s - 1, i, j])
                assert q == 0 or (q > 0) == (sign > 0)                    # every slice carries the sign of a
                assert abs(q) <= 2 ** beta - 1                            # I_{beta+1}, Section 5.2
                rem_new = rem - abs(q) * grid
                assert 0 <= rem_new < grid                                # truncation: the next beta bits
                rem = rem_new
            assert rem < two(int(e[i]) + 1 - k * beta)                    # the bound on V_k of Section 5.1


def test_bitmask_split_of_columns_is_the_transpose():
    _, B = inputs.phi_pair(1, 23, 5, 1.0, seed=62)
    S, e = oracle.split_cols(B, 7, 7, form="bitmask")
    St, et = oracle.split_rows(np.ascontiguousarray(B.T), 7, 7, form="bitmask")
    assert np.array_equal(e, et) and np.array_equal(S, St.transpose(0, 2, 1))


@pytest.mark.parametrize("n", [1, 2, 100, 255, 256, 257, 5000, 16384, 16385, 65536, 2 ** 17, 2 ** 17 + 1, 2 ** 20, 2 ** 29])
def test_wide_r_is_the_largest_safe_power_of_two(n):
    beta, r = oracle.params(n)
    rw = oracle.r_wide(n, beta)
    bound = (2 ** (beta - 1)) ** 2              # |q| <= 2^(beta-1) for round-to-nearest slices
    assert rw & (rw - 1) == 0 and rw >= r
    assert rw * n * bound <= 2 ** 31 - 1 < 2 * rw * n * bound


def test_wide_chunks_of_extreme_rn_slices_fit_int32():
    n = 16384
    beta, r = oracle.params(n)
    rw = oracle.r_wide(n, beta)
    assert (r, rw) == (8, 16)
    SA = np.full((rw + 1, 1, n), 64, dtype=np.int8)
    SB = np.full((rw + 1, n, 1), -64, dtype=np.int8)
    assert oracle.group_chunk(SA, SB, rw + 1, 1, rw)[0, 0] == -rw * n * 4096


def walk(A, B, k, split, accumulate):
    """The schedule re-walked in exact rationals from the oracle's slices (one correctly rounded
    FP64 addition per chunk)."""
    m, n = A.shape
    p = B.shape[1]
    beta, r = oracle.params(n)
    r = {"grouped": r, "per_pair": 1, "wide": oracle.r_wide(n, beta)}[accumulate]
    form = "bitmask" if split == "bitmask" else "int"
    SA, eA = oracle.split_rows(A, k, beta, form=form)
    SB, eB = oracle.split_cols(B, k, beta, form=form)
    SA64, SB64 = SA.astype(np.int64), SB.astype(np.int64)
    D = [[0.0] * p for _ in range(m)]
    w = 0
    for g in range(2, k + 2):
        q, C = 0, np.zeros((m, p), dtype=np.int64)
        for s in range(1, g):
            q += 1
            C += SA64[s - 1] @ SB64[g - s - 1]
            if q == r or s == g - 1:
                w += 1
                assert np.abs(C).max() < 2 ** 31
                for i in range(m):
                    for j in range(p):
                        term = Fraction(int(C[i, j])) * Fraction(2) ** (int(eA[i]) + int(eB[j]) + 2 - beta * g)
                        D[i][j] = float(Fraction(D[i][j]) + term)
                q, C = 0, np.zeros((m, p), dtype=np.int64)
    return np.array(D), w


@pytest.mark.parametrize("split,accumulate", [("bitmask", "grouped"), ("bitmask", "per_pair"), ("rn", "wide"),
                                              ("rn", "per_pair")])
@pytest.mark.parametrize("m,n,p,k", [(3, 40, 2, 7), (2, 65536, 2, 6)])
def test_variants_equal_their_brute_force_walk(split, accumulate, m, n, p, k):
    A, B = inputs.phi_pair(m, n, p, 1.0, seed=63)
    D, w = oracle.dgemm_variant(A, B, k, split, accumulate, return_addends=True)
    Dbf, wbf = walk(A, B, k, split, accumulate)
    assert w == wbf
    assert np.array_equal(D, Dbf)
    if accumulate == "per_pair":
        assert w == k * (k + 1) // 2          # Section 3.2: a sum of k(k+1)/2 FP64 matrices


def test_default_variant_is_the_main_path_and_wide_differs_only_in_rounding():
    A, B = inputs.phi_pair(20, 65536, 6, 0.5, seed=64)       # r = 2, r_wide = 4
    k = 9
    D = oracle.dgemm(A, B, k)
    assert np.array_equal(oracle.dgemm_variant(A, B, k, "rn", "grouped"), D)
    Dw, w = oracle.dgemm_variant(A, B, k, "rn", "wide", return_addends=True)
    assert w < oracle.count_addends(k, 2)
    absab = np.abs(A) @ np.abs(B)
    assert (np.abs(Dw - D) <= 2 * oracle.count_addends(k, 2) * U * absab).all()


def test_accuracy_ordering_reported_in_section_4_1():
    # round-to-nearest slices are at least as accurate as bit-mask slices for the same k (below the
    # FP64 floor), and per-pair accumulation is no better than grouped accumulation
    A, B = inputs.phi_pair(96, 96, 96, 2.0, seed=65)
    hi, lo = oracle.dot2_gemm(A, B)
    absab = np.abs(A) @ np.abs(B)

    def err(split, acc, k):
        return float((np.abs((oracle.dgemm_variant(A, B, k, split, acc) - hi) - lo) / absab).max())

    for k in (6, 7, 8, 9):
        assert err("rn", "grouped", k) <= 1.05 * err("bitmask", "grouped", k)
    assert err("bitmask", "grouped", 12) <= err("bitmask", "per_pair", 12) * 1.001
