"""Pins for the oracle's parameter functions (beta, r, number of FP64 addends).

Each check compares the oracle's integer-only code with something it does not
contain: the paper's real-valued formulas evaluated with math.log2, facts the
paper states in prose, the overflow inequality of Section 5.2, and the closed
form w of Section 5.2.
"""
import math

import pytest

import oracle


def paper_beta(n):  # the formula for beta of Section 2, evaluated as printed
    return min(7, math.floor((31 - math.log2(n)) / 2))


def paper_r(n, beta):  # the definition of r of Section 3.2, evaluated as printed
    return max(1, 2 ** (31 - 2 * beta - math.ceil(math.log2(n))))


SWEEP = sorted(set(
    [1, 2, 3, 5, 7, 100, 255, 256, 257, 1000, 1024, 4096, 5000, 8192, 16384, 65536]
    + [2 ** e + d for e in range(1, 30) for d in (-1, 0, 1) if 2 ** e + d >= 1]
    + [3 * 2 ** e for e in range(0, 27)]))


@pytest.mark.parametrize("n", SWEEP)
def test_beta_r_match_printed_formulas(n):
    if n > 2 ** 29:
        pytest.skip("outside the paper's assumption n <= 2^29")
    beta, r = oracle.params(n)
    assert beta == paper_beta(n)
    assert r == paper_r(n, beta)


def test_facts_stated_in_prose():
    # Section 4.1: beta < 7 exactly when n > 2^17.
    assert oracle.params(2 ** 17)[0] == 7
    assert oracle.params(2 ** 17 + 1)[0] == 6
    # Section 2: beta >= 1 is equivalent to n <= 2^29.
    assert oracle.params(2 ** 29)[0] == 1
    assert oracle.params(2 ** 29 + 1)[0] == 0
    # Algorithm 7 (r >= k version) prints beta = 7 for its regime.
    for n in (256, 1024, 8192):
        beta, r = oracle.params(n)
        assert beta == 7 and r >= 12


@pytest.mark.parametrize("n", [n for n in SWEEP if n <= 2 ** 29])
def test_r_products_cannot_overflow_int32(n):
    # Section 5.2: slices are bounded by 2^beta - 1, so r products of inner
    # length n stay within INT32.
    beta, r = oracle.params(n)
    assert r * n * (2 ** beta - 1) ** 2 <= 2 ** 31 - 1


@pytest.mark.parametrize("k", range(1, 21))
@pytest.mark.parametrize("r", [1, 2, 4, 8, 16, 32, 512])
def test_addend_count_matches_closed_form(k, r):
    # Section 5.2: w = ceil(k/r) * (k - (r/2) * floor((k-1)/r))
    w = math.ceil(k / r) * (k - (r / 2) * ((k - 1) // r))
    assert oracle.count_addends(k, r) == w
    sched = oracle.chunks(k, r)
    assert len(sched) == w
    # every kept pair (s, t), s + t <= k + 1, appears exactly once (Section 3.2: k(k+1)/2 products)
    pairs = [(s, g - s) for (g, s0, s1) in sched for s in range(s0, s1 + 1)]
    assert len(pairs) == k * (k + 1) // 2 == len(set(pairs))
    assert all(1 <= s and 1 <= t and s + t <= k + 1 for s, t in pairs)
    assert all(s1 - s0 + 1 <= r for (_, s0, s1) in sched)
    # groups ascend, chunks ascend inside a group
    assert sched == sorted(sched)
