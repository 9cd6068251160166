"""The oracle against the worked examples the paper prints (tests/golden/, each line cited there)."""
import os

import numpy as np
import pytest

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "section3_1_split_examples.txt")


def cases():
    out = []
    with open(GOLDEN) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            strategy, x, beta, *values = line.split()
            out.append((strategy, float(x), int(beta), [float(v) for v in values]))
    return out


@pytest.mark.parametrize("strategy,x,beta,values", cases())
def test_printed_split_examples(strategy, x, beta, values):
    k = len(values)
    X = np.array([[x]])
    if strategy == "bitmask":
        e = oracle.exponents_floor(X, by_col=False)
        S, _ = oracle.split_rows(X, k, beta, form="bitmask", eA=e)
        got = [float(S[s, 0, 0]) * 2.0 ** (int(e[0]) + 1 - (s + 1) * beta) for s in range(k)]
    elif strategy == "nearest_per_slice":
        S, E = oracle.split_per_slice(X, k, beta, by_col=False)
        got = [float(S[s, 0, 0]) * 2.0 ** (int(E[s, 0]) + 1 - beta) for s in range(k)]
    else:
        raise AssertionError(strategy)
    assert got == values
    assert sum(got) == x
