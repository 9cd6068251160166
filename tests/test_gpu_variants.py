"""GPU parity for the comparison variants (bit-mask split, per-pair and wide accumulation)."""
import numpy as np
import pytest

import oracle
from paper_2409_13313_amd import inputs

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def oz():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU: the HIP path has no CPU fallback")
    from paper_2409_13313_amd import ozimmu
    return ozimmu


def dev(x):
    return torch.from_numpy(np.ascontiguousarray(x)).cuda()


@pytest.mark.parametrize("rows,n,phi,k,seed", [(256, 256, 0.5, 8, 0), (300, 200, 4.0, 14, 1), (65, 1029, 1.0, 20, 2),
                                               (40, 20000, 1.0, 6, 3)])      # rows too long for the one-pass kernel
def test_bitmask_slices_bit_exact(oz, rows, n, phi, k, seed):
    A, B = inputs.phi_pair(rows, n, rows, phi, seed=seed)
    A[1, :] = 0.0
    A[2, 0] = 2.0 ** 9        # a power-of-two row maximum: floor and ceil exponents coincide
    beta, _ = oracle.params(n)
    want, e_want = oracle.split_rows(A, k, beta, form="bitmask")
    SA, eA = oz.split_A(dev(A), k, split="bitmask")
    assert np.array_equal(eA.cpu().numpy(), e_want)
    assert np.array_equal(oz.export_slices(rows, n, k, SA).cpu().numpy(), want)
    wantb, eb_want = oracle.split_cols(B, k, beta, form="bitmask")
    SB, eB = oz.split_B(dev(B), k, split="bitmask")
    assert np.array_equal(eB.cpu().numpy(), eb_want)
    assert np.array_equal(oz.export_slices(rows, n, k, SB).cpu().numpy().transpose(0, 2, 1), wantb)


@pytest.mark.parametrize("split,accumulate", [("bitmask", "grouped"), ("bitmask", "per_pair"), ("rn", "per_pair"),
                                              ("rn", "wide"), ("rn", "grouped")])
@pytest.mark.parametrize("m,n,p,k,phi", [(300, 520, 270, 9, 2.0), (130, 65536, 70, 6, 1.0)])
def test_variants_match_oracle_bit_for_bit(oz, split, accumulate, m, n, p, k, phi):
    A, B = inputs.phi_pair(m, n, p, phi, seed=71)
    want = oracle.dgemm_variant(A, B, k, split, accumulate)
    got = oz.dgemm_variant(dev(A), dev(B), k, split, accumulate).cpu().numpy()
    assert np.isfinite(got).all()
    assert (np.abs(got - want) <= 2 * np.spacing(np.abs(want))).all()
    assert np.array_equal(got, want)


def test_wide_r_and_mode_errors(oz):
    for n in (256, 5000, 16384, 65536, 2 ** 17 + 1):
        beta, _ = oracle.params(n)
        assert oz.r_wide(n) == oracle.r_wide(n, beta)
    A = torch.zeros((4, 4), dtype=torch.float64, device="cuda")
    with pytest.raises(oz.OzimmuError):
        oz.dgemm_variant(A, A, 4, "bitmask", "wide")      # wide chunks need round-to-nearest slices
