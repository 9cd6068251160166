"""GPU parity for the round-to-nearest split with one scale per slice (Algorithm 5) and ozIMMU_RN."""
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


# short vectors (3, 17) make the per-slice scales differ from the shared-scale ones; 1029 and 700 are ragged
# against every tile; phi = 4 spreads the exponents
@pytest.mark.parametrize("rows,n,phi,k,seed", [(256, 256, 0.5, 8, 0), (300, 17, 4.0, 14, 1), (65, 1029, 1.0, 20, 2),
                                               (700, 3, 2.0, 9, 3), (5, 2 ** 17 + 128, 0.5, 4, 4)])
def test_per_slice_split_bit_exact(oz, rows, n, phi, k, seed):
    A, B = inputs.phi_pair(rows, n, rows, phi, seed=seed)
    A[1, :] = 0.0
    A[2, :] = 0.0
    A[2, n // 2] = -0.7
    A[3, 0] = 2.0 ** 9
    B[:, 1] = 0.0
    B[:, 2] = 0.0
    B[n // 3, 2] = 1.0 / 3.0
    beta, _ = oracle.params(n)
    want, e_want = oracle.split_per_slice(A, k, beta, by_col=False)
    SA, eA = oz.split_A(dev(A), k, split="per_slice")
    assert np.array_equal(eA.cpu().numpy(), e_want)
    assert np.array_equal(oz.export_slices(rows, n, k, SA).cpu().numpy(), want)
    wantb, eb_want = oracle.split_per_slice(B, k, beta, by_col=True)
    SB, eB = oz.split_B(dev(B), k, split="per_slice")
    assert np.array_equal(eB.cpu().numpy(), eb_want)
    assert np.array_equal(oz.export_slices(rows, n, k, SB).cpu().numpy().transpose(0, 2, 1), wantb)


def test_per_slice_split_of_strided_operands(oz):
    A, B = inputs.phi_pair(70, 131, 90, 2.0, seed=5)
    beta, _ = oracle.params(131)
    bigA = torch.full((70, 140), 7.0, dtype=torch.float64, device="cuda")
    bigA[:, :131] = dev(A)
    bigB = torch.full((131, 97), 7.0, dtype=torch.float64, device="cuda")
    bigB[:, :90] = dev(B)
    SA, eA = oz.split_A(bigA[:, :131], 6, split="per_slice")
    SB, eB = oz.split_B(bigB[:, :90], 6, split="per_slice")
    want, e_want = oracle.split_per_slice(A, 6, beta, by_col=False)
    wantb, eb_want = oracle.split_per_slice(B, 6, beta, by_col=True)
    assert np.array_equal(eA.cpu().numpy(), e_want) and np.array_equal(eB.cpu().numpy(), eb_want)
    assert np.array_equal(oz.export_slices(70, 131, 6, SA).cpu().numpy(), want)
    assert np.array_equal(oz.export_slices(90, 131, 6, SB).cpu().numpy().transpose(0, 2, 1), wantb)


@pytest.mark.parametrize("m,n,p,k,phi", [(300, 520, 270, 9, 2.0), (257, 5, 513, 7, 4.0), (40, 3, 30, 12, 1.0),
                                         (130, 65536, 70, 6, 1.0)])
def test_ozimmu_rn_matches_oracle_bit_for_bit(oz, m, n, p, k, phi):
    A, B = inputs.phi_pair(m, n, p, phi, seed=72)
    want = oracle.dgemm_per_slice(A, B, k)
    got = oz.dgemm_variant(dev(A), dev(B), k, "per_slice", "per_pair").cpu().numpy()
    assert np.isfinite(got).all()
    assert (np.abs(got - want) <= 2 * np.spacing(np.abs(want))).all()
    assert np.array_equal(got, want)


def test_phase_calls_reproduce_the_fused_path(oz):
    m, n, p, k = 150, 9, 140, 5
    A, B = inputs.phi_pair(m, n, p, 2.0, seed=73)
    beta, _ = oracle.params(n)
    dA, dB = dev(A), dev(B)
    SA, eA = oz.split_A(dA, k, split="per_slice")
    SB, eB = oz.split_B(dB, k, split="per_slice")
    D = torch.empty((m, p), dtype=torch.float64, device="cuda")
    first = True
    for g in range(2, k + 2):
        for s in range(1, g):
            C = oz.gemm_group(m, n, p, SA, k, SB, k, g, s, s)
            oz.accumulate(C, eA[s - 1], eB[g - s - 1], beta, 2, first, D)   # g = 2: factor 2^(e + f + 2 - 2 beta)
            first = False
    fused = oz.dgemm_variant(dA, dB, k, "per_slice", "per_pair")
    assert torch.equal(D, fused)
    assert np.array_equal(fused.cpu().numpy(), oracle.dgemm_per_slice(A, B, k))


def test_mode_errors_and_workspace_size(oz):
    A = torch.zeros((4, 4), dtype=torch.float64, device="cuda")
    for acc in ("grouped", "wide"):
        with pytest.raises(oz.OzimmuError):
            oz.dgemm_variant(A, A, 4, "per_slice", acc)       # per-slice scales share no shift inside a group
    # the least workspace of the shared-scale splits has no room for the remainders of the per-slice split
    small = torch.empty(oz.workspace_bytes_min(300, 520, 270, 8), dtype=torch.uint8, device="cuda")
    A, B = inputs.phi_pair(300, 520, 270, 0.5, seed=74)
    with pytest.raises(oz.OzimmuError):
        oz.dgemm_variant(dev(A), dev(B), 8, "per_slice", "per_pair", workspace=small)
