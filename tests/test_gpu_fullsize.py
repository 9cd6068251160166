"""GPU parity at the benchmark's full sizes, in the launch configuration
bench.py times (ozimmu_dgemm, fused epilogue): sampled rows/columns of D are
recomputed by the oracle, which needs only those rows of A and columns of B."""
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


FULL = [
    (4096, 4096, 4096, 0.0, [3, 8, 12]),          # Section 4.3 workload (throughput against accuracy, phi = 0)
    (8192, 8192, 8192, 0.5, [6, 8, 10]),          # config 3
    (16384, 16384, 16384, 0.5, [8, 12, 14]),      # config 4 (headline)
    (16384, 16384, 16384, 4.0, [8, 12, 14]),      # config 4, wide exponent range
    (4096, 65536, 4096, 1.0, [10]),               # config 5: r = 2, 30 chunks
]


@pytest.mark.parametrize("m,n,p,phi,ks", FULL)
def test_full_size_sampled_entries(oz, m, n, p, phi, ks):
    A, B = inputs.phi_pair(m, n, p, phi, seed=0)
    dA = torch.from_numpy(A).cuda()
    dB = torch.from_numpy(B).cuda()
    # one row in every band of 256 rows and one column in every band of 256 columns (every tile row and
    # tile column of the kernel's 256 x 256 output tiles), plus the first and last row / column
    I = inputs.band_indices(m, 256, seed=1)
    J = inputs.band_indices(p, 256, seed=2)
    D = torch.empty((m, p), dtype=torch.float64, device="cuda")
    native = torch.mm(dA, dB)
    bound = torch.mm(dA.abs(), dB.abs())          # |A||B|: the scale of the error bounds of Section 5
    # unit in the first place of the largest entry of every row of A / column of B (g and f of Section 5)
    g = torch.ldexp(torch.ones(m, dtype=torch.float64, device="cuda"), torch.frexp(dA.abs().amax(1))[1] - 1)
    f = torch.ldexp(torch.ones(p, dtype=torch.float64, device="cuda"), torch.frexp(dB.abs().amax(0))[1] - 1)
    beta, _ = oracle.params(n)
    for k in ks:
        D.fill_(float("nan"))                     # a tile the kernel never wrote would stay NaN
        print(f"full-size case m={m} n={n} p={p} k={k}", flush=True)
        ws = oz.alloc_workspace(m, n, p, k)
        oz.dgemm(dA, dB, k, D=D, workspace=ws)
        got = D[torch.from_numpy(I).cuda()][:, torch.from_numpy(J).cuda()].cpu().numpy()
        want = oracle.dgemm_sub(A, B, k, I, J)
        sp = np.spacing(np.abs(want))
        assert np.isfinite(got).all()
        assert (np.abs(got - want) <= 2 * sp).all()
        assert np.array_equal(got, want)
        # properties that hold at any size: every entry of D was written, and every entry agrees with the
        # native FP64 product within the truncation bound of Section 5.2, 4 (k+1) n 2^(-beta k) g f^T, plus
        # the rounding of both products (catches a tile computed from wrong operands)
        assert torch.isfinite(D).all()
        trunc = 4.0 * (k + 1) * n * 2.0 ** (-beta * k) * torch.outer(g, f)
        assert bool(((D - native).abs() <= trunc + 1e-11 * bound).all())
        del ws
