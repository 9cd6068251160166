"""The allocation-free entry point ozimmu_dgemm_static (workspace = a static device array inside the library)
against ozimmu_dgemm with a caller workspace: bit-identical D, on two calls in a row, the second one smaller,
so that whatever the first call left in the shared array must not leak into the second."""
import ctypes

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


def test_static_workspace_entry_point_matches_dgemm_twice_in_a_row(oz):
    oz.init()
    cases = [(700, 1100, 600, 9, 1.0, 71),      # several tiles, ragged, cut tail round possible
             (130, 300, 70, 5, 0.5, 72)]        # smaller: runs on the leftovers of the first call
    for (m, n, p, k, phi, seed) in cases:
        print(f"static-workspace case m={m} n={n} p={p} k={k}", flush=True)
        A, B = inputs.phi_pair(m, n, p, phi, seed=seed)
        dA, dB = torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda()
        want = oz.dgemm(dA, dB, k)
        D = torch.full((m, p), float("nan"), dtype=torch.float64, device="cuda")
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        rc = oz._lib.ozimmu_dgemm_static(m, n, p, dA.data_ptr(), n, dB.data_ptr(), p, D.data_ptr(), p, k,
                                         torch.cuda.current_stream().cuda_stream)
        assert rc == 0
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        assert torch.equal(D, want)
        ref = oracle.dgemm(A, B, k)
        got = D.cpu().numpy()
        assert (np.abs(got - ref) <= 2 * np.spacing(np.abs(ref))).all()
        assert np.array_equal(got, ref)


def test_static_workspace_entry_point_rejects_what_does_not_fit(oz):
    # 4096^3 with k = 8 needs 268 MB of slices alone: more than the 64 MiB the library holds
    assert oz.slices_bytes(4096, 4096, 8) > oz.STATIC_WORKSPACE_BYTES
    fake = 4096   # never dereferenced: the size check comes first
    rc = oz._lib.ozimmu_dgemm_static(4096, 4096, 4096, fake, 4096, fake, 4096, fake, 4096, 8, None)
    assert rc == -4
    assert oz._lib.ozimmu_dgemm_static(-1, 4, 4, fake, 4, fake, 4, fake, 4, 8, None) == -2
    assert oz._lib.ozimmu_dgemm_static(4, 4, 4, fake, 4, fake, 4, fake, 4, 0, None) == -3
