"""GPU parity: the HIP path (through the C ABI) against the CPU oracle on the
same seeded inputs.  Integer results (exponents, INT8 slices, INT32 products)
must match bit for bit; D must lie within 2 ulp of the oracle's D (the target
stated for this build; bit equality is what the arithmetic predicts, because
both sides perform the same single rounded FP64 addition per chunk)."""
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


def ulp_distance(got, want):
    """|got - want| in units of ulp(want) (spacing of FP64 at want)."""
    want = np.asarray(want, dtype=np.float64)
    sp = np.spacing(np.abs(want))
    return np.abs(np.asarray(got) - want) / sp


def assert_within_2ulp(got, want):
    assert np.isfinite(got).all()
    d = ulp_distance(got, want)
    assert d.max() <= 2.0, f"max ulp distance {d.max()}"


def special_matrix():
    rows = [
        [1.0, -0.7, 0.3, 1.2345 * 2.0 ** -10, 0.0, 2.5 / 64, 3.5 / 64, -2.5 / 64],
        [0.0] * 8,
        [3.0, -3.0, 1.5, 0.75, 2.0 ** -60, -2.0 ** -61, 1e-300, 2.9999999999999996],
        [2.0 ** -1070, -2.0 ** -1074, 3 * 2.0 ** -1074, 0.0, 2.0 ** -1072, 0, 0, 0],
        [2.0 ** 900, -1.0, 2.0 ** 899 + 2.0 ** 860, 5e269, -2.0 ** 900, 1e-5, 0, 7.0],
        [-5.0, 4.999999999999999, 0.5 + 2.0 ** -53, 0.5 - 2.0 ** -54, 1 / 3, -2 / 3, 0.1, 6.5],
        [2.0 ** -7 * 1.5, 2.0 ** -7 * 0.5, 2.0 ** -14 * 0.5, 2.0 ** -14 * 1.5, 1.0, 0, 0, 0],
    ]
    return np.array(rows, dtype=np.float64)


# --------------------------------------------------------------------------- split
SPLIT_CASES = [(256, 256, 0.5, 8, 0), (300, 200, 4.0, 14, 1), (1, 5, 1.0, 3, 2), (513, 1000, 2.0, 9, 3),
               (64, 1029, 0.5, 20, 4), (5, 2 ** 17 + 5, 1.0, 4, 5),
               # the three row-split kernels of A: row in registers (<= 4096, <= 16384 padded), two passes beyond
               (20, 4096, 1.0, 5, 6), (40, 4097, 1.0, 6, 7), (33, 16384, 0.5, 8, 8), (9, 16385, 2.0, 5, 9)]


@pytest.mark.parametrize("rows,n,phi,k,seed", SPLIT_CASES)
def test_split_A_bit_exact(oz, rows, n, phi, k, seed):
    A, _ = inputs.phi_pair(rows, n, 1, phi, seed=seed)
    beta, _ = oracle.params(n)
    want, e_want = oracle.split_rows(A, k, beta)
    SA, eA = oz.split_A(dev(A), k)
    got = oz.export_slices(rows, n, k, SA).cpu().numpy()
    assert np.array_equal(eA.cpu().numpy(), e_want)
    assert np.array_equal(got, want)


@pytest.mark.parametrize("cols,n,phi,k,seed", SPLIT_CASES)
def test_split_B_bit_exact(oz, cols, n, phi, k, seed):
    _, B = inputs.phi_pair(1, n, cols, phi, seed=seed)
    beta, _ = oracle.params(n)
    want, e_want = oracle.split_cols(B, k, beta)              # [k][n][p]
    SB, eB = oz.split_B(dev(B), k)
    got = oz.export_slices(cols, n, k, SB).cpu().numpy()      # [k][p][n]
    assert np.array_equal(eB.cpu().numpy(), e_want)
    assert np.array_equal(got.transpose(0, 2, 1), want)


def test_split_special_values_and_strided_inputs(oz):
    X = special_matrix()
    k = 16
    beta, _ = oracle.params(X.shape[1])
    want, e_want = oracle.split_rows(X, k, beta)
    # odd leading dimension and an unaligned base pointer (scalar-load path)
    big = torch.zeros((X.shape[0], 11), dtype=torch.float64, device="cuda")
    view = big[:, 1:9]
    view.copy_(dev(X))
    SA, eA = oz.split_A(view, k)
    assert np.array_equal(eA.cpu().numpy(), e_want)
    assert np.array_equal(oz.export_slices(X.shape[0], X.shape[1], k, SA).cpu().numpy(), want)
    # the same numbers as columns of B
    Bt = np.ascontiguousarray(X.T)
    beta_b, _ = oracle.params(Bt.shape[0])
    want_b, eb_want = oracle.split_cols(Bt, k, beta_b)
    bigb = torch.zeros((Bt.shape[0], 13), dtype=torch.float64, device="cuda")
    vb = bigb[:, 3:3 + Bt.shape[1]]
    vb.copy_(dev(Bt))
    SB, eB = oz.split_B(vb, k)
    assert np.array_equal(eB.cpu().numpy(), eb_want)
    assert np.array_equal(oz.export_slices(Bt.shape[1], Bt.shape[0], k, SB).cpu().numpy().transpose(0, 2, 1), want_b)


# --------------------------------------------------------------------------- integer products
def test_all_pair_products_bit_exact_config1(oz):
    # m = n = p = 256, phi = 0.5, seed 0, k = 8: all 36 kept pairs
    m = n = p = 256
    k = 8
    A, B = inputs.phi_pair(m, n, p, 0.5, seed=0)
    beta, r = oracle.params(n)
    SAo, _ = oracle.split_rows(A, k, beta)
    SBo, _ = oracle.split_cols(B, k, beta)
    SA, _ = oz.split_A(dev(A), k)
    SB, _ = oz.split_B(dev(B), k)
    count = 0
    for s in range(1, k + 1):
        for t in range(1, k + 2 - s):
            C = oz.gemm_group(m, n, p, SA, k, SB, k, s + t, s, s).cpu().numpy()
            assert np.array_equal(C, oracle.pair_product(SAo, SBo, s, t)), (s, t)
            count += 1
    assert count == 36


@pytest.mark.parametrize("m,n,p,k,chunks", [
    (300, 520, 270, 6, [(2, 1, 1), (7, 1, 6), (7, 2, 4), (5, 4, 4)]),
    (257, 129, 513, 4, [(5, 1, 4), (3, 2, 2)]),
    (33, 4000, 17, 9, [(10, 1, 9), (10, 3, 7)]),
])
def test_group_chunks_bit_exact_ragged(oz, m, n, p, k, chunks):
    A, B = inputs.phi_pair(m, n, p, 1.0, seed=17)
    beta, _ = oracle.params(n)
    SAo, _ = oracle.split_rows(A, k, beta)
    SBo, _ = oracle.split_cols(B, k, beta)
    SA, _ = oz.split_A(dev(A), k)
    SB, _ = oz.split_B(dev(B), k)
    for (g, s0, s1) in chunks:
        # leading dimension larger than p, and a poisoned buffer to catch out-of-range stores
        buf = torch.full((m + 1, p + 3), -7, dtype=torch.int32, device="cuda")
        oz.gemm_group(m, n, p, SA, k, SB, k, g, s0, s1, C=buf[:m, :p])
        got = buf.cpu().numpy()
        assert np.array_equal(got[:m, :p], oracle.group_chunk(SAo, SBo, g, s0, s1)), (g, s0, s1)
        assert (got[m:, :] == -7).all() and (got[:, p:] == -7).all()


def test_extreme_slice_values_long_inner_dimension(oz):
    # a_ij = 1 = 2^eA gives q_1 = +64 (the largest slice magnitude), b_ij = -1 gives -64;
    # with n = 16384 the pair product is -64 * 64 * n = -2^26 in every entry.
    n, k = 16384, 8
    A = np.full((3, n), 1.0)
    B = np.full((n, 2), -1.0)
    SA, eA = oz.split_A(dev(A), k)
    SB, eB = oz.split_B(dev(B), k)
    C = oz.gemm_group(3, n, 2, SA, k, SB, k, 2, 1, 1).cpu().numpy()
    assert (C == -64 * 64 * n).all()
    assert not oz.gemm_group(3, n, 2, SA, k, SB, k, 3, 1, 2).cpu().numpy().any()


@pytest.mark.parametrize("n,k", [(16384, 8), (2 ** 17 + 128, 6), (2 ** 17, 5)])
def test_near_maximal_slices_everywhere_stay_inside_int32(oz, n, k):
    # every entry is the same x = 2^e (h - 1/2 - 2^-20) / h, h = 2^(beta-1): its first slice is h - 1, its second
    # h (the largest magnitudes), in every row and column, so every chunk sum is as large as the data can make
    # it; with the sign pattern below the products keep one sign along the whole inner dimension.  Pair
    # products, chunk sums over r pairs and D must still be the oracle's.
    beta, r = oracle.params(n)
    h = 2.0 ** (beta - 1)
    x = (h - 0.5 - 2.0 ** -20) / h
    m, p = 5, 3
    A = np.full((m, n), x)
    B = np.full((n, p), x)
    A[1] = -x                      # a row of the other sign
    B[:, 2] = -x
    SAo, _ = oracle.split_rows(A, k, beta)
    SBo, _ = oracle.split_cols(B, k, beta)
    assert SAo[0].max() == h - 1 and SAo[1].max() == h
    SA, eA = oz.split_A(dev(A), k)
    SB, eB = oz.split_B(dev(B), k)
    assert np.array_equal(oz.export_slices(m, n, k, SA).cpu().numpy(), SAo)
    assert np.array_equal(oz.export_slices(p, n, k, SB).cpu().numpy().transpose(0, 2, 1), SBo)
    for (g, s0, s1) in [(2, 1, 1), (4, 2, 2), (3, 1, min(2, r)), (k + 1, 1, min(k, r))]:
        C = oz.gemm_group(m, n, p, SA, k, SB, k, g, s0, s1).cpu().numpy()
        assert np.array_equal(C, oracle.group_chunk(SAo, SBo, g, s0, s1)), (g, s0, s1)
    assert np.array_equal(oz.dgemm(dev(A), dev(B), k).cpu().numpy(), oracle.dgemm(A, B, k))


# --------------------------------------------------------------------------- accumulation
def test_accumulate_matches_oracle_bit_exact(oz):
    rng = np.random.Generator(np.random.PCG64(3))
    m, p, beta, g = 70, 300, 7, 5
    C = rng.integers(-2 ** 31, 2 ** 31, size=(m, p)).astype(np.int32)
    eA = rng.integers(-30, 30, size=m).astype(np.int32)
    eB = rng.integers(-30, 30, size=p).astype(np.int32)
    D0 = rng.standard_normal((m, p)) * 2.0 ** rng.integers(-20, 20, size=(m, p))
    for first in (True, False):
        want = D0.copy()
        oracle.accumulate(want, C, eA, eB, beta, g, first)
        D = dev(D0.copy())
        oz.accumulate(dev(C), dev(eA), dev(eB), beta, g, first, D)
        assert np.array_equal(D.cpu().numpy(), want)


# --------------------------------------------------------------------------- whole path
DGEMM_CASES = [
    (256, 256, 256, 8, 0.5, 0),        # config 1
    (300, 520, 270, 10, 2.0, 1),       # ragged in every dimension, several tiles
    (1, 1, 1, 1, 0.5, 2),
    (2, 3, 5, 20, 4.0, 3),
    (513, 129, 257, 3, 1.0, 4),
    (1024, 1024, 1024, 6, 2.0, 5),     # config 2 (ends of the k sweep)
    (1024, 1024, 1024, 12, 0.5, 6),
    (260, 65536, 130, 5, 1.0, 7),      # r = 2: several chunks per group
    (64, 2 ** 17 + 128, 40, 4, 0.5, 8),  # beta = 6
]


@pytest.mark.parametrize("m,n,p,k,phi,seed", DGEMM_CASES)
def test_dgemm_within_2ulp_of_oracle(oz, m, n, p, k, phi, seed):
    A, B = inputs.phi_pair(m, n, p, phi, seed=seed)
    want = oracle.dgemm(A, B, k)
    D = torch.full((m, p), float("nan"), dtype=torch.float64, device="cuda")
    oz.dgemm(dev(A), dev(B), k, D=D)
    got = D.cpu().numpy()
    assert_within_2ulp(got, want)
    assert np.array_equal(got, want), "expected bit equality (same single rounding per chunk)"


# config 2: m = n = p = 1024, phi in {0.5, 1, 2}, k = 6 .. 12 (Section 4.1 workload).  The ends of the sweep are
# compared in full above; here every (phi, k) on rows / columns sampled from every band of 128
@pytest.mark.parametrize("phi", [0.5, 1.0, 2.0])
def test_dgemm_config2_sweep_sampled(oz, phi):
    m = n = p = 1024
    A, B = inputs.phi_pair(m, n, p, phi, seed=0)
    dA, dB = dev(A), dev(B)
    I = inputs.band_indices(m, 128, seed=21)
    J = inputs.band_indices(p, 128, seed=22)
    tI, tJ = torch.from_numpy(I).cuda(), torch.from_numpy(J).cuda()
    for k in range(6, 13):
        D = torch.full((m, p), float("nan"), dtype=torch.float64, device="cuda")
        oz.dgemm(dA, dB, k, D=D)
        assert torch.isfinite(D).all()
        got = D[tI][:, tJ].cpu().numpy()
        want = oracle.dgemm_sub(A, B, k, I, J)
        assert_within_2ulp(got, want)
        assert np.array_equal(got, want), (phi, k)


def test_dgemm_exact_on_small_integers_and_edge_shapes(oz):
    A, B = inputs.small_int_pair(130, 300, 70, 64, seed=4)
    want = (A.astype(np.int64) @ B.astype(np.int64)).astype(np.float64)
    for k in (1, 4):
        assert np.array_equal(oz.dgemm(dev(A), dev(B), k).cpu().numpy(), want)
    # n == 0: D = +0; m == 0 / p == 0: nothing to do
    D = torch.full((4, 6), float("nan"), dtype=torch.float64, device="cuda")
    oz.dgemm(torch.empty((4, 0), dtype=torch.float64, device="cuda"),
             torch.empty((0, 6), dtype=torch.float64, device="cuda"), 8, D=D)
    assert (D == 0).all() and not torch.signbit(D).any()
    out = oz.dgemm(torch.empty((0, 5), dtype=torch.float64, device="cuda"), dev(np.ones((5, 3))), 8)
    assert out.shape == (0, 3)
    # zero rows / columns inside a matrix
    A[3, :] = 0.0
    B[:, 5] = 0.0
    got = oz.dgemm(dev(A), dev(B), 3).cpu().numpy()
    assert np.array_equal(got, (A.astype(np.int64) @ B.astype(np.int64)).astype(np.float64))
    assert not np.signbit(got[3]).any()


def test_dgemm_strided_operands_and_reused_workspace(oz):
    m, n, p, k = 200, 333, 150, 7
    A, B = inputs.phi_pair(m, n, p, 1.0, seed=12)
    want = oracle.dgemm(A, B, k)
    Abig = torch.zeros((m, n + 5), dtype=torch.float64, device="cuda")
    Bbig = torch.zeros((n, p + 7), dtype=torch.float64, device="cuda")
    Dbig = torch.full((m, p + 2), -1.0, dtype=torch.float64, device="cuda")
    Abig[:, 2:2 + n] = dev(A)
    Bbig[:, 1:1 + p] = dev(B)
    ws = oz.alloc_workspace(m, n, p, k)
    ws.fill_(0x5A)                      # stale bytes in the workspace must not leak into the result
    for _ in range(2):
        oz.dgemm(Abig[:, 2:2 + n], Bbig[:, 1:1 + p], k, D=Dbig[:, :p], workspace=ws)
    got = Dbig.cpu().numpy()
    assert np.array_equal(got[:, :p], want)
    assert (got[:, p:] == -1.0).all()


def test_fused_and_phase_paths_agree(oz):
    m, n, p, k = 300, 700, 280, 6
    A, B = inputs.phi_pair(m, n, p, 0.5, seed=13)
    beta, r = oz.params(n)
    assert (beta, r) == oracle.params(n)
    SA, eA = oz.split_A(dev(A), k)
    SB, eB = oz.split_B(dev(B), k)
    D1 = torch.empty((m, p), dtype=torch.float64, device="cuda")
    D2 = torch.empty((m, p), dtype=torch.float64, device="cuda")
    first = True
    sched = oracle.chunks(k, r)
    assert len(sched) == oz.num_chunks(n, k)
    for (g, s0, s1) in sched:
        C = oz.gemm_group(m, n, p, SA, k, SB, k, g, s0, s1)
        oz.accumulate(C, eA, eB, beta, g, first, D1)
        oz.gemm_group_accumulate(m, n, p, SA, k, SB, k, g, s0, s1, eA, eB, first, D2)
        first = False
    want = oracle.dgemm(A, B, k)
    assert np.array_equal(D1.cpu().numpy(), want)
    assert np.array_equal(D2.cpu().numpy(), want)


def test_argument_errors_are_reported(oz):
    A = torch.zeros((4, 4), dtype=torch.float64, device="cuda")
    with pytest.raises(oz.OzimmuError):
        oz.dgemm(A, A, 0)
    with pytest.raises(oz.OzimmuError):
        oz.dgemm(A, A, 21)
    with pytest.raises(oz.OzimmuError):
        oz.dgemm(A, A, 8, workspace=torch.empty(256, dtype=torch.uint8, device="cuda"))


def test_dgemm_captured_in_a_hip_graph_replays_bit_identically(oz):
    # the call enqueues kernels only (counters are cleared by a fill kernel, not a memset), so it can be
    # captured; every replay must reproduce the eager result, also after eager work in between
    m, n, p, k = 300, 520, 270, 8
    A, B = inputs.phi_pair(m, n, p, 0.5, seed=41)
    dA, dB = torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda()
    ws = oz.alloc_workspace(m, n, p, k)
    eager = oz.dgemm(dA, dB, k, workspace=ws).clone()     # also the warm-up that sets the kernel attributes
    D = torch.zeros((m, p), dtype=torch.float64, device="cuda")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        oz.dgemm(dA, dB, k, D=D, workspace=ws)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        oz.dgemm(dA, dB, k, D=D, workspace=ws)
    for rep in range(4):
        D.fill_(float(rep))                                # eager work between the replays
        other = oz.dgemm(dB.T.contiguous(), dA.T.contiguous(), k) if rep == 2 else None   # its own workspace
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(D, eager), f"replay {rep}"
        del other
    want = oracle.dgemm(A, B, k)
    assert (np.abs(eager.cpu().numpy() - want) <= 2 * np.spacing(np.abs(want))).all()


def test_queue_schedule_captured_in_a_hip_graph_replays_bit_identically(oz):
    # 320 tiles: the default schedule is the queue (its counters are cleared by a fill kernel, its waits are
    # bounded); every replay must reproduce the eager result
    m, n, p, k = 4096, 300, 5120, 4
    A, B = inputs.phi_pair(m, n, p, 0.5, seed=43)
    dA, dB = torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda()
    ws = oz.alloc_workspace(m, n, p, k)
    eager = oz.dgemm(dA, dB, k, workspace=ws).clone()
    assert torch.equal(eager, oz.dgemm_variant(dA, dB, k, "rn", "grouped", schedule="one_launch"))
    D = torch.zeros((m, p), dtype=torch.float64, device="cuda")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        oz.dgemm(dA, dB, k, D=D, workspace=ws)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        oz.dgemm(dA, dB, k, D=D, workspace=ws)
    for rep in range(3):
        D.fill_(float(rep))
        ws[-(1 << 20):].fill_(0x33)                        # stale counters behind the blocks
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(D, eager), f"replay {rep}"


def test_first_library_call_of_a_process_inside_a_graph_capture_after_init(oz):
    # the per-device set-up (kernel attributes, symbol address) is not legal inside a stream capture: a process whose
    # very first library call is a captured one must call ozimmu_init before.  Run in a child process, so that the
    # library is really fresh there.
    import subprocess
    import sys
    code = r"""
import sys
import numpy as np
import torch
sys.path.insert(0, %r)
from paper_2409_13313_amd import inputs, ozimmu
m, n, p, k = 300, 520, 270, 6
A, B = inputs.phi_pair(m, n, p, 0.5, seed=43)
dA, dB = torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda()
ws = ozimmu.alloc_workspace(m, n, p, k)
D = torch.zeros((m, p), dtype=torch.float64, device="cuda")
ozimmu.init()                                  # the only library call before the capture
side = torch.cuda.Stream()
side.wait_stream(torch.cuda.current_stream())
torch.cuda.synchronize()
graph = torch.cuda.CUDAGraph()
with torch.cuda.graph(graph):
    ozimmu.dgemm(dA, dB, k, D=D, workspace=ws)
outs = []
for rep in range(3):
    D.fill_(float(rep))
    torch.cuda.synchronize()
    graph.replay()
    torch.cuda.synchronize()
    outs.append(D.clone())
eager = ozimmu.dgemm(dA, dB, k)
torch.cuda.synchronize()
assert all(torch.equal(o, eager) for o in outs)
import oracle
assert np.array_equal(eager.cpu().numpy(), oracle.dgemm(A, B, k))
print("CAPTURE_OK")
""" % (str(__import__("os").path.dirname(__import__("os").path.dirname(__import__("os").path.abspath(__file__)))),)
    pr = subprocess.run([sys.executable, "-c", code], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True,
                        timeout=240)
    assert pr.returncode == 0 and "CAPTURE_OK" in pr.stdout, pr.stdout[-3000:]

