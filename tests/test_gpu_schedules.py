"""GPU parity of the ways the schedule is run: one persistent launch with the fused epilogue; the split-inner
way for tiles too few to fill the chip (per chunk: partial INT32 sums by integer atomics + accumulation kernel);
the chunk-parallel way for outputs of few tiles (all chunks in one launch, each with INT32 blocks of its own,
then one kernel that adds them in the order of Algorithm 6).  All must give the oracle's D bit for bit."""
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


def queue_workspace(oz, m, n, p, k, sets=3):
    """A workspace with room for the blocks of the queue schedule whatever the size (the recommended size holds
    them only for outputs of more than 256 tiles): `sets` sets of chunks x min(tiles, 256) blocks + counters."""
    tiles = -(-m // 256) * -(-p // 256)
    blocks = sets * oz.num_chunks(n, k) * min(tiles, 256) + 2
    return torch.empty(oz.workspace_bytes_min(m, n, p, k) + blocks * 4 * 256 * 256, dtype=torch.uint8, device="cuda")


SHAPES = [
    (300, 520, 270, 8, 0.5),       # 4 tiles, 12 inner tiles: 3 parts
    (513, 1029, 257, 6, 2.0),      # 6 ragged tiles, 20 inner tiles: 5 parts
    (130, 65536, 70, 5, 1.0),      # 1 tile, r = 2, 16 parts, parts that start inside a slice pair
    (1024, 1024, 1024, 12, 0.5),   # 16 tiles, 4 parts, chunks of up to 12 pairs
    (256, 256, 256, 8, 0.5),       # one group of stages per pair: nothing to cut, falls back to one launch
    (40, 2 ** 17 + 128, 64, 4, 0.5),   # beta = 6
    (1536, 512, 1792, 8, 0.5),     # 42 tiles x 8 chunks: more work items than workgroups in the chunk-parallel launch
]


@pytest.mark.parametrize("schedule", ["one_launch", "split_inner", "chunk_parallel", "queue", "auto"])
@pytest.mark.parametrize("m,n,p,k,phi", SHAPES)
def test_both_schedules_match_the_oracle_bit_for_bit(oz, m, n, p, k, phi, schedule):
    A, B = inputs.phi_pair(m, n, p, phi, seed=91)
    want = oracle.dgemm(A, B, k)
    D = torch.full((m, p), float("nan"), dtype=torch.float64, device="cuda")
    ws = queue_workspace(oz, m, n, p, k) if schedule == "queue" else None
    oz.dgemm_variant(dev(A), dev(B), k, "rn", "grouped", D=D, workspace=ws, schedule=schedule)
    got = D.cpu().numpy()
    assert np.isfinite(got).all()
    assert (np.abs(got - want) <= 2 * np.spacing(np.abs(want))).all()
    assert np.array_equal(got, want)


@pytest.mark.parametrize("split,accumulate", [("bitmask", "grouped"), ("bitmask", "per_pair"), ("rn", "wide")])
def test_split_inner_schedule_with_the_comparison_variants(oz, split, accumulate):
    m, n, p, k = 300, 2000, 270, 9
    A, B = inputs.phi_pair(m, n, p, 2.0, seed=92)
    want = oracle.dgemm_variant(A, B, k, split, accumulate)
    got = oz.dgemm_variant(dev(A), dev(B), k, split, accumulate, schedule="split_inner").cpu().numpy()
    assert np.array_equal(got, want)


def test_split_inner_with_strided_output_and_reused_workspace(oz):
    m, n, p, k = 200, 3000, 150, 7
    A, B = inputs.phi_pair(m, n, p, 1.0, seed=93)
    want = oracle.dgemm(A, B, k)
    Dbig = torch.full((m, p + 3), -1.0, dtype=torch.float64, device="cuda")
    ws = oz.alloc_workspace(m, n, p, k)
    ws.fill_(0x5A)                       # stale bytes (also in the partial-sum buffer) must not leak
    for _ in range(2):
        oz.dgemm_variant(dev(A), dev(B), k, "rn", "grouped", D=Dbig[:, :p], workspace=ws, schedule="split_inner")
    got = Dbig.cpu().numpy()
    assert np.array_equal(got[:, :p], want) and (got[:, p:] == -1.0).all()


@pytest.mark.parametrize("split,accumulate", [("bitmask", "grouped"), ("bitmask", "per_pair"), ("rn", "wide"),
                                              ("rn", "per_pair")])
def test_chunk_parallel_schedule_with_the_comparison_variants(oz, split, accumulate):
    m, n, p, k = 300, 2000, 270, 9
    A, B = inputs.phi_pair(m, n, p, 2.0, seed=94)
    want = oracle.dgemm_variant(A, B, k, split, accumulate)
    got = oz.dgemm_variant(dev(A), dev(B), k, split, accumulate, schedule="chunk_parallel").cpu().numpy()
    assert np.array_equal(got, want)


def test_chunk_parallel_with_strided_output_reused_workspace_and_step_v(oz):
    m, n, p, k = 700, 1100, 300, 7
    A, B = inputs.phi_pair(m, n, p, 1.0, seed=95)
    want = oracle.dgemm(A, B, k)
    Dbig = torch.full((m, p + 3), -1.0, dtype=torch.float64, device="cuda")
    ws = oz.alloc_workspace(m, n, p, k)
    ws.fill_(0x5A)                       # stale bytes in the blocks must not leak
    for _ in range(2):
        oz.dgemm_variant(dev(A), dev(B), k, "rn", "grouped", D=Dbig[:, :p], workspace=ws, schedule="chunk_parallel")
    got = Dbig.cpu().numpy()
    assert np.array_equal(got[:, :p], want) and (got[:, p:] == -1.0).all()
    # the GEMM-routine form takes the same way by default at this size: step (v) in the accumulation kernel
    C0 = np.random.Generator(np.random.PCG64(96)).standard_normal((m, p))
    for alpha, beta in ((-1.5, 0.0), (0.75, -0.25)):
        C = dev(C0)
        oz.gemm_ex(False, False, alpha, dev(A), dev(B), beta, C, k)
        assert np.array_equal(C.cpu().numpy(), oracle.gemm_ex(False, False, alpha, A, B, beta, C0, k))


def test_small_workspace_falls_back_to_the_other_schedules(oz):
    # a workspace without room for the chunk-parallel blocks (the least one, or the library's static array)
    # gives the same D through the other schedules; the requirement is not monotone in k, the least one is
    m, n, p, k = 1024, 1024, 1024, 20
    assert oz.workspace_bytes(m, n, p, k) > oz.STATIC_WORKSPACE_BYTES >= oz.workspace_bytes_min(m, n, p, k)
    # (inner dimension 65536: chunks of two pairs; the 30 chunks of k = 10 fit the queue's sets of blocks, the 36 of
    # k = 11 would need more than 2 GiB per set and fall back to the persistent launch)
    assert oz.workspace_bytes(8192, 65536, 8192, 10) > oz.workspace_bytes(8192, 65536, 8192, 11)
    assert oz.workspace_bytes_min(8192, 65536, 8192, 10) < oz.workspace_bytes_min(8192, 65536, 8192, 11)
    A, B = inputs.phi_pair(m, n, p, 0.5, seed=97)
    dA, dB = dev(A), dev(B)
    want = oz.dgemm(dA, dB, k)
    D = torch.empty((m, p), dtype=torch.float64, device="cuda")
    oz.dgemm_static(dA, dB, k, D)
    assert torch.equal(D, want)
    least = torch.empty(oz.workspace_bytes_min(m, n, p, k), dtype=torch.uint8, device="cuda")
    assert torch.equal(oz.dgemm(dA, dB, k, workspace=least), want)
    with pytest.raises(oz.OzimmuError):
        oz.dgemm(dA, dB, k, workspace=least[:-256])


def test_schedule_flags_are_validated(oz):
    A = torch.zeros((4, 4), dtype=torch.float64, device="cuda")
    ws = oz.alloc_workspace(4, 4, 4, 4)
    st = torch.cuda.current_stream().cuda_stream
    D = torch.empty((4, 4), dtype=torch.float64, device="cuda")
    for bad in (0x300, 0x1000, 0x500, 0xc00, 0x103 | 0x200):
        rc = oz._lib.ozimmu_dgemm_variant(4, 4, 4, A.data_ptr(), 4, A.data_ptr(), 4, D.data_ptr(), 4, 4, 0, bad,
                                          ws.data_ptr(), ws.numel(), st)
        assert rc == -3


@pytest.mark.parametrize("m,n,p,k", [(4352, 520, 4096, 4),     # 272 tiles: one round of 256 + 16 in the tail
                                     (4100, 1029, 4000, 3),    # the tail is the ragged last band (4 rows)
                                     (4352, 300, 4352, 5),     # 289 tiles: tail of 33
                                     (3000, 700, 3300, 4)])    # 156 ragged tiles: too many to cut, one launch whatever is asked
def test_last_partial_round_cut_along_the_inner_dimension(oz, m, n, p, k):
    A, B = inputs.phi_pair(m, n, p, 1.0, seed=94)
    dA, dB = dev(A), dev(B)
    out = {}
    for schedule in ("one_launch", "split_inner", "chunk_parallel", "auto"):
        D = torch.full((m, p), float("nan"), dtype=torch.float64, device="cuda")
        oz.dgemm_variant(dA, dB, k, "rn", "grouped", D=D, schedule=schedule)
        assert torch.isfinite(D).all(), schedule          # every tile written, by one path or the other
        out[schedule] = D
    assert torch.equal(out["one_launch"], out["split_inner"])
    assert torch.equal(out["one_launch"], out["chunk_parallel"])
    assert torch.equal(out["one_launch"], out["auto"])
    I = inputs.sample_indices(m, 48, seed=1)
    J = inputs.sample_indices(p, 48, seed=2)
    want = oracle.dgemm_sub(A, B, k, I, J)
    got = out["split_inner"][torch.from_numpy(I).cuda()][:, torch.from_numpy(J).cuda()].cpu().numpy()
    assert np.array_equal(got, want)


@pytest.mark.parametrize("col_shift,extra", [(0, 0), (0, 1), (1, 2)])
def test_fused_epilogue_with_and_without_the_alignment_for_staging(oz, col_shift, extra):
    # 600 x 600: four tiles wholly inside D (their later chunks fetch the old D through LDS when D is 16-byte
    # aligned with an even leading dimension) and five edge tiles (always the plain loads).  An odd leading
    # dimension or a base shifted by one element switches the staging off; the bits must not change.
    m, n, p, k = 600, 300, 600, 6
    A, B = inputs.phi_pair(m, n, p, 1.0, seed=97)
    want = oracle.dgemm(A, B, k)
    Dbig = torch.full((m, p + col_shift + extra), -7.0, dtype=torch.float64, device="cuda")
    view = Dbig[:, col_shift:col_shift + p]
    oz.dgemm_variant(dev(A), dev(B), k, "rn", "grouped", D=view, schedule="one_launch")
    got = Dbig.cpu().numpy()
    assert np.array_equal(got[:, col_shift:col_shift + p], want)
    assert (got[:, :col_shift] == -7.0).all() and (got[:, col_shift + p:] == -7.0).all()


@pytest.mark.parametrize("m,n,p,k,sets", [(4608, 300, 4352, 5, 3),    # 306 tiles: two rounds, the second partly filled
                                          (8192, 256, 8192, 4, 3),    # 1024 tiles: four rounds on three sets of blocks
                                          (8192, 256, 8192, 4, 2),    # the same on two sets (the least that is accepted)
                                          (4100, 1029, 4000, 3, 3),   # ragged edge tiles
                                          (2304, 40000, 2300, 9, 3)]) # 81 tiles, r = 4: 18 chunks (three batches of 8)
def test_queue_schedule_matches_the_persistent_launch_and_sampled_oracle_entries(oz, m, n, p, k, sets):
    A, B = inputs.phi_pair(m, n, p, 1.0, seed=98)
    dA, dB = dev(A), dev(B)
    ref = torch.full((m, p), float("nan"), dtype=torch.float64, device="cuda")
    oz.dgemm_variant(dA, dB, k, "rn", "grouped", D=ref, schedule="one_launch")
    ws = queue_workspace(oz, m, n, p, k, sets)
    ws.fill_(0x5A)                       # stale bytes in the blocks and counters must not leak
    # (odd k: an odd leading dimension, D then goes out in 8-byte stores instead of 16-byte ones)
    Dbig = torch.full((m, p + 2 + k % 2), -3.0, dtype=torch.float64, device="cuda")
    for _ in range(2):                   # the second call finds the first one's counters
        oz.dgemm_variant(dA, dB, k, "rn", "grouped", D=Dbig[:, :p], workspace=ws, schedule="queue")
    assert torch.equal(Dbig[:, :p], ref) and bool((Dbig[:, p:] == -3.0).all())
    I = inputs.sample_indices(m, 40, seed=3)
    J = inputs.sample_indices(p, 40, seed=4)
    want = oracle.dgemm_sub(A, B, k, I, J)
    got = ref[torch.from_numpy(I).cuda()][:, torch.from_numpy(J).cuda()].cpu().numpy()
    assert np.array_equal(got, want)


def test_default_schedule_of_a_large_output_is_bit_identical_with_step_v(oz):
    # 1056 tiles: the default is the queue (full rounds) here; step (v) rides on its tile accumulation
    m, n, p, k = 8192, 300, 8448, 4
    A, B = inputs.phi_pair(m, n, p, 0.5, seed=99)
    dA, dB = dev(A), dev(B)
    ref = oz.dgemm_variant(dA, dB, k, "rn", "grouped", schedule="one_launch")
    assert torch.equal(oz.dgemm(dA, dB, k), ref)
    C0 = torch.from_numpy(np.random.Generator(np.random.PCG64(100)).standard_normal((m, p))).cuda()
    for alpha, beta in ((-1.5, 0.0), (0.75, -0.25)):
        C = C0.clone()
        oz.gemm_ex(False, False, alpha, dA, dB, beta, C, k)
        t1 = alpha * ref
        want = t1 if beta == 0.0 else t1 + beta * C0
        assert torch.equal(C, want)


def test_default_schedule_repeated_calls_give_the_same_bits(oz):
    # 592 tiles in three rounds on recycled blocks: every call of a run must reproduce the persistent launch's D
    # (the blocks written by one XCD are read by another; a stale value would show as a difference here)
    m, n, p, k = 4096, 256, 9472, 8
    A, B = inputs.phi_pair(m, n, p, 1.0, seed=101)
    dA, dB = dev(A), dev(B)
    ref = oz.dgemm_variant(dA, dB, k, "rn", "grouped", schedule="one_launch")
    ws = oz.alloc_workspace(m, n, p, k)
    D = torch.empty_like(ref)
    for rep in range(25):
        D.fill_(float("nan"))
        oz.dgemm(dA, dB, k, D=D, workspace=ws)
        assert torch.equal(D, ref), f"call {rep}"


@pytest.mark.parametrize("split,accumulate", [("bitmask", "grouped"), ("rn", "wide"), ("bitmask", "per_pair")])
def test_default_schedule_of_a_large_output_with_the_comparison_variants(oz, split, accumulate):
    # 272 tiles: the queue by default where its blocks fit (one per chunk: per-pair accumulation has 15 of them at
    # k = 5), else the persistent launch; either way the bits of the forced persistent launch and of the oracle
    m, n, p, k = 4096, 300, 4352, 5
    A, B = inputs.phi_pair(m, n, p, 2.0, seed=102)
    dA, dB = dev(A), dev(B)
    ref = oz.dgemm_variant(dA, dB, k, split, accumulate, schedule="one_launch")
    got = oz.dgemm_variant(dA, dB, k, split, accumulate)
    assert torch.equal(got, ref)
    I = inputs.sample_indices(m, 32, seed=5)
    J = inputs.sample_indices(p, 32, seed=6)
    want = oracle.dgemm_variant(A[I], B[:, J], k, split, accumulate)
    assert np.array_equal(got[torch.from_numpy(I).cuda()][:, torch.from_numpy(J).cuda()].cpu().numpy(), want)
