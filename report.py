"""Secondary measurements on one MI355X (the headline number is bench.py's):

  --accuracy   m=n=p=1024, phi in {0.5, 1, 2}, k = 6..12: error of the emulated product against a
               compensated (Dot2) product, next to native FP64 (torch.mm)         [Section 4.1 workload]
  --phases     m=n=p=8192, phi=0.5, k in {6, 8, 10}: time of split A, split B, chunk GEMMs and
               FP64 accumulation run as separate phases, and of the fused call    [Section 4.2 workload]
  --long-inner m=p=4096, n=65536, phi=1, k=10 (r = 2: 30 chunks for 55 products)
  --variants   accuracy (1024^3, phi=2) and time (16384^3; 4096x65536x4096) of the variants of Section 4:
               ozIMMU_H, ozIMMU_EF, ozIMMU, ozIMMU_RN, and the wide-chunk option

  --perf-vs-accuracy  m=n=p=4096, phi=0, k = 3..12: throughput against accuracy for the four methods of
               Section 4 and native FP64                                          [Section 4.3 workload]
  --small-beta m=p=2048, n=2^18 (beta = 6, r = 2) next to n=2^17 (beta = 7, r = 1): the loss of accuracy
               per slice beyond n = 2^17                                          [Section 4.1 remark]

  --sizes      m=n=p in {1024 .. 16384}, k in {4, 8, 12}: time of ozimmu_dgemm against native FP64   [Section 4.2]

  --small      m=n=p in {256, 1024}, k=8: single-call latency (median of 100) next to native FP64, and the time of
               the CPU oracle for the same product run in full

  --schedules  outputs of few tiles: the one-launch schedule against the split-inner one and native FP64

  --breakdown  time shares of split / INT8 GEMMs / FP64 accumulation with the phases run as separate kernels,
               for the accumulation per slice pair (Algorithm 4) and per chunk (Algorithm 6)   [Section 4.2]

Prints markdown tables.  The Dot2 reference comes from the CPU oracle package, which is test
infrastructure; nothing here feeds back into the HIP path.
"""
from __future__ import annotations

import argparse
import os
import sys

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def _median_ms(fn, reps):
    import torch
    times = []
    for _ in range(reps):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        fn()
        e1.record()
        torch.cuda.synchronize()
        times.append(e0.elapsed_time(e1))
    times.sort()
    return times[len(times) // 2]


def accuracy():
    import numpy as np
    import torch
    import oracle
    from paper_2409_13313_amd import inputs, ozimmu
    n = 1024
    print(f"### accuracy, m=n=p={n}: max |D - R| / (|A||B|) over all entries, R = Dot2 product\n")
    print("| phi | " + " | ".join(f"k={k}" for k in range(6, 13)) + " | native FP64 |")
    print("|---|" + "---|" * 8)
    for phi in (0.5, 1.0, 2.0):
        A, B = inputs.phi_pair(n, n, n, phi, seed=0)
        hi, lo = oracle.dot2_gemm(A, B)
        absab = np.abs(A) @ np.abs(B)
        dA, dB = torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda()
        row = []
        for k in range(6, 13):
            D = ozimmu.dgemm(dA, dB, k).cpu().numpy()
            row.append(float((np.abs((D - hi) - lo) / absab).max()))
        nat = torch.mm(dA, dB).cpu().numpy()
        e_nat = float((np.abs((nat - hi) - lo) / absab).max())
        print(f"| {phi} | " + " | ".join(f"{e:.2e}" for e in row) + f" | {e_nat:.2e} |")
    print()


def phases(m, n, p, phi, ks, reps=5):
    import torch
    from paper_2409_13313_amd import inputs, ozimmu
    A, B = inputs.phi_pair(m, n, p, phi, seed=0)
    dA, dB = torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda()
    beta, r = ozimmu.params(n)
    print(f"### phases, m={m} n={n} p={p}, phi={phi} (beta={beta}, r={r}); median of {reps}, ms\n")
    print("| k | products | chunks | split A | split B | chunk GEMMs (INT32 out) | FP64 accumulation (separate) | "
          "fused GEMM+accumulation | ozimmu_dgemm | effective TFLOP/s | INT8 TOP/s of fused phase |")
    print("|---|---|---|---|---|---|---|---|---|---|---|")
    D = torch.empty((m, p), dtype=torch.float64, device="cuda")
    C = torch.empty((m, p), dtype=torch.int32, device="cuda")
    scratch = ozimmu.alloc_scratch()
    for k in ks:
        SA, eA = ozimmu.split_A(dA, k)
        SB, eB = ozimmu.split_B(dB, k)
        ws = ozimmu.alloc_workspace(m, n, p, k)
        sched = [(g, s0, min(s0 + r - 1, g - 1)) for g in range(2, k + 2) for s0 in range(1, g, r)]

        def gemms():
            for (g, s0, s1) in sched:
                ozimmu.gemm_group(m, n, p, SA, k, SB, k, g, s0, s1, C=C, scratch=scratch)

        def accs():
            for i, (g, s0, s1) in enumerate(sched):
                ozimmu.accumulate(C, eA, eB, beta, g, i == 0, D)

        def fused():
            for i, (g, s0, s1) in enumerate(sched):
                ozimmu.gemm_group_accumulate(m, n, p, SA, k, SB, k, g, s0, s1, eA, eB, i == 0, D, scratch=scratch)

        ozimmu.dgemm(dA, dB, k, D=D, workspace=ws)
        torch.cuda.synchronize()
        t_sa = _median_ms(lambda: ozimmu.split_A(dA, k), reps)
        t_sb = _median_ms(lambda: ozimmu.split_B(dB, k), reps)
        t_g = _median_ms(gemms, reps)
        t_a = _median_ms(accs, reps)
        t_f = _median_ms(fused, reps)
        t_all = _median_ms(lambda: ozimmu.dgemm(dA, dB, k, D=D, workspace=ws), reps)
        pairs = k * (k + 1) // 2
        print(f"| {k} | {pairs} | {len(sched)} | {t_sa:.3f} | {t_sb:.3f} | {t_g:.3f} | {t_a:.3f} | {t_f:.3f} | "
              f"{t_all:.3f} | {2.0 * m * n * p / t_all / 1e9:.1f} | {2.0 * m * n * p * pairs / t_f / 1e9:.0f} |")
        del SA, SB, ws
    print()


def variants():
    """Accuracy and time of the variants compared in Section 4, on the same inputs."""
    import numpy as np
    import torch
    import oracle
    from paper_2409_13313_amd import inputs, ozimmu
    combos = [("rn", "grouped", "ozIMMU_H"), ("rn", "wide", "H, wide chunks"), ("bitmask", "grouped", "ozIMMU_EF"),
              ("bitmask", "per_pair", "ozIMMU"), ("per_slice", "per_pair", "ozIMMU_RN"),
              ("rn", "per_pair", "RN split, per pair")]
    n = 1024
    A, B = inputs.phi_pair(n, n, n, 2.0, seed=0)
    hi, lo = oracle.dot2_gemm(A, B)
    absab = np.abs(A) @ np.abs(B)
    dA, dB = torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda()
    print(f"### variants, accuracy at m=n=p={n}, phi=2: max |D - R| / (|A||B|), R = Dot2 product\n")
    print("| variant | " + " | ".join(f"k={k}" for k in range(7, 12)) + " |")
    print("|---|" + "---|" * 5)
    for split, acc, name in combos:
        row = []
        for k in range(7, 12):
            D = ozimmu.dgemm_variant(dA, dB, k, split, acc).cpu().numpy()
            row.append(float((np.abs((D - hi) - lo) / absab).max()))
        print(f"| {name} | " + " | ".join(f"{e:.2e}" for e in row) + " |")
    nat = torch.mm(dA, dB).cpu().numpy()
    print(f"| native FP64 | {float((np.abs((nat - hi) - lo) / absab).max()):.2e} | | | | |\n")
    del dA, dB
    for (m, nn, p, ks) in [(16384, 16384, 16384, [8, 12, 14]), (4096, 65536, 4096, [10])]:
        A, B = inputs.phi_pair(m, nn, p, 0.5, seed=0)
        dA, dB = torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda()
        D = torch.empty((m, p), dtype=torch.float64, device="cuda")
        beta, r = ozimmu.params(nn)
        print(f"### variants, time at m={m} n={nn} p={p} (r={r}, wide r={ozimmu.r_wide(nn)}); median of 3, ms "
              f"(effective TFLOP/s)\n")
        print("| k | " + " | ".join(name for _, _, name in combos) + " |")
        print("|---|" + "---|" * len(combos))
        for k in ks:
            ws = ozimmu.alloc_workspace(m, nn, p, k, split="per_slice")      # the largest of the variants
            cells = []
            for split, acc, name in combos:
                ozimmu.dgemm_variant(dA, dB, k, split, acc, D=D, workspace=ws)
                t = _median_ms(lambda: ozimmu.dgemm_variant(dA, dB, k, split, acc, D=D, workspace=ws), 3)
                cells.append(f"{t:.2f} ({2.0 * m * nn * p / t / 1e9:.1f})")
            print(f"| {k} | " + " | ".join(cells) + " |")
            del ws
        print()
        del dA, dB, D


def _sampled_errors(D, A, B, I, J, hi, lo, absab):
    """(max |D-R|/|R|, max |D-R|/(|A||B|)) over the sampled entries D[I][:, J]; R = hi + lo (Dot2)."""
    import numpy as np
    got = D[I][:, J].cpu().numpy()
    diff = np.abs((got - hi) - lo)
    return float((diff / np.abs(hi)).max()), float((diff / absab).max())


def perf_vs_accuracy(n=4096, phi=0.0, sample=256, reps=5):
    import numpy as np
    import torch
    import oracle
    from paper_2409_13313_amd import inputs, ozimmu
    methods = [("rn", "grouped", "ozIMMU_H"), ("bitmask", "grouped", "ozIMMU_EF"), ("bitmask", "per_pair", "ozIMMU"),
               ("per_slice", "per_pair", "ozIMMU_RN")]
    A, B = inputs.phi_pair(n, n, n, phi, seed=0)
    I = inputs.sample_indices(n, sample, seed=1)
    J = inputs.sample_indices(n, sample, seed=2)
    Asub, Bsub = np.ascontiguousarray(A[I]), np.ascontiguousarray(B[:, J])
    hi, lo = oracle.dot2_gemm(Asub, Bsub)
    absab = np.abs(Asub) @ np.abs(Bsub)
    dA, dB = torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda()
    tI, tJ = torch.from_numpy(I).cuda(), torch.from_numpy(J).cuda()
    D = torch.empty((n, n), dtype=torch.float64, device="cuda")
    flops = 2.0 * n ** 3
    print(f"### throughput against accuracy, m=n=p={n}, phi={phi}; median of {reps}; errors over a {sample}x{sample} "
          f"sample of D against a Dot2 product R: e1 = max |D-R|/|R|, e2 = max |D-R|/(|A||B|)\n")
    torch.mm(dA, dB, out=D)
    t = _median_ms(lambda: torch.mm(dA, dB, out=D), reps)
    e1, e2 = _sampled_errors(D, A, B, tI, tJ, hi, lo, absab)
    print(f"native FP64 (torch.mm): {flops / t / 1e9:.1f} TFLOP/s, e1 = {e1:.2e}, e2 = {e2:.2e}\n")
    print("| k | " + " | ".join(f"{name}: TFLOP/s, e1, e2" for _, _, name in methods) + " |")
    print("|---|" + "---|" * len(methods))
    ws = ozimmu.alloc_workspace(n, n, n, list(range(3, 13)), split="per_slice")
    for k in range(3, 13):
        cells = []
        for split, acc, name in methods:
            ozimmu.dgemm_variant(dA, dB, k, split, acc, D=D, workspace=ws)
            e1, e2 = _sampled_errors(D, A, B, tI, tJ, hi, lo, absab)
            t = _median_ms(lambda: ozimmu.dgemm_variant(dA, dB, k, split, acc, D=D, workspace=ws), reps)
            cells.append(f"{flops / t / 1e9:.1f}, {e1:.1e}, {e2:.1e}")
        print(f"| {k} | " + " | ".join(cells) + " |")
    print()


def small_beta(m=2048, p=2048, phi=0.5, sample=64, reps=3):
    import numpy as np
    import torch
    import oracle
    from paper_2409_13313_amd import inputs, ozimmu
    print(f"### beyond n = 2^17 (beta < 7): m=p={m}, phi={phi}; e2 = max |D-R|/(|A||B|) over a {sample}x{sample} sample, "
          f"time = median of {reps}\n")
    print("| n | beta | r | " + " | ".join(f"k={k}: e2, ms" for k in (8, 9, 10, 11, 12)) + " | native FP64: e2, ms |")
    print("|---|---|---|" + "---|" * 6)
    for n in (2 ** 17, 2 ** 18):
        A, B = inputs.phi_pair(m, n, p, phi, seed=0)
        I = inputs.sample_indices(m, sample, seed=1)
        J = inputs.sample_indices(p, sample, seed=2)
        Asub, Bsub = np.ascontiguousarray(A[I]), np.ascontiguousarray(B[:, J])
        hi, lo = oracle.dot2_gemm(Asub, Bsub)
        absab = np.abs(Asub) @ np.abs(Bsub)
        dA, dB = torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda()
        tI, tJ = torch.from_numpy(I).cuda(), torch.from_numpy(J).cuda()
        D = torch.empty((m, p), dtype=torch.float64, device="cuda")
        beta, r = ozimmu.params(n)
        ws = ozimmu.alloc_workspace(m, n, p, list(range(3, 13)))
        cells = []
        for k in (8, 9, 10, 11, 12):
            ozimmu.dgemm(dA, dB, k, D=D, workspace=ws)
            _, e2 = _sampled_errors(D, A, B, tI, tJ, hi, lo, absab)
            t = _median_ms(lambda: ozimmu.dgemm(dA, dB, k, D=D, workspace=ws), reps)
            cells.append(f"{e2:.1e}, {t:.2f}")
        torch.mm(dA, dB, out=D)
        _, e2 = _sampled_errors(D, A, B, tI, tJ, hi, lo, absab)
        t = _median_ms(lambda: torch.mm(dA, dB, out=D), reps)
        print(f"| {n} | {beta} | {r} | " + " | ".join(cells) + f" | {e2:.1e}, {t:.2f} |")
        del dA, dB, D, ws
    print()


def sizes(ns=(1024, 2048, 3072, 4096, 5120, 6144, 7168, 8192, 9216, 10240, 12288, 14336, 16384), ks=(4, 8, 12), reps=5):
    import torch
    from paper_2409_13313_amd import inputs, ozimmu
    print(f"### ozimmu_dgemm against native FP64 (torch.mm) over the matrix size, phi=0.5; median of {reps}, ms "
          f"(speed-up over native)\n")
    print("| m=n=p | native FP64 ms (TFLOP/s) | " + " | ".join(f"k={k}" for k in ks) + " | k=8, one launch forced |")
    print("|---|---|" + "---|" * (len(ks) + 1))
    for n in ns:
        A, B = inputs.phi_pair(n, n, n, 0.5, seed=0)
        dA, dB = torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda()
        D = torch.empty((n, n), dtype=torch.float64, device="cuda")
        ws = ozimmu.alloc_workspace(n, n, n, list(ks))
        torch.mm(dA, dB, out=D)
        t_nat = _median_ms(lambda: torch.mm(dA, dB, out=D), reps)
        cells = []
        for k in ks:
            ozimmu.dgemm(dA, dB, k, D=D, workspace=ws)
            t = _median_ms(lambda: ozimmu.dgemm(dA, dB, k, D=D, workspace=ws), reps)
            cells.append(f"{t:.3f} ({t_nat / t:.2f}x)")
        one = lambda: ozimmu.dgemm_variant(dA, dB, 8, "rn", "grouped", D=D, workspace=ws, schedule="one_launch")
        one()
        cells.append(f"{_median_ms(one, reps):.3f}")
        print(f"| {n} | {t_nat:.3f} ({2.0 * n ** 3 / t_nat / 1e9:.1f}) | " + " | ".join(cells) + " |")
        del dA, dB, D, ws
    print()


def small(reps=100):
    """Configurations 1 and 2 of the benchmark list as single calls: latency of one ozimmu_dgemm (median of `reps`,
    after one warm-up) next to native FP64, and the CPU oracle's time for the same product, run in full."""
    import time
    import torch
    import oracle
    from paper_2409_13313_amd import inputs, ozimmu
    print(f"### single-call latency of small products, phi=0.5, k=8; median of {reps} calls after one warm-up\n")
    print("| m=n=p | ozimmu_dgemm (us) | effective TFLOP/s | native FP64 torch.mm (us) | CPU oracle, full product (s) "
          "| oracle threads | D identical to the oracle's |")
    print("|---|---|---|---|---|---|---|")
    for n in (256, 1024):
        A, B = inputs.phi_pair(n, n, n, 0.5, seed=0)
        dA, dB = torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda()
        D = torch.empty((n, n), dtype=torch.float64, device="cuda")
        ws = ozimmu.alloc_workspace(n, n, n, 8)
        ozimmu.dgemm(dA, dB, 8, D=D, workspace=ws)
        t = _median_ms(lambda: ozimmu.dgemm(dA, dB, 8, D=D, workspace=ws), reps)
        got = D.cpu().numpy()
        torch.mm(dA, dB, out=D)
        t_nat = _median_ms(lambda: torch.mm(dA, dB, out=D), reps)
        t0 = time.perf_counter()
        want = oracle.dgemm(A, B, 8)
        t_cpu = time.perf_counter() - t0
        print(f"| {n} | {t * 1e3:.1f} | {2.0 * n ** 3 / t / 1e9:.2f} | {t_nat * 1e3:.1f} | {t_cpu:.2f} | "
              f"{oracle.num_threads()} | {bool((got == want).all())} |")
    print()


def schedules(k=8, reps=5):
    import torch
    from paper_2409_13313_amd import inputs, ozimmu
    shapes = [(512, 512, 512), (1024, 1024, 1024), (2048, 2048, 2048), (2560, 2560, 2560), (3072, 3072, 3072),
              (4096, 4096, 4096), (5120, 5120, 5120), (3072, 16384, 3072),
              (1024, 16384, 1024), (1024, 65536, 1024), (2048, 131072, 2048), (512, 131072, 512), (256, 262144, 256)]
    print(f"### outputs of few 256 x 256 tiles (or with a partly filled last round), k={k}, phi=0.5; "
          f"median of {reps}, ms (effective TFLOP/s)\n")
    print("| m x n x p | tiles | one launch | split inner | chunk parallel | queue | what the library picks | native FP64 |")
    print("|---|---|---|---|---|---|---|---|")
    for (m, n, p) in shapes:
        A, B = inputs.phi_pair(m, n, p, 0.5, seed=0)
        dA, dB = torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda()
        D = torch.empty((m, p), dtype=torch.float64, device="cuda")
        # room for the blocks of every way, also where the library would not ask for them (the queue below 256 tiles)
        tiles = ((m + 255) // 256) * ((p + 255) // 256)
        extra = (3 * ozimmu.num_chunks(n, k) * min(tiles, 256) + 2) * 4 * 256 * 256
        ws = torch.empty(ozimmu.workspace_bytes(m, n, p, k) + extra, dtype=torch.uint8, device="cuda")
        flops = 2.0 * m * n * p
        cells = []
        for sched in ("one_launch", "split_inner", "chunk_parallel", "queue", "auto"):
            run = lambda: ozimmu.dgemm_variant(dA, dB, k, "rn", "grouped", D=D, workspace=ws, schedule=sched)
            run()
            t = _median_ms(run, reps)
            cells.append(f"{t:.3f} ({flops / t / 1e9:.1f})")
        torch.mm(dA, dB, out=D)
        t = _median_ms(lambda: torch.mm(dA, dB, out=D), reps)
        print(f"| {m} x {n} x {p} | {tiles} | " + " | ".join(cells) + f" | {t:.3f} ({flops / t / 1e9:.1f}) |")
        del dA, dB, D, ws
    print()


def breakdown(n=8192, ks=(6, 8, 10, 12), reps=3):
    """The paper's time-breakdown figures, with this library's phase-level kernels: how much of the
    un-fused run is FP64 accumulation when every slice pair is accumulated on its own and when the
    pairs of a chunk are summed in INT32 first."""
    import torch
    from paper_2409_13313_amd import inputs, ozimmu
    A, B = inputs.phi_pair(n, n, n, 0.5, seed=0)
    dA, dB = torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda()
    beta, r = ozimmu.params(n)
    D = torch.empty((n, n), dtype=torch.float64, device="cuda")
    C = torch.empty((n, n), dtype=torch.int32, device="cuda")
    scratch = ozimmu.alloc_scratch()
    print(f"### time breakdown with separate kernels per phase, m=n=p={n}, phi=0.5 (r={r}); median of {reps}, ms (share)\n")
    print("| k | accumulation | split A+B | INT8 GEMMs | FP64 accumulation | total | fused ozimmu_dgemm |")
    print("|---|---|---|---|---|---|---|")
    for k in ks:
        SA, eA = ozimmu.split_A(dA, k)
        SB, eB = ozimmu.split_B(dB, k)
        ws = ozimmu.alloc_workspace(n, n, n, k)
        t_split = _median_ms(lambda: (ozimmu.split_A(dA, k), ozimmu.split_B(dB, k)), reps)
        ozimmu.dgemm(dA, dB, k, D=D, workspace=ws)
        t_fused = _median_ms(lambda: ozimmu.dgemm(dA, dB, k, D=D, workspace=ws), reps)
        for label, rr in (("per slice pair (Algorithm 4)", 1), (f"per chunk of <= {r} (Algorithm 6)", r)):
            sched = [(g, s0, min(s0 + rr - 1, g - 1)) for g in range(2, k + 2) for s0 in range(1, g, rr)]

            def gemms():
                for (g, s0, s1) in sched:
                    ozimmu.gemm_group(n, n, n, SA, k, SB, k, g, s0, s1, C=C, scratch=scratch)

            def accs():
                for i, (g, s0, s1) in enumerate(sched):
                    ozimmu.accumulate(C, eA, eB, beta, g, i == 0, D)

            gemms(); accs()
            t_g, t_a = _median_ms(gemms, reps), _median_ms(accs, reps)
            tot = t_split + t_g + t_a
            print(f"| {k} | {label}: {len(sched)} additions | {t_split:.2f} ({100 * t_split / tot:.0f} %) | "
                  f"{t_g:.2f} ({100 * t_g / tot:.0f} %) | {t_a:.2f} ({100 * t_a / tot:.0f} %) | {tot:.2f} | {t_fused:.2f} |")
        del SA, SB, ws
    print()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--accuracy", action="store_true")
    ap.add_argument("--phases", action="store_true")
    ap.add_argument("--long-inner", action="store_true")
    ap.add_argument("--variants", action="store_true")
    ap.add_argument("--perf-vs-accuracy", action="store_true")
    ap.add_argument("--small-beta", action="store_true")
    ap.add_argument("--sizes", action="store_true")
    ap.add_argument("--schedules", action="store_true")
    ap.add_argument("--small", action="store_true")
    ap.add_argument("--breakdown", action="store_true")
    args = ap.parse_args()
    import torch
    if not torch.cuda.is_available():
        print("report.py needs a GPU", file=sys.stderr)
        return 3
    if args.accuracy:
        accuracy()
    if args.phases:
        phases(8192, 8192, 8192, 0.5, [6, 8, 10])
    if args.long_inner:
        phases(4096, 65536, 4096, 1.0, [10], reps=3)
    if args.variants:
        variants()
    if args.perf_vs_accuracy:
        perf_vs_accuracy()
    if args.small_beta:
        small_beta()
    if args.sizes:
        sizes()
    if args.schedules:
        schedules()
    if args.small:
        small()
    if args.breakdown:
        breakdown()
    return 0


if __name__ == "__main__":
    sys.exit(main())
