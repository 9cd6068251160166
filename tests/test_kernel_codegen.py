"""Code-generation check of the chunk GEMM kernel (CPU only: hipcc cross-compiles).

The main loop orders its global -> LDS copies with hand-written `s_waitcnt vmcnt(N)` whose N counts exactly the copies
in flight.  The compiler knows nothing of those copies, but its own waits use the same counter: a register spill
reload, or any ordinary load still pending when the loop is entered, makes it put a `vmcnt` wait INTO the loop that
also waits for the copies and stalls the pipeline (measured: 6 to 9 % of the run time, with bit-identical results,
so no parity test sees it).  This test compiles the kernel to assembly and looks at the loop."""
import os
import re
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "paper_2409_13313_amd", "csrc", "ozimmu_gemm.hip")
FLAGS = ["-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC", "-ffp-contract=off",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument"]


@pytest.mark.skipif(shutil.which("hipcc") is None, reason="needs hipcc")
def test_no_compiler_made_memory_wait_inside_the_mfma_loop(tmp_path):
    out = str(tmp_path / "gemm.s")
    pr = subprocess.run(["hipcc", *FLAGS, "--cuda-device-only", "-S", SRC, "-o", out],
                        stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert pr.returncode == 0, pr.stdout[-3000:]
    text = open(out).read()
    checked = 0
    for mode in (0, 1, 2, 3):
        m = re.search(r"^_ZN12_GLOBAL__N_16k_gemmILi%dELi4EEEvN3ozk8GemmArgsEii:.*?s_endpgm" % mode, text, re.S | re.M)
        assert m, f"k_gemm<{mode},4> not found in the assembly"
        lines = m.group(0).split("\n")
        mfma = [i for i, l in enumerate(lines) if "v_mfma_i32_16x16x64_i8" in l]
        # 4 stages x 64 MFMAs in the steady-state group, the same in the tail group
        assert len(mfma) == 512, (mode, len(mfma))
        loop = lines[mfma[0]:mfma[-1] + 1]
        waits = [re.search(r"vmcnt\((\d+)\)", l).group(1) for l in loop if "s_waitcnt" in l and "vmcnt" in l]
        # the hand-written ones: one per stage; 8 copies may stay in flight, none at the end of a chunk
        assert sorted(waits) == ["0", "0"] + ["8"] * 6, (mode, waits)
        # (the steady-state group; in the tail group, run once per chunk, the compiler may park a few values for the
        # epilogue - stores only: a reload would bring one of its own waits, which the list above would show)
        steady = lines[mfma[0]:mfma[255] + 1]
        assert not any("scratch_" in l or "buffer_load" in l or "buffer_store" in l for l in steady), mode
        assert not any("scratch_load" in l or "buffer_load" in l for l in loop), mode
        # a fragment fetched in one sub-step (4 MFMAs) is first used four sub-steps later: the compiler's waits for
        # LDS data in the steady state must leave the three youngest fetches pending
        lgkm = [int(re.search(r"lgkmcnt\((\d+)\)", l).group(1)) for l in steady if "s_waitcnt" in l and "lgkmcnt" in l]
        assert lgkm and min(lgkm) >= 3, (mode, sorted(set(lgkm)))
        # three of four tile copies rely on the M0 that the first one set: nothing else in the loop may write M0
        m0 = [l.strip() for l in loop if re.search(r"\bm0\b", l)]
        assert m0 and all(l.startswith("s_add_u32 m0,") for l in m0), (mode, m0[:4])
        # issue slots: with one wave per SIMD an instruction issues every 4 cycles and a 4-pass MFMA lasts 16, so three
        # other instructions fit behind an MFMA and a longer run delays the next one (a dozen scalar instructions of
        # cursor bookkeeping in one gap, an M0 set-up per copy: 2 to 3 % of the run time)
        code = [l.strip() for l in steady]
        code = [l for l in code if l and not l.startswith(";") and not l.startswith(".")]
        at = [i for i, l in enumerate(code) if l.startswith("v_mfma")]
        for a, b in zip(at, at[1:]):
            gap = code[a + 1:b]
            limit = 5 if any(l.startswith("s_barrier") for l in gap) else 3
            assert len(gap) <= limit, (mode, gap)
        checked += 1
    assert checked == 4
