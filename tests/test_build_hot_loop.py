"""Build-time guard for the grouped GEMM kernels: no register reloads inside the k loop.

The kernels keep their tile loads in flight with hand-placed vmcnt waits.  A register the compiler spills and reloads
inside the k loop is a scratch load on the same counter, followed by a wait for everything outstanding, i.e. a stall of
a whole memory latency per k-step (measured: 2x on the kernel).  The compiler decides this silently, so the check is
made on the generated code: between the first and the last MFMA of every instantiation there must be no scratch load
(one is tolerated in the fused-order dgrad2 kernel and in the e4m3 FC1 kernel: there it sits in the ragged-last-step
path, which runs at most once per tile and not at all when the contraction is a multiple of the step).

The second guard is for waits the compiler adds on its own.  The k loop has a path without any vmcnt wait (the wave that
touches L2 lines has no tile loads to wait for).  When vector loads issued before the loop (an epilogue's read-ahead)
may, as far as the compiler can tell, still be writing their registers on that path, it puts a vmcnt wait in front of
the first reuse of each such register; if the allocation gave them to the MFMA fragments, that is a wait in front of
the fragment reads of every k-step, which also waits for the tile loads issued just before (measured: +20 % on the
kernel).  Whether it happens depends on the register allocation, so it is checked on the generated code: no vmcnt wait
may stand directly in front of an LDS fragment read between the first and the last MFMA.
"""
import os
import re
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "paper_2505_11432_amd", "csrc", "gemm_mfma.hip")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


@pytest.fixture(scope="module")
def kernels(tmp_path_factory):
    """(name, instructions without comments or blank lines, up to s_endpgm) of every instantiation of the kernel."""
    if shutil.which(HIPCC) is None and not os.path.exists(HIPCC):
        pytest.skip("hipcc not found")
    out = tmp_path_factory.mktemp("asm") / "gemm.s"
    cmd = [HIPCC, "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Xclang", "-target-feature", "-Xclang",
           "-packed-fp32-ops", "-S", "--cuda-device-only", "-o", str(out), SRC]
    res = subprocess.run(cmd, capture_output=True, text=True)
    assert res.returncode == 0, res.stderr[-2000:]
    lines = out.read_text().split("\n")
    starts = [i for i, l in enumerate(lines) if re.match(r"_ZN3moe4mfma23grouped_gemm_dma_kernel.*: ; @", l)]
    assert len(starts) >= 12, "expected every instantiation of the kernel in the assembly"
    starts.append(len(lines))
    found = []
    for a, b in zip(starts, starts[1:]):
        name = lines[a].split(":")[0]
        body = [l.split(";")[0].rstrip() for l in lines[a + 1:b]]
        body = [l for l in body if l.strip()]
        end = max(i for i, l in enumerate(body) if "s_endpgm" in l)
        found.append((name, body[:end]))
    return found


def _mfma_span(name, body):
    mf = [i for i, l in enumerate(body) if "v_mfma" in l]
    assert mf, name
    return mf[0], mf[-1]


def test_no_scratch_loads_between_the_mfmas(kernels):
    bad = {}
    for name, body in kernels:
        first, last = _mfma_span(name, body)
        reloads = sum(1 for i in range(first, last) if "scratch_load" in body[i])
        allowed = 1 if ("EpiE5" in name or "EpiE1EDF16bh" in name) else 0
        if reloads > allowed:
            bad[name] = reloads
    assert not bad, f"register reloads inside the k loop: {bad}"


def test_no_vmcnt_wait_in_front_of_fragment_reads(kernels):
    bad = {}
    for name, body in kernels:
        first, last = _mfma_span(name, body)
        n = sum(1 for i in range(first, last)
                if re.search(r"s_waitcnt vmcnt\(\d+\)\s*$", body[i]) and any("ds_read" in x for x in body[i + 1:i + 3]))
        if n:
            bad[name] = n
    assert not bad, f"compiler-added vmcnt waits guarding fragment registers inside the k loop: {bad}"
