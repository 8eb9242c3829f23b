"""Build-time guard for the grouped GEMM kernels: no register reloads inside the k loop.

The kernels keep their tile loads in flight with hand-placed vmcnt waits.  A register the compiler spills and reloads
inside the k loop is a scratch load on the same counter, followed by a wait for everything outstanding, i.e. a stall of
a whole memory latency per k-step (measured: 2x on the kernel).  The compiler decides this silently, so the check is
made on the generated code: between the first and the last MFMA of every instantiation there must be no scratch load
(one is tolerated in the fused-order dgrad2 kernel and in the e4m3 FC1 kernel: there it sits in the ragged-last-step
path, which runs at most once per tile and not at all when the contraction is a multiple of the step).
"""
import os
import re
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "paper_2505_11432_amd", "csrc", "gemm_mfma.hip")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


@pytest.mark.skipif(shutil.which(HIPCC) is None and not os.path.exists(HIPCC), reason="hipcc not found")
def test_no_scratch_loads_between_the_mfmas(tmp_path):
    out = tmp_path / "gemm.s"
    cmd = [HIPCC, "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Xclang", "-target-feature", "-Xclang",
           "-packed-fp32-ops", "-S", "--cuda-device-only", "-o", str(out), SRC]
    res = subprocess.run(cmd, capture_output=True, text=True)
    assert res.returncode == 0, res.stderr[-2000:]
    lines = out.read_text().split("\n")
    starts = [i for i, l in enumerate(lines) if re.match(r"_ZN3moe4mfma23grouped_gemm_dma_kernel.*: ; @", l)]
    assert len(starts) >= 12, "expected every instantiation of the kernel in the assembly"
    starts.append(len(lines))
    bad = {}
    for a, b in zip(starts, starts[1:]):
        name = lines[a].split(":")[0]
        body = lines[a:b]
        end = max(i for i, l in enumerate(body) if "s_endpgm" in l)
        body = body[:end]
        mf = [i for i, l in enumerate(body) if "v_mfma" in l]
        assert mf, name
        reloads = sum(1 for i in range(mf[0], mf[-1]) if "scratch_load" in body[i])
        allowed = 1 if ("EpiE5" in name or "EpiE1EDF16bh" in name) else 0
        if reloads > allowed:
            bad[name] = reloads
    assert not bad, f"register reloads inside the k loop: {bad}"
