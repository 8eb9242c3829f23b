"""Text summaries of rocprofv3 output for this library's kernels.

    rocprofv3 --kernel-trace --stats --output-format csv -d DIR -o bench -- python3 bench.py ...
    python -m paper_2505_11432_amd.profile_summary trace DIR/.../bench_kernel_trace.csv [layer steps in the trace]

    rocprofv3 --pmc SQ_BUSY_CYCLES SQ_VALU_MFMA_BUSY_CYCLES --output-format csv -d DIR -o bench -- python3 bench.py ...
    python -m paper_2505_11432_amd.profile_summary pmc DIR/.../bench_counter_collection.csv

Kernel names are shortened to labels; the legend printed under every table says how a label is made
from the (demangled or mangled) kernel name, so a row can be traced back to the profiler's own name.
"""
from __future__ import annotations

import collections
import csv
import re
import sys

LEGEND = """labels: grouped_gemm<BMxBNxBK sS wMxN LAYOUT MODE EPILOGUE out=T in=T> are the template arguments of
  moe::mfma::grouped_gemm_dma_kernel<BM, BN, BKT, NSTAGE, WM, WN, LA, LB, MODE, EPI, TC, TIN> in that order:
  LAYOUT from (LA, LB): (0,0) NT = both operands K-major (forward), (0,1) NN = B N-major (dgrad), (1,1) TN = both
  M/N-major (wgrad); MODE 0 rowseg (rows segmented by expert), 1 kseg (contraction segmented: weight gradient),
  2 plain; EPI 0 store, 1 swiglu (FC1), 2 swiglu_bwd (dgrad2), 3 bias_f32 (router), 4 swiglu_w, 5 swiglu_bwd_w
  (gate weight folded in); TC f = fp32 output, else bf16; TIN h = e4m3 operands, else bf16 (where the profiler
  prints the type pair as "bool _Accum", 128-deep steps mean e4m3 operands with bf16 output).
  Other kernels: the function name without namespaces and template arguments."""

_LAYOUT = {(0, 0): "NT", (0, 1): "NN", (1, 1): "TN", (1, 0): "TT"}
_MODE = {0: "rowseg", 1: "kseg", 2: "plain"}
_EPI = {0: "store", 1: "swiglu", 2: "swiglu_bwd", 3: "bias_f32", 4: "swiglu_w", 5: "swiglu_bwd_w"}


def label(name: str) -> str:
    """Short label of a kernel from its mangled (_ZN...) or demangled name."""
    if "grouped_gemm_dma_kernel" in name:
        tail = name[name.index("grouped_gemm_dma_kernel"):]
        if tail.startswith("grouped_gemm_dma_kernel<"):                       # demangled
            nums = [int(v) for v in re.findall(r"(?<![\w.])(\d+)(?![\w.])", tail)][:10]
            out_f32 = bool(re.search(r",\s*float\s*,", tail))
            in_fp8 = "unsigned char" in tail
            if "_Accum" in tail and len(nums) >= 3:
                # rocprofv3's demangler garbles the pair "__bf16, unsigned char" (it prints "bool _Accum"): only the
                # e4m3 kernels have 128-deep steps, and of those only the fp32-output ones demangle correctly
                in_fp8, out_f32 = nums[2] == 128, False
        else:                                                                 # Itanium mangling: Li<n>E ints, L<enum type>E<n>E enums
            ints = [int(v) for v in re.findall(r"Li(\d+)E", tail)][:6]
            enums = [int(v) for v in re.findall(r"L(?:NS\d+_\d+[A-Za-z]+E|S\d*_)(\d+)E", tail)][:4]
            nums = ints + enums
            types = re.findall(r"DF16b|f|h", re.sub(r"Li\d+E", "", tail.split("Epi", 1)[-1].split("EEv", 1)[0])[2:])
            out_f32 = bool(types) and types[0] == "f"
            in_fp8 = len(types) > 1 and types[-1] == "h"
        if len(nums) == 10:
            bm, bn, bk, ns, wm, wn, la, lb, mode, epi = nums
            return (f"grouped_gemm<{bm}x{bn}x{bk} s{ns} w{wm}x{wn} {_LAYOUT.get((la, lb), '??')} {_MODE.get(mode, '?')} "
                    f"{_EPI.get(epi, '?')} out={'f32' if out_f32 else 'bf16'} in={'e4m3' if in_fp8 else 'bf16'}>")
        return "grouped_gemm<?> " + tail[:80]
    m = re.search(r"([a-z][a-z0-9_]*_kernel)", name)
    if m:
        return m.group(1)
    return name[:70]


def _rows(path: str):
    with open(path, newline="") as fh:
        yield from csv.DictReader(fh)


def trace(path: str, steps: int = 0) -> str:
    """Per-kernel count / mean / min / max duration from a rocprofv3 kernel-trace csv.  With `steps` (the number
    of layer steps in the trace), a kernel launched n > 1 times per step is listed per position in the step
    ("#1" ... "#n", in launch order), since those launches do different work (FC2 and dgrad1, wgrad2 and wgrad1)."""
    rows = sorted(_rows(path), key=lambda r: int(r["Start_Timestamp"]))
    agg = collections.OrderedDict()
    for r in rows:
        dur = (int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3
        agg.setdefault(label(r["Kernel_Name"]), []).append(dur)
    if steps > 0:
        split = collections.OrderedDict()
        for k, v in agg.items():
            n = len(v) // steps
            if k.startswith("grouped_gemm<") and n > 1 and len(v) == n * steps:
                for i in range(n):
                    split[f"{k} #{i + 1}"] = v[i::n]
            else:
                split[k] = v
        agg = split
    total = sum(sum(v) for v in agg.values())
    lines = [f"{'kernel':<86}{'calls':>7}{'avg_us':>10}{'min_us':>10}{'max_us':>10}{'total_ms':>10}{'pct':>6}"]
    for k, v in sorted(agg.items(), key=lambda kv: -sum(kv[1])):
        lines.append(f"{k:<86}{len(v):>7}{sum(v) / len(v):>10.1f}{min(v):>10.1f}{max(v):>10.1f}{sum(v) / 1e3:>10.2f}"
                     f"{100 * sum(v) / total:>6.1f}")
    return "\n".join(lines) + "\n" + LEGEND


def pmc(path: str) -> str:
    """Per-kernel mean of every counter in a rocprofv3 counter-collection csv (one row per dispatch and counter)."""
    agg = collections.OrderedDict()
    counters = []
    for r in _rows(path):
        c = r["Counter_Name"]
        if c not in counters:
            counters.append(c)
        agg.setdefault(label(r["Kernel_Name"]), collections.defaultdict(list))[c].append(float(r["Counter_Value"]))
    lines = []
    for g0 in range(0, len(counters), 3):                      # three counters per block keeps the lines readable
        group = counters[g0:g0 + 3]
        lines.append(f"{'kernel':<86}{'dispatches':>11}" + "".join(f"{c:>32}" for c in group))
        for k, d in agg.items():
            n = max(len(v) for v in d.values())
            lines.append(f"{k:<86}{n:>11}" + "".join(f"{(sum(d[c]) / len(d[c]) if d[c] else float('nan')):>32,.1f}" for c in group))
        lines.append("")
    return "\n".join(lines) + "\n(mean per dispatch)\n" + LEGEND


def main(argv) -> int:
    if len(argv) not in (3, 4) or argv[1] not in ("trace", "pmc"):
        sys.stderr.write(__doc__)
        return 2
    print(trace(argv[2], int(argv[3]) if len(argv) == 4 else 0) if argv[1] == "trace" else pmc(argv[2]))
    return 0


if __name__ == "__main__":
    sys.exit(main(sys.argv))
