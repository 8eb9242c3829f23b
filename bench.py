#!/usr/bin/env python3
"""Benchmark of the MoE-layer hot path on one MI355X.

A "step" is one forward + backward pass of the whole path (router matmul, gating, dispatch, expert
grouped GEMMs with SwiGLU, combine, and every gradient) over one batch of seeded synthetic input
of the Mixtral-8x7B layer shape (T=8192, d=4096, E=8, top-2, d_ff=14336, bf16).  Inputs and weights
are resident in HBM before the timed region starts.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA, published
PEAK_FP8_TFLOPS = 5000.0       # MI355X dense fp8 MFMA, published
PEAK_HBM_GBPS = 8000.0
# L2-fill + write-back bytes per grouped-GEMM launch (average of the six launches of one step) come from the
# committed rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE summary of the same command: a stored figure, read from that
# file's TRAFFIC_BYTES_PER_LAUNCH line (counters cannot be collected from inside a timing run).
TRAFFIC_SUMMARY = {"mixtral": "profiles/grouped_gemm_mixtral_hbm_counters.txt"}


def stored_traffic(workload):
    """(bytes per launch, source file) from the committed counter summary of this workload, or (None, None)."""
    rel = TRAFFIC_SUMMARY.get(workload)
    if rel is None or not os.path.exists(os.path.join(ROOT, rel)):
        return None, None
    for line in open(os.path.join(ROOT, rel)):
        if line.startswith("TRAFFIC_BYTES_PER_LAUNCH"):
            return float(line.split("=")[1].split()[0]), rel
    return None, None


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="mixtral", help="synthetic workload name (see synth/moe_inputs.py)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-tokens", type=int, default=0, help="tokens in the oracle's timed sample (0 = T/4)")
    ap.add_argument("--fp8-backward", action="store_true",
                    help="fp8 configurations only: run the four backward GEMMs on e4m3 operands as well")
    ap.add_argument("--capacity-factor", type=float, default=0.0,
                    help="bf16 configurations: device-level token dropping with capacity = factor * T*k / devices (0 = dropless)")
    ap.add_argument("--balance-alpha", type=float, default=0.0, help="add the device-level auxiliary balance loss (0 = off)")
    ap.add_argument("--devices", type=int, default=8, help="expert groups (GPUs of the node) for the two switches above")
    ap.add_argument("--fused", action="store_true",
                    help="bf16 only: the paper's Section 4.1 / 4.2 operator order (FC1 selects its rows from x inside the "
                         "kernel, gate weight after SwiGLU, gate gradient from the dgrad2 epilogue, no dispatched input "
                         "or FC2 output kept for the backward)")
    ap.add_argument("--keep-a", action="store_true",
                    help="bf16, plain order: keep the FC2 input from the forward (M*f*2 bytes) instead of writing it again in "
                         "the backward")
    ap.add_argument("--graph", action="store_true",
                    help="time K replays of one HIP graph holding the whole step (forward + backward) instead of K eager "
                         "steps; the per-call times and the roofline figure then come from an extra eager pass of K steps")
    ap.add_argument("--ceilings", action="store_true",
                    help="also measure the practical ceilings (register-only MFMA loop, plain copy, library GEMM as context) "
                         "and report the GEMM figure as a fraction of the measured MFMA-loop rate beside the published peak")
    ap.add_argument("--no-permute-large", action="store_true", help="skip the dispatch / combine timing on the large row buffers")
    ap.add_argument("--permute-only", default=None, metavar="WORKLOAD",
                    help="time only dispatch / combine / gate gradient on this workload's activations and print that block")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one 1 GiB device-to-device copy, the known-size reference for HBM byte counters")
    return ap.parse_args()


def ensure_built():
    # builds when the library is missing or was built from other sources than the ones in the tree
    from paper_2505_11432_amd.build import ensure_built as ensure
    ensure()


def to_dev_bf16(a, torch):
    import numpy as np
    from synth.moe_inputs import bf16_bits
    bits = bf16_bits(a).view(np.int16)
    return torch.from_numpy(bits).to("cuda:0").view(torch.bfloat16)


def cpu_baseline_fp8(cfg, inp, tokens, fp8_backward=False):
    import numpy as np
    from threadpoolctl import threadpool_info
    from oracle import moe_oracle as O
    x, dy = inp["x"][:tokens], inp["dy"][:tokens]
    t0 = time.perf_counter()
    z = O.router_logits(x, inp["W_r"], inp["bias"]).astype(np.float32)
    fwd = O.layer_fwd_fp8(x, z, inp["W1"], inp["W2"], cfg.k, cfg.renorm)
    (O.layer_bwd_fp8_gemm if fp8_backward else O.layer_bwd_fp8)(x, z, inp["W1"], inp["W2"], cfg.k, dy, fwd, cfg.renorm)
    dt = time.perf_counter() - t0
    threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    return {"value": tokens / dt, "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
            "sample": f"first {tokens} of {cfg.T} tokens, all {cfg.E} experts and full d, d_ff; numpy float64 "
                      f"forward+backward with the E4M3 casts (weights cast included), {dt:.1f} s"}


def cpu_baseline(cfg, inp, tokens):
    """The oracle as it stands, timed on the host cores on the first `tokens` tokens."""
    import numpy as np
    from threadpoolctl import threadpool_info
    from oracle import moe_oracle as O
    x = inp["x"][:tokens]
    dy = inp["dy"][:tokens]
    t0 = time.perf_counter()
    z = O.router_logits(x, inp["W_r"], inp["bias"]).astype(np.float32)
    if cfg.expert_range is None:
        fwd = O.layer_fwd(x, z, inp["W1"], inp["W2"], cfg.k, cfg.renorm)
        O.layer_bwd(x, z, inp["W1"], inp["W2"], cfg.k, dy, fwd, cfg.renorm, W_r=inp["W_r"])
    else:
        lo, hi = cfg.expert_range
        fwd = O.layer_fwd_range(x, z, inp["W1"], inp["W2"], cfg.k, lo, hi, cfg.renorm)
        O.layer_bwd_range(x, z, inp["W1"], inp["W2"], cfg.k, dy, fwd)
    dt = time.perf_counter() - t0
    threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    return {"value": tokens / dt, "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
            "sample": f"first {tokens} of {cfg.T} tokens, all {len(cfg.local_experts)} " +
                      ("local " if cfg.expert_range else "") + "experts and full d, d_ff; "
                      f"numpy float64 forward+backward, {dt:.1f} s"}


def permute_large(name="finegrained", reps=20):
    """Dispatch, combine and gate gradient alone on the activations of a workload whose row buffers (>= 600 MB per
    pass) do not fit the 256 MB Infinity Cache, so the figure is an HBM rate.  Activations and routing only: no
    expert weights are drawn.  Bytes per call are the algorithmic ones: every token row and every dispatched row
    crosses HBM once ((T + T*k) * d * 2 for bf16; the gate gradient only reads)."""
    import numpy as np
    import torch
    from paper_2505_11432_amd import binding as B
    from synth.moe_inputs import CONFIGS, make_inputs
    cfg = CONFIGS[name]
    inp = make_inputs(cfg, seed=0, with_weights=False)
    dev = "cuda:0"
    T, d, E, k, M = cfg.T, cfg.d, cfg.E, cfg.k, cfg.M
    x, dy = to_dev_bf16(inp["x"], torch), to_dev_bf16(inp["dy"], torch)
    w_r = to_dev_bf16(np.ascontiguousarray(inp["W_r"].T), torch)
    bias = torch.from_numpy(inp["bias"]).to(dev) if cfg.bias != "none" else None
    i32 = dict(dtype=torch.int32, device=dev)
    logits = torch.empty((T, E), device=dev)
    idx, w = torch.empty((T, k), **i32), torch.empty((T, k), device=dev)
    counts, offsets = torch.empty((E,), **i32), torch.empty((E + 1,), **i32)
    perm, inv_perm = torch.empty((M,), **i32), torch.empty((M,), **i32)
    ws = torch.empty((max(B.moe_workspace_bytes(T, 16, E, k, 16, B.BF16), 256),), dtype=torch.uint8, device=dev)
    xp = torch.empty((M, d), dtype=torch.bfloat16, device=dev)
    y = torch.empty((T, d), dtype=torch.bfloat16, device=dev)
    dw = torch.empty((T, k), device=dev)
    B.moe_router_fwd(x, w_r, bias, logits)
    B.moe_route(logits, k, cfg.renorm, idx, w, counts, offsets, perm, inv_perm, ws)
    calls = {
        "dispatch": lambda: B.moe_dispatch(x, None, inv_perm, None, k, xp, None),
        "dispatch_scaled": lambda: B.moe_dispatch(x, None, inv_perm, w.view(-1), k, xp, None),
        "combine": lambda: B.moe_combine(xp, None, inv_perm, w, k, y),
        "combine_unweighted": lambda: B.moe_combine(xp, None, inv_perm, None, k, y),
        "gate_grad": lambda: B.moe_gate_grad(dy, xp, None, inv_perm, k, dw),
    }
    nbytes = float(T + M) * d * 2
    out = {"workload": f"{cfg.name}: T={T} d_model={d} E={E} top-{k}, bf16 rows, activations and routing only",
           "bytes_per_call": nbytes, "reps": reps, "ms": {}, "gbps": {}, "peak": PEAK_HBM_GBPS}
    for cname, fn in calls.items():
        for _ in range(3):
            fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / reps
        out["ms"][cname] = ms
        out["gbps"][cname] = nbytes / ms / 1e6
    out["frac"] = {c: v / PEAK_HBM_GBPS for c, v in out["gbps"].items()}
    return out


def ceilings(cfg, fp8_path=False):
    """The practical ceilings beside the published peaks (include/moe_ceilings.h): a register-only MFMA loop on
    constant and on random operand bits, a plain 1 GiB copy and read, and, as context only, the library GEMM
    (torch.matmul) on one expert's FC1 shape and on all dispatched rows at once."""
    import ctypes
    import torch
    from paper_2505_11432_amd.build import CEILINGS_LIB_PATH
    lib = ctypes.CDLL(CEILINGS_LIB_PATH)
    P, I, Z = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
    lib.moe_ceiling_mfma_loop.argtypes = [I, P, I, I, P, P]
    lib.moe_ceiling_mfma_lds_loop.argtypes = [P, I, I, P, P]
    lib.moe_ceiling_mfma_lds_dma_loop.argtypes = [P, P, Z, I, I, I, P, P]
    lib.moe_ceiling_copy.argtypes = [P, P, Z, P]
    lib.moe_ceiling_read.argtypes = [P, Z, P, P]
    dev = "cuda:0"
    stream = torch.cuda.current_stream().cuda_stream
    wgs = torch.cuda.get_device_properties(0).multi_processor_count
    sink = torch.zeros((wgs * 512,), device=dev)
    g = torch.Generator(device="cpu").manual_seed(0)

    def timed(fn, reps):
        fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    def mfma(fp8, operands, iters=100000):
        ms = timed(lambda: lib.moe_ceiling_mfma_loop(int(fp8), operands.data_ptr(), iters, wgs, sink.data_ptr(), stream), 3)
        return wgs * 8 * iters * 8 * 2.0 * 32 * 32 * (64 if fp8 else 16) / ms / 1e9

    n_lane_slots = 2 * 6 * 64
    def bf16_operands(values):            # values [slots, 8] float -> 32 bytes per lane (bf16 in the first 16)
        buf = torch.zeros((n_lane_slots, 16), dtype=torch.bfloat16)
        buf[:, :8] = values.to(torch.bfloat16)
        return buf.to(dev)
    out = {}
    out["mfma_loop_bf16_const_tflops"] = mfma(False, bf16_operands(torch.ones((n_lane_slots, 8))))
    out["mfma_loop_bf16_random_tflops"] = mfma(False, bf16_operands(torch.randn((n_lane_slots, 8), generator=g)))
    out["mfma_loop_bf16_weightlike_tflops"] = mfma(False, bf16_operands(0.02 * torch.randn((n_lane_slots, 8), generator=g)))
    image = torch.randn((65536,), generator=g).to(torch.bfloat16).to(dev)                     # 128 KiB of N(0,1) bf16
    ms = timed(lambda: lib.moe_ceiling_mfma_lds_loop(image.data_ptr(), 40000, wgs, sink.data_ptr(), stream), 3)
    out["mfma_lds_fed_loop_bf16_random_tflops"] = wgs * 8 * 40000 * 8 * 2.0 * 32 * 32 * 16 / ms / 1e9
    # the same with the kernel's global -> LDS traffic beside it (64 KiB per workgroup and k-step from an L2-resident
    # 4 MiB buffer): loads only, loads + the loaders' wait at the step end, loads + wait + a barrier per step
    feed = torch.randn((2 * 1024 * 1024,), generator=g).to(torch.bfloat16).to(dev)
    for key, flags in (("loads", 1), ("loads_wait", 3), ("loads_wait_barrier", 7)):
        ms = timed(lambda: lib.moe_ceiling_mfma_lds_dma_loop(image.data_ptr(), feed.data_ptr(), feed.numel() * 2, 40000, flags, wgs,
                                                             sink.data_ptr(), stream), 3)
        out[f"mfma_lds_fed_loop_with_{key}_tflops"] = wgs * 8 * 40000 * 8 * 2.0 * 32 * 32 * 16 / ms / 1e9
    codes = torch.randint(0, 0x7f, (n_lane_slots, 32), generator=g, dtype=torch.int16)          # finite e4m3 magnitudes
    codes = (codes | (torch.randint(0, 2, (n_lane_slots, 32), generator=g, dtype=torch.int16) << 7)).to(torch.uint8)
    out["mfma_loop_fp8_const_tflops"] = mfma(True, torch.full((n_lane_slots, 32), 0x38, dtype=torch.uint8).to(dev))
    out["mfma_loop_fp8_random_tflops"] = mfma(True, codes.to(dev))
    nbytes = 1 << 30
    src = torch.randint(0, 255, (nbytes,), dtype=torch.uint8, device=dev)
    dst = torch.empty_like(src)
    ms = timed(lambda: lib.moe_ceiling_copy(src.data_ptr(), dst.data_ptr(), nbytes, stream), 10)
    out["copy_gbps"] = 2.0 * nbytes / ms / 1e6
    ms = timed(lambda: lib.moe_ceiling_read(src.data_ptr(), nbytes, sink.data_ptr(), stream), 10)
    out["read_gbps"] = nbytes / ms / 1e6
    del src, dst
    # context only: the vendor library on dense GEMMs of the FC1 shape, same value distributions as the workload
    rows_e = cfg.M // cfg.E
    for name, rows in (("library_gemm_fc1_one_expert_tflops", rows_e), ("library_gemm_fc1_all_rows_tflops", cfg.M)):
        a = torch.randn((rows, cfg.d), generator=g).to(torch.bfloat16).to(dev)
        w = (0.02 * torch.randn((2 * cfg.f, cfg.d), generator=g)).to(torch.bfloat16).to(dev)
        c = torch.empty((rows, 2 * cfg.f), dtype=torch.bfloat16, device=dev)
        ms = timed(lambda: torch.matmul(a, w.t(), out=c), 10)
        out[name] = 2.0 * rows * cfg.d * 2 * cfg.f / ms / 1e9
        del a, w, c
    # the weight-gradient shape of one expert: [2f, rows_e] x [rows_e, d], contraction over the expert's tokens
    dh = torch.randn((rows_e, 2 * cfg.f), generator=g).to(torch.bfloat16).to(dev)
    xe = torch.randn((rows_e, cfg.d), generator=g).to(torch.bfloat16).to(dev)
    c = torch.empty((2 * cfg.f, cfg.d), dtype=torch.bfloat16, device=dev)
    ms = timed(lambda: torch.matmul(dh.t(), xe, out=c), 10)
    out["library_gemm_wgrad1_one_expert_tflops"] = 2.0 * rows_e * cfg.d * 2 * cfg.f / ms / 1e9
    del dh, xe, c
    out["note"] = ("mfma_loop_*: register-only loop of 32x32 MFMAs, 8 waves per CU; const = all-ones operands, random = "
                   "N(0,1) bf16 / uniformly random finite e4m3 codes, weightlike = N(0, 0.02); mfma_lds_fed_loop: the bf16 loop with "
                   "its fragments read from LDS (N(0,1) data) at the grouped GEMM's ratio; _with_loads / _loads_wait / _loads_wait_barrier: "
                   "plus 64 KiB of direct-to-LDS loads per workgroup and 64-deep k-step from an L2-resident buffer, the loading waves' "
                   "wait at the end of each step, and a workgroup barrier per step; library_gemm_*: "
                   f"torch.matmul on the FC1 shape [rows,{cfg.d}] x [{cfg.d},{2 * cfg.f}] and on one expert's weight-gradient "
                   "shape, bf16, context only")
    return out


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
              f"--gpus {args.gpus} is not supported.", file=sys.stderr)
        sys.exit(2)
    ensure_built()
    import numpy as np
    import torch
    from paper_2505_11432_amd import binding as B          # fails loudly if the HIP library is missing
    if args.permute_only:
        torch.cuda.set_device(0)
        print(json.dumps({"permute_large": permute_large(args.permute_only)}))
        return
    from paper_2505_11432_amd.layer import MoELayer
    from synth.moe_inputs import CONFIGS, make_inputs

    cfg = CONFIGS[args.config]
    assert cfg.dtype in ("bf16", "fp8"), "the benchmark workloads are the bf16 / fp8 configurations"
    fp8 = cfg.dtype == "fp8"
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    torch.cuda.set_device(0)
    t0 = time.time()
    inp = make_inputs(cfg, seed=0)
    x, dy = to_dev_bf16(inp["x"], torch), to_dev_bf16(inp["dy"], torch)
    w_r = to_dev_bf16(np.ascontiguousarray(inp["W_r"].T), torch)
    bias = torch.from_numpy(inp["bias"]).to("cuda:0") if cfg.bias != "none" else None
    w1, w2 = to_dev_bf16(inp["W1"], torch), to_dev_bf16(inp["W2"], torch)
    devices = min(args.devices, cfg.E)
    capacity = (devices, int(math.ceil(args.capacity_factor * cfg.T * cfg.k / devices))) if args.capacity_factor > 0 else None
    balance = (devices, args.balance_alpha) if args.balance_alpha > 0 else None
    layer = MoELayer(cfg.T, cfg.d, cfg.E, cfg.k, cfg.f, dtype=torch.bfloat16, renorm=cfg.renorm, fp8=fp8,
                     expert_range=cfg.expert_range, capacity=capacity, balance=balance, fused=args.fused,
                     keep_a=args.keep_a)
    if args.fused and fp8:
        print("bench.py: --fused is a bf16 path", file=sys.stderr)
        sys.exit(2)
    if fp8:
        layer.set_fp8_weights(w1, w2)       # parameters are kept in E4M3 across steps (Section 7): outside the timed loop
        if args.fp8_backward:
            layer.set_fp8_backward_weights(w1, w2)
    elif args.fp8_backward:
        print("bench.py: --fp8-backward needs an fp8 configuration (--config mixtral_fp8)", file=sys.stderr)
        sys.exit(2)
    torch.cuda.synchronize()
    setup_s = time.time() - t0

    def step():
        if fp8:
            layer.forward_fp8(x, w_r, bias)
            if args.fp8_backward:
                layer.backward_fp8_gemm(x, w_r, dy)
            else:
                layer.backward_fp8(x, w_r, w1, w2, dy)
        else:
            layer.forward(x, w_r, bias, w1, w2)
            layer.backward(x, w_r, w1, w2, dy)

    if args.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda:0")     # 1 GiB read + 1 GiB written
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    start, end = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    if args.graph:
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
        graph.replay()
        torch.cuda.synchronize()
        start.record()
        for _ in range(args.steps):
            graph.replay()
        end.record()
        torch.cuda.synchronize()
        total_ms = start.elapsed_time(end)
        layer.timers = {}
        for _ in range(args.steps):
            step()
    else:
        # inside the timed region only the two calls that hold the six GEMM launches are bracketed with events (the
        # roofline figure); the other calls are timed in a second, untimed pass, because every event record between
        # two calls leaves the GPU idle for about 10 us
        layer.timers = {}
        layer.timer_filter = {"expert_ffn_fwd", "expert_ffn_bwd"}
        torch.cuda.synchronize()
        start.record()
        for _ in range(args.steps):
            step()
        end.record()
        torch.cuda.synchronize()
        total_ms = start.elapsed_time(end)
    per_call = {k: v / args.steps for k, v in layer.timer_ms().items()}
    if layer.timer_filter is not None:
        layer.timers, layer.timer_filter = {}, None
        for _ in range(args.steps):
            step()
        other = {k: v / args.steps for k, v in layer.timer_ms().items()}
        other.update(per_call)                  # the GEMM calls keep their figures from the timed region
        per_call = {k: other[k] for k in other}
    layer.timers = None
    ms_per_step = total_ms / args.steps

    counts = layer.counts.cpu().tolist()
    # dispatched rows: all T*k, or the rows of the local experts for an expert-parallel share
    M = cfg.M if cfg.expert_range is None else int(sum(counts[e] for e in cfg.local_experts))
    if capacity is not None:
        M = int(sum(counts))                                   # rows kept after dropping
    gemm_flops = 18.0 * M * cfg.d * cfg.f                      # three matmuls per routed token, fwd + 2x bwd
    # bf16 path: these two calls are exactly the six GEMM launches (fp8 path: plus the two row casts in the forward)
    gemm_ms = per_call["expert_ffn_fwd"] + per_call["expert_ffn_bwd"]
    gemm_tflops = gemm_flops / gemm_ms / 1e9
    # Each GEMM is priced against the peak of the cores it runs on (the casts inside the two calls count as time):
    # bf16 path 2.5 PFLOP/s; all six on e4m3 operands 5.0; e4m3 forward with bf16 backward: the blend that the
    # forward's 6*M*d*f at 5.0 and the backward's 12*M*d*f at 2.5 would take.
    if not fp8:
        peak = PEAK_BF16_TFLOPS
    elif args.fp8_backward:
        peak = PEAK_FP8_TFLOPS
    else:
        peak = 18.0 / (6.0 / PEAK_FP8_TFLOPS + 12.0 / PEAK_BF16_TFLOPS)
    # algorithmic bytes of the row movers: what is read plus what is written, in the types that are moved
    esz_rows = 1 if fp8 else 2                                   # dispatched rows: e4m3 codes or bf16
    tokens_read = int((layer.inv_perm.view(cfg.T, cfg.k) >= 0).any(dim=1).sum())     # dispatch skips tokens without a local row
    dispatch_bytes = float(tokens_read + M) * cfg.d * esz_rows + (float(tokens_read + M) * 4 if fp8 else 0.0)
    combine_bytes = float(M) * cfg.d * esz_rows + float(cfg.T) * cfg.d * 2 + (float(M) * 4 if fp8 else 0.0)
    traffic, traffic_source = stored_traffic(cfg.name) if not (fp8 or args.fused or capacity or balance) else (None, None)

    out = {
        "metric": "MoE layer fwd+bwd tokens/s; grouped-GEMM TFLOPS as % of MI355X MFMA peak",
        "value": cfg.T / (ms_per_step / 1e3),
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "fp8" if fp8 else "bf16", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: T={cfg.T} d_model={cfg.d} E={cfg.E} top-{cfg.k} d_ff={cfg.f} SwiGLU, " +
                               (("e4m3 dispatched activations / returned outputs, all six expert GEMMs on e4m3 operands, "
                                 if args.fp8_backward else
                                 "e4m3 dispatched activations / expert GEMMs / returned outputs forward, bf16 backward, ")
                                if fp8 else "bf16 weights/activations, ") + "fp32 accumulate, fp32 weight gradients" +
                               (f"; expert-parallel share: experts {cfg.expert_range[0]}..{cfg.expert_range[1] - 1} local, "
                                f"{M} of {cfg.M} dispatched rows, tokens = the all-gathered tokens" if cfg.expert_range else "") +
                               (f"; capacity {capacity[1]} rows per device over {capacity[0]} devices, {M} of {cfg.M} rows kept"
                                if capacity else "") + (f"; balance loss alpha={args.balance_alpha}" if balance else "") +
                               ("; fused operator order (row select inside FC1, gate weight after SwiGLU, FC1 input rows "
                                "produced again in the backward)" if args.fused else "") +
                               ("; FC2 input kept from the forward" if args.keep_a else ""),
                   "tokens": cfg.T, "expert_rows": counts},
        "roofline": {"bound": "mfma", "kernel": "grouped_gemm_kernel (6 launches per step: FC1+SwiGLU, FC2, "
                                                "dgrad2+SwiGLU', wgrad2, dgrad1, wgrad1)",
                     "achieved": gemm_tflops, "peak": peak, "unit": "TFLOP/s",
                     "frac": gemm_tflops / peak,
                     "traffic": traffic, "traffic_source": traffic_source,
                     "flops_per_launch_avg": gemm_flops / 6, "launch_ms_avg": gemm_ms / 6},
        "gemm_tflops": {"fwd": 6.0 * M * cfg.d * cfg.f / per_call["expert_ffn_fwd"] / 1e9,
                        "bwd": 12.0 * M * cfg.d * cfg.f / per_call["expert_ffn_bwd"] / 1e9},
        # activations held from the forward to the backward, beyond x itself and the routing tables
        "kept_activation_bytes": (M * 2 * cfg.f * 2 + M * 8) if args.fused else (M * 2 * cfg.f * 2 + 2 * M * cfg.d * (1 if fp8 else 2)
                                                                                   + (M * cfg.f * 2 if args.keep_a else 0)),
        "hbm_gbps": {"dispatch": dispatch_bytes / per_call["dispatch"] / 1e6 if "dispatch" in per_call else None,
                     "combine": combine_bytes / per_call["combine"] / 1e6,
                     "dispatch_bytes": dispatch_bytes, "combine_bytes": combine_bytes,
                     "peak": PEAK_HBM_GBPS,
                     "note": "this workload's row buffers may fit the 256 MB Infinity Cache; permute_large is the HBM figure"},
        "ms_per_call": per_call,
        "setup_s": setup_s,
        "launch": "one HIP graph per step" if args.graph else "eager",
    }
    if not args.no_permute_large:
        del layer
        torch.cuda.empty_cache()
        out["permute_large"] = permute_large("finegrained")
    if args.ceilings:
        out["ceilings"] = ceilings(cfg)
        key = "mfma_loop_fp8_random_tflops" if (fp8 and args.fp8_backward) else "mfma_loop_bf16_random_tflops"
        out["roofline"]["measured_ceiling"] = out["ceilings"][key]
        out["roofline"]["frac_of_measured_ceiling"] = gemm_tflops / out["ceilings"][key]
        if not fp8:
            # the same loop fed from LDS with the kernel's direct-to-LDS loads, waits and barriers beside it
            k_loop = out["ceilings"]["mfma_lds_fed_loop_with_loads_wait_barrier_tflops"]
            out["roofline"]["k_loop_ceiling"] = k_loop
            out["roofline"]["frac_of_k_loop_ceiling"] = gemm_tflops / k_loop
    if not args.no_cpu_baseline:
        tokens = args.cpu_tokens or max(cfg.T // 4, 1)
        out["cpu_baseline"] = (cpu_baseline_fp8(cfg, inp, tokens, args.fp8_backward) if fp8
                               else cpu_baseline(cfg, inp, tokens))
    print(json.dumps(out))


if __name__ == "__main__":
    main()
