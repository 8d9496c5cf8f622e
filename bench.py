#!/usr/bin/env python3
"""Throughput of spatio-temporal Monarch attention on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--iters T] [--no-cpu-baseline]

One step = one call of the whole path (every sweep's R-update and L-update, the apply-to-V
and the first-frame recomputation) on a seeded synthetic workload that is already resident
in HBM.  Prints ONE JSON line: effective TFLOP/s (algorithmic FLOPs of the method / time),
ms per call, the roofline position of the dominant kernel (the blocked-softmax R-update)
from HIP-event phase timings taken in this run, the HBM-bound L-update's GB/s, and the CPU
oracle timed on the host cores on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

BF16_MFMA_PEAK_TFLOPS = 2500.0   # MI355X dense bf16 (published)
HBM_PEAK_GBS = 8000.0            # MI355X HBM3E (published)


def cpu_baseline(wl, q_bits, k_bits, v_bits, positions=1024, rows=1024, min_seconds=12.0, max_heads=8):
    """The oracle as it stands: per head, `positions` query positions followed through the
    whole iteration (all T frames) plus `rows` first-frame rows recomputed exactly; heads are
    added until about `min_seconds` of CPU work have been timed."""
    import numpy as np
    from oracle import vmonarch_oracle as O

    rng = np.random.default_rng(5)
    pos = np.sort(rng.choice(wl.b, size=min(positions, wl.b), replace=False))
    T, b, d, N = wl.T, wl.b, wl.d, wl.N
    s = len(pos)
    per_head = s * ((wl.iters - 1) * 4 * T * b * d + 6 * T * b * d + wl.iters * 4 * T * T * d)
    if wl.recompute:
        per_head += min(rows, s) * 4 * N * d
    dt, flops, nheads = 0.0, 0.0, 0
    while dt < min_seconds and nheads < min(max_heads, len(q_bits)):
        q, k, v = (O.widen_bf16(x[nheads]) for x in (q_bits, k_bits, v_bits))
        t0 = time.perf_counter()
        O.monarch_attention(q, k, v, wl.T, wl.b, wl.iters, recompute=False, positions=pos)
        if wl.recompute:
            O.first_frame_attention(q, k, v, wl.b, rows=pos[:rows])
        dt += time.perf_counter() - t0
        flops += per_head
        nheads += 1
    try:
        cores = len(os.sched_getaffinity(0))
    except AttributeError:  # pragma: no cover
        cores = os.cpu_count() or 1
    omp = os.environ.get("OMP_NUM_THREADS")
    if omp and omp.isdigit():
        cores = min(cores, int(omp))
    return {
        "value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": cores, "kind": "oracle",
        "sample": f"{nheads} head(s), {s} of {b} query positions x all {T} frames through {wl.iters} sweeps"
                  + (f" + {min(rows, s)} first-frame rows over all {N} keys" if wl.recompute else "")
                  + f", fp64 NumPy, {dt:.1f} s",
        "seconds": dt,
    }


def mfma_probe(torch, binding, dev, cus=256, iters=20000):
    """Sustained rate of the bare bf16 matrix instruction with nothing else running, on all-zero and on
    random-normal operands: the device's matrix pipe is power-limited, so the second figure, not the
    published peak, is what a kernel fed with real data can reach at best."""
    res = {}
    g = torch.Generator(device="cpu")
    g.manual_seed(7)
    for name in ("zeros", "random_normal"):
        n = cus * 512 * 64
        ops = torch.zeros(n, dtype=torch.bfloat16) if name == "zeros" else torch.randn(n, generator=g).to(torch.bfloat16)
        ops = ops.to(dev)
        binding.mfma_probe(ops, cus, 1000)
        torch.cuda.synchronize()
        best = float("inf")
        for _ in range(3):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            _, fl = binding.mfma_probe(ops, cus, iters)
            e1.record()
            torch.cuda.synchronize()
            best = min(best, e0.elapsed_time(e1))
        res[name] = fl / (best * 1e-3) / 1e12
    return res


def recorded_traffic(kernel_that_ran):
    """HBM bytes per launch of the dominant kernel from the committed rocprofv3 --pmc summary (FETCH_SIZE and
    WRITE_SIZE runs scaled by a copy of known size), or None.  The summary names the kernel it was taken from:
    when another kernel ran (a different variant, a renamed or replaced kernel) the figure would be stale and is
    withheld."""
    path = os.path.join(ROOT, "profiles", "attention_long-81x28x52_hbm_traffic.txt")
    kernel, value = None, None
    try:
        for line in open(path):
            if line.startswith("dominant_kernel:"):
                kernel = line.split(":", 1)[1].strip()
            if line.startswith("dominant_kernel_hbm_bytes_per_launch:"):
                value = float(line.split(":", 1)[1])
    except OSError:
        return None
    if kernel is None or value is None or not kernel.startswith(kernel_that_ran):
        print(f"bench.py: profiles/ holds HBM traffic of '{kernel}', the dominant kernel of this run is "
              f"'{kernel_that_ran}': roofline.traffic withheld", file=sys.stderr)
        return None
    return value


def sweep_frames(args) -> int:
    """Context for the paper's speed-versus-length figure (Sec. 4.3): spatial size 28 x 52, T = 20 .. 48
    latent frames, 12 heads, d = 128, 2 sweeps + first-frame recomputation, against exact dense
    attention over the same tokens computed by this library's own blocked-softmax kernel (one
    "frame" holding all N tokens).  One JSON line per T."""
    import torch

    from paper_2601_22275_amd import binding, synth

    dev = torch.device("cuda:0")
    binding.lib()
    if args.flash_variant is not None:
        binding.set_flash_variant(args.flash_variant)
    heads, Hs, Ws, d = 12, 28, 52, 128
    for T in list(range(20, 49, 4)) + [81]:   # the figure's range, then the headline length
        wl = synth.Workload(f"sweep-{T}x28x52", 20 + T, 1, heads, T, Hs, Ws, d, "bf16", 2, True)
        q, k, v = synth.make_inputs(wl)
        tq, tk, tv = (torch.from_numpy(x).to(dev).view(torch.bfloat16).view(1, heads, wl.N, d) for x in (q, k, v))
        out = torch.empty_like(tq)

        def timed(f):
            for _ in range(args.warmup):
                f()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(args.steps):
                f()
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / args.steps

        ms_monarch = timed(lambda: binding.attention(tq, tk, tv, T, Hs, Ws, 2, True, out=out))
        ms_dense = timed(lambda: binding.first_frame_attention(tq, tk, tv, 1, 1, wl.N, out))
        fl = synth.algorithmic_flops(1, heads, T, wl.b, d, 2, True)
        print(json.dumps({"T": T, "N": wl.N, "monarch_ms": ms_monarch, "dense_ms": ms_dense,
                          "dense_over_monarch": ms_dense / ms_monarch, "monarch_tflops": fl / ms_monarch / 1e9,
                          "dense_tflops": 4.0 * heads * wl.N * wl.N * d / ms_dense / 1e9}), flush=True)
    return 0


def sweep_budget(args) -> int:
    """The paper's computation-budget study (App. "Various Monarch Computation Budgets"): N = 2^15 tokens as m blocks of
    b tokens for every power-of-two split from (8, 4096) to (512, 64), 12 heads, d = 64, 2 sweeps.  One JSON line per
    split: ms per call, the method's FLOPs for that split and the phase times."""
    import torch

    from paper_2601_22275_amd import binding, synth

    dev = torch.device("cuda:0")
    binding.lib()
    if args.flash_variant is not None:
        binding.set_flash_variant(args.flash_variant)
    for m, b in synth.BUDGET_SPLITS:
        wl = synth.WORKLOADS[f"budget-{m}x{b}"]
        q, k, v = synth.make_inputs(wl)
        tq, tk, tv = (torch.from_numpy(x).to(dev).view(torch.bfloat16).view(1, wl.heads, wl.N, wl.d) for x in (q, k, v))
        out = torch.empty_like(tq)
        ws = torch.empty(binding.workspace_bytes(1, wl.heads, wl.T, wl.Hs, wl.Ws, wl.d, wl.iters, wl.recompute, 2),
                         dtype=torch.uint8, device=dev)
        binding.set_workspace(ws)

        def step():
            binding.attention(tq, tk, tv, wl.T, wl.Hs, wl.Ws, wl.iters, wl.recompute, out=out)

        for _ in range(args.warmup):
            step()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(args.steps):
            step()
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / args.steps
        binding.set_phase_timing(True)
        acc = {}
        for _ in range(args.steps):
            step()
            for name, t in binding.get_phase_timing():
                acc.setdefault(name, []).append(t)
        binding.set_phase_timing(False)
        binding.set_workspace(None)
        fl = synth.algorithmic_flops(1, wl.heads, wl.T, wl.b, wl.d, wl.iters, wl.recompute)
        print(json.dumps({"m": m, "b": b, "N": wl.N, "ms": ms, "gflop_per_call": fl / 1e9, "tflops": fl / ms / 1e9,
                          "phase_ms": {n: sum(x) / len(x) for n, x in acc.items()}}), flush=True)
    return 0


def bench_backward(args) -> int:
    """Backward of one blocked-softmax pass with entropy (Alg. 2) on the workload's per-frame problems:
    dq, dk, dv for every (head, frame) from K, V, the forward outputs and seeded random dO, dH.  One JSON
    line; FLOPs counted as Alg. 2's five b x b x d products per problem (the three passes issue eight)."""
    import numpy as np
    import torch

    from paper_2601_22275_amd import binding, synth

    dev = torch.device("cuda:0")
    binding.lib()
    wl = synth.WORKLOADS[args.workload]
    q, k, v = synth.make_inputs(wl)
    tq, tk, tv = (torch.from_numpy(x).to(dev).view(torch.bfloat16).view(wl.B, wl.heads, wl.N, wl.d) for x in (q, k, v))
    g = torch.Generator(device="cpu")
    g.manual_seed(3)
    dO = torch.randn(wl.B, wl.heads, wl.N, wl.d, generator=g).to(torch.bfloat16).to(dev)
    dH = torch.randn(wl.B, wl.heads, wl.N, generator=g).to(dev)
    s = 1.0 / math.sqrt(wl.d)
    _, cL, y, lse = binding.r_update_lse(tq, None, tk, tv, wl.T, wl.Hs, wl.Ws, s, 0.1)
    H = (-cL).contiguous()

    def step():
        return binding.entropy_attention_bwd(tq, None, tk, tv, y, dO, lse, H, dH, wl.T, wl.Hs, wl.Ws, s, 0.1)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(args.steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / args.steps
    fl = 10.0 * wl.B * wl.heads * wl.T * wl.b * wl.b * wl.d
    print(json.dumps({"metric": "Alg. 2 backward of the blocked-softmax pass, TFLOP/s (five products per problem / time)",
                      "value": fl / ms / 1e9, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
                      "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
                      "dtype": "bf16", "data": "synthetic", "issued_tflops": 1.6 * fl / ms / 1e9,
                      "config": {"workload": wl.name, "heads": wl.heads, "T": wl.T, "b": wl.b, "d": wl.d}}))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="long-81x28x52")
    ap.add_argument("--iters", type=int, default=None,
                    help="number of alternating sweeps (default: the workload's; the 720p workload is also run with 1 and 3 "
                         "to separate the cost of a sweep)")
    ap.add_argument("--entropy", choices=["online", "identity"], default="online")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--flash-variant", type=int, choices=[0, 1, 2], default=None,
                    help="bf16 MFMA R-update kernels: 0 two waves per SIMD, 1 one wave per SIMD with two query tiles per "
                         "wave, 2 the latter for the update with values only (default: the library's setting)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one token-permutation copy of known size (reference for HBM byte counters)")
    ap.add_argument("--backward", action="store_true",
                    help="time the Alg. 2 backward of the workload's per-frame softmax blocks instead of the forward path")
    ap.add_argument("--graph", action="store_true",
                    help="capture one call in a HIP graph and time replays (for launch-bound small workloads)")
    ap.add_argument("--sweep-budget", action="store_true",
                    help="time the (m, b) splits of N = 2^15 tokens from (8, 4096) to (512, 64) instead of the benchmark")
    ap.add_argument("--sweep-frames", action="store_true",
                    help="time T = 20..48 frames of 28x52 tokens against exact dense attention instead of the benchmark")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no sharding, no collectives); use --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    from paper_2601_22275_amd import binding, synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    if args.sweep_frames:
        return sweep_frames(args)
    if args.sweep_budget:
        return sweep_budget(args)
    if args.backward:
        return bench_backward(args)
    binding.lib()  # fail loudly when the HIP library is missing
    wl = synth.WORKLOADS[args.workload]
    if args.iters is not None:
        if args.iters < 1:
            print("bench.py: --iters must be at least 1", file=sys.stderr)
            return 2
        import dataclasses
        wl = dataclasses.replace(wl, iters=args.iters)
    dev = torch.device("cuda:0")
    bf16 = wl.dtype == "bf16"

    t0 = time.perf_counter()
    q, k, v = synth.make_inputs(wl)
    gen_s = time.perf_counter() - t0

    def up(x):
        t = torch.from_numpy(x).to(dev)
        if bf16:
            t = t.view(torch.bfloat16)
        return t.view(wl.B, wl.heads, wl.N, wl.d)

    tq, tk, tv = up(q), up(k), up(v)
    out = torch.empty_like(tq)
    ws_bytes = binding.workspace_bytes(wl.B, wl.heads, wl.T, wl.Hs, wl.Ws, wl.d, wl.iters, wl.recompute, 2 if bf16 else 4)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
    binding.set_workspace(ws)
    binding.set_entropy_mode(binding.ENTROPY_IDENTITY if args.entropy == "identity" else binding.ENTROPY_ONLINE)
    if args.flash_variant is not None:
        binding.set_flash_variant(args.flash_variant)

    def eager_step():
        binding.attention(tq, tk, tv, wl.T, wl.Hs, wl.Ws, wl.iters, wl.recompute, out=out)

    step = eager_step
    if args.graph:
        # the call only enqueues kernels once the workspace is the caller's: capture it once, replay it
        eager_step()
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            eager_step()
        step = graph.replay

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # ---- timed region: exactly K steps, inputs resident, events on the launch stream ----
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    evs[0].record()
    for i in range(args.steps):
        step()
        evs[i + 1].record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    per_step = sorted(evs[i].elapsed_time(evs[i + 1]) for i in range(args.steps))
    ms = wall * 1e3 / args.steps
    flops = synth.algorithmic_flops(wl.B, wl.heads, wl.T, wl.b, wl.d, wl.iters, wl.recompute)
    tflops = flops / (ms * 1e-3) / 1e12

    # ---- per-phase durations of the same call, HIP events recorded by the library between
    # its kernels on this stream (a second, instrumented pass over K steps)
    binding.set_phase_timing(True)
    phase_ms = {}
    for _ in range(args.steps):
        eager_step()
        for name, t in binding.get_phase_timing():
            phase_ms.setdefault(name, []).append(t)
    binding.set_phase_timing(False)
    phases = {n: sum(x) / len(x) for n, x in phase_ms.items()}

    BH, T, b, d, N = wl.B * wl.heads, wl.T, wl.b, wl.d, wl.N
    elem = 2 if bf16 else 4
    roofline = None
    hbm_phase = None
    variant = binding.get_flash_variant()
    fused = bf16 and d in (64, 128) and args.entropy == "online" and binding.get_fused_apply() and variant == 0
    if "r_update_last" in phases:
        # dominant kernel (the longest single launch of a call): the R-update of the last sweep, which forms
        # the logits, R K (alpha_L), c_L and R V (y) in one launch: three b x b x d products per frame.
        # (With the two-pass form the phase is two launches.)
        fl, t_ms = 6.0 * BH * T * b * b * d, phases["r_update_last"]
        if bf16 and d in (64, 128) and variant in (1, 2):
            kern, what = "flash2_kernel", "flash2_kernel (last R-update: logits, R K, c_L and R V in one launch, one wave per SIMD)"
        elif fused:
            kern, what = "flash_kv_kernel", "flash_kv_kernel (last R-update: logits, R K, c_L and R V in one launch)"
        else:
            kern, what = "flash_kernel", "R-update of the last sweep (two launches: R K pass and R V pass)"
        ach = fl / (t_ms * 1e-3) / 1e12
        roofline = {"bound": "mfma", "achieved": ach, "peak": BF16_MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                    "frac": ach / BF16_MFMA_PEAK_TFLOPS,
                    "traffic": recorded_traffic(kern) if wl.name == "long-81x28x52" and wl.iters == 2 and d == 128 else None,
                    "kernel": what,
                    "flops_per_launch": fl, "ms_per_launch": t_ms}
        if "r_update" in phases:
            # the fitting sweeps' R-update (logits + R K), one launch each
            fl2, t2 = 4.0 * BH * T * b * b * d, phases["r_update"]
            two_tiles = variant == 1 or (variant == 2 and d == 64)
            roofline["fitting_r_update"] = {"kernel": "flash2_kernel (logits + R K)" if two_tiles else "flash_kernel (logits + R K)",
                                            "flops_per_launch": fl2,
                                            "ms_per_launch": t2, "achieved": fl2 / (t2 * 1e-3) / 1e12,
                                            "frac": fl2 / (t2 * 1e-3) / 1e12 / BF16_MFMA_PEAK_TFLOPS}
        if "first_frame" in phases:
            fl3, t3 = 4.0 * BH * b * N * d, phases["first_frame"]
            ff_kernel = "flash2_kernel" if bf16 and d in (64, 128) and variant != 0 else "flash_kernel"
            roofline["first_frame"] = {"kernel": ff_kernel + " over key ranges + merge (exact attention of frame 0)",
                                       "flops_per_launch": fl3, "ms_per_launch": t3,
                                       "achieved": fl3 / (t3 * 1e-3) / 1e12,
                                       "frac": fl3 / (t3 * 1e-3) / 1e12 / BF16_MFMA_PEAK_TFLOPS}

    def hbm(kernel, by, t_ms):
        return {"kernel": kernel, "bytes_per_launch": by, "ms_per_launch": t_ms, "achieved": by / (t_ms * 1e-3) / 1e9,
                "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": by / (t_ms * 1e-3) / 1e9 / HBM_PEAK_GBS}

    hbm_phase = {}
    if "l_update" in phases:
        # fitting L-update: reads q and alpha_L, writes alpha_R (3 token tensors); reads c_L, writes c_R
        hbm_phase["l_update"] = hbm("L-update of a fitting sweep (q, alpha_L, c_L -> alpha_R, c_R)",
                                    3.0 * BH * N * d * elem + 2.0 * BH * N * 4, phases["l_update"])
    if "l_update_last" in phases:
        # final L-update: reads q, alpha_L, y, writes out (4 token tensors); reads c_L
        hbm_phase["l_update_last"] = hbm("L-update of the last sweep with the apply-to-V (q, alpha_L, c_L, y -> out)",
                                         4.0 * BH * N * d * elem + 1.0 * BH * N * 4, phases["l_update_last"])
    # the stride permutation as a stand-alone copy (never on the fused path): reads and writes every token row once
    perm_out = torch.empty_like(tq)
    binding.permute_tokens(tq, wl.T, wl.Hs, wl.Ws, True, out=perm_out)
    torch.cuda.synchronize()
    pe = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    nperm = max(3, min(args.steps, 10))
    pe[0].record()
    for _ in range(nperm):
        binding.permute_tokens(tq, wl.T, wl.Hs, wl.Ws, True, out=perm_out)
    pe[1].record()
    torch.cuda.synchronize()
    hbm_phase["permute_tokens"] = hbm("vmonarch_permute_tokens, frame-major -> position-major copy of q",
                                      2.0 * BH * N * d * elem, pe[0].elapsed_time(pe[1]) / nperm)
    # context, not a kernel of this library: the runtime's own device-to-device copy of the same tensor
    pe[0].record()
    for _ in range(nperm):
        perm_out.copy_(tq)
    pe[1].record()
    torch.cuda.synchronize()
    hbm_phase["device_copy"] = hbm("device-to-device copy of q by the HIP runtime (context: what a plain copy reaches)",
                                   2.0 * BH * N * d * elem, pe[0].elapsed_time(pe[1]) / nperm)
    del perm_out

    if args.copy_calibration:
        # reads and writes B*heads*N*d*elem bytes each: the yardstick for FETCH_SIZE / WRITE_SIZE
        binding.permute_tokens(tq, wl.T, wl.Hs, wl.Ws, True)
        torch.cuda.synchronize()

    probe = mfma_probe(torch, binding, dev, torch.cuda.get_device_properties(0).multi_processor_count)
    if roofline is not None:
        roofline["sustained_mfma_tflops"] = probe
        roofline["frac_of_sustained_random"] = roofline["achieved"] / probe["random_normal"]

    cpu = None
    if not args.no_cpu_baseline and bf16:
        cpu = cpu_baseline(wl, q, k, v)

    rec = {
        "metric": "spatio-temporal Monarch attention, effective TFLOP/s (algorithmic FLOPs / time per call)",
        "value": tflops, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms, "ms_per_step_median": per_step[len(per_step) // 2], "ms_per_step_min": per_step[0],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if bf16 else "f32", "data": "synthetic",
        "pct_bf16_mfma_peak": 100.0 * tflops / BF16_MFMA_PEAK_TFLOPS,
        "algorithmic_tflop_per_call": flops / 1e12,
        "config": {"workload": wl.name, "B": wl.B, "heads": wl.heads, "T": wl.T, "Hs": wl.Hs, "Ws": wl.Ws,
                   "N": wl.N, "d": wl.d, "iters": wl.iters, "recompute": bool(wl.recompute),
                   "entropy": args.entropy, "flash_variant": variant, "launch": "hip graph replay" if args.graph else "eager",
                   "input_generation_s": gen_s},
        "phase_ms": phases,
        "roofline": roofline,
        "hbm_phase": hbm_phase,
        "cpu_baseline": cpu,
    }
    print(json.dumps(rec))
    return 0


if __name__ == "__main__":
    sys.exit(main())
