#!/usr/bin/env python3
"""Benchmark of the transposable N:M mask finder on one MI355X.

One "step" is one pass of the whole hot path (matrix maximum, tile load, all T Dykstra iterations, sort, greedy
selection, local search, mask write) = one call of tsenor_mask_ex over the headline workload: transposable 16:32
on a 4096x14336 bf16 matrix with Wanda-style importance, T = 300, entropy weight 0.005 * max importance.
Inputs are synthetic (seeded) and already resident in HBM when the timed region starts.

Prints ONE JSON line: whole-job throughput in masked weights/s over the timed tsenor_mask_ex calls, the roofline
of the dominant kernel (its duration from HIP events at the stage boundaries of a second, equally long run of
the same calls), and the CPU oracle timed on a bounded sample.  `--workload all` measures every configuration,
writes one such line per configuration into --out-dir and prints the headline one.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "masked weights/s (Dykstra+rounding), 16:32 @4096x14336; % of roofline"
HEADLINE = "cfg3_16of32_4096x14336"

# ---- roofline of the dominant kernel (tile load + Algorithm 1 + sort): bound by vector-ALU issue ---------------
# Useful work: the vector operations per matrix entry and Dykstra iteration that the linear-domain form of
# Algorithm 1 needs: capped entry (multiply with clamp), row-sum add, column-sum multiply-add, row rescale of the
# entry = 4 (a multiply-add counts once: it is one issue slot).
# Peak: one double-precision wave instruction per SIMD every 4 cycles = 16 lanes/clk/SIMD:
# 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz = 39.32 T lane-operations/s (the published 78.6 TFLOP/s counts every
# operation as a multiply-add, i.e. twice).
PEAK_F64_TLANEOPS = 256 * 4 * 16 * 2.4e9 / 1e12
# Single-precision iterations (TSENOR_FLAG_FP32_ITERATIONS): packed fp32 instructions are not used, and the rate
# measured on this chip for plain v_mul_f32 / v_add_f32 / v_fma_f32 is 48-57 T lane-operations/s
# (profiles/issue_rates_mi355x.md); the upper end is taken as the peak.
PEAK_F32_PLAIN_TLANEOPS = 57.0
# A coarser model of the method (5 full-rate vector operations + 1 quarter-rate exponential per entry and
# iteration = 9 lane-cycles), kept only as a comparison figure: this kernel has no transcendental in its loop.
NINE_OP_MODEL_LANE_OPS = 9.0


def useful_ops_per_entry_iter(M: int, fp32: bool) -> float:
    # (the double-precision mode of the 64 x 64 kernel cannot keep the capped entries in registers and computes
    # them twice)
    return 5.0 if (M == 64 and not fp32) else 4.0


# Vector instructions the compiled default-mode iteration loop issues per wave and iteration, and the matrix
# entries a wave holds (counted in the ISA of the built library, `v_*` lines between the loop label and its
# branch; cross-lane ds_swizzle and LDS accesses issue on another pipeline and are not counted).  Keyed by
# (M, small tiles).
LOOP_VALU_PER_WAVE_ITER = {
    (4, False): (108, 1024), (4, True): (36, 256), (8, False): (104, 1024), (8, True): (40, 256),
    (16, False): (176, 2048), (16, True): (98, 1024), (32, False): (164, 2048), (32, True): (110, 1024),
    (64, False): (384, 4096),
}
# a matrix with fewer blocks than this runs the small-tile instantiation (the library's own choice, mirrored here
# only to pick the row of the table above)
SMALL_TILES_BELOW_BLOCKS = {False: {4: 100000, 8: 13000, 16: 40000, 32: 3200, 64: 0},     # default mode
                            True: {4: 55000, 8: 12000, 16: 9000, 32: 2100, 64: 0}}         # with the fp32 flag


def recorded_traffic(workload: str, fp32: bool):
    """HBM bytes of the dominant kernel and of the whole pass, per launch, as recorded in the committed
    rocprofv3 summary of this workload (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, scaled by a copy of known size;
    not measured in this run)."""
    out = {"kernel": None, "pass": None}
    tag = "fp32" if fp32 else "fp64"
    path = os.path.join(ROOT, "profiles", f"all_kernels_{workload}.md")
    try:
        for line in open(path):
            if line.startswith(f"traffic_bytes_per_launch dykstra_sort_kernel {tag}"):
                out["kernel"] = int(line.split(":")[1])
            if line.startswith(f"traffic_bytes_per_pass {tag}"):
                out["pass"] = int(line.split(":")[1])
    except OSError:
        pass
    return out


def cpu_model() -> str:
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def timed_calls(torch, fn, steps):
    """`steps` calls of fn enqueued back to back, bracketed by a device synchronisation on both sides.
    Returns (wall ms per step, HIP-event ms per step on the current stream)."""
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    start.record()
    for _ in range(steps):
        fn()
    stop.record()
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t0) * 1e3 / steps
    return wall, start.elapsed_time(stop) / steps


def per_pass_ms(torch, fn, trials):
    """`trials` calls of fn, each between its own pair of events on the current stream (enqueued back to back, one
    synchronisation at the end).  Returns (median, min) in ms: the per-trial statistics beside the mean."""
    pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(trials)]
    torch.cuda.synchronize()
    for a, b in pairs:
        a.record()
        fn()
        b.record()
    torch.cuda.synchronize()
    ms = sorted(a.elapsed_time(b) for a, b in pairs)
    mid = len(ms) // 2
    return (ms[mid] if len(ms) % 2 else 0.5 * (ms[mid - 1] + ms[mid])), ms[0]


def bench_layer(args):
    """Secondary workload: the seven projection matrices of one 8B decoder layer (fp32, 16:32, Wanda-style
    importance) through ONE tsenor_mask_batched call per step.  Wall-clock only (no per-kernel split)."""
    import torch

    from paper_2505_23949_amd import binding, synth

    dev = torch.device("cuda:0")
    ws = synth.layer_workloads(0)
    keep, probs = [], []
    for w in ws:
        g = synth.generate(w)
        W = torch.from_numpy(g["W_store"]).to(dev)
        cs = torch.from_numpy(g["col_scale"]).to(dev)
        mask = torch.empty(W.shape, dtype=torch.uint8, device=dev)
        flags = binding.TSENOR_FLAG_FP32_ITERATIONS if args.precision == "fp32" else 0
        probs.append(binding.make_problem(W, w.N, w.M, w.tau, w.iters, mask=mask, col_scale=cs, tau_mode=w.tau_mode,
                                          flags=flags, tol=args.tol))
        keep += [W, cs, mask]
    work = torch.empty(binding.tsenor_workspace_bytes(probs), dtype=torch.uint8, device=dev)
    for _ in range(args.warmup):
        binding.tsenor_mask_batched(probs, work)
    ms_per_step, ms_events = timed_calls(torch, lambda: binding.tsenor_mask_batched(probs, work), args.steps)
    ms_median, ms_min = per_pass_ms(torch, lambda: binding.tsenor_mask_batched(probs, work), max(args.steps, 10))
    weights = sum(w.rows * w.cols for w in ws)
    return {
        "metric": "masked weights/s (Dykstra+rounding), 16:32, one 8B decoder layer per batched call",
        "value": round(weights / (ms_per_step * 1e-3), 1), "unit": "masked weights/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "ms_per_step_hip_events": round(ms_events, 4), "ms_per_step_median": round(ms_median, 4),
        "ms_per_step_min": round(ms_min, 4), "trials": max(args.steps, 10), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32" if args.precision == "fp32" else "f64",
        "data": "synthetic",
        "config": {"workload": "cfg4_layer", "matrices": [[w.rows, w.cols] for w in ws], "weights": weights,
                   "N": 16, "M": 32, "iters": 300, "tau": 0.005, "tau_mode": "rel_matrix_max", "storage": "f32",
                   "importance": "wanda", **({"tol": args.tol} if args.tol > 0.0 else {})},
        "roofline": None, "cpu_baseline": None,
    }


def bench_slab_loop(args):
    """Secondary workload, the call shape of a column-by-column pruning loop (Sec. 4, SparseGPT integration): the
    headline matrix taken M columns at a time, cols/M dependent tsenor_mask_ex calls of a rows x M slab each on
    one stream (here every slab is solved under its own matrix maximum)."""
    import numpy as np
    import torch

    from paper_2505_23949_amd import binding, synth

    dev = torch.device("cuda:0")
    w = synth.CONFIGS[HEADLINE]
    g = synth.generate(w)
    W = torch.from_numpy(g["W_store"].view(np.int16)).to(dev).view(torch.bfloat16)
    cs = torch.from_numpy(g["col_scale"]).to(dev)
    mask = torch.empty(W.shape, dtype=torch.uint8, device=dev)
    nslabs = w.cols // w.M
    probs = []
    for k in range(nslabs):
        sl = slice(k * w.M, (k + 1) * w.M)
        # the mask slab is a strided view: the library writes masks with leading dimension `cols` of the problem,
        # so every slab gets a contiguous buffer of its own
        probs.append((W[:, sl], cs[sl]))
    slab_masks = torch.empty((nslabs, w.rows, w.M), dtype=torch.uint8, device=dev)
    plist = [binding.make_problem(Wk, w.N, w.M, w.tau, w.iters, mask=slab_masks[k], col_scale=ck,
                                  tau_mode=w.tau_mode) for k, (Wk, ck) in enumerate(probs)]
    work = torch.empty(binding.tsenor_workspace_bytes([plist[0]]), dtype=torch.uint8, device=dev)

    def one_pass():
        for p in plist:
            binding.tsenor_mask_ex(p, work)

    for _ in range(max(args.warmup // 2, 1)):
        one_pass()
    steps = max(args.steps // 4, 1)
    ms_per_step, ms_events = timed_calls(torch, one_pass, steps)
    ms_median, ms_min = per_pass_ms(torch, one_pass, 10)
    weights = w.rows * w.cols
    return {
        "metric": f"masked weights/s, {w.N}:{w.M}, {nslabs} dependent calls of a {w.rows}x{w.M} slab",
        "value": round(weights / (ms_per_step * 1e-3), 1), "unit": "masked weights/s", "n_gpus": 1,
        "steps": steps, "warmup": max(args.warmup // 2, 1), "ms_per_step": round(ms_per_step, 4),
        "ms_per_step_hip_events": round(ms_events, 4), "ms_per_step_median": round(ms_median, 4),
        "ms_per_step_min": round(ms_min, 4), "trials": 10, "ms_per_call": round(ms_per_step / nslabs, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f64", "data": "synthetic",
        "config": {"workload": "slab_loop", "rows": w.rows, "cols": w.cols, "N": w.N, "M": w.M, "iters": w.iters,
                   "tau": w.tau, "tau_mode": "rel_matrix_max (per slab)", "storage": w.dtype, "importance": w.dist,
                   "calls_per_step": nslabs},
        "roofline": None, "cpu_baseline": None,
    }


def bench_matrix(args, name):
    import numpy as np
    import torch
    from dataclasses import replace

    from paper_2505_23949_amd import binding, synth

    w = synth.CONFIGS[name]
    if args.rows and args.cols:
        w = w.scaled(args.rows, args.cols)
    if args.iters >= 0:
        w = replace(w, iters=args.iters)
    if args.absolute_tau:
        w = replace(w, tau_mode=synth.TAU_ABSOLUTE)
    dev = torch.device("cuda:0")
    g = synth.generate(w)
    if w.dtype == "bf16":
        W = torch.from_numpy(g["W_store"].view(np.int16)).to(dev).view(torch.bfloat16)
    else:
        W = torch.from_numpy(g["W_store"]).to(dev)
    cs = None if g["col_scale"] is None else torch.from_numpy(g["col_scale"]).to(dev)
    weights = w.rows * w.cols
    nblocks = weights // (w.M * w.M)
    steps = args.steps
    fp32_flag = binding.TSENOR_FLAG_FP32_ITERATIONS
    # a matrix this small runs on the small tiles, which iterate in double whatever the flag says
    small_launch = nblocks < SMALL_TILES_BELOW_BLOCKS[True][w.M]
    headline_fp32 = args.precision == "fp32" and not small_launch
    no_cpu, no_modes = args.no_cpu_baseline, args.no_other_modes
    if args.tol > 0.0:
        no_cpu = no_modes = True

    if args.calibrate_copy:
        ref_in = torch.zeros(64 * 1024 * 1024, dtype=torch.float32, device=dev)
        ref_out = torch.empty_like(ref_in)
        torch.add(ref_in, 1.0, out=ref_out)
        torch.cuda.synchronize()
        del ref_in, ref_out

    entry_iters = float(weights) * w.iters
    esize = 2 if w.dtype == "bf16" else 4
    work = None

    def run_mode(fp32, tol=0.0):
        """One mode of the library on the workload: `steps` timed calls of tsenor_mask_ex, then the same number of
        passes with events at the stage boundaries.  Returns its part of the bench line and its mask."""
        nonlocal work
        mask = torch.empty(W.shape, dtype=torch.uint8, device=dev)
        done = torch.zeros(nblocks, dtype=torch.int32, device=dev) if tol > 0.0 else None
        prob = binding.make_problem(W, w.N, w.M, w.tau, w.iters, mask=mask, col_scale=cs, tau_mode=w.tau_mode,
                                    flags=fp32_flag if fp32 else 0, tol=tol, iters_done_out=done)
        if work is None:
            work = torch.empty(binding.tsenor_workspace_bytes([prob]), dtype=torch.uint8, device=dev)
        # A settling run of `steps` passes comes first: the chip's clock takes some tens of milliseconds of load to
        # settle after the idle time of the set-up (kernel durations fall by ~10 % over the first 15-20 passes).
        # Then the warm-up steps, the timed region, and the staged run (events at the stage boundaries).
        binding.tsenor_mask_ex_profile(prob, work, steps)
        for _ in range(args.warmup):
            binding.tsenor_mask_ex(prob, work)
        # ---- timed region: exactly `steps` calls of tsenor_mask_ex, enqueued back to back on the current stream
        ms_per_step, ms_events = timed_calls(torch, lambda: binding.tsenor_mask_ex(prob, work), steps)
        # (outside the timed region) the same call trial by trial, for the median and the minimum
        ms_median, ms_min = per_pass_ms(torch, lambda: binding.tsenor_mask_ex(prob, work), max(steps, 10))
        stage_ms, clock_mhz = binding.tsenor_mask_ex_profile(prob, work, steps, want_clock=True)
        dyk_ms = stage_ms[1]
        out = {"dtype": "f32" if fp32 else "f64", "value": round(weights / (ms_per_step * 1e-3), 1),
               "ms_per_step": round(ms_per_step, 4), "ms_per_step_hip_events": round(ms_events, 4),
               "ms_per_step_median": round(ms_median, 4), "ms_per_step_min": round(ms_min, 4),
               "trials": max(steps, 10)}
        if tol > 0.0:
            out.update({"tol": tol, "mean_iterations": round(float(done.float().mean()), 1),
                        "kernel_ms": round(dyk_ms, 4)})
            return out, mask
        ops = useful_ops_per_entry_iter(w.M, fp32)
        achieved = ops * entry_iters / (dyk_ms * 1e-3) / 1e12
        peak = PEAK_F32_PLAIN_TLANEOPS if fp32 else PEAK_F64_TLANEOPS
        plain = not (args.rows or args.absolute_tau or args.iters >= 0)
        traffic = recorded_traffic(w.name, fp32) if plain else {"kernel": None, "pass": None}
        roofline = {
            "bound": "alu", "kernel": f"dykstra_sort_kernel<{w.M}{', fp32 iterations' if fp32 else ''}>",
            "achieved": round(achieved, 3), "peak": round(peak, 3), "unit": "T lane-ops/s",
            "frac": round(achieved / peak, 4), "traffic": traffic["kernel"], "kernel_ms": round(dyk_ms, 4),
            "useful_ops_per_entry_iteration": ops,
            "note": ("bound by vector-ALU issue, not memory. achieved = useful vector operations (a multiply-add is "
                     "one) x rows x cols x T / kernel time, kernel time from HIP events at the stage boundaries of "
                     f"{steps} back-to-back passes; peak = "
                     + ("the rate measured on this chip for plain (unpacked) fp32 multiplies and adds; the published "
                        "157.3 TFLOP/s (78.6 T multiply-adds/s) needs the packed instructions, which are not used"
                        if fp32 else "256 CUs x 4 SIMDs x 16 lanes/clk x 2.4 GHz, the fp64 vector issue rate")
                     + "; traffic = HBM bytes per launch recorded in profiles/ (rocprofv3 --pmc FETCH_SIZE, "
                       "WRITE_SIZE), not measured in this run"),
            "stage_ms": {n: round(v, 4) for n, v in zip(binding.STAGE_NAMES, stage_ms)},
            "staged_ms_per_step": round(sum(stage_ms), 4),
            "shader_clock_mhz_in_loop": round(clock_mhz, 1),
            "vs_9op_model": round(NINE_OP_MODEL_LANE_OPS * entry_iters / (dyk_ms * 1e-3) / 1e12 / peak, 4),
            "algorithmic_bytes_per_pass": weights * (esize + 1) + (0 if cs is None else 4 * w.cols),
            "pass_traffic_recorded_in_profiles": traffic["pass"],
        }
        if fp32:
            roofline["frac_of_published_fp32_vector_rate"] = round(achieved / (2 * PEAK_F64_TLANEOPS), 4)
        if traffic["pass"]:
            roofline["pass_traffic_over_algorithmic"] = round(
                traffic["pass"] / roofline["algorithmic_bytes_per_pass"], 2)
        if not fp32 and w.iters > 0:
            small = nblocks < SMALL_TILES_BELOW_BLOCKS[False][w.M]
            counted = LOOP_VALU_PER_WAVE_ITER.get((w.M, small))
            if counted:
                # second view of the same measurement: the vector instructions the loop issues against the issue
                # slots of the chip (1024 SIMDs, one double-precision wave instruction per 4 cycles), at the
                # peak clock and at the clock the kernel's first wave saw
                per_wave, entries = counted
                issued = per_wave * (weights / entries) * w.iters
                roofline["loop_valu_per_wave_iteration"] = per_wave
                roofline["loop_issue_frac_of_peak_clock"] = round(issued / (1024 * (dyk_ms * 1e-3) * 2.4e9 / 4.0), 4)
                if clock_mhz > 0:
                    roofline["loop_issue_frac_of_held_clock"] = round(
                        issued / (1024 * (dyk_ms * 1e-3) * clock_mhz * 1e6 / 4.0), 4)
        out["roofline"] = roofline
        return out, mask

    def same_blocks(a, b):
        diff = (a != b).view(w.rows // w.M, w.M, w.cols // w.M, w.M).any(dim=3).any(dim=1)
        return round(1.0 - float(diff.float().mean()), 6)

    # the optional modes first, the headline mode last
    other_mode = early_exit = early_exit32 = None
    if not no_modes:
        if small_launch:
            other_mode, mask_o = None, None
        else:
            other_mode, mask_o = run_mode(not headline_fp32)
        early_exit, mask_e = run_mode(False, 1e-5)
        early_exit32, mask_e32 = run_mode(True, 1e-5)
    if args.tol > 0.0:
        main_mode, mask = run_mode(headline_fp32, args.tol)
        main_mode["roofline"] = None
    else:
        main_mode, mask = run_mode(headline_fp32)
    if not no_modes:
        if other_mode is not None:
            other_mode["blocks_identical_to_headline_mode"] = same_blocks(mask_o, mask)
        early_exit["blocks_identical_to_headline_mode"] = same_blocks(mask_e, mask)
        early_exit32["blocks_identical_to_headline_mode"] = same_blocks(mask_e32, mask)
        del mask_o, mask_e, mask_e32

    # the rounding counters of the headline mode, from a call of its own (asking for them adds two tiny kernels)
    stats = torch.zeros(4, dtype=torch.int64, device=dev)
    binding.tsenor_mask_ex(binding.make_problem(W, w.N, w.M, w.tau, w.iters, mask=torch.empty_like(mask), col_scale=cs,
                                                tau_mode=w.tau_mode, flags=fp32_flag if headline_fp32 else 0,
                                                stats_out=stats, tol=args.tol), work)
    torch.cuda.synchronize()
    stats_host = stats.cpu().numpy().tolist()
    mask_host = mask.cpu().numpy()          # host copy of the result for the check against the oracle below

    cpu_baseline = None
    if not no_cpu:
        import oracle
        from oracle import exact

        imp = oracle.importance(g["W_f32"], g["col_scale"])
        te = oracle.tau_eff(imp, w.tau, w.tau_mode)       # the matrix maximum is taken over the whole matrix
        nthreads = oracle.num_threads()

        def cpu_leg(rows_s, threads):
            oracle.set_threads(threads)
            imp_s = np.ascontiguousarray(imp[:rows_s])
            t0 = time.perf_counter()
            log_S = oracle.dykstra(imp_s, w.N, w.M, te, w.iters)
            m_ref, _ = oracle.round_plan(log_S, imp_s, w.N, w.M)
            secs = time.perf_counter() - t0
            same = (exact.blocks(m_ref, w.M) == exact.blocks(mask_host[:rows_s], w.M)).all(axis=(1, 2))
            return secs, int(same.sum()), int(same.size)

        # bounded samples: about 10 s on all threads and about 10 s on one (the oracle does ~6e6 weights/s on
        # 16 threads and ~4e5 on one thread for the 16:32 workload; the other block sizes are within 2x)
        per_weight = max(w.iters, 1) / 300.0
        rows_all = max(w.M, min(w.rows, int(6.0e7 / per_weight / w.cols) // w.M * w.M))
        rows_one = max(w.M, min(w.rows, int(3.7e6 / per_weight / w.cols) // w.M * w.M))
        if args.cpu_sample_rows:
            rows_all = max(w.M, min(w.rows, args.cpu_sample_rows // w.M * w.M))
        secs_all, same_all, blocks_all = cpu_leg(rows_all, nthreads)
        secs_one, same_one, blocks_one = cpu_leg(rows_one, 1)
        oracle.set_threads(nthreads)
        cpu_baseline = {
            "value": round(rows_all * w.cols / secs_all, 1), "unit": "masked weights/s", "cores": nthreads,
            "kind": "oracle",
            "sample": f"first {rows_all} rows of the {w.rows}x{w.cols} matrix ({rows_all * w.cols} weights, "
                      f"{secs_all:.1f} s on {nthreads} threads), tau_eff from the whole matrix",
            "one_thread": {"value": round(rows_one * w.cols / secs_one, 1), "cores": 1,
                           "sample": f"first {rows_one} rows ({rows_one * w.cols} weights, {secs_one:.1f} s)"},
            "cpu_model": cpu_model(), "host_cpus_visible": os.cpu_count(),
            "compiler": "gcc -O2 -std=c99 -fopenmp, no fast-math; OpenMP over blocks",
            "gpu_mask_equals_oracle_on_sample": same_all == blocks_all and same_one == blocks_one,
            "gpu_blocks_identical_to_oracle_on_sample": [same_all, blocks_all],
        }

    headline = w.name == HEADLINE and (w.rows, w.cols) == (4096, 14336) and not args.absolute_tau
    precision = ("iterations after the fourth in fp32 (TSENOR_FLAG_FP32_ITERATIONS); first four iterations, sort "
                 "keys and swap scores in fp64" if headline_fp32 else
                 "fp64 throughout (a launch this small runs on the small tiles, to which the fp32 flag does not apply)"
                 if small_launch else "fp64 throughout (the library's default)")
    return {
        "metric": METRIC if headline else
        f"masked weights/s (Dykstra+rounding), {w.N}:{w.M} @{w.rows}x{w.cols}; % of roofline",
        "value": main_mode["value"], "unit": "masked weights/s", "n_gpus": 1, "steps": steps,
        "warmup": args.warmup, "ms_per_step": main_mode["ms_per_step"],
        "ms_per_step_hip_events": main_mode["ms_per_step_hip_events"],
        "ms_per_step_median": main_mode["ms_per_step_median"], "ms_per_step_min": main_mode["ms_per_step_min"],
        "trials": main_mode["trials"],
        "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": main_mode["dtype"], "data": "synthetic",
        "config": {"workload": w.name, "rows": w.rows, "cols": w.cols, "N": w.N, "M": w.M, "iters": w.iters,
                   "tau": w.tau, "tau_mode": "rel_matrix_max" if w.tau_mode else "absolute",
                   "storage": w.dtype, "importance": w.dist, "precision": precision, "rounding_stats": stats_host,
                   **({"tol": args.tol, "mean_iterations": main_mode["mean_iterations"]} if args.tol > 0.0 else {})},
        "roofline": main_mode["roofline"], "cpu_baseline": cpu_baseline,
        ("fp64_mode" if headline_fp32 else "fp32_iterations_mode"): other_mode,
        "early_exit_mode": early_exit, "early_exit_fp32_mode": early_exit32,
    }


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default=HEADLINE,
                    help="a configuration name, cfg4_layer, slab_loop, or all (one line per configuration into "
                         "--out-dir, the headline line on stdout)")
    ap.add_argument("--out-dir", default=os.path.join(ROOT, "gpurun_out"),
                    help="where --workload all writes bench_<name>.json")
    ap.add_argument("--rows", type=int, default=0, help="override rows (debug)")
    ap.add_argument("--cols", type=int, default=0, help="override cols (debug)")
    ap.add_argument("--iters", type=int, default=-1, help="override the iteration count T (debug)")
    ap.add_argument("--absolute-tau", action="store_true",
                    help="secondary line: K = tau * importance as Algorithm 1 prints it, with the workload's "
                         "coefficient as tau (no matrix-maximum pre-pass; a nearly flat kernel)")
    ap.add_argument("--tol", type=float, default=0.0,
                    help="early exit of the iterations (tsenor_problem.tol); not the headline configuration, the "
                         "CPU baseline and the other modes are skipped with it")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-rows", type=int, default=0,
                    help="rows of the matrix the CPU oracle is timed on with all threads (default: sized for ~10 s)")
    ap.add_argument("--precision", choices=("fp32", "fp64"), default="fp32",
                    help="arithmetic of the Dykstra iterations in the headline figure: fp32 (the precision the method "
                         "is run at, TSENOR_FLAG_FP32_ITERATIONS; checked to plan 1e-4 / 99.9 %% of blocks / 1e-5 "
                         "retained importance against the fp64 oracle) or fp64 (the library's default: masks equal "
                         "to the oracle's by construction).  The other one is reported beside it")
    ap.add_argument("--no-other-modes", "--no-fp32-mode", dest="no_other_modes", action="store_true",
                    help="skip the secondary timings of the optional modes (for profiling runs)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one elementwise pass over 256 MiB (reads 256 MiB, writes 256 MiB): the "
                         "known-size reference for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE readings")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (blocks are independent, so the path would shard by "
              "block range with no communication); run with --gpus 1", file=sys.stderr)
        return 2

    from paper_2505_23949_amd import binding, synth

    binding.load()

    def run(name):
        if name == "cfg4_layer":
            return bench_layer(args)
        if name == "slab_loop":
            return bench_slab_loop(args)
        return bench_matrix(args, name)

    if args.workload == "all":
        os.makedirs(args.out_dir, exist_ok=True)
        headline = None
        for name in [n for n in synth.CONFIGS if n != HEADLINE] + ["cfg4_layer", "slab_loop", HEADLINE]:
            print(f"bench.py: {name}", file=sys.stderr, flush=True)
            out = run(name)
            with open(os.path.join(args.out_dir, f"bench_{name}.json"), "w") as fh:
                fh.write(json.dumps(out) + "\n")
            headline = out
        print(json.dumps(headline), flush=True)
    else:
        print(json.dumps(run(args.workload)), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
