#!/usr/bin/env python3
"""Throughput of the SOAR NVFP4 hot path on one MI355X.

A "step" is one pass of the whole path (absmax -> Eq. 1-2 statistics -> Eq. 5
global scale -> Eq. 6 block scales -> Eq. 8 search -> pack) over every tensor of
the workload, enqueued through the C-ABI batch entry point with the weights
already resident in HBM.  Default workload: the 36-layer 8B-class decoder
(252 bf16 tensors, 6.95e9 weights, search radius 4).

Prints ONE JSON line: metric, value (GB/s of bf16 input), ms_per_step, the roofline of the dominant
kernel, the per-kernel times and the oracle timed on the host cores.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
BYTES_3PASS = 6.5625           # per bf16 weight: three reads + codes + scales
BYTES_SEARCH = 2.5625          # search kernel alone: one read + codes + scales
BYTES_STATS = 2.0
BYTES_ABSMAX = 2.0
# HBM bytes per weight that a kernel really moves, and vector instructions it really executes, come from
# rocprofv3 counter runs (FETCH_SIZE / WRITE_SIZE scaled by a plain copy of known size; SQ_INSTS_VALU): the
# figures live in profiles/pmc_table.json, one entry per (algorithm, workload, dtype, kernel), beside the
# summaries they were taken from.  No entry, no figure: the JSON line then carries null and says why.
PMC_TABLE = os.path.join(ROOT, "profiles", "pmc_table.json")


def pmc_entry(algorithm, workload, dtype, kernel, layers=0, search="auto"):
    """-> (entry or None, reason)"""
    if layers:
        return None, "measured on the whole workload only, not on a --layers subset"
    try:
        with open(PMC_TABLE) as f:
            table = json.load(f)
    except (OSError, ValueError) as e:
        return None, f"{os.path.relpath(PMC_TABLE, ROOT)} not readable ({e.__class__.__name__})"
    for e in table.get("entries", []):
        if (e["algorithm"], e["workload"], e["dtype"], e["kernel"], e.get("search", "auto")) == \
                (algorithm, f"config{workload}", dtype, kernel, search):
            return e, e.get("source", "")
    return None, f"no counter run recorded for ({algorithm}, config{workload}, {dtype}, {kernel}, search {search})"


def traffic_per_launch(algorithm, workload, dtype, kernel, weights_per_launch, layers=0):
    e, why = pmc_entry(algorithm, workload, dtype, kernel, layers)
    if e is None or "read_B_per_weight" not in e:
        return None, why
    return (e["read_B_per_weight"] + e["written_B_per_weight"]) * weights_per_launch, why


# Iterated path (--algorithm paper): arithmetic-bound.  Per block, factor beta and iteration the
# method needs 16 products w*r, 16 roundings onto E2M1, 16 decoded values and, per stored-scale
# candidate, 16 residuals (one fused op each) and 16 fused square-accumulates.
VALU_PEAK_TFLOPS = 157.3       # MI355X FP32 vector, published (packed FP32)
VALU_LANE_OPS_PEAK = 256 * 4 * 16 * 2.4e9   # one non-packed 32-bit op per lane: CUs x SIMDs x lanes/clk x clock


def iter_flops_per_block_beta(ncand, nelem=16):
    """floating-point operations the method's definition asks for per block and factor: nelem products w*r, and per
    stored-scale candidate nelem fused residuals and nelem fused square-accumulates (2 operations each).  The
    roundings onto E2M1 and the decoded values are conversions, not floating-point operations, and are not counted."""
    return nelem + ncand * (nelem * 2 + nelem * 2)


def iter_lane_ops_per_block_beta(ncand, nelem=16):
    """the plain loop as vector instructions per lane: nelem multiplications, nelem/2 two-element conversions each way,
    2 nelem fused operations per candidate (a model: used where no counter run has measured the executed count)"""
    return nelem + nelem // 2 + nelem // 2 + ncand * 2 * nelem


def alu_roofline(kernel, algorithm, workload, dtype, search, layers, steps_blocks_factors, ncand, t_kernel, nelem=16):
    """Roofline of an arithmetic-bound kernel: executed vector instructions per lane against the rate at which the
    part issues them unpacked (256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz: one 32-bit operation per lane and cycle; the
    published 157.3 TFLOP/s is this rate x 2 for fused multiply-add x 2 for packed FP32, which this build does not
    emit).  The executed count per (block, factor) comes from a SQ_INSTS_VALU counter run (profiles/pmc_table.json);
    without one the plain loop's instruction count stands in and the line says so.  The method-definition
    floating-point rate is reported beside it."""
    e, why = pmc_entry(algorithm, workload, dtype, kernel, layers, search)
    if e is not None and "valu_lane_insts_per_block_factor" in e:
        per_step, source = e["valu_lane_insts_per_block_factor"], why
    else:
        per_step, source = iter_lane_ops_per_block_beta(ncand, nelem), "modelled (plain loop): " + why
    lane_ops = steps_blocks_factors * per_step
    flops = steps_blocks_factors * iter_flops_per_block_beta(ncand, nelem)
    return {"kernel": kernel, "bound": "alu", "achieved": lane_ops / t_kernel / 1e12, "peak": VALU_LANE_OPS_PEAK / 1e12,
            "unit": "T lane-op/s", "frac": lane_ops / t_kernel / VALU_LANE_OPS_PEAK, "traffic": None,
            "executed_lane_insts_per_block_factor": per_step, "executed_count_source": source,
            "method_flops_per_block_factor": iter_flops_per_block_beta(ncand, nelem),
            "method_tflops": flops / t_kernel / 1e12,
            "method_tflops_frac_of_packed_fma_peak": flops / t_kernel / 1e12 / VALU_PEAK_TFLOPS,
            "block_factor_steps_per_step": steps_blocks_factors}


def iterated_params(B, args, streams):
    stop = 0.0 if args.no_early_stop else args.early_stop_rel
    if args.algorithm == "paper":
        p = B.soar_paper_params(iters=args.iters or None, early_stop_rel=stop, tiles_per_wg=args.tpw, streams=streams)
    else:
        method = B.SOAR_METHOD_CJSO_ONLY if args.algorithm == "cjso-only" else B.SOAR_METHOD_DSS_ONLY
        p = B.soar_arm_params(method, iters=args.iters or 15, early_stop_rel=stop, tiles_per_wg=args.tpw, streams=streams)
    p.search_mode = B.SOAR_SEARCH_AUTO if args.search == "auto" else B.SOAR_SEARCH_FULL
    return p


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", type=int, default=4, choices=[1, 2, 3, 4, 5])
    ap.add_argument("--layers", type=int, default=0, help="workloads 4/5: first N layers only (0 = all)")
    ap.add_argument("--search", choices=["auto", "full"], default="auto")
    ap.add_argument("--tpw", type=int, default=0, help="force tiles per workgroup (0 = library default)")
    ap.add_argument("--tpw-absmax", type=int, default=0, help="single-step / rtn: force the maximum pass alone (0 = as --tpw)")
    ap.add_argument("--tpw-search", type=int, default=0, help="single-step / rtn: force the search pass alone (0 = as --tpw)")
    ap.add_argument("--streams", type=int, default=0, help="0 = library default, 1 = caller's stream only")
    ap.add_argument("--one-launch", choices=["auto", "never"], default="auto",
                    help="single tensors: let the library take its one-launch kernels (default) or hold it to three passes")
    ap.add_argument("--algorithm", choices=["single-step", "paper", "cjso-only", "dss-only", "rtn", "rtn-amax", "mxfp4", "mxfp4-dss",
                                               "dequantize", "recon-error", "copy-calibration"],
                    default="single-step",
                    help="single-step: Algorithm 1 with T = 1, beta = {1} (the headline path); "
                         "paper: T = 15, 101 beta factors, bracket candidates, early stop 1e-3; "
                         "cjso-only / dss-only: the arms of the paper's component study (T = 15, early stop); "
                         "rtn: plain NVFP4 (two passes); "
                         "rtn-amax: plain NVFP4 with each tensor's maximum supplied (one pass); "
                         "mxfp4 / mxfp4-dss: MXFP4 conversion, plain or with the decoupled scale search; "
                         "dequantize / recon-error: Eq. 3 / Eq. 4 on the stored form of every tensor (one call per tensor); "
                         "copy-calibration: no quantization at all -- a plain 1 GiB device copy, five times, whose known "
                         "traffic scales the FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run")
    ap.add_argument("--iters", type=int, default=0, help="--algorithm paper: override T")
    ap.add_argument("--no-early-stop", action="store_true", help="--algorithm paper: run all T iterations")
    ap.add_argument("--early-stop-rel", type=float, default=1e-3,
                    help="iterated algorithms: stop after an iteration that gains less than this fraction (Appendix B.3: 1e-3)")
    ap.add_argument("--dtype", choices=["bf16", "fp32"], default="bf16",
                    help="element type of the weights (NVFP4 algorithms only; every byte figure scales with it)")
    ap.add_argument("--graph", action="store_true",
                    help="capture one step into a HIP graph (caller's stream only) and time its replays")
    ap.add_argument("--reps", type=int, default=7,
                    help="after the timed region: this many separately timed steps, reported as median and min (0 = none)")
    ap.add_argument("--cold", action="store_true",
                    help="with --reps: write a 1 GiB scratch buffer before every repetition (caches hold none of the input)")
    ap.add_argument("--per-tensor", action="store_true",
                    help="--algorithm dequantize / recon-error: one call per tensor instead of the batch entry point")
    ap.add_argument("--search-stats", action="store_true",
                    help="single-step: after the timed region, one more pass with the library's diagnostic counters on: how "
                         "often the certified Eq. 8 search handed a block over to the exhaustive loop")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-widened", action="store_true",
                    help="default run only: leave out the short timed runs of the other entry points (widened_paths)")
    ap.add_argument("--no-kernel-timing", action="store_true")
    return ap.parse_args()


def run(args):
    """one benchmark as the flags say -> the dict of its JSON line"""
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no sharding, no collectives); "
              f"--gpus {args.gpus} is not supported", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2605_12245_amd import binding as B
    from paper_2605_12245_amd import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(2)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    B.lib()

    if args.algorithm == "copy-calibration":
        return copy_calibration(torch, dev)

    if args.algorithm in ("mxfp4", "mxfp4-dss"):
        if args.dtype != "bf16":
            print("bench.py: --dtype fp32 is wired for the NVFP4 algorithms only", file=sys.stderr)
            sys.exit(2)
        return bench_mxfp4(args, torch, B, synth, dev)

    if args.algorithm in ("dequantize", "recon-error"):
        return bench_stored_form(args, torch, B, synth, dev)

    specs = synth.workload_specs(args.workload)
    per_layer = {4: 7, 5: 3}.get(args.workload, 1)
    if args.layers and args.workload in (4, 5):
        specs = specs[: args.layers * per_layer]
    K = specs[0].dss_radius
    mode = B.SOAR_SEARCH_AUTO if args.search == "auto" else B.SOAR_SEARCH_FULL

    # ---- resident inputs and outputs
    t0 = time.time()
    weights, outs = [], []
    for s in specs:
        w = synth.make_weight(s, dev, torch.float32 if args.dtype == "fp32" else torch.bfloat16)
        weights.append(w)
        outs.append(B.Quantized(torch.empty((s.rows, s.cols // 2), dtype=torch.uint8, device=dev),
                                torch.empty((s.rows, s.cols // 16), dtype=torch.uint8, device=dev),
                                torch.empty(1, dtype=torch.float32, device=dev),
                                torch.empty(1, dtype=torch.float64, device=dev),
                                torch.empty(1, dtype=torch.int32, device=dev)))
    torch.cuda.synchronize()
    gen_s = time.time() - t0
    E = sum(s.numel for s in specs)
    es = 4.0 if args.dtype == "fp32" else 2.0                       # bytes per weight read
    BYTES_ABSMAX = BYTES_STATS = es
    BYTES_SEARCH = es + 0.5625
    BYTES_3PASS = 3.0 * es + 0.5625
    paper = args.algorithm in ("paper", "cjso-only", "dss-only")      # the iterated path
    rtn_amax = args.algorithm in ("rtn", "rtn-amax")                  # plain NVFP4
    one_launch = B.SOAR_RESIDENT_AUTO if args.one_launch == "auto" else B.SOAR_RESIDENT_NEVER
    amax_in = [None] * len(specs)
    if rtn_amax:
        if args.algorithm == "rtn-amax":
            # the supplied maxima: measured here, outside the timed region, as a calibration pass would
            amax_in = [w.abs().max().float().reshape(1) for w in weights]
        params = B.soar_default_params(B.SOAR_METHOD_RTN, 0, mode, args.tpw, args.streams)
        params.resident = one_launch
        params.tiles_per_wg_absmax, params.tiles_per_wg_search = args.tpw_absmax, args.tpw_search
    elif paper:
        params = iterated_params(B, args, args.streams)
        for o in outs:
            o.iters_run = torch.zeros(1, dtype=torch.int32, device=dev)
            o.sse_trace = torch.full((params.iters + 1,), float("nan"), dtype=torch.float64, device=dev)
    else:
        params = B.soar_default_params(B.SOAR_METHOD_SOAR, K, mode, args.tpw, args.streams)
        params.resident = one_launch
        params.tiles_per_wg_absmax, params.tiles_per_wg_search = args.tpw_absmax, args.tpw_search
    descs = [B.make_desc(w, o, a) for w, o, a in zip(weights, outs, amax_in)]
    ws = B.new_batch_workspace(descs, params, dev)

    def enqueue():
        B.quantize_batch(descs, params, ws)

    step = enqueue
    if args.graph:
        params.streams = 1                      # one stream: every launch of the step lands in the capture
        enqueue()
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            enqueue()
        step = graph.replay

    # ---- timed region
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    t_wall0 = time.perf_counter()
    e0.record()
    for _ in range(args.steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t_wall0) * 1e3
    ms_per_step = e0.elapsed_time(e1) / args.steps
    gbs_in = es * E / (ms_per_step * 1e-3) / 1e9

    per_tensor_sse = [float(o.sse.item()) for o in outs]
    sse_soar = sum(per_tensor_sse)
    statuses = [int(o.status.item()) for o in outs]

    # ---- separately timed repetitions (small workloads: median / min, warm or cold)
    reps = None
    if args.reps > 0:
        scratch = torch.empty(1 << 28, dtype=torch.float32, device=dev) if args.cold else None
        times = []
        for _ in range(args.reps):
            if scratch is not None:
                scratch.fill_(1.0)
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            step()
            b.record()
            torch.cuda.synchronize()
            times.append(a.elapsed_time(b))
        times.sort()
        med = times[len(times) // 2]
        reps = {"n": args.reps, "cold": bool(args.cold), "median_ms": med, "min_ms": times[0],
                "median_GBps_in": es * E / (med * 1e-3) / 1e9,
                "median_hbm_frac": (BYTES_SEARCH if args.algorithm == "rtn-amax" else
                                    2.0 * es + 0.5625 if args.algorithm == "rtn" else BYTES_3PASS) * E / (med * 1e-3) / 1e9 / HBM_PEAK_GBS
                if not paper else None}

    # ---- per-kernel durations: HIP events around every launch, on the stream it is
    # launched on; same steps again, on one stream so that a kernel's duration is its own
    roofline = None
    kernels = {}
    iters_run = [int(o.iters_run.item()) for o in outs] if paper else None
    if paper and not args.no_kernel_timing:
        n_prof = min(args.steps, 2)
        p_one = iterated_params(B, args, 1)
        B.soar_kernel_timing_enable(True)
        for _ in range(n_prof):
            B.quantize_batch(descs, p_one, ws)
        torch.cuda.synchronize()
        names = {B.SOAR_KERNEL_INIT: "init", B.SOAR_KERNEL_ABSMAX: "absmax",
                 B.SOAR_KERNEL_ITER_INIT: "iter_init", B.SOAR_KERNEL_ITER: "iter"}
        for kid, nm in names.items():
            ms, n = B.soar_kernel_timing_read(kid)
            kernels[nm] = {"launches": n, "total_ms": ms, "avg_us": (ms / n * 1e3) if n else None,
                           "ms_per_step": ms / n_prof}
        B.soar_kernel_timing_enable(False)
        ncand = 2 if params.dd_mode == B.SOAR_DD_BRACKET else 2 * params.dss_radius + 1
        block_iters = sum(it * (s.numel // 16) for it, s in zip(iters_run, specs))       # per step
        t_iter = kernels["iter"]["ms_per_step"] * 1e-3
        if args.algorithm == "cjso-only":
            # no search: an iteration reads the weights and the carried ratio and writes ratio, codes and scale
            per_w = 2.0 + 0.25 + 0.25 + 0.5625
            gbs = block_iters * 16 * per_w / t_iter / 1e9
            roofline = {"kernel": "k_cjso", "bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                        "frac": gbs / HBM_PEAK_GBS, "traffic": None, "algorithmic_bytes_per_weight_and_iteration": per_w,
                        "block_iterations_per_step": block_iters,
                        "timed_loops_per_step": kernels["iter"]["launches"] / n_prof,
                        "note": "all iteration launches of a step together (launches of tensors that have stopped return "
                                "at once): one HIP-event bracket per launch group round its T launches, on the launch "
                                "stream, single-stream pass"}
            # the same kernel where every launch has work: three iterations, no early stop
            B.soar_kernel_timing_enable(True)          # drops the events of the pass above
            p_work = B.soar_arm_params(B.SOAR_METHOD_CJSO_ONLY, iters=3, early_stop_rel=0.0, tiles_per_wg=args.tpw, streams=1)
            for _ in range(n_prof):
                B.quantize_batch(descs, p_work, ws)
            torch.cuda.synchronize()
            ms_w, n_w = B.soar_kernel_timing_read(B.SOAR_KERNEL_ITER)
            B.soar_kernel_timing_enable(False)
            if ms_w > 0:
                gbs_w = 3 * n_prof * E * per_w / (ms_w * 1e-3) / 1e9
                roofline["working_launches"] = {
                    "achieved": gbs_w, "frac": gbs_w / HBM_PEAK_GBS, "iterations": 3, "early_stop": False,
                    "note": "same tensors, every launch with work (T = 3, no stop): the kernel's own rate; the figure above "
                            "also carries the launches that find their tensors stopped"}
        else:
            roofline = alu_roofline("k_iter", args.algorithm, args.workload, args.dtype, args.search, args.layers,
                                    block_iters * params.n_beta, ncand, t_iter)
            roofline["timed_loops_per_step"] = kernels["iter"]["launches"] / n_prof
            roofline["note"] = ("all k_iter launches of a step together (launches of tensors that have stopped return at "
                                "once): one HIP-event bracket per launch group round its T launches, on the launch "
                                "stream, single-stream pass")
    elif not args.no_kernel_timing:
        n_prof = min(args.steps, 5)
        p_one = B.soar_default_params(B.SOAR_METHOD_RTN if rtn_amax else B.SOAR_METHOD_SOAR, 0 if rtn_amax else K,
                                      mode, args.tpw, streams=1)
        p_one.resident = one_launch
        p_one.tiles_per_wg_absmax, p_one.tiles_per_wg_search = args.tpw_absmax, args.tpw_search
        B.soar_kernel_timing_enable(True)
        for _ in range(n_prof):
            B.quantize_batch(descs, p_one, ws)
        torch.cuda.synchronize()
        names = {B.SOAR_KERNEL_INIT: "init", B.SOAR_KERNEL_ABSMAX: "absmax",
                 B.SOAR_KERNEL_STATS: "stats", B.SOAR_KERNEL_SEARCH: "search", B.SOAR_KERNEL_RESIDENT: "resident"}
        # the one-launch kernel of a single tensor is the whole path and reads the weights once
        per_elem = {"absmax": BYTES_ABSMAX, "stats": BYTES_STATS, "search": BYTES_SEARCH, "init": 0.0,
                    "resident": BYTES_SEARCH}
        for kid, nm in names.items():
            ms, n = B.soar_kernel_timing_read(kid)
            kernels[nm] = {"launches": n, "total_ms": ms, "avg_us": (ms / n * 1e3) if n else None,
                           "ms_per_step": ms / n_prof,
                           "GBps": (per_elem[nm] * E * n_prof / (ms * 1e-3) / 1e9) if ms > 0 and per_elem[nm] else None}
        B.soar_kernel_timing_enable(False)
        dom = max(("absmax", "stats", "search", "resident"), key=lambda k: kernels[k]["total_ms"])
        kernels = {k: v for k, v in kernels.items() if v["launches"]}
        achieved = kernels[dom]["GBps"]
        traffic, traffic_source = traffic_per_launch(args.algorithm, args.workload, args.dtype, "k_" + dom,
                                                     E / (kernels[dom]["launches"] / n_prof), args.layers)
        roofline = {"kernel": "k_" + dom, "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": achieved / HBM_PEAK_GBS, "traffic": traffic, "traffic_source": traffic_source,
                    "algorithmic_bytes_per_weight": per_elem[dom],
                    "weights_per_launch": E / (kernels[dom]["launches"] / n_prof),
                    "avg_launch_us": kernels[dom]["avg_us"],
                    "note": "per-launch HIP-event durations on the launch stream, single-stream pass"
                            + ("; the one-launch kernel reads the weights once, so its algorithmic bytes are those of the "
                               "search pass alone; it is bound by its arithmetic and by two trips across the grid, "
                               "not by memory" if dom == "resident" else "")}

    # ---- diagnostics of the certified search (untimed pass, counters on)
    search_stats = None
    if args.search_stats and args.algorithm == "single-step":
        B.soar_search_stats_enable(True)
        B.quantize_batch(descs, params, ws)
        c = B.soar_search_stats_read()
        B.soar_search_stats_enable(False)
        search_stats = dict(c, block_fraction=c["blocks_handed_over"] / max(1, c["blocks"]),
                            wave_step_fraction=c["wave_steps_with_hand_over"] / max(1, c["wave_steps"]))

    # ---- "MSE vs RTN": the plain max-based NVFP4 of Sec. 3.1 on the same tensors
    if args.algorithm in ("rtn", "rtn-amax"):
        per_tensor_rtn = list(per_tensor_sse)      # the timed path is that conversion
    else:
        p_rtn = B.soar_default_params(B.SOAR_METHOD_RTN, 0)
        for o in outs:
            o.iters_run = o.sse_trace = None       # plain descriptors: the single-step entry
        B.quantize_batch([B.make_desc(w, o) for w, o in zip(weights, outs)], p_rtn, ws)
        torch.cuda.synchronize()
        per_tensor_rtn = [float(o.sse.item()) for o in outs]
    sse_rtn = sum(per_tensor_rtn)
    ratios = sorted(a / b for a, b in zip(per_tensor_sse, per_tensor_rtn) if b > 0)

    # ---- oracle on the host cores, bounded sample of the same workload
    cpu = None
    if not args.no_cpu_baseline:
        import numpy as np
        import oracle
        # about ten seconds of oracle time on the machine's host cores
        sample = specs[: 16 * per_layer] if args.workload == 4 else specs[: 2 * per_layer] if args.workload == 5 else specs[:1]
        if paper:
            sample = sample[:1]
        host = [w.cpu().contiguous().numpy() if args.dtype == "fp32" else
                w.cpu().contiguous().view(torch.int16).numpy().view(np.uint16) for w in weights[: len(sample)]]
        n_el = sum(s.numel for s in sample)
        t1 = time.perf_counter()
        if paper:
            sample, host = sample[:1], host[:1]
            n_el = sample[0].numel
            t1 = time.perf_counter()
            oracle.quantize_iter(host[0], iters=params.iters, n_beta=params.n_beta, beta_lo=params.beta_lo,
                                 beta_hi=params.beta_hi, dd_mode=params.dd_mode, dss_radius=params.dss_radius,
                                 early_stop_rel=params.early_stop_rel,
                                 arm={B.SOAR_METHOD_SOAR: oracle.ARM_SOAR, B.SOAR_METHOD_CJSO_ONLY: oracle.ARM_CJSO_ONLY,
                                      B.SOAR_METHOD_DSS_ONLY: oracle.ARM_DSS_ONLY}[params.method])
        for s, h in zip(sample, host):
            if paper:
                break
            if args.algorithm == "rtn-amax":
                oracle.quantize_rtn_amax(h, float(amax_in[0].item()))
                continue
            if args.algorithm == "rtn":
                oracle.quantize(h, oracle.METHOD_RTN, 0)
                continue
            oracle.quantize(h, oracle.METHOD_SOAR, s.dss_radius)
        dt = time.perf_counter() - t1
        # one thread, a slice of the first tensor: nanoseconds per weight of the same function
        nthreads = oracle.threads()
        rows1 = max(1, min(host[0].shape[0], (1 << 20) // host[0].shape[1]))
        piece = np.ascontiguousarray(host[0][:rows1])
        oracle.set_threads(1)
        t2 = time.perf_counter()
        if paper:
            oracle.quantize_iter(piece, iters=1, n_beta=params.n_beta, beta_lo=params.beta_lo, beta_hi=params.beta_hi,
                                 dd_mode=params.dd_mode, dss_radius=params.dss_radius, early_stop_rel=0.0,
                                 arm={B.SOAR_METHOD_SOAR: oracle.ARM_SOAR, B.SOAR_METHOD_CJSO_ONLY: oracle.ARM_CJSO_ONLY,
                                      B.SOAR_METHOD_DSS_ONLY: oracle.ARM_DSS_ONLY}[params.method])
        elif rtn_amax:
            oracle.quantize(piece, oracle.METHOD_RTN, 0)
        else:
            oracle.quantize(piece, oracle.METHOD_SOAR, K)
        ns1 = (time.perf_counter() - t2) * 1e9 / piece.size
        oracle.set_threads(nthreads)
        cpu = {"value": es * n_el / dt / 1e9, "unit": f"GB/s {args.dtype} in", "cores": oracle.threads(),
               "single_thread_ns_per_weight": ns1,
               "single_thread_note": "one iteration" if paper else "whole path",
               "kind": "oracle", "seconds": dt, "weights_per_s": n_el / dt,
               "sample": f"first {len(sample)} tensor(s) of the workload ({n_el} weights), whole path"}

    out = {
        "metric": {"single-step": "nvfp4_soar_quantize_throughput", "paper": "nvfp4_soar_full_algorithm_throughput",
                   "cjso-only": "nvfp4_cjso_only_throughput", "dss-only": "nvfp4_dss_only_throughput",
                   "rtn": "nvfp4_rtn_throughput", "rtn-amax": "nvfp4_rtn_supplied_amax_throughput"}[args.algorithm],
        "value": gbs_in,
        "unit": f"GB/s {args.dtype} in",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": f"config{args.workload}", "tensors": len(specs), "weights": E,
                   "dss_radius": K, "search": args.search, "entry_point": "soar_quantize_batch",
                   "input": f"{args.dtype}, resident in HBM", "algorithm": args.algorithm, "hip_graph": bool(args.graph),
                   **({"iters": params.iters, "n_beta": params.n_beta, "beta": [params.beta_lo, params.beta_hi],
                       "dd_mode": "bracket" if params.dd_mode == B.SOAR_DD_BRACKET else "window",
                       "early_stop_rel": params.early_stop_rel,
                       "iterations_run_min_mean_max": [min(iters_run), sum(iters_run) / len(iters_run), max(iters_run)]}
                      if paper else {})},
        "weights_per_s": E / (ms_per_step * 1e-3),
        "hbm_frac_3pass": (BYTES_3PASS * E / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS) if not rtn_amax else None,
        "hbm_frac_3pass_note": "algorithmic bytes per weight (three reads of the weights, codes and scales written once) / "
                               "time / 8 TB/s: a rate of bytes the method has to touch.  Launch groups of at most 256 MiB "
                               "are found in the last-level cache by the second and third pass, so this is not a DRAM "
                               "rate for workloads 1-4; workload 5 (470 MB tensors: nothing stays cached) is",
        "hbm_frac_single_touch": BYTES_SEARCH * E / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "mse_vs_rtn": sse_soar / sse_rtn if sse_rtn > 0 else None,
        "mse_vs_rtn_per_tensor_min_median_max": [ratios[0], ratios[len(ratios) // 2], ratios[-1]] if ratios else None,
        "sse_soar": sse_soar, "sse_rtn": sse_rtn,
        "repetitions": reps,
        "status_bits_or": int(np_or(statuses)),
        "wall_ms_per_step": wall_ms / args.steps,
        "gen_seconds": gen_s,
        "kernels": kernels,
        "roofline": roofline,
        "search_hand_over": search_stats,
        "cpu_baseline": cpu,
    }
    return out


def copy_calibration(torch, dev, gib=1.0, reps=5):
    """A dtype-preserving element-wise copy (torch's vectorized kernel): 1 GiB read and 1 GiB written per
    dispatch.  Under `rocprofv3 --pmc FETCH_SIZE` (then WRITE_SIZE) its counter values per dispatch, against
    the 1 048 576 KiB really moved, give the scale factors of those counters."""
    n = int(gib * (1 << 30)) // 4
    src = torch.arange(n, dtype=torch.int32, device=dev)
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        torch.add(src, 0, out=dst)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / reps
    return ({"metric": "copy_calibration", "bytes_read_per_dispatch": n * 4, "bytes_written_per_dispatch": n * 4,
                      "dispatches": reps, "ms_per_dispatch": ms, "GBps_read_plus_written": 2 * n * 4 / (ms * 1e-3) / 1e9,
                      "kernel": "torch vectorized_elementwise_kernel"})


def bench_stored_form(args, torch, B, synth, dev):
    """Eq. 3 (soar_dequantize_batch) or Eq. 4 (soar_recon_error_batch) over every tensor of the workload, on
    the stored form the single-step path produced; --per-tensor: one soar_dequantize / soar_recon_error call
    per tensor instead."""
    import numpy as np
    specs = synth.workload_specs(args.workload)
    per_layer = {4: 7, 5: 3}.get(args.workload, 1)
    if args.layers and args.workload in (4, 5):
        specs = specs[: args.layers * per_layer]
    deq = args.algorithm == "dequantize"
    tdt = torch.float32 if args.dtype == "fp32" else torch.bfloat16
    es = 4.0 if args.dtype == "fp32" else 2.0
    code = B.SOAR_FP32 if args.dtype == "fp32" else B.SOAR_BF16
    weights = [synth.make_weight(s, dev, tdt) for s in specs]
    qs = B.quantize_tensors(weights, B.soar_default_params(B.SOAR_METHOD_SOAR, specs[0].dss_radius))
    torch.cuda.synchronize()
    E = sum(s.numel for s in specs)
    st = torch.cuda.current_stream().cuda_stream
    one_by_one = args.per_tensor
    if deq:
        backs = [torch.empty((s.rows, s.cols), dtype=tdt, device=dev) for s in specs]
        descs = [B.stored_desc(q, out=o) for q, o in zip(qs, backs)]

        def step():
            if not one_by_one:
                rc = B.soar_dequantize_batch(descs, st)
                assert rc == B.SOAR_OK, rc
                return
            for s, q, o in zip(specs, qs, backs):
                rc = B.soar_dequantize(q.codes.data_ptr(), q.scales.data_ptr(), q.global_scale.data_ptr(), s.rows, s.cols,
                                       code, o.data_ptr(), s.cols, st)
                assert rc == B.SOAR_OK, rc
    else:
        sses = torch.zeros(len(specs), dtype=torch.float64, device=dev)
        descs = [B.stored_desc(q, w=w, sse=sses[k:k + 1]) for k, (q, w) in enumerate(zip(qs, weights))]

        def step():
            if not one_by_one:
                rc = B.soar_recon_error_batch(descs, st)
                assert rc == B.SOAR_OK, rc
                return
            for k, (s, q, w) in enumerate(zip(specs, qs, weights)):
                rc = B.soar_recon_error(w.data_ptr(), code, s.rows, s.cols, s.cols, q.codes.data_ptr(), q.scales.data_ptr(),
                                        q.global_scale.data_ptr(), sses.data_ptr() + 8 * k, st)
                assert rc == B.SOAR_OK, rc

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(args.steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    ms_per_step = e0.elapsed_time(e1) / args.steps
    per_w = (0.5625 + es) if deq else (es + 0.5625)       # codes + scale bytes, and the weights written or read
    kid, kname = (B.SOAR_KERNEL_DEQUANT, "k_dequant") if deq else (B.SOAR_KERNEL_RECON, "k_recon")
    kernels, roofline = {}, None
    if not args.no_kernel_timing:
        n_prof = min(args.steps, 5)
        B.soar_kernel_timing_enable(True)
        for _ in range(n_prof):
            step()
        torch.cuda.synchronize()
        ms, n = B.soar_kernel_timing_read(kid)
        B.soar_kernel_timing_enable(False)
        kernels[kname[2:]] = {"launches": n, "total_ms": ms, "avg_us": ms / n * 1e3, "ms_per_step": ms / n_prof}
        gbs = per_w * E * n_prof / (ms * 1e-3) / 1e9
        traffic, traffic_source = traffic_per_launch(args.algorithm, args.workload, args.dtype, kname, E / (n / n_prof), args.layers)
        roofline = {"kernel": kname, "bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": gbs / HBM_PEAK_GBS, "traffic": traffic, "traffic_source": traffic_source,
                    "algorithmic_bytes_per_weight": per_w,
                    "weights_per_launch": E / (n / n_prof), "avg_launch_us": ms / n * 1e3,
                    "note": "per-launch HIP-event durations on the launch stream, "
                            + ("one launch per tensor" if one_by_one else "up to 8 tensors per launch")
                            + ("" if deq else " (with the small launch that clears the sums)")}
    extra = {}
    if not deq:
        got = float(sses.sum().item())
        want = sum(float(q.sse.item()) for q in qs)
        extra["sse_recon"] = got
        extra["sse_from_quantize"] = want
        extra["sse_rel_diff"] = abs(got - want) / want if want > 0 else 0.0
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        k = 4 if len(specs) > 4 else 0
        q = qs[k]
        c, sc, a = q.codes.cpu().numpy(), q.scales.cpu().numpy(), float(q.global_scale.item())
        h = weights[k].cpu().contiguous()
        h = h.numpy() if args.dtype == "fp32" else h.view(torch.int16).numpy().view(np.uint16)
        reps = 0
        t1 = time.perf_counter()
        while time.perf_counter() - t1 < 10.0:
            if deq:
                oracle.dequantize(c, sc, a, oracle.FP32 if args.dtype == "fp32" else oracle.BF16)
            else:
                oracle.recon_error(h, c, sc, a)
            reps += 1
        dt = (time.perf_counter() - t1) / reps
        cpu = {"value": es * h.size / dt / 1e9, "unit": f"GB/s {args.dtype} " + ("out" if deq else "in"), "cores": oracle.threads(),
               "kind": "oracle", "seconds": dt, "weights_per_s": h.size / dt,
               "sample": f"tensor {k} ({specs[k].name}, {h.size} weights), {reps} repetitions"}
    return ({
        "metric": "nvfp4_dequantize_throughput" if deq else "nvfp4_recon_error_throughput",
        "value": es * E / (ms_per_step * 1e-3) / 1e9, "unit": f"GB/s {args.dtype} " + ("out" if deq else "in"), "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"config{args.workload}", "tensors": len(specs), "weights": E,
                   "entry_point": ("soar_dequantize" if deq else "soar_recon_error") + ("" if one_by_one else "_batch"),
                   "algorithm": args.algorithm,
                   "stored_form": "single-step SOAR output, resident in HBM"},
        "weights_per_s": E / (ms_per_step * 1e-3), "hbm_frac_of_step": per_w * E / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
        **extra, "kernels": kernels, "roofline": roofline, "cpu_baseline": cpu})


def bench_mxfp4(args, torch, B, synth, dev):
    """MXFP4 conversion of every tensor of the workload through soar_mxfp4_quantize_batch."""
    specs = synth.workload_specs(args.workload)
    per_layer = {4: 7, 5: 3}.get(args.workload, 1)
    if args.layers and args.workload in (4, 5):
        specs = specs[: args.layers * per_layer]
    dss = args.algorithm == "mxfp4-dss"
    p = B.soar_mx_default_params(dss=dss, tiles_per_wg=args.tpw, streams=args.streams)
    weights = [synth.make_weight(s, dev) for s in specs]
    outs = [B.mx_new_outputs(s.rows, s.cols, dev) for s in specs]
    descs = [B.mx_make_desc(w, o) for w, o in zip(weights, outs)]
    ws = torch.empty(B.soar_mxfp4_batch_workspace_bytes(descs, p), dtype=torch.uint8, device=dev)
    E = sum(s.numel for s in specs)
    torch.cuda.synchronize()

    def step(params=p):
        B.mx_quantize_batch(descs, params, ws)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(args.steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    ms_per_step = e0.elapsed_time(e1) / args.steps
    sse = sum(float(o.sse.item()) for o in outs)
    status = np_or(int(o.status.item()) for o in outs)

    kernels, roofline = {}, None
    if not args.no_kernel_timing:
        n_prof = min(args.steps, 2 if dss else 5)
        p_one = B.soar_mx_default_params(dss=dss, tiles_per_wg=args.tpw, streams=1)     # launches must not overlap
        B.soar_kernel_timing_enable(True)
        for _ in range(n_prof):
            step(p_one)
        torch.cuda.synchronize()
        for kid, nm in ((B.SOAR_KERNEL_INIT, "init"), (B.SOAR_KERNEL_MX, "mx")):
            ms, n = B.soar_kernel_timing_read(kid)
            kernels[nm] = {"launches": n, "total_ms": ms, "avg_us": (ms / n * 1e3) if n else None, "ms_per_step": ms / n_prof}
        B.soar_kernel_timing_enable(False)
        t_mx = kernels["mx"]["ms_per_step"] * 1e-3
        if dss:
            ncand = 2 * p.radius + 1
            roofline = alu_roofline("k_mx", args.algorithm, args.workload, "bf16", "auto", args.layers,
                                    (E // 32) * p.n_beta, ncand, t_mx, nelem=32)
            roofline["note"] = "all k_mx launches of a step together; HIP-event durations on the launch stream, single-stream pass"
        else:
            per_w = 2.0 + 0.5 + 1.0 / 32.0
            gbs = per_w * E / t_mx / 1e9
            traffic, traffic_source = traffic_per_launch(args.algorithm, args.workload, "bf16", "k_mx",
                                                         E / (kernels["mx"]["launches"] / n_prof), args.layers)
            roofline = {"kernel": "k_mx", "bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                        "frac": gbs / HBM_PEAK_GBS, "traffic": traffic, "traffic_source": traffic_source,
                        "algorithmic_bytes_per_weight": per_w,
                        "weights_per_launch": E / (kernels["mx"]["launches"] / n_prof),
                        "avg_launch_us": kernels["mx"]["avg_us"],
                        "note": "per-launch HIP-event durations on the launch stream, single-stream pass, up to 8 tensors per launch"}

    # the way back: soar_mxfp4_dequantize_batch, bf16 out (2 + 1/2 + 1/32 bytes per weight)
    backs = [torch.empty((s.rows, s.cols), dtype=torch.bfloat16, device=dev) for s in specs]
    st = torch.cuda.current_stream().cuda_stream

    back_descs = [B.mx_stored_desc(o, b) for o, b in zip(outs, backs)]

    def back():
        rc = B.soar_mxfp4_dequantize_batch(back_descs, st)
        assert rc == B.SOAR_OK, rc
    back()
    torch.cuda.synchronize()
    d0, d1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    d0.record()
    for _ in range(3):
        back()
    d1.record()
    torch.cuda.synchronize()
    deq_ms = d0.elapsed_time(d1) / 3
    del backs

    # error of the plain conversion, for the ratio the paper's table is about
    p_plain = B.soar_mx_default_params(dss=False)
    step(p_plain)
    torch.cuda.synchronize()
    sse_plain = sum(float(o.sse.item()) for o in outs)

    cpu = None
    if not args.no_cpu_baseline:
        import numpy as np
        import oracle
        h = weights[0].cpu().contiguous().view(torch.int16).numpy().view(np.uint16)
        if dss:
            h = np.ascontiguousarray(h[: max(1, h.shape[0] // 4)])
        t1 = time.perf_counter()
        oracle.mxfp4_quantize(h, dss, p.n_beta, p.beta_lo, p.beta_hi, p.radius)
        dt = time.perf_counter() - t1
        cpu = {"value": 2.0 * h.size / dt / 1e9, "unit": "GB/s bf16 in", "cores": oracle.threads(), "kind": "oracle",
               "seconds": dt, "weights_per_s": h.size / dt,
               "sample": f"first {h.shape[0]} rows of the first tensor ({h.size} weights), whole path"}
    return ({
        "metric": "mxfp4_dss_quantize_throughput" if dss else "mxfp4_quantize_throughput",
        "value": 2.0 * E / (ms_per_step * 1e-3) / 1e9, "unit": "GB/s bf16 in", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"config{args.workload}", "tensors": len(specs), "weights": E,
                   "entry_point": "soar_mxfp4_quantize_batch", "input": "bf16, resident in HBM", "algorithm": args.algorithm,
                   "n_beta": p.n_beta if dss else None, "beta": [p.beta_lo, p.beta_hi] if dss else None,
                   "radius": p.radius if dss else None},
        "weights_per_s": E / (ms_per_step * 1e-3), "mse_vs_plain_mxfp4": sse / sse_plain if sse_plain > 0 else None,
        "sse": sse, "sse_plain": sse_plain, "status_bits_or": status,
        "dequantize": {"entry_point": "soar_mxfp4_dequantize_batch (bf16 out)", "ms_per_step": deq_ms,
                       "hbm_frac": 2.53125 * E / (deq_ms * 1e-3) / 1e9 / HBM_PEAK_GBS},
        "kernels": kernels, "roofline": roofline,
        "cpu_baseline": cpu})


def np_or(xs):
    r = 0
    for x in xs:
        r |= x
    return r


# The other entry points on the same workload, a few steps each, so that one default run times every path this
# build has (whole-job figures, weights resident in HBM; no per-kernel events, no host baseline: the run of
# each --algorithm by itself reports those).
WIDENED = (("paper", 2, 1), ("cjso-only", 3, 1), ("dss-only", 2, 1), ("rtn-amax", 10, 2), ("mxfp4-dss", 2, 1),
           ("dequantize", 10, 2), ("recon-error", 10, 2))


def widened_paths(args):
    import torch
    rows = {}
    for alg, steps, warmup in WIDENED:
        a = argparse.Namespace(**vars(args))
        a.algorithm, a.steps, a.warmup = alg, steps, warmup
        a.no_cpu_baseline = a.no_kernel_timing = True
        a.reps, a.search_stats, a.graph, a.cold = 0, False, False, False
        d = run(a)
        rows[alg] = {k: d.get(k) for k in ("metric", "value", "unit", "ms_per_step", "steps", "warmup", "weights_per_s")}
        for k in ("mse_vs_rtn", "mse_vs_plain_mxfp4"):
            if d.get(k) is not None:
                rows[alg][k] = d[k]
        if d.get("config", {}).get("iterations_run_min_mean_max"):
            rows[alg]["iterations_run_min_mean_max"] = d["config"]["iterations_run_min_mean_max"]
        torch.cuda.empty_cache()
    return rows


def main():
    args = parse_args()
    out = run(args)
    headline = (args.algorithm == "single-step" and args.workload == 4 and not args.layers and args.dtype == "bf16"
                and not args.graph)
    if headline and not args.no_widened:
        out["widened_paths"] = widened_paths(args)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
