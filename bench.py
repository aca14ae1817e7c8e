#!/usr/bin/env python3
"""Benchmark of the FFT convolution hot path on one MI355X.

One "step" is one pass of the whole hot path over one batch of synthetic input
already resident in HBM: the three forward transforms (x, w, dL/dy), the three
per-bin contractions and the three inverse transforms + crops, i.e. fprop, bprop
and accGrad of one layer with every spectrum computed once and reused.

Prints ONE JSON line on stdout.  `value` is direct-equivalent GFLOP/s of the
step: 3 * 2*S*f*f'*(n-k+1)^2*k^2 divided by the step time (the direct method's
operation count of the paper's Sec. 2.2 table, times two for multiply+add).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_FP32_MFMA_TFLOPS = 157.3
PEAK_HBM_GBS = 8000.0
EVENT_EVERY = 4   # steps between event-bracketed steps inside the timed region


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def cpu_baseline(layer, x, w, g, budget_s=18.0):
    """Time the fp64 direct-sum oracle on a bounded sample of the same layer."""
    from oracle import direct
    from paper_1312_5851_amd import workloads as wl
    S, f, fo, n, k = layer.S, layer.f, layer.fo, layer.n, layer.k
    totals = (S * fo, S * f, fo * f)
    # probe with a few units to size the sample to the budget (a third of it per pass)
    counts = []
    t_meas = []
    fns = (lambda u: direct.fprop(x, w, u), lambda u: direct.bprop(g, w, n, u), lambda u: direct.accgrad(g, x, k, u))
    xs = [a.astype(np.float64) for a in (x, w, g)]
    x, w, g = xs
    for p, (fn, total) in enumerate(zip(fns, totals)):
        probe = wl.sample_units(total, min(total, 16), layer.seed + 70 + p)
        t0 = time.perf_counter(); fn(probe); dt = max(time.perf_counter() - t0, 1e-4)
        cnt = int(max(16, min(total, (budget_s / 3.0) / (dt / len(probe)))))
        u = wl.sample_units(total, cnt, layer.seed + 80 + p)
        t0 = time.perf_counter(); fn(u); dt = time.perf_counter() - t0
        counts.append(len(u)); t_meas.append(dt)
    # every unit of a pass costs the same, so full-pass time = sample time * total / count
    full_s = sum(t * tot / c for t, tot, c in zip(t_meas, totals, counts))
    return {
        "value": 3 * layer.direct_flops / full_s / 1e9,
        "unit": "GFLOP/s (direct-equivalent)",
        "cores": direct.num_threads(),
        "kind": "oracle",
        "sample": (f"fp64 direct loops on {counts[0]}/{totals[0]} fprop maps, {counts[1]}/{totals[1]} bprop maps, "
                   f"{counts[2]}/{totals[2]} accGrad kernels of the same layer ({sum(t_meas):.1f} s), "
                   f"extrapolated per pass by units total / units run"),
        "extrapolated_step_s": full_s,
    }


def copy_bandwidth():
    """Read+write rate of a plain 1 GiB device copy (larger than the 256 MB memory-side cache):
    what a kernel that only moves data gets out of HBM on this machine, as context for the FFT stages."""
    import torch
    n = 256 * 1024 * 1024
    src = torch.empty(n, dtype=torch.float32, device="cuda").fill_(1.0)
    dst = torch.empty_like(src)
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    reps = 20
    for _ in range(5):
        dst.copy_(src)
    ev0.record()
    for _ in range(reps):
        dst.copy_(src)
    ev1.record(); ev1.synchronize()
    return reps * 2 * 4 * n / (ev0.elapsed_time(ev1) * 1e-3) / 1e9


def measure(layer, args, inputs=None):
    """Times args.steps steps of the whole hot path on one layer; returns the JSON record."""
    import torch
    from paper_1312_5851_amd import fftconv as fc
    from paper_1312_5851_amd import workloads as wl

    x, w, g = inputs if inputs is not None else wl.make_inputs(layer)
    xd, wd, gd = (torch.from_numpy(a).cuda() for a in (x, w, g))
    plan = fc.Plan(layer.S, layer.f, layer.fo, layer.n, layer.k)
    plan.alloc_workspace()
    y = torch.empty(layer.shapes()[2], dtype=torch.float32, device="cuda")
    dx = torch.empty_like(xd)
    dw = torch.empty_like(wd)

    def step():
        plan.invalidate()
        plan.fprop(xd, wd, y)
        plan.bprop(gd, wd, dx)
        plan.accgrad(gd, xd, dw)

    if args.calibration_copy:
        # a copy of known size in the same process: rocprofv3's FETCH_SIZE / WRITE_SIZE readings for
        # it give the factor that turns the counters into bytes
        src = torch.empty(64 * 1024 * 1024, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    step()   # first launches: code objects load, LDS limits are raised
    torch.cuda.synchronize()
    plan.profile_read()
    stage_ms = {name: [0.0, 0] for name in fc.STAGE_NAMES}
    gemm_names = ("cgemm_fprop", "cgemm_bprop", "cgemm_accgrad")

    def drain():
        for name, (ms, cnt) in plan.profile_read().items():
            stage_ms[name][0] += ms
            stage_ms[name][1] += cnt

    # Auxiliary measurements come first (per-pass times, memory-efficient mode, per-stage table), the
    # warm-up and timed steps of the headline figure last: a card coming out of idle runs the same
    # kernels up to 30 % slower during its first ~30 ms under load (per-dispatch durations of a
    # rocprofv3 kernel trace: the contraction of this layer falls from 120 to 90 us over 60 steps), and
    # the figure of interest is the sustained rate.
    # per-pass times, warm (operand spectra cached) and cold (pass includes its forward transforms)
    # bprop and accGrad are timed in alternation, the way a training step calls them: with all spectra cached the
    # first of the two also forms the other's result spectrum (one launch over the spectrum of dL/dy), so the
    # pair is the meaningful unit; "warm" = operand spectra cached, "cold" = the pass transforms its operands first.
    def time_passes(fns, slots, iters=20):
        evs = [torch.cuda.Event(enable_timing=True) for _ in range(len(fns) + 1)]
        out = []
        for cold in (False, True):
            ts = [[] for _ in fns]
            for _ in range(iters + 3):
                for i, fn in enumerate(fns):
                    if cold:
                        plan.invalidate(slots[i])
                    evs[i].record(); fn(); evs[i + 1].record(); evs[i + 1].synchronize()
                    ts[i].append(evs[i].elapsed_time(evs[i + 1]))
            out.append([float(np.median(t[3:])) for t in ts])
        return [{"warm_ms": w, "cold_ms": c} for w, c in zip(*out)]

    plan.fprop(xd, wd, y); plan.bprop(gd, wd, dx); plan.accgrad(gd, xd, dw)
    (p_f,) = time_passes([lambda: plan.fprop(xd, wd, y)], [fc.SPEC_X | fc.SPEC_W])
    p_b, p_a = time_passes([lambda: plan.bprop(gd, wd, dx), lambda: plan.accgrad(gd, xd, dw)],
                           [fc.SPEC_G | fc.SPEC_W, fc.SPEC_G | fc.SPEC_X])
    passes = {"fprop": p_f, "bprop": p_b, "accgrad": p_a}
    passes["bprop"]["note"] = passes["accgrad"]["note"] = "timed in alternation bprop, accGrad, bprop, ..."
    for v in passes.values():
        v["warm_direct_equiv_gflops"] = layer.direct_flops / (v["warm_ms"] * 1e-3) / 1e9
        v["cold_direct_equiv_gflops"] = layer.direct_flops / (v["cold_ms"] * 1e-3) / 1e9

    # The paper's memory-efficient mode (Sec. 2.3; all of its own timings assume it): no spectrum is
    # reused, so a step runs six forward transforms instead of three, in a three-slot workspace.
    lean = fc.Plan(layer.S, layer.f, layer.fo, layer.n, layer.k, flags=fc.RECOMPUTE)
    lean.alloc_workspace()

    def lean_step():
        lean.fprop(xd, wd, y)
        lean.bprop(gd, wd, dx)
        lean.accgrad(gd, xd, dw)

    for _ in range(3):
        lean_step()
    torch.cuda.synchronize()
    lean_steps = min(args.steps, 30)
    t0 = time.perf_counter()
    for _ in range(lean_steps):
        lean_step()
    torch.cuda.synchronize()
    lean_ms = (time.perf_counter() - t0) * 1e3 / lean_steps
    memory_efficient = {"ms_per_step": lean_ms, "steps": lean_steps,
                        "direct_equiv_gflops": 3 * layer.direct_flops / (lean_ms * 1e-3) / 1e9,
                        "workspace_bytes": lean.workspace_bytes, "cached_workspace_bytes": plan.workspace_bytes,
                        "paper_ram_bytes": fc.paper_ram_bytes(layer.S, layer.n, layer.f, layer.fo)}
    lean.ws = None
    lean.close()

    # A few steps with every stage bracketed, for the per-stage table.
    plan.profile_enable(not args.no_stage_events)
    for _ in range(min(args.steps, 20)):
        step()
    torch.cuda.synchronize()
    drain()
    plan.profile_enable(False)
    stages = {name: (ms / cnt if cnt else None) for name, (ms, cnt) in stage_ms.items()}

    # ---- the headline figure: W warm-up steps, then exactly K timed steps
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    plan.profile_read()
    stage_ms = {name: [0.0, 0] for name in fc.STAGE_NAMES}

    # Timed region.  The dominant kernel (the contraction, three launches per step) is bracketed
    # with HIP events on every EVENT_EVERY-th step; a bracket costs queue time (all nine stages on
    # every step add ~65 us to a 0.53 ms step), so the other steps run unbracketed.
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        if not args.no_stage_events:
            plan.profile_enable(gemm_names if i % EVENT_EVERY == 0 else False)
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    drain()
    ms_per_step = elapsed * 1e3 / args.steps
    # the same number of steps again with no event brackets at all, reported beside the timed region
    plan.profile_enable(False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_per_step_unbracketed = (time.perf_counter() - t0) * 1e3 / args.steps
    gemm_live = {n: (stage_ms[n][0] / stage_ms[n][1] if stage_ms[n][1] else None) for n in gemm_names}
    gemm_live_launches = sum(stage_ms[n][1] for n in gemm_names)

    # roofline of the dominant kernel: the per-bin contraction (three launches per step).
    # Algorithmic work of one launch: a complex multiply-add (8 real flops) per (s, i, j) triple
    # and per stored bin.  The kernel issues fewer matrix-core flops than that (three real
    # products per complex product instead of four), reported next to it as "issued".
    B = plan.num_bins
    algo_flops = plan.contraction_flops * 8.0 / 6.0   # = 8 S f f' B for a layer that is not tiled
    roofline = None
    # (a layer with f <= 4 has no contraction launch in fprop, whose product is formed inside the inverse
    # transform, and one launch for bprop and accGrad together, timed with the pass that comes first)
    timed = [n for n in gemm_names if gemm_live[n]]
    # products one launch forms: with f > 4 and all spectra cached, bprop's launch also forms accGrad's product
    # (one joint launch over the spectrum of dL/dy), and accGrad has no contraction launch of its own
    products = {n: 1 for n in gemm_names}
    if layer.f > 4 and gemm_live["cgemm_bprop"] and not gemm_live["cgemm_accgrad"]:
        products["cgemm_bprop"] = 2
    if timed:
        gemm_ms = float(np.mean([gemm_live[n] for n in timed]))
        per_launch = float(np.mean([products[n] for n in timed]))   # products per launch, mean over the launches
        achieved = per_launch * algo_flops / (gemm_ms * 1e-3) / 1e12
        issued = per_launch * plan.contraction_flops / (gemm_ms * 1e-3) / 1e12
        traffic = None
        tpath = os.path.join(ROOT, "profiles", f"traffic_{layer.name}.json")
        if os.path.exists(tpath):
            traffic = json.load(open(tpath)).get("cgemm_hbm_bytes_per_launch")
        rocprof_us, rocprof_products = None, 1.0
        if os.path.exists(tpath):
            rocprof_us = json.load(open(tpath)).get("cgemm_rocprof_avg_us")
            rocprof_products = json.load(open(tpath)).get("cgemm_products_per_launch", 1.0)
        roofline = {"bound": "mfma", "achieved": achieved, "peak": PEAK_FP32_MFMA_TFLOPS, "unit": "TFLOP/s",
                    "frac": achieved / PEAK_FP32_MFMA_TFLOPS, "traffic": traffic,
                    # the same launches priced three ways: algorithmic flops (8 per complex multiply-add, the
                    # speed-up-equivalent figure), flops the matrix cores actually issue (6: three real products),
                    # both on the event clock of this run; and the issued fraction on rocprofv3's kernel durations
                    # of the stored profile of this workload, if there is one
                    "frac_algorithmic": achieved / PEAK_FP32_MFMA_TFLOPS,
                    "frac_issued": issued / PEAK_FP32_MFMA_TFLOPS,
                    "clock": "HIP events recorded on the launch stream around each contraction launch (includes "
                             "dispatch latency; reads a few us above rocprofv3's kernel duration)",
                    "rocprof_avg_launch_us": rocprof_us,
                    "frac_issued_rocprof": (rocprof_products * plan.contraction_flops / (rocprof_us * 1e-6) / 1e12 / PEAK_FP32_MFMA_TFLOPS
                                            if rocprof_us else None),
                    "launches": {n: {"avg_ms": gemm_live[n], "products": products[n]} for n in timed},
                    "kernel": ("bin_cgemm_kernel (fprop) and bin_cgemm_bprop_accgrad_kernel (both other products in one launch)"
                               if products["cgemm_bprop"] == 2 else
                               "bin_cgemm_kernel" if layer.f > 4 else "streaming kernels for f <= 4 (skinny_kernels.hpp)") +
                              " (mean of the " + "/".join(n[6:] for n in timed) + " launches)",
                    "avg_launch_ms": gemm_ms, "launches_timed": gemm_live_launches,
                    "timing": f"HIP events around the contraction launches of every {EVENT_EVERY}th timed step",
                    "flops_per_launch": per_launch * algo_flops,
                    "issued_mfma_flops_per_launch": per_launch * plan.contraction_flops, "issued_TFLOPs": issued,
                    "issued_frac": issued / PEAK_FP32_MFMA_TFLOPS}
        # With few maps on one side (f = 3) the product has less arithmetic per byte than the chip's
        # ridge point: the same launches are then bound by HBM, and that is the roof to price them against.
        min_bytes = 8.0 * B * (plan.slot_maps(fc.SPEC_X) + plan.slot_maps(fc.SPEC_W) + plan.slot_maps(fc.SPEC_G))
        roofline["min_bytes_per_launch"] = min_bytes   # one product alone; the joint launch reads dL/dy's spectrum once for two
        if algo_flops / min_bytes < PEAK_FP32_MFMA_TFLOPS * 1e12 / (PEAK_HBM_GBS * 1e9):
            gbs = min_bytes / (gemm_ms * 1e-3) / 1e9
            roofline.update({"bound": "hbm", "achieved": gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                             "frac": gbs / PEAK_HBM_GBS, "mfma_TFLOPs": achieved})
    # HBM-side view of the transform stages: algorithmic bytes = unpadded real map + stored half spectrum
    # (images, image extent, transforms): a layer with n > 64 runs one transform per tile
    (L, _), (nt, _), (nt2, _) = plan.tiling   # bench layers are square
    T, T2 = nt * nt, nt2 * nt2
    ext = {"fft_x": (layer.S * layer.f, layer.n, layer.S * layer.f * T),
           "fft_w": (layer.fo * layer.f, layer.k, layer.fo * layer.f),
           "fft_g": (layer.S * layer.fo, layer.no, layer.S * layer.fo * (T + T2) / 2 if L else layer.S * layer.fo),
           "ifft_y": (layer.S * layer.fo, layer.no, layer.S * layer.fo * T),
           "ifft_dx": (layer.S * layer.f, layer.n, layer.S * layer.f * T2),
           "ifft_dw": (layer.fo * layer.f, layer.k, layer.fo * layer.f)}
    stage_report = {}
    for name, ms in stages.items():
        if ms is None:
            continue
        rec = {"avg_ms": ms}
        if name in ext:
            images, e, transforms = ext[name]
            nbytes = images * 4 * e * e + transforms * 8 * B
            if name == "ifft_y" and stages.get("cgemm_fprop") is None:
                # fprop of a layer with f <= 4: no output spectrum exists, the kernel reads the spectra of x and w
                nbytes = images * 4 * e * e + 8 * B * (plan.slot_maps(fc.SPEC_X) + plan.slot_maps(fc.SPEC_W))
                rec["fused_product"] = True
            rec["algorithmic_bytes"] = nbytes
            rec["GBps"] = nbytes / (ms * 1e-3) / 1e9
            rec["frac_hbm_peak"] = rec["GBps"] / PEAK_HBM_GBS
        else:
            # (after the timed steps every stage is bracketed: which launches exist is the same as in the timed region)
            npr = 2 if (name == "cgemm_bprop" and layer.f > 4 and stages.get("cgemm_accgrad") is None) else 1
            rec["products"] = npr
            rec["TFLOPs"] = npr * algo_flops / (ms * 1e-3) / 1e12
            rec["frac_mfma_peak"] = rec["TFLOPs"] / PEAK_FP32_MFMA_TFLOPS
            rec["issued_frac_mfma_peak"] = npr * plan.contraction_flops / (ms * 1e-3) / 1e12 / PEAK_FP32_MFMA_TFLOPS
        stage_report[name] = rec

    out = {
        "metric": "direct-equiv GFLOP/s + ms per fprop/bprop/accGrad, fp32, 1 MI355X",
        "value": 3 * layer.direct_flops / (ms_per_step * 1e-3) / 1e9,
        "unit": "GFLOP/s (direct-equivalent, fprop+bprop+accGrad step)",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "ms_per_step_unbracketed": ms_per_step_unbracketed,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{layer.name}: S={layer.S} f={layer.f} f'={layer.fo} n={layer.n} k={layer.k} "
                               f"(N={plan.fft_size}, {B} bins" + (f", {nt}x{nt} / {nt2}x{nt2} tiles of {L}" if L else "") +
                               "); step = FFT(x,w,dL/dy) + 3 contractions + 3 inverse+crop",
                   "seed": layer.seed},
        "passes": passes,
        "memory_efficient_mode": memory_efficient,
        "stages": stage_report,
        "roofline": roofline,
    }
    return out


def write_report(args):
    """Per-point numbers for every layer: ms per pass (warm / cold), direct-equivalent GFLOP/s, stage fractions."""
    import copy
    from paper_1312_5851_amd import workloads as wl
    a = copy.copy(args)
    a.steps, a.warmup, a.calibration_copy = 20, 3, False
    layers = (list(wl.CONFIGS.values()) + wl.sweep_layers() + wl.paper_table_layers() + wl.fig3_layers()
              + wl.large_layers())
    recs = []
    for layer in layers:
        log(f"report: {layer.name}")
        r = measure(layer, a)
        r.pop("roofline", None)
        recs.append(r)
    json.dump(recs, open(args.report + ".json", "w"), indent=1)
    open(args.report + ".md", "w").write(render_report(layers, recs))


def render_report(layers, recs):
    """The per-layer table of write_report as markdown."""
    head = ("# All layers: BASELINE configs, n x k sweep, paper-table columns, speed-figure axes, tiled layers (one MI355X)\n\n"
            "Command: `python bench.py --report PATH` (per layer: per-pass times, memory-efficient mode, stage table, "
            "then 3 warm-up and 20 timed steps, i.e. the order of the default bench line).  \"no-cache step\" is the same step in the "
            "memory-efficient mode (plan flag RECOMPUTE: every pass transforms its operands again, three-slot workspace).  "
            "bprop and accGrad are timed in alternation: with all spectra cached the first of the two also forms the other's result "
            "spectrum, so their warm times belong together (accGrad's is then the inverse transform alone).  Stage percentages use HIP "
            "events recorded around every launch, on algorithmic bytes / flops against 8 TB/s and 157.3 TFLOP/s; the events read 2-3 us "
            "above rocprofv3's kernel durations, which matters for the 10-20 us transform launches of N <= 16 (rocprofv3 durations: "
            "hot_path_*.md).  Contraction: the first column is matrix-core utilisation in the sense of flops issued (6 per complex "
            "multiply-add: three real products), the second prices the same launches at the 8 flops of the textbook complex "
            "multiply-add and can pass 100; with more than four input maps and both result spectra under 192 MiB, bprop's launch forms "
            "accGrad's product too (one figure for both, `-` for accGrad); for layers with f = 3 the contractions of bprop and accGrad "
            "are one streaming kernel bound by HBM (its matrix-core percentage says nothing) and fprop has no contraction launch "
            "(`-`): its products are formed inside the inverse transform, whose percentage then counts the output bytes and the small "
            "operand spectra only.  `large_*` layers (n > 64) run on overlapping tiles; their transform percentages count image bytes "
            "once plus one spectrum per tile.\n\n")
    lines = ["| layer | S,f,f',n,k | step ms | no-cache step ms | direct-equiv TFLOP/s (step) | fprop warm/cold ms | bprop warm/cold ms | "
             "accGrad warm/cold ms | FFT stages % of 8 TB/s (x,w,g / y,dx,dw) | contraction, % of 157.3 TFLOP/s on issued flops "
             "(fprop,bprop,accGrad) | the same on algorithmic flops |",
             "|---|---|---|---|---|---|---|---|---|---|---|"]
    for layer, r in zip(layers, recs):
        st, ps = r["stages"], r["passes"]
        pct = lambda n: f"{100 * st[n].get('frac_hbm_peak', st[n].get('frac_mfma_peak', 0)):.0f}" if n in st else "-"
        iss = lambda n: f"{100 * st[n]['issued_frac_mfma_peak']:.0f}" if n in st else "-"
        lines.append(f"| {layer.name} | {layer.S},{layer.f},{layer.fo},{layer.n},{layer.k} | {r['ms_per_step']:.3f} | "
                     f"{r['memory_efficient_mode']['ms_per_step']:.3f} | {r['value'] / 1e3:.1f} | " +
                     " | ".join(f"{ps[p]['warm_ms']:.3f} / {ps[p]['cold_ms']:.3f}" for p in ("fprop", "bprop", "accgrad")) +
                     f" | {pct('fft_x')},{pct('fft_w')},{pct('fft_g')} / {pct('ifft_y')},{pct('ifft_dx')},{pct('ifft_dw')} | "
                     f"{iss('cgemm_fprop')},{iss('cgemm_bprop')},{iss('cgemm_accgrad')} | "
                     f"{pct('cgemm_fprop')},{pct('cgemm_bprop')},{pct('cgemm_accgrad')} |")
    return head + "\n".join(lines) + "\n"


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="mid", help="layer name from paper_1312_5851_amd.workloads")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-stage-events", action="store_true", help="do not bracket kernels with HIP events")
    ap.add_argument("--report", metavar="PATH", help="also measure the four headline layers, the n x k sweep, the "
                    "paper's table columns and its figure's three axes (fewer steps each) and write PATH.json and PATH.md")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run a plain 256 MiB device copy three times (reference for HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on exactly one GPU (every box has one); --gpus must be 1")

    import torch
    from paper_1312_5851_amd import fftconv as fc
    from paper_1312_5851_amd import workloads as wl

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    layer = wl.by_name(args.workload)
    inputs = wl.make_inputs(layer)
    # the plain-copy rate first: it is context for the transform stages, and the card has left its idle
    # clocks by the time the warm-up steps start
    # (not in a counter-calibration run: its only copy launches must be the 256 MiB ones)
    copy_gbps = None if args.calibration_copy else copy_bandwidth()
    out = measure(layer, args, inputs)
    out["hbm_copy_GBps"] = copy_gbps
    x, w, g = inputs
    if not args.no_cpu_baseline:
        log("timing the CPU oracle on a bounded sample ...")
        out["cpu_baseline"] = cpu_baseline(layer, x, w, g)
    print(json.dumps(out), flush=True)
    if args.report:
        write_report(args)


if __name__ == "__main__":
    main()
