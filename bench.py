#!/usr/bin/env python3
"""Benchmark of the GLEAM module step on one MI355X.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload 0..4] [--only] [--no-cpu-baseline] [--calibrate]

One step = one gleam_module_fwd + one gleam_module_bwd (data-consistency step, prox forward, local loss,
module-confined backward), all inputs resident in HBM before the timed region.  The headline workload (3, the
default) is the largest of the five synthetic configurations that fits one GPU: the 3D volume (256x160x160, 8 coils,
3D transform, 3x3x3 prox with 32 channels, fp32).  The other four (0 tiny 2D, 1 knee-shaped 2D, 2 brain-shaped 2D with
bf16 convolutions, 4 2D+t cine) are measured in the same run and reported in the `workloads` block (--only skips
them; --workload N makes another one the headline).

Prints ONE JSON line: module steps/s of the headline workload; `roofline` of its dominant convolution kernel
(HIP-event timed inside the library on the launch stream; `achieved` = flops issued on the matrix cores / time,
`effective_tflops` = the direct convolution's flops / time, which is larger for the Winograd kernels); the SENSE
normal operator's bandwidth; greedy-iteration, two-iteration-module and MoDL-module times; and `cpu_baseline`,
the CPU oracle timed on the host cores on a bounded sample of the same workload (a reported baseline, not a target).
"""
import argparse
import dataclasses
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_FP32_MFMA_TFLOPS = 157.3
PEAK_BF16_MFMA_TFLOPS = 2500.0
PEAK_HBM_GBS = 8000.0

# HBM traffic per launch (bytes), keyed by (workload, launch label of the dominant kernel), from the two rocprofv3
# --pmc runs (FETCH_SIZE, then WRITE_SIZE, KiB per dispatch) of `bench.py --workload N --only --steps 2 --warmup 1
# --no-cpu-baseline --calibrate` summarised in profiles/module_step_<workload>_hbm_traffic.txt.  Scaling: the 256 MiB
# calibration copy of the same run reads 131 100 KiB on FETCH_SIZE (factor 2.0: the counter counts 64-byte units of
# 128-byte requests) and 262 144 KiB on WRITE_SIZE (factor 1.0).  A pair without a profile of its own reports null.
MEASURED_TRAFFIC = {
    ("knee2d_640x368_c15_b2", "conv_fwd+dgrad_64to64_t9"): 1.126e5 * 1024 * 2.0 + 1.192e5 * 1024 * 1.0,
    ("knee2d_640x368_c15_b2", "conv_wgrad_64to64_t9"): 1.18465e5 * 1024 * 2.0 + 6.56e4 * 1024 * 1.0,
    ("vol3d_256x160x160_c8_b1", "conv_fwd+dgrad_32to32_t27"): 1.292e6 * 1024 * 2.0 + 8.202e5 * 1024 * 1.0,
    ("vol3d_256x160x160_c8_b1", "conv_wgrad_32to32_t27"): 8.663e5 * 1024 * 2.0 + 9.939e4 * 1024 * 1.0,
    ("cine2dt_20x192x160_c8_b1", "conv_fwd+dgrad_64to64_t9"): 1.36e5 * 1024 * 2.0 + 1.536e5 * 1024 * 1.0,
    ("cine2dt_20x192x160_c8_b1", "conv_wgrad_64to64_t9"): 1.539e5 * 1024 * 2.0 + 6.56e4 * 1024 * 1.0,
    ("brain2d_640x320_c16_b4_bf16", "conv_bf16_fwd+dgrad_128to128_t9"): 1.235e5 * 1024 * 2.0 + 2.0907e5 * 1024 * 1.0,
    ("brain2d_640x320_c16_b4_bf16", "conv_bf16_wgrad_128to128_t9"): 2.091e5 * 1024 * 2.0 + 6.918e4 * 1024 * 1.0,
}

WORKLOAD_NAMES = ("tiny2d", "knee2d", "brain2d bf16", "vol3d", "cine2dt")


def aggregate(records):
    agg = {}
    for name, flops, nbytes, ms, mfma in records:
        a = agg.setdefault(name, {"launches": 0, "ms": 0.0, "flops": 0.0, "bytes": 0.0, "mfma_flops": 0.0})
        a["launches"] += 1
        a["ms"] += ms
        a["flops"] += flops
        a["bytes"] += nbytes
        a["mfma_flops"] += mfma
    return agg


def prox_text(prox):
    ls = prox.layers
    taps = sorted({f"{l.kt}x{l.kd}x{l.kh}x{l.kw}" for l in ls})
    skips = sum(1 for l in ls if l.skip_src >= 0)
    return (f"{len(ls)} convs, {max(l.cout for l in ls[:-1])} ch, kernels (t,d,h,w) {'/'.join(taps)}, "
            f"{skips} skip adds, {'bf16 operands + fp32 accumulate' if prox.dtype == 1 else 'fp32'}")


def cpu_sample(case, idx):
    """A bounded sample of the workload for the oracle (about 10-30 s of CPU work): (case to run, fraction of one
    module step it stands for, description).  The oracle's cost is linear in the pixels of the prox and the sample
    keeps the architecture, the coils and the transform lengths of the in-plane axes."""
    g = case.geom
    if idx == 2:      # brain-shaped: one of the four batch samples
        c = dataclasses.replace(case, geom=dataclasses.replace(g, B=1), x_true=case.x_true[:1], S=case.S[:1], M=case.M[:1],
                                y=case.y[:1], x_in=case.x_in[:1])
        return c, 1.0 / g.B, f"batch sample 1 of {g.B} (whole images, all {g.C} coils)"
    if idx == 3:      # 3D volume: a slab of 32 of the 256 read-out partitions (timing only: a cropped k-space is not a
        D = 32        # measurement of the cropped volume, and the values are not used)
        import numpy as np
        c = dataclasses.replace(case, geom=dataclasses.replace(g, D=D), x_true=case.x_true[:, :, :D], S=case.S[:, :, :D],
                                M=case.M[:, :, :D], y=np.ascontiguousarray(case.y[:, :, :, :D]), x_in=case.x_in[:, :, :D])
        return c, D / g.D, (f"slab of {D} of the {g.D} partitions along the read-out (arrays cropped along D: the prox and "
                            f"the in-plane transforms at full size, the transform along D at length {D})")
    return case, 1.0, "whole module steps of the workload (full batch)"


def cpu_baseline(case, idx, min_seconds=3.0, max_reps=5):
    """Times the oracle (as it stands) on a bounded sample of the workload, forward + backward, and scales the rate to
    whole module steps of the workload."""
    from oracle import gleam_oracle as og
    c, frac, what = cpu_sample(case, idx)
    g = c.geom
    reps, t0 = 0, time.perf_counter()
    while True:
        f = og.module_fwd(g, c.prox, c.x_in, c.S, c.M, c.y, c.alpha, c.theta, c.x_true)
        og.module_bwd(c.prox, c.theta, f)
        reps += 1
        dt = time.perf_counter() - t0
        if dt >= min_seconds or reps >= max_reps:
            break
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    return {"value": reps * frac / dt, "unit": "module steps/s", "cores": int(cores), "kind": "oracle",
            "sample": f"{what}: {reps} pass(es), fwd + bwd of the float64 numpy oracle, {dt:.1f} s; rate scaled by the "
                      f"sample's share of a step ({frac:.4g})"}


def conv_rooflines(agg, steps, peak, workload):
    """Per GPU kernel (forward and data gradient of one layer shape are one kernel): average launch time, rate of the
    flops issued on the matrix cores and its fraction of the peak, rate in direct-convolution flops."""
    groups = {}
    for k, v in agg.items():
        if not (k.startswith("conv_") and v["mfma_flops"] > 0):
            continue
        if "_2to" in k or "to2_" in k:      # the two-channel first / last layers are HBM-bound (about 9 flop/B)
            continue
        key = k.replace("conv_fwd_", "conv_fwd+dgrad_").replace("conv_dgrad_", "conv_fwd+dgrad_") \
               .replace("conv_bf16_fwd_", "conv_bf16_fwd+dgrad_").replace("conv_bf16_dgrad_", "conv_bf16_fwd+dgrad_")
        b = groups.setdefault(key, {"launches": 0, "ms": 0.0, "flops": 0.0, "mfma_flops": 0.0})
        for f in b:
            b[f] += v[f]
    out = {}
    for key, d in groups.items():
        sec = d["ms"] * 1e-3
        issued = d["mfma_flops"] / sec / 1e12
        out[key] = {"kernel": key + (" (Winograd F(2x2,3x3): 4/9 of the direct flops issued)" if d["mfma_flops"] < 0.99 * d["flops"] else ""),
                    "bound": "mfma", "achieved": issued, "peak": peak, "unit": "TFLOP/s", "frac": issued / peak,
                    "effective_tflops": d["flops"] / sec / 1e12,
                    "algorithmic_flops_per_launch": d["flops"] / d["launches"],
                    "avg_launch_ms": d["ms"] / d["launches"], "launches_per_step": d["launches"] / steps,
                    "ms_per_step": d["ms"] / steps, "traffic": MEASURED_TRAFFIC.get((workload, key))}
    return out


def sense_block(gb, torch, sr, steps, warmup):
    """gleam_sense_normal on its own: algorithmic bytes / HIP-event time of its sweeps."""
    for _ in range(warmup):
        sr.run()
    torch.cuda.synchronize()
    gb.gleam_profile_begin()
    for _ in range(steps):
        sr.run()
    sagg = aggregate(gb.gleam_profile_end())
    s_ms = sum(v["ms"] for v in sagg.values()) / steps
    s_bytes = sum(v["bytes"] for v in sagg.values()) / steps
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        sr.run()
    torch.cuda.synchronize()
    wall = 1e3 * (time.perf_counter() - t0) / steps
    gbs = s_bytes / (s_ms * 1e-3) / 1e9
    return {"bound": "hbm", "achieved": gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": gbs / PEAK_HBM_GBS,
            "algorithmic_bytes": s_bytes, "kernel_ms": s_ms, "wall_ms_per_call": wall,
            "sweeps": {k: v["ms"] / v["launches"] for k, v in sagg.items()}}


def measure(idx, steps, warmup, full, with_cpu):
    """Everything reported for one workload.  full: also the per-kernel table, the single-axis SENSE path and the
    greedy / two-iteration / MoDL legs (the headline); otherwise the compact entry of the `workloads` block."""
    import torch
    from paper_2207_08393_amd import binding as gb
    from paper_2207_08393_amd import synth
    from paper_2207_08393_amd.runner import DeepModuleRunner, GreedyRunner, ModlRunner, ModuleRunner, SenseRunner

    case = synth.make_case(idx)
    peak = PEAK_BF16_MFMA_TFLOPS if case.prox.dtype == 1 else PEAK_FP32_MFMA_TFLOPS
    g = case.geom
    r = ModuleRunner(case)
    torch.cuda.synchronize()
    for _ in range(warmup):
        r.step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        r.step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0

    # the same steps again with every kernel bracketed by HIP events on the launch stream
    gb.gleam_profile_begin()
    for _ in range(steps):
        r.step()
    agg = aggregate(gb.gleam_profile_end())
    convs = conv_rooflines(agg, steps, peak, case.name)
    dom = max(convs.values(), key=lambda d: d["ms_per_step"]) if convs else None
    mfma = {k: v for k, v in agg.items() if k.startswith("conv_") and not ("_2to" in k or "to2_" in k)}
    conv_ms = sum(v["ms"] for v in mfma.values())
    conv_all = {"effective_tflops": sum(v["flops"] for v in mfma.values()) / (conv_ms * 1e-3) / 1e12,
                "issued_tflops": sum(v["mfma_flops"] for v in mfma.values()) / (conv_ms * 1e-3) / 1e12,
                "ms_per_step": conv_ms / steps}
    conv_all["issued_frac_of_mfma_peak"] = conv_all["issued_tflops"] / peak
    del r

    sr = SenseRunner(g, case.x_in, case.S, case.M)
    sense = sense_block(gb, torch, sr, steps, warmup)
    del sr

    res = {"workload": case.name, "value": steps / dt, "ms_per_step": 1e3 * dt / steps, "timed_seconds": dt,
           "dtype": "bf16" if case.prox.dtype == 1 else "f32", "roofline": dom, "conv_all": conv_all, "sense_normal": sense,
           "case": case}
    if full:
        res["conv_kernels"] = convs
        res["kernels"] = {k: {"avg_ms": v["ms"] / v["launches"], "per_step": v["launches"] / steps,
                              "tflops": (v["flops"] / (v["ms"] * 1e-3) / 1e12) if v["flops"] else None,
                              "gbs": v["bytes"] / (v["ms"] * 1e-3) / 1e9} for k, v in sorted(agg.items())}
        # When the mask does not depend on the outermost transformed axis (the line masks of the 2D workloads, the
        # fully sampled read-out of the 3D one) that transform cancels in A^H A: the library's own check and its
        # k-space-to-hybrid-space transform give the same problem with one transformed axis less (exact, not an
        # approximation).  Reported beside the general path, each against its own algorithmic bytes.
        reduced = None
        gfull = gb.make_geom(g)
        if g.ndim_fft >= 2 and gb.gleam_mask_constant_along_outer_axis(gfull, case.M):
            s1 = SenseRunner(synth.Geom(g.ndim_fft - 1, g.B, g.C, g.T, g.D, g.H, g.W, g.centred), case.x_in, case.S, case.M)
            b1 = sense_block(gb, torch, s1, steps, warmup)
            del s1
            reduced = {"ndim_fft": g.ndim_fft - 1, "sense_normal": {k: b1[k] for k in ("kernel_ms", "algorithmic_bytes", "achieved", "unit", "frac", "sweeps")}}
            r1 = ModuleRunner(case, separable=True)
            for _ in range(warmup):
                r1.step()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(steps):
                r1.step()
            torch.cuda.synchronize()
            dt1 = time.perf_counter() - t0
            reduced["module_ms_per_step"] = 1e3 * dt1 / steps
            reduced["module_steps_per_s"] = steps / dt1
            reduced["note"] = ("same x, S, mask and results as the headline step; the measured k-space was taken to hybrid "
                               "space once by gleam_kspace_to_hybrid (not timed: once per scan)")
            del r1
        res["reduced_problem"] = reduced

        # one greedy training iteration (Alg. 1): all M modules of the workload in order, each fwd + bwd + Adam
        gr = GreedyRunner(case, [case.theta] * case.n_modules, lr=1e-4)
        gr.iteration(1)
        torch.cuda.synchronize()
        n_it = max(2, steps // case.n_modules)
        t0 = time.perf_counter()
        for k in range(n_it):
            gr.iteration(2 + k)
        torch.cuda.synchronize()
        greedy_ms = 1e3 * (time.perf_counter() - t0) / n_it
        # activation memory: greedy training keeps one module's activations at a time; end-to-end backpropagation
        # through the same N = M modules would keep all of them (estimate, not built)
        mem = {"activations_one_module_bytes": gr.saved_bytes, "workspace_bytes": gr.ws_bytes,
               "greedy_peak_bytes": gr.saved_bytes + gr.ws_bytes,
               "end_to_end_estimate_bytes": case.n_modules * gr.saved_bytes + gr.ws_bytes,
               "ratio": (case.n_modules * gr.saved_bytes + gr.ws_bytes) / (gr.saved_bytes + gr.ws_bytes)}
        del gr
        res["greedy_iteration"] = {"modules": case.n_modules, "ms": greedy_ms, "iterations_per_s": 1e3 / greedy_ms,
                                   "includes": "fwd + bwd + Adam update of every module, detached hand-off", "memory": mem}

        # a module of two unrolled iterations (N/M = 2): fwd + bwd through both prox networks and the DC step between
        dr = DeepModuleRunner(case, [case.theta, case.theta])
        dr.step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n_it):
            dr.step()
        torch.cuda.synchronize()
        res["deep_module"] = {"iterations_per_module": 2, "ms": 1e3 * (time.perf_counter() - t0) / n_it,
                              "includes": "fwd + bwd of one module holding two unrolled iterations"}
        del dr

        # one MoDL module (Eq. 6-8) on the same data: prox, 10 CG steps forward, 10 CG steps backward, prox backward
        mr = ModlRunner(case, 0.05, 10)
        mr.step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n_it):
            mr.step()
        torch.cuda.synchronize()
        res["modl_module"] = {"mu": 0.05, "cg_steps": 10, "ms": 1e3 * (time.perf_counter() - t0) / n_it,
                              "includes": "fwd + bwd of one MoDL module: prox, 10 CG steps each way (20 A^H A sweeps)"}
        del mr
    torch.cuda.empty_cache()
    if with_cpu:
        res["cpu_baseline"] = cpu_baseline(case, idx)
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=40)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--only", action="store_true", help="measure the headline workload only (no `workloads` block)")
    ap.add_argument("--calibrate", action="store_true",
                    help="also run one plain 256 MiB device copy (known size) so that rocprofv3 --pmc "
                         "FETCH_SIZE / WRITE_SIZE readings can be scaled to bytes")
    ap.add_argument("--workload", type=int, default=3, choices=range(5),
                    help="headline configuration: 0 tiny2d, 1 knee2d, 2 brain2d bf16, 3 vol3d (default: the largest), 4 cine2dt")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no sharding, no collectives); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch

    if args.calibrate:
        a = torch.ones(64 * 1024 * 1024, device="cuda")     # 256 MiB of float32
        b = torch.empty_like(a)
        b.copy_(a)
        torch.cuda.synchronize()
        del a, b
    cpu = not args.no_cpu_baseline
    head = measure(args.workload, args.steps, args.warmup, True, cpu)
    case = head.pop("case")
    g = case.geom
    out = {"metric": "GLEAM module fwd+bwd steps/s", "value": head["value"], "unit": "module steps/s",
           "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": head["ms_per_step"],
           "timed_seconds": head["timed_seconds"],
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": head["dtype"], "data": "synthetic",
           "config": {"workload": case.name, "image": [d_ for d_ in (g.T, g.D, g.H, g.W) if d_ > 1],
                      "fft_dims": g.ndim_fft, "coils": g.C, "batch": g.B, "prox": prox_text(case.prox),
                      "loss": "l1" if case.prox.loss_kind == 1 else "l2",
                      "modules_per_greedy_iteration": case.n_modules},
           "roofline": head["roofline"], "conv_kernels": head["conv_kernels"], "conv_all": head["conv_all"],
           "sense_normal": head["sense_normal"], "reduced_problem": head["reduced_problem"], "kernels": head["kernels"],
           "greedy_iteration": head["greedy_iteration"], "deep_module": head["deep_module"],
           "modl_module": head["modl_module"]}
    if cpu:
        out["cpu_baseline"] = head["cpu_baseline"]
    del case
    if not args.only:
        others = {}
        for idx in range(5):
            if idx == args.workload:
                continue
            # the small workloads get as many steps as it takes to time about as long as the headline does
            m = measure(idx, max(args.steps, 20), args.warmup, False, cpu)
            m.pop("case")
            name = m.pop("workload")
            m["steps_per_s"] = m.pop("value")
            rf, sn = m["roofline"], m["sense_normal"]
            m["dominant_conv_frac"] = rf["frac"] if rf else None
            m["sense_normal_frac"] = sn["frac"]
            m["sense_normal"] = {k: sn[k] for k in ("achieved", "unit", "frac", "algorithmic_bytes", "kernel_ms")}
            others[name] = m
        out["workloads"] = others
    print(json.dumps(out))


if __name__ == "__main__":
    main()
