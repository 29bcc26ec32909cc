#!/usr/bin/env python3
"""Benchmark of the GLEAM module step on one MI355X.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload 0..4]

One step = one gleam_module_fwd + one gleam_module_bwd (data-consistency step, prox forward, local loss,
module-confined backward), all inputs resident in HBM before the timed region.  The default workload (1) is
the knee-shaped 2D one (640x368, 15 coils, batch 2, fp32, 64-channel two-resblock prox); --workload picks
another of the five synthetic configurations (0 tiny 2D, 2 brain-shaped bf16, 3 3D volume, 4 2D+t cine).
Prints ONE JSON line with the module steps/s, the roofline of the dominant kernel (HIP-event timed inside
the library), the SENSE normal operator's bandwidth, and the CPU oracle timed on the host cores as a
reported baseline (default workload and the small ones only: the oracle needs minutes on the others).
"""
import argparse
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

# HBM traffic per launch (bytes) from the two rocprofv3 --pmc runs (FETCH_SIZE, then WRITE_SIZE, KiB per
# dispatch) of `bench.py --steps 2 --warmup 1 --no-cpu-baseline --calibrate`, summarised in
# profiles/module_step_knee2d_hbm_traffic.txt.  Scaling: the 256 MiB calibration copy reads 131 100 KiB on
# FETCH_SIZE (factor 2.0: the counter under-reports 128-byte requests) and 262 144 KiB on WRITE_SIZE (1.0).
MEASURED_TRAFFIC = {
    "conv_wino_kernel<RELU> fwd+dgrad 64->64 3x3 (Winograd F(2x2,3x3))": 1.126e5 * 1024 * 2.0 + 1.192e5 * 1024 * 1.0,
    "wgrad_wino_kernel<RELU> wgrad 64->64 3x3 (Winograd F(2x2,3x3))": 1.18465e5 * 1024 * 2.0 + 6.56e4 * 1024 * 1.0,
}

# library launch label -> GPU kernel it runs (forward and data gradient of a 64->64 layer are one kernel)
KERNEL_OF = {
    "conv_fwd_64to64_t9": "conv_wino_kernel<RELU> fwd+dgrad 64->64 3x3 (Winograd F(2x2,3x3))",
    "conv_dgrad_64to64_t9": "conv_wino_kernel<RELU> fwd+dgrad 64->64 3x3 (Winograd F(2x2,3x3))",
    "conv_wgrad_64to64_t9": "wgrad_wino_kernel<RELU> wgrad 64->64 3x3 (Winograd F(2x2,3x3))",
}


def aggregate(records):
    agg = {}
    for name, flops, nbytes, ms in records:
        a = agg.setdefault(name, {"launches": 0, "ms": 0.0, "flops": 0.0, "bytes": 0.0})
        a["launches"] += 1
        a["ms"] += ms
        a["flops"] += flops
        a["bytes"] += nbytes
    return agg


def prox_text(prox):
    ls = prox.layers
    taps = sorted({f"{l.kt}x{l.kd}x{l.kh}x{l.kw}" for l in ls})
    skips = sum(1 for l in ls if l.skip_src >= 0)
    return (f"{len(ls)} convs, {max(l.cout for l in ls[:-1])} ch, kernels (t,d,h,w) {'/'.join(taps)}, "
            f"{skips} skip adds, {'bf16 operands + fp32 accumulate' if prox.dtype == 1 else 'fp32'}")


def cpu_baseline(case, min_seconds=10.0, max_reps=3):
    """Times the oracle (as it stands) on whole module steps of the workload: full batch, forward + backward,
    repeated until min_seconds of CPU work have been spent (at most max_reps times)."""
    from oracle import gleam_oracle as og
    g = case.geom
    reps, t0 = 0, time.perf_counter()
    while True:
        f = og.module_fwd(g, case.prox, case.x_in, case.S, case.M, case.y, case.alpha, case.theta, case.x_true)
        og.module_bwd(case.prox, case.theta, f)
        reps += 1
        dt = time.perf_counter() - t0
        if dt >= min_seconds or reps >= max_reps:
            break
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    return {"value": reps / dt, "unit": "module steps/s", "cores": int(cores), "kind": "oracle",
            "sample": f"{reps} whole module step(s) of the workload (full batch of {g.B}, fwd + bwd of the float64 "
                      f"numpy oracle) in {dt:.1f} s"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate", action="store_true",
                    help="also run one plain 256 MiB device copy (known size) so that rocprofv3 --pmc "
                         "FETCH_SIZE / WRITE_SIZE readings can be scaled to bytes")
    ap.add_argument("--workload", type=int, default=1, choices=range(5),
                    help="synthetic configuration: 0 tiny2d, 1 knee2d (default), 2 brain2d bf16, 3 vol3d, 4 cine2dt")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no sharding, no collectives); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2207_08393_amd import binding as gb
    from paper_2207_08393_amd import synth
    from paper_2207_08393_amd.runner import ModuleRunner, SenseRunner

    if args.calibrate:
        a = torch.ones(64 * 1024 * 1024, device="cuda")     # 256 MiB of float32
        b = torch.empty_like(a)
        b.copy_(a)
        torch.cuda.synchronize()
        del a, b
    case = synth.make_case(args.workload)
    peak = PEAK_BF16_MFMA_TFLOPS if case.prox.dtype == 1 else PEAK_FP32_MFMA_TFLOPS
    g = case.geom
    r = ModuleRunner(case)
    sr = SenseRunner(g, case.x_in, case.S, case.M)
    torch.cuda.synchronize()

    for _ in range(args.warmup):
        r.step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        r.step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = 1e3 * dt / args.steps

    # the same steps again with every kernel bracketed by HIP events on the launch stream
    gb.gleam_profile_begin()
    for _ in range(args.steps):
        r.step()
    agg = aggregate(gb.gleam_profile_end())
    mfma = {k: v for k, v in agg.items() if k.startswith("conv_")}
    by_kernel = {}
    for k, v in mfma.items():
        b = by_kernel.setdefault(KERNEL_OF.get(k, k), {"launches": 0, "ms": 0.0, "flops": 0.0, "bytes": 0.0})
        for f in b:
            b[f] += v[f]
    dom = max(by_kernel, key=lambda k: by_kernel[k]["ms"])
    d = by_kernel[dom]
    avg_ms = d["ms"] / d["launches"]
    achieved = d["flops"] / d["launches"] / (avg_ms * 1e-3) / 1e12
    roofline = {"kernel": dom, "bound": "mfma", "achieved": achieved, "peak": peak,
                "unit": "TFLOP/s", "frac": achieved / peak, "avg_launch_ms": avg_ms,
                "launches_per_step": d["launches"] / args.steps, "traffic": MEASURED_TRAFFIC.get(dom)}
    if "Winograd" in dom:
        # algorithmic flops are those of the direct 3x3 convolution; F(2x2,3x3) executes 16 multiplications per
        # 2x2 outputs and channel pair instead of 36, so the matrix cores run 4/9 of them
        roofline["executed_tflops"] = achieved * 16.0 / 36.0
        roofline["executed_frac"] = achieved * 16.0 / 36.0 / peak
        roofline["note"] = ("achieved counts the direct convolution's flops (2*9*K*N per pixel); the Winograd kernel "
                            "executes 4/9 of them on the matrix cores, so frac can exceed 1")
    conv_ms = sum(v["ms"] for v in mfma.values())
    conv_tflops = sum(v["flops"] for v in mfma.values()) / (conv_ms * 1e-3) / 1e12
    kernels = {k: {"avg_ms": v["ms"] / v["launches"], "per_step": v["launches"] / args.steps,
                   "tflops": (v["flops"] / (v["ms"] * 1e-3) / 1e12) if v["flops"] else None,
                   "gbs": v["bytes"] / (v["ms"] * 1e-3) / 1e9} for k, v in sorted(agg.items())}

    # SENSE normal operator A^H A on its own: algorithmic bytes / event time of its three sweeps
    for _ in range(args.warmup):
        sr.run()
    torch.cuda.synchronize()
    gb.gleam_profile_begin()
    for _ in range(args.steps):
        sr.run()
    sagg = aggregate(gb.gleam_profile_end())
    s_ms = sum(v["ms"] for v in sagg.values()) / args.steps
    s_bytes = sum(v["bytes"] for v in sagg.values()) / args.steps
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        sr.run()
    torch.cuda.synchronize()
    s_wall_ms = 1e3 * (time.perf_counter() - t0) / args.steps
    sense = {"bound": "hbm", "achieved": s_bytes / (s_ms * 1e-3) / 1e9, "peak": PEAK_HBM_GBS, "unit": "GB/s",
             "frac": s_bytes / (s_ms * 1e-3) / 1e9 / PEAK_HBM_GBS, "algorithmic_bytes": s_bytes,
             "kernel_ms": s_ms, "wall_ms_per_call": s_wall_ms,
             "sweeps": {k: v["ms"] / v["launches"] for k, v in sagg.items()}}

    # The same operator when the mask does not depend on the outermost transformed axis (the line masks of the 2D
    # workloads; the read-out of the 3D one): that transform cancels, and with one transformed axis less the 2D
    # workloads run the whole operator in a single sweep (ndim_fft = 1).  Reported beside the general path.
    single = None
    if g.ndim_fft == 2 and bool((case.M == case.M[..., :1, :]).all()):
        g1 = synth.Geom(1, g.B, g.C, g.T, g.D, g.H, g.W)
        s1 = SenseRunner(g1, case.x_in, case.S, case.M)
        for _ in range(args.warmup):
            s1.run()
        torch.cuda.synchronize()
        gb.gleam_profile_begin()
        for _ in range(args.steps):
            s1.run()
        a1 = aggregate(gb.gleam_profile_end())
        ms1 = sum(v["ms"] for v in a1.values()) / args.steps
        b1 = sum(v["bytes"] for v in a1.values()) / args.steps
        single = {"kernel_ms": ms1, "algorithmic_bytes": b1, "achieved": b1 / (ms1 * 1e-3) / 1e9, "unit": "GB/s",
                  "frac": b1 / (ms1 * 1e-3) / 1e9 / PEAK_HBM_GBS,
                  "note": "ndim_fft = 1 on the same x, S, mask: equals the 2D operator because the mask is constant along H"}
        del s1
    sense["single_axis"] = single

    # one greedy training iteration (Alg. 1): all M modules of the workload in order, each fwd + bwd + Adam
    from paper_2207_08393_amd.runner import GreedyRunner
    del sr
    gr = GreedyRunner(case, [case.theta] * case.n_modules, lr=1e-4)
    gr.iteration(1)
    torch.cuda.synchronize()
    n_it = max(2, args.steps // case.n_modules)
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

    # a module of two unrolled iterations (N/M = 2): fwd + bwd through both prox networks and the DC step between
    from paper_2207_08393_amd.runner import DeepModuleRunner
    dr = DeepModuleRunner(case, [case.theta, case.theta])
    dr.step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(n_it):
        dr.step()
    torch.cuda.synchronize()
    deep_ms = 1e3 * (time.perf_counter() - t0) / n_it
    del dr

    # one MoDL module (Eq. 6-8) on the same data: prox, 10 CG steps forward, 10 CG steps backward, prox backward
    from paper_2207_08393_amd.runner import ModlRunner
    mr = ModlRunner(case, 0.05, 10)
    mr.step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(n_it):
        mr.step()
    torch.cuda.synchronize()
    modl_ms = 1e3 * (time.perf_counter() - t0) / n_it
    del mr

    out = {"metric": "GLEAM module fwd+bwd steps/s", "value": args.steps / dt, "unit": "module steps/s",
           "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": "bf16" if case.prox.dtype == 1 else "f32", "data": "synthetic",
           "config": {"workload": case.name, "image": [d_ for d_ in (g.T, g.D, g.H, g.W) if d_ > 1],
                      "fft_dims": g.ndim_fft, "coils": g.C, "batch": g.B, "prox": prox_text(case.prox),
                      "loss": "l1" if case.prox.loss_kind == 1 else "l2",
                      "modules_per_greedy_iteration": case.n_modules},
           "roofline": roofline,
           "conv_all": {"tflops": conv_tflops, "frac_of_mfma_peak": conv_tflops / peak,
                        "ms_per_step": conv_ms / args.steps},
           "sense_normal": sense, "kernels": kernels,
           "greedy_iteration": {"modules": case.n_modules, "ms": greedy_ms, "iterations_per_s": 1e3 / greedy_ms,
                                "includes": "fwd + bwd + Adam update of every module, detached hand-off",
                                "memory": mem}}
    out["deep_module"] = {"iterations_per_module": 2, "ms": deep_ms,
                          "includes": "fwd + bwd of one module holding two unrolled iterations"}
    out["modl_module"] = {"mu": 0.05, "cg_steps": 10, "ms": modl_ms,
                          "includes": "fwd + bwd of one MoDL module: prox, 10 CG steps each way (20 A^H A sweeps)"}
    if not args.no_cpu_baseline and args.workload in (0, 1, 4):
        out["cpu_baseline"] = cpu_baseline(case)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
