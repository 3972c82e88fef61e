#!/usr/bin/env python3
"""Benchmark of the Lightplane Renderer hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config large]

One step = one pass of the whole hot path over one batch of synthetic rays: forward
(sample, interpolate, decode, composite), MSE loss gradient, zeroing of the gradient
buffers, backward (recompute, emission-absorption VJP, MLP backward, scatter into the
grid and MLP gradients).  Inputs are resident in HBM before the timed region.  Prints
ONE JSON line: ray-samples/s of forward+backward; three roofline views of the dominant kernel
(the backward) over its HIP-event duration, with the one that binds first; and the CPU oracle
timed on a bounded ray subset of the same workload on this machine's host cores.

Roofline views (`roofline`):
  * "mfma": the MLP contractions run on the bf16 matrix cores with fp32 operands split into
    hi + lo, three products per multiply-add.  achieved = 3 products x 3 F FLOP per sample
    (recompute, input gradients, weight gradients; F = the MLP's forward FLOPs) x samples /
    duration, against the dense bf16 peak.  This is the unit the kernel is closest to, together
    with the vector ALU work that feeds it (the kernel is bound by instruction issue, see
    profiles/), so it is reported as THE bound;
  * "hbm_effective": the algorithmic no-reuse bytes (every sample re-reads its corners and adds a
    gradient of the same size) / duration against the HBM peak: an EFFECTIVE bandwidth, met
    mostly from the caches (it can exceed the peak where the reuse is high);
  * "hbm_counters": the HBM bytes the profiler's FETCH_SIZE / WRITE_SIZE counters saw per launch
    (`traffic`, from profiles/) / duration.
"""
from __future__ import annotations

import argparse
import json
import sys
import time

import numpy as np

HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0

# HBM bytes per launch of the backward kernel from two rocprofv3 --pmc runs (FETCH_SIZE scaled
# by 2.0, WRITE_SIZE by 1.0 against a 1 GiB copy kernel in the same run); the summary with the
# commands is profiles/large_voxel256_fwd_bwd_kernels.md.  None = not measured for that workload.
MEASURED_BWD_HBM_BYTES = {"large": 19.51e9 + 65.42e9}
# 64-byte lines of atomic adds per launch of the backward kernel: TCC_ATOMIC (each request is one line,
# written through as 64 bytes: WRITE_SIZE / 64 gives the same number); profiles/atomic_line_rate.md.
MEASURED_BWD_ATOMIC_LINES = {"large": 65.42e9 / 64, "batched": 257.0e9 / 64, "voxel": 171758784.0,
                             "contract": 140152160.0, "single_scene": 15266496.0, "decoder": 52144736.0,
                             "hash": 10885988.0}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="large",
                    help="workload: tiny | single_scene | voxel | batched | large")
    ap.add_argument("--math", default="default", choices=["default", "generic", "bf16x3"])
    ap.add_argument("--aabb", type=float, default=None,
                    help="half-width of the grid box (default: the workload's, which contains every sample; "
                         "1.0 = the object box, about half the samples clamp to the border)")
    ap.add_argument("--grid-dtype", default="f32", choices=["f32", "bf16", "f16"],
                    help="storage type of the grid on the GPU (gradients stay f32)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=20.0)
    ap.add_argument("--also", default="tiny,single_scene,voxel,batched,large:bf16,contract,decoder,decoder_paper,"
                                      "hash,hexplane,splat_naive,splat_mlp",
                    help="further workloads reported for context under 'also' (comma-separated, '' to skip; "
                         "name:bf16 / name:f16 = that workload with the grid stored in reduced precision)")
    ap.add_argument("--coexecution", action="store_true",
                    help="instead of the benchmark: time how one SIMD overlaps matrix and vector instructions "
                         "(one JSON line)")
    ap.add_argument("--atomic-rate", action="store_true",
                    help="instead of the benchmark: time how many 64-byte lines of fp32 atomic adds the GPU retires "
                         "per second (one JSON line)")
    ap.add_argument("--ws-phases", action="store_true",
                    help="with a measurement build of the library (LP_EXTRA_HIPCC_FLAGS=-DLP_WS_PHASES python "
                         "paper_2404_19760_amd/build.py): after the run, print where the two roles of the two-wave "
                         "backward spend their cycles (a second JSON line)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 1 GiB device-to-device copy kernel (reference for HBM counters)")
    return ap.parse_args()


def cpu_baseline(inp, budget_s: float):
    """The oracle as it stands, forward + backward, on a strided ray subset sized to take
    about `budget_s` seconds on this machine's cores."""
    import lp_inputs
    import oracle
    rng = np.random.default_rng(5)

    def run(n):
        sub = inp.subset(lp_inputs.strided_ray_subset(inp.n_rays, n, offset=1))
        prob = oracle.Problem(sub)
        p = (rng.standard_normal((sub.n_rays, 3)) / sub.n_rays)
        t0 = time.perf_counter()
        oracle.render_fwd(prob)
        oracle.render_bwd(prob, p)      # recomputes the forward internally, then reverses it
        return time.perf_counter() - t0, sub.n_rays

    t_probe, n_probe = run(min(1024, inp.n_rays))
    n = int(max(n_probe, min(inp.n_rays, n_probe * budget_s / max(t_probe, 1e-3))))
    t, n = run(n)
    return {"value": n * inp.samples / t, "unit": "ray-samples/s", "cores": oracle.num_threads(),
            "kind": "oracle", "sample": f"{n} of {inp.n_rays} rays (every {max(1, inp.n_rays // n)}th), "
            f"all {inp.samples} samples each, fp64 forward + stored-forward reverse-mode backward, {t:.1f} s"}


def measure(lp, torch, name, mode, steps, warmup, calibrate_copy=False, grid_dtype="f32", aabb=None,
            measure_memory=False):
    """Times `steps` forward+backward steps of workload `name`; returns the result fields."""
    import lp_inputs
    w = lp_inputs.WORKLOADS[name]
    inp = lp_inputs.make_inputs(name, aabb=aabb)
    dev = "cuda:0"
    grid, mlp, rays, bg = lp.to_device(inp, dev)
    if grid_dtype != "f32":
        grid.data = [t.to(torch.bfloat16 if grid_dtype == "bf16" else torch.float16) for t in grid.data]
    target = torch.from_numpy(inp.target).to(dev)
    dec = lp.decoder_to_device(inp.decoder, dev) if inp.decoder is not None else None
    if dec is None:
        fast = lp.lp_has_fast_path(grid, mlp) and mode != lp.LP_MATH_GENERIC
    else:
        fast = lp.lp_dec_has_fast_path(grid, dec) and mode != lp.LP_MATH_GENERIC

    m = rays.n_rays
    rgb = torch.empty((m, 3), device=dev); alpha = torch.empty(m, device=dev)
    depth = torch.empty(m, device=dev); cache = torch.empty(m, device=dev)
    d_grid = [torch.zeros_like(t, dtype=torch.float32) for t in grid.data]
    if dec is None:
        params = [mlp.weights, mlp.biases]
        ws = torch.empty(lp.lp_bwd_workspace_bytes(grid, mlp, rays, mode), dtype=torch.uint8, device=dev)
    else:
        params = [dec.opacity.weights, dec.opacity.biases, dec.feature.weights, dec.feature.biases]
        ws = torch.empty(lp.lp_dec_workspace_bytes(grid, dec, rays, mode)[1], dtype=torch.uint8, device=dev)
    grads = [[torch.zeros_like(t) for t in lst] for lst in params]
    if inp.scene is None:
        inv = torch.full((m, 1), 2.0 / (3.0 * m), device=dev)
    else:
        counts = torch.bincount(rays.scene.long(), minlength=inp.n_scenes).float()
        inv = (2.0 / (3.0 * counts[rays.scene.long()]))[:, None]

    ev = lambda: torch.cuda.Event(enable_timing=True)

    def step(timed: bool):
        # events on torch's current stream, which is the stream the library launches on
        e0, e1, e2, e3 = ev(), ev(), ev(), ev()
        e0.record()
        if dec is None:
            lp.lp_render_fwd(grid, mlp, rays, bg, rgb, alpha, depth, cache, mode)
        else:
            lp.lp_render_dec_fwd(grid, dec, rays, bg, rgb, alpha, depth, cache, ws, mode)
        e1.record()
        d_rgb = (rgb - target) * inv                      # MSE loss gradient
        for t in d_grid + [t for lst in grads for t in lst]:
            t.zero_()
        e2.record()
        if dec is None:
            lp.lp_render_bwd(grid, mlp, rays, bg, d_rgb, None, None, cache, d_grid, grads[0], grads[1], ws, mode)
        else:
            lp.lp_render_dec_bwd(grid, dec, rays, bg, d_rgb, None, None, cache, d_grid, *grads, ws, mode)
        e3.record()
        return (e0, e1, e2, e3) if timed else None

    if calibrate_copy:
        # a copy kernel of known traffic (1 GiB read + 1 GiB written) for scaling the
        # FETCH_SIZE / WRITE_SIZE counters of a profiler run of this same command
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    for _ in range(warmup):
        step(False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    events = [step(True) for _ in range(steps)]
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    fwd_ms = float(np.mean([e0.elapsed_time(e1) for e0, e1, _, _ in events]))
    bwd_ms = float(np.mean([e2.elapsed_time(e3) for _, _, e2, e3 in events]))
    mid_ms = float(np.mean([e1.elapsed_time(e2) for _, e1, e2, _ in events]))   # loss gradient + zeroing
    memory = None
    if measure_memory and dec is None:
        # Device memory a forward + backward needs beyond its inputs and the gradient buffers:
        # outputs (20 B per ray), the cached scalar (4 B per ray), the upstream gradient and the
        # workspace; measured as the allocator's peak over one step, at S and at 4 S samples.
        import dataclasses
        memory = {"state_kept_for_backward_bytes_per_ray": 4}
        for mult in (1, 4):
            r2 = dataclasses.replace(rays, samples=inp.samples * mult)
            torch.cuda.synchronize()
            torch.cuda.reset_peak_memory_stats()
            base = torch.cuda.memory_allocated()
            o = [torch.empty((m, 3), device=dev), torch.empty(m, device=dev), torch.empty(m, device=dev),
                 torch.empty(m, device=dev)]
            w2 = torch.empty(lp.lp_bwd_workspace_bytes(grid, mlp, r2, mode), dtype=torch.uint8, device=dev)
            lp.lp_render_fwd(grid, mlp, r2, bg, o[0], o[1], o[2], o[3], mode)
            g2 = (o[0] - target) * inv
            lp.lp_render_bwd(grid, mlp, r2, bg, g2, None, None, o[3], d_grid, grads[0], grads[1], w2, mode)
            torch.cuda.synchronize()
            memory["peak_extra_bytes_at_%dS" % mult] = int(torch.cuda.max_memory_allocated() - base)
            memory["workspace_bytes_at_%dS" % mult] = int(w2.numel())
            del o, w2, g2
    return dict(w=w, inp=inp, fast=fast, rays=m, samples=m * inp.samples, elapsed=elapsed,
                fwd_ms=fwd_ms, bwd_ms=bwd_ms, mid_ms=mid_ms, memory=memory)


def measure_splat(lp, torch, name, steps, warmup):
    """Times the Splatter (forward: push + normalise; backward for a random output gradient)."""
    import lp_inputs
    w = lp_inputs.SPLAT_WORKLOADS[name]
    sp = lp_inputs.make_splat_inputs(name)
    target, rays, splat = lp.splat_to_device(sp)
    theta, theta_w = lp.splat_fwd(target, rays, splat)
    g = [torch.randn_like(t) for t in theta]
    d_feats = torch.empty_like(splat.feats)
    d_prior = [] if splat.prior is None else [torch.zeros_like(t) for t in splat.prior.data]
    dW = [] if splat.mlp is None else [torch.zeros_like(t) for t in splat.mlp.weights]
    db = [] if splat.mlp is None else [torch.zeros_like(t) for t in splat.mlp.biases]
    ws = torch.empty(lp.lp_splat_bwd_workspace_bytes(target, rays, splat), dtype=torch.uint8, device="cuda:0")
    ev = lambda: torch.cuda.Event(enable_timing=True)
    times = []
    for it in range(warmup + steps):
        e0, e1, e2 = ev(), ev(), ev()
        e0.record()
        lp.lp_splat_fwd(target, rays, splat, theta, theta_w)
        e1.record()
        for t in d_prior + dW + db:
            t.zero_()
        lp.lp_splat_bwd(target, rays, splat, theta_w, g, d_feats, d_prior, dW, db, ws)
        e2.record()
        torch.cuda.synchronize()
        if it >= warmup:
            times.append((e0.elapsed_time(e1), e1.elapsed_time(e2)))
    fwd_ms, bwd_ms = [float(np.mean(x)) for x in zip(*times)]
    pts = w.ray_samples
    return {"workload": name, "points": pts, "value": pts / ((fwd_ms + bwd_ms) * 1e-3), "unit": "points/s fwd+bwd",
            "fwd_ms": fwd_ms, "bwd_ms": bwd_ms, "mlp": w.hidden is not None,
            "fwd_push_GBs": w.push_bytes_per_sample * pts / (fwd_ms * 1e-3) / 1e9}


def main():
    args = parse()
    if args.gpus != 1:
        print(f"bench.py: this build runs on ONE GPU (no collectives, no sharding); --gpus {args.gpus} "
              "is not supported", file=sys.stderr)
        sys.exit(2)
    import torch
    import paper_2404_19760_amd as lp

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the Renderer has no CPU path", file=sys.stderr)
        sys.exit(2)
    if args.coexecution:
        ns = lp.lp_diag_coexecution()
        print(json.dumps({
            "measurement": "overlap of 32x32x16 bf16 matrix products (32 cycles) with vector multiply-adds (4 cycles) on one SIMD",
            "one_wave_ns_per_product_followed_by_K_multiply_adds": {"K=0": ns[0], "K=4": ns[1], "K=8": ns[2], "K=12": ns[3]},
            "two_waves_w_and_w_plus_4_ns_per_iteration": {"8 products only": ns[4], "64 multiply-adds only": ns[5], "both": ns[6]},
            "two_waves_w_and_w_plus_1_ns_per_iteration": {"8 products only": ns[7], "64 multiply-adds only": ns[8], "both": ns[9]}}))
        return
    if args.atomic_rate:
        r = lp.lp_diag_atomic_rate()
        print(json.dumps({
            "measurement": "64-byte lines of fp32 atomic adds retired per second (2048 workgroups of 4 waves, 16 lanes per line)",
            "random_lines_in_256MiB": {"4 lines per instruction": r[0], "2 lines per instruction": r[1], "1 line per instruction": r[2]},
            "random_lines_in_256KiB_4_per_instruction": r[3],
            "neighbouring_lines_4_per_instruction": {"256MiB": r[4], "256KiB": r[5]}}))
        return
    mode = {"default": lp.LP_MATH_DEFAULT, "generic": lp.LP_MATH_GENERIC, "bf16x3": lp.LP_MATH_BF16X3}[args.math]
    r = measure(lp, torch, args.config, mode, args.steps, args.warmup, args.calibrate_copy, args.grid_dtype, args.aabb,
                measure_memory=not args.calibrate_copy)
    w, inp, fast, m, samples = r["w"], r["inp"], r["fast"], r["rays"], r["samples"]
    elapsed, fwd_avg, bwd_avg = r["elapsed"], r["fwd_ms"], r["bwd_ms"]

    ms_per_step = 1e3 * elapsed / args.steps
    g_write = w.gather_bytes_per_sample                                   # fp32 gradient bytes per sample
    g_bytes = g_write if args.grid_dtype == "f32" else g_write // 2       # bytes a sample reads from the grid
    # dominant kernel: the backward (re-reads the gather bytes and adds the fp32 gradient bytes)
    bwd_gbs = (g_bytes + g_write) * samples / (bwd_avg * 1e-3) / 1e9
    fwd_gbs = g_bytes * samples / (fwd_avg * 1e-3) / 1e9
    # arithmetic view: MLP FLOPs per sample F (forward), 4 F forward + backward (recompute, dX, dW),
    # plus the interpolation (2 FLOP per corner and channel, again in the backward's recompute and scatter)
    interp = 2 * w.corners * w.channels
    f_fwd, f_all = w.mlp_flop_per_sample + interp, 4 * w.mlp_flop_per_sample + 3 * interp
    step_s = elapsed / args.steps
    bwd_flop = (9 if fast else 3) * w.mlp_flop_per_sample
    bwd_tflops = bwd_flop * samples / (bwd_avg * 1e-3) / 1e12
    traffic = MEASURED_BWD_HBM_BYTES.get(args.config) if fast and args.grid_dtype == "f32" and args.aabb is None else None
    lines = MEASURED_BWD_ATOMIC_LINES.get(args.config) if fast and args.grid_dtype == "f32" and args.aabb is None else None
    atomic_peak = lp.lp_diag_atomic_rate()[0]     # measured now, on this GPU
    out = {
        "metric": "ray-samples/sec fwd+bwd (Renderer hot path)",
        "value": samples / (elapsed / args.steps),
        "unit": "ray-samples/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32 (MLP contractions: bf16 hi+lo split, 3 MFMA products, f32 accumulate)" if fast else "f32",
        "data": "synthetic",
        "config": {"workload": f"{args.config}: {'voxel' if w.kind == 0 else 'triplane'} "
                               f"{w.n_scenes}x{w.res[0]}^{3 if w.kind == 0 else 2}x{w.channels}ch, "
                               f"{m} rays x {w.samples} samples, MLP {'-'.join(map(str, w.mlp_dims))}",
                   "rays": m, "samples_per_ray": w.samples, "ray_samples": samples, "grid_dtype": args.grid_dtype,
                   "aabb_half_width": inp.aabb_max[0],
                   "kernels": "mfma" if fast else "generic"},
        "fwd": {"ms": fwd_avg, "ray_samples_per_s": samples / (fwd_avg * 1e-3),
                "mfma_bf16_TFLOPs": (3 if fast else 1) * w.mlp_flop_per_sample * samples / (fwd_avg * 1e-3) / 1e12,
                "frac_mfma_bf16_peak": ((3 * w.mlp_flop_per_sample * samples / (fwd_avg * 1e-3) / 1e12
                                         / MFMA_BF16_PEAK_TFLOPS) if fast else None),
                "hbm_effective_GBs": fwd_gbs, "hbm_effective_frac": fwd_gbs / HBM_PEAK_GBS},
        "fwd_bwd_hbm_effective": {"GBs": (2 * g_bytes + g_write) * samples / ((fwd_avg + bwd_avg) * 1e-3) / 1e9,
                                  "frac": (2 * g_bytes + g_write) * samples / ((fwd_avg + bwd_avg) * 1e-3) / 1e9
                                  / HBM_PEAK_GBS},
        "loss_grad_and_zeroing_ms": r["mid_ms"],
        "memory": r["memory"],
        "fp32_equivalent": {"flop_per_sample_fwd": f_fwd, "flop_per_sample_fwd_bwd": f_all,
                            "fwd_TFLOPs": f_fwd * samples / (fwd_avg * 1e-3) / 1e12,
                            "fwd_bwd_TFLOPs": f_all * samples / step_s / 1e12,
                            "note": "algorithmic fp32 FLOPs of MLP + interpolation; for comparison with plain fp32 "
                                    "vector code (peak 157.3 TFLOP/s), not a roofline of this kernel"},
        "roofline": {"kernel": "lp_render_bwd", "bound": "mfma" if fast else "alu",
                     "achieved": bwd_tflops, "peak": MFMA_BF16_PEAK_TFLOPS if fast else 157.3,
                     "unit": "TFLOP/s", "frac": bwd_tflops / (MFMA_BF16_PEAK_TFLOPS if fast else 157.3),
                     "traffic": traffic, "ms": bwd_avg,
                     "flop_per_sample": bwd_flop,
                     "flop_counting": ("3 bf16 products per fp32 multiply-add x 3 F (recompute, dX, dW), F = MLP forward FLOPs"
                                       if fast else "3 F fp32 (recompute, dX, dW), F = MLP forward FLOPs"),
                     "hbm_effective": {"bound": "hbm-effective (no-reuse algorithmic bytes, served mostly from caches)",
                                       "achieved": bwd_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                       "frac": bwd_gbs / HBM_PEAK_GBS, "bytes_per_sample": g_bytes + g_write},
                     "hbm_counters": None if traffic is None else
                     {"bound": "hbm (FETCH_SIZE + WRITE_SIZE per launch, profiles/)",
                      "achieved": traffic / (bwd_avg * 1e-3) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                      "frac": traffic / (bwd_avg * 1e-3) / 1e9 / HBM_PEAK_GBS},
                     "atomic_lines": None if lines is None else
                     {"bound": "atomic adds of whole 64-byte lines (lines per launch from the counters in profiles/; "
                               "peak measured in this run by lp_diag_atomic_rate, random lines in 256 MiB)",
                      "achieved": lines / (bwd_avg * 1e-3), "peak": atomic_peak, "unit": "lines/s",
                      "frac": lines / (bwd_avg * 1e-3) / atomic_peak}},
    }
    # further workloads for context (short runs), e.g. the single-scene configuration and the
    # paper's experimental Renderer shape with contract coordinates
    del r
    import gc
    gc.collect()   # the main workload's host buffers go back before the short context runs are timed
    for entry in [n for n in args.also.split(",") if n and n != args.config]:
        torch.cuda.empty_cache()
        name, _, gdt = entry.partition(":")
        if name in __import__("lp_inputs").SPLAT_WORKLOADS:
            out.setdefault("also", []).append(measure_splat(lp, torch, name, max(3, args.steps // 2), 2))
            continue
        k = max(3, args.steps // 2)
        o = measure(lp, torch, name, mode, k, 5, grid_dtype=gdt or "f32")
        ow = o["w"]
        gw = ow.gather_bytes_per_sample
        gr = gw if not gdt else gw // 2
        nine_f = (9 if o["fast"] else 3) * ow.mlp_flop_per_sample
        out.setdefault("also", []).append(
            {"workload": entry, "ray_samples": o["samples"], "value": o["samples"] / (o["elapsed"] / k),
             "unit": "ray-samples/s", "fwd_ms": o["fwd_ms"], "bwd_ms": o["bwd_ms"], "grid_dtype": gdt or "f32",
             "contract_a": ow.contract_a, "two_mlp_decoder": ow.dec_hidden is not None, "kernels": "mfma" if o["fast"] else "generic",
             "bwd_mfma_bf16_frac": (nine_f * o["samples"] / (o["bwd_ms"] * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS
                                    if o["fast"] and ow.dec_hidden is None else None),
             "fwd_bwd_hbm_effective_frac": (2 * gr + gw) * o["samples"]
             / ((o["fwd_ms"] + o["bwd_ms"]) * 1e-3) / 1e9 / HBM_PEAK_GBS,
             "bwd_atomic_lines_frac": (MEASURED_BWD_ATOMIC_LINES[name] / (o["bwd_ms"] * 1e-3) / atomic_peak
                                       if name in MEASURED_BWD_ATOMIC_LINES and o["fast"] and not gdt else None)})
        del o
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(inp, args.cpu_seconds)
    print(json.dumps(out))
    if args.ws_phases:
        try:
            cyc = lp.lp_diag_ws_phases()
        except lp.LightplaneError:
            print("bench.py: --ws-phases needs a measurement build: LP_EXTRA_HIPCC_FLAGS=-DLP_WS_PHASES python "
                  "paper_2404_19760_amd/build.py", file=sys.stderr)
            sys.exit(2)
        chain = ["step start", "sampling issue", "forward", "hand-over h1 h2", "Eq. (2)", "hand-over output gradients",
                 "chain link 1 (dZ2)", "hand-over dZ2", "chain link 2 (dZ1)", "hand-over features, records, dZ1",
                 "interpolation of the next features"]
        weights = ["step start", "h2 taken + transposed", "wait for output gradients", "dWo", "h1 transposed", "wait for dZ2",
                   "dW2", "features taken + transposed", "wait for dZ1", "feature gradient + dW1", "walk"]
        def shares(names, vals):
            tot = max(sum(vals), 1)
            return {n: round(c / tot, 4) for n, c in zip(names, vals)}
        print(json.dumps({"two_wave_backward_phase_shares": {"chain_wave": shares(chain, cyc[:11]),
                                                              "weights_wave": shares(weights, cyc[16:27])},
                          "note": "shares of the cycles between marks, summed over all waves and all launches of this "
                                  "run; waits for the partner are inside the hand-over / wait phases"}))



if __name__ == "__main__":
    main()
