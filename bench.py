#!/usr/bin/env python3
"""Benchmark of the cache-aware CNN inference path on one MI355X.

Workload (default): 64 independent 224x224 video streams, one batch per time step, through the VGG-16-style stack
in bf16 (fp32 accumulation).  A step is one frame of every stream through the whole hot path: block matching against
the previous frame, merge + region propagation, and the stack in which every convolution copies its reusable pixels
from the previous frame's cached output and computes only the rest.  Frames are resident in HBM before the timed
region starts.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--dtype f32|bf16] [--streams n] [--repeats r]

Prints one JSON line: whole-job frames/s with the cache (`value`, the median over `repeats` timed regions of K steps)
and without it (`no_cache`, same number of steps), the roofline of the dominant convolution kernel measured with HIP
events during the run, the shifted copy against the HBM peak, the matching, the single-stream fp32 configuration as a
sub-record, and the CPU oracle timed on a bounded sample of the same video.

    python bench.py --traffic-calib     a plain 256 MiB device copy and nothing else (run under rocprofv3 --pmc
                                        FETCH_SIZE / WRITE_SIZE: gives the bytes per counter unit)
"""
from __future__ import annotations

import argparse
import json
import os
import re
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_TFLOPS = {"f32": 157.3, "bf16": 2500.0}     # MI355X dense matrix peaks
PEAK_INT8_TOPS = 5000.0
PEAK_HBM_GBS = 8000.0
TARGET_CONV_FRAC = 0.5                           # the bar asked of the bf16 convolutions
TARGET_COPY_FRAC = 0.6


def read_traffic_table(streams, dtype):
    """HBM traffic per launch of the conv kernels from the rocprofv3 --pmc summary of this workload under
    profiles/ (lines `traffic | kernel | FETCH_SIZE avg | WRITE_SIZE avg`, and a `calibration` line with the KiB of
    HBM traffic per counter unit measured with `--traffic-calib`).  Returns (table, scale) or (None, None)."""
    path = os.path.join(ROOT, "profiles", f"vgg16_224_{dtype}_{streams}streams_hbm_traffic.txt")
    if not os.path.exists(path):
        return None, None
    table, scale = {}, None
    with open(path) as fh:
        for line in fh:
            parts = [p.strip() for p in line.split("|")]
            if parts[0] == "traffic" and len(parts) >= 4:
                table[parts[1]] = (float(parts[2]), float(parts[3]))
            elif parts[0] == "calibration" and len(parts) >= 3:
                scale = (float(parts[1]), float(parts[2]))
    return (table, scale) if table and scale else (None, None)


def traffic_calib():
    import torch
    dev = torch.device("cuda:0")
    n = 256 << 20
    src = torch.empty(n, dtype=torch.uint8, device=dev).random_(0, 255)
    dst = torch.empty_like(src)
    for _ in range(5):
        dst.copy_(src)
    torch.cuda.synchronize()
    print(json.dumps({"traffic_calib": "device copy", "bytes_read": n, "bytes_written": n, "launches": 5}))


def run_workload(args, n, dtype, steps, warmup, repeats, detail, cpu_frames, exact_masks=None, torus=None, pool_cache=None,
                 k_skip=None):
    import numpy as np
    import torch
    from paper_1712_01670_amd import binding, synth

    dev = torch.device("cuda:0")
    H = W = 224
    n_frames = 30
    layers = synth.vgg16()
    ws, bs = synth.he_weights(layers, 1)
    seed0 = 2000 if n == 1 else 5000           # configs[1] names one video, configs[4] per-stream seeds
    videos = np.stack([synth.panning_video(seed0 + s, n_frames=n_frames, H=H, W=W) for s in range(n)])  # [n][T][H][W][3]
    dev_video = torch.from_numpy(np.ascontiguousarray(videos.transpose(1, 0, 2, 3, 4))).to(dev)
    dt = binding.DC_BF16 if dtype == "bf16" else binding.DC_F32
    method = binding.DC_MATCH_DIAMOND if args.matcher == "ds" else binding.DC_MATCH_EXHAUSTIVE
    exact = (args.regions == "exact" if exact_masks is None else exact_masks) and not args.host_plan
    torus = args.torus if torus is None else torus

    def make_runner(on_torus):
        return binding.StackRunner(layers, ws, bs, n, H, W, 3, block=16, radius=16, dtype=dt, expiry=args.expiry,
                                   match_method=method, k_skip=args.k_skip if k_skip is None else k_skip,
                                   device_plan=not args.host_plan,
                                   exact_masks=exact,
                                   cache_pool_add=exact and (args.cache_pool_add if pool_cache is None else pool_cache),
                                   no_reuse=synth.no_reuse_flags(layers, args.min_reuse_macs) if args.min_reuse_macs > 0 else None,
                                   torus=on_torus)
    runner = make_runner(torus)

    def run_steps(k, start, collect=None, force_full=False, runner=runner):
        """Run k steps through the cyclic video starting at global step `start`."""
        for i in range(start, start + k):
            f = i % n_frames
            if f == 0:
                runner.reset()          # the video wraps: a scene cut
            nxt = (i + 1) % n_frames
            runner.step(dev_video[f], force_full=force_full,
                        next_frames=dev_video[nxt] if (args.lookahead and nxt != 0 and not force_full) else None)
            if collect is not None:
                collect(i, f)

    # ---- warm-up, then the timed region (K steps, `repeats` times; the median counts) ----
    run_steps(warmup, 0)
    torch.cuda.synchronize()
    times = []
    pos = warmup
    for _ in range(repeats):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        run_steps(steps, pos)
        torch.cuda.synchronize()
        times.append(time.perf_counter() - t0)
        pos += steps
    elapsed = statistics.median(times)
    fps = steps * n / elapsed

    # ---- every frame in full (no cache): same number of steps, same repeats ----
    # A stack that computes every frame in full has no reason to keep one buffer per tensor: it alternates two, so
    # that a layer of the next frame only waits for the same layer of this one.  The baseline gets that arrangement.
    full_runner = make_runner(False) if torus else runner
    run_steps(min(warmup, 5), 0, force_full=True, runner=full_runner)
    times_full = []
    for _ in range(repeats):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        run_steps(steps, 0, force_full=True, runner=full_runner)
        torch.cuda.synchronize()
        times_full.append(time.perf_counter() - t0)
    fps_full = steps * n / statistics.median(times_full)
    if full_runner is not runner:
        del full_runner

    out = {"value": fps, "ms_per_step": elapsed / steps * 1e3, "repeat_ms_per_step": [t / steps * 1e3 for t in times],
           "no_cache": {"value": fps_full, "unit": "frames/s", "steps": steps, "repeats": repeats,
                        "saving": 1.0 - fps_full / fps}}
    if not detail:
        del runner
        return out

    # ---- same steps again, one at a time, with HIP-event brackets around every conv GEMM / copy launch ----
    runner.enable_profile(True)
    shapes = runner.shapes
    per_kernel = {}      # kernel name -> [flops_alg, ms, launches, flops_issued]
    copy = dict(ms=0.0, bytes=0.0, launches=0)
    agg = dict(reuse=[], macs_full=0, macs_needed=0, macs_issued=0, cached_frames=0, full_frames=0, layer_reuse={})

    def collect(i, f):
        torch.cuda.synchronize()
        st = runner.read_stats()
        ls = runner.layer_stats()
        agg["macs_full"] += st.macs_full
        agg["macs_needed"] += st.macs_needed
        agg["macs_issued"] += st.macs_issued
        if st.full:
            agg["full_frames"] += 1
        else:
            agg["cached_frames"] += 1
            agg["reuse"].append(st.n_reusable_blocks / st.n_blocks)
            for li, L in enumerate(layers):          # reusable output pixels per conv layer on the cached frames
                if L["type"] == synth.CONV:
                    ho, wo, _ = shapes[li + 1]
                    rec = agg["layer_reuse"].setdefault(li, [0, 0])
                    rec[0] += ls["reused_px"][li]
                    rec[1] += n * ho * wo
        for li, (g_ms, c_ms) in runner.profile_ms().items():
            L = layers[li]
            ho, wo, co = shapes[li + 1]
            kh, kw = synth.conv_geometry(L)[:2]
            mac_px = kh * kw * L["cin"] * L["cout"]
            reused = 0 if st.full else ls["reused_px"][li]
            if g_ms is not None:
                name = binding.conv_kernel_name(ls["kernel_id"][li])
                rec = per_kernel.setdefault(name, [0.0, 0.0, 0, 0.0])
                rec[0] += 2.0 * (n * ho * wo - reused) * mac_px
                rec[1] += g_ms
                rec[2] += 1
                rec[3] += 2.0 * ls["issued_macs"][li]
            if c_ms is not None:
                copy["ms"] += c_ms
                copy["launches"] += 1
        copy["bytes"] += st.copy_bytes

    k_prof = min(steps, 60)
    run_steps(k_prof, 0, collect)
    runner.enable_profile(False)

    dname, (dflops, dms, dlaunch, dissued) = max(per_kernel.items(), key=lambda kv: kv[1][1])
    all_flops = sum(v[0] for v in per_kernel.values())
    all_ms = sum(v[1] for v in per_kernel.values())
    peak = PEAK_TFLOPS[dtype]
    table, scale = read_traffic_table(n, dtype)
    traffic = None
    if table and dname in table:
        traffic = (table[dname][0] * scale[0] + table[dname][1] * scale[1]) * 1024.0
    roofline = {
        "bound": "mfma", "kernel": dname,
        "achieved": dflops / (dms * 1e-3) / 1e12, "peak": peak, "unit": "TFLOP/s",
        "frac": dflops / (dms * 1e-3) / 1e12 / peak, "target_frac": TARGET_CONV_FRAC if dtype == "bf16" else None,
        "avg_launch_us": dms / dlaunch * 1e3, "launches": dlaunch,
        "issued_tflops": dissued / (dms * 1e-3) / 1e12,
        "traffic": traffic,
        "traffic_note": "HBM bytes per launch from the rocprofv3 FETCH_SIZE / WRITE_SIZE summary under profiles/ "
                        "(calibrated against a plain copy; a constant of that profile run, not measured in this run)",
        "all_conv": {"achieved": all_flops / (all_ms * 1e-3) / 1e12, "frac": all_flops / (all_ms * 1e-3) / 1e12 / peak,
                     "ms_per_step": all_ms / k_prof},
        "per_kernel": {k: {"frac": v[0] / (v[1] * 1e-3) / 1e12 / peak, "avg_launch_us": v[1] / v[2] * 1e3, "launches": v[2]}
                       for k, v in sorted(per_kernel.items(), key=lambda kv: -kv[1][1])},
        "copy": {"bound": "hbm", "achieved": (copy["bytes"] / (copy["ms"] * 1e-3) / 1e9) if copy["ms"] else None,
                 "peak": PEAK_HBM_GBS, "unit": "GB/s", "target_frac": TARGET_COPY_FRAC,
                 "frac": (copy["bytes"] / (copy["ms"] * 1e-3) / 1e9 / PEAK_HBM_GBS) if copy["ms"] else None,
                 "avg_launch_us": (copy["ms"] / copy["launches"] * 1e3) if copy["launches"] else None},
    }
    if not copy["launches"]:
        roofline["copy"]["note"] = ("nothing is copied: every conv output stays in one buffer and its origin moves "
                                    "(see shifted_copies for the same workload with the copies)")

    if dtype == "bf16":     # what the matrix cores sustain on this GPU under its power limit, measured now
        regs, lds = binding.dc_probe_mfma_rate(0), binding.dc_probe_mfma_rate(1)
        roofline["sustained_mfma"] = {
            "registers_only": regs, "with_lds_reads": lds, "unit": "TFLOP/s",
            "frac_of_with_lds_reads": roofline["achieved"] / lds,
            "note": "v_mfma_f32_16x16x32_bf16, 4x4 tiles per wavefront, 8 wavefronts on every CU, 30 launches of 0.3 ms back to "
                    "back, the last one timed: operands in registers, and re-read from LDS every step as the conv kernels do"}

    # ---- the matching alone (Steps 1-4), HIP events on the launch stream; allocations are outside the events ----
    torch.cuda.synchronize()
    mbs = synth.max_block_ssd(16, 3)
    for f in range(1, 4):
        binding.dc_match_blocks_opt(dev_video[f], dev_video[f - 1], 16, 16, mbs, method, args.k_skip)
    torch.cuda.synchronize()
    match_ms = 0.0
    k_match = n_frames - 1
    for f in range(1, n_frames):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.empty(1, device=dev)      # nothing pending on the stream when the first event is recorded
        e0.record()
        binding.dc_match_blocks_opt(dev_video[f], dev_video[f - 1], 16, 16, mbs, method, args.k_skip)
        e1.record()
        torch.cuda.synchronize()
        match_ms += e0.elapsed_time(e1)
    match_us = match_ms / k_match * 1e3
    match_bytes = 2.0 * n * H * W * 3 + n * (H // 16) * (W // 16) * 13.0      # both frames once; mv, ssd, mask per block
    match_terms = float(n) * (H // 16) * (W // 16) * 16 * 16 * 3 * 33 * 33      # candidates inside the frame or not
    peak_terms = 256 * 64 * 2.4e9 * 4 / 1e12       # 256 CUs x 64 lanes x 2.4 GHz x 4 bytes per packed dot instruction
    rate = None if args.matcher == "ds" else match_terms / (match_us * 1e-6) / 1e12
    roofline["match"] = {
        "bound": "alu", "avg_launch_us": match_us,
        "achieved": rate, "peak": peak_terms, "unit": "T squared differences/s",
        "frac": None if rate is None else rate / peak_terms,
        "frac_of_int8_mfma_peak": None if rate is None else rate / (PEAK_INT8_TOPS / 2.0),
        "hbm_GBps": match_bytes / (match_us * 1e-6) / 1e9,
        "hbm_frac": match_bytes / (match_us * 1e-6) / 1e9 / PEAK_HBM_GBS,
        "note": "Steps 1-4 of the matching for all streams, alone on the GPU.  The search is bound by integer arithmetic "
                "and LDS traffic, not by HBM.  `peak` = packed 8-bit dot products on the vector ALUs; the kernel runs its "
                "cross terms on the int8 matrix cores, whose peak (5.0 POP/s = 2.5 P multiply-adds/s) gives "
                "frac_of_int8_mfma_peak (the diamond search evaluates a data-dependent number of candidates: no rate)"}

    # ---- oracle on the host cores, bounded sample of the same workload ----
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import oracle as oc
        ref = oc.Stream(layers, ws, bs, H, W, 3, block=16, radius=16, bf16=(dtype == "bf16"), expiry=args.expiry,
                        diamond=(args.matcher == "ds"), k_skip=args.k_skip, exact_masks=exact,
                        cache_pool_add=exact and args.cache_pool_add,
                        no_reuse=synth.no_reuse_flags(layers, args.min_reuse_macs) if args.min_reuse_macs > 0 else None)
        k_cpu = min(cpu_frames, n_frames)
        t0 = time.perf_counter()
        for f in range(k_cpu):
            ref.step(videos[0, f])
        cpu_s = time.perf_counter() - t0
        n_cpu_full = len(range(0, k_cpu, args.expiry)) if args.expiry > 0 else 1
        cpu = {"value": k_cpu / cpu_s, "unit": "frames/s", "cores": oc.num_threads(), "kind": "oracle",
               "sample": f"first {k_cpu} frames of stream 0 of the same videos ({n_cpu_full} full + {k_cpu - n_cpu_full} "
                         f"cached), {cpu_s:.1f} s; the other {n - 1} streams are the same work per frame"}

    steps_all = agg["cached_frames"] + agg["full_frames"]
    out.update({
        "config_detail": {"mean_block_reuse": float(np.mean(agg["reuse"])) if agg["reuse"] else 0.0,
                          "full_frame_fraction": agg["full_frames"] / max(steps_all, 1),
                          "mac_fraction_needed": agg["macs_needed"] / max(agg["macs_full"], 1),
                          "mac_fraction_issued": agg["macs_issued"] / max(agg["macs_full"], 1),
                          # rho_l: share of a conv layer's output pixels that are reused, cached frames only
                          "conv_layer_reuse": {str(li): round(r[0] / max(r[1], 1), 4) for li, r in sorted(agg["layer_reuse"].items())}},
        "effective_tflops": 2.0 * agg["macs_full"] / max(steps_all, 1) * steps / elapsed / 1e12,
        "roofline": roofline, "cpu_baseline": cpu})
    del runner
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=120)
    ap.add_argument("--warmup", type=int, default=30)
    ap.add_argument("--repeats", type=int, default=5, help="timed regions of K steps; the median is reported")
    ap.add_argument("--dtype", choices=["f32", "bf16"], default="bf16")
    ap.add_argument("--streams", type=int, default=64)
    ap.add_argument("--expiry", type=int, default=10, help="full recompute every N frames (Section 5 default 10)")
    ap.add_argument("--matcher", choices=["es", "ds"], default="es",
                    help="Step 2 of the matching: exhaustive search, or the diamond search of Section 4")
    ap.add_argument("--k-skip", type=int, default=1, help="search every k-th block row and column only (Section 4)")
    ap.add_argument("--lookahead", action="store_true",
                    help="start the matching of the next frame at the end of a step (dc_prefetch_match), as a decoder "
                         "one frame ahead would allow")
    ap.add_argument("--host-plan", action="store_true",
                    help="merge / propagate / list the dirty units on the host (one wait per frame) instead of on the GPU")
    ap.add_argument("--regions", choices=["exact", "rect"], default="exact",
                    help="what is reused: the pixels of the exact reuse maps (Table 2's rule per pixel, planned on the GPU), or "
                         "the rectangles of Step 5 propagated by Table 2 as the paper prints it")
    ap.add_argument("--cache-pool-add", action="store_true",
                    help="with exact maps: max-pooling layers take their outputs from the cache too (Section 5)")
    ap.add_argument("--copies", action="store_true",
                    help="reuse by shifted copies into a second buffer per tensor; the default keeps every conv "
                         "output in one buffer addressed from a moving origin (a torus), so that nothing is copied")
    ap.add_argument("--min-reuse-macs", type=int, default=0,
                    help="conv layers with fewer multiply-adds per output element (k*k*cin) are computed in full on every "
                         "frame instead of using the cache (0: every conv layer uses the cache, as in the paper)")
    ap.add_argument("--no-single", action="store_true", help="skip the single-stream fp32 sub-record")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-frames", type=int, default=30)
    ap.add_argument("--traffic-calib", action="store_true")
    args = ap.parse_args()
    args.torus = not args.copies and not args.host_plan
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (streams are independent and would shard "
              "across GPUs without communication); run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    torch.cuda.set_device(torch.device("cuda:0"))
    if args.traffic_calib:
        traffic_calib()
        return

    n = args.streams
    main_rec = run_workload(args, n, args.dtype, args.steps, args.warmup, args.repeats, True, args.cpu_frames)
    single = None
    if not args.no_single and not (n == 1 and args.dtype == "f32"):
        # configs[1]: the small configuration (one fp32 stream), frames/s and saving only
        single = run_workload(args, 1, "f32", 300, 30, args.repeats, False, 0)
        single["config"] = {"workload": "configs[1]: one 30-frame 224x224x3 synthetic panning video, VGG-16-style stack, fp32",
                            "streams": 1, "steps": 300}
    which = "configs[4]: 64 streams" if n == 64 else ("configs[1]: one stream" if n == 1 else f"{n} streams")
    detail = main_rec.pop("config_detail")
    out = {
        "metric": "frames/s cache-aware CNN at fixed reuse ratio + % of MFMA/HBM peak",
        "value": main_rec.pop("value"), "unit": "frames/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": main_rec.pop("ms_per_step"), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": args.dtype, "data": "synthetic",
        "config": {"workload": f"{which} x 30-frame 224x224x3 synthetic panning videos (per-stream seeds), one batch per "
                               "time step, VGG-16-style 13-conv stack, 16x16 blocks, search +/-16, tau=20",
                   "streams": n, "matcher": ("exhaustive search" if args.matcher == "es" else "diamond search") + f", k-skip {args.k_skip}",
                   "cache_expiry_frames": args.expiry, "frames_per_video": 30, "repeats": args.repeats,
                   "planning": "host" if args.host_plan else "device",
                   "reusable_regions": "exact maps (Table 2's rule per pixel)" if (args.regions == "exact" and not args.host_plan)
                                       else "rectangles (Table 2 as printed)",
                   "cached_layers": "conv, max-pooling, add" if (args.cache_pool_add and args.regions == "exact" and not args.host_plan)
                                    else "conv",
                   "min_reuse_macs": args.min_reuse_macs, "reuse_by": "moving origins (conv outputs on a torus, no copies)" if args.torus else "shifted copies",
                   "lookahead_frames": 1 if args.lookahead else 0, **detail},
    }
    out.update(main_rec)
    if single is not None:
        out["single_stream_f32"] = single
    if args.regions == "exact" and not args.host_plan and not args.no_single:
        # the paper's own form of the regions (rectangles) on the same workload: frames/s and saving only
        rect = run_workload(args, n, args.dtype, args.steps, args.warmup, args.repeats, False, 0, exact_masks=False)
        rect["config"] = {"reusable_regions": "rectangles (Table 2 as printed)", "streams": n, "steps": args.steps}
        out["rectangles"] = rect
    if args.torus and not args.no_single:
        # the same workload with reuse by shifted copies into a second buffer per tensor: frames/s and saving only
        cp = run_workload(args, n, args.dtype, args.steps, args.warmup, args.repeats, False, 0, torus=False)
        cp["config"] = {"reuse_by": "shifted copies", "streams": n, "steps": args.steps}
        out["shifted_copies"] = cp
    if args.torus and args.regions == "exact" and not args.cache_pool_add and not args.no_single:
        # the same workload with the max-pooling layers through the cache as well (their outputs on a torus of their
        # own): another reading of the method's values (Section 5: the cache extends to other layer types)
        pc = run_workload(args, n, args.dtype, args.steps, args.warmup, args.repeats, False, 0, pool_cache=True)
        pc["config"] = {"cached_layers": "conv, max-pooling", "streams": n, "steps": args.steps}
        out["poolings_cached"] = pc
    if args.k_skip == 1 and not args.no_single:
        # the same workload with Step 2 on every second block row and column only (Section 4's k-skip, k = 2)
        ks = run_workload(args, n, args.dtype, args.steps, args.warmup, args.repeats, False, 0, k_skip=2)
        ks["config"] = {"matcher": ("exhaustive search" if args.matcher == "es" else "diamond search") + ", k-skip 2",
                        "streams": n, "steps": args.steps}
        out["k_skip_2"] = ks
    print(json.dumps(out))


if __name__ == "__main__":
    main()
