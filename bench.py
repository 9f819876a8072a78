#!/usr/bin/env python3
"""Benchmark of the cache-aware CNN inference path on one MI355X.

A step is one frame of the synthetic 224x224 video through the whole hot path:
block matching against the previous frame, merge + region propagation, and the
VGG-16-style stack in which every convolution copies its reusable pixels from the
previous frame's cached output and computes only the rest.  Frames are resident in
HBM before the timed region starts.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--dtype f32|bf16] [--streams n]

Prints one JSON line: whole-job frames/s with the cache (`value`) and without it (`no_cache`), the roofline of
the dominant convolution kernel measured with HIP events during the run, and the CPU oracle timed on a bounded
sample of the same video.
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

PEAK_TFLOPS = {"f32": 157.3, "bf16": 2500.0}     # MI355X dense matrix peaks
PEAK_HBM_GBS = 8000.0

# HBM traffic per launch of the conv kernels on this workload, from two rocprofv3 --pmc runs of this file
# (profiles/vgg16_224_f32_hbm_traffic.txt): kernel -> (FETCH_SIZE, WRITE_SIZE) counter averages.  A plain
# 256 MiB device copy reads 131085 / 262144 on the same counters, hence the scale factors.
PMC_TRAFFIC = {
    "conv_fast_kernel<float, 3, 16, 1, 2, 4, 1>": (7625.5, 3142.0),
    "conv_fast_kernel<float, 3, 16, 2, 2, 4, 1>": (8938.4, 9088.0),
    "conv_fast_kernel<float, 3, 16, 3, 2, 4, 1>": (4191.0, 3664.1),
    "conv_fast_kernel<float, 3, 16, 4, 2, 4, 1>": (6366.4, 8362.7),
    "conv_fast_kernel<float, 3, 32, 1, 2, 4, 1>": (7245.5, 1986.0),
}
PMC_SCALE = (2.0, 1.0)      # KiB of HBM traffic per counter unit (fetch, write)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=300)
    ap.add_argument("--warmup", type=int, default=30)
    ap.add_argument("--dtype", choices=["f32", "bf16"], default="f32")
    ap.add_argument("--streams", type=int, default=1)
    ap.add_argument("--expiry", type=int, default=10, help="full recompute every N frames (Section 5 default 10)")
    ap.add_argument("--matcher", choices=["es", "ds"], default="es",
                    help="Step 2 of the matching: exhaustive search, or the diamond search of Section 4")
    ap.add_argument("--k-skip", type=int, default=1, help="search every k-th block row and column only (Section 4)")
    ap.add_argument("--lookahead", action="store_true",
                    help="start the matching of the next frame at the end of a step (dc_prefetch_match), as a decoder "
                         "one frame ahead would allow")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-frames", type=int, default=30)
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (streams are independent and would shard "
              "across GPUs without communication); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_1712_01670_amd import binding, synth

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    H = W = 224
    n_frames = 30
    n = args.streams
    layers = synth.vgg16()
    ws, bs = synth.he_weights(layers, 1)
    videos = np.stack([synth.panning_video(2000 + s, n_frames=n_frames, H=H, W=W) for s in range(n)])  # [n][T][H][W][3]
    dev_video = torch.from_numpy(np.ascontiguousarray(videos.transpose(1, 0, 2, 3, 4))).to(dev)
    dt = binding.DC_BF16 if args.dtype == "bf16" else binding.DC_F32
    runner = binding.StackRunner(layers, ws, bs, n, H, W, 3, block=16, radius=16, dtype=dt, expiry=args.expiry,
                                 match_method=binding.DC_MATCH_DIAMOND if args.matcher == "ds" else binding.DC_MATCH_EXHAUSTIVE,
                                 k_skip=args.k_skip)

    def run_steps(k, start, collect=None):
        """Run k steps through the cyclic video starting at global step `start`."""
        for i in range(start, start + k):
            f = i % n_frames
            if f == 0:
                runner.reset()          # the video wraps: a scene cut
            nxt = (i + 1) % n_frames
            runner.step(dev_video[f], next_frames=dev_video[nxt] if (args.lookahead and nxt != 0) else None)
            if collect is not None:
                collect(i, f)

    # ---- warm-up, then the timed region ----
    run_steps(args.warmup, 0)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run_steps(args.steps, args.warmup)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    fps = args.steps * n / elapsed

    # ---- same steps again with HIP-event brackets around every conv GEMM / copy launch ----
    runner.enable_profile(True)
    conv_ids = [i for i, L in enumerate(layers) if L["type"] == synth.CONV]
    shapes = runner.shapes
    per_kernel = {}      # kernel name -> [flops_alg, ms, launches, flops_issued]
    copy_ms = copy_bytes = 0.0
    copy_launches = 0
    agg = dict(reuse=[], macs_full=0, macs_needed=0, macs_issued=0, cached_frames=0, full_frames=0)

    def collect(i, f):
        torch.cuda.synchronize()
        st = runner.stats
        ls = runner.layer_stats()
        agg["macs_full"] += st.macs_full
        agg["macs_needed"] += st.macs_needed
        agg["macs_issued"] += st.macs_issued
        if st.full:
            agg["full_frames"] += 1
        else:
            agg["cached_frames"] += 1
            agg["reuse"].append(st.n_reusable_blocks / st.n_blocks)
        nonlocal copy_ms, copy_bytes, copy_launches
        for li, (g_ms, c_ms) in runner.profile_ms().items():
            L = layers[li]
            ho, wo, co = shapes[li + 1]
            mac_px = L["k"] * L["k"] * L["cin"] * L["cout"]
            reused = 0 if st.full else ls["reused_px"][li]
            if g_ms is not None:
                name = binding.conv_kernel_name(ls["kernel_id"][li])
                rec = per_kernel.setdefault(name, [0.0, 0.0, 0, 0.0])
                rec[0] += 2.0 * (n * ho * wo - reused) * mac_px
                rec[1] += g_ms
                rec[2] += 1
                rec[3] += 2.0 * ls["issued_macs"][li]
            if c_ms is not None:
                copy_ms += c_ms
                copy_launches += 1
        copy_bytes += st.copy_bytes

    run_steps(args.steps, args.warmup + args.steps, collect)
    runner.enable_profile(False)

    dom = max(per_kernel.items(), key=lambda kv: kv[1][1])
    dname, (dflops, dms, dlaunch, dissued) = dom
    all_flops = sum(v[0] for v in per_kernel.values())
    all_ms = sum(v[1] for v in per_kernel.values())
    peak = PEAK_TFLOPS[args.dtype]
    roofline = {
        "bound": "mfma", "kernel": dname,
        "achieved": dflops / (dms * 1e-3) / 1e12, "peak": peak, "unit": "TFLOP/s",
        "frac": dflops / (dms * 1e-3) / 1e12 / peak,
        "avg_launch_us": dms / dlaunch * 1e3, "launches": dlaunch,
        "issued_tflops": dissued / (dms * 1e-3) / 1e12,
        "traffic": (sum(c * f for c, f in zip(PMC_TRAFFIC[dname], PMC_SCALE)) * 1024.0
                    if (args.dtype == "f32" and n == 1 and dname in PMC_TRAFFIC) else None),
        "traffic_unit": "bytes of HBM traffic per launch (rocprofv3 FETCH_SIZE + WRITE_SIZE, calibrated)",
        "all_conv": {"achieved": all_flops / (all_ms * 1e-3) / 1e12, "frac": all_flops / (all_ms * 1e-3) / 1e12 / peak,
                     "ms_per_step": all_ms / args.steps},
        "copy": {"bound": "hbm", "achieved": (copy_bytes / (copy_ms * 1e-3) / 1e9) if copy_ms else None,
                 "peak": PEAK_HBM_GBS, "unit": "GB/s",
                 "frac": (copy_bytes / (copy_ms * 1e-3) / 1e9 / PEAK_HBM_GBS) if copy_ms else None,
                 "avg_launch_us": (copy_ms / copy_launches * 1e3) if copy_launches else None},
    }

    # ---- the matching alone (Steps 1-4), HIP events on the launch stream; allocations are outside the events ----
    torch.cuda.synchronize()
    method = binding.DC_MATCH_DIAMOND if args.matcher == "ds" else binding.DC_MATCH_EXHAUSTIVE
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
    roofline["match"] = {
        "bound": "alu", "avg_launch_us": match_us,
        "achieved": None if args.matcher == "ds" else match_terms / (match_us * 1e-6) / 1e12, "peak": peak_terms,
        "unit": "T squared differences/s",
        "frac": None if args.matcher == "ds" else match_terms / (match_us * 1e-6) / 1e12 / peak_terms,
        "hbm_GBps": match_bytes / (match_us * 1e-6) / 1e9,
        "hbm_frac": match_bytes / (match_us * 1e-6) / 1e9 / PEAK_HBM_GBS,
        "note": "Steps 1-4 of the matching for all streams, alone on the GPU; the search is bound by integer arithmetic "
                "and LDS traffic, not by HBM; peak = packed 8-bit dot products on the vector ALUs (the diamond "
                "search evaluates a data-dependent number of candidates: no fixed term count)"}

    # ---- frames computed in full every time (no cache) for the saving ----
    torch.cuda.synchronize()
    k_full = max(10, args.steps // 5)
    t0 = time.perf_counter()
    for i in range(k_full):
        runner.step(dev_video[i % n_frames], force_full=True)
    torch.cuda.synchronize()
    fps_full = k_full * n / (time.perf_counter() - t0)

    # ---- oracle on the host cores, bounded sample of the same workload ----
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import oracle as oc
        ref = oc.Stream(layers, ws, bs, H, W, 3, block=16, radius=16, bf16=(args.dtype == "bf16"), expiry=args.expiry,
                        diamond=(args.matcher == "ds"), k_skip=args.k_skip)
        k_cpu = min(args.cpu_frames, n_frames)
        t0 = time.perf_counter()
        for f in range(k_cpu):
            ref.step(videos[0, f])
        cpu_s = time.perf_counter() - t0
        n_cpu_full = len(range(0, k_cpu, args.expiry)) if args.expiry > 0 else 1
        cpu = {"value": k_cpu / cpu_s, "unit": "frames/s", "cores": oc.num_threads(), "kind": "oracle",
               "sample": f"first {k_cpu} frames of stream 0 of the same video ({n_cpu_full} full + {k_cpu - n_cpu_full} cached), "
                         f"{cpu_s:.1f} s"}

    steps_all = agg["cached_frames"] + agg["full_frames"]
    out = {
        "metric": "frames/s cache-aware CNN at fixed reuse ratio + % of MFMA/HBM peak",
        "value": fps, "unit": "frames/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": elapsed / args.steps * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": args.dtype, "data": "synthetic",
        "config": {"workload": "configs[1]: 30-frame 224x224x3 synthetic panning video, VGG-16-style 13-conv stack, "
                               "16x16 blocks, search +/-16, tau=20",
                   "streams": n, "matcher": ("exhaustive search" if args.matcher == "es" else "diamond search") + f", k-skip {args.k_skip}",
                   "cache_expiry_frames": args.expiry, "frames_per_video": n_frames,
                   "lookahead_frames": 1 if args.lookahead else 0,
                   "mean_block_reuse": float(np.mean(agg["reuse"])) if agg["reuse"] else 0.0,
                   "full_frame_fraction": agg["full_frames"] / max(steps_all, 1),
                   "mac_fraction_needed": agg["macs_needed"] / max(agg["macs_full"], 1),
                   "mac_fraction_issued": agg["macs_issued"] / max(agg["macs_full"], 1)},
        "effective_tflops": 2.0 * agg["macs_full"] / max(steps_all, 1) * args.steps / elapsed / 1e12,
        "no_cache": {"value": fps_full, "unit": "frames/s", "saving": 1.0 - fps_full / fps},
        "roofline": roofline,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
