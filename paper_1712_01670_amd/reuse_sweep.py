#!/usr/bin/env python3
"""Frame time of the cache-aware path against the input reuse ratio (Section 7.2 reports the
saving per scenario; here the scenario is synthetic and the reuse ratio is the knob).

For every target reuse ratio a 60-frame video is generated (panning background under moving
rectangles of fresh noise whose sizes are calibrated to the non-reusable fraction, scene cut at
the middle), resident in HBM, and run three ways on one GPU:
  cached   every frame but the first of a scene goes through matching + cached convolution
           (no expiry), which isolates the cost of a cached frame;
  expiry   as deployed: a full frame every N frames (Section 5, N = 10);
  full     every frame computed in full (no cache).
One JSON line per ratio: measured reuse ratio, fraction of MACs needed and issued, frames/s of
the three modes and the saving 1 - t_mode / t_full.

    python paper_1712_01670_amd/reuse_sweep.py [--net darknet19|vgg16|resnet50|alexnet|googlenet] [--size 416] [--dtype bf16|f32]
                                               [--streams n] [--matcher es|ds] [--k-skip k]
                                               [--pan dx,dy] [--in-place] [--extend-borders]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--net", choices=["darknet19", "vgg16", "resnet50", "alexnet", "googlenet"], default="darknet19")
    ap.add_argument("--size", type=int, default=416)
    ap.add_argument("--dtype", choices=["bf16", "f32"], default="bf16")
    ap.add_argument("--ratios", default="0,0.25,0.5,0.75,0.95")
    ap.add_argument("--frames", type=int, default=60)
    ap.add_argument("--repeats", type=int, default=3)
    ap.add_argument("--expiry", type=int, default=10)
    ap.add_argument("--streams", type=int, default=1, help="independent videos processed as one batch per step")
    ap.add_argument("--matcher", choices=["es", "ds"], default="es")
    ap.add_argument("--k-skip", type=int, default=1)
    ap.add_argument("--pan", default="2,0", help="background motion in pixels per frame; 0,0 is a static camera")
    ap.add_argument("--lookahead", action="store_true",
                    help="hand the next frame over one step early, so that its matching starts then (dc_prefetch_match)")
    ap.add_argument("--extend-borders", action="store_true",
                    help="border case of the region rule for streams that did not move (beyond the paper's table)")
    ap.add_argument("--host-plan", action="store_true",
                    help="merge / propagate / list the dirty units on the host (one wait per frame) instead of on the GPU")
    ap.add_argument("--exact-masks", action="store_true", help="exact reuse maps instead of rectangles (planned on the GPU)")
    ap.add_argument("--cache-pool-add", action="store_true", help="with --exact-masks: max-pooling and add layers use the cache too")
    ap.add_argument("--torus", action="store_true", help="conv outputs on a torus: nothing is copied (planned on the GPU)")
    ap.add_argument("--min-reuse-macs", type=int, default=0,
                    help="conv layers with fewer multiply-adds per output element (k*k*cin) do not use the cache")
    ap.add_argument("--in-place", action="store_true",
                    help="let frames in which no stream moved update the cached tensors in place (no copies)")
    args = ap.parse_args()
    pan = tuple(int(v) for v in args.pan.split(","))

    import numpy as np
    import torch
    from paper_1712_01670_amd import binding, synth

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    H = W = args.size
    layers = {"darknet19": synth.darknet19, "vgg16": synth.vgg16, "resnet50": synth.resnet50_trunk,
              "alexnet": synth.alexnet, "googlenet": synth.googlenet}[args.net]()
    layers = synth.resolve_global_pooling(layers, H, W, 3)
    ws, bs = synth.he_weights(layers, 1, residual_scale=0.5 if args.net == "resnet50" else 1.0, input_shape=(H, W, 3))
    dt = binding.DC_BF16 if args.dtype == "bf16" else binding.DC_F32
    cut = args.frames // 2

    def timed(runner, video, mode):
        def one_pass(collect):
            macs = [0, 0, 0]
            reuse = []
            for f in range(args.frames):
                scene_start = f == 0 or f == cut
                if scene_start:
                    runner.reset()
                nxt = f + 1
                ahead = args.lookahead and mode != "full" and nxt < args.frames and nxt != cut
                runner.step(video[f], force_full=(mode == "full"), next_frames=video[nxt] if ahead else None)
                if collect:
                    torch.cuda.synchronize()
                    st = runner.read_stats()
                    macs[0] += st.macs_full; macs[1] += st.macs_needed; macs[2] += st.macs_issued
                    if not st.full:
                        reuse.append(st.n_reusable_blocks / st.n_blocks)
            return macs, reuse
        macs, reuse = one_pass(True)          # warm-up and statistics
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.repeats):
            one_pass(False)
        torch.cuda.synchronize()
        dt_s = (time.perf_counter() - t0) / (args.repeats * args.frames)
        return dt_s, macs, reuse

    for i, r in enumerate(float(x) for x in args.ratios.split(",")):
        vids = np.stack([synth.reuse_sweep_video(4000 + i + 100 * s, r, n_frames=args.frames, H=H, W=W, cut_at=cut, pan=pan)
                         for s in range(args.streams)])                       # [streams][T][H][W][3]
        video = torch.from_numpy(np.ascontiguousarray(vids.transpose(1, 0, 2, 3, 4))).to(dev)
        out = {"target_reuse": r, "net": args.net, "size": args.size, "dtype": args.dtype, "frames": args.frames,
               "streams": args.streams, "matcher": args.matcher, "k_skip": args.k_skip, "pan": list(pan), "in_place": bool(args.in_place), "extend_borders": bool(args.extend_borders),
               "lookahead": bool(args.lookahead), "planning": "host" if (args.host_plan or args.in_place) else "device", "exact_masks": bool(args.exact_masks), "cache_pool_add": bool(args.cache_pool_add and args.exact_masks), "min_reuse_macs": args.min_reuse_macs, "torus": bool(args.torus),
               "video": "panning background under moving noise rectangles sized for the target ratio, scene cut at the middle"}
        for mode, expiry in (("cached", 1 << 30), ("expiry", args.expiry), ("full", 1 << 30)):
            runner = binding.StackRunner(layers, ws, bs, args.streams, H, W, 3, block=16, radius=16, dtype=dt, expiry=expiry,
                                         match_method=binding.DC_MATCH_DIAMOND if args.matcher == "ds" else binding.DC_MATCH_EXHAUSTIVE,
                                         k_skip=args.k_skip, in_place=args.in_place, extend_borders=args.extend_borders,
                                         device_plan=not args.host_plan, exact_masks=args.exact_masks and not args.host_plan and not args.in_place,
                                         cache_pool_add=args.cache_pool_add and args.exact_masks and not args.host_plan and not args.in_place,
                                         no_reuse=synth.no_reuse_flags(layers, args.min_reuse_macs) if args.min_reuse_macs > 0 else None,
                                         # the all-full baseline alternates two buffers per tensor as without a torus
                                         torus=args.torus and mode != "full" and not args.host_plan and not args.in_place)
            t, macs, reuse = timed(runner, video, mode)
            out[mode] = {"frames_per_s": args.streams / t, "ms_per_frame": t * 1e3 / args.streams}
            if mode != "full":
                out[mode]["mac_fraction_needed"] = macs[1] / max(macs[0], 1)
                out[mode]["mac_fraction_issued"] = macs[2] / max(macs[0], 1)
            if mode == "cached":
                out["measured_reuse"] = float(np.mean(reuse)) if reuse else 0.0
            del runner
        for mode in ("cached", "expiry"):
            out[mode]["saving"] = 1.0 - out[mode]["ms_per_frame"] / out["full"]["ms_per_frame"]
        print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
