"""GPU parity of dc_run_stack (whole per-frame path) against the oracle: match results,
reuse masks and propagated rectangles bit-exact; every tensor within 1e-4 (fp32) or
2e-2 (bf16) of the oracle, relative to the tensor's largest magnitude."""
import numpy as np
import pytest
import torch

from paper_1712_01670_amd import binding, synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _rel_err(got, want):
    scale = max(float(np.abs(want).max()), 1e-30)
    return float(np.abs(got - want).max()) / scale


def _elem_err(got, want):
    """Element-wise variant: |g - o| / max(|o|, 1e-3 * max|o|), the floor keeps values near zero from deciding."""
    scale = max(float(np.abs(want).max()), 1e-30)
    return float((np.abs(got - want) / np.maximum(np.abs(want), 1e-3 * scale)).max())


def _run_both(oracle, layers, videos, block, radius, bf16, in_place=False, device_plan=None, exact_masks=False, **kw):
    exact_masks = exact_masks or bool(kw.get("cache_pool_add"))
    if kw.get("torus"):      # torus frames are planned on the GPU
        device_plan = True
    """Every frame of every stream against the oracle, with the frame planned on the host and (unless in-place frames
    are asked for, which only the host plans) once more with the frame planned on the GPU."""
    modes = [False] if in_place else ([False, True] if device_plan is None else [bool(device_plan)])
    if exact_masks:          # exact reuse maps exist on the GPU only
        modes = [True]
    first = None
    for dp in modes:
        res = _run_one(oracle, layers, videos, block, radius, bf16, in_place=in_place, device_plan=dp, exact_masks=exact_masks, **kw)
        if first is None:
            first = res
        else:
            assert res[1] == first[1]
    return first


def _run_one(oracle, layers, videos, block, radius, bf16, expiry=0, seed=1, bias_scale=0.05,
             residual_scale=1.0, check_tensors=None, resets=(), diamond=False, k_skip=1, in_place=False,
             extend_borders=False, device_plan=False, exact_masks=False, cache_pool_add=False, no_reuse=None, torus=False):
    """videos: uint8 [n_streams][T][H][W][C].  Compares every frame of every stream."""
    n, T, H, W, C = videos.shape
    ws, bs = synth.he_weights(layers, seed, bias_scale=bias_scale, residual_scale=residual_scale, input_shape=(H, W, C))
    tol = 2e-2 if bf16 else 1e-4
    dt = binding.DC_BF16 if bf16 else binding.DC_F32
    runner = binding.StackRunner(layers, ws, bs, n, H, W, C, block=block, radius=radius, dtype=dt, expiry=expiry,
                                 want_regions=True, k_skip=k_skip, in_place=in_place, extend_borders=extend_borders,
                                 match_method=binding.DC_MATCH_DIAMOND if diamond else binding.DC_MATCH_EXHAUSTIVE,
                                 device_plan=device_plan, exact_masks=exact_masks, cache_pool_add=cache_pool_add, no_reuse=no_reuse,
                                 torus=torus, want_origins=torus)
    streams = [oracle.Stream(layers, ws, bs, H, W, C, block=block, radius=radius, bf16=bf16, expiry=expiry,
                             diamond=diamond, k_skip=k_skip, extend_borders=extend_borders, exact_masks=exact_masks,
                             cache_pool_add=cache_pool_add, no_reuse=no_reuse)
               for _ in range(n)]
    dev_video = torch.from_numpy(np.ascontiguousarray(videos.transpose(1, 0, 2, 3, 4))).to(DEV)
    worst = worst_elem = 0.0
    reuse = []
    runner.in_place_frames = []
    shapes = runner.shapes
    for t in range(T):
        print(f"[stack] frame {t}/{T} n={n} {H}x{W} bf16={bf16} planned on the {'GPU' if device_plan else 'host'}"
              f"{', exact reuse maps' if exact_masks else ''}", flush=True)
        if t in resets:
            runner.reset()
            for s in streams:
                s.reset()
        tensors = runner.step(dev_video[t])
        torch.cuda.synchronize()
        runner.in_place_frames.append(bool(runner.last_in_place))
        got = [x.float().cpu().numpy() for x in runner.logical_tensors(tensors)]
        blocks = needed = 0
        for s in range(n):
            want = streams[s].step(videos[s, t])
            assert bool(runner.last_full) == bool(want["full"])
            if not want["full"]:
                m = want["match"]
                assert np.array_equal(runner.mv[s].cpu().numpy(), m["mv"])
                assert np.array_equal(runner.best_ssd[s].cpu().numpy().view(np.uint32), m["best_ssd"])
                assert runner.gmv[s].cpu().numpy().tolist() == m["gmv"].tolist()
                assert int(runner.n_pass[s]) == m["n_pass"]
                assert np.array_equal(runner.mask[s].cpu().numpy(), m["mask"])
                regs = runner.regions(s)
                for ti in range(len(layers) + 1):
                    if exact_masks:              # no rectangle lists in this mode; the maps are checked by the counters below
                        assert len(regs[ti]["rects"]) == 0
                        continue
                    assert regs[ti]["rects"].tolist() == want["rects"][ti].tolist(), (t, s, ti)
                    assert list(regs[ti]["dxy"]) == want["dxy"][ti].tolist()
                reuse.append(float(m["mask"].mean()))
                blocks += int(m["mask"].sum())
                for li, L in enumerate(layers):
                    if L["type"] == synth.CONV:
                        ho, wo, _ = shapes[li + 1]
                        reused = (int(want["masks"][li + 1].sum()) if exact_masks else
                                  int(sum(int(r[2]) * int(r[3]) for r in want["rects"][li + 1])))
                        if no_reuse is not None and no_reuse[li]:
                            reused = 0
                        kh, kw = synth.conv_geometry(L)[:2]
                        needed += (ho * wo - reused) * kh * kw * runner.layers[li]["cin"] * L["cout"]
            for ti in (check_tensors or range(len(layers) + 1)):
                g = got[ti][s]
                if ti == 0:          # tensor 0 may carry zero padding channels
                    assert not g[..., C:].any()
                    g = g[..., :C]
                e = _rel_err(g, want["tensors"][ti])
                worst = max(worst, e)
                worst_elem = max(worst_elem, _elem_err(g, want["tensors"][ti]))
                assert e <= tol, (t, s, ti, e)
        if not runner.last_full:     # the library's work counters against the oracle's masks and rectangles
            st = runner.read_stats()
            assert st.n_reusable_blocks == blocks and st.n_overflow_streams == 0
            assert st.macs_needed == needed and st.macs_issued >= st.macs_needed
    print(f"[stack] worst error relative to the tensor's largest magnitude {worst:.3e} (bound {tol:g}); element-wise "
          f"with floor 1e-3 of that magnitude {worst_elem:.3e}; mean block reuse {np.mean(reuse) if reuse else 0:.3f}", flush=True)
    return runner, reuse


@pytest.mark.parametrize("bf16", [False, True])
def test_tiny_config(oracle, bf16):
    f1, f2 = synth.tiny_pair(0)
    video = np.stack([f1, f2, f2, f1])[None]
    runner, reuse = _run_both(oracle, synth.tiny_net(), video, 8, 8, bf16)
    assert abs(reuse[0] - 45 / 64) < 1e-9
    assert reuse[1] == 1.0


def test_tiny_exact_shift_equals_full_forward_on_gpu(oracle):
    # the invariant of the oracle also holds for the HIP path: with an exact shift by a multiple of
    # the total stride the cached frame reproduces the full forward (copies are bit copies; recomputed
    # pixels go through the same kernel)
    layers = synth.tiny_net()
    f1, f2 = synth.shifted_pair(10, 64, 64, (4, -2))
    ws, bs = synth.he_weights(layers, 1, bias_scale=0.05)
    r = binding.StackRunner(layers, ws, bs, 1, 64, 64, 3, block=8, radius=8)
    d1, d2 = torch.from_numpy(f1[None]).to(DEV), torch.from_numpy(f2[None]).to(DEV)
    r.step(d1)
    cached = [t.clone() for t in r.step(d2)]
    torch.cuda.synchronize()
    assert r.read_stats().n_reusable_blocks >= 40
    r.reset()
    full = r.step(d2)
    for a, b in zip(cached, full):
        assert torch.equal(a, b)


def test_vgg16_224_first_frames(oracle):
    video = synth.panning_video(2000, n_frames=3)[None]
    _run_both(oracle, synth.vgg16(), video, 16, 16, False, bias_scale=0.0)


@pytest.mark.parametrize("k_skip", [1, 2])
def test_diamond_search_in_the_whole_path(oracle, k_skip):
    # the paper's matcher (diamond search, k-skip) feeding the same region logic and cached convolutions
    f1, f2 = synth.tiny_pair(0)
    runner, reuse = _run_both(oracle, synth.tiny_net(), np.stack([f1, f2, f2, f1])[None], 8, 8, False,
                              diamond=True, k_skip=k_skip)
    assert reuse[1] == 1.0
    v = np.stack([synth.panning_video(5100 + s, n_frames=4, H=96, W=96, fg=((24, 24),), margin=32) for s in range(2)])
    runner, reuse = _run_both(oracle, synth.vgg16(), v, 16, 16, False, bias_scale=0.0, diamond=True, k_skip=k_skip,
                              check_tensors=(0, 1, 2, 5, 10, 17))
    assert max(reuse) > 0.3


def test_exhaustive_search_with_k_skip_in_the_whole_path(oracle):
    f1, f2 = synth.tiny_pair(0)
    _run_both(oracle, synth.tiny_net(), np.stack([f1, f2, f2, f1])[None], 8, 8, False, k_skip=2)


@pytest.mark.parametrize("bf16", [False, True])
def test_alexnet_style_stack_small(oracle, bf16):
    """Every layer type of Table 2 in one stack: 11x11 stride-4 first layer, LRN, pooling, fully-connected, softmax
    (a narrow AlexNet at its 227x227 input size; the paper's 10-pixel blocks)."""
    layers = synth.alexnet(n_classes=40, width=0.25)
    video = np.stack([synth.panning_video(300 + s, n_frames=3, H=227, W=227) for s in range(2)])
    runner, reuse = _run_both(oracle, layers, video, 10, 8, bf16)
    assert len(reuse) == 4 and min(reuse) > 0.2


def test_alexnet_full_width_fp32(oracle):
    """The AlexNet-style stack at its real widths (96-256-384-384-256 channels, 4096-wide fully-connected layers),
    227x227, the paper's 10-pixel blocks: every tensor of a full and a cached frame against the oracle."""
    layers = synth.alexnet()
    video = synth.panning_video(310, n_frames=2, H=227, W=227)[None]
    _run_both(oracle, layers, video, 10, 8, False, bias_scale=0.02)


@pytest.mark.parametrize("bf16", [False, True])
def test_dave_orig_stack(oracle, bf16):
    """The steering network: a 66x200 frame (not square), 5x5 stride-2 convolutions without padding, channel counts
    (24, 36, 48) that are not whole 16-byte vectors in bf16, four fully-connected layers."""
    layers = synth.dave_orig()
    video = np.stack([synth.panning_video(800 + s, n_frames=3, H=66, W=200, fg=((16, 24),)) for s in range(2)])
    runner, reuse = _run_both(oracle, layers, video, 10, 8, bf16, bias_scale=0.02)
    assert runner.shapes[5] == (1, 18, 64) and runner.shapes[-1] == (1, 1, 1)


def test_googlenet_full_width_bf16(oracle):
    """The GoogLeNet-style stack at its real widths, 224x224, bf16: a full and a cached frame."""
    layers = synth.resolve_global_pooling(synth.googlenet(), 224, 224, 3)
    video = synth.panning_video(410, n_frames=2, H=224, W=224)[None]
    _run_both(oracle, layers, video, 16, 8, True, bias_scale=0.02)


def test_googlenet_style_stack_small(oracle):
    """Inception modules: four branches of different depth joined by a concat; global average pooling at the end."""
    layers = synth.resolve_global_pooling(synth.googlenet(n_classes=24, width=0.25), 224, 224, 3)
    assert sum(L["type"] == synth.CONV for L in layers) == 57
    video = np.stack([synth.panning_video(400 + s, n_frames=3, H=224, W=224) for s in range(1)])
    _run_both(oracle, layers, video, 16, 8, True)


def _static_then_moving(seed, H, W, n_static, n_moving):
    """A camera that stands still (only a small object moves), then pans, then stands still again."""
    still = synth.panning_video(seed, n_frames=n_static, H=H, W=W, fg=((24, 24),), pan_speeds=(0,))
    moving = synth.panning_video(seed, n_frames=n_static + n_moving, H=H, W=W, fg=((24, 24),), pan_speeds=(2,),
                                 redraw_every=100)[n_static:]
    return np.concatenate([still, moving, still[::-1]])


@pytest.mark.parametrize("bf16", [False, True])
def test_in_place_frames_of_a_static_camera(oracle, bf16):
    """No stream moves: the conv outputs are updated in the previous frame's buffers and nothing is copied; the
    values are the oracle's (which knows nothing of buffers)."""
    layers = synth.vgg16()[:7]
    video = np.stack([synth.panning_video(500 + s, n_frames=4, H=96, W=96, fg=((24, 24),), pan_speeds=(0,)) for s in range(2)])
    runner, reuse = _run_both(oracle, layers, video, 16, 8, bf16, in_place=True)
    assert runner.in_place_frames == [False, True, True, True]
    assert runner.stats.copy_bytes == 0 and runner.stats.macs_needed < runner.stats.macs_full
    assert min(reuse) > 0.5


def test_border_case_of_a_static_camera(oracle):
    """extend_borders: windows may reach into the zero padding when the stream did not move; regions and tensors
    follow the oracle with the same option, and more pixels are reused than with the printed rule."""
    layers = synth.vgg16()[:10]
    video = np.stack([_static_then_moving(700 + s, 96, 96, 3, 2) for s in range(2)])
    needed = {}
    for ext in (False, True):
        runner, _ = _run_both(oracle, layers, video, 16, 8, True, in_place=True, extend_borders=ext)
        needed[ext] = runner.stats.macs_needed          # last frame: static again
        assert runner.in_place_frames[-1]
    assert needed[True] < needed[False]


def test_in_place_and_copied_frames_mix(oracle):
    """Static and moving stretches in one video: in-place frames where every stream's motion is zero, shifted copies
    elsewhere, parity on every frame; and bit-identical tensors with the option off."""
    layers = synth.resnet50_trunk()[:14]
    video = np.stack([_static_then_moving(600 + s, 96, 96, 3, 3) for s in range(2)])
    runner, _ = _run_both(oracle, layers, video, 16, 8, True, residual_scale=0.5, in_place=True)
    flags = runner.in_place_frames
    assert flags[1] and flags[2] and not any(flags[3:6]) and flags[-1], flags
    ws, bs = synth.he_weights(layers, 1, bias_scale=0.05, residual_scale=0.5, input_shape=(96, 96, 3))
    dev_video = torch.from_numpy(np.ascontiguousarray(video.transpose(1, 0, 2, 3, 4))).to(DEV)
    runs = [binding.StackRunner(layers, ws, bs, 2, 96, 96, 3, block=16, radius=8, dtype=binding.DC_BF16, in_place=ip)
            for ip in (False, True)]
    for t in range(video.shape[1]):
        outs = []
        for r in runs:
            tensors = r.step(dev_video[t])
            torch.cuda.synchronize()
            outs.append([x.clone() for x in tensors])
        for a, b in zip(*outs):
            assert torch.equal(a, b), t


def test_vgg16_two_streams_bf16_small(oracle):
    # batch mode: per-stream caches, per-stream motion, one launch per layer
    v = np.stack([synth.panning_video(5000 + s, n_frames=3, H=96, W=96, fg=((24, 24),), margin=32) for s in range(2)])
    _run_both(oracle, synth.vgg16(), v, 16, 16, True, bias_scale=0.0)


def test_expiry_and_reset(oracle):
    f1, f2 = synth.tiny_pair(3)
    video = np.stack([f1, f2, f2, f1, f1, f2])[None]
    _run_both(oracle, synth.tiny_net(), video, 8, 8, False, expiry=3, resets=(4,))


def test_resnet_stage_small(oracle):
    layers = synth.resnet50_trunk()[:23]     # stem, pool, stage 1 (3 blocks), first block of stage 2
    v = synth.panning_video(3000, n_frames=3, H=96, W=96, fg=((24, 24),), margin=32)[None]
    _run_both(oracle, layers, v, 16, 16, True, bias_scale=0.0, residual_scale=0.5)
    _run_both(oracle, layers, v, 16, 16, False, bias_scale=0.0, residual_scale=0.5)


@pytest.mark.parametrize("bf16", [False, True])
def test_darknet_with_leaky_relu_small(oracle, bf16):
    """The published Darknet activation (leaky ReLU, slope 0.1) through every conv kernel family: first layer, 3x3,
    1x1, and the register-weight kernel's fallback."""
    layers = synth.darknet19(leaky=True)[:12]
    video = np.stack([synth.panning_video(900 + s, n_frames=3, H=96, W=96, fg=((24, 24),)) for s in range(2)])
    _run_both(oracle, layers, video, 16, 8, bf16)


def test_darknet_head_small(oracle):
    layers = synth.darknet19()[:12]
    v = synth.reuse_sweep_video(4001, 0.75, n_frames=3, H=128, W=128, cut_at=2)[None]
    _run_both(oracle, layers, v, 16, 16, True, bias_scale=0.0, resets=(2,))


# ---- full-size configurations -------------------------------------------------------------------

def _sampled_conv_check(oracle, layers, ws, bs, tensors, li, stream, bf16, n_samples, rng, tol):
    """Recompute sampled output pixels of conv layer li from the GPU's own input tensor with the oracle's
    direct loop (valid for pixels that were computed, i.e. on a full frame)."""
    L = layers[li]
    x = tensors[L["in0"]][stream].float().cpu().numpy()
    y = tensors[li + 1][stream].float().cpu().numpy()
    w = oracle.round_bf16(ws[li]) if bf16 else ws[li]
    if w.shape[-1] < x.shape[-1]:     # input channels padded by the runner
        wp = np.zeros(w.shape[:3] + (x.shape[-1],), np.float32)
        wp[..., :w.shape[-1]] = w
        w = wp
    k, s, p = L["k"], L["s"], L["p"]
    Ho, Wo, _ = y.shape
    scale = float(np.abs(y).max()) + 1e-30
    for _ in range(n_samples):
        oy, ox = int(rng.integers(0, Ho)), int(rng.integers(0, Wo))
        # window of the input around the sampled pixel, zero padded
        win = np.zeros((k, k, x.shape[-1]), np.float32)
        for ky in range(k):
            for kx in range(k):
                iy, ix = oy * s - p + ky, ox * s - p + kx
                if 0 <= iy < x.shape[0] and 0 <= ix < x.shape[1]:
                    win[ky, kx] = x[iy, ix]
        want = oracle.conv_cached(win, w, bs[li], k, 1, 0, L["relu"], bf16=bf16)[0, 0]
        assert np.abs(y[oy, ox] - want).max() / scale <= tol, (li, oy, ox)


def test_resnet50_trunk_224_bf16_full_size(oracle):
    """configs[2] at full size: two frames through the GPU path; frame 0 against the oracle's whole stack
    (full compute), frame 1 (cached) for rectangles bit-exact and features within tolerance."""
    layers = synth.resnet50_trunk()
    video = synth.panning_video(2000, n_frames=2)[None]
    _run_both(oracle, layers, video, 16, 16, True, bias_scale=0.0, residual_scale=0.5)


def test_darknet19_416_bf16_cached_frame_and_scene_cut(oracle):
    """configs[3] at full size (416x416, 19 conv layers, bf16, moving noise rectangles at half reuse): the last two
    frames of the first scene and the first two of the second, with the cache dropped at the cut as the config
    says.  Every tensor of the full frames and of the cached frames (reused pixels are the oracle's shifted cache,
    the others its convolution), match results, masks and rectangles against the oracle's stream."""
    layers = synth.darknet19()
    video = synth.reuse_sweep_video(4002, 0.5, n_frames=60)[28:32][None]
    runner, reuse = _run_both(oracle, layers, video, 16, 16, True, bias_scale=0.0, resets=(2,))
    assert len(reuse) == 2 and all(0.45 < r < 0.6 for r in reuse)


@pytest.mark.parametrize("device_plan,exact,torus", [(False, False, False), (True, False, False), (True, True, False),
                                                     (True, True, True)])
def test_throughput_mode_64_streams_bf16_sampled(oracle, device_plan, exact, torus):
    """configs[4] launch configuration: 64 streams in one batch, VGG-16-style, bf16, planned on the host, on the GPU, on
    the GPU with exact reuse maps, and the same with the conv outputs on a torus (what bench.py times).  Three streams
    are followed by the oracle over four time steps (everything compared); the others are checked for bit-exact match
    results on the cached steps."""
    layers = synth.vgg16()
    n, T = 64, 4 if torus else 3
    videos = np.stack([synth.panning_video(5000 + s, n_frames=T) for s in range(n)])
    ws, bs = synth.he_weights(layers, 1)
    r = binding.StackRunner(layers, ws, bs, n, 224, 224, 3, block=16, radius=16, dtype=binding.DC_BF16, want_regions=True,
                            device_plan=device_plan, exact_masks=exact, torus=torus, want_origins=torus)
    followed = [0, 31, 63]
    refs = {s: oracle.Stream(layers, ws, bs, 224, 224, 3, block=16, radius=16, bf16=True, exact_masks=exact) for s in followed}
    dv = torch.from_numpy(np.ascontiguousarray(videos.transpose(1, 0, 2, 3, 4))).to(DEV)
    for t in range(T):
        print(f"[batch64] step {t}", flush=True)
        tensors = r.step(dv[t])
        torch.cuda.synchronize()
        if torus:       # only the followed streams are rolled back to their logical layout
            moved = r.origins.copy()
            tensors = [x if not moved[followed, ti].any() else
                       {s: torch.roll(x[s], shifts=(-int(moved[s, ti, 1]), -int(moved[s, ti, 0])), dims=(0, 1)) for s in followed}
                       for ti, x in enumerate(tensors)]
        for s in followed:
            want = refs[s].step(videos[s, t])
            for ti in range(1, len(layers) + 1):
                g = tensors[ti][s].float().cpu().numpy()
                assert _rel_err(g, want["tensors"][ti]) <= 2e-2, (t, s, ti)
            if t > 0 and not exact:
                regs = r.regions(s)
                for ti in range(len(layers) + 1):
                    assert regs[ti]["rects"].tolist() == want["rects"][ti].tolist()
        if t > 0:
            if exact:       # the maps themselves: the multiply-adds the library counted are those of the oracle's maps
                assert r.read_stats().n_overflow_streams == 0
            masks = r.mask.cpu().numpy()
            gmv = r.gmv.cpu().numpy()
            for s in range(0, n, 7):
                m = oracle.match_blocks(videos[s, t], videos[s, t - 1], 16, 16, synth.max_block_ssd(16))
                assert np.array_equal(masks[s], m["mask"]) and gmv[s].tolist() == m["gmv"].tolist()


@pytest.mark.parametrize("bf16", [False, True])
def test_exact_reuse_maps_tiny_and_vgg(oracle, bf16):
    """dc_match_options.exact_masks: the conv layers reuse the pixels of the exact maps; tensors and work counters
    against the oracle's stream in the same mode."""
    f1, f2 = synth.tiny_pair(0)
    runner, reuse = _run_both(oracle, synth.tiny_net(), np.stack([f1, f2, f2, f1])[None], 8, 8, bf16, exact_masks=True)
    assert abs(reuse[0] - 45 / 64) < 1e-9
    v = np.stack([synth.panning_video(5000 + s, n_frames=3, H=96, W=96, fg=((24, 24),), margin=32) for s in range(2)])
    _run_both(oracle, synth.vgg16(), v, 16, 16, bf16, bias_scale=0.0, exact_masks=True)


def test_exact_reuse_maps_other_stacks(oracle):
    v = synth.panning_video(3000, n_frames=3, H=96, W=96, fg=((24, 24),), margin=32)[None]
    _run_both(oracle, synth.resnet50_trunk()[:23], v, 16, 16, True, bias_scale=0.0, residual_scale=0.5, exact_masks=True)
    v = synth.reuse_sweep_video(4001, 0.75, n_frames=3, H=128, W=128, cut_at=2)[None]
    _run_both(oracle, synth.darknet19()[:12], v, 16, 16, True, bias_scale=0.0, resets=(2,), exact_masks=True)
    layers = synth.alexnet(n_classes=40, width=0.25)
    video = np.stack([synth.panning_video(300 + s, n_frames=3, H=227, W=227) for s in range(2)])
    _run_both(oracle, layers, video, 10, 8, False, exact_masks=True)
    video = np.stack([_static_then_moving(700 + s, 96, 96, 3, 2) for s in range(2)])
    _run_both(oracle, synth.vgg16()[:10], video, 16, 8, True, extend_borders=True, exact_masks=True)


def test_exact_reuse_maps_vgg16_224_save_more(oracle):
    """configs[1] with exact maps: parity on the first frames, and fewer multiply-adds needed than with rectangles."""
    video = synth.panning_video(2000, n_frames=3)[None]
    exact, _ = _run_both(oracle, synth.vgg16(), video, 16, 16, False, bias_scale=0.0, exact_masks=True)
    rect, _ = _run_both(oracle, synth.vgg16(), video, 16, 16, False, bias_scale=0.0, device_plan=True)
    assert exact.read_stats().macs_needed < rect.read_stats().macs_needed


def _pool_add_stack(c=8):
    conv = lambda cin, cout, i, relu=1: dict(type=synth.CONV, k=3, s=1, p=1, cin=cin, cout=cout, relu=relu, in0=i, in1=-1)
    return [conv(3, c, 0), dict(type=synth.MAXPOOL, k=2, s=2, p=0, cin=c, cout=c, relu=0, in0=1, in1=-1),
            conv(c, c, 2), conv(c, c, 3, 0), dict(type=synth.ADD, k=1, s=1, p=0, cin=c, cout=c, relu=1, in0=4, in1=2),
            dict(type=synth.MAXPOOL, k=3, s=2, p=1, cin=c, cout=c, relu=0, in0=5, in1=-1), conv(c, c, 6)]


@pytest.mark.parametrize("bf16", [False, True])
def test_cached_pool_and_add_layers(oracle, bf16):
    """dc_match_options.cache_pool_add: max-pooling and add outputs come from the cache where their maps are set
    (Section 5).  The case is one where the option changes the result, so a library that ignored it would fail."""
    layers = _pool_add_stack()
    f1, f2 = synth.tiny_pair(0)                   # a noisy frame moved by (3, -2): not a multiple of the strides
    video = np.stack([f1, f2, f2, f1])[None]
    H, W, C = f1.shape
    ws, bs = synth.he_weights(layers, 1, bias_scale=0.05, input_shape=(H, W, C))
    on = oracle.Stream(layers, ws, bs, H, W, C, block=8, radius=8, bf16=bf16, exact_masks=True, cache_pool_add=True)
    off = oracle.Stream(layers, ws, bs, H, W, C, block=8, radius=8, bf16=bf16, exact_masks=True)
    a = [on.step(f) for f in (f1, f2)][1]["tensors"][2]
    b = [off.step(f) for f in (f1, f2)][1]["tensors"][2]
    assert _rel_err(a, b) > 0.05
    _run_both(oracle, layers, video, 8, 8, bf16, cache_pool_add=True)
    # several streams, a scene cut and a forced full frame in between
    video = np.stack([synth.reuse_sweep_video(4100 + s, 0.75, n_frames=5, H=96, W=96, cut_at=3) for s in range(3)])
    _run_both(oracle, layers, video, 8, 8, bf16, cache_pool_add=True, resets=(2,))


def test_cached_pool_and_add_in_the_model_stacks(oracle):
    v = np.stack([synth.panning_video(5000 + s, n_frames=3, H=96, W=96, fg=((24, 24),), margin=32) for s in range(2)])
    _run_both(oracle, synth.vgg16(), v, 16, 16, True, bias_scale=0.0, cache_pool_add=True)
    v = synth.panning_video(3000, n_frames=3, H=96, W=96, fg=((24, 24),), margin=32)[None]
    _run_both(oracle, synth.resnet50_trunk()[:23], v, 16, 16, True, bias_scale=0.0, residual_scale=0.5, cache_pool_add=True)
    v = synth.reuse_sweep_video(4001, 0.75, n_frames=3, H=128, W=128)[None]
    _run_both(oracle, synth.darknet19()[:12], v, 16, 16, False, bias_scale=0.0, cache_pool_add=True)


def test_cache_pool_add_needs_exact_maps_and_previous_outputs(oracle):
    layers = _pool_add_stack()
    f1, f2 = synth.tiny_pair(0)
    H, W, C = f1.shape
    ws, bs = synth.he_weights(layers, 1, input_shape=(H, W, C))
    r = binding.StackRunner(layers, ws, bs, 1, H, W, C, block=8, radius=8, dtype=binding.DC_F32, device_plan=True,
                            exact_masks=True, cache_pool_add=True)
    r.match_options.exact_masks = 0
    with pytest.raises(binding.DcError) as e:
        r.step(torch.from_numpy(f1[None]).to(DEV))
    assert e.value.status == -4
    torch.cuda.synchronize()


@pytest.mark.parametrize("exact", [False, True])
def test_conv_layers_that_do_not_use_the_cache(oracle, exact):
    """dc_match_options.no_reuse: flagged conv layers are computed in full, the others reuse; planned on the host and on
    the GPU, rectangles and exact maps."""
    layers = synth.tiny_net()
    f1, f2 = synth.tiny_pair(0)
    video = np.stack([f1, f2, f2, f1])[None]
    for flags in ([0, 1, 0], [1, 0, 1], [1, 1, 1]):
        _run_both(oracle, layers, video, 8, 8, False, exact_masks=exact, no_reuse=np.array(flags, np.uint8))
    # the break-even policy on a model stack: layers with few multiply-adds per output are not cached
    v = np.stack([synth.panning_video(5000 + s, n_frames=3, H=96, W=96, fg=((24, 24),), margin=32) for s in range(2)])
    layers = synth.vgg16()
    flags = synth.no_reuse_flags(layers, 600)
    assert flags.tolist()[:5] == [1, 1, 0, 1, 0] and flags.sum() == 3
    _run_both(oracle, layers, v, 16, 16, True, bias_scale=0.0, exact_masks=exact, no_reuse=flags)
    layers = synth.resnet50_trunk()[:23]
    v = synth.panning_video(3000, n_frames=3, H=96, W=96, fg=((24, 24),), margin=32)[None]
    _run_both(oracle, layers, v, 16, 16, True, bias_scale=0.0, residual_scale=0.5, exact_masks=exact,
              no_reuse=synth.no_reuse_flags(layers, 600))


@pytest.mark.parametrize("bf16", [False, True])
def test_stack_with_kernels_that_are_not_square_or_dilated(oracle, bf16):
    """1 x 7 / 7 x 1 pairs, dilated 3 x 3 and 5 x 3 kernels (dc_layer.k2 / p2 / dil) through the whole path: regions,
    exact maps, copies and the general conv kernels, planned on the host and on the GPU."""
    layers = synth.factorised_net(16)
    video = np.stack([synth.panning_video(900 + s, n_frames=3, H=96, W=96, fg=((24, 24),), margin=32) for s in range(2)])
    runner, reuse = _run_both(oracle, layers, video, 8, 8, bf16)
    assert max(reuse) > 0.3
    _run_both(oracle, layers, video, 8, 8, bf16, exact_masks=True)
    f1, f2 = synth.tiny_pair(0)
    _run_both(oracle, layers, np.stack([f1, f2, f2])[None], 8, 8, bf16, extend_borders=True)


def _torus_stack(c=64):
    """first layer on a padded pixel vector, 3x3 layers with whole 64-byte rows, 2x2 poolings: what the torus mode takes"""
    return synth.small_vgg(c)


@pytest.mark.parametrize("exact", [False, True])
@pytest.mark.parametrize("bf16", [False, True])
def test_conv_outputs_on_a_torus(oracle, bf16, exact):
    """dc_match_options.torus: nothing is copied, every conv output is one buffer whose origin moves with the frames; the
    tensors, read from their origins, are those of the oracle's stream (and of the copying path)."""
    layers = _torus_stack()
    # a pan that crosses the seams several times, streams that move differently, a scene cut, an expiry in between
    video = np.stack([synth.panning_video(7000 + s, n_frames=7, H=96, W=96, fg=((24, 24),), margin=32) for s in range(3)])
    runner, reuse = _run_one(oracle, layers, video, 16, 16, bf16, device_plan=True, exact_masks=exact, torus=True, resets=(4,),
                             expiry=3, bias_scale=0.0)
    assert max(reuse) > 0.3 and runner.torus
    # the tiny pair: motion (-3, +2), then a frame that does not move, then back
    f1, f2 = synth.tiny_pair(0)
    _run_one(oracle, _torus_stack(64), np.stack([f1, f2, f2, f1, f2])[None], 8, 8, bf16, device_plan=True, exact_masks=exact, torus=True)


def test_torus_vgg16_two_streams(oracle):
    v = np.stack([synth.panning_video(5000 + s, n_frames=4, H=96, W=96, fg=((24, 24),), margin=32) for s in range(2)])
    runner, _ = _run_one(oracle, synth.vgg16(), v, 16, 16, True, device_plan=True, exact_masks=True, torus=True, bias_scale=0.0)
    assert runner.origins.any()          # some origin moved
    assert runner.read_stats().copy_bytes == 0


def test_torus_tensors_read_without_a_wait(oracle):
    """dc_torus_read with the device address of the frame's origins (origins_dev_out): the logical tensors without any
    host wait, equal to those rolled on the host from origins_out; full frames (no origins) included."""
    layers = synth.small_vgg()
    video = np.stack([synth.panning_video(7600 + s, n_frames=6, H=96, W=96, fg=((24, 24),), margin=32) for s in range(3)])
    ws, bs = synth.he_weights(layers, 1, bias_scale=0.05)
    r = binding.StackRunner(layers, ws, bs, 3, 96, 96, 3, block=16, radius=16, dtype=binding.DC_BF16, device_plan=True,
                            exact_masks=True, cache_pool_add=True, torus=True, want_origins=True, expiry=4)
    dv = torch.from_numpy(np.ascontiguousarray(video.transpose(1, 0, 2, 3, 4))).to(DEV)
    moved = False
    for t in range(6):
        tensors = r.step(dv[t])
        got = [r.read_tensor(ti, tensors) for ti in range(len(layers) + 1)]      # queued behind the frame, nothing waited for
        torch.cuda.synchronize()
        want = r.logical_tensors(tensors)
        moved = moved or bool(r.origins.any())
        for ti in range(len(layers) + 1):
            assert torch.equal(got[ti], want[ti]), (t, ti)
    assert moved
    # odd channel counts and element sizes take the narrower vectors
    x = torch.randn((2, 5, 7, 3), device=DEV)
    org = torch.tensor([[3, 1], [6, 4]], dtype=torch.int32, device=DEV)
    out = torch.empty_like(x)
    L = binding.lib()
    import ctypes as C
    assert L.dc_torus_read(C.c_void_p(x.data_ptr()), C.c_void_p(out.data_ptr()), C.c_void_p(org.data_ptr()), 2, 2, 5, 7, 3,
                           binding.DC_F32, None) == 0
    torch.cuda.synchronize()
    for s in range(2):
        assert torch.equal(out[s], torch.roll(x[s], shifts=(-int(org[s, 1]), -int(org[s, 0])), dims=(0, 1)))
    assert L.dc_torus_read(C.c_void_p(x.data_ptr()), C.c_void_p(x.data_ptr()), None, 2, 2, 5, 7, 3, binding.DC_F32, None) == -1


@pytest.mark.parametrize("bf16", [False, True])
def test_poolings_on_the_torus_too(oracle, bf16):
    """torus with cache_pool_add: the poolings' outputs are cache values on a torus of their own, a pooled pixel whose map
    bit is set is not touched; the oracle's stream with max-pooling through the cache gives the logical tensors."""
    video = np.stack([synth.panning_video(7100 + s, n_frames=7, H=96, W=96, fg=((24, 24),), margin=32) for s in range(3)])
    runner, reuse = _run_one(oracle, _torus_stack(), video, 16, 16, bf16, device_plan=True, exact_masks=True, cache_pool_add=True,
                             torus=True, resets=(4,), expiry=3)
    assert max(reuse) > 0.3 and runner.origins[:, 3].any()       # tensor 3 is the first pooling's output
    v = np.stack([synth.panning_video(5000 + s, n_frames=4, H=96, W=96, fg=((24, 24),), margin=32) for s in range(2)])
    _run_one(oracle, synth.vgg16(), v, 16, 16, bf16, device_plan=True, exact_masks=True, cache_pool_add=True, torus=True, bias_scale=0.0)
    if bf16:     # enough units for the register-weight kernel in the second layer, whose output the first pooling reads
        v32 = np.stack([synth.panning_video(7700 + s, n_frames=4, H=96, W=96, fg=((24, 24),), margin=32) for s in range(32)])
        runner, _ = _run_one(oracle, synth.small_vgg(), v32, 16, 16, True, device_plan=True, exact_masks=True, cache_pool_add=True,
                             torus=True, resets=(2,))
        assert runner.layer_stats()["kernel_id"][1] == 130


def test_torus_with_the_border_case_and_layers_outside_the_cache(oracle):
    layers = _torus_stack()
    video = np.stack([_static_then_moving(700 + s, 96, 96, 3, 2) for s in range(2)])
    _run_one(oracle, layers, video, 16, 8, True, extend_borders=True, device_plan=True, exact_masks=True, torus=True)
    flags = np.zeros(len(layers), np.uint8)
    flags[1] = flags[4] = 1
    v = np.stack([synth.panning_video(7200 + s, n_frames=5, H=96, W=96, fg=((24, 24),), margin=32) for s in range(2)])
    _run_one(oracle, layers, v, 16, 16, False, device_plan=True, exact_masks=False, torus=True, no_reuse=flags)


@pytest.mark.parametrize("bf16,leaky", [(True, False), (False, True)])
def test_torus_darknet_with_1x1_layers(oracle, bf16, leaky):
    """The Darknet-19-style stack on a torus: 3x3 layers, 1x1 bottlenecks (the 1x1 kernel reads and writes through
    origins), 2x2 poolings, maps with ragged units (13 x 13 at the end), ReLU or leaky ReLU."""
    video = np.stack([synth.panning_video(7500 + s, n_frames=5, H=208, W=208, fg=((48, 48),), margin=32) for s in range(2)])
    runner, reuse = _run_one(oracle, synth.darknet19(leaky=leaky)[:17], video, 16, 8, bf16, device_plan=True, exact_masks=True,
                             torus=True, resets=(3,), bias_scale=0.02)
    assert max(reuse) > 0.3 and runner.origins.any() and runner.shapes[-1][0] == 13


def test_torus_on_a_frame_whose_maps_do_not_fit_the_lds(oracle):
    """640 x 480: the reuse bitmaps of the stack (more than 128 KB) are built in the workspace; the origins come from the
    same planning kernel.  One full and two cached frames of one stream."""
    video = synth.panning_video(7400, n_frames=3, H=480, W=640, fg=((96, 96),), margin=64)[None]
    runner, reuse = _run_one(oracle, synth.small_vgg(), video, 16, 16, True, device_plan=True, exact_masks=True, torus=True,
                             bias_scale=0.0)
    assert max(reuse) > 0.5 and runner.origins.any()


def test_torus_with_more_streams_than_the_origin_tables_hold(oracle):
    """Beyond 2048 streams the persistent kernels do not keep the origins in LDS: the first layer loads them from memory
    and the 64-channel layers take the tiled GEMM kernel.  2100 small streams (three videos, repeated); six are compared."""
    layers = synth.small_vgg()
    n, T, H, W = 2100, 3, 32, 32
    base = np.stack([synth.panning_video(7300 + s, n_frames=T, H=H, W=W, fg=((8, 8),), margin=16) for s in range(3)])
    videos = base[np.arange(n) % 3]
    ws, bs = synth.he_weights(layers, 1, bias_scale=0.05)
    r = binding.StackRunner(layers, ws, bs, n, H, W, 3, block=16, radius=8, dtype=binding.DC_BF16, device_plan=True,
                            exact_masks=True, torus=True, want_origins=True)
    followed = [0, 1, 2, 1037, 2098, 2099]
    refs = {s: oracle.Stream(layers, ws, bs, H, W, 3, block=16, radius=8, bf16=True, exact_masks=True) for s in followed}
    dv = torch.from_numpy(np.ascontiguousarray(videos.transpose(1, 0, 2, 3, 4))).to(DEV)
    reused = 0
    for t in range(T):
        print(f"[many streams] step {t}", flush=True)
        tensors = r.step(dv[t])
        torch.cuda.synchronize()
        org = r.origins.copy()
        for s in followed:
            want = refs[s].step(videos[s, t])
            for ti in range(1, len(layers) + 1):
                g = torch.roll(tensors[ti][s], shifts=(-int(org[s, ti, 1]), -int(org[s, ti, 0])), dims=(0, 1)).float().cpu().numpy()
                assert _rel_err(g, want["tensors"][ti]) <= 2e-2, (t, s, ti)
        if t > 0:
            reused += int(r.read_stats().n_reusable_blocks)
    assert reused > 0


def test_torus_is_refused_for_stacks_it_cannot_take(oracle):
    layers = synth.resnet50_trunk()[:10]         # 1x1 and strided layers, adds
    H = W = 64
    ws, bs = synth.he_weights(layers, 1, input_shape=(H, W, 3))
    r = binding.StackRunner(layers, ws, bs, 1, H, W, 3, block=16, radius=8, dtype=binding.DC_BF16, device_plan=True, torus=True)
    with pytest.raises(binding.DcError) as e:
        r.step(torch.zeros((1, H, W, 3), dtype=torch.uint8, device=DEV))
    assert e.value.status == -4
    torch.cuda.synchronize()


def test_border_case_planned_on_the_gpu(oracle):
    """extend_borders with the frame planned on the GPU (copy path: in-place frames are the host's)."""
    layers = synth.vgg16()[:10]
    video = np.stack([_static_then_moving(700 + s, 96, 96, 3, 2) for s in range(2)])
    _run_both(oracle, layers, video, 16, 8, True, extend_borders=True, device_plan=True)


@pytest.mark.parametrize("n_streams,bf16", [(1, False), (3, True)])
def test_frames_planned_on_the_gpu_without_any_wait(oracle, n_streams, bf16):
    """Frames planned on the GPU, two in flight, issued back to back: the host never waits for a frame (no regions
    are asked for), expiry and a scene cut included; every tensor of every frame is cloned on the caller's stream and
    compared with the oracle at the end, and the work counters of the last frame are read once everything is done."""
    layers = synth.vgg16()[:10]
    T, H, W = 9, 96, 96
    videos = np.stack([synth.panning_video(6100 + s, n_frames=T, H=H, W=W, fg=((24, 24),), margin=32) for s in range(n_streams)])
    ws, bs = synth.he_weights(layers, 1, bias_scale=0.05)
    dt = binding.DC_BF16 if bf16 else binding.DC_F32
    r = binding.StackRunner(layers, ws, bs, n_streams, H, W, 3, block=16, radius=8, dtype=dt, expiry=4, device_plan=True)
    refs = [oracle.Stream(layers, ws, bs, H, W, 3, block=16, radius=8, bf16=bf16, expiry=4) for _ in range(n_streams)]
    dv = torch.from_numpy(np.ascontiguousarray(videos.transpose(1, 0, 2, 3, 4))).to(DEV)
    torch.cuda.synchronize()
    kept = []
    for t in range(T):
        if t == 6:
            r.reset()
        kept.append([x.clone() for x in r.step(dv[t])])
    torch.cuda.synchronize()
    tol = 2e-2 if bf16 else 1e-4
    last_blocks = 0
    for t in range(T):
        for s in range(n_streams):
            if t == 6:
                refs[s].reset()
            want = refs[s].step(videos[s, t])
            for ti in range(1, len(layers) + 1):
                assert _rel_err(kept[t][ti][s].float().cpu().numpy(), want["tensors"][ti]) <= tol, (t, s, ti)
            if t == T - 1:
                assert not want["full"]
                last_blocks += int(want["match"]["mask"].sum())
    assert r.read_stats().n_reusable_blocks == last_blocks


@pytest.mark.parametrize("net,size,bf16", [("vgg16", 96, False), ("resnet", 64, True)])
def test_overlap_modes_give_identical_tensors(net, size, bf16):
    """Two frames in flight, matching on a second stream only, and everything on the caller's stream run the
    same kernels with the same plans: every tensor of every frame must be bit-identical, also when the frames
    are issued back to back without any synchronisation in between (Section 7.6: asynchronous stages)."""
    H = W = size
    if net == "vgg16":
        layers = synth.vgg16()
        ws, bs = synth.he_weights(layers, 3, bias_scale=0.05)
    else:
        layers = synth.resnet50_trunk()[:24]       # stem, pool, the first two bottleneck blocks
        ws, bs = synth.he_weights(layers, 3, bias_scale=0.05, residual_scale=0.5)
    T = 14
    video = torch.from_numpy(synth.panning_video(77, n_frames=T, H=H, W=W, fg=((24, 24), (16, 32)))).to(DEV)
    frames = [video[t:t + 1].contiguous() for t in range(T)]
    torch.cuda.synchronize()
    dt = binding.DC_BF16 if bf16 else binding.DC_F32
    results = {}
    for mode, kw in (("pipeline", dict(overlap=True, pipeline=True)), ("overlap", dict(overlap=True, pipeline=False)),
                     ("plain", dict(overlap=False))):
        print(f"[overlap modes] {net} {mode}", flush=True)
        runner = binding.StackRunner(layers, ws, bs, 1, H, W, 3, block=16, radius=16, dtype=dt, expiry=5, **kw)
        kept = []
        for stop in (3, 8, T):                        # the tensors are read when a run of frames has drained
            runner.reset()
            for t in range(stop):
                tensors = runner.step(frames[t])      # no synchronisation between the frames of a run
            torch.cuda.synchronize()
            kept.append([x.clone() for x in tensors])
        results[mode] = kept
        del runner
    for mode in ("overlap", "plain"):
        for f, (a, b) in enumerate(zip(results["pipeline"], results[mode])):
            for i, (x, y) in enumerate(zip(a, b)):
                assert torch.equal(x, y), (net, mode, f, i)


def test_pipelined_frames_with_irregular_buffer_alternation():
    """With two frames in flight the library skips the cross-stream wait for a tensor whose buffer is the one its
    work stream used last and not the previous frame's, and records no event for it; a caller that then reuses the
    previous frame's buffer after all must still get the same tensors (the library waits for the whole previous
    frame instead).  The runner's choice of the set for the tensors that are not conv outputs is overridden
    frame by frame with a pattern that holds every transition; frames are issued without synchronisation."""
    H = W = 96
    layers = synth.vgg16()
    ws, bs = synth.he_weights(layers, 3, bias_scale=0.05)
    T = 14
    video = torch.from_numpy(synth.panning_video(78, n_frames=T, H=H, W=W, fg=((24, 24), (16, 32)))).to(DEV)
    frames = [video[t:t + 1].contiguous() for t in range(T)]
    torch.cuda.synchronize()
    pattern = [0, 1, 0, 0, 1, 1, 1, 0, 1, 0, 0, 0, 1, 0]
    finals = {}
    for mode, kw in (("pipeline", dict(overlap=True, pipeline=True)), ("plain", dict(overlap=False))):
        print(f"[irregular alternation] {mode}", flush=True)
        runner = binding.StackRunner(layers, ws, bs, 1, H, W, 3, block=16, radius=16, dtype=binding.DC_F32, expiry=6, **kw)
        kept = []
        for stop in (5, 9, T):
            runner.reset()
            for t in range(stop):
                if mode == "pipeline":
                    runner.cur_other = pattern[t]
                tensors = runner.step(frames[t])
            torch.cuda.synchronize()
            kept.append([x.clone() for x in tensors])
        finals[mode] = kept
        del runner
    for f, (a, b) in enumerate(zip(finals["pipeline"], finals["plain"])):
        for i, (x, y) in enumerate(zip(a, b)):
            assert torch.equal(x, y), (f, i)


def test_pageable_host_workspace_gives_the_same_tensors():
    """The frame's plans reach the device through a kernel that reads the pinned staging buffer, or through an
    asynchronous copy when the host workspace is pageable memory: same tensors either way."""
    H = W = 64
    layers = synth.vgg16()[:7]
    ws, bs = synth.he_weights(layers, 3, bias_scale=0.05)
    T = 6
    video = torch.from_numpy(synth.panning_video(79, n_frames=T, H=H, W=W, fg=((16, 16), (8, 24)))).to(DEV)
    frames = [video[t:t + 1].contiguous() for t in range(T)]
    torch.cuda.synchronize()
    outs = {}
    for pinned in (True, False):
        print(f"[host workspace] pinned={pinned}", flush=True)
        runner = binding.StackRunner(layers, ws, bs, 1, H, W, 3, block=16, radius=16, dtype=binding.DC_F32)
        if not pinned:
            runner.ws_host = torch.empty(runner.ws_host.numel(), dtype=torch.uint8)
        kept = []
        for t in range(T):
            tensors = runner.step(frames[t])
            torch.cuda.synchronize()
            kept.append([x.clone() for x in tensors])
        assert runner.stats.n_reusable_blocks > 0
        outs[pinned] = kept
        del runner
    for a, b in zip(outs[True], outs[False]):
        for x, y in zip(a, b):
            assert torch.equal(x, y)


def test_lookahead_matching_gives_the_same_tensors():
    """Section 7.6: the matching of the next frame started one step early (dc_prefetch_match) must change
    nothing but the time at which it runs: same tensors and the same masks as without it, across cache expiry,
    a scene cut, and a look-ahead that names a frame other than the one that follows (it must be ignored)."""
    H = W = 96
    layers = synth.vgg16()[:10]
    ws, bs = synth.he_weights(layers, 3, bias_scale=0.05)
    T = 12
    video = torch.from_numpy(synth.panning_video(80, n_frames=T, H=H, W=W, fg=((24, 24), (16, 32)))).to(DEV)
    frames = [video[t:t + 1].contiguous() for t in range(T)]
    torch.cuda.synchronize()
    order = list(range(T)) + [3, 4, 5]              # a jump back: a scene cut handled by reset()
    results = {}
    for look in (False, True):
        print(f"[lookahead] {look}", flush=True)
        runner = binding.StackRunner(layers, ws, bs, 1, H, W, 3, block=16, radius=16, dtype=binding.DC_F32, expiry=5)
        kept = []
        for j, t in enumerate(order):
            if j == T:
                runner.reset()
            nxt = None
            if look and j + 1 < len(order):
                nxt = frames[order[j + 1]]
                if j == 6:
                    nxt = frames[0]                 # wrong guess: the next call must match again itself
            tensors = runner.step(frames[t], next_frames=nxt)
            torch.cuda.synchronize()
            kept.append(([x.clone() for x in tensors], runner.stats.n_reusable_blocks, runner.stats.full))
        results[look] = kept
        del runner
    assert any(not full and reusable > 0 for _, reusable, full in results[True])
    for j, ((a, ra, fa), (b, rb, fb)) in enumerate(zip(results[False], results[True])):
        assert (ra, fa) == (rb, fb), j
        for i, (x, y) in enumerate(zip(a, b)):
            assert torch.equal(x, y), (j, i)


def test_lookahead_matching_without_synchronisation():
    """The same with two frames in flight and no synchronisation between the steps."""
    H = W = 96
    layers = synth.vgg16()
    ws, bs = synth.he_weights(layers, 3, bias_scale=0.05)
    T = 14
    video = torch.from_numpy(synth.panning_video(81, n_frames=T, H=H, W=W, fg=((24, 24), (16, 32)))).to(DEV)
    frames = [video[t:t + 1].contiguous() for t in range(T)]
    torch.cuda.synchronize()
    finals = {}
    for look in (False, True):
        runner = binding.StackRunner(layers, ws, bs, 1, H, W, 3, block=16, radius=16, dtype=binding.DC_F32, expiry=6)
        kept = []
        for stop in (4, 9, T):
            runner.reset()
            for t in range(stop):
                tensors = runner.step(frames[t], next_frames=frames[t + 1] if (look and t + 1 < stop) else None)
            torch.cuda.synchronize()
            kept.append([x.clone() for x in tensors])
        finals[look] = kept
        del runner
    for a, b in zip(finals[False], finals[True]):
        for x, y in zip(a, b):
            assert torch.equal(x, y)
