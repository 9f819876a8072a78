"""The entry point that allocates nothing (dc_cached_conv_layer_noalloc: the library's static device scratch, rectangles
as kernel arguments, unit list built on the GPU) against dc_cached_conv_layer with caller workspaces: same inputs,
same outputs, on two calls in a row, the second with a smaller input; then its size limits."""
import ctypes as C

import numpy as np
import pytest
import torch

from paper_1712_01670_amd import binding, synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _case(seed, n, H, W, cin, cout, bf16, k=3, p=1):
    rng = np.random.default_rng(seed)
    td = torch.bfloat16 if bf16 else torch.float32
    layer = dict(type=synth.CONV, k=k, s=1, p=p, cin=cin, cout=cout, relu=1, in0=0, in1=-1)
    x = torch.from_numpy(rng.standard_normal((n, H, W, cin)).astype(np.float32)).to(DEV).to(td)
    w = torch.from_numpy((rng.standard_normal((cout, k, k, cin)) * np.sqrt(2.0 / (cin * k * k))).astype(np.float32)).to(DEV).to(td)
    b = torch.from_numpy(rng.standard_normal(cout).astype(np.float32) * 0.1).to(DEV)
    prev = torch.from_numpy(rng.standard_normal((n, H, W, cout)).astype(np.float32)).to(DEV).to(td)
    regions = []
    for s in range(n):      # disjoint rectangles on a coarse grid, a source offset that keeps the source inside the map
        dx, dy = int(rng.integers(-2, 3)), int(rng.integers(-2, 3))
        rects = []
        gy, gx = max(H // 3, 1), max(W // 3, 1)
        for cy in range(3):
            for cx in range(3):
                if rng.random() < 0.6:
                    x0, y0 = cx * gx + int(rng.integers(0, 3)), cy * gy + int(rng.integers(0, 3))
                    x1, y1 = min((cx + 1) * gx - int(rng.integers(0, 3)), W), min((cy + 1) * gy - int(rng.integers(0, 3)), H)
                    x0, x1 = max(x0, -dx, 0), min(x1, W - dx, W)
                    y0, y1 = max(y0, -dy, 0), min(y1, H - dy, H)
                    if x1 > x0 and y1 > y0:
                        rects.append([x0, y0, x1 - x0, y1 - y0])
        regions.append((np.array(rects, np.int32).reshape(-1, 4), (dx, dy)))
    return layer, x, w, b, prev, regions


def _compare(layer, x, w, b, prev, regions, bf16):
    want = binding.dc_cached_conv_layer(layer, x, w, b, prev, regions)
    got = torch.full_like(want, float("nan"))
    binding.dc_cached_conv_layer_noalloc(layer, x, w, b, got, prev, regions)
    torch.cuda.synchronize()
    a, g = want.float().cpu().numpy(), got.float().cpu().numpy()
    assert np.isfinite(g).all()
    tol = 2e-2 if bf16 else 1e-4
    assert np.abs(a - g).max() <= tol * max(np.abs(a).max(), 1e-30)
    if regions is not None:     # reusable pixels are bit copies of the cache on both sides
        n, H, W, _ = a.shape
        for s, (rects, _) in enumerate(regions):
            for (rx, ry, rw, rh) in rects:
                assert np.array_equal(a[s, ry:ry + rh, rx:rx + rw], g[s, ry:ry + rh, rx:rx + rw])
        assert sum(len(r[0]) for r in regions) > 0


@pytest.mark.parametrize("bf16", [False, True])
def test_no_alloc_conv_layer_two_calls_in_a_row(bf16):
    print("[no_alloc] first call: 3 streams 40x52, 32 -> 64 channels, bf16 =", bf16, flush=True)
    _compare(*_case(1, 3, 40, 52, 32, 64, bf16), bf16)
    print("[no_alloc] second call, smaller: 2 streams 18x22", flush=True)
    _compare(*_case(2, 2, 18, 22, 32, 64, bf16), bf16)
    print("[no_alloc] every pixel computed, deep K on a small map (partial sums in the static scratch)", flush=True)
    layer, x, w, b, prev, _ = _case(3, 2, 14, 14, 256, 128, bf16)
    _compare(layer, x, w, b, None, None, bf16)
    print("[no_alloc] 1x1 layer with rectangles", flush=True)
    _compare(*_case(4, 2, 20, 28, 64, 64, bf16, k=1, p=0), bf16)


def test_no_alloc_conv_layer_rejects_what_does_not_fit():
    L = binding.lib()
    layer, x, w, b, prev, regions = _case(5, 2, 16, 16, 32, 64, False)
    out = torch.empty_like(prev)
    Lc = binding.layers_to_c([layer])
    regs, keep = binding._alloc_regions(40, 130)
    for i in range(40):
        regs[i].n = 0
    call = lambda n, H, W: L.dc_cached_conv_layer_noalloc(Lc, binding._ptr(x), binding._ptr(w), None, None, binding._ptr(prev),
                                                          binding._ptr(out), n, H, W, regs, 0, None)
    assert call(33, 16, 16) == -6                      # more streams than the kernel arguments hold
    regs[0].n = 129
    for j in range(129):
        keep[0][j] = binding.Rect(0, 0, 1, 1)
    assert call(2, 16, 16) in (-3, -6)                 # overlapping rectangles are refused first, else too many
    for j in range(129):
        keep[0][j] = binding.Rect(j % 16, j // 16, 1, 1)
    assert call(2, 16, 16) == -6                       # 129 rectangles
    regs[0].n = 0
    assert call(32, 1600, 1600) == -5                  # a plan beyond the static scratch (nothing is touched)
    assert call(2, 16, 16) == 0
    torch.cuda.synchronize()
