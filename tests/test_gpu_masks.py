"""GPU parity of the exact reuse maps (dc_propagate_masks: Section 5's propagation per pixel) against the oracle's
oc_propagate_masks: every bit of every tensor's map and every source offset, on random block masks and motions."""
import numpy as np
import pytest
import torch

from paper_1712_01670_amd import binding, synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _mixed_stack():
    C_ = lambda k, s, p, i: dict(type=synth.CONV, k=k, s=s, p=p, cin=4, cout=4, relu=1, in0=i, in1=-1)
    return [C_(3, 1, 1, 0), C_(5, 1, 2, 1),
            dict(type=synth.MAXPOOL, k=2, s=2, p=0, cin=4, cout=4, relu=0, in0=2, in1=-1),
            C_(3, 1, 1, 3), C_(1, 1, 0, 3),
            dict(type=synth.ADD, k=1, s=1, p=0, cin=4, cout=4, relu=1, in0=4, in1=5),
            dict(type=synth.LRN, k=3, s=1, p=0, cin=4, cout=4, relu=0, in0=6, in1=-1, within=1, alpha=1e-4, beta=0.75, kappa=1.0),
            C_(3, 2, 1, 7),
            dict(type=synth.MAXPOOL, k=3, s=2, p=1, cin=4, cout=4, relu=0, in0=8, in1=-1),
            dict(type=synth.RELU, k=1, s=1, p=0, cin=4, cout=4, relu=0, in0=9, in1=-1),
            C_(7, 1, 3, 10),
            dict(type=synth.CONCAT, k=1, s=1, p=0, cin=8, cout=8, relu=0, in0=10, in1=11, in2=-1, in3=-1),
            dict(type=synth.CONV, k=3, s=3, p=0, cin=8, cout=4, relu=0, in0=12, in1=-1),     # word path in two 64-column pieces
            dict(type=synth.CONV, k=3, s=9, p=1, cin=4, cout=4, relu=0, in0=7, in1=-1)]      # a stride only the bit-by-bit path takes


def _check(oracle, layers, H, W, Ch, block, n, seed, density=0.8, max_motion=9):
    rng = np.random.default_rng(seed)
    gh, gw = H // block, W // block
    bm = (rng.random((n, gh, gw)) < density).astype(np.uint8)
    bm[0] = 1                                              # one stream with everything matched
    gmv = rng.integers(-max_motion, max_motion + 1, (n, 2)).astype(np.int32)
    gmv[0] = 0
    if n > 2:
        gmv[2] = 0                                         # and one that did not move with a ragged mask
    for ext in (False, True):
        print(f"[masks] {len(layers)} layers {H}x{W} block {block} streams {n} border case {ext}", flush=True)
        got, dxy = binding.dc_propagate_masks(layers, H, W, Ch, block, torch.from_numpy(bm).to(DEV), torch.from_numpy(gmv).to(DEV), ext)
        for s in range(n):
            want = oracle.propagate_masks(layers, H, W, bm[s], block, int(gmv[s, 0]), int(gmv[s, 1]), extend_borders=ext)
            assert np.array_equal(dxy[s], want["dxy"]), s
            for t, m in enumerate(want["masks"]):
                assert np.array_equal(got[t][s], m.astype(bool)), (s, t, ext)
        assert got[1][0].any()


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_mixed_stack_random_masks(oracle, seed):
    _check(oracle, _mixed_stack(), 70, 92, 4, 8, 5, seed)                     # remainder strips on both axes, 35-bit rows
    _check(oracle, _mixed_stack(), 64, 256, 4, 16, 3, 10 + seed, density=0.95, max_motion=20)   # rows of several words


def test_model_stacks(oracle):
    _check(oracle, synth.vgg16(), 224, 224, 3, 16, 4, 20)
    _check(oracle, synth.resnet50_trunk(), 224, 224, 3, 16, 3, 21, density=0.9)
    _check(oracle, synth.resolve_global_pooling(synth.googlenet(n_classes=24, width=0.25), 224, 224, 3), 224, 224, 3, 16, 2, 22, density=0.9)
    _check(oracle, synth.alexnet(n_classes=40, width=0.25), 227, 227, 3, 10, 3, 23, density=0.9, max_motion=12)
    _check(oracle, synth.darknet19(), 416, 416, 3, 16, 2, 24, density=0.9, max_motion=16)
    _check(oracle, synth.dave_orig(), 66, 200, 3, 10, 3, 25, density=0.9)
    _check(oracle, synth.factorised_net(8), 96, 128, 3, 8, 4, 26, density=0.9)      # kernels that are not square, dilation


def test_large_frame_maps_built_in_the_workspace(oracle):
    """A frame whose bitmaps (more than 128 KB per stream) do not fit the workgroup's LDS: the same maps, built in the
    workspace instead."""
    _check(oracle, _mixed_stack()[:6], 1000, 1100, 4, 16, 2, 30, density=0.9, max_motion=20)
