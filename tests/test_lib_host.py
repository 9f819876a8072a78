"""CPU-only checks of libdeepcache.so: it loads, exports every symbol the header
declares, rejects bad arguments before touching the GPU, and its host region logic
(merge + propagation) equals the oracle bit for bit."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_1712_01670_amd import binding, synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "deepcache.h")).read()
    body = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(dc_[a-z_]+)\s*\(", body))
    assert {"dc_match_blocks", "dc_propagate_regions", "dc_cached_conv_layer", "dc_run_stack"} <= declared
    L = binding.lib()
    for name in declared:
        assert hasattr(L, name), name
    assert declared == set(binding.EXPORTS)
    assert L.dc_status_string(0) == b"ok"
    assert L.dc_status_string(-5) == b"workspace too small"


def test_no_torch_types_in_the_header():
    header = open(os.path.join(ROOT, "include", "deepcache.h")).read()
    assert "torch" not in header and "at::" not in header and "hip/" not in header


def test_argument_errors_are_reported_before_any_launch():
    L = binding.lib()
    # null pointers
    assert L.dc_match_blocks(None, None, 1, 64, 64, 3, 8, 8, 0, None, None, None, None, None, None) == -2
    one = C.c_void_p(16)  # never dereferenced: validation fails first
    assert L.dc_match_blocks(one, one, 0, 64, 64, 3, 8, 8, 0, one, one, one, one, one, None) == -1
    assert L.dc_match_blocks(one, one, 1, 64, 64, 3, 128, 8, 0, one, one, one, one, one, None) == -3
    assert L.dc_match_blocks(one, one, 1, 64, 64, 3, 8, 200, 0, one, one, one, one, one, None) == -4
    assert L.dc_match_blocks_ds(None, None, 1, 64, 64, 3, 8, 8, 1, 0, None, None, None, None, None, None) == -2
    assert L.dc_match_blocks_ds(one, one, 1, 64, 64, 3, 8, 8, 0, 0, one, one, one, one, one, None) == -1    # k_skip
    assert L.dc_match_blocks_ds(one, one, 1, 64, 64, 3, 128, 8, 1, 0, one, one, one, one, one, None) == -3  # block > frame
    assert L.dc_match_blocks_ds(one, one, 1, 64, 64, 3, 8, 20000, 1, 0, one, one, one, one, one, None) == -4
    assert L.dc_match_blocks_ds(one, one, 1, 4096, 4096, 4, 200, 8, 1, 0, one, one, one, one, one, None) == -4  # 32-bit sums
    opt = binding.MatchOptions(7, 1)
    assert L.dc_match_blocks_opt(one, one, 1, 64, 64, 3, 8, 8, C.byref(opt), 0, one, one, one, one, one, None) == -1    # method
    opt = binding.MatchOptions(0, 0)
    assert L.dc_match_blocks_opt(one, one, 1, 64, 64, 3, 8, 8, C.byref(opt), 0, one, one, one, one, one, None) == -1    # k_skip
    assert L.dc_match_blocks_opt(None, one, 1, 64, 64, 3, 8, 8, None, 0, one, one, one, one, one, None) == -2
    # look-ahead matching: handle and buffers are checked before anything is touched
    assert L.dc_prefetch_match(None, one, one, 1, 64, 64, 3, 8, 8, 0, None, one, one, one, one, one, one, 4096) == -2
    assert L.dc_prefetch_match(one, one, one, 1, 64, 64, 3, 8, 8, 0, None, one, one, one, one, None, one, 4096) == -2
    assert L.dc_prefetch_match(one, one, one, 0, 64, 64, 3, 8, 8, 0, None, one, one, one, one, one, one, 4096) == -1
    assert L.dc_prefetch_match(one, one, one, 1, 64, 4, 3, 8, 8, 0, None, one, one, one, one, one, one, 4096) == -3   # block > frame
    assert L.dc_prefetch_match(one, one, one, 1, 64, 64, 3, 8, 8, 0, None, one, one, one, one, one, one, 16) == -5
    bad = binding.layers_to_c([dict(type=0, k=3, s=0, p=1, cin=3, cout=8, relu=1, in0=0, in1=-1)])
    two = C.c_void_p(32)
    assert L.dc_torus_read(None, one, None, 2, 1, 8, 8, 4, 0, None) == -2
    assert L.dc_torus_read(one, one, None, 2, 1, 8, 8, 4, 0, None) == -1          # in place
    assert L.dc_torus_read(one, two, None, 2, 1, 8, 8, 4, 7, None) == -1          # dtype
    assert L.dc_torus_read(one, two, one, 1, 1, 8, 8, 4, 0, None) == -1           # stride below one entry
    assert L.dc_torus_read(one, two, None, 2, 70000, 8, 8, 4, 0, None) == -4      # rows beyond the grid
    assert L.dc_cached_conv_layer(bad, one, one, None, None, None, one, 1, 8, 8, None, 0, None, 0, None, 0, None) == -1
    ok = binding.layers_to_c([dict(type=0, k=3, s=1, p=1, cin=3, cout=8, relu=1, in0=0, in1=-1)])
    assert L.dc_cached_conv_layer(ok, one, one, None, None, None, one, 1, 8, 8, None, 7, None, 0, None, 0, None) == -1
    assert L.dc_cached_conv_layer(ok, None, one, None, None, None, one, 1, 8, 8, None, 0, None, 0, None, 0, None) == -2
    # packed weights exist for the layers the 3x3 stride-1 GEMM kernel takes, and are a permutation of the plain ones
    nb = C.c_size_t(1)
    assert L.dc_packed_weights_bytes(ok, 0, C.byref(nb)) == 0 and nb.value == 0
    big = binding.layers_to_c([dict(type=0, k=3, s=1, p=1, cin=32, cout=128, relu=1, in0=0, in1=-1)])
    assert L.dc_packed_weights_bytes(big, 0, C.byref(nb)) == 0 and nb.value == 128 * 9 * 32 * 4
    assert L.dc_packed_weights_bytes(big, 1, C.byref(nb)) == 0 and nb.value == 128 * 9 * 32 * 2
    odd = binding.layers_to_c([dict(type=0, k=3, s=1, p=1, cin=24, cout=128, relu=1, in0=0, in1=-1)])
    assert L.dc_packed_weights_bytes(odd, 1, C.byref(nb)) == 0 and nb.value == 0      # 48-byte channel runs
    assert L.dc_packed_weights_bytes(big, 5, C.byref(nb)) == -1
    assert L.dc_pack_conv_weights(ok, one, 0, C.c_void_p(32), None) == -3
    assert L.dc_pack_conv_weights(big, one, 0, None, None) == -2
    assert L.dc_pack_conv_weights(big, one, 0, one, None) == -1                         # in place
    # kernel ids of dc_stack_stats.layer_kernel_id name the instantiation a profiler shows
    assert binding.conv_kernel_name(64) == "conv_fast_kernel<float, 3, 16, 1, 2, 4, 1>"
    assert binding.conv_kernel_name(64 + 3 * 8 + 4) == "conv_fast_kernel<__hip_bfloat16, 3, 64, 5, 2, 4, 1>"
    assert binding.conv_kernel_name(96 + 2) == "conv_first_kernel<float, 4>"
    assert binding.conv_kernel_name(102 + 2 + 1) == "conv_stem_kernel<__hip_bfloat16, 2>"
    assert binding.conv_kernel_name(107) == "conv_stem11_kernel<__hip_bfloat16>"
    assert binding.conv_kernel_name(108) == "conv_pw_kernel<float, 2>"
    assert binding.conv_kernel_name(128) == "conv_pw_kernel<__hip_bfloat16, 4>"
    assert binding.conv_kernel_name(110 + 3) == "conv_fast_kernel<__hip_bfloat16, 3, 32, 4, 4, 2, 4>"
    assert binding.conv_kernel_name(110 + 8 + 4) == "conv_fast_kernel<__hip_bfloat16, 3, 64, 1, 4, 2, 2>"
    assert binding.conv_kernel_name(126) == "conv_regw_kernel<2, 2, false>"
    assert binding.conv_kernel_name(130) == "conv_regw_kernel<2, 2, true>"
    assert binding.conv_kernel_name(129) == "conv_fast_kernel<__hip_bfloat16, 3, 32, 3, 6, 2, 4>"
    with pytest.raises(binding.DcError):
        binding.conv_kernel_name(131)
    # overlapping rectangles are rejected
    regs, keep = binding._alloc_regions(1, 2)
    keep[0][0] = binding.Rect(0, 0, 4, 4)
    keep[0][1] = binding.Rect(2, 2, 4, 4)
    regs[0].n = 2
    assert L.dc_cached_conv_layer(ok, one, one, None, None, one, C.c_void_p(32), 1, 8, 8, regs, 0, one, 1 << 20, one,
                                  1 << 20, None) == -3
    # a layer table whose channel counts do not chain
    layers = synth.tiny_net()
    layers[1] = dict(layers[1], cin=17)
    with pytest.raises(binding.DcError) as e:
        binding.dc_propagate_regions(layers, 64, 64, 8, np.ones((8, 8), np.uint8), 0, 0)
    assert e.value.status == -3
    with pytest.raises(binding.DcError) as e:
        binding.dc_propagate_regions(synth.tiny_net(), 64, 64, 8, np.ones((4, 8), np.uint8), 0, 0)
    assert e.value.status == -3
    with pytest.raises(binding.DcError) as e:
        binding.dc_propagate_regions(synth.tiny_net(), 64, 64, 8, np.ones((8, 8), np.uint8), 0, 0, cap=0)
    assert e.value.status in (-2, -6)


def _compare(oracle, layers, H, W, B, mask, mx, my, extend=False):
    got = binding.dc_propagate_regions(layers, H, W, B, mask, mx, my, extend_borders=extend)
    r0 = oracle.merge_blocks(mask, B)
    want = oracle.propagate(layers, H, W, r0, mx, my, extend_borders=extend)
    for t in range(len(layers) + 1):
        assert got[t]["rects"].tolist() == want["rects"][t].tolist(), t
        assert list(got[t]["dxy"]) == want["dxy"][t].tolist(), t
        assert got[t]["cum_stride"] == want["cum_stride"][t]
        assert list(got[t]["hw"]) == want["hw"][t].tolist()


@pytest.mark.parametrize("net,H,W,B", [("tiny", 64, 64, 8), ("vgg", 224, 224, 16), ("resnet", 224, 224, 16),
                                       ("darknet", 416, 416, 16), ("vgg", 100, 132, 10)])
def test_host_regions_equal_oracle(oracle, net, H, W, B):
    layers = dict(tiny=synth.tiny_net, vgg=synth.vgg16, resnet=synth.resnet50_trunk, darknet=synth.darknet19)[net]()
    rng = np.random.default_rng(len(net) * 100 + H)
    gh, gw = H // B, W // B
    for trial in range(25):
        dens = rng.choice([0.0, 0.3, 0.7, 0.9, 0.97, 1.0])
        mask = (rng.random((gh, gw)) < dens).astype(np.uint8)
        if trial % 3 == 0:   # a solid region with a hole: the typical panning-background case
            mask[:] = 1
            y, x = int(rng.integers(0, gh - 2)), int(rng.integers(0, gw - 2))
            mask[y:y + 3, x:x + 2] = 0
        mx, my = int(rng.integers(-B, B + 1)), int(rng.integers(-B, B + 1))
        _compare(oracle, layers, H, W, B, mask, mx, my)
    _compare(oracle, layers, H, W, B, np.ones((gh, gw), np.uint8), 0, 0)
    _compare(oracle, layers, H, W, B, np.zeros((gh, gw), np.uint8), 3, -2)


def _random_layers(rng, H, W):
    """A random layer table: convs and pools with assorted kernels / strides / paddings, ReLUs, and adds of
    same-shaped tensors, kept valid (every map stays at least as large as the next kernel)."""
    layers, shapes = [], [(H, W, 8)]
    for _ in range(int(rng.integers(3, 9))):
        a = len(shapes) - 1
        h, w, c = shapes[a]
        kind = rng.choice(["conv", "conv", "conv", "pool", "relu", "add"])
        if kind == "add":
            same = [t for t in range(len(shapes) - 1) if shapes[t] == shapes[a]]
            if not same:
                kind = "relu"
            else:
                layers.append(dict(type=synth.ADD, k=1, s=1, p=0, cin=c, cout=c, relu=int(rng.integers(0, 2)), in0=a,
                                   in1=int(rng.choice(same))))
                shapes.append((h, w, c))
                continue
        if kind == "relu":
            layers.append(dict(type=synth.RELU, k=1, s=1, p=0, cin=c, cout=c, relu=1, in0=a, in1=-1))
            shapes.append((h, w, c))
            continue
        k = int(rng.choice([1, 2, 3, 3, 5, 7]))
        s_ = int(rng.choice([1, 1, 2, 3]))
        p_ = int(rng.integers(0, k))
        if h + 2 * p_ < k or w + 2 * p_ < k:
            k, s_, p_ = 1, 1, 0
        ho, wo = (h + 2 * p_ - k) // s_ + 1, (w + 2 * p_ - k) // s_ + 1
        if kind == "pool":
            layers.append(dict(type=synth.MAXPOOL, k=k, s=s_, p=p_, cin=c, cout=c, relu=0, in0=a, in1=-1))
            shapes.append((ho, wo, c))
        else:
            co = int(rng.choice([8, 16]))
            layers.append(dict(type=synth.CONV, k=k, s=s_, p=p_, cin=c, cout=co, relu=1, in0=a, in1=-1))
            shapes.append((ho, wo, co))
    return layers


def test_host_regions_equal_oracle_on_random_layer_tables(oracle):
    rng = np.random.default_rng(2024)
    for trial in range(60):
        H, W, B = int(rng.integers(20, 90)), int(rng.integers(20, 90)), int(rng.choice([4, 5, 8]))
        layers = _random_layers(rng, H, W)
        gh, gw = H // B, W // B
        mask = (rng.random((gh, gw)) < rng.choice([0.5, 0.8, 0.95, 1.0])).astype(np.uint8)
        mx, my = int(rng.integers(-2 * B, 2 * B + 1)), int(rng.integers(-2 * B, 2 * B + 1))
        _compare(oracle, layers, H, W, B, mask, mx, my)


def _random_layers_all_types(rng, H, W):
    """As _random_layers, with LRN (both windows), average pooling, concats of 2-4 earlier tensors of the current
    spatial size, and sometimes a fully-connected / softmax tail."""
    layers, shapes = [], [(H, W, 8)]
    for _ in range(int(rng.integers(4, 11))):
        a = len(shapes) - 1
        h, w, c = shapes[a]
        kind = rng.choice(["conv", "conv", "pool", "avg", "lrn", "lrnw", "concat", "concat", "relu"])
        if kind == "concat":
            same = [t for t in range(1, len(shapes)) if shapes[t][:2] == (h, w)]
            if len(same) < 2:
                kind = "conv"
            else:
                m = int(rng.integers(2, min(4, len(same)) + 1))
                ins = [int(t) for t in rng.choice(same, size=m, replace=False)]
                cs = [shapes[t][2] for t in ins]
                layers.append(synth._concat(cs, ins))
                shapes.append((h, w, sum(cs)))
                continue
        if kind in ("lrn", "lrnw"):
            size = int(rng.choice([1, 3, 5]))
            layers.append(synth._lrn(c, size, a, within=(kind == "lrnw")))
            shapes.append((h, w, c))
            continue
        if kind == "relu":
            layers.append(dict(type=synth.RELU, k=1, s=1, p=0, cin=c, cout=c, relu=1, in0=a, in1=-1))
            shapes.append((h, w, c))
            continue
        k = int(rng.choice([1, 2, 3, 3, 5]))
        s_ = int(rng.choice([1, 1, 2]))
        p_ = int(rng.integers(0, k))
        if h + 2 * p_ < k or w + 2 * p_ < k:
            k, s_, p_ = 1, 1, 0
        ho, wo = (h + 2 * p_ - k) // s_ + 1, (w + 2 * p_ - k) // s_ + 1
        if kind in ("pool", "avg"):
            layers.append((synth._pool if kind == "pool" else synth._avgpool)(c, k, s_, p_, a))
            shapes.append((ho, wo, c))
        else:
            co = int(rng.choice([8, 16]))
            layers.append(synth._conv(c, co, k, s_, p_, True, a))
            shapes.append((ho, wo, co))
    if rng.random() < 0.5:
        c = shapes[-1][2]
        layers.append(synth._fc(c, 12, True, len(layers)))
        layers.append(dict(type=synth.RELU, k=1, s=1, p=0, cin=12, cout=12, relu=1, in0=len(layers), in1=-1))
        layers.append(synth._softmax(12, len(layers)))
    return layers


def test_host_regions_equal_oracle_with_every_layer_type(oracle):
    rng = np.random.default_rng(77)
    seen = set()
    for trial in range(80):
        H, W, B = int(rng.integers(24, 90)), int(rng.integers(24, 90)), int(rng.choice([4, 5, 8]))
        layers = _random_layers_all_types(rng, H, W)
        seen |= {L["type"] for L in layers}
        gh, gw = H // B, W // B
        mask = (rng.random((gh, gw)) < rng.choice([0.6, 0.9, 1.0])).astype(np.uint8)
        mx, my = int(rng.integers(-B, B + 1)), int(rng.integers(-B, B + 1))
        _compare(oracle, layers, H, W, B, mask, mx, my)
    assert seen >= {synth.CONV, synth.MAXPOOL, synth.AVGPOOL, synth.LRN, synth.CONCAT, synth.FC, synth.SOFTMAX}
    for net, H in ((synth.alexnet(), 227), (synth.resolve_global_pooling(synth.googlenet(), 224, 224, 3), 224)):
        gh = H // 16
        mask = np.ones((gh, gh), np.uint8)
        mask[3:5, 2:9] = 0
        _compare(oracle, net, H, H, 16, mask, 5, -3)


def test_layer_table_validation_of_the_new_types():
    L = binding.lib()
    one = C.c_void_p(16)
    regs, keep = binding._alloc_regions(4, 8)
    mask = np.ones((4, 4), np.uint8)

    def status(layers):
        return L.dc_propagate_regions(binding.layers_to_c(layers), len(layers), 32, 32, 8, mask.ctypes.data_as(C.c_void_p),
                                      4, 4, 0, 0, regs)
    conv = synth._conv(3, 8, 3, 1, 1, True, 0)
    assert status([conv, synth._lrn(8, 5, 1)]) == 0
    assert status([conv, synth._lrn(8, 4, 1)]) == -1                                    # even window
    assert status([conv, synth._lrn(16, 5, 1)]) == -3                                   # channel mismatch
    assert status([conv, conv, synth._concat([8, 8], [1, 2])]) == 0
    assert status([conv, conv, synth._concat([8, 4], [1, 2])]) == -3                    # wrong channel sum
    assert status([conv, conv, dict(synth._concat([8, 8], [1, 2]), in2=-1, in3=1)]) == -3   # in3 without in2
    assert status([conv, synth._pool(8, 2, 2, 0, 1), synth._concat([8, 8], [1, 2])]) == -3   # sizes differ
    assert status([conv, synth._fc(8, 10, False, 1), synth._softmax(10, 2)]) == 0
    assert status([conv, synth._fc(4, 10, False, 1)]) == -3
    assert status([conv, synth._avgpool(8, 3, 2, 3, 1)]) == -1                          # padding >= kernel


def test_host_regions_with_the_border_case_equal_oracle(oracle):
    rng = np.random.default_rng(99)
    grew = 0
    for trial in range(60):
        B = int(rng.choice([4, 8]))
        H, W = B * int(rng.integers(4, 12)), B * int(rng.integers(4, 12)) + int(rng.integers(0, 3))
        layers = _random_layers_all_types(rng, H, W) if trial % 2 else _random_layers(rng, H, W)
        gh, gw = H // B, W // B
        mask = (rng.random((gh, gw)) < rng.choice([0.8, 0.95, 1.0])).astype(np.uint8)
        mx, my = (0, 0) if trial % 3 else (int(rng.integers(-B, B + 1)), int(rng.integers(-B, B + 1)))
        _compare(oracle, layers, H, W, B, mask, mx, my, extend=True)
        if (mx, my) == (0, 0):
            r0 = oracle.merge_blocks(mask, B)
            a = oracle.propagate(layers, H, W, r0, 0, 0)
            b = oracle.propagate(layers, H, W, r0, 0, 0, extend_borders=True)
            area = lambda pr: sum(int(r[2]) * int(r[3]) for t in pr["rects"] for r in t)
            assert area(b) >= area(a)
            grew += area(b) > area(a)
    assert grew > 10


def test_reuse_sweep_generator_hits_its_target_ratio(oracle):
    """The sweep's moving noise rectangles are sized so that the measured share of reusable blocks (Step 4 of the
    oracle's matcher) is the target within 3 points; zero means fresh noise, and the entering column caps 0.95."""
    from paper_1712_01670_amd import synth
    for i, target in enumerate((0.0, 0.25, 0.5, 0.75, 0.95)):
        v = synth.reuse_sweep_video(4000 + i, target, n_frames=8, cut_at=4)
        got = []
        for f in (1, 2, 3, 5, 6):
            m = oracle.match_blocks(v[f], v[f - 1], 16, 16, synth.max_block_ssd(16))
            got.append(float(m["mask"].mean()))
            if target > 0:
                assert m["gmv"].tolist() == [2, 0]
        assert abs(np.mean(got) - target) <= 0.03, (target, got)
    # across the cut nothing matches
    v = synth.reuse_sweep_video(4003, 0.75, n_frames=8, cut_at=4)
    assert oracle.match_blocks(v[4], v[3], 16, 16, synth.max_block_ssd(16))["mask"].sum() == 0
