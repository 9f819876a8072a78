"""Pins for the oracle's cache-aware layers and whole-stack behaviour (Section 5
"Reuse", Section 3 workflow): library convolution / pooling, bf16 bit patterns, and
the three invariants: zero reuse == full forward, identical frames -> full reuse,
exact shifted copy == full forward on reused pixels."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

from paper_1712_01670_amd import synth


def _torch_conv(x, w, b, s, p, relu):
    xt = torch.from_numpy(x.astype(np.float64)).permute(2, 0, 1)[None]
    wt = torch.from_numpy(w.astype(np.float64)).permute(0, 3, 1, 2)
    bt = None if b is None else torch.from_numpy(b.astype(np.float64))
    y = F.conv2d(xt, wt, bt, stride=s, padding=p)
    if relu:
        y = y.clamp_min(0)
    return y[0].permute(1, 2, 0).numpy()


@pytest.mark.parametrize("k,s,p,cin,cout,relu", [
    (3, 1, 1, 3, 8, True), (3, 2, 1, 5, 7, False), (1, 1, 0, 6, 4, True), (1, 2, 0, 6, 4, False),
    (7, 2, 3, 3, 5, True), (5, 1, 0, 2, 3, False), (3, 1, 0, 4, 4, True)])
def test_conv_matches_library(oracle, k, s, p, cin, cout, relu):
    rng = np.random.default_rng(k * 100 + s * 10 + p)
    x = rng.standard_normal((13, 17, cin)).astype(np.float32)
    w = rng.standard_normal((cout, k, k, cin)).astype(np.float32)
    b = rng.standard_normal(cout).astype(np.float32)
    got = oracle.conv_cached(x, w, b, k, s, p, relu)
    want = _torch_conv(x, w, b, s, p, relu)
    assert got.shape == want.shape
    np.testing.assert_allclose(got, want, rtol=1e-6, atol=1e-6)
    got = oracle.conv_cached(x, w, None, k, s, p, relu)
    np.testing.assert_allclose(got, _torch_conv(x, w, None, s, p, relu), rtol=1e-6, atol=1e-6)


def test_conv_identity_kernel(oracle):
    rng = np.random.default_rng(0)
    x = rng.standard_normal((6, 7, 4)).astype(np.float32)
    w = np.zeros((4, 3, 3, 4), np.float32)
    for c in range(4):
        w[c, 1, 1, c] = 1.0
    assert np.array_equal(oracle.conv_cached(x, w, None, 3, 1, 1, False), x)
    # one-hot tap at (ky=0,kx=2) reads the pixel up-right; zero padding outside
    w[:] = 0
    for c in range(4):
        w[c, 0, 2, c] = 1.0
    y = oracle.conv_cached(x, w, None, 3, 1, 1, False)
    want = np.zeros_like(x)
    want[1:, :-1] = x[:-1, 1:]
    assert np.array_equal(y, want)


@pytest.mark.parametrize("k,s,p", [(2, 2, 0), (3, 2, 1), (3, 1, 1)])
def test_maxpool_matches_library(oracle, k, s, p):
    rng = np.random.default_rng(k)
    x = rng.standard_normal((11, 14, 5)).astype(np.float32)
    got = oracle.maxpool(x, k, s, p)
    want = F.max_pool2d(torch.from_numpy(x).permute(2, 0, 1)[None], k, s, p)[0].permute(1, 2, 0).numpy()
    assert np.array_equal(got, want)


def test_bf16_rounding_bit_patterns(oracle):
    def bits(f):
        return np.array([f], np.float32).view(np.uint32)[0]

    def frombits(u):
        return np.array([u], np.uint32).view(np.float32)[0]
    cases = [
        (0x3F800000, 0x3F800000),  # 1.0 exact
        (0x3F808000, 0x3F800000),  # tie, even mantissa below -> stays
        (0x3F818000, 0x3F820000),  # tie, odd mantissa -> rounds up to even
        (0x3F808001, 0x3F810000),  # just above the tie
        (0x3F807FFF, 0x3F800000),  # just below the tie
        (0xBF818000, 0xBF820000),  # sign is untouched
        (0x3FFFFFFF, 0x40000000),  # mantissa carry into the exponent
        (0x00000000, 0x00000000),
    ]
    for u, want in cases:
        got = bits(oracle.round_bf16(np.array([frombits(u)], np.float32))[0])
        assert got == want, (hex(u), hex(got), hex(want))
    rng = np.random.default_rng(2)
    a = (rng.standard_normal(20000) * 10 ** rng.uniform(-6, 6, 20000)).astype(np.float32)
    want = torch.from_numpy(a).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(oracle.round_bf16(a), want)


def test_frame_to_tensor_is_exact_in_bf16(oracle):
    f = np.arange(256, dtype=np.uint8).reshape(16, 16, 1)
    t = oracle.frame_to_tensor(f)
    assert np.array_equal(t.ravel(), (np.arange(256) - 128) / 128.0)
    assert np.array_equal(oracle.round_bf16(t), t)


def test_cached_conv_copies_exactly_where_masked(oracle):
    rng = np.random.default_rng(4)
    x = rng.standard_normal((10, 12, 3)).astype(np.float32)
    w = rng.standard_normal((5, 3, 3, 3)).astype(np.float32)
    cache = rng.standard_normal((10, 12, 5)).astype(np.float32)
    mask = np.zeros((10, 12), np.uint8)
    mask[2:6, 3:9] = 1
    full = oracle.conv_cached(x, w, None, 3, 1, 1, True)
    out = oracle.conv_cached(x, w, None, 3, 1, 1, True, cache_prev=cache, mask=mask, dxy=(2, -1))
    m = mask.astype(bool)
    assert np.array_equal(out[~m], full[~m])
    # out[y][x] = cache[y-1][x+2] on the mask
    assert np.array_equal(out[2:6, 3:9], cache[1:5, 5:11])


def _run_video(oracle, layers, frames, block, radius, bf16=False, expiry=0, seed=1, bias_scale=0.1, exact_masks=False,
               cache_pool_add=False, no_reuse=None):
    ws, bs = synth.he_weights(layers, seed, bias_scale=bias_scale)
    H, W, C = frames[0].shape
    st = oracle.Stream(layers, ws, bs, H, W, C, block=block, radius=radius, bf16=bf16, expiry=expiry, exact_masks=exact_masks,
                       cache_pool_add=cache_pool_add, no_reuse=no_reuse)
    outs = []
    for f in frames:
        r = st.step(f)
        r["tensors"] = [t.copy() for t in r["tensors"]]
        outs.append(r)
    return outs, (ws, bs)


def _full_forward(oracle, layers, ws, bs, frame, bf16=False):
    H, W, C = frame.shape
    st = oracle.Stream(layers, ws, bs, H, W, C, bf16=bf16)
    return [t.copy() for t in st.step(frame)["tensors"]]


def test_invariant_zero_reuse_is_full_forward(oracle):
    # two unrelated frames: no block passes -> empty region lists -> bit-identical to full forward
    rng = np.random.default_rng(6)
    layers = synth.tiny_net()
    frames = [rng.integers(0, 256, (64, 64, 3)).astype(np.uint8) for _ in range(2)]
    outs, (ws, bs) = _run_video(oracle, layers, frames, 8, 8)
    assert outs[1]["match"]["n_pass"] == 0 and all(len(r) == 0 for r in outs[1]["rects"])
    full = _full_forward(oracle, layers, ws, bs, frames[1])
    for a, b in zip(outs[1]["tensors"], full):
        assert np.array_equal(a, b)


def test_invariant_identical_frames_full_reuse(oracle):
    rng = np.random.default_rng(8)
    layers = synth.tiny_net()
    f = rng.integers(0, 256, (64, 64, 3)).astype(np.uint8)
    outs, _ = _run_video(oracle, layers, [f, f], 8, 8)
    m = outs[1]["match"]
    assert m["mask"].all() and m["gmv"].tolist() == [0, 0]
    assert outs[1]["rects"][0].tolist() == [[0, 0, 64, 64]]
    # the padding ring is lost layer by layer (no border extension), the rest is reused
    assert outs[1]["rects"][1].tolist() == [[1, 1, 62, 62]]
    for a, b in zip(outs[0]["tensors"], outs[1]["tensors"]):
        assert np.array_equal(a, b)


@pytest.mark.parametrize("bf16", [False, True])
def test_invariant_exact_shift_equals_full_forward(oracle, bf16):
    # content moved by a multiple of the total stride (2): every reused value was produced by
    # the same arithmetic on identical inputs, so the cached frame equals the full forward.
    layers = synth.tiny_net()
    f1, f2 = synth.shifted_pair(10, 64, 64, (4, -2))
    outs, (ws, bs) = _run_video(oracle, layers, [f1, f2], 8, 8, bf16=bf16)
    m = outs[1]["match"]
    assert m["gmv"].tolist() == [-4, 2] and m["mask"].sum() >= 40
    full = _full_forward(oracle, layers, ws, bs, f2, bf16=bf16)
    reused = 0
    for t in range(1, len(layers) + 1):
        assert np.array_equal(outs[1]["tensors"][t], full[t]), t
        reused += sum(int(w) * int(h) for _, _, w, h in outs[1]["rects"][t])
    assert reused > 1000      # the test is not vacuous: many pixels were copied


def test_misaligned_shift_is_exact_only_through_stride_one(oracle):
    layers = synth.tiny_net()
    f1, f2 = synth.shifted_pair(12, 64, 64, (3, -2))
    outs, (ws, bs) = _run_video(oracle, layers, [f1, f2], 8, 8)
    full = _full_forward(oracle, layers, ws, bs, f2)
    assert np.array_equal(outs[1]["tensors"][1], full[1])          # stride 1: exact
    assert not np.array_equal(outs[1]["tensors"][2], full[2])      # stride 2, dx=3: approximate


def test_cached_values_really_come_from_cache(oracle):
    # with sensor noise the reused pixels differ from a recomputation but equal the shifted cache
    layers = synth.tiny_net()
    f1, f2 = synth.tiny_pair(0)
    outs, (ws, bs) = _run_video(oracle, layers, [f1, f2], 8, 8)
    full = _full_forward(oracle, layers, ws, bs, f2)
    t = 1
    mask = oracle.rasterize(outs[1]["rects"][t], 64, 64).astype(bool)
    assert mask.sum() > 1500
    dx, dy = outs[1]["dxy"][t]
    prev = outs[0]["tensors"][t]
    cur = outs[1]["tensors"][t]
    ys, xs = np.nonzero(mask)
    assert np.array_equal(cur[ys, xs], prev[ys + dy, xs + dx])
    assert not np.array_equal(cur[ys, xs], full[t][ys, xs])
    assert np.array_equal(cur[~mask], full[t][~mask])


def test_expiry_forces_full_frames(oracle):
    layers = synth.tiny_net()
    rng = np.random.default_rng(3)
    f = rng.integers(0, 256, (64, 64, 3)).astype(np.uint8)
    outs, _ = _run_video(oracle, layers, [f] * 7, 8, 8, expiry=3)
    assert [o["full"] for o in outs] == [True, False, False, True, False, False, True]


def test_resnet_block_runs_and_reuses(oracle):
    # first stage of the residual trunk on a small frame: DAG wiring + add intersection
    layers = synth.resnet50_trunk()[:12]
    f1, f2 = synth.shifted_pair(14, 64, 64, (0, 0))
    outs, (ws, bs) = _run_video(oracle, layers, [f1, f2], 8, 4, bias_scale=0.0)
    for a, b in zip(outs[0]["tensors"], outs[1]["tensors"]):
        assert np.array_equal(a, b)
    assert len(outs[1]["rects"][12]) == 1


@pytest.mark.parametrize("extend", [False, True])
def test_invariant_static_scene_is_exact(oracle, extend):
    """A stream that did not move, blocks accepted only when identical (bound 0): every reused pixel has the same
    inputs as in the previous frame, so the cached frame equals the full forward bit for bit, with the printed
    rule and with the border case; the border case reuses more."""
    rng = np.random.default_rng(21)
    layers = synth.vgg16()[:7]
    H = W = 64
    f0 = rng.integers(0, 256, (H, W, 3)).astype(np.uint8)
    f1 = f0.copy()
    f1[24:40, 8:24] = rng.integers(0, 256, (16, 16, 3))            # one changed patch (2 x 2 blocks of 8)
    ws, bs = synth.he_weights(layers, 3, bias_scale=0.1)
    st = oracle.Stream(layers, ws, bs, H, W, 3, block=8, radius=4, max_ssd=0, extend_borders=extend)
    st.step(f0)
    out = st.step(f1)
    assert out["match"]["gmv"].tolist() == [0, 0] and int(out["match"]["mask"].sum()) == 64 - 4
    full = _full_forward(oracle, layers, ws, bs, f1)
    for a, b in zip(out["tensors"], full):
        assert np.array_equal(a, b)
    reused = [int(oracle.rasterize(out["rects"][t], *out["hw"][t]).sum()) for t in range(1, len(layers) + 1)]
    test_invariant_static_scene_is_exact.reused[extend] = reused
    if len(test_invariant_static_scene_is_exact.reused) == 2:
        plain, ext = (test_invariant_static_scene_is_exact.reused[e] for e in (False, True))
        assert all(e >= p for e, p in zip(ext, plain)) and sum(ext) > sum(plain)


test_invariant_static_scene_is_exact.reused = {}


def test_leaky_relu_of_a_convolution(oracle):
    """relu == 2: v < 0 -> 0.1 v, applied to the same sums as the other two settings."""
    rng = np.random.default_rng(31)
    x = rng.standard_normal((9, 11, 5)).astype(np.float32)
    w = rng.standard_normal((6, 3, 3, 5)).astype(np.float32)
    b = rng.standard_normal(6).astype(np.float32)
    plain = oracle.conv_cached(x, w, b, 3, 1, 1, 0).astype(np.float64)
    assert (plain < 0).any() and (plain > 0).any()
    assert np.allclose(oracle.conv_cached(x, w, b, 3, 1, 1, 2), np.where(plain > 0, plain, 0.1 * plain), rtol=1e-6, atol=1e-7)
    assert np.allclose(oracle.conv_cached(x, w, b, 3, 1, 1, 1), np.maximum(plain, 0), rtol=1e-6, atol=1e-7)
    one = np.full((1, 1, 1), -2.0, np.float32)                      # hand value: -2 * 3 = -6 -> -0.6
    assert abs(float(oracle.conv_cached(one, np.full((1, 1, 1, 1), 3.0, np.float32), None, 1, 1, 0, 2)[0, 0, 0]) + 0.6) < 1e-7


# ---- the same invariants with exact reuse maps instead of rectangles ---------------------------------------------
def test_exact_masks_zero_reuse_is_full_forward(oracle):
    rng = np.random.default_rng(6)
    layers = synth.tiny_net()
    frames = [rng.integers(0, 256, (64, 64, 3)).astype(np.uint8) for _ in range(2)]
    outs, (ws, bs) = _run_video(oracle, layers, frames, 8, 8, exact_masks=True)
    assert outs[1]["match"]["n_pass"] == 0 and all(not m.any() for m in outs[1]["masks"])
    for a, b in zip(outs[1]["tensors"], _full_forward(oracle, layers, ws, bs, frames[1])):
        assert np.array_equal(a, b)


def test_exact_masks_identical_frames_lose_only_the_padding_ring(oracle):
    rng = np.random.default_rng(8)
    layers = synth.tiny_net()           # 3x3 p1 s1; 3x3 p1 s2; 3x3 p1 s1
    f = rng.integers(0, 256, (64, 64, 3)).astype(np.uint8)
    outs, _ = _run_video(oracle, layers, [f, f], 8, 8, exact_masks=True)
    m = outs[1]["masks"]
    assert m[0].all()
    want1 = np.zeros((64, 64), bool); want1[1:63, 1:63] = True          # windows inside the map
    want2 = np.zeros((32, 32), bool); want2[1:31, 1:31] = True          # taps 2o-1 .. 2o+1 inside [1, 62]
    want3 = np.zeros((32, 32), bool); want3[2:30, 2:30] = True
    assert np.array_equal(m[1].astype(bool), want1) and np.array_equal(m[2].astype(bool), want2)
    assert np.array_equal(m[3].astype(bool), want3)
    for a, b in zip(outs[0]["tensors"], outs[1]["tensors"]):
        assert np.array_equal(a, b)


@pytest.mark.parametrize("bf16", [False, True])
def test_exact_masks_exact_shift_equals_full_forward(oracle, bf16):
    # more pixels are copied than with rectangles, and every copied value still equals the recomputed one
    layers = synth.tiny_net()
    f1, f2 = synth.shifted_pair(10, 64, 64, (4, -2))
    f2 = f2.copy()
    f2[24:40, 8:24] = np.random.default_rng(3).integers(0, 256, (16, 16, 3))     # a hole: the region is not one rectangle
    exact, (ws, bs) = _run_video(oracle, layers, [f1, f2], 8, 8, bf16=bf16, exact_masks=True)
    rect, _ = _run_video(oracle, layers, [f1, f2], 8, 8, bf16=bf16)
    full = _full_forward(oracle, layers, ws, bs, f2, bf16=bf16)
    more = 0
    for t in range(1, len(layers) + 1):
        assert np.array_equal(exact[1]["tensors"][t], full[t]), t
        reused_rect = sum(int(w) * int(h) for _, _, w, h in rect[1]["rects"][t])
        assert int(exact[1]["masks"][t].sum()) >= reused_rect
        more += int(exact[1]["masks"][t].sum()) - reused_rect
    assert more > 100


def test_exact_masks_values_come_from_the_cache(oracle):
    # a noisy second frame: reused pixels are the previous frame's values at the offset, bit for bit, and differ
    # from what a recomputation gives
    layers = synth.tiny_net()
    f1, f2 = synth.tiny_pair(0)
    outs, (ws, bs) = _run_video(oracle, layers, [f1, f2], 8, 8, exact_masks=True)
    full = _full_forward(oracle, layers, ws, bs, f2)
    for t in (1, 2, 3):
        m = outs[1]["masks"][t].astype(bool)
        dx, dy = (int(v) for v in outs[1]["dxy"][t])
        ys, xs = np.nonzero(m)
        assert len(ys) > 50
        assert np.array_equal(outs[1]["tensors"][t][ys, xs], outs[0]["tensors"][t][ys + dy, xs + dx])
        assert np.array_equal(outs[1]["tensors"][t][~m], full[t][~m]) or t > 1      # layer 1 reads exact inputs
        assert not np.array_equal(outs[1]["tensors"][t][m], full[t][m])


# ---- max-pooling and add layers that use the cache too (Section 5: the cache extends to other layer types) ---------
def _pool_add_stack():
    C_ = lambda cin, cout, i, relu=1: dict(type=synth.CONV, k=3, s=1, p=1, cin=cin, cout=cout, relu=relu, in0=i, in1=-1)
    return [C_(3, 8, 0), dict(type=synth.MAXPOOL, k=2, s=2, p=0, cin=8, cout=8, relu=0, in0=1, in1=-1),
            C_(8, 8, 2), C_(8, 8, 3, 0), dict(type=synth.ADD, k=1, s=1, p=0, cin=8, cout=8, relu=1, in0=4, in1=2),
            dict(type=synth.MAXPOOL, k=3, s=2, p=1, cin=8, cout=8, relu=0, in0=5, in1=-1), C_(8, 8, 6)]


def test_cached_pool_and_add_exact_shift_equals_full_forward(oracle):
    layers = _pool_add_stack()           # total stride 4
    f1, f2 = synth.shifted_pair(10, 64, 64, (8, -4))
    f2 = f2.copy()
    f2[24:40, 8:24] = np.random.default_rng(3).integers(0, 256, (16, 16, 3))
    outs, (ws, bs) = _run_video(oracle, layers, [f1, f2], 8, 8, exact_masks=True, cache_pool_add=True)
    assert outs[1]["match"]["gmv"].tolist() == [-8, 4]
    full = _full_forward(oracle, layers, ws, bs, f2)
    for t in range(1, len(layers) + 1):
        assert np.array_equal(outs[1]["tensors"][t], full[t]), t
    for t in (2, 5, 6):                  # the pooling and add outputs were really taken from the cache
        m = outs[1]["masks"][t].astype(bool)
        dx, dy = (int(v) for v in outs[1]["dxy"][t])
        ys, xs = np.nonzero(m)
        assert len(ys) > 20
        assert np.array_equal(outs[1]["tensors"][t][ys, xs], outs[0]["tensors"][t][ys + dy, xs + dx])


def test_cached_pool_and_add_take_their_values_from_the_cache(oracle):
    # a noisy frame moved by (3, -2): not a multiple of the strides, so a pooled value from the cache differs from
    # the pooling of the current (copied) conv output; the option decides which one the stream holds
    layers = _pool_add_stack()
    f1, f2 = synth.tiny_pair(0)
    on, _ = _run_video(oracle, layers, [f1, f2], 8, 8, exact_masks=True, cache_pool_add=True)
    off, _ = _run_video(oracle, layers, [f1, f2], 8, 8, exact_masks=True)
    for t in (2, 5, 6):
        m = on[1]["masks"][t].astype(bool)
        dx, dy = (int(v) for v in on[1]["dxy"][t])
        ys, xs = np.nonzero(m)
        assert len(ys) > 10
        assert np.array_equal(on[1]["tensors"][t][ys, xs], on[0]["tensors"][t][ys + dy, xs + dx])
    assert np.array_equal(on[1]["tensors"][1], off[1]["tensors"][1])            # nothing changes before the first pooling
    assert not np.array_equal(on[1]["tensors"][2], off[1]["tensors"][2])
    # without any reuse the option changes nothing
    rng = np.random.default_rng(6)
    frames = [rng.integers(0, 256, (64, 64, 3)).astype(np.uint8) for _ in range(2)]
    a, (ws, bs) = _run_video(oracle, layers, frames, 8, 8, exact_masks=True, cache_pool_add=True)
    for x, y in zip(a[1]["tensors"], _full_forward(oracle, layers, ws, bs, frames[1])):
        assert np.array_equal(x, y)


@pytest.mark.parametrize("exact", [False, True])
def test_conv_layers_that_do_not_use_the_cache(oracle, exact):
    """no_reuse: a flagged conv layer is computed in full from whatever its input holds; the others keep reusing
    from their own caches, and the regions do not change."""
    layers = synth.tiny_net()
    f1, f2 = synth.tiny_pair(0)
    base, (ws, bs) = _run_video(oracle, layers, [f1, f2], 8, 8, exact_masks=exact)
    conv = [i for i, L in enumerate(layers) if L["type"] == synth.CONV]
    # every conv layer flagged: the cached frame is the full forward, bit for bit
    all_off, _ = _run_video(oracle, layers, [f1, f2], 8, 8, exact_masks=exact, no_reuse=[1] * len(layers))
    for x, y in zip(all_off[1]["tensors"], _full_forward(oracle, layers, ws, bs, f2)):
        assert np.array_equal(x, y)
    # no layer flagged: the default
    none_off, _ = _run_video(oracle, layers, [f1, f2], 8, 8, exact_masks=exact, no_reuse=[0] * len(layers))
    for x, y in zip(none_off[1]["tensors"], base[1]["tensors"]):
        assert np.array_equal(x, y)
    # only the second conv layer flagged
    flags = [0] * len(layers)
    flags[conv[1]] = 1
    mixed, _ = _run_video(oracle, layers, [f1, f2], 8, 8, exact_masks=exact, no_reuse=flags)
    t1, t2, t3 = conv[0] + 1, conv[1] + 1, conv[2] + 1
    assert np.array_equal(mixed[1]["tensors"][t1], base[1]["tensors"][t1])          # before it nothing changes
    L = layers[conv[1]]
    want = oracle.conv_cached(mixed[1]["tensors"][L["in0"]], ws[conv[1]], bs[conv[1]], L["k"], L["s"], L["p"], bool(L["relu"]))
    assert np.array_equal(mixed[1]["tensors"][t2], want)                             # the layer itself: a plain convolution of its input
    assert not np.array_equal(mixed[1]["tensors"][t2], base[1]["tensors"][t2])      # which is not what the cache held
    # the layer behind it still takes its reusable pixels from its own cache
    m = (mixed[1]["masks"][t3].astype(bool) if exact else oracle.rasterize(mixed[1]["rects"][t3], *mixed[1]["tensors"][t3].shape[:2]).astype(bool))
    dx, dy = (int(v) for v in mixed[1]["dxy"][t3])
    ys, xs = np.nonzero(m)
    assert len(ys) > 10
    assert np.array_equal(mixed[1]["tensors"][t3][ys, xs], mixed[0]["tensors"][t3][ys + dy, xs + dx])
    # the regions are the same with and without flags
    for t in range(len(layers) + 1):
        assert np.array_equal(mixed[1]["rects"][t], base[1]["rects"][t])
        if exact:
            assert np.array_equal(mixed[1]["masks"][t], base[1]["masks"][t])
