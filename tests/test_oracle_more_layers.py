"""Pins of the oracle's remaining layer types and their rows of Table 2 (LRN, concat, fully-connected, softmax,
average pooling).  Every pin is independent of the oracle: hand-computed values, the table's printed formulas,
brute force over pixels, and library routines (torch, scipy, numpy) for the special cases they implement."""
import numpy as np
import pytest
import scipy.special
import torch
import torch.nn.functional as F


def _nchw(x):
    return torch.from_numpy(np.ascontiguousarray(x.transpose(2, 0, 1))[None]).double()


def _hwc(t):
    return t[0].permute(1, 2, 0).numpy()


# ---- arithmetic -------------------------------------------------------------------------------------------------
def test_lrn_across_channels_hand_value(oracle):
    # one pixel, channels (1, 2, 3), window 3, alpha/n = 1, beta = 1, kappa = 1:
    # 1/(1+1+4), 2/(1+1+4+9), 3/(1+4+9)
    x = np.array([[[1.0, 2.0, 3.0]]], np.float32)
    got = oracle.lrn(x, 3, alpha=3.0, beta=1.0, kappa=1.0)
    assert np.allclose(got[0, 0], [1 / 6, 2 / 15, 3 / 14], rtol=1e-7)


def test_lrn_within_channel_hand_value(oracle):
    # 2x2 map, one channel, window 3: every window holds all four values (sum of squares 30), n = 9
    x = np.array([[[1.0], [2.0]], [[3.0], [4.0]]], np.float32)
    got = oracle.lrn(x, 3, alpha=9.0, beta=0.5, kappa=6.0, within=True)
    assert np.allclose(got[:, :, 0], np.array([[1, 2], [3, 4]]) / 6.0, rtol=1e-7)


@pytest.mark.parametrize("size,alpha,beta,kappa", [(5, 1e-4, 0.75, 2.0), (3, 0.3, 0.5, 1.0), (7, 2.0, 1.25, 1.5)])
def test_lrn_across_channels_matches_torch(oracle, size, alpha, beta, kappa):
    rng = np.random.default_rng(size)
    x = (rng.standard_normal((9, 11, 13)) * 3).astype(np.float32)
    want = _hwc(F.local_response_norm(_nchw(x), size, alpha=alpha, beta=beta, k=kappa))
    got = oracle.lrn(x, size, alpha, beta, kappa)
    assert np.allclose(got, want, rtol=2e-7, atol=1e-9)


@pytest.mark.parametrize("size", [3, 5])
def test_lrn_within_channel_matches_padded_window_average(oracle, size):
    rng = np.random.default_rng(40 + size)
    x = (rng.standard_normal((10, 12, 6)) * 2).astype(np.float32)
    alpha, beta, kappa = 0.7, 0.75, 1.3
    t = _nchw(x)
    avg = F.avg_pool2d(t * t, size, stride=1, padding=size // 2, count_include_pad=True)   # zeros outside, divisor size^2
    want = _hwc(t / (kappa + alpha * avg) ** beta)
    got = oracle.lrn(x, size, alpha, beta, kappa, within=True)
    assert np.allclose(got, want, rtol=2e-7, atol=1e-9)


def test_concat_matches_numpy(oracle):
    rng = np.random.default_rng(3)
    xs = [rng.standard_normal((5, 7, c)).astype(np.float32) for c in (3, 8, 1, 6)]
    assert np.array_equal(oracle.concat(xs), np.concatenate(xs, axis=2))
    assert np.array_equal(oracle.concat(xs[:2]), np.concatenate(xs[:2], axis=2))


def test_fc_matches_matmul_and_whole_map_convolution(oracle):
    rng = np.random.default_rng(4)
    x = rng.standard_normal((6, 6, 10)).astype(np.float32)
    w = (rng.standard_normal((17, 6 * 6 * 10)) * 0.1).astype(np.float32)
    b = rng.standard_normal(17).astype(np.float32)
    want = w.astype(np.float64) @ x.reshape(-1).astype(np.float64) + b
    got = oracle.fc(x, w, b, relu=False)
    assert got.shape == (1, 1, 17)
    assert np.allclose(got.reshape(-1), want, rtol=1e-6, atol=1e-6)
    assert np.allclose(oracle.fc(x, w, b, relu=True).reshape(-1), np.maximum(want, 0), rtol=1e-6, atol=1e-6)
    # a fully-connected layer is the convolution whose kernel covers the whole map (pinned against scipy elsewhere)
    conv = oracle.conv_cached(x, w.reshape(17, 6, 6, 10), b, 6, 1, 0, False)
    assert np.array_equal(conv.reshape(-1), got.reshape(-1))
    # bf16 storage: rounded once
    assert np.array_equal(oracle.fc(x, w, b, False, bf16=True), oracle.round_bf16(got))


def test_softmax_matches_scipy(oracle):
    rng = np.random.default_rng(5)
    x = (rng.standard_normal((3, 4, 21)) * 5).astype(np.float32)
    got = oracle.softmax(x)
    assert np.allclose(got, scipy.special.softmax(x.astype(np.float64), axis=2), rtol=1e-6, atol=1e-9)
    assert np.allclose(got.sum(axis=2), 1.0, atol=1e-6)
    assert np.allclose(oracle.softmax(x + 100.0), got, rtol=1e-5, atol=1e-8)      # shift invariance
    big = np.array([[[1000.0, 1000.0, -1000.0]]], np.float32)                    # no overflow
    assert np.allclose(oracle.softmax(big)[0, 0], [0.5, 0.5, 0.0])


@pytest.mark.parametrize("k,s,p", [(7, 1, 0), (3, 2, 1), (2, 2, 0), (5, 3, 2)])
def test_avgpool_matches_torch(oracle, k, s, p):
    rng = np.random.default_rng(k * 10 + s)
    x = rng.standard_normal((14, 9, 5)).astype(np.float32)
    want = _hwc(F.avg_pool2d(_nchw(x), k, stride=s, padding=p, count_include_pad=False))
    got = oracle.avgpool(x, k, s, p)
    assert got.shape == want.shape
    assert np.allclose(got, want, rtol=1e-6, atol=1e-7)


def test_global_avgpool_is_the_mean(oracle):
    rng = np.random.default_rng(6)
    x = rng.standard_normal((7, 7, 12)).astype(np.float32)
    assert np.allclose(oracle.avgpool(x, 7, 1, 0)[0, 0], x.astype(np.float64).mean(axis=(0, 1)), rtol=1e-6, atol=1e-7)


# ---- Table 2 rows -------------------------------------------------------------------------------------------------
def test_lrn_row_of_table_2(oracle):
    # the row as printed: x' = x + r, y' = y + r, w' = w - 2r, h' = h - 2r
    assert oracle.dt_lrn((10, 20, 30, 12), 2) == (12, 22, 26, 8)
    assert oracle.dt_lrn((0, 0, 5, 5), 2) == (2, 2, 1, 1)
    assert oracle.dt_lrn((3, 3, 4, 9), 2) is None
    assert oracle.dt_lrn((7, 8, 9, 10), 0) == (7, 8, 9, 10)


def test_lrn_row_is_window_containment(oracle):
    # brute force: the output pixels whose (2r+1)^2 window lies wholly inside the rectangle
    H, W = 20, 24
    for rect in [(3, 2, 10, 9), (0, 0, 24, 20), (5, 5, 3, 3), (18, 1, 6, 12)]:
        for r in (1, 2):
            inside = np.zeros((H, W), bool)
            x, y, w, h = rect
            inside[y:y + h, x:x + w] = True
            want = np.zeros((H, W), bool)
            for yy in range(H):
                for xx in range(W):
                    ys, xs = range(yy - r, yy + r + 1), range(xx - r, xx + r + 1)
                    want[yy, xx] = all(0 <= a < H and 0 <= b < W and inside[a, b] for a in ys for b in xs)
            got = oracle.dt_lrn(rect, r)
            mask = oracle.rasterize([got] if got else [], H, W).astype(bool)
            assert np.array_equal(mask, want), (rect, r)


def _L(**kw):
    return dict(kw)


def test_propagation_rows_of_the_new_layer_types(oracle):
    H = W = 40
    layers = [
        _L(type=0, k=3, s=1, p=1, cin=3, cout=4, relu=1, in0=0),                      # t1
        _L(type=4, k=5, cin=4, cout=4, in0=1, within=0, alpha=1e-4, beta=0.75, kappa=2.0),    # t2: window over channels
        _L(type=4, k=5, cin=4, cout=4, in0=1, within=1, alpha=1e-4, beta=0.75, kappa=2.0),    # t3: 5x5 pixels
        _L(type=0, k=5, s=1, p=2, cin=4, cout=4, relu=1, in0=1),                      # t4
        _L(type=5, cin=12, cout=12, in0=2, in1=3, in2=4),                             # t5: concat of t2, t3, t4
        _L(type=8, k=2, s=2, p=0, cin=12, cout=12, in0=5),                            # t6: average pooling
        _L(type=6, cin=12, cout=10, relu=0, in0=6),                                   # t7: fully connected
        _L(type=7, cin=10, cout=10, in0=7),                                           # t8: softmax
    ]
    rects0 = [(4, 6, 20, 16), (28, 2, 10, 30)]
    pr = oracle.propagate(layers, H, W, rects0, 0, 0)
    r = [sorted(map(tuple, t.tolist())) for t in pr["rects"]]
    t1 = sorted([(5, 7, 18, 14), (29, 3, 8, 28)])
    assert r[1] == t1
    assert r[2] == t1                                                   # channel window: nothing changes in the pixel grid
    assert r[3] == sorted([(7, 9, 14, 10), (31, 5, 4, 24)])             # printed row with r = 2
    assert r[4] == sorted([(7, 9, 14, 10), (31, 5, 4, 24)])             # a 5x5 convolution erodes alike
    # concat: the overlap, here by brute force over pixels
    masks = [oracle.rasterize(pr["rects"][t], H, W).astype(bool) for t in (2, 3, 4)]
    assert np.array_equal(oracle.rasterize(pr["rects"][5], H, W).astype(bool), masks[0] & masks[1] & masks[2])
    assert r[6] == sorted([(4, 5, 6, 4), (16, 3, 1, 11)])               # 2x2 stride-2 windows inside (7,9,14,10), (31,5,4,24)
    assert len(r[7]) == 0 and len(r[8]) == 0                            # (0,0,0,0)
    assert tuple(pr["hw"][7]) == (1, 1) and tuple(pr["hw"][6]) == (20, 20)


def test_concat_row_with_several_rectangles_per_input(oracle):
    H = W = 32
    layers = [
        _L(type=0, k=1, s=1, p=0, cin=3, cout=2, relu=0, in0=0),
        _L(type=0, k=3, s=1, p=1, cin=3, cout=2, relu=0, in0=0),
        _L(type=0, k=5, s=1, p=2, cin=3, cout=2, relu=0, in0=0),
        _L(type=0, k=7, s=1, p=3, cin=3, cout=2, relu=0, in0=0),
        _L(type=5, cin=8, cout=8, in0=1, in1=2, in2=3, in3=4),
    ]
    rects0 = [(0, 0, 12, 32), (14, 3, 9, 9), (16, 16, 16, 12)]
    pr = oracle.propagate(layers, H, W, rects0, 0, 0)
    want = np.ones((H, W), bool)
    for t in (1, 2, 3, 4):
        want &= oracle.rasterize(pr["rects"][t], H, W).astype(bool)
    assert np.array_equal(oracle.rasterize(pr["rects"][5], H, W).astype(bool), want)
    # with rectangles that do not overlap each other, the overlap of the lists is the most eroded input
    assert np.array_equal(want, oracle.rasterize(pr["rects"][4], H, W).astype(bool))


# ---- whole stack --------------------------------------------------------------------------------------------------
def _small_alexnet_like():
    return [
        _L(type=0, k=5, s=2, p=2, cin=3, cout=8, relu=1, in0=0),
        _L(type=4, k=3, cin=8, cout=8, in0=1, within=0, alpha=0.125, beta=0.75, kappa=1.0),   # constants exact in fp32
        _L(type=1, k=3, s=2, p=0, cin=8, cout=8, in0=2),
        _L(type=0, k=3, s=1, p=1, cin=8, cout=8, relu=1, in0=3),
        _L(type=0, k=1, s=1, p=0, cin=8, cout=4, relu=1, in0=3),
        _L(type=5, cin=12, cout=12, in0=4, in1=5),
        _L(type=8, k=3, s=2, p=1, cin=12, cout=12, in0=6),
        _L(type=6, cin=12, cout=16, relu=1, in0=7),
        _L(type=6, cin=16, cout=5, relu=0, in0=8),
        _L(type=7, cin=5, cout=5, in0=9),
    ]


def _weights(layers, shapes, seed):
    rng = np.random.default_rng(seed)
    ws, bs = [], []
    for i, L in enumerate(layers):
        if L["type"] == 0:
            ws.append((rng.standard_normal((L["cout"], L["k"], L["k"], L["cin"])) * np.sqrt(2.0 / (L["k"] ** 2 * L["cin"]))).astype(np.float32))
            bs.append((rng.standard_normal(L["cout"]) * 0.1).astype(np.float32))
        elif L["type"] == 6:
            K = int(np.prod(shapes[L["in0"]]))
            ws.append((rng.standard_normal((L["cout"], K)) * np.sqrt(2.0 / K)).astype(np.float32))
            bs.append((rng.standard_normal(L["cout"]) * 0.1).astype(np.float32))
        else:
            ws.append(None); bs.append(None)
    return ws, bs


def test_stack_with_every_layer_type_is_the_composition_of_its_layers(oracle):
    from paper_1712_01670_amd import synth
    layers = _small_alexnet_like()
    H = W = 48
    st = oracle.Stream(layers, [None] * len(layers), [None] * len(layers), H, W)
    ws, bs = _weights(layers, st.shapes, 1)
    st = oracle.Stream(layers, ws, bs, H, W, block=8, radius=4)
    prev, cur = synth.shifted_pair(11, H, W, (2, -1))
    out0 = st.step(prev)
    t = [oracle.frame_to_tensor(prev)]
    for i, L in enumerate(layers):
        a = t[L["in0"]]
        ty = L["type"]
        if ty == 0: t.append(oracle.conv_cached(a, ws[i], bs[i], L["k"], L["s"], L["p"], L["relu"]))
        elif ty == 1: t.append(oracle.maxpool(a, L["k"], L["s"], L["p"]))
        elif ty == 4: t.append(oracle.lrn(a, L["k"], L["alpha"], L["beta"], L["kappa"], L["within"]))
        elif ty == 5: t.append(oracle.concat([t[L["in0"]], t[L["in1"]]]))
        elif ty == 6: t.append(oracle.fc(a, ws[i], bs[i], L["relu"]))
        elif ty == 7: t.append(oracle.softmax(a))
        elif ty == 8: t.append(oracle.avgpool(a, L["k"], L["s"], L["p"]))
    for i in range(len(layers) + 1):
        assert np.array_equal(out0["tensors"][i], t[i]), i
    assert abs(float(out0["tensors"][-1].sum()) - 1.0) < 1e-6
    # second frame: the convolutions reuse, the other layers are recomputed; nothing is reusable after the first fc
    out1 = st.step(cur)
    assert len(out1["rects"][1]) > 0 and len(out1["rects"][8]) == 0 and len(out1["rects"][10]) == 0
    # identical frame: every tensor equals the previous frame's
    out2 = st.step(cur)
    for i in range(len(layers) + 1):
        assert np.array_equal(out2["tensors"][i], out1["tensors"][i]), i


# ---- element-wise add and ReLU ------------------------------------------------------------------------------------
def test_add_hand_values(oracle):
    # exact binary fractions: every sum is exact in fp32, so the expected values are plain arithmetic
    a = np.array([1.5, -2.0, 0.25, -0.5, 1e3, -0.0], np.float32)
    b = np.array([2.0, 1.0, -0.25, -1.0, -1e3 + 0.5, 0.0], np.float32)
    assert oracle.add(a, b, relu=False).tolist() == [3.5, -1.0, 0.0, -1.5, 0.5, 0.0]
    assert oracle.add(a, b, relu=True).tolist() == [3.5, 0.0, 0.0, 0.0, 0.5, 0.0]
    # the operands are not interchanged with anything else: a + b, not a - b or b alone
    assert oracle.add(a, np.zeros_like(a), relu=False).tolist() == a.tolist()
    assert oracle.add(np.zeros_like(b), b, relu=False).tolist() == b.tolist()


def test_add_bf16_rounds_the_sum_once_to_nearest_even(oracle):
    # bf16 keeps 8 significant bits: the spacing at 1.0 is 2^-7
    e = lambda k: float(2.0 ** -k)
    cases = [
        (1.0, e(9), 1.0),                           # below half a step: down
        (1.0, e(8), 1.0),                           # exactly half, lower neighbour even: down
        (1.0 + e(7), e(8), 1.0 + e(6)),             # exactly half, lower neighbour odd: up
        (1.0, e(8) + e(20), 1.0 + e(7)),            # just above half: up (the sum is not rounded to the tie first)
        (-1.0, -e(8), -1.0),                        # ties behave the same for negative sums
        (0.5, 0.25, 0.75),                          # representable: unchanged
    ]
    a = np.array([c[0] for c in cases], np.float32)
    b = np.array([c[1] for c in cases], np.float32)
    want = [c[2] for c in cases]
    assert oracle.add(a, b, relu=False, bf16=True).tolist() == want
    # ReLU acts on the sum, then the result is rounded
    assert oracle.add(a, b, relu=True, bf16=True).tolist() == [max(w, 0.0) for w in want]
    # without bf16 nothing is rounded beyond fp32
    assert oracle.add(a, b, relu=False).tolist() == [float(np.float32(x) + np.float32(y)) for x, y, _ in cases]


def test_add_matches_numpy_on_random_values(oracle):
    rng = np.random.default_rng(5)
    a = rng.standard_normal(4099).astype(np.float32) * 7
    b = rng.standard_normal(4099).astype(np.float32) * 7
    want = (a.astype(np.float64) + b.astype(np.float64))
    assert np.array_equal(oracle.add(a, b, relu=False), want.astype(np.float32))
    assert np.array_equal(oracle.add(a, b, relu=True), np.maximum(want, 0.0).astype(np.float32))
    bf = torch.from_numpy(np.maximum(want, 0.0)).to(torch.bfloat16).float().numpy()
    assert np.array_equal(oracle.add(a, b, relu=True, bf16=True), bf)


def test_relu_hand_values(oracle):
    x = np.array([-1.0, 0.0, 2.5, -0.0, 1e-30, -1e-30, 3.0e38, -3.0e38], np.float32)
    got = oracle.relu(x)
    assert got.tolist() == [0.0, 0.0, 2.5, 0.0, float(np.float32(1e-30)), 0.0, float(np.float32(3.0e38)), 0.0]
    assert not np.signbit(got).any()          # negative zero does not survive either
    rng = np.random.default_rng(6)
    y = rng.standard_normal(1000).astype(np.float32)
    assert np.array_equal(oracle.relu(y), np.maximum(y, 0))      # positives pass unchanged, bit for bit


def test_relu_and_add_layers_inside_a_stack(oracle):
    # conv (identity weights) -> ReLU layer -> add(ReLU output, conv output): out = max(x, 0) + x, by hand per element
    from paper_1712_01670_amd import synth
    layers = [dict(type=synth.CONV, k=1, s=1, p=0, cin=2, cout=2, relu=0, in0=0, in1=-1),
              dict(type=synth.RELU, k=1, s=1, p=0, cin=2, cout=2, relu=0, in0=1, in1=-1),
              dict(type=synth.ADD, k=1, s=1, p=0, cin=2, cout=2, relu=0, in0=2, in1=1)]
    w = [np.eye(2, dtype=np.float32).reshape(2, 1, 1, 2), None, None]
    st = oracle.Stream(layers, w, [None, None, None], 4, 4, 2, block=2, radius=1)
    frame = np.arange(32, dtype=np.uint8).reshape(4, 4, 2) * 8
    res = st.step(frame)
    x = (frame.astype(np.float64) - 128.0) / 128.0
    assert np.array_equal(res["tensors"][2], np.maximum(x, 0).astype(np.float32))
    assert np.array_equal(res["tensors"][3], (np.maximum(x, 0) + x).astype(np.float32))
