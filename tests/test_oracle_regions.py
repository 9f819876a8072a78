"""Pins for the oracle's region logic: Section 4 Step 5 (merge) and Section 5 Table 2
(region transformation), against the paper's worked examples and brute force."""
import itertools
import os

import numpy as np
import pytest

from paper_1712_01670_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "region_examples.txt")


def _golden():
    rows = []
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        name, rin, ksp, rout, _ = [f.strip() for f in line.split("|")]
        rows.append((name, tuple(map(int, rin.split())), tuple(map(int, ksp.split())),
                     tuple(map(int, rout.split()))))
    return rows


@pytest.mark.parametrize("name,rin,ksp,rout", _golden())
def test_paper_worked_examples(oracle, name, rin, ksp, rout):
    assert oracle.dt_window(rin, *ksp) == rout


def test_paper_example_source_rect_keeps_offset(oracle):
    # Section 5: the previous-frame block (120,120,100,40) goes through the same rule;
    # the offset 20 px becomes 10 px after the stride-2 layer and the sizes agree.
    cur = oracle.dt_window((100, 100, 100, 40), 11, 2, 5)
    src = oracle.dt_window((120, 120, 100, 40), 11, 2, 5)
    assert src == (cur[0] + 10, cur[1] + 10, cur[2], cur[3])
    # following pooling layer k3 s2 p1 shrinks it again
    assert oracle.dt_window(cur, 3, 2, 1) == (27, 27, 22, 7)


def test_erosion_pixel_counts(oracle):
    # Section 4: two separate 5x5 blocks keep 18 px, the merged 5x10 keeps 24 px
    a = oracle.dt_window((0, 0, 5, 5), 3, 1, 1)
    b = oracle.dt_window((0, 0, 10, 5), 3, 1, 1)
    assert 2 * a[2] * a[3] == 18
    assert b[2] * b[3] == 24


def _brute(rect, k, s, p, Win, Hin):
    """All output pixels whose k x k window lies wholly inside rect (padding never does)."""
    x, y, w, h = rect
    Wo, Ho = (Win + 2 * p - k) // s + 1, (Hin + 2 * p - k) // s + 1
    ok = np.zeros((Ho, Wo), bool)
    for Y in range(Ho):
        for X in range(Wo):
            x0, y0 = X * s - p, Y * s - p
            ok[Y, X] = (x0 >= x and x0 + k <= x + w and y0 >= y and y0 + k <= y + h)
    return ok


@pytest.mark.parametrize("k,s", [(1, 1), (1, 2), (2, 2), (3, 1), (3, 2), (7, 2), (11, 2), (3, 3), (5, 1)])
def test_dt_window_is_exact_window_containment(oracle, k, s):
    rng = np.random.default_rng(k * 10 + s)
    Win, Hin = 37, 29
    for p in range(0, 6):
        if Win + 2 * p < k:
            continue
        for _ in range(40):
            x = int(rng.integers(0, Win - 1)); y = int(rng.integers(0, Hin - 1))
            w = int(rng.integers(1, Win - x + 1)); h = int(rng.integers(1, Hin - y + 1))
            ok = _brute((x, y, w, h), k, s, p, Win, Hin)
            r = oracle.dt_window((x, y, w, h), k, s, p)
            got = np.zeros_like(ok)
            if r is not None:
                got[r[1]:r[1] + r[3], r[0]:r[0] + r[2]] = True
                assert r[0] >= 0 and r[1] >= 0 and r[0] + r[2] <= ok.shape[1] and r[1] + r[3] <= ok.shape[0]
            assert np.array_equal(ok, got), (x, y, w, h, k, s, p)


def test_table2_other_rows(oracle):
    # activation: unchanged; overlap of rectangles for multi-input layers
    L = [dict(type=synth.RELU, k=1, s=1, p=0, cin=4, cout=4, relu=0, in0=0, in1=-1)]
    out = oracle.propagate(L, 32, 32, [(4, 6, 10, 12)], 0, 0)
    assert out["rects"][1].tolist() == [[4, 6, 10, 12]]
    assert oracle.dt_overlap((0, 0, 10, 10), (5, 6, 10, 10)) == (5, 6, 5, 4)
    assert oracle.dt_overlap((0, 0, 5, 5), (5, 0, 5, 5)) is None


def _check_merge(oracle, mask, B):
    rects = oracle.merge_blocks(mask, B)
    cover = np.zeros((mask.shape[0] * B, mask.shape[1] * B), np.int32)
    for x, y, w, h in rects:
        assert x % B == 0 and y % B == 0 and w % B == 0 and h % B == 0 and w > 0 and h > 0
        cover[y:y + h, x:x + w] += 1
    want = np.kron(mask, np.ones((B, B), np.int32))
    assert np.array_equal(cover, want)  # disjoint and union == mask
    return rects


def test_merge_invariants_random(oracle):
    rng = np.random.default_rng(7)
    for trial in range(200):
        gh, gw = int(rng.integers(1, 12)), int(rng.integers(1, 12))
        mask = (rng.random((gh, gw)) < rng.random()).astype(np.uint8)
        _check_merge(oracle, mask, int(rng.integers(1, 5)))


def test_merge_hand_cases(oracle):
    # full grid -> one rectangle
    assert oracle.merge_blocks(np.ones((3, 4), np.uint8), 8).tolist() == [[0, 0, 32, 24]]
    assert oracle.merge_blocks(np.zeros((3, 4), np.uint8), 8).tolist() == []
    # L shape: the first run claims the top row, then extends while the whole run is set
    m = np.array([[1, 1, 1],
                  [1, 1, 0],
                  [1, 1, 0]], np.uint8)
    assert oracle.merge_blocks(m, 2).tolist() == [[0, 0, 6, 2], [0, 2, 4, 4]]
    # a hole splits rows
    m = np.array([[1, 1, 1],
                  [1, 0, 1],
                  [1, 1, 1]], np.uint8)
    assert oracle.merge_blocks(m, 1).tolist() == [[0, 0, 3, 1], [0, 1, 1, 2], [2, 1, 1, 2], [1, 2, 1, 1]]


def test_adjacent_blocks_merge_beats_separate(oracle):
    # Section 4: adjacent properly-matched blocks share the offset and merge into one
    m = np.array([[1, 1]], np.uint8)
    r = oracle.merge_blocks(m, 5)
    assert r.tolist() == [[0, 0, 10, 5]]


def test_propagate_vgg_against_rasterized_brute_force(oracle):
    """Chain of convs and pools: the propagated rectangles of every tensor must equal,
    pixel for pixel, the set found by testing each output window against the input
    reusable set layer by layer (motion 0, so no clipping interferes)."""
    L = synth.vgg16()[:7]
    H = W = 64
    rects0 = [(0, 0, 32, 48), (32, 16, 32, 16), (48, 48, 16, 16)]
    out = oracle.propagate(L, H, W, rects0, 0, 0)
    for li, layer in enumerate(L):
        a, t = layer["in0"], li + 1
        ha, wa = out["hw"][a]
        ho, wo = out["hw"][t]
        want = np.zeros((ho, wo), bool)
        for r in out["rects"][a]:
            want |= _brute(tuple(r), layer["k"], layer["s"], layer["p"], wa, ha)
        got = oracle.rasterize(out["rects"][t], ho, wo).astype(bool)
        assert np.array_equal(want, got), li
    assert out["cum_stride"].tolist() == [1, 1, 1, 2, 2, 2, 4, 4]


def test_propagate_offsets_and_clipping(oracle):
    L = synth.tiny_net()
    # motion (4,-2): a multiple of the total stride 2 in x and y
    out = oracle.propagate(L, 64, 64, [(0, 8, 56, 48)], 4, -2)
    assert out["dxy"].tolist() == [[4, -2], [4, -2], [2, -1], [2, -1]]
    # every source rectangle stays inside its map
    for t, rects in enumerate(out["rects"]):
        h, w = out["hw"][t]
        dx, dy = out["dxy"][t]
        for x, y, ww, hh in rects:
            assert 0 <= x + dx and x + dx + ww <= w and 0 <= y + dy and y + dy + hh <= h
    # rounding of a misaligned motion: halves away from zero
    out = oracle.propagate(L, 64, 64, [(8, 8, 40, 40)], 3, -1)
    assert out["dxy"].tolist() == [[3, -1], [3, -1], [2, -1], [2, -1]]
    out = oracle.propagate(L, 64, 64, [(8, 8, 40, 40)], -3, 1)
    assert out["dxy"].tolist() == [[-3, 1], [-3, 1], [-2, 1], [-2, 1]]
    out = oracle.propagate(L, 64, 64, [(8, 8, 40, 40)], 1, -5)
    assert out["dxy"].tolist() == [[1, -5], [1, -5], [1, -3], [1, -3]]
    # a rectangle whose source would leave the map is clipped at the input
    out = oracle.propagate(L, 64, 64, [(56, 0, 8, 64)], 4, 0)
    assert out["rects"][0].tolist() == [[56, 0, 4, 64]]


def test_propagate_residual_intersection(oracle):
    # branch a: conv3x3 p1 (erodes), branch b: identity shortcut; add -> overlap
    L = [dict(type=synth.CONV, k=3, s=1, p=1, cin=4, cout=4, relu=1, in0=0, in1=-1),
         dict(type=synth.ADD, k=1, s=1, p=0, cin=4, cout=4, relu=1, in0=1, in1=0)]
    out = oracle.propagate(L, 32, 32, [(8, 8, 16, 16)], 0, 0)
    assert out["rects"][1].tolist() == [[9, 9, 14, 14]]
    assert out["rects"][2].tolist() == [[9, 9, 14, 14]]
    # resnet trunk: both inputs of every add have the same cumulative stride
    R = synth.resnet50_trunk()
    out = oracle.propagate(R, 224, 224, [(0, 0, 224, 224)], 0, 0)
    for i, l in enumerate(R):
        if l["type"] == synth.ADD:
            assert out["cum_stride"][l["in0"]] == out["cum_stride"][l["in1"]]
            assert tuple(out["hw"][l["in0"]]) == tuple(out["hw"][l["in1"]])
    assert out["cum_stride"][-1] == 32


# ---- border case for a stream that did not move (an extension beyond Table 2) ------------------------------------
def test_border_extension_is_in_bounds_window_containment(oracle):
    """Brute force: an output pixel is reusable iff every tap of its window that lies inside the map lies inside the
    rectangle (the taps in the zero padding read zeros in both frames)."""
    rng = np.random.default_rng(12)
    for trial in range(300):
        wa, ha = int(rng.integers(5, 20)), int(rng.integers(5, 20))
        k = int(rng.choice([1, 2, 3, 5, 7]))
        s = int(rng.choice([1, 2, 3]))
        p = int(rng.integers(0, k))
        if wa + 2 * p < k or ha + 2 * p < k:
            continue
        x, y = int(rng.integers(0, wa)), int(rng.integers(0, ha))
        w, h = int(rng.integers(1, wa - x + 1)), int(rng.integers(1, ha - y + 1))
        if trial % 3 == 0: x, w = 0, wa                     # touches both sides
        if trial % 4 == 0: y = 0
        if trial % 5 == 0: h = ha - y
        wo, ho = (wa + 2 * p - k) // s + 1, (ha + 2 * p - k) // s + 1
        want = np.zeros((ho, wo), bool)
        for oy in range(ho):
            for ox in range(wo):
                taps = [(oy * s - p + ky, ox * s - p + kx) for ky in range(k) for kx in range(k)]
                inb = [(a, b) for a, b in taps if 0 <= a < ha and 0 <= b < wa]
                want[oy, ox] = len(inb) > 0 and all(y <= a < y + h and x <= b < x + w for a, b in inb)
        got = oracle.dt_window_ext((x, y, w, h), k, s, p, wa, ha)
        mask = oracle.rasterize([got] if got else [], ho, wo).astype(bool)
        assert np.array_equal(mask, want), (wa, ha, k, s, p, (x, y, w, h), got)
        # away from the borders it is the printed rule
        if x > 0 and y > 0 and x + w < wa and y + h < ha:
            assert got == oracle.dt_window((x, y, w, h), k, s, p)


def test_border_extension_only_for_zero_motion(oracle):
    from paper_1712_01670_amd import synth
    layers = synth.vgg16()
    rects0 = [(0, 0, 224, 224)]
    plain = oracle.propagate(layers, 224, 224, rects0, 0, 0)
    ext = oracle.propagate(layers, 224, 224, rects0, 0, 0, extend_borders=True)
    moved = oracle.propagate(layers, 224, 224, rects0, 3, 0, extend_borders=True)
    moved_plain = oracle.propagate(layers, 224, 224, rects0, 3, 0)
    for t in range(len(layers) + 1):
        h, w = ext["hw"][t]
        assert ext["rects"][t].tolist() == [[0, 0, w, h]]                      # identical frames: everything reusable
        assert moved["rects"][t].tolist() == moved_plain["rects"][t].tolist()   # a moving stream: the printed rule
    # the printed rule loses a ring per layer: the last 14x14 maps keep almost nothing
    assert plain["rects"][len(layers)].size == 0 or np.prod(plain["rects"][len(layers)][0][2:]) <= 4


# ---- exact reuse maps (Section 5's propagation applied per pixel instead of per rectangle) ------------------------
def _np_window_and(mask, k, s, p, ignore_padding=False):
    """out[o] = AND over the k x k window at o*s - p of `mask`; taps outside the map count as `ignore_padding`."""
    H, W = mask.shape
    Ho, Wo = (H + 2 * p - k) // s + 1, (W + 2 * p - k) // s + 1
    pad = np.full((H + 2 * p + k, W + 2 * p + k), bool(ignore_padding))
    pad[p:p + H, p:p + W] = mask.astype(bool)
    out = np.ones((Ho, Wo), bool)
    for ky in range(k):
        for kx in range(k):
            out &= pad[ky:ky + (Ho - 1) * s + 1:s, kx:kx + (Wo - 1) * s + 1:s]
    return out


def _np_source_inside(mask, dx, dy):
    H, W = mask.shape
    ys, xs = np.mgrid[0:H, 0:W]
    return mask & (xs + dx >= 0) & (xs + dx < W) & (ys + dy >= 0) & (ys + dy < H)


def _np_exact_masks(layers, H, W, block_mask, B, mx, my, ext=False):
    from paper_1712_01670_amd import synth
    ext = ext and mx == 0 and my == 0
    rha = lambda m, d: int(np.sign(m)) * ((2 * abs(m) + d) // (2 * d))
    full = np.zeros((H, W), bool)
    px = np.kron(np.asarray(block_mask, bool), np.ones((B, B), bool))
    full[:px.shape[0], :px.shape[1]] = px[:H, :W]
    masks, cum = [_np_source_inside(full, mx, my)], [1]
    for L in layers:
        a = masks[L["in0"]]
        c = cum[L["in0"]]
        if L["type"] in (synth.CONV, synth.MAXPOOL, synth.AVGPOOL):
            m = _np_window_and(a, L["k"], L["s"], L["p"], ext)
            c *= L["s"]
        elif L["type"] == synth.LRN and L.get("within", 0):
            m = _np_window_and(a, L["k"], 1, (L["k"] - 1) // 2, ext)
        elif L["type"] == synth.ADD:
            m = a & masks[L["in1"]]
        elif L["type"] == synth.CONCAT:
            m = a.copy()
            for key in ("in1", "in2", "in3"):
                if L.get(key, -1) >= 0:
                    m &= masks[L[key]]
        elif L["type"] in (synth.FC, synth.SOFTMAX):
            m = np.zeros((1, 1) if L["type"] == synth.FC else a.shape, bool)
        else:
            m = a.copy()
        cum.append(c)
        masks.append(_np_source_inside(m, rha(mx, c), rha(my, c)))
    return masks


def _mixed_stack():
    from paper_1712_01670_amd import synth
    C_ = lambda k, s, p, i: dict(type=synth.CONV, k=k, s=s, p=p, cin=4, cout=4, relu=1, in0=i, in1=-1)
    return [C_(3, 1, 1, 0),                                                                   # 1
            C_(5, 1, 2, 1),                                                                   # 2
            dict(type=synth.MAXPOOL, k=2, s=2, p=0, cin=4, cout=4, relu=0, in0=2, in1=-1),    # 3
            C_(3, 1, 1, 3),                                                                   # 4  branch a
            C_(1, 1, 0, 3),                                                                   # 5  branch b
            dict(type=synth.ADD, k=1, s=1, p=0, cin=4, cout=4, relu=1, in0=4, in1=5),         # 6
            dict(type=synth.LRN, k=3, s=1, p=0, cin=4, cout=4, relu=0, in0=6, in1=-1, within=1, alpha=1e-4, beta=0.75, kappa=1.0),  # 7
            C_(3, 2, 1, 7),                                                                   # 8
            dict(type=synth.MAXPOOL, k=3, s=2, p=1, cin=4, cout=4, relu=0, in0=8, in1=-1),    # 9
            dict(type=synth.RELU, k=1, s=1, p=0, cin=4, cout=4, relu=0, in0=9, in1=-1),       # 10
            C_(7, 1, 3, 10),                                                                  # 11
            dict(type=synth.CONCAT, k=1, s=1, p=0, cin=8, cout=8, relu=0, in0=10, in1=11, in2=-1, in3=-1)]  # 12


@pytest.mark.parametrize("seed", range(6))
def test_exact_masks_are_the_per_pixel_rule(oracle, seed):
    # a pixel is reusable iff every tap of its window is reusable and inside the map, and its source is inside the
    # map: an independent array formulation (shifted slices of a padded map) on random block masks and motions
    rng = np.random.default_rng(seed)
    layers = _mixed_stack()
    H, W, B = 70, 92, 8                       # 8 x 11 blocks and a remainder strip on both axes
    bm = (rng.random((H // B, W // B)) < 0.8).astype(np.uint8)
    mx, my = (0, 0) if seed == 0 else (int(rng.integers(-9, 10)), int(rng.integers(-9, 10)))
    for ext in (False, True):
        got = oracle.propagate_masks(layers, H, W, bm, B, mx, my, extend_borders=ext)
        want = _np_exact_masks(layers, H, W, bm, B, mx, my, ext)
        for t, (g, w_) in enumerate(zip(got["masks"], want)):
            assert np.array_equal(g.astype(bool), w_), (t, ext)
        rects = oracle.propagate(layers, H, W, oracle.merge_blocks(bm, B), mx, my, extend_borders=ext)
        assert np.array_equal(got["dxy"], rects["dxy"]) and np.array_equal(got["hw"], rects["hw"])
        for t, m in enumerate(got["masks"]):   # the rectangles never claim a pixel the exact map does not
            r = oracle.rasterize(rects["rects"][t], *m.shape).astype(bool)
            assert not (r & ~m.astype(bool)).any(), t
        assert got["masks"][1].sum() > 0


def test_exact_masks_equal_the_rectangle_rule_for_a_single_rectangle(oracle):
    from paper_1712_01670_amd import synth
    layers = synth.vgg16()[:10]
    bm = np.zeros((6, 6), np.uint8)
    bm[1:5, 2:6] = 1                                                # one 4 x 4-block rectangle
    for (mx, my) in ((0, 0), (3, -2), (-16, 8)):
        got = oracle.propagate_masks(layers, 96, 96, bm, 16, mx, my)
        rects = oracle.propagate(layers, 96, 96, oracle.merge_blocks(bm, 16), mx, my)
        for t, m in enumerate(got["masks"]):
            assert len(rects["rects"][t]) <= 1
            assert np.array_equal(m, oracle.rasterize(rects["rects"][t], *m.shape)), (t, mx, my)


def test_exact_masks_do_not_pay_for_seams(oracle):
    # Section 4's arithmetic: two 5x5 blocks under a 3x3 kernel keep 3x3 pixels each (18) when they are propagated
    # apart, 3x8 = 24 as one 5x10 rectangle.  The exact map of their union holds 24 however Step 5 cuts it.
    from paper_1712_01670_amd import synth
    conv = [dict(type=synth.CONV, k=3, s=1, p=1, cin=1, cout=1, relu=0, in0=0, in1=-1)]
    bm = np.zeros((4, 5), np.uint8)
    bm[1, 1:3] = 1
    exact = oracle.propagate_masks(conv, 20, 25, bm, 5, 0, 0)["masks"][1]
    assert int(exact.sum()) == 24 and exact[6:9, 6:14].all()
    apart = oracle.propagate(conv, 20, 25, [(5, 5, 5, 5), (10, 5, 5, 5)], 0, 0)
    assert sum(int(r[2]) * int(r[3]) for r in apart["rects"][1]) == 18
    merged = oracle.propagate(conv, 20, 25, oracle.merge_blocks(bm, 5), 0, 0)
    assert [tuple(int(v) for v in r) for r in merged["rects"][1]] == [(6, 6, 8, 3)]
    # an L-shaped region: three rectangles' worth of seams in any decomposition, none in the exact map
    bm = np.zeros((4, 5), np.uint8)
    bm[0:3, 1] = 1
    bm[2, 1:4] = 1
    exact = oracle.propagate_masks(conv, 20, 25, bm, 5, 0, 0)["masks"][1]
    rect = oracle.propagate(conv, 20, 25, oracle.merge_blocks(bm, 5), 0, 0)["rects"][1]
    # column: x 6..8, y 1..13 (the map's top row is lost to the padding); bar: x 6..18, y 11..13
    assert int(exact.sum()) == 3 * 13 + 13 * 3 - 9
    assert sum(int(r[2]) * int(r[3]) for r in rect) < int(exact.sum())
