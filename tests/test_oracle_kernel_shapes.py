"""Pins for conv layers whose kernel is not square or is dilated (k2 / p2 / dil of a layer): the convolution against
torch in fp64, the region rule against brute-force window containment, the exact maps against brute force over the
taps, and the stream invariants on a stack made of such layers."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

from paper_1712_01670_amd import synth


CASES = [  # kh, kw, s, ph, pw, dil
    (1, 7, 1, 0, 3, 1), (7, 1, 1, 3, 0, 1), (3, 3, 1, 2, 2, 2), (3, 1, 2, 1, 0, 1), (5, 3, 1, 4, 2, 2),
    (2, 5, 3, 0, 1, 1), (3, 3, 2, 3, 3, 3), (1, 1, 1, 0, 0, 1),
]


@pytest.mark.parametrize("case", CASES)
def test_convolution_matches_torch(oracle, case):
    kh, kw, s, ph, pw, dil = case
    rng = np.random.default_rng(sum(case))
    x = rng.standard_normal((19, 23, 5)).astype(np.float32)
    w = rng.standard_normal((6, kh, kw, 5)).astype(np.float32)
    b = rng.standard_normal(6).astype(np.float32)
    got = oracle.conv_cached(x, w, b, kh, s, ph, False, k2=kw, p2=pw, dil=dil)
    want = F.conv2d(torch.from_numpy(x).double().permute(2, 0, 1)[None], torch.from_numpy(w).double().permute(0, 3, 1, 2),
                    torch.from_numpy(b).double(), stride=s, padding=(ph, pw), dilation=dil)[0].permute(1, 2, 0).numpy()
    assert got.shape == want.shape
    assert np.allclose(got, want, rtol=1e-6, atol=1e-6)
    # rows are k, columns k2: the transposed kernel with swapped paddings is the convolution of the transposed image
    if kh != kw:
        xt = np.ascontiguousarray(x.transpose(1, 0, 2))
        wt = np.ascontiguousarray(w.transpose(0, 2, 1, 3))
        assert np.array_equal(oracle.conv_cached(xt, wt, b, kw, s, pw, False, k2=kh, p2=ph, dil=dil).transpose(1, 0, 2), got)


@pytest.mark.parametrize("case", CASES)
def test_region_rule_is_window_containment(oracle, case):
    """An output pixel is in the propagated rectangle iff the whole span of its kernel lies in the input rectangle."""
    kh, kw, s, ph, pw, dil = case
    ew, eh = (kw - 1) * dil + 1, (kh - 1) * dil + 1
    rng = np.random.default_rng(1 + sum(case))
    for _ in range(60):
        x, y = int(rng.integers(0, 20)), int(rng.integers(0, 20))
        w, h = int(rng.integers(1, 25)), int(rng.integers(1, 25))
        got = oracle.dt_window2((x, y, w, h), ew, eh, s, pw, ph)
        ok = np.zeros((64, 64), bool)
        for oy in range(64):
            for ox in range(64):
                x0, y0 = ox * s - pw, oy * s - ph
                ok[oy, ox] = x0 >= x and x0 + ew <= x + w and y0 >= y and y0 + eh <= y + h
        if not ok.any():
            assert got is None
            continue
        ys, xs = np.nonzero(ok)
        assert got == (xs.min(), ys.min(), xs.max() - xs.min() + 1, ys.max() - ys.min() + 1)
        assert ok[ys.min():ys.max() + 1, xs.min():xs.max() + 1].all()


def _brute_masks(layers, H, W, bm, B, mx, my):
    """Exact maps by the definition: every tap of the window inside the map and reusable, source inside the map."""
    hw, cs, masks = [(H, W)], [1], []
    m0 = np.zeros((H, W), bool)
    for y in range(H):
        for x in range(W):
            by, bx = y // B, x // B
            m0[y, x] = by < bm.shape[0] and bx < bm.shape[1] and bool(bm[by, bx]) and 0 <= x + mx < W and 0 <= y + my < H
    masks.append(m0)
    for L in layers:
        ha, wa = hw[L["in0"]]
        ma = masks[L["in0"]]
        kh, kw, ph, pw, dil = synth.conv_geometry(L)
        s = L["s"]
        ho, wo = (ha + 2 * ph - ((kh - 1) * dil + 1)) // s + 1, (wa + 2 * pw - ((kw - 1) * dil + 1)) // s + 1
        c = cs[L["in0"]] * s
        rd = lambda v: int(np.sign(v) * ((2 * abs(v) + c) // (2 * c)))
        dx, dy = rd(mx), rd(my)
        m = np.zeros((ho, wo), bool)
        for y in range(ho):
            for x in range(wo):
                ok = 0 <= x + dx < wo and 0 <= y + dy < ho
                for ky in range(kh):
                    for kx in range(kw):
                        iy, ix = y * s - ph + ky * dil, x * s - pw + kx * dil
                        ok = ok and 0 <= iy < ha and 0 <= ix < wa and bool(ma[iy, ix])
                m[y, x] = ok
        hw.append((ho, wo)); cs.append(c); masks.append(m)
    return masks


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_exact_maps_against_brute_force_over_the_taps(oracle, seed):
    layers = synth.factorised_net(4)
    H, W, B = 48, 64, 8
    rng = np.random.default_rng(seed)
    bm = (rng.random((H // B, W // B)) < 0.8).astype(np.uint8)
    mx, my = int(rng.integers(-6, 7)), int(rng.integers(-6, 7))
    got = oracle.propagate_masks(layers, H, W, bm, B, mx, my)
    want = _brute_masks(layers, H, W, bm, B, mx, my)
    assert any(m.any() for m in want[2:])
    for t, m in enumerate(want):
        assert np.array_equal(got["masks"][t].astype(bool), m), t
    # the rectangles of the same frame stay inside the maps (a dilated kernel's rectangle asks for the whole span)
    rects = oracle.propagate(layers, H, W, oracle.merge_blocks(bm, B), mx, my)
    for t in range(len(layers) + 1):
        r = oracle.rasterize(rects["rects"][t], *want[t].shape).astype(bool)
        assert not (r & ~want[t]).any(), t


def test_stream_invariants_on_a_stack_of_such_layers(oracle):
    layers = synth.factorised_net(8)       # total stride 4
    ws, bs = synth.he_weights(layers, 3, bias_scale=0.1)
    H = W = 64
    # exact shift by a multiple of the total stride with one fresh patch: bit-identical to the full forward
    f1, f2 = synth.shifted_pair(11, H, W, (8, -4))
    f2 = f2.copy()
    f2[24:40, 8:24] = np.random.default_rng(3).integers(0, 256, (16, 16, 3))
    for exact in (False, True):
        st = oracle.Stream(layers, ws, bs, H, W, 3, block=8, radius=8, exact_masks=exact)
        st.step(f1)
        r = st.step(f2)
        assert r["match"]["gmv"].tolist() == [-8, 4]
        reused = (r["masks"][-1].sum() if exact else sum(int(q[2]) * int(q[3]) for q in r["rects"][2]))
        assert reused > 0
        full = oracle.Stream(layers, ws, bs, H, W, 3).step(f2)["tensors"]
        for a, b in zip(r["tensors"], full):
            assert np.array_equal(a, b)
    # unrelated frames: nothing reusable, the full forward
    rng = np.random.default_rng(6)
    g1, g2 = (rng.integers(0, 256, (H, W, 3)).astype(np.uint8) for _ in range(2))
    st = oracle.Stream(layers, ws, bs, H, W, 3, block=8, radius=8)
    st.step(g1)
    for a, b in zip(st.step(g2)["tensors"], oracle.Stream(layers, ws, bs, H, W, 3).step(g2)["tensors"]):
        assert np.array_equal(a, b)
