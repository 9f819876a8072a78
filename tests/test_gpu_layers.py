"""GPU parity of the per-layer entry points against the oracle (Section 5 "Reuse")."""
import numpy as np
import pytest
import torch

from paper_1712_01670_amd import binding, synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _to_dev(a, bf16):
    t = torch.from_numpy(np.ascontiguousarray(a)).to(DEV)
    return t.to(torch.bfloat16) if bf16 else t


def _to_np(t):
    return t.float().cpu().numpy()


def _rel_err(got, want):
    scale = max(float(np.abs(want).max()), 1e-30)
    return float(np.abs(got - want).max()) / scale


def _layer(cin, cout, k, s, p, relu):
    return dict(type=synth.CONV, k=k, s=s, p=p, cin=cin, cout=cout, relu=int(relu), in0=0, in1=-1)


CONV_CASES = [
    # H, W, cin, cout, k, s, p, relu
    (20, 37, 3, 16, 3, 1, 1, True),      # first-layer shape, ragged tiles
    (33, 18, 16, 32, 3, 2, 1, True),     # stride 2
    (16, 16, 32, 32, 3, 1, 1, False),
    (29, 31, 64, 64, 3, 1, 1, True),     # 64-channel, several tiles and a ragged tail
    (14, 14, 128, 256, 3, 1, 1, True),   # small map, wide
    (28, 28, 64, 128, 1, 1, 0, True),    # 1x1
    (28, 28, 128, 64, 1, 2, 0, False),   # 1x1 stride 2 (projection shortcut)
    (40, 40, 3, 64, 7, 2, 3, True),      # stem
    (9, 11, 5, 7, 3, 1, 0, True),        # odd channel counts: scalar load path
    (10, 10, 40, 136, 3, 1, 1, True),    # cin not a multiple of the chunk, cout ragged
]


@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("case", CONV_CASES)
def test_full_conv_matches_oracle(oracle, case, bf16):
    H, W, cin, cout, k, s, p, relu = case
    print(f"[conv] case={case} bf16={bf16}", flush=True)
    rng = np.random.default_rng(abs(hash(case)) % 2 ** 31)
    x = rng.standard_normal((2, H, W, cin)).astype(np.float32)
    w = (rng.standard_normal((cout, k, k, cin)) * np.sqrt(2.0 / (cin * k * k))).astype(np.float32)
    b = (rng.standard_normal(cout) * 0.1).astype(np.float32)
    if bf16:
        x, w = oracle.round_bf16(x), oracle.round_bf16(w)
    got = _to_np(binding.dc_cached_conv_layer(_layer(cin, cout, k, s, p, relu), _to_dev(x, bf16), _to_dev(w, bf16),
                                              torch.from_numpy(b).to(DEV)))
    for n in range(2):
        want = oracle.conv_cached(x[n], w, b, k, s, p, relu, bf16=bf16)
        assert got[n].shape == want.shape
        assert _rel_err(got[n], want) <= (2e-2 if bf16 else 1e-4), (case, n)


@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("case", [(40, 52, 16, 64, 3, 1, 1), (31, 45, 32, 32, 3, 2, 1), (24, 24, 64, 160, 1, 1, 0)])
def test_cached_conv_matches_oracle(oracle, case, bf16):
    H, W, cin, cout, k, s, p = case
    print(f"[cached conv] case={case} bf16={bf16}", flush=True)
    rng = np.random.default_rng(sum(case))
    n = 3
    x = rng.standard_normal((n, H, W, cin)).astype(np.float32)
    w = (rng.standard_normal((cout, k, k, cin)) * np.sqrt(2.0 / (cin * k * k))).astype(np.float32)
    b = (rng.standard_normal(cout) * 0.1).astype(np.float32)
    Ho, Wo = (H + 2 * p - k) // s + 1, (W + 2 * p - k) // s + 1
    cache = rng.standard_normal((n, Ho, Wo, cout)).astype(np.float32)
    if bf16:
        x, w, cache = oracle.round_bf16(x), oracle.round_bf16(w), oracle.round_bf16(cache)
    # per-stream regions: stream 0 large rect + sliver, stream 1 nothing, stream 2 everything that fits
    regions = [
        (np.array([[2, 1, Wo - 9, Ho - 9], [Wo - 6, 3, 2, 5]], np.int32), (3, -1)),
        (np.zeros((0, 4), np.int32), (0, 0)),
        (np.array([[0, 0, Wo - 2, Ho - 1]], np.int32), (2, 1)),
    ]
    got = _to_np(binding.dc_cached_conv_layer(_layer(cin, cout, k, s, p, True), _to_dev(x, bf16), _to_dev(w, bf16),
                                              torch.from_numpy(b).to(DEV), cache_prev=_to_dev(cache, bf16),
                                              regions=regions))
    for i in range(n):
        mask = oracle.rasterize(regions[i][0], Ho, Wo)
        want = oracle.conv_cached(x[i], w, b, k, s, p, True, cache_prev=cache[i], mask=mask, dxy=regions[i][1], bf16=bf16)
        m = mask.astype(bool)
        assert np.array_equal(got[i][m], want[m]), "copied pixels must be bit-identical"
        assert _rel_err(got[i], want) <= (2e-2 if bf16 else 1e-4), (case, i)


def _random_regions(rng, oracle, Ho, Wo):
    """Disjoint rectangles (merged from a random grid mask) whose sources stay inside the map."""
    cell = int(rng.choice([2, 3, 5]))
    mask = (rng.random((Ho // cell, Wo // cell)) < rng.choice([0.3, 0.6, 0.9])).astype(np.uint8)
    rects = oracle.merge_blocks(mask, cell)
    dx, dy = int(rng.integers(-4, 5)), int(rng.integers(-4, 5))
    out = []
    for x, y, w, h in rects.tolist():
        x0, y0 = max(x, -dx, 0), max(y, -dy, 0)
        x1, y1 = min(x + w, Wo - dx, Wo), min(y + h, Ho - dy, Ho)
        if x1 > x0 and y1 > y0:
            out.append([x0, y0, x1 - x0, y1 - y0])
    return np.array(out, np.int32).reshape(-1, 4), (dx, dy)


@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("seed", range(6))
def test_cached_conv_random_regions(oracle, seed, bf16):
    """Random layer shapes of both kernel families with random disjoint reusable rectangles per stream:
    copied pixels bit-identical, recomputed ones within tolerance, nothing else touched."""
    rng = np.random.default_rng(100 + seed)
    k, s, p = [(3, 1, 1), (3, 1, 1), (1, 1, 0), (3, 2, 1), (5, 1, 2), (3, 1, 0)][seed]
    cin = int(rng.choice([16, 32, 64])) if seed < 2 else int(rng.choice([8, 16, 24]))
    cout = int(rng.choice([64, 128])) if seed < 2 else int(rng.choice([16, 40, 64]))
    H, W = int(rng.integers(18, 40)), int(rng.integers(18, 44))
    print(f"[cached conv random] seed={seed} bf16={bf16} {H}x{W} cin={cin} cout={cout} k={k} s={s} p={p}", flush=True)
    n = 3
    x = rng.standard_normal((n, H, W, cin)).astype(np.float32)
    w = (rng.standard_normal((cout, k, k, cin)) * np.sqrt(2.0 / (cin * k * k))).astype(np.float32)
    b = (rng.standard_normal(cout) * 0.1).astype(np.float32)
    Ho, Wo = (H + 2 * p - k) // s + 1, (W + 2 * p - k) // s + 1
    cache = rng.standard_normal((n, Ho, Wo, cout)).astype(np.float32)
    if bf16:
        x, w, cache = oracle.round_bf16(x), oracle.round_bf16(w), oracle.round_bf16(cache)
    regions = [_random_regions(rng, oracle, Ho, Wo) for _ in range(n)]
    got = _to_np(binding.dc_cached_conv_layer(_layer(cin, cout, k, s, p, True), _to_dev(x, bf16), _to_dev(w, bf16),
                                              torch.from_numpy(b).to(DEV), cache_prev=_to_dev(cache, bf16),
                                              regions=regions))
    for i in range(n):
        mask = oracle.rasterize(regions[i][0], Ho, Wo)
        want = oracle.conv_cached(x[i], w, b, k, s, p, True, cache_prev=cache[i], mask=mask, dxy=regions[i][1], bf16=bf16)
        m = mask.astype(bool)
        assert np.array_equal(got[i][m], want[m]), "copied pixels must be bit-identical"
        assert _rel_err(got[i], want) <= (2e-2 if bf16 else 1e-4), (seed, i)


# 3x3 stride-1 layers with whole 64-byte channel rows take the compile-time-shaped GEMM kernel; the launch
# heuristics are overridden so that every shape of that kernel is exercised at a size the oracle handles:
# (arrangement, units per workgroup, K split, chunk index); arrangement 1 exists for bf16 only.
FAST_CASES = [
    # H, W, cin, cout, tuning
    (22, 30, 32, 64, (0, 1, -1, 0)),     # one unit per workgroup
    (22, 30, 64, 64, (0, 5, -1, 1)),     # odd unit count, longer channel chunk
    (22, 30, 64, 128, (0, 16, 1, 0)),    # full workgroup tile, more units in the tile than in the map's last group
    (14, 14, 128, 64, (0, 3, 4, 0)),     # K split among 4 workgroups + reduction kernel
    (13, 17, 256, 128, (0, 2, 8, 1)),    # K split, ragged map
    (22, 30, 64, 128, (1, 7, 1, 0)),     # 128 channels per workgroup
    (22, 30, 64, 256, (1, 16, 2, 0)),    # ... with a K split
    (22, 30, 64, 64, (2, 11, 1, 0)),     # 64 channels per workgroup in two blocks per wavefront (bf16)
    (14, 14, 128, 192, (2, 4, 2, 1)),
    (19, 23, 128, 128, (-1, -1, -1, -1)),  # the library's own choice
    (22, 30, 64, 64, (3, -1, -1, -1)),    # bf16: persistent kernel with the weights in registers (plain weights)
    (37, 41, 64, 128, (3, -1, -1, -1)),   # ... two channel tiles, more unit groups than one step, ragged map
    (22, 30, 64, 128, (4, 18, 1, 0)),     # bf16: twelve wavefronts, 18 units per workgroup (96 units: the last group holds 6)
    (45, 61, 32, 256, (4, 13, 1, 0)),     # ... 13 units: one row of wavefronts with three units, five with two
    (30, 34, 96, 128, (4, 17, 3, 0)),     # ... with a K split
]


@pytest.mark.parametrize("cached", [False, True])
@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("case", FAST_CASES)
def test_fast_conv_kernel_shapes(oracle, case, bf16, cached):
    H, W, cin, cout, tuning = case
    print(f"[fast conv] case={case} bf16={bf16} cached={cached}", flush=True)
    rng = np.random.default_rng(H * 1000 + W * 10 + cin + cout)
    n = 2
    x = rng.standard_normal((n, H, W, cin)).astype(np.float32)
    w = (rng.standard_normal((cout, 3, 3, cin)) * np.sqrt(2.0 / (cin * 9))).astype(np.float32)
    b = (rng.standard_normal(cout) * 0.1).astype(np.float32)
    cache = rng.standard_normal((n, H, W, cout)).astype(np.float32)
    if bf16:
        x, w, cache = oracle.round_bf16(x), oracle.round_bf16(w), oracle.round_bf16(cache)
    regions = None
    if cached:
        regions = [(np.array([[1, 2, W - 7, H - 6], [W - 5, 1, 3, 4]], np.int32), (2, -1)),
                   (np.array([[0, 0, W - 1, H - 3]], np.int32), (1, 2))]
    binding.dc_conv_tuning(*tuning)
    try:
        layer, wd = _layer(cin, cout, 3, 1, 1, True), _to_dev(w, bf16)
        got = _to_np(binding.dc_cached_conv_layer(layer, _to_dev(x, bf16), wd, torch.from_numpy(b).to(DEV),
                                                  cache_prev=_to_dev(cache, bf16) if cached else None, regions=regions))
        # the same layer reading the packed copy of the weights: same products in the same order
        wp = binding.dc_pack_conv_weights(layer, wd)
        assert wp is not None
        es = 2 if bf16 else 4
        raw = wd.view(torch.uint8).cpu().numpy().reshape(cout // 16, 16, 9, cin * es // 64, 64)
        assert np.array_equal(wp.view(torch.uint8).cpu().numpy().reshape(cout // 16, cin * es // 64, 9, 16, 64),
                              raw.transpose(0, 3, 2, 1, 4)), "layout [cout/16][64-byte chunk][tap][16][64 bytes]"
        # plain weights zeroed: the result shows that the kernel reads the packed copy
        plain = wd if tuning[0] == 3 else torch.zeros_like(wd)     # arrangement 3 reads the plain layout
        got_p = _to_np(binding.dc_cached_conv_layer(layer, _to_dev(x, bf16), plain, torch.from_numpy(b).to(DEV),
                                                    cache_prev=_to_dev(cache, bf16) if cached else None, regions=regions,
                                                    packed=wp))
    finally:
        binding.dc_conv_tuning()
    assert np.array_equal(got, got_p), "packed weights must not change a bit"
    for i in range(n):
        if cached:
            mask = oracle.rasterize(regions[i][0], H, W)
            want = oracle.conv_cached(x[i], w, b, 3, 1, 1, True, cache_prev=cache[i], mask=mask, dxy=regions[i][1], bf16=bf16)
            m = mask.astype(bool)
            assert np.array_equal(got[i][m], want[m]), "copied pixels must be bit-identical"
        else:
            want = oracle.conv_cached(x[i], w, b, 3, 1, 1, True, bf16=bf16)
        assert _rel_err(got[i], want) <= (2e-2 if bf16 else 1e-4), (case, i)


def test_register_weight_kernel_without_relu_and_bias(oracle):
    """The persistent bf16 kernel for 64 input channels: negative outputs survive when the layer has no ReLU,
    and a missing bias is zero."""
    H, W, cin, cout = 26, 34, 64, 64
    rng = np.random.default_rng(5)
    x = oracle.round_bf16(rng.standard_normal((3, H, W, cin)).astype(np.float32))
    w = oracle.round_bf16((rng.standard_normal((cout, 3, 3, cin)) * np.sqrt(2.0 / (cin * 9))).astype(np.float32))
    binding.dc_conv_tuning(3, -1, -1, -1)
    try:
        got = _to_np(binding.dc_cached_conv_layer(_layer(cin, cout, 3, 1, 1, False), _to_dev(x, True), _to_dev(w, True), None))
    finally:
        binding.dc_conv_tuning()
    assert (got < 0).mean() > 0.3
    for i in range(3):
        want = oracle.conv_cached(x[i], w, None, 3, 1, 1, False, bf16=True)
        assert _rel_err(got[i], want) <= 2e-2


@pytest.mark.parametrize("cached", [False, True])
@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("cout", [16, 32, 64, 128])
def test_first_layer_kernel(oracle, cout, bf16, cached):
    """Input pixels of one 16-byte vector (4 fp32 / 8 bf16 channels): the kernel without LDS staging."""
    H, W = 21, 26
    cin = 8 if bf16 else 4
    print(f"[first layer] cout={cout} bf16={bf16} cached={cached}", flush=True)
    rng = np.random.default_rng(cout + 7)
    n = 2
    x = rng.standard_normal((n, H, W, cin)).astype(np.float32)
    w = (rng.standard_normal((cout, 3, 3, cin)) * np.sqrt(2.0 / (cin * 9))).astype(np.float32)
    b = (rng.standard_normal(cout) * 0.1).astype(np.float32)
    cache = rng.standard_normal((n, H, W, cout)).astype(np.float32)
    if bf16:
        x, w, cache = oracle.round_bf16(x), oracle.round_bf16(w), oracle.round_bf16(cache)
    regions = None
    if cached:
        regions = [(np.array([[3, 1, W - 8, H - 5]], np.int32), (-2, 1)), (np.zeros((0, 4), np.int32), (0, 0))]
    got = _to_np(binding.dc_cached_conv_layer(_layer(cin, cout, 3, 1, 1, True), _to_dev(x, bf16), _to_dev(w, bf16),
                                              torch.from_numpy(b).to(DEV),
                                              cache_prev=_to_dev(cache, bf16) if cached else None, regions=regions))
    for i in range(n):
        if cached:
            mask = oracle.rasterize(regions[i][0], H, W)
            want = oracle.conv_cached(x[i], w, b, 3, 1, 1, True, cache_prev=cache[i], mask=mask, dxy=regions[i][1], bf16=bf16)
            m = mask.astype(bool)
            assert np.array_equal(got[i][m], want[m])
        else:
            want = oracle.conv_cached(x[i], w, b, 3, 1, 1, True, bf16=bf16)
        assert _rel_err(got[i], want) <= (2e-2 if bf16 else 1e-4), (cout, i)


@pytest.mark.parametrize("cached", [False, True])
@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("cout", [16, 64, 96])
@pytest.mark.parametrize("geom", [(7, 2, 3), (11, 4, 0), (11, 4, 2)])
def test_stem_kernel(oracle, geom, cout, bf16, cached):
    """7x7 stride-2 and 11x11 stride-4 convolutions over 16-byte input pixels (the first layers of the residual and
    the AlexNet-style networks); odd and even sizes, so that the last output row reads past the input on one side
    only."""
    H, W = (45, 54) if geom[0] == 7 else (75, 91)
    k, s, p = geom
    Ho, Wo = (H + 2 * p - k) // s + 1, (W + 2 * p - k) // s + 1
    cin = 8 if bf16 else 4
    print(f"[stem] geom={geom} cout={cout} bf16={bf16} cached={cached}", flush=True)
    rng = np.random.default_rng(cout + 11)
    n = 2
    x = rng.standard_normal((n, H, W, cin)).astype(np.float32)
    w = (rng.standard_normal((cout, k, k, cin)) * np.sqrt(2.0 / (cin * k * k))).astype(np.float32)
    b = (rng.standard_normal(cout) * 0.1).astype(np.float32)
    cache = rng.standard_normal((n, Ho, Wo, cout)).astype(np.float32)
    if bf16:
        x, w, cache = oracle.round_bf16(x), oracle.round_bf16(w), oracle.round_bf16(cache)
    regions = None
    if cached:
        regions = [(np.zeros((0, 4), np.int32), (0, 0)), (np.array([[2, 3, Wo - 9, Ho - 6], [Wo - 6, 4, 3, 6]], np.int32), (1, -2))]
    got = _to_np(binding.dc_cached_conv_layer(_layer(cin, cout, k, s, p, True), _to_dev(x, bf16), _to_dev(w, bf16),
                                              torch.from_numpy(b).to(DEV),
                                              cache_prev=_to_dev(cache, bf16) if cached else None, regions=regions))
    assert got.shape == (n, Ho, Wo, cout)
    for i in range(n):
        if cached:
            mask = oracle.rasterize(regions[i][0], Ho, Wo)
            want = oracle.conv_cached(x[i], w, b, k, s, p, True, cache_prev=cache[i], mask=mask, dxy=regions[i][1], bf16=bf16)
            m = mask.astype(bool)
            assert np.array_equal(got[i][m], want[m])
        else:
            want = oracle.conv_cached(x[i], w, b, k, s, p, True, bf16=bf16)
        assert _rel_err(got[i], want) <= (2e-2 if bf16 else 1e-4), (cout, i)


def test_cached_conv_everything_reusable_launches_no_gemm(oracle):
    rng = np.random.default_rng(1)
    x = rng.standard_normal((1, 16, 16, 16)).astype(np.float32)
    w = rng.standard_normal((32, 3, 3, 16)).astype(np.float32)
    cache = rng.standard_normal((1, 16, 16, 32)).astype(np.float32)
    got = _to_np(binding.dc_cached_conv_layer(_layer(16, 32, 3, 1, 1, True), _to_dev(x, False), _to_dev(w, False), None,
                                              cache_prev=_to_dev(cache, False),
                                              regions=[(np.array([[0, 0, 16, 16]], np.int32), (0, 0))]))
    assert np.array_equal(got, cache)


@pytest.mark.parametrize("bf16", [False, True])
def test_uncached_layers(oracle, bf16):
    rng = np.random.default_rng(2)
    x = rng.standard_normal((2, 23, 30, 24)).astype(np.float32)
    y = rng.standard_normal((2, 23, 30, 24)).astype(np.float32)
    if bf16:
        x, y = oracle.round_bf16(x), oracle.round_bf16(y)
    for k, s, p in [(2, 2, 0), (3, 2, 1)]:
        got = _to_np(binding.dc_maxpool_layer(_to_dev(x, bf16), k, s, p))
        for n in range(2):
            assert np.array_equal(got[n], oracle.maxpool(x[n], k, s, p))
    for relu in (0, 1):
        got = _to_np(binding.dc_add_layer(_to_dev(x, bf16), _to_dev(y, bf16), relu))
        assert np.array_equal(got, oracle.add(x, y, relu, bf16=bf16))
    f = rng.integers(0, 256, (2, 9, 11, 3)).astype(np.uint8)
    dt = binding.DC_BF16 if bf16 else binding.DC_F32
    got = _to_np(binding.dc_frame_to_tensor(torch.from_numpy(f).to(DEV), dt))
    assert np.array_equal(got, oracle.frame_to_tensor(f))
    for ct in (4, 8):      # a tensor pixel of exactly 16 bytes (fp32 x 4, bf16 x 8) takes the per-pixel kernel
        got = _to_np(binding.dc_frame_to_tensor(torch.from_numpy(f).to(DEV), dt, c_tensor=ct))
        assert np.array_equal(got[..., :3], oracle.frame_to_tensor(f)) and not got[..., 3:].any()
    # element counts that are not whole 16-byte vectors
    xs, ys = x[:, :5, :7, :3].copy(), y[:, :5, :7, :3].copy()
    for relu in (0, 1):
        got = _to_np(binding.dc_add_layer(_to_dev(xs, bf16), _to_dev(ys, bf16), relu))
        assert np.array_equal(got, oracle.add(xs, ys, relu, bf16=bf16))


@pytest.mark.parametrize("bf16", [False, True])
def test_lrn_avgpool_concat_softmax_layers(oracle, bf16):
    """The un-cached layer types of Table 2 besides pooling and add, each against the oracle."""
    print(f"[more layers] bf16={bf16}", flush=True)
    rng = np.random.default_rng(9)
    tol = 2e-2 if bf16 else 1e-4
    n = 2
    for ch in (24, 7, 8):          # whole 16-byte vectors per pixel (several, one) and an odd channel count
        x = (rng.standard_normal((n, 13, 17, ch)) * 2).astype(np.float32)
        if bf16:
            x = oracle.round_bf16(x)
        xd = _to_dev(x, bf16)
        for size, within in [(5, False), (3, False), (1, False), (7, False), (3, True), (5, True)]:
            got = _to_np(binding.dc_lrn_layer(xd, size, 0.5, 0.75, 2.0, within))
            for i in range(n):
                assert _rel_err(got[i], oracle.lrn(x[i], size, 0.5, 0.75, 2.0, within, bf16=bf16)) <= tol, (ch, size, within)
        for k, s, p in [(3, 2, 1), (2, 2, 0), (13, 1, 0), (5, 3, 2)]:
            got = _to_np(binding.dc_avgpool_layer(xd, k, s, p))
            for i in range(n):
                assert _rel_err(got[i], oracle.avgpool(x[i], k, s, p, bf16=bf16)) <= tol, (ch, k, s, p)
            got = _to_np(binding.dc_maxpool_layer(xd, k, s, p))
            for i in range(n):
                assert np.array_equal(got[i], oracle.maxpool(x[i], k, s, p)), (ch, k, s, p)
    for cs in [(24, 8, 16), (24, 3), (5, 7, 24, 1), (8, 8)]:       # whole 16-byte vectors and odd channel counts
        parts = [np.ascontiguousarray(rng.standard_normal((n, 13, 17, c)).astype(np.float32)) for c in cs]
        if bf16:
            parts = [oracle.round_bf16(q) for q in parts]
        got = _to_np(binding.dc_concat_layer([_to_dev(q, bf16) for q in parts]))
        for i in range(n):
            assert np.array_equal(got[i], oracle.concat([q[i] for q in parts])), cs
    for c in (10, 64, 1000, 1024, 1500):      # up to 1024 channels stay in registers
        v = (rng.standard_normal((n, 2, 3, c)) * 4).astype(np.float32)
        if bf16:
            v = oracle.round_bf16(v)
        got = _to_np(binding.dc_softmax_layer(_to_dev(v, bf16)))
        for i in range(n):
            want = oracle.softmax(v[i], bf16=bf16)
            assert np.abs(got[i] - want).max() <= tol * max(float(want.max()), 1e-30), c


@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("n,shape,cout", [(1, (6, 6, 32), 100), (3, (5, 5, 7), 33), (20, (1, 1, 256), 64), (5, (2, 3, 24), 1),
                                          (16, (2, 2, 64), 30), (37, (3, 3, 16), 50), (18, (1, 1, 40), 3)])
def test_fully_connected_layer(oracle, n, shape, cout, bf16):
    print(f"[fc] n={n} shape={shape} cout={cout} bf16={bf16}", flush=True)
    rng = np.random.default_rng(n * 100 + cout)
    K = int(np.prod(shape))
    x = rng.standard_normal((n,) + shape).astype(np.float32)
    w = (rng.standard_normal((cout, K)) * np.sqrt(2.0 / K)).astype(np.float32)
    b = (rng.standard_normal(cout) * 0.1).astype(np.float32)
    if bf16:
        x, w = oracle.round_bf16(x), oracle.round_bf16(w)
    for relu, bias in [(True, b), (False, None)]:
        got = _to_np(binding.dc_fc_layer(_to_dev(x, bf16), _to_dev(w, bf16), None if bias is None else torch.from_numpy(bias).to(DEV), relu))
        assert got.shape == (n, 1, 1, cout)
        want = np.stack([oracle.fc(x[i], w, bias, relu, bf16=bf16) for i in range(n)])
        assert _rel_err(got, want) <= (2e-2 if bf16 else 1e-4)


PW_CASES = [
    # H, W, cin, cout, stride
    (13, 18, 64, 64, 1),       # one chunk in bf16, two in fp32
    (13, 18, 96, 24, 1),       # last chunk half empty (bf16), cout below one channel tile
    (9, 9, 1024, 72, 1),       # more chunks than ring stages; channel tile with a tail
    (14, 14, 256, 200, 1),
    (8, 8, 8, 8, 1),           # a single 16-byte vector per pixel (bf16)
    (27, 21, 128, 136, 2),     # strided projection, odd map
    (28, 28, 64, 256, 2),
]


@pytest.fixture
def pw_tile(request):
    """Forces the 1x1 kernel's tile (units per workgroup) for one test."""
    binding.dc_conv_tuning(units_per_workgroup=request.param)
    yield request.param
    binding.dc_conv_tuning()


@pytest.mark.parametrize("cached", [False, True])
@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("pw_tile", [4, 8], indirect=True)
@pytest.mark.parametrize("case", PW_CASES)
def test_pointwise_kernel(oracle, case, pw_tile, bf16, cached):
    """1x1 convolutions (stride 1 and 2) on the GEMM kernel with the staged K ring, both tile sizes."""
    H, W, cin, cout, s = case
    print(f"[pointwise] case={case} tile={pw_tile} bf16={bf16} cached={cached}", flush=True)
    rng = np.random.default_rng(sum(case) + 3)
    n = 3
    Ho, Wo = (H - 1) // s + 1, (W - 1) // s + 1
    x = rng.standard_normal((n, H, W, cin)).astype(np.float32)
    w = (rng.standard_normal((cout, 1, 1, cin)) * np.sqrt(2.0 / cin)).astype(np.float32)
    b = (rng.standard_normal(cout) * 0.1).astype(np.float32)
    cache = rng.standard_normal((n, Ho, Wo, cout)).astype(np.float32)
    if bf16:
        x, w, cache = oracle.round_bf16(x), oracle.round_bf16(w), oracle.round_bf16(cache)
    regions = None
    if cached:
        regions = [(np.array([[1, 0, Wo - 3, Ho - 2]], np.int32), (1, 1)), (np.zeros((0, 4), np.int32), (0, 0)),
                   (np.array([[0, 1, 2, Ho - 2], [3, 2, Wo - 4, 3]], np.int32), (1, 0))]
    got = _to_np(binding.dc_cached_conv_layer(_layer(cin, cout, 1, s, 0, True), _to_dev(x, bf16), _to_dev(w, bf16),
                                              torch.from_numpy(b).to(DEV),
                                              cache_prev=_to_dev(cache, bf16) if cached else None, regions=regions))
    assert got.shape == (n, Ho, Wo, cout)
    for i in range(n):
        if cached:
            mask = oracle.rasterize(regions[i][0], Ho, Wo)
            want = oracle.conv_cached(x[i], w, b, 1, s, 0, True, cache_prev=cache[i], mask=mask, dxy=regions[i][1], bf16=bf16)
            m = mask.astype(bool)
            assert np.array_equal(got[i][m], want[m])
        else:
            want = oracle.conv_cached(x[i], w, b, 1, s, 0, True, bf16=bf16)
        assert _rel_err(got[i], want) <= (2e-2 if bf16 else 1e-4), (case, i)


@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("case", [(20, 24, 4, 32, 3, 1, 1), (20, 24, 64, 64, 3, 1, 1), (20, 24, 64, 128, 1, 1, 0), (21, 25, 32, 48, 5, 2, 2),
                                  (21, 25, 6, 10, 3, 1, 1), (12, 12, 512, 64, 3, 1, 1)])
def test_leaky_relu_in_every_conv_kernel(oracle, case, bf16):
    """relu = 2 (leaky, slope 0.1) in the epilogue of the first-layer, 3x3, 1x1, general, element-load and split-K
    kernels."""
    H, W, cin, cout, k, s, p = case
    if bf16 and cin == 4:
        cin = 8
    print(f"[leaky] case={case} bf16={bf16}", flush=True)
    rng = np.random.default_rng(sum(case) + 1)
    x = rng.standard_normal((2, H, W, cin)).astype(np.float32)
    w = (rng.standard_normal((cout, k, k, cin)) * np.sqrt(2.0 / (cin * k * k))).astype(np.float32)
    b = (rng.standard_normal(cout) * 0.1).astype(np.float32)
    if bf16:
        x, w = oracle.round_bf16(x), oracle.round_bf16(w)
    got = _to_np(binding.dc_cached_conv_layer(_layer(cin, cout, k, s, p, 2), _to_dev(x, bf16), _to_dev(w, bf16), torch.from_numpy(b).to(DEV)))
    for i in range(2):
        want = oracle.conv_cached(x[i], w, b, k, s, p, 2, bf16=bf16)
        assert (want < 0).any()
        assert _rel_err(got[i], want) <= (2e-2 if bf16 else 1e-4), (case, i)


# Launches of the general kernel with at least three workgroups on every two CUs switch to short stages of the
# narrowest channel chunk (one kernel row of taps, or about a dozen taps where four wavefronts share a stage):
# shapes that reach that many workgroups at a size the oracle still handles.
SHORT_STAGE_CASES = [
    # n, H, W, cin, cout, k, s, p
    (12, 64, 64, 32, 128, 3, 2, 1),     # 384 workgroups of 4 units x 64 channels: 3 taps per stage
    (6, 48, 48, 16, 128, 5, 1, 2),      # 432 workgroups: 5 taps per stage
    (16, 28, 28, 16, 32, 5, 1, 2),      # 392 workgroups of 2 units x 32 channels: 13 + 12 taps (tap tail)
    (12, 62, 66, 40, 72, 3, 2, 0),      # channel tail in the chunk, ragged channel tile, no padding
]


@pytest.mark.parametrize("cached", [False, True])
@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("case", SHORT_STAGE_CASES)
def test_general_kernel_short_stages(oracle, case, bf16, cached):
    n, H, W, cin, cout, k, s, p = case
    print(f"[short stages] case={case} bf16={bf16} cached={cached}", flush=True)
    rng = np.random.default_rng(sum(case) + 7)
    x = rng.standard_normal((n, H, W, cin)).astype(np.float32)
    w = (rng.standard_normal((cout, k, k, cin)) * np.sqrt(2.0 / (cin * k * k))).astype(np.float32)
    b = (rng.standard_normal(cout) * 0.1).astype(np.float32)
    Ho, Wo = (H + 2 * p - k) // s + 1, (W + 2 * p - k) // s + 1
    cache = rng.standard_normal((n, Ho, Wo, cout)).astype(np.float32)
    if bf16:
        x, w, cache = oracle.round_bf16(x), oracle.round_bf16(w), oracle.round_bf16(cache)
    regions = None
    if cached:      # few reusable pixels, so that the launch keeps its many workgroups
        regions = []
        for i in range(n):
            rw, rh = int(rng.integers(2, 7)), int(rng.integers(2, 7))
            rx, ry = int(rng.integers(2, Wo - rw - 2)), int(rng.integers(2, Ho - rh - 2))
            regions.append((np.array([[rx, ry, rw, rh]], np.int32), (int(rng.integers(-2, 3)), int(rng.integers(-2, 3)))))
    got = _to_np(binding.dc_cached_conv_layer(_layer(cin, cout, k, s, p, True), _to_dev(x, bf16), _to_dev(w, bf16),
                                              torch.from_numpy(b).to(DEV),
                                              cache_prev=_to_dev(cache, bf16) if cached else None, regions=regions))
    for i in range(n):
        if cached:
            mask = oracle.rasterize(regions[i][0], Ho, Wo)
            want = oracle.conv_cached(x[i], w, b, k, s, p, True, cache_prev=cache[i], mask=mask, dxy=regions[i][1], bf16=bf16)
            m = mask.astype(bool)
            assert np.array_equal(got[i][m], want[m]), "copied pixels must be bit-identical"
        else:
            want = oracle.conv_cached(x[i], w, b, k, s, p, True, bf16=bf16)
        assert _rel_err(got[i], want) <= (2e-2 if bf16 else 1e-4), (case, i)


KERNEL_SHAPE_CASES = [
    # H, W, cin, cout, kh, kw, s, ph, pw, dil
    (23, 31, 16, 32, 1, 7, 1, 0, 3, 1),      # a row kernel
    (23, 31, 16, 32, 7, 1, 1, 3, 0, 1),      # a column kernel
    (26, 30, 32, 64, 3, 3, 1, 2, 2, 2),      # dilated by 2, same size
    (33, 29, 32, 32, 3, 1, 2, 1, 0, 1),      # column kernel with stride 2
    (24, 28, 16, 48, 5, 3, 1, 4, 2, 2),      # not square and dilated
    (19, 21, 5, 7, 2, 5, 3, 0, 1, 1),        # odd channel counts (element loads), stride 3
    (30, 30, 8, 16, 3, 3, 1, 3, 3, 3),       # dilated by 3
]


@pytest.mark.parametrize("cached", [False, True])
@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("case", KERNEL_SHAPE_CASES)
def test_kernels_that_are_not_square_or_dilated(oracle, case, bf16, cached):
    """dc_layer.k2 / p2 / dil: the general conv kernels with a kernel of k rows x k2 columns and taps dil pixels apart."""
    H, W, cin, cout, kh, kw, s, ph, pw, dil = case
    print(f"[kernel shapes] case={case} bf16={bf16} cached={cached}", flush=True)
    rng = np.random.default_rng(sum(case))
    n = 2
    x = rng.standard_normal((n, H, W, cin)).astype(np.float32)
    w = (rng.standard_normal((cout, kh, kw, cin)) * np.sqrt(2.0 / (cin * kh * kw))).astype(np.float32)
    b = (rng.standard_normal(cout) * 0.1).astype(np.float32)
    layer = dict(type=synth.CONV, k=kh, s=s, p=ph, cin=cin, cout=cout, relu=1, in0=0, in1=-1, k2=kw, p2=pw, dil=dil)
    Ho, Wo, _ = synth.tensor_shapes([layer], H, W, cin)[1]
    cache = rng.standard_normal((n, Ho, Wo, cout)).astype(np.float32)
    if bf16:
        x, w, cache = oracle.round_bf16(x), oracle.round_bf16(w), oracle.round_bf16(cache)
    regions = None
    if cached:
        regions = [(np.array([[1, 2, Wo - 4, Ho - 5]], np.int32), (1, -1)), (np.array([[0, 0, Wo - 2, Ho - 1]], np.int32), (1, 0))]
    got = _to_np(binding.dc_cached_conv_layer(layer, _to_dev(x, bf16), _to_dev(w, bf16), torch.from_numpy(b).to(DEV),
                                              cache_prev=_to_dev(cache, bf16) if cached else None, regions=regions))
    assert got.shape == (n, Ho, Wo, cout)
    for i in range(n):
        if cached:
            mask = oracle.rasterize(regions[i][0], Ho, Wo)
            want = oracle.conv_cached(x[i], w, b, kh, s, ph, True, cache_prev=cache[i], mask=mask, dxy=regions[i][1], bf16=bf16,
                                      k2=kw, p2=pw, dil=dil)
            m = mask.astype(bool)
            assert np.array_equal(got[i][m], want[m])
        else:
            want = oracle.conv_cached(x[i], w, b, kh, s, ph, True, bf16=bf16, k2=kw, p2=pw, dil=dil)
        assert _rel_err(got[i], want) <= (2e-2 if bf16 else 1e-4), (case, i)


def test_raster_positions_of_a_large_batch(oracle):
    """40 streams of 416 x 416: the product of a unit's raster position and the units per map passes 2^32, where the
    kernels' division by a magic number is one too large and is corrected.  First-layer shape and a 3x3 layer; the first
    and the last stream against the oracle."""
    n, H, W = 40, 416, 416
    for cin, cout in ((8, 32), (32, 64)):
        rng = np.random.default_rng(cin)
        x = oracle.round_bf16(rng.standard_normal((n, H, W, cin)).astype(np.float32))
        w = oracle.round_bf16((rng.standard_normal((cout, 3, 3, cin)) * np.sqrt(2.0 / (cin * 9))).astype(np.float32))
        got = binding.dc_cached_conv_layer(_layer(cin, cout, 3, 1, 1, True), _to_dev(x, True), _to_dev(w, True), None)
        torch.cuda.synchronize()
        for s in (0, n - 1):
            want = oracle.conv_cached(x[s], w, None, 3, 1, 1, True, bf16=True)
            assert _rel_err(got[s].float().cpu().numpy(), want) <= 2e-2, (cin, s)
