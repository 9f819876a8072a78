"""Seeded synthetic inputs: video frames, layer tables and weights.

This module feeds both the HIP path and the CPU oracle.  It holds none of the
method's arithmetic (no matching, no region logic, no convolution): it only
draws frames, describes network stacks as plain data and draws weights.

The videos stand in for the paper's phone-camera clips (Section 7.1 uses UCF101
and a driving set, neither of which can be shipped): a textured background
that pans by a few pixels per frame (camera motion) with rigid foreground
rectangles that move on their own (moving objects), which is the structure
Section 4 designs the matcher for.
"""
from __future__ import annotations

import numpy as np

# layer types (plain data; each side maps them to its own C enum)
CONV, MAXPOOL, RELU, ADD, LRN, CONCAT, FC, SOFTMAX, AVGPOOL = 0, 1, 2, 3, 4, 5, 6, 7, 8

# fields a layer's dict may leave out
LAYER_DEFAULTS = dict(k=1, s=1, p=0, relu=0, in1=-1, in2=-1, in3=-1, within=0, alpha=0.0, beta=0.0, kappa=1.0,
                      k2=0, p2=0, dil=1)


# --------------------------------------------------------------------------- #
# layer tables                                                                #
# --------------------------------------------------------------------------- #
def _conv(cin, cout, k, s, p, relu, in0):
    return dict(type=CONV, k=k, s=s, p=p, cin=cin, cout=cout, relu=int(relu), in0=in0, in1=-1)


def conv_geometry(L):
    """(kernel rows, kernel columns, padding rows, padding columns, dilation) of a conv layer: k2 > 0 gives the kernel
    k rows x k2 columns with paddings p / p2, dil > 1 puts the taps dil pixels apart."""
    if L["type"] != CONV:
        return L["k"], L["k"], L["p"], L["p"], 1
    k2 = L.get("k2", 0)
    return L["k"], (k2 if k2 > 0 else L["k"]), L["p"], (L.get("p2", 0) if k2 > 0 else L["p"]), max(1, L.get("dil", 1))


def _pool(c, k, s, p, in0):
    return dict(type=MAXPOOL, k=k, s=s, p=p, cin=c, cout=c, relu=0, in0=in0, in1=-1)


def _add(c, in0, in1, relu):
    return dict(type=ADD, k=1, s=1, p=0, cin=c, cout=c, relu=int(relu), in0=in0, in1=in1)


def _avgpool(c, k, s, p, in0):
    return dict(type=AVGPOOL, k=k, s=s, p=p, cin=c, cout=c, relu=0, in0=in0, in1=-1)


def _lrn(c, size, in0, within=0, alpha=1e-4, beta=0.75, kappa=1.0):
    return dict(type=LRN, k=size, s=1, p=0, cin=c, cout=c, relu=0, in0=in0, in1=-1, within=int(within),
                alpha=alpha, beta=beta, kappa=kappa)


def _concat(cs, ins):
    ins = list(ins) + [-1] * (4 - len(ins))
    return dict(type=CONCAT, k=1, s=1, p=0, cin=sum(cs), cout=sum(cs), relu=0, in0=ins[0], in1=ins[1], in2=ins[2],
                in3=ins[3])


def _fc(cin, cout, relu, in0):
    return dict(type=FC, k=1, s=1, p=0, cin=cin, cout=cout, relu=int(relu), in0=in0, in1=-1)


def _softmax(c, in0):
    return dict(type=SOFTMAX, k=1, s=1, p=0, cin=c, cout=c, relu=0, in0=in0, in1=-1)


def _chain(spec, cin):
    """spec: list of ('c', cout, k, s, p) or ('p', k, s, p).  Tensor 0 is the input."""
    layers = []
    c = cin
    for item in spec:
        t = len(layers)  # producer tensor id of the next layer's input
        if item[0] == "c":
            _, cout, k, s, p = item
            layers.append(_conv(c, cout, k, s, p, True, t))
            c = cout
        else:
            _, k, s, p = item
            layers.append(_pool(c, k, s, p, t))
    return layers


def no_reuse_flags(layers, min_macs):
    """A cache setting for a stack: flag [n_layers] (uint8) the conv layers with fewer than min_macs multiply-adds per
    output element (k * k * cin of the layer table as given); flagged layers are computed in full on every frame."""
    return np.array([1 if (L["type"] == CONV and conv_geometry(L)[0] * conv_geometry(L)[1] * L["cin"] < min_macs) else 0
                     for L in layers], np.uint8)


def factorised_net(c=16):
    """A small stack with kernels that are not square and with dilated ones (the 1 x 7 / 7 x 1 pairs of later
    inception-style networks, the dilated 3 x 3 of segmentation networks): 3 -> c 3x3, c -> c 1x7, c -> c 7x1,
    max-pooling 2x2, c -> 2c 3x3 dilated by 2, 2c -> 2c 3x1 stride 2, 2c -> 2c 5x3 dilated by 2, 2c -> 2c 1x1."""
    C_ = lambda cin, cout, k, s, p, i, **kw: dict(type=CONV, k=k, s=s, p=p, cin=cin, cout=cout, relu=1, in0=i, in1=-1, **kw)
    return [C_(3, c, 3, 1, 1, 0),
            C_(c, c, 1, 1, 0, 1, k2=7, p2=3),
            C_(c, c, 7, 1, 3, 2, k2=1, p2=0),
            _pool(c, 2, 2, 0, 3),
            C_(c, 2 * c, 3, 1, 2, 4, dil=2),
            C_(2 * c, 2 * c, 3, 2, 1, 5, k2=1, p2=0),
            C_(2 * c, 2 * c, 5, 1, 4, 6, k2=3, p2=2, dil=2),
            C_(2 * c, 2 * c, 1, 1, 0, 7)]


def tiny_net():
    """3 conv layers: 3->16 s1, 16->32 s2, 32->32 s1, all 3x3 p1 + ReLU."""
    return _chain([("c", 16, 3, 1, 1), ("c", 32, 3, 2, 1), ("c", 32, 3, 1, 1)], 3)


def small_vgg(c=64):
    """Five 3x3 conv layers of c, c, 2c, 2c, 2c channels with 2x2 poolings after the second and the fourth: the
    smallest stack with the layer shapes of the VGG-style trunk (whole 64-byte channel rows for c = 64)."""
    return _chain([("c", c, 3, 1, 1), ("c", c, 3, 1, 1), ("p", 2, 2, 0), ("c", 2 * c, 3, 1, 1), ("c", 2 * c, 3, 1, 1),
                   ("p", 2, 2, 0), ("c", 2 * c, 3, 1, 1)], 3)


def vgg16():
    """VGG-16-style trunk: 13 conv3x3 p1 ReLU and 4 maxpool 2x2 s2."""
    spec = []
    for block, (c, n) in enumerate([(64, 2), (128, 2), (256, 3), (512, 3), (512, 3)]):
        spec += [("c", c, 3, 1, 1)] * n
        if block < 4:
            spec.append(("p", 2, 2, 0))
    return _chain(spec, 3)


def darknet19(leaky=False):
    """Darknet-19-style stack: 3x3 convs with 1x1 bottlenecks, 5 maxpools, 1x1 head.  `leaky`: the activation of
    the published network (leaky ReLU, slope 0.1) instead of ReLU."""
    spec = [("c", 32, 3, 1, 1), ("p", 2, 2, 0), ("c", 64, 3, 1, 1), ("p", 2, 2, 0)]
    for c, n in [(128, 3), (256, 3)]:
        for i in range(n):
            spec.append(("c", c, 3, 1, 1) if i % 2 == 0 else ("c", c // 2, 1, 1, 0))
        spec.append(("p", 2, 2, 0))
    for i in range(5):
        spec.append(("c", 512, 3, 1, 1) if i % 2 == 0 else ("c", 256, 1, 1, 0))
    spec.append(("p", 2, 2, 0))
    for i in range(5):
        spec.append(("c", 1024, 3, 1, 1) if i % 2 == 0 else ("c", 512, 1, 1, 0))
    spec.append(("c", 1024, 1, 1, 0))
    layers = _chain(spec, 3)
    if leaky:
        for L in layers:
            if L["type"] == CONV:
                L["relu"] = 2
    return layers


def resnet50_trunk():
    """ResNet-50-style conv trunk (no BN): 7x7 s2 stem, maxpool 3x3 s2, stages [3,4,6,3]
    of 1x1/3x3/1x1 bottlenecks, projection shortcut on each stage's first block,
    add then ReLU."""
    layers = [_conv(3, 64, 7, 2, 3, True, 0)]
    layers.append(_pool(64, 3, 2, 1, 1))
    x = 2  # tensor id of the running block input
    cin = 64
    for stage, (width, n) in enumerate([(64, 3), (128, 4), (256, 6), (512, 3)]):
        for b in range(n):
            s = 2 if (b == 0 and stage > 0) else 1
            cout = 4 * width
            layers.append(_conv(cin, width, 1, 1, 0, True, x))
            a = len(layers)
            layers.append(_conv(width, width, 3, s, 1, True, a))
            bb = len(layers)
            layers.append(_conv(width, cout, 1, 1, 0, False, bb))
            main = len(layers)
            if b == 0:
                layers.append(_conv(cin, cout, 1, s, 0, False, x))
                short = len(layers)
            else:
                short = x
            layers.append(_add(cout, main, short, True))
            x = len(layers)
            cin = cout
    return layers


def alexnet(n_classes=1000, width=1.0):
    """AlexNet-style stack in one tower (Table 3, REC_1): 5 convolutions (11x11 s4, 5x5, three 3x3), LRN over 5
    channels after the first two, three 3x3 s2 max-poolings, three fully-connected layers and a softmax.
    `width` scales every channel count (tests use a narrow copy)."""
    c = lambda v: max(8, int(v * width) // 8 * 8)
    L = []
    L.append(_conv(3, c(96), 11, 4, 0, True, 0))
    L.append(_lrn(c(96), 5, len(L), alpha=1e-4, beta=0.75, kappa=2.0))
    L.append(_pool(c(96), 3, 2, 0, len(L)))
    L.append(_conv(c(96), c(256), 5, 1, 2, True, len(L)))
    L.append(_lrn(c(256), 5, len(L), alpha=1e-4, beta=0.75, kappa=2.0))
    L.append(_pool(c(256), 3, 2, 0, len(L)))
    L.append(_conv(c(256), c(384), 3, 1, 1, True, len(L)))
    L.append(_conv(c(384), c(384), 3, 1, 1, True, len(L)))
    L.append(_conv(c(384), c(256), 3, 1, 1, True, len(L)))
    L.append(_pool(c(256), 3, 2, 0, len(L)))
    L.append(_fc(c(256), c(4096), True, len(L)))
    L.append(_fc(c(4096), c(4096), True, len(L)))
    L.append(_fc(c(4096), n_classes, False, len(L)))
    L.append(_softmax(n_classes, len(L)))
    return L


def dave_orig():
    """The steering network of Table 3 (DRV): five convolutions without padding (three 5x5 stride 2 with 24, 36 and
    48 channels, two 3x3 with 64) on a 66x200 frame, then fully-connected layers of 100, 50, 10 and 1 outputs."""
    L = []
    L.append(_conv(3, 24, 5, 2, 0, True, 0))
    L.append(_conv(24, 36, 5, 2, 0, True, len(L)))
    L.append(_conv(36, 48, 5, 2, 0, True, len(L)))
    L.append(_conv(48, 64, 3, 1, 0, True, len(L)))
    L.append(_conv(64, 64, 3, 1, 0, True, len(L)))
    L.append(_fc(64, 100, True, len(L)))
    L.append(_fc(100, 50, True, len(L)))
    L.append(_fc(50, 10, True, len(L)))
    L.append(_fc(10, 1, False, len(L)))
    return L


def googlenet(n_classes=1000, width=1.0):
    """GoogLeNet-style stack (Table 3, REC_2): stem, nine inception modules (four branches joined by a concat),
    global average pooling, one fully-connected layer and a softmax: 57 convolutions.  Poolings use zero padding
    where the published network rounds the output size up."""
    c = lambda v: max(8, int(v * width) // 8 * 8)
    L = []
    L.append(_conv(3, c(64), 7, 2, 3, True, 0))
    L.append(_pool(c(64), 3, 2, 1, len(L)))
    L.append(_lrn(c(64), 5, len(L)))
    L.append(_conv(c(64), c(64), 1, 1, 0, True, len(L)))
    L.append(_conv(c(64), c(192), 3, 1, 1, True, len(L)))
    L.append(_lrn(c(192), 5, len(L)))
    L.append(_pool(c(192), 3, 2, 1, len(L)))
    x, cin = len(L), c(192)

    def inception(x, cin, n1, n3r, n3, n5r, n5, npj):
        L.append(_conv(cin, c(n1), 1, 1, 0, True, x)); b1 = len(L)
        L.append(_conv(cin, c(n3r), 1, 1, 0, True, x))
        L.append(_conv(c(n3r), c(n3), 3, 1, 1, True, len(L))); b2 = len(L)
        L.append(_conv(cin, c(n5r), 1, 1, 0, True, x))
        L.append(_conv(c(n5r), c(n5), 5, 1, 2, True, len(L))); b3 = len(L)
        L.append(_pool(cin, 3, 1, 1, x))
        L.append(_conv(cin, c(npj), 1, 1, 0, True, len(L))); b4 = len(L)
        cs = [c(n1), c(n3), c(n5), c(npj)]
        L.append(_concat(cs, [b1, b2, b3, b4]))
        return len(L), sum(cs)

    x, cin = inception(x, cin, 64, 96, 128, 16, 32, 32)
    x, cin = inception(x, cin, 128, 128, 192, 32, 96, 64)
    L.append(_pool(cin, 3, 2, 1, x)); x = len(L)
    x, cin = inception(x, cin, 192, 96, 208, 16, 48, 64)
    x, cin = inception(x, cin, 160, 112, 224, 24, 64, 64)
    x, cin = inception(x, cin, 128, 128, 256, 24, 64, 64)
    x, cin = inception(x, cin, 112, 144, 288, 32, 64, 64)
    x, cin = inception(x, cin, 256, 160, 320, 32, 128, 128)
    L.append(_pool(cin, 3, 2, 1, x)); x = len(L)
    x, cin = inception(x, cin, 256, 160, 320, 32, 128, 128)
    x, cin = inception(x, cin, 384, 192, 384, 48, 128, 128)
    L.append(dict(_avgpool(cin, 7, 1, 0, x), k=-1)); x = len(L)     # k = -1: replaced by the map size (global pooling)
    L.append(_fc(cin, n_classes, False, x))
    L.append(_softmax(n_classes, len(L)))
    return L


def resolve_global_pooling(layers, H, W, C):
    """Layer tables may mark a pooling as global with k = -1: returns a copy with the map size filled in."""
    out = []
    shapes = [(H, W, C)]
    for L in layers:
        L = dict(L)
        h, w, _ = shapes[L["in0"]]
        if L["type"] in (MAXPOOL, AVGPOOL) and L["k"] < 0:
            assert h == w, "global pooling of a square map"
            L["k"], L["s"], L["p"] = h, 1, 0
        out.append(L)
        shapes.append(tensor_shapes([dict(L, in0=0)], h, w, shapes[L["in0"]][2])[1])
    return out


def tensor_shapes(layers, H, W, C):
    """(H, W, C) of every tensor; tensor 0 is the input, tensor i+1 is layer i's output."""
    shapes = [(H, W, C)]
    for L in layers:
        h, w, _ = shapes[L["in0"]]
        if L["type"] in (CONV, MAXPOOL, AVGPOOL):
            kh, kw, ph, pw, dil = conv_geometry(L)
            ho = (h + 2 * ph - ((kh - 1) * dil + 1)) // L["s"] + 1
            wo = (w + 2 * pw - ((kw - 1) * dil + 1)) // L["s"] + 1
            shapes.append((ho, wo, L["cout"]))
        elif L["type"] == FC:
            shapes.append((1, 1, L["cout"]))
        else:
            shapes.append((h, w, L["cout"]))
    return shapes


def he_weights(layers, seed, bias_scale=0.0, residual_scale=1.0, input_shape=None):
    """He-normal weights N(0, 2/(cin*k*k)) in [cout][k][k][cin] order and biases; a fully-connected layer gets
    [cout][h*w*cin] with variance 2/(h*w*cin), for which `input_shape` = (H, W, C) of tensor 0 is needed.

    `residual_scale` multiplies the conv that feeds in0 of every ADD layer (keeps
    activations of deep residual stacks in a tame range without normalisation layers).
    Returns two lists indexed by layer (None for layers without weights)."""
    rng = np.random.default_rng(seed)
    feeds_add = {L["in0"] - 1 for L in layers if L["type"] == ADD}
    ws, bs = [], []
    shapes = tensor_shapes(layers, *input_shape) if input_shape is not None else None
    for i, L in enumerate(layers):
        if L["type"] == FC:
            K = int(np.prod(shapes[L["in0"]]))
            ws.append(np.ascontiguousarray(rng.standard_normal((L["cout"], K)) * np.sqrt(2.0 / K), dtype=np.float32))
            bs.append(np.ascontiguousarray(rng.standard_normal(L["cout"]) * bias_scale, dtype=np.float32))
            continue
        if L["type"] != CONV:
            ws.append(None)
            bs.append(None)
            continue
        cin, cout = L["cin"], L["cout"]
        kh, kw = conv_geometry(L)[:2]
        w = rng.standard_normal((cout, kh, kw, cin)) * np.sqrt(2.0 / (cin * kh * kw))
        if i in feeds_add:
            w = w * residual_scale
        b = rng.standard_normal(cout) * bias_scale
        ws.append(np.ascontiguousarray(w, dtype=np.float32))
        bs.append(np.ascontiguousarray(b, dtype=np.float32))
    return ws, bs


# --------------------------------------------------------------------------- #
# frames                                                                      #
# --------------------------------------------------------------------------- #
def _box_blur5(img):
    """5x5 box blur, edge-replicated, integer rounding (sum+12)//25, per channel."""
    H, W, _ = img.shape
    pad = np.pad(img.astype(np.int64), ((2, 2), (2, 2), (0, 0)), mode="edge")
    acc = np.zeros(img.shape, dtype=np.int64)
    for dy in range(5):
        for dx in range(5):
            acc += pad[dy:dy + H, dx:dx + W]
    return ((acc + 12) // 25).astype(np.uint8)


def tiny_pair(seed=0, H=64, W=64, shift=(3, -2), sigma=2.0, patch=(24, 24, 16)):
    """Two frames: a blurred-noise image, and the same content moved by `shift`
    (+x right, +y down) with sensor noise and one square patch of fresh noise.

    Returns (frame1, frame2) as uint8 [H][W][3]."""
    rng = np.random.default_rng(seed)
    f1 = _box_blur5(rng.integers(0, 256, size=(H, W, 3), dtype=np.int64).astype(np.uint8))
    sx, sy = shift
    ys = np.clip(np.arange(H) - sy, 0, H - 1)
    xs = np.clip(np.arange(W) - sx, 0, W - 1)
    moved = f1[ys][:, xs].astype(np.float64)
    noisy = np.rint(moved + rng.normal(0.0, sigma, size=moved.shape))
    f2 = np.clip(noisy, 0, 255).astype(np.uint8)
    px, py, ps = patch
    if ps > 0:
        f2[py:py + ps, px:px + ps] = rng.integers(0, 256, size=(ps, ps, 3), dtype=np.int64).astype(np.uint8)
    return f1, f2


def shifted_pair(seed, H, W, shift, C=3):
    """Noise-free pair: frame2 is frame1's content moved by `shift` (edge-replicated)."""
    rng = np.random.default_rng(seed)
    f1 = _box_blur5(rng.integers(0, 256, size=(H, W, C), dtype=np.int64).astype(np.uint8))
    sx, sy = shift
    ys = np.clip(np.arange(H) - sy, 0, H - 1)
    xs = np.clip(np.arange(W) - sx, 0, W - 1)
    return f1, np.ascontiguousarray(f1[ys][:, xs])


def _value_noise(rng, size, lattices=(64, 32, 16, 8, 4)):
    """Multi-octave value noise, `size` x `size` x 3, amplitude halving per octave,
    smoothstep interpolation, channels independent, quantised to uint8."""
    out = np.zeros((size, size, 3), dtype=np.float64)
    amp, total = 1.0, 0.0
    coords = np.arange(size, dtype=np.float64)
    for lat in lattices:
        n = size // lat + 2
        grid = rng.random((n, n, 3))
        g = coords / lat
        i0 = np.floor(g).astype(np.int64)
        t = g - i0
        t = t * t * (3.0 - 2.0 * t)
        ty = t[:, None, None]
        tx = t[None, :, None]
        a = grid[i0][:, i0]
        b = grid[i0][:, i0 + 1]
        c = grid[i0 + 1][:, i0]
        d = grid[i0 + 1][:, i0 + 1]
        out += amp * ((a * (1 - tx) + b * tx) * (1 - ty) + (c * (1 - tx) + d * tx) * ty)
        total += amp
        amp *= 0.5
    out /= total
    return np.clip(np.rint(out * 255.0), 0, 255).astype(np.uint8)


_DIRS = [(1, 0), (1, 1), (0, 1), (-1, 1), (-1, 0), (-1, -1), (0, -1), (1, -1)]


def panning_video(seed, n_frames=30, H=224, W=224, fg=((48, 48), (32, 64)),
                  pan_speeds=(1, 2, 3), fg_speeds=(4, 5, 6), redraw_every=10,
                  margin=96):
    """Value-noise background panning `pan_speeds` px/frame in a compass direction that
    is redrawn every `redraw_every` frames, plus rigid uniform-noise rectangles
    (h, w) moving `fg_speeds` px/frame and bouncing at the edges.  No sensor noise.

    Returns uint8 [n_frames][H][W][3]."""
    rng = np.random.default_rng(seed)
    size = ((max(H, W) + 2 * margin + 63) // 64) * 64
    canvas = _value_noise(rng, size)
    ox, oy = (size - W) // 2, (size - H) // 2
    objs = []
    for (h, w) in fg:
        tex = rng.integers(0, 256, size=(h, w, 3), dtype=np.int64).astype(np.uint8)
        x = int(rng.integers(0, W - w + 1))
        y = int(rng.integers(0, H - h + 1))
        sp = int(rng.choice(fg_speeds))
        dx, dy = _DIRS[int(rng.integers(0, 8))]
        objs.append([tex, x, y, dx * sp, dy * sp])
    frames = np.empty((n_frames, H, W, 3), dtype=np.uint8)
    vx = vy = 0
    for f in range(n_frames):
        if f % redraw_every == 0:
            sp = int(rng.choice(pan_speeds))
            dx, dy = _DIRS[int(rng.integers(0, 8))]
            vx, vy = dx * sp, dy * sp
        if f > 0:
            ox = int(np.clip(ox + vx, 0, size - W))
            oy = int(np.clip(oy + vy, 0, size - H))
        img = canvas[oy:oy + H, ox:ox + W].copy()
        for o in objs:
            tex, x, y, ux, uy = o
            if f > 0:
                x += ux
                y += uy
                if x < 0 or x + tex.shape[1] > W:
                    ux = -ux
                    x = int(np.clip(x, 0, W - tex.shape[1]))
                if y < 0 or y + tex.shape[0] > H:
                    uy = -uy
                    y = int(np.clip(y, 0, H - tex.shape[0]))
                o[1], o[2], o[3], o[4] = x, y, ux, uy
            img[y:y + tex.shape[0], x:x + tex.shape[1]] = tex
        frames[f] = img
    return frames


def _sweep_dirty_fraction(boxes, pan, H, W, block, frames):
    """Share of blocks that a foreground box touches in a frame or whose counterpart one frame earlier (the block
    moved back along the pan) was touched or lay outside the frame, averaged over `frames` (index >= 1).  Geometry
    only: it sizes the foreground, the matcher is not involved."""
    gh, gw = H // block, W // block
    by, bx = np.mgrid[0:gh, 0:gw]
    x0, y0 = bx * block, by * block

    def touched(f, xa, ya):       # blocks [xa, xa+block) x [ya, ya+block) that meet a box of frame f
        hit = (xa < 0) | (ya < 0) | (xa + block > W) | (ya + block > H)
        for (x, y, w, h) in boxes[f]:
            hit |= (xa < x + w) & (xa + block > x) & (ya < y + h) & (ya + block > y)
        return hit
    tot = 0.0
    for f in frames:
        tot += float((touched(f, x0, y0) | touched(f - 1, x0 + pan[0], y0 + pan[1])).mean())
    return tot / max(len(frames), 1)


def reuse_sweep_video(seed, target_reuse, n_frames=60, H=416, W=416, block=16,
                      pan=(2, 0), cut_at=30, fg_speeds=(4, 5, 6)):
    """The reuse-ratio sweep: a value-noise background panning `pan` px/frame under moving noise rectangles
    (their texture is drawn afresh every frame, so they never match; they move `fg_speeds` px/frame and bounce at the
    edges), a new background (scene cut) at frame `cut_at`.  The rectangles' sizes are scaled so that the share
    of blocks they spoil (touched now, or touched one frame ago where the block came from) leaves about
    `target_reuse` of the blocks reusable; the column of blocks that enters the frame caps the ratio near
    1 - block/W per panned block column.  target_reuse <= 0: every frame is fresh noise.

    Returns uint8 [n_frames][H][W][3]."""
    rng = np.random.default_rng(seed)
    margin = abs(pan[0]) * n_frames + abs(pan[1]) * n_frames + 8
    size = ((max(H, W) + 2 * margin + 63) // 64) * 64
    frames = np.empty((n_frames, H, W, 3), dtype=np.uint8)
    if target_reuse <= 0.0:
        for f in range(n_frames):
            frames[f] = rng.integers(0, 256, size=(H, W, 3), dtype=np.int64).astype(np.uint8)
        return frames
    # trajectories of the rectangles' centres and their base sizes (fractions of the frame edge)
    n_box = 12
    base = rng.uniform(0.10, 0.30, size=(n_box, 2))
    centre = rng.uniform(0.2, 0.8, size=(n_box, 2)) * (W, H)
    vel = np.array([np.array(_DIRS[int(rng.integers(0, 8))]) * int(rng.choice(fg_speeds)) for _ in range(n_box)], float)
    centres = np.empty((n_frames, n_box, 2))
    c, v = centre.copy(), vel.copy()
    for f in range(n_frames):
        if f > 0:
            c = c + v
            for a, lim in ((0, W), (1, H)):
                out = (c[:, a] < 0) | (c[:, a] > lim)
                v[out, a] = -v[out, a]
                c[:, a] = np.clip(c[:, a], 0, lim)
        centres[f] = c

    def boxes_at(scale):
        out = []
        for f in range(n_frames):
            bl = []
            for i in range(n_box):
                w, h = int(round(base[i, 0] * scale * W)), int(round(base[i, 1] * scale * H))
                if w < 1 or h < 1:
                    continue
                x = int(np.clip(round(centres[f, i, 0] - w / 2), 0, max(W - w, 0)))
                y = int(np.clip(round(centres[f, i, 1] - h / 2), 0, max(H - h, 0)))
                bl.append((x, y, min(w, W), min(h, H)))
            out.append(bl)
        return out
    sample = [f for f in range(1, n_frames) if f != cut_at]
    lo, hi = 0.0, 4.0
    for _ in range(24):                       # the spoiled share grows with the scale: bisection
        mid = 0.5 * (lo + hi)
        if 1.0 - _sweep_dirty_fraction(boxes_at(mid), pan, H, W, block, sample) > target_reuse:
            lo = mid
        else:
            hi = mid
    boxes = boxes_at(lo)
    canvas = None
    ox = oy = 0
    for f in range(n_frames):
        if f == 0 or f == cut_at:
            canvas = _value_noise(rng, size)
            ox, oy = (size - W) // 2, (size - H) // 2
        else:
            ox += pan[0]
            oy += pan[1]
        img = canvas[oy:oy + H, ox:ox + W].copy()
        for (x, y, w, h) in boxes[f]:
            img[y:y + h, x:x + w] = rng.integers(0, 256, size=(h, w, 3), dtype=np.int64).astype(np.uint8)
        frames[f] = img
    return frames


def max_block_ssd(block, channels=3, tau=20):
    """Total per-block SSD bound for a mean squared error of `tau` per sample."""
    return int(tau * block * block * channels)
