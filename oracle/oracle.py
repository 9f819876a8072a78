"""ctypes wrapper around the CPU oracle (deepcache_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, __graft_entry__.smoke() and the
cpu_baseline leg of bench.py.  It imports nothing from the HIP package.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "deepcache_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")


def build(force=False):
    """Compile the oracle with gcc (-O2 -fopenmp)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-std=c99", "-shared", "-fPIC",
                               "-o", _LIB, _SRC, "-lm"])
    return _LIB


class Rect(C.Structure):
    _fields_ = [("x", C.c_int32), ("y", C.c_int32), ("w", C.c_int32), ("h", C.c_int32)]


class Layer(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("type", "k", "s", "p", "cin", "cout", "relu", "in0", "in1", "in2", "in3",
                                         "within")] + [(n, C.c_float) for n in ("alpha", "beta", "kappa")] + \
               [(n, C.c_int32) for n in ("k2", "p2", "dil")]


# value of a field that a layer's dict leaves out
_LAYER_DEFAULTS = dict(k=1, s=1, p=0, relu=0, in1=-1, in2=-1, in3=-1, within=0, alpha=0.0, beta=0.0, kappa=1.0,
                       k2=0, p2=0, dil=1)


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.oc_round_bf16.restype = C.c_float
        _lib.oc_round_bf16.argtypes = [C.c_float]
        _lib.oc_round_bf16_array.argtypes = [C.c_void_p, C.c_size_t]
        _lib.oc_conv_cached.restype = None
        for f in ("oc_avgpool", "oc_lrn", "oc_concat", "oc_fc", "oc_softmax"):
            getattr(_lib, f).restype = None
        _lib.oc_maxpool.restype = None
        _lib.oc_add.restype = None
        _lib.oc_add.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_int, C.c_int, C.c_void_p]
        _lib.oc_frame_to_tensor.argtypes = [C.c_void_p, C.c_size_t, C.c_void_p]
    return _lib


def _p(a):
    return a.ctypes.data_as(C.c_void_p) if a is not None else None


def num_threads():
    return int(lib().oc_num_threads())


def window_out_hw(L, h, w):
    """Output size of a windowed layer (conv, pooling): a conv layer may carry k2 / p2 (kernel columns, their
    padding) and dil (distance between taps)."""
    conv = L["type"] == 0
    kh, kw = L["k"], (L["k2"] if conv and L.get("k2", 0) > 0 else L["k"])
    ph, pw = L["p"], (L.get("p2", 0) if conv and L.get("k2", 0) > 0 else L["p"])
    dil = L.get("dil", 1) if conv and L.get("dil", 1) > 1 else 1
    return (h + 2 * ph - ((kh - 1) * dil + 1)) // L["s"] + 1, (w + 2 * pw - ((kw - 1) * dil + 1)) // L["s"] + 1


def layers_to_c(layers):
    arr = (Layer * len(layers))()
    for i, L in enumerate(layers):
        for f, ct in Layer._fields_:
            v = L[f] if f in L else _LAYER_DEFAULTS[f]
            setattr(arr[i], f, float(v) if ct is C.c_float else int(v))
    return arr


def rects_to_np(rects):
    """list of (x,y,w,h) -> int32 [n][4]"""
    return np.ascontiguousarray(np.array(rects, dtype=np.int32).reshape(-1, 4))


def match_blocks(cur, prev, block, radius, max_ssd, k_skip=1):
    """Section 4, Steps 1-4 (exhaustive search; k_skip > 1: only every k-th block row and column is searched).
    Returns dict(mv, best_ssd, gmv, n_pass, mask)."""
    H, W, Ch = cur.shape
    gh, gw = H // block, W // block
    mv = np.zeros((gh, gw, 2), np.int16)
    best = np.zeros((gh, gw), np.uint32)
    gmv = np.zeros(2, np.int32)
    npass = np.zeros(1, np.int32)
    mask = np.zeros((gh, gw), np.uint8)
    cur = np.ascontiguousarray(cur, np.uint8)
    prev = np.ascontiguousarray(prev, np.uint8)
    if k_skip == 1:
        lib().oc_match_blocks(_p(cur), _p(prev), H, W, Ch, block, radius, C.c_uint32(max_ssd),
                              _p(mv), _p(best), _p(gmv), _p(npass), _p(mask))
    else:
        lib().oc_match_blocks_k(_p(cur), _p(prev), H, W, Ch, block, radius, int(k_skip), C.c_uint32(max_ssd),
                                _p(mv), _p(best), _p(gmv), _p(npass), _p(mask))
    return dict(mv=mv, best_ssd=best, gmv=gmv, n_pass=int(npass[0]), mask=mask)


def match_blocks_ds(cur, prev, block, radius, max_ssd, k_skip=1):
    """Section 4, Steps 1-4 with diamond search in Step 2 and k-skip.  Returns dict(mv, best_ssd, gmv,
    n_pass, mask, rounds); rounds = large-pattern rounds per searched block."""
    H, W, Ch = cur.shape
    gh, gw = H // block, W // block
    mv = np.zeros((gh, gw, 2), np.int16)
    best = np.zeros((gh, gw), np.uint32)
    gmv = np.zeros(2, np.int32)
    npass = np.zeros(1, np.int32)
    mask = np.zeros((gh, gw), np.uint8)
    rounds = np.zeros((gh, gw), np.int32)
    cur = np.ascontiguousarray(cur, np.uint8)
    prev = np.ascontiguousarray(prev, np.uint8)
    lib().oc_match_blocks_ds(_p(cur), _p(prev), H, W, Ch, block, radius, int(k_skip), C.c_uint32(max_ssd),
                             _p(mv), _p(best), _p(gmv), _p(npass), _p(mask), _p(rounds))
    return dict(mv=mv, best_ssd=best, gmv=gmv, n_pass=int(npass[0]), mask=mask, rounds=rounds)


def diamond_search_table(table):
    """Diamond search over a cost table [(2R+1)][(2R+1)] indexed [dy+R][dx+R]; 0xFFFFFFFF = invalid vector.
    Returns ((dx, dy), cost, rounds)."""
    table = np.ascontiguousarray(table, np.uint32)
    R = (table.shape[0] - 1) // 2
    assert table.shape == (2 * R + 1, 2 * R + 1)
    d = np.zeros(2, np.int32)
    best = np.zeros(1, np.uint32)
    rounds = np.zeros(1, np.int32)
    lib().oc_diamond_search_table(_p(table), R, _p(d), _p(best), _p(rounds))
    return (int(d[0]), int(d[1])), int(best[0]), int(rounds[0])


def merge_blocks(mask, block, cap=4096):
    """Section 4, Step 5.  Returns int32 [n][4] rectangles (x,y,w,h) in pixels."""
    mask = np.ascontiguousarray(mask, np.uint8)
    gh, gw = mask.shape
    out = np.zeros((cap, 4), np.int32)
    n = lib().oc_merge_blocks(_p(mask), gh, gw, block, _p(out), cap)
    assert n <= cap
    return out[:n].copy()


def dt_window(rect, k, s, p):
    """Table 2 conv/pool row.  Returns (x,y,w,h) or None."""
    out = Rect()
    ok = lib().oc_dt_window(Rect(*[int(v) for v in rect]), int(k), int(s), int(p), C.byref(out))
    return (out.x, out.y, out.w, out.h) if ok else None


def dt_overlap(a, b):
    out = Rect()
    ok = lib().oc_dt_overlap(Rect(*[int(v) for v in a]), Rect(*[int(v) for v in b]), C.byref(out))
    return (out.x, out.y, out.w, out.h) if ok else None


def dt_lrn(rect, r):
    """Table 2 LRN row for a window of radius r pixels.  Returns (x,y,w,h) or None."""
    out = Rect()
    ok = lib().oc_dt_lrn(Rect(*[int(v) for v in rect]), int(r), C.byref(out))
    return (out.x, out.y, out.w, out.h) if ok else None


def dt_window2(rect, ew, eh, s, pw, ph):
    """Table 2's conv / pooling row for a window that spans ew columns and eh rows, paddings pw / ph."""
    out = Rect()
    ok = lib().oc_dt_window2(Rect(*[int(v) for v in rect]), int(ew), int(eh), int(s), int(pw), int(ph), C.byref(out))
    return (out.x, out.y, out.w, out.h) if ok else None


def dt_window_ext(rect, k, s, p, wa, ha):
    """Conv/pool row with the border case (a rectangle touching a side of the wa x ha map extends beyond it)."""
    out = Rect()
    ok = lib().oc_dt_window_ext(Rect(*[int(v) for v in rect]), int(k), int(s), int(p), int(wa), int(ha), C.byref(out))
    return (out.x, out.y, out.w, out.h) if ok else None


def propagate(layers, H, W, rects0, mx, my, cap=1024, extend_borders=False):
    """Section 5 propagation.  Returns dict(rects=[per tensor int32 [n][4]], dxy, cum_stride, hw)."""
    n = len(layers)
    Lc = layers_to_c(layers)
    r0 = rects_to_np(rects0)
    rects = np.zeros((n + 1, cap, 4), np.int32)
    n_rects = np.zeros(n + 1, np.int32)
    dxy = np.zeros((n + 1, 2), np.int32)
    cs = np.zeros(n + 1, np.int32)
    hw = np.zeros((n + 1, 2), np.int32)
    rc = lib().oc_propagate_ext(Lc, n, int(H), int(W), _p(r0), len(r0), int(mx), int(my), int(extend_borders), _p(rects), cap,
                            _p(n_rects), _p(dxy), _p(cs), _p(hw))
    assert rc == 0, "rect capacity exceeded"
    return dict(rects=[rects[t, :n_rects[t]].copy() for t in range(n + 1)], dxy=dxy,
                cum_stride=cs, hw=hw)


def tensor_hw(layers, H, W):
    """Spatial size of every tensor of the stack."""
    hw = [(int(H), int(W))]
    for L in layers:
        h, w_ = hw[L["in0"]]
        if L["type"] in (0, 1, 8):
            hw.append(window_out_hw(L, h, w_))
        elif L["type"] == 6:
            hw.append((1, 1))
        else:
            hw.append((h, w_))
    return hw


def propagate_masks(layers, H, W, block_mask, block, mx, my, extend_borders=False):
    """Exact reuse maps of every tensor (uint8 [h][w], 1 = reusable).  Returns dict(masks, dxy, cum_stride, hw)."""
    n = len(layers)
    Lc = layers_to_c(layers)
    bm = np.ascontiguousarray(block_mask, np.uint8)
    gh, gw = bm.shape
    masks = [np.zeros(s, np.uint8) for s in tensor_hw(layers, H, W)]
    mp = (C.c_void_p * (n + 1))(*[m.ctypes.data for m in masks])
    dxy = np.zeros((n + 1, 2), np.int32)
    cs = np.zeros(n + 1, np.int32)
    hw = np.zeros((n + 1, 2), np.int32)
    rc = lib().oc_propagate_masks(Lc, n, int(H), int(W), _p(bm), gh, gw, int(block), int(mx), int(my), int(extend_borders),
                                  mp, _p(dxy), _p(cs), _p(hw))
    assert rc == 0
    return dict(masks=masks, dxy=dxy, cum_stride=cs, hw=hw)


def rasterize(rects, H, W):
    r = rects_to_np(rects)
    H, W = int(H), int(W)
    mask = np.zeros((H, W), np.uint8)
    lib().oc_rasterize(_p(r), len(r), int(H), int(W), _p(mask))
    return mask


def round_bf16(a):
    a = np.array(a, dtype=np.float32, copy=True, order="C")
    lib().oc_round_bf16_array(_p(a), a.size)
    return a


def frame_to_tensor(frame):
    frame = np.ascontiguousarray(frame, np.uint8)
    out = np.zeros(frame.shape, np.float32)
    lib().oc_frame_to_tensor(_p(frame), frame.size, _p(out))
    return out


def conv_cached(x, w, bias, k, s, p, relu, cache_prev=None, mask=None, dxy=(0, 0), bf16=False, k2=0, p2=0, dil=1):
    """Section 5 "Reuse".  x [H][W][cin] fp32, w [cout][k][k][cin]; k2 > 0: a kernel of k rows x k2 columns with paddings
    p (rows) and p2 (columns), w [cout][k][k2][cin]; dil: distance between taps."""
    x = np.ascontiguousarray(x, np.float32)
    w = np.ascontiguousarray(w, np.float32)
    Hin, Win, cin = x.shape
    cout = w.shape[0]
    kh, kw, ph, pw = k, (k2 if k2 > 0 else k), p, (p2 if k2 > 0 else p)
    assert w.shape == (cout, kh, kw, cin)
    Ho, Wo = (Hin + 2 * ph - ((kh - 1) * dil + 1)) // s + 1, (Win + 2 * pw - ((kw - 1) * dil + 1)) // s + 1
    out = np.zeros((Ho, Wo, cout), np.float32)
    if bias is not None:
        bias = np.ascontiguousarray(bias, np.float32)
    if mask is not None:
        mask = np.ascontiguousarray(mask, np.uint8)
        cache_prev = np.ascontiguousarray(cache_prev, np.float32)
        assert mask.shape == (Ho, Wo) and cache_prev.shape == out.shape
    lib().oc_conv_cached2(_p(x), Hin, Win, cin, _p(w), _p(bias), cout, kh, kw, s, ph, pw, int(dil), int(relu),
                          _p(cache_prev), _p(mask), int(dxy[0]), int(dxy[1]), int(bf16), _p(out))
    return out


def maxpool(x, k, s, p):
    x = np.ascontiguousarray(x, np.float32)
    H, W, Ch = x.shape
    out = np.zeros(((H + 2 * p - k) // s + 1, (W + 2 * p - k) // s + 1, Ch), np.float32)
    lib().oc_maxpool(_p(x), H, W, Ch, k, s, p, _p(out))
    return out


def avgpool(x, k, s, p, bf16=False):
    x = np.ascontiguousarray(x, np.float32)
    H, W, Cc = x.shape
    out = np.zeros(((H + 2 * p - k) // s + 1, (W + 2 * p - k) // s + 1, Cc), np.float32)
    lib().oc_avgpool(_p(x), H, W, Cc, int(k), int(s), int(p), int(bf16), _p(out))
    return out


def lrn(x, size, alpha, beta, kappa, within=False, bf16=False):
    x = np.ascontiguousarray(x, np.float32)
    H, W, Cc = x.shape
    out = np.zeros_like(x)
    lib().oc_lrn(_p(x), H, W, Cc, int(size), int(within), C.c_double(alpha), C.c_double(beta), C.c_double(kappa),
                 int(bf16), _p(out))
    return out


def concat(xs):
    xs = [np.ascontiguousarray(x, np.float32) for x in xs]
    H, W = xs[0].shape[:2]
    cs = np.array([x.shape[2] for x in xs], np.int32)
    out = np.zeros((H, W, int(cs.sum())), np.float32)
    ptrs = (C.c_void_p * len(xs))(*[x.ctypes.data for x in xs])
    lib().oc_concat(ptrs, _p(cs), len(xs), C.c_size_t(H * W), _p(out))
    return out


def fc(x, w, bias, relu, bf16=False):
    x = np.ascontiguousarray(x, np.float32)
    w = np.ascontiguousarray(w, np.float32)
    cout = w.shape[0]
    assert w.size == cout * x.size
    b = None if bias is None else np.ascontiguousarray(bias, np.float32)
    out = np.zeros((1, 1, cout), np.float32)
    lib().oc_fc(_p(x), C.c_size_t(x.size), _p(w), _p(b), cout, int(relu), int(bf16), _p(out))
    return out


def softmax(x, bf16=False):
    x = np.ascontiguousarray(x, np.float32)
    H, W, Cc = x.shape
    out = np.zeros_like(x)
    lib().oc_softmax(_p(x), C.c_size_t(H * W), Cc, int(bf16), _p(out))
    return out


def add(a, b, relu, bf16=False):
    a = np.ascontiguousarray(a, np.float32)
    b = np.ascontiguousarray(b, np.float32)
    out = np.zeros_like(a)
    lib().oc_add(_p(a), _p(b), a.size, int(relu), int(bf16), _p(out))
    return out


def relu(a):
    a = np.ascontiguousarray(a, np.float32)
    out = np.zeros_like(a)
    lib().oc_relu(_p(a), a.size, _p(out))
    return out


class Stream:
    """One video stream through one stack: holds the previous frame (cache key) and
    the previous feature maps (cache values), Section 3."""

    def __init__(self, layers, weights, biases, H, W, Ch=3, block=16, radius=16, max_ssd=None,
                 bf16=False, expiry=0, cap=1024, diamond=False, k_skip=1, extend_borders=False, exact_masks=False, cache_pool_add=False,
                 no_reuse=None):
        # no_reuse: per layer, non-zero = that conv layer is computed in full on every frame (None: all use the cache)
        self.no_reuse = None if no_reuse is None else np.ascontiguousarray(no_reuse, np.uint8)
        assert self.no_reuse is None or self.no_reuse.shape == (len(layers),)
        self.diamond, self.k_skip, self.extend_borders, self.exact_masks = diamond, k_skip, extend_borders, exact_masks
        self.cache_pool_add = bool(cache_pool_add) and bool(exact_masks)
        self.layers, self.H, self.W, self.Ch = layers, H, W, Ch
        self.block, self.radius, self.bf16, self.expiry, self.cap = block, radius, bf16, expiry, cap
        self.max_ssd = max_ssd if max_ssd is not None else 20 * block * block * Ch
        self.Lc = layers_to_c(layers)
        n = len(layers)
        self.w = [None if w is None else (round_bf16(w) if bf16 else np.ascontiguousarray(w, np.float32))
                  for w in weights]
        self.b = [None if b is None else np.ascontiguousarray(b, np.float32) for b in biases]
        self._wp = (C.c_void_p * n)(*[None if w is None else w.ctypes.data for w in self.w])
        self._bp = (C.c_void_p * n)(*[None if b is None else b.ctypes.data for b in self.b])
        # tensor shapes
        shapes = [(H, W, Ch)]
        for L in layers:
            h, w_, _ = shapes[L["in0"]]
            if L["type"] in (0, 1, 8):
                shapes.append((*window_out_hw(L, h, w_), L["cout"]))
            elif L["type"] == 6:
                shapes.append((1, 1, L["cout"]))
            else:
                shapes.append((h, w_, L["cout"]))
        self.shapes = shapes
        self.bufs = [[np.zeros(s, np.float32) for s in shapes] for _ in range(2)]
        self.prev_frame = None
        self.age = 0  # frames since the last full computation

    def reset(self):
        self.prev_frame = None
        self.age = 0

    def step(self, frame):
        """Process one frame.  Returns dict with tensors (list, current frame), match
        results (or None on a full frame), per-tensor rects / dxy."""
        frame = np.ascontiguousarray(frame, np.uint8)
        n = len(self.layers)
        full = self.prev_frame is None or (self.expiry > 0 and self.age >= self.expiry)
        cur, prev = self.bufs[0], self.bufs[1]
        m = None
        if full:
            r0 = np.zeros((0, 4), np.int32)
            n0, mx, my = -1, 0, 0
            self.age = 1
        else:
            if self.diamond:
                m = match_blocks_ds(frame, self.prev_frame, self.block, self.radius, self.max_ssd, self.k_skip)
            else:
                m = match_blocks(frame, self.prev_frame, self.block, self.radius, self.max_ssd, self.k_skip)
            r0 = merge_blocks(m["mask"], self.block)
            n0, mx, my = len(r0), int(m["gmv"][0]), int(m["gmv"][1])
            self.age += 1
        rects = np.zeros((n + 1, self.cap, 4), np.int32)
        n_rects = np.zeros(n + 1, np.int32)
        dxy = np.zeros((n + 1, 2), np.int32)
        cs = np.zeros(n + 1, np.int32)
        hw = np.zeros((n + 1, 2), np.int32)
        curp = (C.c_void_p * (n + 1))(*[t.ctypes.data for t in cur])
        prevp = (C.c_void_p * (n + 1))(*[t.ctypes.data for t in prev])
        masks = mp = None
        if self.exact_masks and not full:
            masks = propagate_masks(self.layers, self.H, self.W, m["mask"], self.block, mx, my, self.extend_borders)["masks"]
            mp = (C.c_void_p * (n + 1))(*[a.ctypes.data for a in masks])
        rc = lib().oc_run_stack(self.Lc, n, self._wp, self._bp, _p(frame), self.H, self.W, self.Ch,
                                int(self.bf16), _p(r0), n0, mx, my, curp, prevp, _p(rects),
                                self.cap, _p(n_rects), _p(dxy), _p(cs), _p(hw), int(self.extend_borders), mp,
                                int(self.cache_pool_add), None if self.no_reuse is None else _p(self.no_reuse))
        assert rc == 0
        self.bufs = [prev, cur]  # cur becomes next frame's prev
        self.prev_frame = frame.copy()
        return dict(tensors=cur, match=m, rects0=r0, full=full, masks=masks,
                    rects=[rects[t, :n_rects[t]].copy() for t in range(n + 1)],
                    dxy=dxy, cum_stride=cs, hw=hw)
