"""Thin ctypes binding of libdeepcache.so: argument marshalling only.

Every step of the path runs inside the library's kernels; torch is used for device
memory and the HIP stream.  There is no CPU fallback: importing the library fails
loudly if it has not been built.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
import torch

from . import synth

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdeepcache.so")

DC_F32, DC_BF16 = 0, 1
STATUS = {0: "DC_OK", -1: "DC_ERR_INVALID_ARG", -2: "DC_ERR_NULL_PTR", -3: "DC_ERR_BAD_SHAPE",
          -4: "DC_ERR_UNSUPPORTED", -5: "DC_ERR_WORKSPACE", -6: "DC_ERR_CAPACITY", -7: "DC_ERR_HIP"}

EXPORTS = ["dc_status_string", "dc_profile_create", "dc_profile_destroy", "dc_profile_reset",
           "dc_profile_elapsed_ms", "dc_overlap_create", "dc_overlap_destroy", "dc_overlap_pipeline", "dc_prefetch_match", "dc_conv_tuning", "dc_conv_kernel_name", "dc_conv_tile_shape", "dc_match_blocks", "dc_match_blocks_ds", "dc_match_blocks_opt", "dc_propagate_regions", "dc_propagate_regions_opt", "dc_conv_workspace_bytes",
           "dc_packed_weights_bytes", "dc_pack_conv_weights", "dc_cached_conv_layer", "dc_frame_to_tensor", "dc_torus_read", "dc_maxpool_layer", "dc_add_layer", "dc_avgpool_layer", "dc_lrn_layer", "dc_concat_layer", "dc_fc_layer", "dc_softmax_layer",
           "dc_stack_workspace_bytes", "dc_run_stack", "dc_stack_stats_fetch", "dc_cached_conv_layer_noalloc",
           "dc_propagate_masks_size", "dc_propagate_masks", "dc_probe_mfma_rate"]


class DcError(RuntimeError):
    def __init__(self, fn, status):
        super().__init__(f"{fn} returned {STATUS.get(status, status)}")
        self.status = status


class Rect(C.Structure):
    _fields_ = [("x", C.c_int32), ("y", C.c_int32), ("w", C.c_int32), ("h", C.c_int32)]


class Layer(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("type", "k", "s", "p", "cin", "cout", "relu", "in0", "in1", "in2", "in3",
                                         "within")] + [(n, C.c_float) for n in ("alpha", "beta", "kappa")] + \
               [(n, C.c_int32) for n in ("k2", "p2", "dil")]


class Regions(C.Structure):
    _fields_ = [("rects", C.POINTER(Rect)), ("capacity", C.c_int32), ("n", C.c_int32),
                ("dx", C.c_int32), ("dy", C.c_int32), ("cum_stride", C.c_int32),
                ("h", C.c_int32), ("w", C.c_int32)]


class MatchOptions(C.Structure):
    _fields_ = [("method", C.c_int32), ("k_skip", C.c_int32), ("extend_borders", C.c_int32), ("exact_masks", C.c_int32),
                ("cache_pool_add", C.c_int32), ("no_reuse", C.c_void_p), ("torus", C.c_int32), ("origins_out", C.c_void_p),
                ("origins_dev_out", C.POINTER(C.c_void_p)), ("device_plan", C.c_int32)]


DC_MATCH_EXHAUSTIVE, DC_MATCH_DIAMOND = 0, 1


class StackStats(C.Structure):
    _fields_ = [("full", C.c_int32), ("n_blocks", C.c_int32), ("n_reusable_blocks", C.c_int32),
                ("n_overflow_streams", C.c_int32), ("macs_full", C.c_int64), ("macs_needed", C.c_int64), ("macs_issued", C.c_int64),
                ("copy_bytes", C.c_int64), ("layer_reused_px", C.POINTER(C.c_int64)),
                ("layer_issued_macs", C.POINTER(C.c_int64)), ("layer_kernel_id", C.POINTER(C.c_int32)),
                ("profile", C.c_void_p)]


_lib = None


def lib():
    """Load libdeepcache.so (raises if it is missing: there is no fallback path)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} is not built; run `python -m paper_1712_01670_amd.build`")
        L = C.CDLL(LIB_PATH)
        L.dc_status_string.restype = C.c_char_p
        vp, i32, u32, sz = C.c_void_p, C.c_int32, C.c_uint32, C.c_size_t
        L.dc_profile_create.argtypes = [i32, C.POINTER(vp)]
        L.dc_profile_destroy.argtypes = [vp]
        L.dc_profile_reset.argtypes = [vp]
        L.dc_profile_elapsed_ms.argtypes = [vp, i32, C.POINTER(C.c_float)]
        L.dc_overlap_create.argtypes = [C.POINTER(vp)]
        L.dc_overlap_destroy.argtypes = [vp]
        L.dc_overlap_pipeline.argtypes = [vp, i32]
        L.dc_prefetch_match.argtypes = [vp, vp, vp, i32, i32, i32, i32, i32, i32, u32, vp, vp, vp, vp, vp, vp, vp, sz]
        L.dc_conv_tuning.argtypes = [i32, i32, i32, i32]
        L.dc_conv_kernel_name.argtypes = [i32, C.c_char_p, sz]
        L.dc_conv_tile_shape.argtypes = [vp, i32, i32, i32, i32] + [C.POINTER(i32)] * 4
        L.dc_match_blocks.argtypes = [vp, vp, i32, i32, i32, i32, i32, i32, u32, vp, vp, vp, vp, vp, vp]
        L.dc_match_blocks_ds.argtypes = [vp, vp, i32, i32, i32, i32, i32, i32, i32, u32, vp, vp, vp, vp, vp, vp]
        L.dc_match_blocks_opt.argtypes = [vp, vp, i32, i32, i32, i32, i32, i32, vp, u32, vp, vp, vp, vp, vp, vp]
        L.dc_propagate_regions.argtypes = [vp, i32, i32, i32, i32, vp, i32, i32, i32, i32, vp]
        L.dc_propagate_regions_opt.argtypes = [vp, i32, i32, i32, i32, vp, i32, i32, i32, i32, i32, vp]
        L.dc_conv_workspace_bytes.argtypes = [vp, i32, i32, i32, i32, C.POINTER(sz), C.POINTER(sz)]
        L.dc_packed_weights_bytes.argtypes = [vp, i32, C.POINTER(sz)]
        L.dc_pack_conv_weights.argtypes = [vp, vp, i32, vp, vp]
        L.dc_cached_conv_layer.argtypes = [vp, vp, vp, vp, vp, vp, vp, i32, i32, i32, vp, i32, vp, sz, vp, sz, vp]
        L.dc_frame_to_tensor.argtypes = [vp, vp, sz, i32, i32, i32, vp]
        L.dc_maxpool_layer.argtypes = [vp, vp, i32, i32, i32, i32, i32, i32, i32, i32, vp]
        L.dc_torus_read.argtypes = [vp, vp, vp, i32, i32, i32, i32, i32, i32, vp]
        L.dc_add_layer.argtypes = [vp, vp, vp, sz, i32, i32, vp]
        f32 = C.c_float
        L.dc_avgpool_layer.argtypes = [vp, vp, i32, i32, i32, i32, i32, i32, i32, i32, vp]
        L.dc_lrn_layer.argtypes = [vp, vp, i32, i32, i32, i32, i32, i32, f32, f32, f32, i32, vp]
        L.dc_concat_layer.argtypes = [vp, vp, i32, vp, sz, i32, vp]
        L.dc_fc_layer.argtypes = [vp, vp, vp, vp, i32, sz, i32, i32, i32, vp]
        L.dc_softmax_layer.argtypes = [vp, vp, sz, i32, i32, vp]
        L.dc_stack_workspace_bytes.argtypes = [vp, i32, i32, i32, i32, i32, i32, i32, C.POINTER(sz), C.POINTER(sz)]
        L.dc_run_stack.argtypes = [vp, i32, vp, vp, vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, i32, i32, u32, vp, i32, vp,
                                   vp, vp, vp, vp, vp, i32, vp, vp, sz, vp, sz, vp, vp, vp]
        L.dc_stack_stats_fetch.argtypes = [vp, sz, vp]
        L.dc_cached_conv_layer_noalloc.argtypes = [vp, vp, vp, vp, vp, vp, vp, i32, i32, i32, vp, i32, vp]
        L.dc_probe_mfma_rate.argtypes = [i32, vp, sz, C.POINTER(C.c_double), vp]
        L.dc_propagate_masks_size.argtypes = [vp, i32, i32, i32, i32, C.POINTER(sz), vp, C.POINTER(sz)]
        L.dc_propagate_masks.argtypes = [vp, i32, i32, i32, i32, i32, i32, vp, vp, i32, vp, vp, vp, sz, vp]
        for name in EXPORTS:
            if name != "dc_status_string":
                getattr(L, name).restype = i32
        _lib = L
    return _lib


def _check(fn, status):
    if status != 0:
        raise DcError(fn, status)


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr(t):
    return C.c_void_p(t.data_ptr()) if t is not None else None


def layers_to_c(layers):
    arr = (Layer * len(layers))()
    for i, L in enumerate(layers):
        for f, ct in Layer._fields_:
            v = L[f] if f in L else synth.LAYER_DEFAULTS[f]
            setattr(arr[i], f, float(v) if ct is C.c_float else int(v))
    return arr


def torch_dtype(dtype):
    return torch.bfloat16 if dtype == DC_BF16 else torch.float32


# --------------------------------------------------------------------------- #
# entry points (same names as the C ABI)                                      #
# --------------------------------------------------------------------------- #
def dc_match_blocks(cur, prev, block, radius, max_block_ssd):
    """cur, prev: uint8 cuda tensors [n][H][W][C].  Returns dict of cuda tensors."""
    assert cur.is_cuda and cur.dtype == torch.uint8 and cur.is_contiguous() and cur.dim() == 4
    assert prev.shape == cur.shape and prev.is_cuda and prev.dtype == torch.uint8 and prev.is_contiguous()
    n, H, W, Ch = cur.shape
    gh, gw = H // block, W // block
    dev = cur.device
    out = dict(mv=torch.empty((n, gh, gw, 2), dtype=torch.int16, device=dev),
               best_ssd=torch.empty((n, gh, gw), dtype=torch.int32, device=dev),
               gmv=torch.empty((n, 2), dtype=torch.int32, device=dev),
               n_pass=torch.empty((n,), dtype=torch.int32, device=dev),
               mask=torch.empty((n, gh, gw), dtype=torch.uint8, device=dev))
    _check("dc_match_blocks", lib().dc_match_blocks(
        _ptr(cur), _ptr(prev), n, H, W, Ch, block, radius, max_block_ssd, _ptr(out["mv"]),
        _ptr(out["best_ssd"]), _ptr(out["gmv"]), _ptr(out["n_pass"]), _ptr(out["mask"]), _stream()))
    return out


def dc_match_blocks_opt(cur, prev, block, radius, max_block_ssd, method=0, k_skip=1):
    """Either search (method DC_MATCH_EXHAUSTIVE / DC_MATCH_DIAMOND) with k-skip; result as dc_match_blocks."""
    assert cur.is_cuda and cur.dtype == torch.uint8 and cur.is_contiguous() and cur.dim() == 4
    assert prev.shape == cur.shape and prev.is_cuda and prev.dtype == torch.uint8 and prev.is_contiguous()
    n, H, W, Ch = cur.shape
    gh, gw = H // block, W // block
    dev = cur.device
    out = dict(mv=torch.empty((n, gh, gw, 2), dtype=torch.int16, device=dev),
               best_ssd=torch.empty((n, gh, gw), dtype=torch.int32, device=dev),
               gmv=torch.empty((n, 2), dtype=torch.int32, device=dev),
               n_pass=torch.empty((n,), dtype=torch.int32, device=dev),
               mask=torch.empty((n, gh, gw), dtype=torch.uint8, device=dev))
    opt = MatchOptions(int(method), int(k_skip))
    _check("dc_match_blocks_opt", lib().dc_match_blocks_opt(
        _ptr(cur), _ptr(prev), n, H, W, Ch, block, radius, C.byref(opt), max_block_ssd, _ptr(out["mv"]),
        _ptr(out["best_ssd"]), _ptr(out["gmv"]), _ptr(out["n_pass"]), _ptr(out["mask"]), _stream()))
    return out


def dc_match_blocks_ds(cur, prev, block, radius, max_block_ssd, k_skip=1):
    """Diamond search with k-skip; arguments and result as dc_match_blocks."""
    assert cur.is_cuda and cur.dtype == torch.uint8 and cur.is_contiguous() and cur.dim() == 4
    assert prev.shape == cur.shape and prev.is_cuda and prev.dtype == torch.uint8 and prev.is_contiguous()
    n, H, W, Ch = cur.shape
    gh, gw = H // block, W // block
    dev = cur.device
    out = dict(mv=torch.empty((n, gh, gw, 2), dtype=torch.int16, device=dev),
               best_ssd=torch.empty((n, gh, gw), dtype=torch.int32, device=dev),
               gmv=torch.empty((n, 2), dtype=torch.int32, device=dev),
               n_pass=torch.empty((n,), dtype=torch.int32, device=dev),
               mask=torch.empty((n, gh, gw), dtype=torch.uint8, device=dev))
    _check("dc_match_blocks_ds", lib().dc_match_blocks_ds(
        _ptr(cur), _ptr(prev), n, H, W, Ch, block, radius, int(k_skip), max_block_ssd, _ptr(out["mv"]),
        _ptr(out["best_ssd"]), _ptr(out["gmv"]), _ptr(out["n_pass"]), _ptr(out["mask"]), _stream()))
    return out


def _alloc_regions(n, cap):
    regs = (Regions * n)()
    store = [(Rect * cap)() for _ in range(n)]
    for i in range(n):
        regs[i].rects = C.cast(store[i], C.POINTER(Rect))
        regs[i].capacity = cap
    return regs, store


def _regions_to_py(r):
    n = min(r.n, r.capacity)
    rects = np.array([[r.rects[i].x, r.rects[i].y, r.rects[i].w, r.rects[i].h] for i in range(n)],
                     dtype=np.int32).reshape(-1, 4)
    return dict(rects=rects, n=r.n, dxy=(r.dx, r.dy), cum_stride=r.cum_stride, hw=(r.h, r.w))


def dc_propagate_regions(layers, H, W, block, block_mask, mx, my, cap=1024, extend_borders=False):
    """Host call.  block_mask: numpy uint8 [gh][gw].  Returns a list (per tensor) of dicts."""
    mask = np.ascontiguousarray(block_mask, np.uint8)
    gh, gw = mask.shape
    Lc = layers_to_c(layers)
    regs, store = _alloc_regions(len(layers) + 1, cap)
    _check("dc_propagate_regions_opt", lib().dc_propagate_regions_opt(
        Lc, len(layers), H, W, block, mask.ctypes.data_as(C.c_void_p), gh, gw, int(mx), int(my), int(extend_borders), regs))
    return [_regions_to_py(regs[t]) for t in range(len(layers) + 1)]


class _Workspace:
    """Device + pinned host scratch, grown on demand and kept per device."""

    def __init__(self):
        self.dev = None
        self.host = None
        self.busy = None   # event recorded after the last call that read the host staging

    def get(self, dev_bytes, host_bytes, device):
        if self.busy is not None:
            self.busy.synchronize()   # the previous upload must have left the staging buffer
            self.busy = None
        if self.dev is None or self.dev.numel() < dev_bytes or self.dev.device != device:
            self.dev = torch.empty(max(int(dev_bytes), 256), dtype=torch.uint8, device=device)
        if self.host is None or self.host.numel() < host_bytes:
            self.host = torch.empty(max(int(host_bytes), 256), dtype=torch.uint8, pin_memory=True)
        return self.dev, self.host


_conv_ws = _Workspace()


def dc_pack_conv_weights(layer, weights):
    """Packed copy of the weights [cout][3][3][cin] (cuda, fp32 or bf16) of a layer, or None if the layer has
    no packed form."""
    assert weights.is_cuda and weights.is_contiguous()
    dtype = DC_BF16 if weights.dtype == torch.bfloat16 else DC_F32
    Lc = layers_to_c([layer])
    nb = C.c_size_t()
    _check("dc_packed_weights_bytes", lib().dc_packed_weights_bytes(Lc, dtype, C.byref(nb)))
    if nb.value == 0:
        return None
    assert nb.value == weights.numel() * weights.element_size()
    packed = torch.empty_like(weights)
    _check("dc_pack_conv_weights", lib().dc_pack_conv_weights(Lc, _ptr(weights), dtype, _ptr(packed), _stream()))
    return packed


def dc_cached_conv_layer(layer, x, weights, bias, cache_prev=None, regions=None, out=None, packed=None):
    """x [n][Hin][Win][cin] cuda (fp32 or bf16); weights [cout][k][k][cin] same dtype; bias fp32 or None.
    regions: list (per stream) of (rects int32 [m][4], (dx, dy)) for the output tensor, or None.
    packed: the result of dc_pack_conv_weights for `weights`, or None."""
    assert x.is_cuda and x.is_contiguous() and x.dim() == 4
    dtype = DC_BF16 if x.dtype == torch.bfloat16 else DC_F32
    assert weights.dtype == x.dtype and weights.is_contiguous()
    n, Hin, Win, cin = x.shape
    Ho, Wo, _ = synth.tensor_shapes([dict(layer, in0=0)], Hin, Win, cin)[1]
    if out is None:
        out = torch.empty((n, Ho, Wo, layer["cout"]), dtype=x.dtype, device=x.device)
    Lc = layers_to_c([layer])
    regs = None
    keep = None
    max_rects = 1
    if regions is not None:
        assert len(regions) == n
        max_rects = max(1, max(len(r[0]) for r in regions))
        regs, keep = _alloc_regions(n, max_rects)
        for i, (rects, dxy) in enumerate(regions):
            regs[i].n = len(rects)
            regs[i].dx, regs[i].dy = int(dxy[0]), int(dxy[1])
            for j, r in enumerate(rects):
                keep[i][j] = Rect(*[int(v) for v in r])
    db, hb = C.c_size_t(), C.c_size_t()
    _check("dc_conv_workspace_bytes", lib().dc_conv_workspace_bytes(Lc, n, Hin, Win, max_rects, C.byref(db), C.byref(hb)))
    wd, wh = _conv_ws.get(db.value, hb.value, x.device)
    _check("dc_cached_conv_layer", lib().dc_cached_conv_layer(
        Lc, _ptr(x), _ptr(weights), _ptr(packed), _ptr(bias), _ptr(cache_prev), _ptr(out), n, Hin, Win, regs, dtype,
        _ptr(wd), wd.numel(), C.c_void_p(wh.data_ptr()), wh.numel(), _stream()))
    _conv_ws.busy = torch.cuda.Event()
    _conv_ws.busy.record()
    return out


def dc_cached_conv_layer_noalloc(layer, x, weights, bias, out, cache_prev=None, regions=None, packed=None):
    """dc_cached_conv_layer without workspaces (the library's static scratch); `out` is the caller's tensor."""
    assert x.is_cuda and x.is_contiguous() and x.dim() == 4 and out.is_cuda and out.is_contiguous()
    dtype = DC_BF16 if x.dtype == torch.bfloat16 else DC_F32
    assert weights.dtype == x.dtype and weights.is_contiguous() and out.dtype == x.dtype
    n, Hin, Win, cin = x.shape
    Lc = layers_to_c([layer])
    regs = keep = None
    if regions is not None:
        assert len(regions) == n
        regs, keep = _alloc_regions(n, max(1, max(len(r[0]) for r in regions)))
        for i, (rects, dxy) in enumerate(regions):
            regs[i].n = len(rects)
            regs[i].dx, regs[i].dy = int(dxy[0]), int(dxy[1])
            for j, r in enumerate(rects):
                keep[i][j] = Rect(*[int(v) for v in r])
    _check("dc_cached_conv_layer_noalloc", lib().dc_cached_conv_layer_noalloc(
        Lc, _ptr(x), _ptr(weights), _ptr(packed), _ptr(bias), _ptr(cache_prev), _ptr(out), n, Hin, Win, regs, dtype, _stream()))
    return out


def dc_propagate_masks(layers, H, W, Ch, block, block_mask, gmv, extend_borders=False):
    """Exact reuse maps on the GPU.  block_mask: cuda uint8 [n][gh][gw]; gmv: cuda int32 [n][2].  Returns
    (list per tensor of numpy bool [n][h][w], numpy int32 dxy [n][tensors][2])."""
    n = block_mask.shape[0]
    nl = len(layers)
    Lc = layers_to_c(layers)
    words, wsb = C.c_size_t(), C.c_size_t()
    offs = (C.c_int64 * (nl + 1))()
    _check("dc_propagate_masks_size", lib().dc_propagate_masks_size(Lc, nl, H, W, Ch, C.byref(words), offs, C.byref(wsb)))
    dev = block_mask.device
    bitmaps = torch.zeros((n, words.value), dtype=torch.int32, device=dev)
    dxy = torch.zeros((n, nl + 1, 2), dtype=torch.int32, device=dev)
    ws = torch.empty(wsb.value + 4 * n * (nl + 3) + 256, dtype=torch.uint8, device=dev)
    _check("dc_propagate_masks", lib().dc_propagate_masks(Lc, nl, n, H, W, Ch, block, _ptr(block_mask), _ptr(gmv),
                                                          int(extend_borders), _ptr(bitmaps), _ptr(dxy), _ptr(ws), ws.numel(), _stream()))
    torch.cuda.synchronize()
    raw = bitmaps.cpu().numpy().view(np.uint32)
    shapes = synth.tensor_shapes(layers, H, W, Ch)
    masks = []
    for t, (h, w, _) in enumerate(shapes):
        wpr = (w + 31) // 32
        rows = raw[:, offs[t]:offs[t] + h * wpr].reshape(n, h, wpr)
        bits = ((rows[..., None] >> np.arange(32, dtype=np.uint32)) & 1).astype(bool).reshape(n, h, wpr * 32)
        assert not bits[..., w:].any()
        masks.append(bits[..., :w])
    return masks, dxy.cpu().numpy()


def dc_frame_to_tensor(frames, dtype=DC_F32, c_tensor=None):
    cf = frames.shape[-1]
    ct = cf if c_tensor is None else int(c_tensor)
    out = torch.empty(tuple(frames.shape[:-1]) + (ct,), dtype=torch_dtype(dtype), device=frames.device)
    _check("dc_frame_to_tensor", lib().dc_frame_to_tensor(_ptr(frames), _ptr(out), frames.numel() // cf, cf, ct, dtype,
                                                          _stream()))
    return out


def pad_input_channels(layers, weights, Ch, dtype):
    """Give the layers that read tensor 0 a channel run of whole 16-byte vectors: cin is rounded up
    and their weights get zero input channels (the library zero-fills the extra channels of tensor 0).
    Returns (layers, weights, padded channel count)."""
    ve = 8 if dtype == DC_BF16 else 4
    cp = (Ch + ve - 1) // ve * ve
    if cp == Ch:
        return layers, weights, Ch
    layers = [dict(L) for L in layers]
    weights = list(weights)
    for i, L in enumerate(layers):
        if L["in0"] == 0 and L["type"] == synth.CONV:
            w = np.zeros(tuple(weights[i].shape[:3]) + (cp,), np.float32)
            w[..., :Ch] = weights[i]
            weights[i] = w
            L["cin"] = cp
        elif 0 in (L["in0"], L.get("in1", -1), L.get("in2", -1), L.get("in3", -1)):
            return [dict(L) for L in layers], weights, Ch   # a non-conv layer reads the input: leave it alone
    return layers, weights, cp


def dc_maxpool_layer(x, k, s, p):
    n, H, W, Ch = x.shape
    dtype = DC_BF16 if x.dtype == torch.bfloat16 else DC_F32
    out = torch.empty((n, (H + 2 * p - k) // s + 1, (W + 2 * p - k) // s + 1, Ch), dtype=x.dtype, device=x.device)
    _check("dc_maxpool_layer", lib().dc_maxpool_layer(_ptr(x), _ptr(out), n, H, W, Ch, k, s, p, dtype, _stream()))
    return out


def dc_avgpool_layer(x, k, s, p):
    n, H, W, Ch = x.shape
    dtype = DC_BF16 if x.dtype == torch.bfloat16 else DC_F32
    out = torch.empty((n, (H + 2 * p - k) // s + 1, (W + 2 * p - k) // s + 1, Ch), dtype=x.dtype, device=x.device)
    _check("dc_avgpool_layer", lib().dc_avgpool_layer(_ptr(x), _ptr(out), n, H, W, Ch, k, s, p, dtype, _stream()))
    return out


def dc_lrn_layer(x, size, alpha, beta, kappa, within=False):
    n, H, W, Ch = x.shape
    dtype = DC_BF16 if x.dtype == torch.bfloat16 else DC_F32
    out = torch.empty_like(x)
    _check("dc_lrn_layer", lib().dc_lrn_layer(_ptr(x), _ptr(out), n, H, W, Ch, int(size), int(within), C.c_float(alpha),
                                              C.c_float(beta), C.c_float(kappa), dtype, _stream()))
    return out


def dc_concat_layer(xs):
    n, H, W = xs[0].shape[:3]
    dtype = DC_BF16 if xs[0].dtype == torch.bfloat16 else DC_F32
    cs = [int(x.shape[3]) for x in xs]
    out = torch.empty((n, H, W, sum(cs)), dtype=xs[0].dtype, device=xs[0].device)
    ins = (C.c_void_p * len(xs))(*[x.data_ptr() for x in xs])
    chans = (C.c_int32 * len(xs))(*cs)
    _check("dc_concat_layer", lib().dc_concat_layer(ins, chans, len(xs), _ptr(out), C.c_size_t(n * H * W), dtype, _stream()))
    return out


def dc_fc_layer(x, w, bias, relu):
    n = x.shape[0]
    K = x[0].numel()
    cout = w.shape[0]
    assert w.numel() == cout * K and x.is_contiguous() and w.is_contiguous()
    dtype = DC_BF16 if x.dtype == torch.bfloat16 else DC_F32
    out = torch.empty((n, 1, 1, cout), dtype=x.dtype, device=x.device)
    _check("dc_fc_layer", lib().dc_fc_layer(_ptr(x), _ptr(w), _ptr(bias) if bias is not None else None, _ptr(out), n,
                                            C.c_size_t(K), cout, int(relu), dtype, _stream()))
    return out


def dc_softmax_layer(x):
    dtype = DC_BF16 if x.dtype == torch.bfloat16 else DC_F32
    out = torch.empty_like(x)
    Ch = x.shape[-1]
    _check("dc_softmax_layer", lib().dc_softmax_layer(_ptr(x), _ptr(out), C.c_size_t(x.numel() // Ch), Ch, dtype, _stream()))
    return out


def dc_add_layer(a, b, relu):
    dtype = DC_BF16 if a.dtype == torch.bfloat16 else DC_F32
    out = torch.empty_like(a)
    _check("dc_add_layer", lib().dc_add_layer(_ptr(a), _ptr(b), _ptr(out), a.numel(), int(relu), dtype, _stream()))
    return out


class StackRunner:
    """Owns the device buffers of n_streams video streams through one layer stack and
    calls dc_run_stack once per time step.  The cache policy (first frame, expiry every
    `expiry` frames, explicit reset) is decided here and passed down as force_full."""

    def __init__(self, layers, weights, biases, n_streams, H, W, Ch=3, block=16, radius=16,
                 max_block_ssd=None, dtype=DC_F32, expiry=0, max_rects=1024, device="cuda:0",
                 want_regions=False, pad_input=True, overlap=True, pipeline=True, pack_weights=True,
                 match_method=DC_MATCH_EXHAUSTIVE, k_skip=1, in_place=False, extend_borders=False, device_plan=False,
                 exact_masks=False, cache_pool_add=False, no_reuse=None, torus=False, want_origins=False):
        self.device_plan = bool(device_plan) and not in_place
        self.in_place = bool(in_place)
        self.last_in_place = False
        self._in_place_flag = C.c_int32(0)
        self.Ch_tensor = Ch
        if pad_input:
            layers, weights, self.Ch_tensor = pad_input_channels(layers, weights, Ch, dtype)
        self.layers, self.n, self.H, self.W, self.Ch = layers, n_streams, H, W, Ch
        self.block, self.radius, self.dtype, self.expiry = block, radius, dtype, expiry
        self.max_block_ssd = int(max_block_ssd if max_block_ssd is not None else synth.max_block_ssd(block, Ch))
        self.max_rects = max_rects
        self.exact_masks = bool(exact_masks)
        self.cache_pool_add = bool(cache_pool_add) and self.exact_masks
        # no_reuse: per layer, non-zero = that conv layer is computed in full on every frame (host array kept alive here)
        self._no_reuse = None if no_reuse is None else np.ascontiguousarray(no_reuse, np.uint8)
        assert self._no_reuse is None or self._no_reuse.shape == (len(layers),)
        # torus: the conv outputs are one buffer each, addressed from an origin that moves with every cached frame; nothing
        # is copied.  origins [n][tensor][2] = (ox, oy) is filled after every step when want_origins (the call then waits
        # for the planning): logical_tensors() needs it.
        self.torus = bool(torus) and self.device_plan
        self.origins = np.zeros((n_streams, len(layers) + 1, 2), np.int32) if (self.torus and want_origins) else None
        self._origins_dev = C.c_void_p(None)      # device address of the last frame's origins (torus), set by every step
        self.match_options = MatchOptions(int(match_method), int(k_skip), int(extend_borders), int(self.exact_masks),
                                          int(self.cache_pool_add),
                                          None if self._no_reuse is None else self._no_reuse.ctypes.data, int(self.torus),
                                          None if self.origins is None else self.origins.ctypes.data,
                                          C.pointer(self._origins_dev) if self.torus else None, int(self.device_plan))
        self.device = torch.device(device)
        td = torch_dtype(dtype)
        self.Lc = layers_to_c(layers)
        nl = len(layers)
        self.w = [None if w is None else torch.from_numpy(w).to(self.device).to(td).contiguous() for w in weights]
        self.b = [None if b is None else torch.from_numpy(b).to(self.device).float().contiguous() for b in biases]
        self._wp = (C.c_void_p * nl)(*[None if w is None else w.data_ptr() for w in self.w])
        torch.cuda.set_device(self.device)
        self.w_packed = [None if (w is None or not pack_weights or L["type"] != synth.CONV) else dc_pack_conv_weights(L, w)
                         for L, w in zip(layers, self.w)]
        self._wpp = (C.c_void_p * nl)(*[None if w is None else w.data_ptr() for w in self.w_packed])
        self._bp = (C.c_void_p * nl)(*[None if b is None else b.data_ptr() for b in self.b])
        self.shapes = synth.tensor_shapes(layers, H, W, self.Ch_tensor)
        # conv outputs are cache values: two copies (previous / current frame).  The rest is shared, except with
        # two frames in flight: alternating those tensors too spares the library its cross-stream waits for them.
        is_conv = [False] + [L["type"] == synth.CONV for L in layers]
        self._is_conv_out = is_conv
        both = bool(overlap and pipeline) or bool(cache_pool_add and exact_masks)
        # on a torus: the conv outputs, and the max-pooling outputs too when those layers use the cache
        single = [self.torus and (is_conv[t] or (self.cache_pool_add and t > 0 and layers[t - 1]["type"] == synth.MAXPOOL))
                  for t in range(nl + 1)]
        self.bufs = [[], []]
        for t, (h, w, c) in enumerate(self.shapes):
            a = torch.empty((n_streams, h, w, c), dtype=td, device=self.device)
            b = a if single[t] else (torch.empty_like(a) if (is_conv[t] or both) else a)
            self.bufs[0].append(a)
            self.bufs[1].append(b)
        # pointer tables [set of the conv outputs][set of the other tensors]: the two only differ after in-place frames
        self._tp = [[(C.c_void_p * (nl + 1))(*[self.bufs[cc if is_conv[t] else cn][t].data_ptr() for t in range(nl + 1)])
                     for cn in range(2)] for cc in range(2)]
        self.cur_other = 0    # set that receives the next frame's tensors other than conv outputs
        gh, gw = H // block, W // block
        dev = self.device
        self.mv = torch.zeros((n_streams, gh, gw, 2), dtype=torch.int16, device=dev)
        self.best_ssd = torch.zeros((n_streams, gh, gw), dtype=torch.int32, device=dev)
        self.gmv = torch.zeros((n_streams, 2), dtype=torch.int32, device=dev)
        self.n_pass = torch.zeros((n_streams,), dtype=torch.int32, device=dev)
        self.mask = torch.zeros((n_streams, gh, gw), dtype=torch.uint8, device=dev)
        db, hb = C.c_size_t(), C.c_size_t()
        _check("dc_stack_workspace_bytes", lib().dc_stack_workspace_bytes(
            self.Lc, nl, n_streams, H, W, Ch, block, max_rects, C.byref(db), C.byref(hb)))
        self.ws_dev = torch.empty(max(db.value, 256), dtype=torch.uint8, device=dev)
        self.ws_host = torch.empty(max(hb.value, 256), dtype=torch.uint8, pin_memory=True)
        self.prev_frames = None   # the caller's tensor of the previous step (cache key), kept by reference
        self.cur = 0          # index of the buffer set that receives the next frame
        self.have_prev = False
        self.age = 0
        self.stats = StackStats()
        self._reused = (C.c_int64 * nl)()
        self._issued = (C.c_int64 * nl)()
        self.stats.layer_reused_px = C.cast(self._reused, C.POINTER(C.c_int64))
        self.stats.layer_issued_macs = C.cast(self._issued, C.POINTER(C.c_int64))
        self._kid = (C.c_int32 * nl)()
        self.stats.layer_kernel_id = C.cast(self._kid, C.POINTER(C.c_int32))
        self.overlap = None
        if overlap:
            h = C.c_void_p()
            _check("dc_overlap_create", lib().dc_overlap_create(C.byref(h)))
            self.overlap = h
            if pipeline:
                _check("dc_overlap_pipeline", lib().dc_overlap_pipeline(h, 2))
        torch.cuda.synchronize(dev)   # weights and buffers are complete before any internal stream reads them
        self.regs = None
        if want_regions:
            self.regs, self._regs_store = _alloc_regions(n_streams * (nl + 1), max_rects)

    def __del__(self):
        try:
            if self.overlap:
                torch.cuda.synchronize()
                lib().dc_overlap_destroy(self.overlap)
                self.overlap = None
        except Exception:
            pass

    def reset(self):
        """Drop the cache (scene cut): the next frame is computed in full."""
        self.have_prev = False
        self.prev_frames = None
        self.age = 0

    def step(self, frames, force_full=False, next_frames=None):
        """frames: uint8 cuda tensor [n][H][W][C], resident (its producer has completed: the library reads it on
        streams of its own) and contiguous; it is kept by reference as the next step's previous frame, so the
        caller must not overwrite it before that step has run.  Returns the list of this frame's tensors, valid
        once the current stream is synchronised.  next_frames: the tensor the next step will be called with, if
        the caller has it already (a decoder one frame ahead): its matching is started at the end of this step
        (dc_prefetch_match), so the next step does not wait for it; mv / mask then belong to that frame."""
        assert frames.is_cuda and frames.dtype == torch.uint8 and frames.is_contiguous()
        assert tuple(frames.shape) == (self.n, self.H, self.W, self.Ch)
        c, p = self.cur, 1 - self.cur
        cn = self.cur_other
        full = force_full or not self.have_prev or (self.expiry > 0 and self.age >= self.expiry)
        _check("dc_run_stack", lib().dc_run_stack(
            self.Lc, len(self.layers), self._wp, self._wpp, self._bp, _ptr(frames), _ptr(self.prev_frames),
            self._tp[c][cn], self._tp[p][1 - cn if self.cache_pool_add else cn], self.n, self.H, self.W, self.Ch, self.dtype, self.block, self.radius,
            self.max_block_ssd, C.byref(self.match_options), int(full),
            C.byref(self._in_place_flag) if self.in_place else None, _ptr(self.mv), _ptr(self.best_ssd), _ptr(self.gmv), _ptr(self.n_pass),
            _ptr(self.mask), self.max_rects, self.regs, _ptr(self.ws_dev), self.ws_dev.numel(),
            C.c_void_p(self.ws_host.data_ptr()), self.ws_host.numel(), C.byref(self.stats), self.overlap, _stream()))
        if full and self.origins is not None:
            self.origins[:] = 0          # a full frame writes every tensor at its buffer's start
        self.age = 1 if full else self.age + 1
        self.have_prev = True
        self.prev_frames = frames
        self.last_full = full
        self.last_in_place = self.in_place and self._in_place_flag.value != 0
        self.cur_other = 1 - cn
        if not self.last_in_place:      # (an in-place frame updated the conv outputs in the previous frame's buffers)
            self.cur = p
        if next_frames is not None and self.overlap and not (self.expiry > 0 and self.age >= self.expiry):
            assert next_frames.is_cuda and next_frames.dtype == torch.uint8 and next_frames.is_contiguous()
            assert tuple(next_frames.shape) == (self.n, self.H, self.W, self.Ch)
            _check("dc_prefetch_match", lib().dc_prefetch_match(
                self.overlap, _ptr(next_frames), _ptr(frames), self.n, self.H, self.W, self.Ch, self.block, self.radius,
                self.max_block_ssd, C.byref(self.match_options), _ptr(self.mv), _ptr(self.best_ssd), _ptr(self.gmv),
                _ptr(self.n_pass), _ptr(self.mask), C.c_void_p(self.ws_host.data_ptr()), self.ws_host.numel()))
        if self.last_in_place:
            return [self.bufs[p if self._is_conv_out[t] else cn][t] for t in range(len(self.bufs[c]))]
        return [self.bufs[c if self._is_conv_out[t] else cn][t] for t in range(len(self.bufs[c]))]

    def read_tensor(self, t, tensors):
        """With torus: tensor t of the last step in its logical layout, written by dc_torus_read on the current stream
        (no wait for anything; without torus the tensor itself)."""
        x = tensors[t]
        if not self.torus:
            return x
        out = torch.empty_like(x)
        n, h, w, c = x.shape
        base = self._origins_dev.value
        _check("dc_torus_read", lib().dc_torus_read(_ptr(x), _ptr(out), C.c_void_p(base + 8 * t) if base else None,
                                                    2 * (len(self.layers) + 1), n, h, w, c, self.dtype, _stream()))
        return out

    def logical_tensors(self, tensors):
        """With torus: the tensors of the last step in their logical layout (copies; needs want_origins and a synchronised
        stream).  Pixel (x, y) of stream s of a tensor on the torus lies at ((x + ox) mod w, (y + oy) mod h) of its buffer."""
        if not self.torus:
            return tensors
        assert self.origins is not None
        out = []
        for t, x in enumerate(tensors):
            if not self.origins[:, t].any():
                out.append(x)
                continue
            out.append(torch.stack([torch.roll(x[s], shifts=(-int(self.origins[s, t, 1]), -int(self.origins[s, t, 0])), dims=(0, 1))
                                    for s in range(self.n)]))
        return out

    def read_stats(self):
        """Work counters of the last step (call after the stream has been synchronised): a frame planned on the GPU
        leaves them in the host workspace."""
        if self.device_plan and not self.last_full:
            _check("dc_stack_stats_fetch", lib().dc_stack_stats_fetch(C.c_void_p(self.ws_host.data_ptr()), self.ws_host.numel(),
                                                                      C.byref(self.stats)))
        return self.stats

    def enable_profile(self, on=True):
        """Attach (or detach) HIP-event brackets around every conv GEMM and copy launch."""
        if on and not self.stats.profile:
            h = C.c_void_p()
            _check("dc_profile_create", lib().dc_profile_create(2 * len(self.layers), C.byref(h)))
            self.stats.profile = h
        elif not on and self.stats.profile:
            lib().dc_profile_destroy(self.stats.profile)
            self.stats.profile = None

    def profile_ms(self):
        """After a synchronised step: dict layer -> (gemm_ms or None, copy_ms or None)."""
        nl = len(self.layers)
        out = {}
        for i, L in enumerate(self.layers):
            if L["type"] != synth.CONV:
                continue
            vals = []
            for slot in (i, nl + i):
                ms = C.c_float()
                rc = lib().dc_profile_elapsed_ms(self.stats.profile, slot, C.byref(ms))
                vals.append(ms.value if rc == 0 else None)
            out[i] = tuple(vals)
        lib().dc_profile_reset(self.stats.profile)
        return out

    def tile_shape(self, i):
        """(th, tw, nt, cfg) of conv layer i."""
        h, w, _ = self.shapes[self.layers[i]["in0"]]
        v = [C.c_int32() for _ in range(4)]
        _check("dc_conv_tile_shape", lib().dc_conv_tile_shape(layers_to_c([self.layers[i]]), self.n, h, w, self.dtype,
                                                            *[C.byref(x) for x in v]))
        return tuple(x.value for x in v)

    def regions(self, stream=0):
        """Regions of every tensor of `stream` for the last step (needs want_regions=True)."""
        nl = len(self.layers)
        return [_regions_to_py(self.regs[stream * (nl + 1) + t]) for t in range(nl + 1)]

    def layer_stats(self):
        nl = len(self.layers)
        return dict(reused_px=[self._reused[i] for i in range(nl)], issued_macs=[self._issued[i] for i in range(nl)],
                    kernel_id=[self._kid[i] for i in range(nl)])


def dc_probe_mfma_rate(lds_reads, device="cuda:0"):
    """Sustained bf16 MFMA rate in TFLOP/s (operands in registers, or re-read from LDS as the conv kernels do)."""
    scratch = torch.empty(4 << 20, dtype=torch.uint8, device=device)
    tf = C.c_double()
    _check("dc_probe_mfma_rate", lib().dc_probe_mfma_rate(int(lds_reads), _ptr(scratch), scratch.numel(), C.byref(tf), _stream()))
    return tf.value


def dc_conv_tuning(arrangement=-1, units_per_workgroup=-1, k_split=-1, chunk_index=-1):
    """Process-wide override of the conv launch heuristics (tests, experiments); -1 = automatic."""
    _check("dc_conv_tuning", lib().dc_conv_tuning(arrangement, units_per_workgroup, k_split, chunk_index))


def conv_kernel_name(kernel_id):
    buf = C.create_string_buffer(160)
    _check("dc_conv_kernel_name", lib().dc_conv_kernel_name(int(kernel_id), buf, 160))
    return buf.value.decode()
