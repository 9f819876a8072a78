// Internal declarations shared by the translation units of libdeepcache.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <functional>
#include <vector>

#include "deepcache.h"

namespace dc {

// ---- device-side plan records -------------------------------------------------
// One reusable rectangle of a conv layer's output, with its stream and source offset.
struct RectDev {
    int32_t x, y, w, h;
    int32_t stream, dx, dy, pad;
};
// One output tile (ty, tx in tile units) that holds at least one non-reusable pixel.
struct TileDev {
    int32_t stream, ty, tx;
    int32_t reuse_mask;  // bit 4*row + column: that pixel of the 4x4 tile is reusable and keeps the copied value
};
// Per-stream slice of the rectangle table.
struct RangeDev {
    int32_t begin, count;
};

// ---- tile geometry ------------------------------------------------------------
struct ConvTiling {
    int cfg;     // index into the kernel table
    int th, tw;  // output pixels per tile (rows, columns)
    int nt;      // output channels per workgroup
};
ConvTiling pick_tiling(const dc_layer& L, int Hout, int Wout, int n_streams, int dtype);

// ---- host region logic (dc_regions.cpp) ---------------------------------------
struct TensorRegions {
    std::vector<dc_rect> rects;
    int dx = 0, dy = 0, cum_stride = 1, h = 0, w = 0;
};
void merge_blocks(const uint8_t* mask, int gh, int gw, int B, std::vector<dc_rect>& out);
// extend_borders: for a stream with zero motion, windows may reach into the zero padding (see dc_match_options)
int propagate(const dc_layer* L, int n_layers, int H, int W, const std::vector<dc_rect>& rects0,
              int mx, int my, std::vector<TensorRegions>& out, bool extend_borders = false);
int validate_layers(const dc_layer* L, int n_layers, int H, int W, int C,
                    std::vector<int>* hs, std::vector<int>* ws, std::vector<int>* cs);

struct LayerPlan {
    std::vector<RectDev> rects;    // all streams
    std::vector<RangeDev> ranges;  // [n_streams]
    std::vector<TileDev> tiles;    // dirty tiles, all streams (empty when they were written to the staging buffer directly)
    size_t n_tiles = 0;            // number of dirty tiles, all streams
    int64_t reused_px = 0;
};
// Runs fn(0) .. fn(n-1) on the calling thread and a small pool of host threads (created on first use, at most
// 16 in all); returns when all are done.  Calls from several threads are serialised.  n < 4 runs inline.
void parallel_for(int n, const std::function<void(int)>& fn);
// Classify the tiles of one stream's output map against its rectangles and append.
void plan_stream(const dc_rect* rects, int n, int dx, int dy, int stream, int Hout, int Wout,
                 int th, int tw, LayerPlan& plan);

// ---- kernel launchers -----------------------------------------------------------
// Kernel rows / columns, paddings along y / x, distance between taps and the kernel's span in pixels, for a conv
// layer (k2, p2, dil of dc_layer); any other windowed layer: k x k, p, 1.
struct WindowGeom { int kh, kw, ph, pw, dil, eh, ew; };
inline WindowGeom window_geom(const dc_layer& l) {
    WindowGeom g{l.k, l.k, l.p, l.p, 1, l.k, l.k};
    if (l.type == DC_CONV) {
        if (l.k2 > 0) { g.kw = l.k2; g.pw = l.p2; }
        if (l.dil > 1) g.dil = l.dil;
        g.eh = (g.kh - 1) * g.dil + 1;
        g.ew = (g.kw - 1) * g.dil + 1;
    }
    return g;
}
inline bool plain_square(const dc_layer& l) { return !(l.type == DC_CONV && (l.k2 > 0 || l.dil > 1)); }

struct ConvLaunch {
    const void* in;
    const void* w;
    const void* w_packed = nullptr;   // optional: the same weights in the layout of launch_pack_weights
    const float* bias;
    void* out;
    int n_streams, Hin, Win, Cin, Hout, Wout, Cout, k, s, p, relu, dtype;
    int kw = 0, pw = 0, dil = 1;      // kw > 0: k rows x kw columns, paddings p / pw; dil: distance between taps
    // Tensors on a torus (optional, device): (ox, oy) of stream s at origin[s * origin_stride + 0 / 1]; nullptr: none.
    // Only the 3x3 stride-1 GEMM kernel and the first-layer kernels take them (the launch fails otherwise).
    const int32_t* in_origin = nullptr;
    const int32_t* out_origin = nullptr;
    int origin_stride = 0;
    ConvTiling tiling;
    const TileDev* tiles;  // device; nullptr: every tile of every stream
    int n_tiles;           // ignored when tiles == nullptr; with n_tiles_dev the capacity of the list
    const int* n_tiles_dev = nullptr;   // device: length of a list built on the GPU (the launch is sized for n_tiles)
    long n_tiles_hint = -1;             // with n_tiles_dev: a guess of that length for the launch heuristics (-1: none)
    const RectDev* rects;  // device
    const RangeDev* ranges;
    int* kernel_id = nullptr;  // out (host): which instantiation ran
    void* scratch = nullptr;   // device memory for partial sums when K is split among workgroups (optional)
    size_t scratch_bytes = 0;
};

// Upper bound of the scratch a convolution launch can make use of.
constexpr size_t kConvScratchBytes = (size_t)32 << 20;
// n_units: list length the launch must cover; n_hint: the length to tune for (equal unless the list is built on the GPU)
bool launch_conv_fast(const ConvLaunch& c, long n_units, long n_hint, hipStream_t st, hipError_t* err);
// Packed weights of a layer the 3x3 stride-1 GEMM kernel runs: [cout/16][cin*es/64][9][16][64 bytes], i.e. the
// 64-byte channel runs that one load instruction brings into LDS are contiguous.  0 bytes: no packed form.
size_t packed_weights_bytes(int k, int s, int cin, int cout, int dtype);
hipError_t launch_pack_weights(const void* w, void* packed, int cin, int cout, int dtype, hipStream_t st);
void conv_kernel_name(int id, char* buf, size_t n);
void conv_fast_kernel_name(int id, char* buf, size_t n);
void conv_set_tuning(int geom, int g, int ks, int kci);
hipError_t launch_conv(const ConvLaunch& c, hipStream_t st);

hipError_t launch_shifted_copy(const RectDev* rects_dev, int n_rects, int max_rect_w, int max_rect_h,
                               const void* prev, void* out, int Hout, int Wout, int Cout,
                               int dtype, hipStream_t st);
// Per-layer operands of the all-layers copy; RectDev::pad indexes this table.
struct CopyLayerDev {
    const void* prev;
    void* out;
    int32_t Hout, Wout, pv, pad;   // pv: 16-byte vectors per pixel
};
hipError_t launch_shifted_copy_all(const RectDev* rects_dev, int n_rects, const CopyLayerDev* layers_dev,
                                   size_t max_vec_per_rect, hipStream_t st);
hipError_t launch_match(const uint8_t* cur, const uint8_t* prev, int n_streams, int H, int W, int C,
                        int B, int R, int k_skip, uint32_t max_ssd, int16_t* mv, uint32_t* best_ssd,
                        int32_t* gmv, int32_t* n_pass, uint8_t* mask, hipStream_t st);
// Steps 1-4 with the diamond search in Step 2; only the blocks on every k-th grid row and column are searched.
hipError_t launch_match_diamond(const uint8_t* cur, const uint8_t* prev, int n_streams, int H, int W, int C, int B,
                                int R, int k_skip, uint32_t max_ssd, int16_t* mv, uint32_t* best_ssd, int32_t* gmv,
                                int32_t* n_pass, uint8_t* mask, hipStream_t st);
hipError_t launch_frame_to_tensor(const uint8_t* f, void* out, size_t n_pixels, int cf, int ct, int dtype,
                                  hipStream_t st);
// out[s][y][x] = in[s][(y + oy) mod H][(x + ox) mod W], (ox, oy) = origin[s * origin_stride + 0 / 1] (nullptr: a copy)
hipError_t launch_torus_read(const void* in, void* out, int n_streams, int H, int W, size_t pixel_bytes,
                             const int32_t* origin, int origin_stride, hipStream_t st);
hipError_t launch_maxpool(const void* in, void* out, int n_streams, int Hin, int Win, int C, int k,
                          int s, int p, int dtype, hipStream_t st);
hipError_t launch_add(const void* a, const void* b, void* out, size_t n, int relu, int dtype,
                      hipStream_t st);
// Max-pooling and add layers that use the cache (exact reuse maps): where the output tensor's bitmap is set the
// output is prev at +(dx, dy), elsewhere it is computed.  16-byte vectors of channels only (C * element size % 16 == 0).
struct CachedMap {
    const uint32_t* bitmaps;   // all streams' bitmaps
    int64_t bm_words;          // words per stream
    int32_t bm_off;            // first word of this tensor's bitmap
    const int32_t* dxy;        // [stream][n_tensors][2]
    int32_t n_tensors, tensor;
};
// 2 x 2 / stride 2 max-pooling of a tensor stored on a torus (origin [stream * origin_stride + 0 / 1] = ox, oy).
// out_origin != nullptr: the output lies on a torus too.  M != nullptr: the layer uses the cache, which on a torus
// means that a pixel whose bit is set in the output's reuse bitmap is left as it is.
hipError_t launch_maxpool2x2_torus(const void* in, void* out, int n_streams, int Hin, int Win, int C, int dtype,
                                   const int32_t* origin, const int32_t* out_origin, int origin_stride, const CachedMap* M,
                                   hipStream_t st);
hipError_t launch_maxpool_cached(const void* in, const void* prev, void* out, int n_streams, int Hin, int Win, int C, int k,
                                 int s, int p, int dtype, const CachedMap& M, hipStream_t st);
hipError_t launch_add_cached(const void* a, const void* b, const void* prev, void* out, int n_streams, int H, int W, int C,
                             int relu, int dtype, const CachedMap& M, hipStream_t st);
hipError_t launch_avgpool(const void* in, void* out, int n_streams, int Hin, int Win, int C, int k,
                          int s, int p, int dtype, hipStream_t st);
hipError_t launch_lrn(const void* in, void* out, int n_streams, int H, int W, int C, int size, int within,
                      float alpha, float beta, float kappa, int dtype, hipStream_t st);
// ins/cs: host arrays of n_in device pointers and channel counts
hipError_t launch_concat(const void* const* ins, const int* cs, int n_in, void* out, size_t n_pixels, int dtype,
                         hipStream_t st);
hipError_t launch_softmax(const void* in, void* out, size_t n_pixels, int C, int dtype, hipStream_t st);
// x: [n_streams][K], w: [cout][K], out: [n_streams][cout]
hipError_t launch_fc(const void* x, const void* w, const float* bias, void* out, int n_streams, size_t K, int cout,
                     int relu, int dtype, hipStream_t st);
// Producer tensors of a DC_CONCAT layer in channel order; returns their number (2..4).
int concat_inputs(const dc_layer& l, int* ids);

// ---- planning on the GPU (dc_plan.hip): Step 5 of Section 4 and the propagation of Section 5 without the host ------
// The host path above reads the block mask back, plans and uploads; here three small kernels do the same from the
// mask in device memory, so that a cached frame needs no host wait:
//   plan_regions_kernel  one wavefront per stream: merge (Step 5), then every layer's row of Table 2 in turn
//   plan_masks_kernel    per conv layer, stream and 256 units: the 16-bit mask of reusable pixels of every 4x4 unit
//   plan_lists_kernel    compacts the units with a non-reusable pixel into the layer's list (stream-major, raster
//                        order: the order of the host path) and leaves the list lengths and the work counters
// The convolutions are then launched for the longest possible list and read its length from memory; the reusable
// pixels are copied per unit from the masks (shifted_copy_units_kernel).
constexpr int kPlanMaxTensors = 192;     // tensors of a stack the device tables hold
constexpr int kPlanMaxRects = 256;       // rectangles per list (a longer list: the stream reuses nothing)
constexpr int kPlanChunk = 256;          // units per workgroup of the mask / list kernels
struct PlanLayerDev {                    // one layer; tensor i + 1 is its output
    int32_t type, k, s, p, in0, in1, in2, in3, within;
    int32_t kw, pw, dil;                 // conv layers: kernel columns, their padding, distance between taps (k, p: rows)
};
struct PlanTensorDev { int32_t h, w, cum_stride, bm_off; };   // bm_off: first word of the tensor's bitmap (exact maps)
struct PlanConvDev {                     // one conv layer's share of the plan area (offsets in bytes from its start)
    int32_t tensor, Hout, Wout, units_x, units_y, n_chunks;
    int32_t no_reuse;                    // 1: this layer is computed in full on every frame (its unit masks are all zero)
    int32_t pad1;
    int64_t umask_off, count_off, list_off, pad2;
};
// What the list kernel leaves for the host, per frame: {reusable blocks, overflowed streams, 0, 0}, then per conv
// layer {reused pixels (int64), list length (int32), 0}.
struct PlanStatsHead { int32_t n_reusable_blocks, n_overflow_streams, pad0, pad1; };
struct PlanStatsConv { int64_t reused_px; int32_t n_units, pad; };
struct PlanDev {                         // device addresses of one frame's plan, handed to the kernels by value
    const PlanLayerDev* layers;
    const PlanTensorDev* tensors;
    const PlanConvDev* convs;
    int32_t n_layers, n_convs, n_streams, cap;
    dc_rect* rects;                      // [stream][tensor][cap]
    int32_t* nrect;                      // [stream][tensor]
    int32_t* dxy;                        // [stream][tensor][2]
    int32_t* stream_info;                // [stream][2]: reusable blocks, 1 if a list overflowed
    unsigned char* area;                 // base of the per-layer arrays (PlanConvDev offsets)
    int32_t* n_units;                    // [conv]
    void* stats;                         // PlanStatsHead + n_convs x PlanStatsConv; device memory or pinned host memory
    // exact reuse maps (optional): one bit per pixel, rows of (w + 31) / 32 words, tensor t of stream s at
    // bitmaps + s * bm_words + tensors[t].bm_off
    uint32_t* bitmaps;
    int64_t bm_words;
    // Conv outputs kept on a torus (optional): origin [stream][tensor][2] = (ox, oy), the buffer position of the
    // tensor's pixel (0, 0); this frame's = the previous frame's + the tensor's offset, modulo the map's size, for
    // conv outputs, (0, 0) for every other tensor.  origin_prev == nullptr: the previous frame left none (all zero).
    int32_t* origin;
    const int32_t* origin_prev;
    int pool_torus;          // 1: the outputs of max-pooling layers lie on a torus as well (they use the cache too)
};
// Position in the buffer of pixel v of a tensor axis of n pixels whose origin is o (0 <= o < n, 0 <= v < n).
__host__ __device__ inline int torus_wrap(int v, int o, int n) { const int p = v + o; return p >= n ? p - n : p; }
hipError_t launch_plan(const PlanDev& P, const uint8_t* block_mask, const int32_t* gmv, int gh, int gw, int block,
                       int extend_borders, int max_chunks, hipStream_t st);
// The same with exact reuse maps instead of rectangles: plan_erode_kernel (one workgroup per stream) derives every
// tensor's bitmap from its producers' (a pixel is reusable iff every tap of its window is), then the unit masks are
// cut out of the bitmaps and listed as above.  with_lists = false stops after the bitmaps.
hipError_t launch_plan_exact(const PlanDev& P, const uint8_t* block_mask, const int32_t* gmv, int gh, int gw, int block,
                             int extend_borders, int max_chunks, bool with_lists, hipStream_t st);
// The same for one conv layer whose rectangles come from the host and are small enough to travel as kernel arguments
// (no staging buffer, no copy): a set-up kernel writes them where the mask and list kernels expect them.
constexpr int kArgMaxRects = 128;        // rectangles of all streams together
constexpr int kArgMaxStreams = 32;
struct PlanArgRects {
    dc_rect r[kArgMaxRects];             // stream after stream
    int32_t first[kArgMaxStreams + 1];   // stream s owns r[first[s]] .. r[first[s + 1] - 1]
    int32_t dxy[kArgMaxStreams][2];      // its source offset
};
// P describes a stack of no layers (the rectangles belong to tensor 0 = the conv output); P.convs must be writable.
hipError_t launch_plan_from_args(const PlanDev& P, const PlanConvDev& conv, const PlanArgRects& R, hipStream_t st);

// One conv layer of the per-unit copy: out[p] = prev[p + d] for every pixel whose bit is set in its unit's mask.
struct CopyUnitsLayer {
    const void* prev;
    void* out;
    const uint16_t* umask;               // [stream][units_y][units_x]
    int32_t tensor, Hout, Wout, units_x, units_y, vec_per_px;
    int32_t units_per_group, vec_shift;   // set by the launcher: units per workgroup; log2(vec_per_px) or -1
};
constexpr int kCopyUnitsMaxLayers = 32;
hipError_t launch_shifted_copy_units(const CopyUnitsLayer* layers, int n_layers, const int32_t* dxy, int n_tensors,
                                     int n_streams, int vec_bytes, hipStream_t st);

// Sustained bf16 MFMA rate (dc_probe.hip): `launches` back-to-back launches of wgs workgroups x 8 wavefronts x steps x
// 16 MFMAs (16x16x32); the duration of the last one.  scratch: 4 MiB of device memory.
hipError_t probe_mfma_rate(int lds_reads, void* scratch, int wgs, int steps, int launches, float* last_ms, hipStream_t st);

// Event pairs for kernel timing (measurement aid).
struct Profile {
    std::vector<hipEvent_t> ev;   // 2 per slot: start, stop
    std::vector<uint8_t> used;
};

// Streams and events of an overlap handle (Section 7.6: the stages can be carried out asynchronously).
//  - aux: the matching of a frame and the read-back of its mask run here, next to the previous frame's layers;
//  - pipeline: consecutive frames alternate between two work streams; layer i of a frame waits for layer i of
//    the previous frame (its cache) and for the previous frame's readers of every single-buffered tensor it
//    overwrites, so two frames are in flight and the second fills the CUs the first leaves idle.  A tensor
//    whose buffer is not the previous frame's but that of the frame before it (a caller that alternates all
//    its tensors, not only the conv outputs) was last used on this same stream and needs neither wait nor event.
struct Overlap {
    hipStream_t aux = nullptr;
    hipEvent_t match_done = nullptr;                  // mask and motion of the current frame are in host memory
    hipEvent_t upload_done[2] = {nullptr, nullptr};   // plan upload from staging half 0 / 1 has completed
    bool pending[2] = {false, false};
    int parity = 0;
    bool pipeline = false;
    hipStream_t work[2] = {nullptr, nullptr};
    hipEvent_t frame_done[2] = {nullptr, nullptr};
    std::vector<hipEvent_t> layer_done[2];            // [frame parity][layer]
    std::vector<char> recorded[2];                    // [frame parity][layer]: that frame recorded layer_done
    bool frame_recorded[2] = {false, false};          // that frame recorded frame_done
    std::vector<const void*> last_cur[2];             // [frame parity]: tensors_cur of that stream's last frame
    int frame_parity = 0;
    // planning on the GPU: matching and planning kernels of consecutive frames run on `aux`, ahead of the layers;
    // a frame's plan lives in one of three areas (two frames in flight and one being planned)
    hipEvent_t plan_done[3] = {nullptr, nullptr, nullptr};   // the plan in that area is complete
    hipEvent_t area_free[3] = {nullptr, nullptr, nullptr};   // the layers of the frame that used the area are done
    bool area_recorded[3] = {false, false, false};
    int plan_counter = 0;
    // look-ahead matching: the arguments of a match already started for the next frame
    struct Prefetch {
        bool valid = false;
        const void *cur = nullptr, *prev = nullptr, *mv = nullptr, *best_ssd = nullptr, *gmv = nullptr, *n_pass = nullptr,
                   *mask = nullptr, *ws_host = nullptr;
        int n_streams = 0, H = 0, W = 0, C = 0, block = 0, radius = 0, method = 0, k_skip = 1;
        uint32_t max_block_ssd = 0;
    } prefetch;
};

inline size_t dtype_size(int dtype) { return dtype == DC_BF16 ? 2 : 4; }
inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

}  // namespace dc
