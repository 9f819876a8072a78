// C ABI entry points: argument validation, host-side planning, kernel sequencing.
#include <algorithm>
#include <chrono>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>

#include "dc_internal.h"

using namespace dc;

namespace {

inline hipStream_t as_stream(void* s) { return reinterpret_cast<hipStream_t>(s); }

#define DC_TRY_HIP(expr)                      \
    do {                                      \
        hipError_t e__ = (expr);              \
        if (e__ != hipSuccess) return DC_ERR_HIP; \
    } while (0)

bool rects_disjoint_inside(const dc_rect* r, int n, int W, int H, int dx, int dy) {
    for (int i = 0; i < n; ++i) {
        if (r[i].w <= 0 || r[i].h <= 0 || r[i].x < 0 || r[i].y < 0 || r[i].x + r[i].w > W ||
            r[i].y + r[i].h > H)
            return false;
        if (r[i].x + dx < 0 || r[i].y + dy < 0 || r[i].x + dx + r[i].w > W || r[i].y + dy + r[i].h > H)
            return false;
        for (int j = 0; j < i; ++j) {
            bool apart = r[i].x + r[i].w <= r[j].x || r[j].x + r[j].w <= r[i].x ||
                         r[i].y + r[i].h <= r[j].y || r[j].y + r[j].h <= r[i].y;
            if (!apart) return false;
        }
    }
    return true;
}

// Bytes of plan data for one conv layer, worst case.
size_t plan_bytes(int n_streams, int Hout, int Wout, const ConvTiling& t, int max_rects) {
    size_t tiles = (size_t)n_streams * ((Hout + t.th - 1) / t.th) * ((Wout + t.tw - 1) / t.tw);
    return align_up(tiles * sizeof(TileDev), 256) + align_up((size_t)n_streams * max_rects * sizeof(RectDev), 256) +
           align_up((size_t)n_streams * sizeof(RangeDev), 256);
}

// Serialise a plan into host staging at `host` and return the three device addresses
// it will have once copied to `dev` (same offsets).
struct PlanAddr {
    const TileDev* tiles;
    const RectDev* rects;
    const RangeDev* ranges;
    size_t bytes;
};
PlanAddr pack_plan(const LayerPlan& plan, unsigned char* host, unsigned char* dev) {
    size_t off = 0;
    PlanAddr a;
    a.tiles = reinterpret_cast<const TileDev*>(dev + off);
    if (!plan.tiles.empty()) std::memcpy(host + off, plan.tiles.data(), plan.tiles.size() * sizeof(TileDev));
    off += align_up(plan.n_tiles * sizeof(TileDev), 256);       // the caller may fill the tile list itself
    a.rects = reinterpret_cast<const RectDev*>(dev + off);
    if (!plan.rects.empty()) std::memcpy(host + off, plan.rects.data(), plan.rects.size() * sizeof(RectDev));
    off += align_up(plan.rects.size() * sizeof(RectDev), 256);
    a.ranges = reinterpret_cast<const RangeDev*>(dev + off);
    if (!plan.ranges.empty()) std::memcpy(host + off, plan.ranges.data(), plan.ranges.size() * sizeof(RangeDev));
    off += align_up(plan.ranges.size() * sizeof(RangeDev), 256);
    a.bytes = off;
    return a;
}

// Channel count of tensor 0: the cin of the layers that read it (they must agree); it may exceed the
// frame's channel count, the extra channels are zero.
int input_channels(const dc_layer* L, int n_layers, int c_frame) {
    int c = -1;
    for (int i = 0; i < n_layers; ++i) {
        if (L[i].type == DC_CONCAT) {             // its cin is the sum of its producers' channels
            int ids[4];
            const int m = concat_inputs(L[i], ids);
            for (int j = 0; j < m; ++j)
                if (ids[j] == 0) return -1;       // a concat reads layer outputs only
            continue;
        }
        if (L[i].in0 == 0 || (L[i].type == DC_ADD && L[i].in1 == 0)) {
            if (c >= 0 && L[i].cin != c) return -1;
            c = L[i].cin;
        }
    }
    return c < 0 ? c_frame : c;
}

int check_conv_layer(const dc_layer* l) {
    if (l->type != DC_CONV) return DC_ERR_INVALID_ARG;
    const WindowGeom g = window_geom(*l);
    if (g.kh < 1 || g.kw < 1 || l->s < 1 || g.ph < 0 || g.pw < 0 || g.ph >= g.eh || g.pw >= g.ew || l->cin < 1 || l->cout < 1)
        return DC_ERR_INVALID_ARG;
    if (l->relu < 0 || l->relu > 2 || l->k2 < 0 || l->dil < 0 || l->dil > 64 || g.kh > 64 || g.kw > 64) return DC_ERR_INVALID_ARG;
    return DC_OK;
}

// Waits for an event by polling: the host thread is needed again within tens of microseconds, which a
// blocking wait's wake-up latency would double.  After 2 ms of polling it blocks instead.
hipError_t spin_wait(hipEvent_t e) {
    const auto t0 = std::chrono::steady_clock::now();
    for (int i = 0;; ++i) {
        const hipError_t q = hipEventQuery(e);
        if (q != hipErrorNotReady) return q;
        if ((i & 63) == 63 && std::chrono::steady_clock::now() - t0 > std::chrono::milliseconds(2))
            return hipEventSynchronize(e);
    }
}

// Small plans (one or a few streams) go from the pinned staging buffer to the device with a kernel that reads
// the host memory through its device address: a launch costs the host a few microseconds where an asynchronous
// copy on an idle stream measured 25.  Large plans (64 streams: megabytes) are faster through the copy engine,
// and pageable staging memory has no device address.
__global__ void __launch_bounds__(256) upload_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n_vec) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n_vec; i += (size_t)gridDim.x * blockDim.x)
        dst[i] = src[i];
}

// Device address of a host buffer: nullptr if it is not pinned.  Asked on every call: a caller may free a
// pinned buffer and pass pageable memory at the same address later.
const unsigned char* device_alias(void* host) {
    void* d = nullptr;
    if (hipHostGetDevicePointer(&d, host, 0) != hipSuccess) { d = nullptr; (void)hipGetLastError(); }
    return static_cast<const unsigned char*>(d);
}

hipError_t upload_plans(void* dst_dev, const unsigned char* src_host, size_t bytes, void* ws_host, hipStream_t st) {
    if (bytes > 256 * 1024) return hipMemcpyAsync(dst_dev, src_host, bytes, hipMemcpyHostToDevice, st);
    const unsigned char* alias = device_alias(ws_host);
    if (!alias || bytes % 16 || reinterpret_cast<uintptr_t>(dst_dev) % 16 || reinterpret_cast<uintptr_t>(src_host) % 16)
        return hipMemcpyAsync(dst_dev, src_host, bytes, hipMemcpyHostToDevice, st);
    const unsigned char* src = alias + (src_host - static_cast<const unsigned char*>(ws_host));
    const size_t n_vec = bytes / 16;
    const unsigned grid = (unsigned)std::min<size_t>((n_vec + 255) / 256, 1024);
    hipLaunchKernelGGL(upload_kernel, dim3(grid), dim3(256), 0, st, reinterpret_cast<const uint4*>(src),
                       static_cast<uint4*>(dst_dev), n_vec);
    return hipGetLastError();
}

// Copy + conv launches of one layer given its packed plan on the device.
struct Bracket {   // records a profile slot around a launch when a profile is attached
    Profile* p; int slot; hipStream_t st;
    Bracket(Profile* p_, int slot_, hipStream_t st_) : p(p_), slot(slot_), st(st_) {
        if (p && slot >= 0 && (size_t)slot < p->used.size()) { (void)hipEventRecord(p->ev[2 * slot], st); }
        else p = nullptr;
    }
    ~Bracket() {
        if (p) { (void)hipEventRecord(p->ev[2 * slot + 1], st); p->used[slot] = 1; }
    }
};

int run_conv_planned(const dc_layer& l, const void* in, const void* w, const float* bias,
                     const void* cache_prev, void* out, int n_streams, int Hin, int Win, int dtype,
                     const ConvTiling& tiling, const LayerPlan* plan, const PlanAddr* addr, hipStream_t st,
                     Profile* prof = nullptr, int gemm_slot = -1, int copy_slot = -1, int* kernel_id = nullptr,
                     bool copy_done = false, void* scratch = nullptr, size_t scratch_bytes = 0,
                     const void* w_packed = nullptr, const TileDev* dev_tiles = nullptr, int dev_capacity = 0,
                     const int* dev_count = nullptr, long dev_hint = -1, const int32_t* in_origin = nullptr,
                     const int32_t* out_origin = nullptr, int origin_stride = 0) {
    const WindowGeom wg = window_geom(l);
    const int Hout = (Hin + 2 * wg.ph - wg.eh) / l.s + 1, Wout = (Win + 2 * wg.pw - wg.ew) / l.s + 1;
    ConvLaunch c;
    c.kernel_id = kernel_id;
    if (kernel_id) *kernel_id = -1;
    c.in = in; c.w = w; c.w_packed = w_packed; c.bias = bias; c.out = out;
    c.n_streams = n_streams; c.Hin = Hin; c.Win = Win; c.Cin = l.cin;
    c.Hout = Hout; c.Wout = Wout; c.Cout = l.cout; c.k = l.k; c.s = l.s; c.p = l.p; c.relu = l.relu;
    if (!plain_square(l)) { c.kw = wg.kw; c.pw = wg.pw; c.dil = wg.dil; }
    c.dtype = dtype; c.tiling = tiling;
    c.scratch = scratch; c.scratch_bytes = scratch_bytes;
    c.in_origin = in_origin; c.out_origin = out_origin; c.origin_stride = origin_stride;
    if (dev_tiles) {      // a list the planning kernels built: its length is in device memory, the copies are done
        c.tiles = dev_tiles; c.n_tiles = dev_capacity; c.n_tiles_dev = dev_count; c.n_tiles_hint = dev_hint;
        c.rects = nullptr; c.ranges = nullptr;
        Bracket b(prof, gemm_slot, st);
        DC_TRY_HIP(launch_conv(c, st));
        return DC_OK;
    }
    if (!plan) {
        c.tiles = nullptr; c.n_tiles = 0; c.rects = nullptr; c.ranges = nullptr;
        Bracket b(prof, gemm_slot, st);
        DC_TRY_HIP(launch_conv(c, st));
        return DC_OK;
    }
    int mw = 0, mh = 0;
    for (const RectDev& r : plan->rects) { mw = r.w > mw ? r.w : mw; mh = r.h > mh ? r.h : mh; }
    if (!plan->rects.empty() && !copy_done) {
        Bracket b(prof, copy_slot, st);
        DC_TRY_HIP(launch_shifted_copy(addr->rects, (int)plan->rects.size(), mw, mh, cache_prev, out, Hout, Wout,
                                       l.cout, dtype, st));
    }
    if (plan->n_tiles) {
        Bracket b(prof, gemm_slot, st);
        c.tiles = addr->tiles; c.n_tiles = (int)plan->n_tiles; c.rects = addr->rects; c.ranges = addr->ranges;
        DC_TRY_HIP(launch_conv(c, st));
    }
    return DC_OK;
}

// ---- planning on the GPU: layout of the tables and of one frame's plan in the device workspace ----
constexpr size_t kDevHostRegion = 64 * 1024;    // tail of the host workspace: header, two counter slots, table staging
constexpr size_t kDevHostSlot = 4096;
constexpr int kPlanMaxConvs = 128;
constexpr uint64_t kDevHostMagic = 0x6463706c616e3031ull;
struct DevHostConv { int32_t layer, cout_bytes; int64_t mac_px, px_total; };
struct DevHostHeader {                          // host-only bookkeeping of the workspace pair
    uint64_t magic, signature;
    const void* ws_dev;
    int32_t n_layers, n_convs, last_slot, n_blocks;
    int64_t macs_full;
    int32_t origin_area;                        // torus frames: the plan area that holds the previous frame's origins (-1: none)
    int32_t torus;                              // 1: the last frame planned here copied nothing
    DevHostConv conv[kPlanMaxConvs];
};
static_assert(sizeof(DevHostHeader) <= kDevHostSlot, "header fits its slot");
static_assert(sizeof(PlanStatsHead) + kPlanMaxConvs * sizeof(PlanStatsConv) <= kDevHostSlot, "counters fit their slot");

struct DevPlanLayout {
    std::vector<PlanLayerDev> layers;
    std::vector<PlanTensorDev> tensors;
    std::vector<PlanConvDev> convs;
    std::vector<int> conv_layer;                // layer index of every conv
    size_t table_bytes = 0, off_tensors = 0, off_convs = 0;
    size_t frame_bytes = 0, off_nrect = 0, off_dxy = 0, off_origin = 0, off_info = 0, off_nunits = 0, off_stats = 0, off_area = 0;
    size_t off_bitmaps = 0;
    int64_t bm_words = 0;                       // words of all bitmaps of one stream (exact reuse maps)
    int cap = 0, max_chunks = 0;
    bool ok = false;
};

// Tables and sizes for n_streams streams of this stack; ok = false if the device kernels cannot take it (the host
// path then plans the frame).
void device_plan_layout(const dc_layer* L, int n_layers, const std::vector<int>& hs, const std::vector<int>& ws,
                        int n_streams, int max_rects, DevPlanLayout& d, const uint8_t* no_reuse = nullptr) {
    d.ok = false;
    const int nt = n_layers + 1;
    if (nt > kPlanMaxTensors) return;
    d.cap = max_rects < kPlanMaxRects ? max_rects : kPlanMaxRects;
    d.layers.resize(n_layers); d.tensors.resize(nt); d.convs.clear(); d.conv_layer.clear();
    d.tensors[0] = PlanTensorDev{hs[0], ws[0], 1, 0};
    int64_t bm = ((int64_t)hs[0] * ((ws[0] + 31) / 32) + 63) / 64 * 64;          // every bitmap starts on a 256-byte line
    for (int i = 0; i < n_layers; ++i) {
        const dc_layer& l = L[i];
        const WindowGeom wg = window_geom(l);
        d.layers[i] = PlanLayerDev{l.type, l.k, l.s, l.p, l.in0, l.in1, l.in2, l.in3, l.within, wg.kw, wg.pw, wg.dil};
        const bool windowed = l.type == DC_CONV || l.type == DC_MAXPOOL || l.type == DC_AVGPOOL;
        const int cum = d.tensors[l.in0].cum_stride * (windowed ? l.s : 1);
        if (bm > 0x7fffffffll) return;
        d.tensors[i + 1] = PlanTensorDev{hs[i + 1], ws[i + 1], cum, (int32_t)bm};
        bm += ((int64_t)hs[i + 1] * ((ws[i + 1] + 31) / 32) + 63) / 64 * 64;
        if (l.type == DC_ADD && d.tensors[l.in1].cum_stride != d.tensors[l.in0].cum_stride) return;
        if (l.type == DC_CONCAT) {
            int ids[4];
            const int m = concat_inputs(l, ids);
            for (int j = 1; j < m; ++j)
                if (d.tensors[ids[j]].cum_stride != d.tensors[l.in0].cum_stride) return;
        }
        if (l.type == DC_CONV) d.conv_layer.push_back(i);
    }
    if ((int)d.conv_layer.size() > kPlanMaxConvs) return;
    d.off_tensors = align_up((size_t)n_layers * sizeof(PlanLayerDev), 256);
    d.off_convs = d.off_tensors + align_up((size_t)nt * sizeof(PlanTensorDev), 256);
    d.table_bytes = d.off_convs + align_up(d.conv_layer.size() * sizeof(PlanConvDev), 256);
    size_t off = align_up((size_t)n_streams * nt * d.cap * sizeof(dc_rect), 256);
    d.off_nrect = off; off += align_up((size_t)n_streams * nt * sizeof(int32_t), 256);
    d.off_dxy = off; off += align_up((size_t)n_streams * nt * 2 * sizeof(int32_t), 256);
    d.off_origin = off; off += align_up((size_t)n_streams * nt * 2 * sizeof(int32_t), 256);
    d.off_info = off; off += align_up((size_t)n_streams * 2 * sizeof(int32_t), 256);
    d.off_nunits = off; off += align_up(d.conv_layer.size() * sizeof(int32_t), 256);
    d.off_stats = off; off += kDevHostSlot;
    d.bm_words = bm;
    d.off_bitmaps = off; off += align_up((size_t)n_streams * (size_t)bm * sizeof(uint32_t), 256);
    d.off_area = off;
    size_t area = 0;
    d.max_chunks = 0;
    for (int layer : d.conv_layer) {
        PlanConvDev c{};
        c.tensor = layer + 1; c.Hout = hs[layer + 1]; c.Wout = ws[layer + 1];
        c.no_reuse = no_reuse && no_reuse[layer] ? 1 : 0;
        c.units_x = (c.Wout + 3) / 4; c.units_y = (c.Hout + 3) / 4;
        const size_t units = (size_t)c.units_x * c.units_y;
        c.n_chunks = (int)((units + kPlanChunk - 1) / kPlanChunk);
        d.max_chunks = c.n_chunks > d.max_chunks ? c.n_chunks : d.max_chunks;
        c.umask_off = (int64_t)area; area += align_up((size_t)n_streams * units * sizeof(uint16_t), 256);
        c.count_off = (int64_t)area; area += align_up((size_t)n_streams * c.n_chunks * 2 * sizeof(int32_t), 256);
        c.list_off = (int64_t)area; area += align_up((size_t)n_streams * units * sizeof(TileDev), 256);
        if (units * (size_t)n_streams > 0x7fffffffull) return;
        d.convs.push_back(c);
    }
    d.frame_bytes = align_up(off + area, 256);
    d.ok = true;
}

// ---- scratch of the entry point that allocates nothing ----
// Device memory that belongs to the library for the life of the process (one copy per GPU the library is loaded
// on): the plan of one conv layer (rectangles, unit masks, counts, unit list) and the partial sums of a split K.
constexpr size_t kStaticScratchBytes = (size_t)16 << 20;
constexpr size_t kStaticPlanBytes = (size_t)6 << 20;      // the plan's share; the rest takes partial sums
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
unsigned char* g_scratch_ptr[kMaxDevices] = {};           // device address of `scratch` on each GPU, asked once

// Address of this GPU's copy of the array (the array's name is not an address host code may use).
int static_scratch(unsigned char** ptr) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return DC_ERR_HIP;
    if (dev < 0 || dev >= kMaxDevices) return DC_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> guard(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return DC_ERR_HIP;
        g_scratch_ptr[dev] = static_cast<unsigned char*>(p);
    }
    *ptr = g_scratch_ptr[dev];
    return DC_OK;
}

uint64_t fnv1a(uint64_t h, const void* p, size_t n) {
    const unsigned char* b = static_cast<const unsigned char*>(p);
    for (size_t i = 0; i < n; ++i) { h ^= b[i]; h *= 0x100000001b3ull; }
    return h;
}

}  // namespace

extern "C" {

const char* dc_status_string(int32_t s) {
    switch (s) {
        case DC_OK: return "ok";
        case DC_ERR_INVALID_ARG: return "invalid argument";
        case DC_ERR_NULL_PTR: return "null pointer";
        case DC_ERR_BAD_SHAPE: return "inconsistent shapes";
        case DC_ERR_UNSUPPORTED: return "unsupported configuration";
        case DC_ERR_WORKSPACE: return "workspace too small";
        case DC_ERR_CAPACITY: return "list capacity exceeded";
        case DC_ERR_HIP: return "HIP runtime error";
        default: return "unknown status";
    }
}

int32_t dc_profile_create(int32_t n_slots, void** profile) {
    if (!profile) return DC_ERR_NULL_PTR;
    if (n_slots < 1 || n_slots > (1 << 20)) return DC_ERR_INVALID_ARG;
    Profile* p = new (std::nothrow) Profile();
    if (!p) return DC_ERR_WORKSPACE;
    p->ev.resize(2 * (size_t)n_slots, nullptr);
    p->used.assign(n_slots, 0);
    for (size_t i = 0; i < p->ev.size(); ++i)
        if (hipEventCreate(&p->ev[i]) != hipSuccess) {
            for (size_t j = 0; j < i; ++j) (void)hipEventDestroy(p->ev[j]);
            delete p;
            return DC_ERR_HIP;
        }
    *profile = p;
    return DC_OK;
}

int32_t dc_profile_destroy(void* profile) {
    if (!profile) return DC_ERR_NULL_PTR;
    Profile* p = static_cast<Profile*>(profile);
    for (hipEvent_t e : p->ev) (void)hipEventDestroy(e);
    delete p;
    return DC_OK;
}

int32_t dc_profile_reset(void* profile) {
    if (!profile) return DC_ERR_NULL_PTR;
    Profile* p = static_cast<Profile*>(profile);
    std::fill(p->used.begin(), p->used.end(), 0);
    return DC_OK;
}

int32_t dc_profile_elapsed_ms(void* profile, int32_t slot, float* ms) {
    if (!profile || !ms) return DC_ERR_NULL_PTR;
    Profile* p = static_cast<Profile*>(profile);
    if (slot < 0 || (size_t)slot >= p->used.size() || !p->used[slot]) return DC_ERR_INVALID_ARG;
    DC_TRY_HIP(hipEventElapsedTime(ms, p->ev[2 * slot], p->ev[2 * slot + 1]));
    return DC_OK;
}

int32_t dc_probe_mfma_rate(int32_t lds_reads, void* scratch_dev, size_t scratch_bytes, double* tflops, void* stream) {
    if (!scratch_dev || !tflops) return DC_ERR_NULL_PTR;
    if (scratch_bytes < ((size_t)4 << 20)) return DC_ERR_WORKSPACE;
    if (reinterpret_cast<uintptr_t>(scratch_dev) % 16) return DC_ERR_INVALID_ARG;
    const int wgs = 256, steps = 1024, launches = 30;       // about 0.3 ms per launch
    float ms = 0.f;
    DC_TRY_HIP(probe_mfma_rate(lds_reads != 0, scratch_dev, wgs, steps, launches, &ms, as_stream(stream)));
    if (!(ms > 0.f)) return DC_ERR_HIP;
    *tflops = (double)wgs * 8 * steps * 16 * 16384.0 / (ms * 1e-3) / 1e12;
    return DC_OK;
}

int32_t dc_overlap_create(void** overlap) {
    if (!overlap) return DC_ERR_NULL_PTR;
    Overlap* o = new (std::nothrow) Overlap();
    if (!o) return DC_ERR_WORKSPACE;
    bool ok = hipStreamCreateWithFlags(&o->aux, hipStreamNonBlocking) == hipSuccess;
    for (int i = 0; i < 2 && ok; ++i) ok = hipEventCreateWithFlags(&o->upload_done[i], hipEventDisableTiming) == hipSuccess;
    for (int i = 0; i < 2 && ok; ++i) ok = hipStreamCreateWithFlags(&o->work[i], hipStreamNonBlocking) == hipSuccess;
    for (int i = 0; i < 2 && ok; ++i) ok = hipEventCreateWithFlags(&o->frame_done[i], hipEventDisableTiming) == hipSuccess;
    ok = ok && hipEventCreateWithFlags(&o->match_done, hipEventDisableTiming) == hipSuccess;
    for (int i = 0; i < 3 && ok; ++i) ok = hipEventCreateWithFlags(&o->plan_done[i], hipEventDisableTiming) == hipSuccess;
    for (int i = 0; i < 3 && ok; ++i) ok = hipEventCreateWithFlags(&o->area_free[i], hipEventDisableTiming) == hipSuccess;
    if (!ok) {
        (void)dc_overlap_destroy(o);
        return DC_ERR_HIP;
    }
    *overlap = o;
    return DC_OK;
}

int32_t dc_overlap_destroy(void* overlap) {
    if (!overlap) return DC_ERR_NULL_PTR;
    Overlap* o = static_cast<Overlap*>(overlap);
    if (o->aux) (void)hipStreamSynchronize(o->aux);
    for (int i = 0; i < 2; ++i) {
        if (o->work[i]) (void)hipStreamSynchronize(o->work[i]);
        if (o->upload_done[i]) (void)hipEventDestroy(o->upload_done[i]);
        if (o->frame_done[i]) (void)hipEventDestroy(o->frame_done[i]);
        for (hipEvent_t e : o->layer_done[i]) (void)hipEventDestroy(e);
        if (o->work[i]) (void)hipStreamDestroy(o->work[i]);
    }
    for (int i = 0; i < 3; ++i) {
        if (o->plan_done[i]) (void)hipEventDestroy(o->plan_done[i]);
        if (o->area_free[i]) (void)hipEventDestroy(o->area_free[i]);
    }
    if (o->match_done) (void)hipEventDestroy(o->match_done);
    if (o->aux) (void)hipStreamDestroy(o->aux);
    delete o;
    return DC_OK;
}

int32_t dc_prefetch_match(void* overlap, const uint8_t* frames_next, const uint8_t* frames_cur,
                          int32_t n_streams, int32_t H, int32_t W, int32_t C, int32_t block, int32_t radius,
                          uint32_t max_block_ssd, const dc_match_options* match_options,
                          int16_t* mv, uint32_t* best_ssd, int32_t* global_mv, int32_t* n_pass,
                          uint8_t* block_mask, void* ws_host, size_t ws_host_bytes) {
    if (!overlap || !frames_next || !frames_cur || !global_mv || !block_mask || !ws_host) return DC_ERR_NULL_PTR;
    if (n_streams < 1 || H < 1 || W < 1 || C < 1 || block < 1) return DC_ERR_INVALID_ARG;
    if (block > H || block > W) return DC_ERR_BAD_SHAPE;
    Overlap* ov = static_cast<Overlap*>(overlap);
    const size_t nb = (size_t)n_streams * (H / block) * (W / block);
    if (ws_host_bytes < align_up(nb, 256) + align_up((size_t)n_streams * 3 * sizeof(int32_t), 256)) return DC_ERR_WORKSPACE;
    if (ov->prefetch.valid) {     // an unused look-ahead is dropped once its kernels are out of the way
        DC_TRY_HIP(hipStreamSynchronize(ov->aux));
        ov->prefetch.valid = false;
    }
    int rc = dc_match_blocks_opt(frames_next, frames_cur, n_streams, H, W, C, block, radius, match_options, max_block_ssd,
                                 mv, best_ssd, global_mv, n_pass, block_mask, ov->aux);
    if (rc) return rc;
    unsigned char* hbase = static_cast<unsigned char*>(ws_host);
    DC_TRY_HIP(hipMemcpyAsync(hbase, block_mask, nb, hipMemcpyDeviceToHost, ov->aux));
    DC_TRY_HIP(hipMemcpyAsync(hbase + align_up(nb, 256), global_mv, (size_t)n_streams * 2 * sizeof(int32_t),
                              hipMemcpyDeviceToHost, ov->aux));
    DC_TRY_HIP(hipEventRecord(ov->match_done, ov->aux));
    Overlap::Prefetch& pf = ov->prefetch;
    pf.cur = frames_next; pf.prev = frames_cur; pf.mv = mv; pf.best_ssd = best_ssd; pf.gmv = global_mv; pf.n_pass = n_pass;
    pf.mask = block_mask; pf.ws_host = ws_host; pf.n_streams = n_streams; pf.H = H; pf.W = W; pf.C = C; pf.block = block;
    pf.radius = radius; pf.max_block_ssd = max_block_ssd;
    pf.method = match_options ? match_options->method : DC_MATCH_EXHAUSTIVE;
    pf.k_skip = match_options ? match_options->k_skip : 1;
    pf.valid = true;
    return DC_OK;
}

int32_t dc_overlap_pipeline(void* overlap, int32_t frames_in_flight) {
    if (!overlap) return DC_ERR_NULL_PTR;
    if (frames_in_flight < 1 || frames_in_flight > 2) return DC_ERR_INVALID_ARG;
    Overlap* o = static_cast<Overlap*>(overlap);
    for (int i = 0; i < 2; ++i) {
        DC_TRY_HIP(hipStreamSynchronize(o->work[i]));
        o->recorded[i].clear();
        o->last_cur[i].clear();
        o->frame_recorded[i] = false;
    }
    if (o->aux) DC_TRY_HIP(hipStreamSynchronize(o->aux));
    for (int i = 0; i < 3; ++i) o->area_recorded[i] = false;
    o->pipeline = frames_in_flight == 2;
    return DC_OK;
}

int32_t dc_conv_tuning(int32_t arrangement, int32_t units_per_workgroup, int32_t k_split, int32_t chunk_index) {
    if (arrangement > 4 || units_per_workgroup > 18 || chunk_index > 1) return DC_ERR_INVALID_ARG;
    conv_set_tuning(arrangement, units_per_workgroup, k_split, chunk_index);
    return DC_OK;
}

int32_t dc_conv_kernel_name(int32_t kernel_id, char* buf, size_t n) {
    if (!buf) return DC_ERR_NULL_PTR;
    if (n < 2 || kernel_id < 0 || kernel_id > 130) return DC_ERR_INVALID_ARG;
    conv_kernel_name(kernel_id, buf, n);
    return DC_OK;
}

int32_t dc_conv_tile_shape(const dc_layer* layer, int32_t n_streams, int32_t Hin, int32_t Win, int32_t dtype,
                           int32_t* th, int32_t* tw, int32_t* nt, int32_t* cfg) {
    if (!layer || !th || !tw || !nt || !cfg) return DC_ERR_NULL_PTR;
    int rc = check_conv_layer(layer);
    if (rc) return rc;
    if (n_streams < 1 || Hin < 1 || Win < 1) return DC_ERR_INVALID_ARG;
    const WindowGeom lg = window_geom(*layer);
    if (Hin + 2 * lg.ph < lg.eh || Win + 2 * lg.pw < lg.ew) return DC_ERR_BAD_SHAPE;
    const int Hout = (Hin + 2 * lg.ph - lg.eh) / layer->s + 1, Wout = (Win + 2 * lg.pw - lg.ew) / layer->s + 1;
    ConvTiling t = pick_tiling(*layer, Hout, Wout, n_streams, dtype);
    *th = t.th; *tw = t.tw; *nt = t.nt; *cfg = t.cfg;
    return DC_OK;
}

static int match_exhaustive(const uint8_t* cur, const uint8_t* prev, int32_t n_streams, int32_t H, int32_t W, int32_t C,
                     int32_t block, int32_t radius, int32_t k_skip, uint32_t max_block_ssd, int16_t* mv,
                     uint32_t* best_ssd, int32_t* global_mv, int32_t* n_pass, uint8_t* block_mask, void* stream) {
    if (!cur || !prev || !mv || !best_ssd || !global_mv || !n_pass || !block_mask) return DC_ERR_NULL_PTR;
    if (n_streams < 1 || n_streams > 65535 || H < 1 || W < 1 || C < 1 || block < 1 || radius < 0 || k_skip < 1)
        return DC_ERR_INVALID_ARG;
    if (block > H || block > W) return DC_ERR_BAD_SHAPE;
    if (radius > 127 || block * C > 256) return DC_ERR_UNSUPPORTED;
    const long rows = block + 2 * radius;
    if (rows * (rows * C + 16) > 60 * 1024) return DC_ERR_UNSUPPORTED;
    // 32-bit sums: B*B*C*255^2 must fit
    if ((double)block * block * C * 65025.0 * 2.0 > 4.0e9) return DC_ERR_UNSUPPORTED;
    DC_TRY_HIP(launch_match(cur, prev, n_streams, H, W, C, block, radius, k_skip, max_block_ssd, mv, best_ssd, global_mv,
                            n_pass, block_mask, as_stream(stream)));
    return DC_OK;
}

int32_t dc_match_blocks(const uint8_t* cur, const uint8_t* prev, int32_t n_streams, int32_t H, int32_t W,
                        int32_t C, int32_t block, int32_t radius, uint32_t max_block_ssd, int16_t* mv,
                        uint32_t* best_ssd, int32_t* global_mv, int32_t* n_pass, uint8_t* block_mask,
                        void* stream) {
    return match_exhaustive(cur, prev, n_streams, H, W, C, block, radius, 1, max_block_ssd, mv, best_ssd, global_mv,
                            n_pass, block_mask, stream);
}

int32_t dc_match_blocks_opt(const uint8_t* cur, const uint8_t* prev, int32_t n_streams, int32_t H, int32_t W,
                            int32_t C, int32_t block, int32_t radius, const dc_match_options* options,
                            uint32_t max_block_ssd, int16_t* mv, uint32_t* best_ssd, int32_t* global_mv,
                            int32_t* n_pass, uint8_t* block_mask, void* stream) {
    const int method = options ? options->method : DC_MATCH_EXHAUSTIVE, k = options ? options->k_skip : 1;
    if (method == DC_MATCH_DIAMOND)
        return dc_match_blocks_ds(cur, prev, n_streams, H, W, C, block, radius, k, max_block_ssd, mv, best_ssd, global_mv,
                                  n_pass, block_mask, stream);
    if (method != DC_MATCH_EXHAUSTIVE) return DC_ERR_INVALID_ARG;
    return match_exhaustive(cur, prev, n_streams, H, W, C, block, radius, k, max_block_ssd, mv, best_ssd, global_mv,
                            n_pass, block_mask, stream);
}

int32_t dc_match_blocks_ds(const uint8_t* cur, const uint8_t* prev, int32_t n_streams, int32_t H, int32_t W,
                           int32_t C, int32_t block, int32_t radius, int32_t k_skip, uint32_t max_block_ssd,
                           int16_t* mv, uint32_t* best_ssd, int32_t* global_mv, int32_t* n_pass, uint8_t* block_mask,
                           void* stream) {
    if (!cur || !prev || !mv || !best_ssd || !global_mv || !n_pass || !block_mask) return DC_ERR_NULL_PTR;
    if (n_streams < 1 || n_streams > 65535 || H < 1 || W < 1 || C < 1 || block < 1 || radius < 0 || k_skip < 1)
        return DC_ERR_INVALID_ARG;
    if (block > H || block > W) return DC_ERR_BAD_SHAPE;
    if (radius > 16383) return DC_ERR_UNSUPPORTED;                                   // vectors are int16
    if ((double)block * block * C * 65025.0 * 2.0 > 4.0e9) return DC_ERR_UNSUPPORTED;   // 32-bit sums
    if ((double)block * W * C >= 2147483648.0) return DC_ERR_UNSUPPORTED;             // 32-bit offsets inside a block
    if ((double)block * block * block * C * C >= 4294967296.0) return DC_ERR_UNSUPPORTED;   // row index by multiplication
    DC_TRY_HIP(launch_match_diamond(cur, prev, n_streams, H, W, C, block, radius, k_skip, max_block_ssd, mv, best_ssd,
                                    global_mv, n_pass, block_mask, as_stream(stream)));
    return DC_OK;
}

int32_t dc_propagate_regions(const dc_layer* layers, int32_t n_layers, int32_t H, int32_t W, int32_t block,
                             const uint8_t* block_mask, int32_t gh, int32_t gw, int32_t mx, int32_t my,
                             dc_regions* regions) {
    return dc_propagate_regions_opt(layers, n_layers, H, W, block, block_mask, gh, gw, mx, my, 0, regions);
}

int32_t dc_propagate_regions_opt(const dc_layer* layers, int32_t n_layers, int32_t H, int32_t W, int32_t block,
                                 const uint8_t* block_mask, int32_t gh, int32_t gw, int32_t mx, int32_t my,
                                 int32_t extend_borders, dc_regions* regions) {
    if (!layers || !block_mask || !regions) return DC_ERR_NULL_PTR;
    if (n_layers < 0 || H < 1 || W < 1 || block < 1 || gh < 0 || gw < 0) return DC_ERR_INVALID_ARG;
    if (gh != H / block || gw != W / block) return DC_ERR_BAD_SHAPE;
    int rc = validate_layers(layers, n_layers, H, W, n_layers ? layers[0].cin : 1, nullptr, nullptr, nullptr);
    if (rc != DC_OK) return rc;
    for (int t = 0; t <= n_layers; ++t)
        if (regions[t].capacity < 0 || (regions[t].capacity > 0 && !regions[t].rects)) return DC_ERR_NULL_PTR;
    std::vector<dc_rect> rects0;
    std::vector<TensorRegions> out;
    try {
        merge_blocks(block_mask, gh, gw, block, rects0);
        rc = propagate(layers, n_layers, H, W, rects0, mx, my, out, extend_borders != 0);
    } catch (const std::bad_alloc&) {
        return DC_ERR_WORKSPACE;
    }
    if (rc != DC_OK) return rc;
    int status = DC_OK;
    for (int t = 0; t <= n_layers; ++t) {
        dc_regions& r = regions[t];
        r.n = (int)out[t].rects.size();
        r.dx = out[t].dx; r.dy = out[t].dy; r.cum_stride = out[t].cum_stride; r.h = out[t].h; r.w = out[t].w;
        int keep = r.n < r.capacity ? r.n : r.capacity;
        if (keep) std::memcpy(r.rects, out[t].rects.data(), keep * sizeof(dc_rect));
        if (r.n > r.capacity) status = DC_ERR_CAPACITY;
    }
    return status;
}

int32_t dc_conv_workspace_bytes(const dc_layer* layer, int32_t n_streams, int32_t Hin, int32_t Win,
                                int32_t max_rects, size_t* dev_bytes, size_t* host_bytes) {
    if (!layer || !dev_bytes || !host_bytes) return DC_ERR_NULL_PTR;
    int rc = check_conv_layer(layer);
    if (rc) return rc;
    if (n_streams < 1 || Hin < 1 || Win < 1 || max_rects < 0) return DC_ERR_INVALID_ARG;
    const WindowGeom lg = window_geom(*layer);
    if (Hin + 2 * lg.ph < lg.eh || Win + 2 * lg.pw < lg.ew) return DC_ERR_BAD_SHAPE;
    const int Hout = (Hin + 2 * lg.ph - lg.eh) / layer->s + 1, Wout = (Win + 2 * lg.pw - lg.ew) / layer->s + 1;
    size_t worst = 0;
    for (int dtype = 0; dtype < 2; ++dtype) {
        size_t b = plan_bytes(n_streams, Hout, Wout, pick_tiling(*layer, Hout, Wout, n_streams, dtype), max_rects);
        worst = b > worst ? b : worst;
    }
    *dev_bytes = align_up(worst, 256) + kConvScratchBytes;   // plan + room for partial sums of a split K
    *host_bytes = worst;
    return DC_OK;
}

int32_t dc_packed_weights_bytes(const dc_layer* layer, int32_t dtype, size_t* bytes) {
    if (!layer || !bytes) return DC_ERR_NULL_PTR;
    if (dtype != DC_F32 && dtype != DC_BF16) return DC_ERR_INVALID_ARG;
    int rc = check_conv_layer(layer);
    if (rc) return rc;
    *bytes = plain_square(*layer) ? packed_weights_bytes(layer->k, layer->s, layer->cin, layer->cout, dtype) : 0;
    return DC_OK;
}

int32_t dc_pack_conv_weights(const dc_layer* layer, const void* weights, int32_t dtype, void* packed, void* stream) {
    if (!layer || !weights || !packed) return DC_ERR_NULL_PTR;
    if (dtype != DC_F32 && dtype != DC_BF16) return DC_ERR_INVALID_ARG;
    int rc = check_conv_layer(layer);
    if (rc) return rc;
    if (!plain_square(*layer) || !packed_weights_bytes(layer->k, layer->s, layer->cin, layer->cout, dtype)) return DC_ERR_BAD_SHAPE;
    if (reinterpret_cast<uintptr_t>(weights) % 16 || reinterpret_cast<uintptr_t>(packed) % 16 || weights == packed)
        return DC_ERR_INVALID_ARG;
    DC_TRY_HIP(launch_pack_weights(weights, packed, layer->cin, layer->cout, dtype, as_stream(stream)));
    return DC_OK;
}

int32_t dc_cached_conv_layer(const dc_layer* layer, const void* in, const void* weights, const void* packed_weights,
                             const float* bias, const void* cache_prev, void* out, int32_t n_streams, int32_t Hin, int32_t Win,
                             const dc_regions* regions, int32_t dtype, void* ws_dev, size_t ws_dev_bytes,
                             void* ws_host, size_t ws_host_bytes, void* stream) {
    if (!layer || !in || !weights || !out) return DC_ERR_NULL_PTR;
    int rc = check_conv_layer(layer);
    if (rc) return rc;
    if (dtype != DC_F32 && dtype != DC_BF16) return DC_ERR_INVALID_ARG;
    if (n_streams < 1 || Hin < 1 || Win < 1) return DC_ERR_INVALID_ARG;
    const WindowGeom lg = window_geom(*layer);
    if (Hin + 2 * lg.ph < lg.eh || Win + 2 * lg.pw < lg.ew) return DC_ERR_BAD_SHAPE;
    const int Hout = (Hin + 2 * lg.ph - lg.eh) / layer->s + 1, Wout = (Win + 2 * lg.pw - lg.ew) / layer->s + 1;
    const ConvTiling tiling = pick_tiling(*layer, Hout, Wout, n_streams, dtype);
    hipStream_t st = as_stream(stream);
    if (!regions || !cache_prev)
        return run_conv_planned(*layer, in, weights, bias, nullptr, out, n_streams, Hin, Win, dtype, tiling, nullptr,
                                nullptr, st, nullptr, -1, -1, nullptr, false, ws_dev, ws_dev ? ws_dev_bytes : 0, packed_weights);
    if (out == cache_prev) return DC_ERR_INVALID_ARG;
    int max_rects = 0;
    for (int s = 0; s < n_streams; ++s) {
        if (regions[s].n < 0 || (regions[s].n > 0 && !regions[s].rects)) return DC_ERR_NULL_PTR;
        if (!rects_disjoint_inside(regions[s].rects, regions[s].n, Wout, Hout, regions[s].dx, regions[s].dy))
            return DC_ERR_BAD_SHAPE;
        max_rects = regions[s].n > max_rects ? regions[s].n : max_rects;
    }
    size_t need = plan_bytes(n_streams, Hout, Wout, tiling, max_rects);
    if (!ws_dev || !ws_host) return DC_ERR_NULL_PTR;
    if (ws_dev_bytes < need || ws_host_bytes < need) return DC_ERR_WORKSPACE;
    LayerPlan plan;
    try {
        for (int s = 0; s < n_streams; ++s)
            plan_stream(regions[s].rects, regions[s].n, regions[s].dx, regions[s].dy, s, Hout, Wout, tiling.th,
                        tiling.tw, plan);
    } catch (const std::bad_alloc&) {
        return DC_ERR_WORKSPACE;
    }
    plan.n_tiles = plan.tiles.size();
    PlanAddr addr = pack_plan(plan, static_cast<unsigned char*>(ws_host), static_cast<unsigned char*>(ws_dev));
    DC_TRY_HIP(hipMemcpyAsync(ws_dev, ws_host, addr.bytes, hipMemcpyHostToDevice, st));
    // whatever the workspace holds beyond the plan serves as scratch for partial sums
    const size_t plan_end = align_up(addr.bytes, 256);
    unsigned char* scratch = plan_end < ws_dev_bytes ? static_cast<unsigned char*>(ws_dev) + plan_end : nullptr;
    return run_conv_planned(*layer, in, weights, bias, cache_prev, out, n_streams, Hin, Win, dtype, tiling, &plan,
                            &addr, st, nullptr, -1, -1, nullptr, false, scratch, scratch ? ws_dev_bytes - plan_end : 0,
                            packed_weights);
}

int32_t dc_cached_conv_layer_noalloc(const dc_layer* layer, const void* in, const void* weights, const void* packed_weights,
                                     const float* bias, const void* cache_prev, void* out, int32_t n_streams, int32_t Hin,
                                     int32_t Win, const dc_regions* regions, int32_t dtype, void* stream) {
    if (!layer || !in || !weights || !out) return DC_ERR_NULL_PTR;
    int rc = check_conv_layer(layer);
    if (rc) return rc;
    if (dtype != DC_F32 && dtype != DC_BF16) return DC_ERR_INVALID_ARG;
    if (n_streams < 1 || Hin < 1 || Win < 1) return DC_ERR_INVALID_ARG;
    const WindowGeom lg = window_geom(*layer);
    if (Hin + 2 * lg.ph < lg.eh || Win + 2 * lg.pw < lg.ew) return DC_ERR_BAD_SHAPE;
    const int Hout = (Hin + 2 * lg.ph - lg.eh) / layer->s + 1, Wout = (Win + 2 * lg.pw - lg.ew) / layer->s + 1;
    const ConvTiling tiling = pick_tiling(*layer, Hout, Wout, n_streams, dtype);
    hipStream_t st = as_stream(stream);
    const bool cached = regions && cache_prev;
    if (cached && out == cache_prev) return DC_ERR_INVALID_ARG;
    // sizes first: the plan of the layer must fit the library's scratch, the rectangles the kernel arguments
    PlanConvDev cv{};
    cv.tensor = 0; cv.Hout = Hout; cv.Wout = Wout; cv.units_x = (Wout + 3) / 4; cv.units_y = (Hout + 3) / 4;
    const size_t units = (size_t)cv.units_x * cv.units_y;
    cv.n_chunks = (int)((units + kPlanChunk - 1) / kPlanChunk);
    PlanArgRects args{};
    int cap = 1;
    size_t off = 0;
    size_t off_rects = 0, off_nrect = 0, off_dxy = 0, off_info = 0, off_nunits = 0, off_stats = 0, off_convs = 0;
    if (cached) {
        if (n_streams > kArgMaxStreams) return DC_ERR_CAPACITY;
        int total = 0;
        for (int s = 0; s < n_streams; ++s) {
            if (regions[s].n < 0 || (regions[s].n > 0 && !regions[s].rects)) return DC_ERR_NULL_PTR;
            if (!rects_disjoint_inside(regions[s].rects, regions[s].n, Wout, Hout, regions[s].dx, regions[s].dy))
                return DC_ERR_BAD_SHAPE;
            if (total + regions[s].n > kArgMaxRects) return DC_ERR_CAPACITY;
            args.first[s] = total;
            for (int j = 0; j < regions[s].n; ++j) args.r[total + j] = regions[s].rects[j];
            total += regions[s].n;
            args.dxy[s][0] = regions[s].dx; args.dxy[s][1] = regions[s].dy;
            cap = regions[s].n > cap ? regions[s].n : cap;
        }
        for (int s = n_streams; s <= kArgMaxStreams; ++s) args.first[s] = total;
        off_rects = off; off += align_up((size_t)n_streams * cap * sizeof(dc_rect), 256);
        off_nrect = off; off += align_up((size_t)n_streams * sizeof(int32_t), 256);
        off_dxy = off; off += align_up((size_t)n_streams * 2 * sizeof(int32_t), 256);
        off_info = off; off += align_up((size_t)n_streams * 2 * sizeof(int32_t), 256);
        off_nunits = off; off += 256;
        off_stats = off; off += 256;
        off_convs = off; off += 256;
        cv.umask_off = (int64_t)off; off += align_up((size_t)n_streams * units * sizeof(uint16_t), 256);
        cv.count_off = (int64_t)off; off += align_up((size_t)n_streams * cv.n_chunks * 2 * sizeof(int32_t), 256);
        cv.list_off = (int64_t)off; off += align_up((size_t)n_streams * units * sizeof(TileDev), 256);
        if (off > kStaticPlanBytes || (size_t)n_streams * units > 0x7fffffffull) return DC_ERR_WORKSPACE;
    }
    unsigned char* base = nullptr;
    rc = static_scratch(&base);
    if (rc) return rc;
    unsigned char* const partial = base + kStaticPlanBytes;
    const size_t partial_bytes = kStaticScratchBytes - kStaticPlanBytes;
    if (!cached)
        return run_conv_planned(*layer, in, weights, bias, nullptr, out, n_streams, Hin, Win, dtype, tiling, nullptr, nullptr,
                                st, nullptr, -1, -1, nullptr, false, partial, partial_bytes, packed_weights);
    PlanDev pd{};
    pd.layers = nullptr; pd.tensors = nullptr;
    pd.convs = reinterpret_cast<const PlanConvDev*>(base + off_convs);
    pd.n_layers = 0; pd.n_convs = 1; pd.n_streams = n_streams; pd.cap = cap;
    pd.rects = reinterpret_cast<dc_rect*>(base + off_rects);
    pd.nrect = reinterpret_cast<int32_t*>(base + off_nrect);
    pd.dxy = reinterpret_cast<int32_t*>(base + off_dxy);
    pd.stream_info = reinterpret_cast<int32_t*>(base + off_info);
    pd.n_units = reinterpret_cast<int32_t*>(base + off_nunits);
    pd.stats = base + off_stats;
    pd.area = base;
    DC_TRY_HIP(launch_plan_from_args(pd, cv, args, st));
    const size_t px_bytes = (size_t)layer->cout * dtype_size(dtype);
    const bool vec16 = px_bytes % 16 == 0 && reinterpret_cast<uintptr_t>(cache_prev) % 16 == 0 && reinterpret_cast<uintptr_t>(out) % 16 == 0;
    const int vb = vec16 ? 16 : (int)dtype_size(dtype);
    const CopyUnitsLayer cl{cache_prev, out, reinterpret_cast<const uint16_t*>(base + cv.umask_off), 0, Hout, Wout,
                            cv.units_x, cv.units_y, (int32_t)(px_bytes / vb), 0, 0};
    DC_TRY_HIP(launch_shifted_copy_units(&cl, 1, pd.dxy, 1, n_streams, vb, st));
    return run_conv_planned(*layer, in, weights, bias, cache_prev, out, n_streams, Hin, Win, dtype, tiling, nullptr, nullptr, st,
                            nullptr, -1, -1, nullptr, true, partial, partial_bytes, packed_weights,
                            reinterpret_cast<const TileDev*>(base + cv.list_off), (int)((size_t)n_streams * units), pd.n_units, -1);
}

int32_t dc_frame_to_tensor(const uint8_t* frames, void* out, size_t n_pixels, int32_t c_frame, int32_t c_tensor,
                           int32_t dtype, void* stream) {
    if (!frames || !out) return DC_ERR_NULL_PTR;
    if (dtype != DC_F32 && dtype != DC_BF16) return DC_ERR_INVALID_ARG;
    if (c_frame < 1 || c_tensor < c_frame) return DC_ERR_INVALID_ARG;
    DC_TRY_HIP(launch_frame_to_tensor(frames, out, n_pixels, c_frame, c_tensor, dtype, as_stream(stream)));
    return DC_OK;
}

int32_t dc_maxpool_layer(const void* in, void* out, int32_t n_streams, int32_t Hin, int32_t Win, int32_t C,
                         int32_t k, int32_t s, int32_t p, int32_t dtype, void* stream) {
    if (!in || !out) return DC_ERR_NULL_PTR;
    if (dtype != DC_F32 && dtype != DC_BF16) return DC_ERR_INVALID_ARG;
    if (n_streams < 1 || Hin < 1 || Win < 1 || C < 1 || k < 1 || s < 1 || p < 0 || p >= k) return DC_ERR_INVALID_ARG;
    if (Hin + 2 * p < k || Win + 2 * p < k) return DC_ERR_BAD_SHAPE;
    DC_TRY_HIP(launch_maxpool(in, out, n_streams, Hin, Win, C, k, s, p, dtype, as_stream(stream)));
    return DC_OK;
}

int32_t dc_torus_read(const void* in, void* out, const int32_t* origins_dev, int32_t origin_stride, int32_t n_streams,
                      int32_t H, int32_t W, int32_t C, int32_t dtype, void* stream) {
    if (!in || !out) return DC_ERR_NULL_PTR;
    if (in == out) return DC_ERR_INVALID_ARG;
    if (dtype != DC_F32 && dtype != DC_BF16) return DC_ERR_INVALID_ARG;
    if (n_streams < 1 || H < 1 || W < 1 || C < 1 || (origins_dev && origin_stride < 2)) return DC_ERR_INVALID_ARG;
    if ((size_t)n_streams * H > 65535) return DC_ERR_UNSUPPORTED;
    DC_TRY_HIP(launch_torus_read(in, out, n_streams, H, W, (size_t)C * dtype_size(dtype), origins_dev, origin_stride, as_stream(stream)));
    return DC_OK;
}

int32_t dc_add_layer(const void* a, const void* b, void* out, size_t n, int32_t relu, int32_t dtype, void* stream) {
    if (!a || !b || !out) return DC_ERR_NULL_PTR;
    if (dtype != DC_F32 && dtype != DC_BF16) return DC_ERR_INVALID_ARG;
    DC_TRY_HIP(launch_add(a, b, out, n, relu, dtype, as_stream(stream)));
    return DC_OK;
}

int32_t dc_avgpool_layer(const void* in, void* out, int32_t n_streams, int32_t Hin, int32_t Win, int32_t C,
                         int32_t k, int32_t s, int32_t p, int32_t dtype, void* stream) {
    if (!in || !out) return DC_ERR_NULL_PTR;
    if (dtype != DC_F32 && dtype != DC_BF16) return DC_ERR_INVALID_ARG;
    if (n_streams < 1 || Hin < 1 || Win < 1 || C < 1 || k < 1 || s < 1 || p < 0 || p >= k) return DC_ERR_INVALID_ARG;
    if (Hin + 2 * p < k || Win + 2 * p < k) return DC_ERR_BAD_SHAPE;
    DC_TRY_HIP(launch_avgpool(in, out, n_streams, Hin, Win, C, k, s, p, dtype, as_stream(stream)));
    return DC_OK;
}

int32_t dc_lrn_layer(const void* in, void* out, int32_t n_streams, int32_t H, int32_t W, int32_t C, int32_t size,
                     int32_t within, float alpha, float beta, float kappa, int32_t dtype, void* stream) {
    if (!in || !out) return DC_ERR_NULL_PTR;
    if (dtype != DC_F32 && dtype != DC_BF16) return DC_ERR_INVALID_ARG;
    if (n_streams < 1 || H < 1 || W < 1 || C < 1 || size < 1 || size % 2 == 0) return DC_ERR_INVALID_ARG;
    DC_TRY_HIP(launch_lrn(in, out, n_streams, H, W, C, size, within != 0, alpha, beta, kappa, dtype, as_stream(stream)));
    return DC_OK;
}

int32_t dc_concat_layer(const void* const* ins, const int32_t* channels, int32_t n_in, void* out, size_t n_pixels,
                        int32_t dtype, void* stream) {
    if (!ins || !channels || !out) return DC_ERR_NULL_PTR;
    if (dtype != DC_F32 && dtype != DC_BF16) return DC_ERR_INVALID_ARG;
    if (n_in < 2 || n_in > 4) return DC_ERR_INVALID_ARG;
    int chans[4];
    for (int j = 0; j < n_in; ++j) {
        if (!ins[j]) return DC_ERR_NULL_PTR;
        if (channels[j] < 1) return DC_ERR_INVALID_ARG;
        if (ins[j] == out) return DC_ERR_INVALID_ARG;
        chans[j] = channels[j];
    }
    DC_TRY_HIP(launch_concat(ins, chans, n_in, out, n_pixels, dtype, as_stream(stream)));
    return DC_OK;
}

int32_t dc_fc_layer(const void* in, const void* weights, const float* bias, void* out, int32_t n_streams, size_t K,
                    int32_t cout, int32_t relu, int32_t dtype, void* stream) {
    if (!in || !weights || !out) return DC_ERR_NULL_PTR;
    if (dtype != DC_F32 && dtype != DC_BF16) return DC_ERR_INVALID_ARG;
    if (n_streams < 1 || K < 1 || cout < 1) return DC_ERR_INVALID_ARG;
    DC_TRY_HIP(launch_fc(in, weights, bias, out, n_streams, K, cout, relu, dtype, as_stream(stream)));
    return DC_OK;
}

int32_t dc_softmax_layer(const void* in, void* out, size_t n_pixels, int32_t C, int32_t dtype, void* stream) {
    if (!in || !out) return DC_ERR_NULL_PTR;
    if (dtype != DC_F32 && dtype != DC_BF16) return DC_ERR_INVALID_ARG;
    if (C < 1) return DC_ERR_INVALID_ARG;
    DC_TRY_HIP(launch_softmax(in, out, n_pixels, C, dtype, as_stream(stream)));
    return DC_OK;
}

int32_t dc_stack_workspace_bytes(const dc_layer* layers, int32_t n_layers, int32_t n_streams, int32_t H, int32_t W,
                                 int32_t C, int32_t block, int32_t max_rects, size_t* dev_bytes, size_t* host_bytes) {
    if (!layers || !dev_bytes || !host_bytes) return DC_ERR_NULL_PTR;
    if (n_layers < 1 || n_streams < 1 || block < 1 || max_rects < 1) return DC_ERR_INVALID_ARG;
    std::vector<int> hs, ws, cs;
    const int c_tensor = input_channels(layers, n_layers, C);
    if (c_tensor < C) return DC_ERR_BAD_SHAPE;
    int rc = validate_layers(layers, n_layers, H, W, c_tensor, &hs, &ws, &cs);
    if (rc) return rc;
    size_t total = 0;
    for (int i = 0; i < n_layers; ++i) {
        if (layers[i].type != DC_CONV) continue;
        size_t worst = 0;
        for (int dtype = 0; dtype < 2; ++dtype) {
            size_t b = plan_bytes(n_streams, hs[i + 1], ws[i + 1],
                                  pick_tiling(layers[i], hs[i + 1], ws[i + 1], n_streams, dtype), max_rects);
            worst = b > worst ? b : worst;
        }
        total += worst;
        total += align_up((size_t)n_streams * max_rects * sizeof(RectDev), 256);   // all-layers copy table
    }
    total += align_up((size_t)n_layers * sizeof(CopyLayerDev), 256);
    const size_t nb = (size_t)n_streams * (H / block) * (W / block);
    size_t match_host = align_up(nb, 256) + align_up((size_t)n_streams * 3 * sizeof(int32_t), 256);
    size_t plans = 2 * align_up(total, 256);       // two frames in flight: a set of plans for each
    try {                                           // planning on the GPU lays the same area out differently
        DevPlanLayout dl;
        device_plan_layout(layers, n_layers, hs, ws, n_streams, max_rects, dl);
        if (dl.ok && 3 * (align_up(dl.table_bytes, 256) + dl.frame_bytes) > plans) plans = 3 * (align_up(dl.table_bytes, 256) + dl.frame_bytes);
    } catch (const std::bad_alloc&) {
        return DC_ERR_WORKSPACE;
    }
    *dev_bytes = plans + 2 * kConvScratchBytes;     // and K-split scratch for each
    // two staging halves (used alternately with an overlap handle); the tail serves the planning on the GPU
    *host_bytes = align_up(2 * total + match_host, 256) + kDevHostRegion;
    return DC_OK;
}

namespace {
// Planning of one frame for dc_run_stack: per (stream, conv layer) lists built in parallel, merged by offset.
struct FramePlan {
    std::vector<int> conv_layers;          // layer indices
    std::vector<LayerPlan> part;           // [stream][conv layer], storage kept between frames
    std::vector<size_t> tile_off;          // [stream][conv layer]: first tile of the part in the layer's list
    std::vector<unsigned char*> tile_dst;  // [conv layer]: the layer's tile list in the staging buffer
    int n_streams = 0;

    // no_reuse (optional): conv layers that are computed in full (planned as if their lists were empty)
    int classify(const dc_layer* layers, int n_layers, int streams, const std::vector<std::vector<TensorRegions>>& regs,
                 const std::vector<int>& hs, const std::vector<int>& ws, const uint8_t* no_reuse) {
        n_streams = streams;
        conv_layers.clear();
        for (int i = 0; i < n_layers; ++i)
            if (layers[i].type == DC_CONV) conv_layers.push_back(i);
        const int nc = (int)conv_layers.size();
        std::vector<int> ok(streams, 1);
        try {
            if (part.size() < (size_t)streams * nc) part.resize((size_t)streams * nc);
            tile_off.assign((size_t)streams * nc, 0);
            tile_dst.assign(nc, nullptr);
        } catch (const std::bad_alloc&) {
            return DC_ERR_WORKSPACE;
        }
        parallel_for(streams, [&](int s) {
            try {
                for (int c = 0; c < nc; ++c) {
                    const int i = conv_layers[c];
                    LayerPlan& lp = part[(size_t)s * nc + c];
                    lp.rects.clear(); lp.ranges.clear(); lp.tiles.clear(); lp.reused_px = 0;
                    const TensorRegions& g = regs[s][i + 1];
                    plan_stream(g.rects.data(), (no_reuse && no_reuse[i]) ? 0 : (int)g.rects.size(), g.dx, g.dy, s, hs[i + 1], ws[i + 1], 4, 4, lp);
                }
            } catch (const std::bad_alloc&) {
                ok[s] = 0;
            }
        });
        for (int s = 0; s < streams; ++s)
            if (!ok[s]) return DC_ERR_WORKSPACE;
        return DC_OK;
    }
    // Lays layer i out in the staging buffer ([tiles][rects][ranges], as pack_plan), fills the small tables and
    // notes where each stream's tiles go.
    PlanAddr finish_layer(int layer, LayerPlan& plan, unsigned char* host, unsigned char* dev) {
        const int nc = (int)conv_layers.size();
        int c = 0;
        while (conv_layers[c] != layer) ++c;
        size_t n_tiles = 0;
        for (int s = 0; s < n_streams; ++s) {
            LayerPlan& lp = part[(size_t)s * nc + c];
            tile_off[(size_t)s * nc + c] = n_tiles;
            n_tiles += lp.tiles.size();
            RangeDev r{(int)plan.rects.size(), (int)lp.rects.size()};
            plan.rects.insert(plan.rects.end(), lp.rects.begin(), lp.rects.end());
            plan.ranges.push_back(r);
            plan.reused_px += lp.reused_px;
        }
        plan.n_tiles = n_tiles;
        tile_dst[c] = host;
        PlanAddr a = pack_plan(plan, host, dev);        // plan.tiles is empty: copies rects and ranges, sizes from n_tiles
        return a;
    }
    void copy_tiles() {
        const int nc = (int)conv_layers.size();
        parallel_for(n_streams, [&](int s) {
            for (int c = 0; c < nc; ++c) {
                const LayerPlan& lp = part[(size_t)s * nc + c];
                if (!lp.tiles.empty())
                    std::memcpy(tile_dst[c] + tile_off[(size_t)s * nc + c] * sizeof(TileDev), lp.tiles.data(),
                                lp.tiles.size() * sizeof(TileDev));
            }
        });
    }
};
FramePlan g_frame_plan;
std::mutex g_frame_plan_mutex;

}  // namespace

int32_t dc_run_stack(const dc_layer* layers, int32_t n_layers, const void* const* weights,
                     const void* const* packed_weights, const float* const* bias,
                     const uint8_t* frames_cur, const uint8_t* frames_prev, void* const* tensors_cur,
                     void* const* tensors_prev, int32_t n_streams, int32_t H, int32_t W, int32_t C,
                     int32_t dtype, int32_t block, int32_t radius, uint32_t max_block_ssd,
                     const dc_match_options* match_options, int32_t force_full, int32_t* in_place,
                     int16_t* mv, uint32_t* best_ssd, int32_t* global_mv, int32_t* n_pass, uint8_t* block_mask,
                     int32_t max_rects, dc_regions* regions_out, void* ws_dev, size_t ws_dev_bytes, void* ws_host,
                     size_t ws_host_bytes, dc_stack_stats* stats, void* overlap, void* stream) {
    if (!layers || !weights || !frames_cur || !tensors_cur) return DC_ERR_NULL_PTR;
    if (dtype != DC_F32 && dtype != DC_BF16) return DC_ERR_INVALID_ARG;
    if (n_layers < 1 || n_streams < 1 || n_streams > 65535 || block < 1 || radius < 0 || max_rects < 1) return DC_ERR_INVALID_ARG;
    std::vector<int> hs, ws, cs;
    const int c_tensor = input_channels(layers, n_layers, C);
    if (c_tensor < C) return DC_ERR_BAD_SHAPE;
    int rc = validate_layers(layers, n_layers, H, W, c_tensor, &hs, &ws, &cs);
    if (rc) return rc;
    for (int t = 0; t <= n_layers; ++t)
        if (!tensors_cur[t]) return DC_ERR_NULL_PTR;
    for (int i = 0; i < n_layers; ++i)
        if ((layers[i].type == DC_CONV || layers[i].type == DC_FC) && !weights[i]) return DC_ERR_NULL_PTR;
    const bool cached = !force_full;
    if (match_options) {
        if (match_options->method != DC_MATCH_EXHAUSTIVE && match_options->method != DC_MATCH_DIAMOND) return DC_ERR_INVALID_ARG;
        if (match_options->k_skip < 1) return DC_ERR_INVALID_ARG;
        if (match_options->exact_masks && (!match_options->device_plan || in_place)) return DC_ERR_UNSUPPORTED;   // planned on the GPU only
        if (match_options->cache_pool_add && !match_options->exact_masks) return DC_ERR_UNSUPPORTED;
        if (match_options->torus && (!match_options->device_plan || in_place)) return DC_ERR_UNSUPPORTED;
    }
    if (cached) {
        if (!frames_prev || !tensors_prev || !mv || !best_ssd || !global_mv || !n_pass || !block_mask || !ws_dev || !ws_host)
            return DC_ERR_NULL_PTR;
        if (block > H || block > W) return DC_ERR_BAD_SHAPE;
        for (int i = 0; i < n_layers; ++i)
            if (layers[i].type == DC_CONV && (!tensors_prev[i + 1] || (tensors_prev[i + 1] == tensors_cur[i + 1]) != (match_options && match_options->torus)))
                return DC_ERR_NULL_PTR;     // two buffers per conv output, or the one buffer of a torus
        size_t need_dev = 0, need_host = 0;
        rc = dc_stack_workspace_bytes(layers, n_layers, n_streams, H, W, C, block, max_rects, &need_dev, &need_host);
        if (rc) return rc;
        if (ws_dev_bytes < need_dev || ws_host_bytes < need_host) return DC_ERR_WORKSPACE;
    }
    if (regions_out)      // checked before anything is launched: every list fits
        for (size_t i = 0; i < (size_t)n_streams * (n_layers + 1); ++i)
            if (regions_out[i].capacity < max_rects || !regions_out[i].rects) return DC_ERR_CAPACITY;
    // max-pooling and add layers that use the cache: their outputs are cache values like the conv outputs
    const uint8_t* const no_reuse = match_options ? match_options->no_reuse : nullptr;
    // Conv outputs on a torus: single-buffered, never copied (see dc_match_options.torus).  Only the layers whose kernels
    // address a torus may touch a conv output.
    const bool torus = match_options && match_options->torus;
    // with cache_pool_add the poolings' outputs are cache values too and lie on a torus like the conv outputs
    const bool pool_torus = torus && match_options->cache_pool_add;
    auto on_torus = [&](int t) {
        return torus && t > 0 && (layers[t - 1].type == DC_CONV || (pool_torus && layers[t - 1].type == DC_MAXPOOL));
    };
    if (torus) {
        const size_t esz = dtype_size(dtype);
        auto conv_output = [&](int t) { return t > 0 && layers[t - 1].type == DC_CONV; };
        for (int i = 0; i < n_layers; ++i) {
            const dc_layer& l = layers[i];
            const int t = i + 1;
            if (l.type == DC_CONV) {
                const bool first = l.in0 == 0 && cs[0] * esz == 16 && l.cout % 16 == 0 &&
                                   ((l.k == 3 && l.s == 1) || (l.k == 7 && l.s == 2) || (l.k == 11 && l.s == 4));
                const bool gemm3 = l.k == 3 && l.s == 1 && l.cout % 64 == 0 && (l.cin * esz) % 64 == 0;
                const bool point = l.k == 1 && l.s == 1 && l.p == 0 && l.cout % 8 == 0 && (l.cin * esz) % 16 == 0;
                if (!plain_square(l) || !(first || gemm3 || point)) return DC_ERR_UNSUPPORTED;
                if (!tensors_prev || tensors_prev[t] != tensors_cur[t]) return DC_ERR_INVALID_ARG;     // one buffer per conv output
            } else if (l.type == DC_MAXPOOL) {
                if ((conv_output(l.in0) || pool_torus) &&
                    !(conv_output(l.in0) && l.k == 2 && l.s == 2 && l.p == 0 && (cs[l.in0] * esz) % 16 == 0 &&
                      (size_t)n_streams * hs[t] <= 65535))
                    return DC_ERR_UNSUPPORTED;
                if (pool_torus && (!tensors_prev || tensors_prev[t] != tensors_cur[t])) return DC_ERR_INVALID_ARG;   // one buffer
            } else {
                if (pool_torus && l.type == DC_ADD) return DC_ERR_UNSUPPORTED;       // an add layer that uses the cache copies
                int ids[4] = {l.in0, l.type == DC_ADD ? l.in1 : -1, -1, -1};
                int m = l.type == DC_ADD ? 2 : 1;
                if (l.type == DC_CONCAT) m = concat_inputs(l, ids);
                for (int j = 0; j < m; ++j)
                    if (on_torus(ids[j])) return DC_ERR_UNSUPPORTED;
            }
        }
    }
    const bool cache_other = cached && match_options && match_options->cache_pool_add && match_options->exact_masks;
    auto uses_cache = [&](int i) { return cache_other && (layers[i].type == DC_MAXPOOL || layers[i].type == DC_ADD); };
    if (cache_other)
        for (int i = 0; i < n_layers; ++i)
            if (uses_cache(i)) {
                if (!tensors_prev[i + 1] || (tensors_prev[i + 1] == tensors_cur[i + 1]) != pool_torus) return DC_ERR_NULL_PTR;
                if ((cs[i + 1] * dtype_size(dtype)) % 16 || (size_t)n_streams * hs[i + 1] > 65535 ||
                    reinterpret_cast<uintptr_t>(tensors_prev[i + 1]) % 16 || reinterpret_cast<uintptr_t>(tensors_cur[i + 1]) % 16)
                    return DC_ERR_UNSUPPORTED;
            }
    Overlap* ov = static_cast<Overlap*>(overlap);
    hipStream_t caller_st = as_stream(stream);
    // a look-ahead match is for the very next call only (the caller may reuse its frame buffers after that)
    Overlap::Prefetch pf;
    if (ov) { pf = ov->prefetch; ov->prefetch.valid = false; }
    // Pipelined: this frame's work goes to one of the handle's two streams, the previous frame's is on the other.
    const bool pipe = ov && ov->pipeline;
    const int fp = pipe ? ov->frame_parity : 0;
    hipStream_t st = pipe ? ov->work[fp] : caller_st;
    if (pipe) {
        try {
            for (int p = 0; p < 2; ++p)
                while ((int)ov->layer_done[p].size() < n_layers) {
                    hipEvent_t e;
                    DC_TRY_HIP(hipEventCreateWithFlags(&e, hipEventDisableTiming));
                    ov->layer_done[p].push_back(e);
                }
        } catch (const std::bad_alloc&) {
            return DC_ERR_WORKSPACE;
        }
    }
    // last layer that reads each tensor: a layer that overwrites a single-buffered tensor waits for it
    std::vector<int> last_reader(n_layers + 1, -1);
    for (int i = 0; i < n_layers; ++i) {
        last_reader[layers[i].in0] = i;
        if (layers[i].type == DC_ADD) last_reader[layers[i].in1] = i;
        if (layers[i].type == DC_CONCAT) {
            int ids[4];
            const int m = concat_inputs(layers[i], ids);
            for (int j = 0; j < m; ++j) last_reader[ids[j]] = i;
        }
    }
    // conv layers wait per run of consecutive conv layers (for the last one of the run): fewer cross-stream
    // dependencies, and the copies of a run go out in one launch
    std::vector<int> run_end(n_layers, -1);
    for (int i = n_layers - 1; i >= 0; --i)
        if (layers[i].type == DC_CONV)
            run_end[i] = (i + 1 < n_layers && layers[i + 1].type == DC_CONV) ? run_end[i + 1] : i;
    // A tensor that holds no cached values (anything but a conv output) may be one buffer for all frames, or the
    // caller may alternate it like the conv outputs.  If this frame's buffer is not the previous frame's but the
    // one this work stream used for its last frame, its last users are on this same stream: no cross-stream
    // wait, and (expecting the caller to go on alternating) no event for the next frame.  Should the next frame
    // then use this frame's buffer after all, it finds no event and waits for the whole frame.
    std::vector<char> fresh(n_layers + 1, 0);
    if (pipe && ov->last_cur[0].size() == (size_t)n_layers + 1 && ov->last_cur[1].size() == (size_t)n_layers + 1)
        for (int t = 0; t <= n_layers; ++t)
            fresh[t] = (t == 0 || layers[t - 1].type != DC_CONV) && ov->last_cur[1 - fp][t] != tensors_cur[t] &&
                       ov->last_cur[fp][t] == tensors_cur[t];
    // only the layers that the next frame can wait for get an event
    std::vector<char> is_target(n_layers, 0);
    if (pipe) {
        if (last_reader[0] >= 0 && !fresh[0]) is_target[last_reader[0]] = 1;
        for (int i = 0; i < n_layers; ++i) {
            if (layers[i].type == DC_CONV) is_target[run_end[i]] = 1;
            if (uses_cache(i)) is_target[i] = 1;          // the next frame reads this layer's output as its cache
            if ((layers[i].type != DC_CONV || in_place || torus) && last_reader[i + 1] >= 0 && !fresh[i + 1])
                is_target[last_reader[i + 1]] = 1;
        }
    }
    int waited = -1;
    auto wait_prev = [&](int w) -> hipError_t {     // the previous frame has finished its layers 0..w
        if (!pipe || w <= waited) return hipSuccess;
        const std::vector<char>& rec = ov->recorded[1 - fp];
        if ((size_t)w < rec.size() && rec[w]) {
            waited = w;
            return hipStreamWaitEvent(st, ov->layer_done[1 - fp][w], 0);
        }
        waited = n_layers;
        return ov->frame_recorded[1 - fp] ? hipStreamWaitEvent(st, ov->frame_done[1 - fp], 0) : hipSuccess;
    };
    auto wait_readers = [&](int t) -> hipError_t {  // before tensor t is overwritten
        return fresh[t] ? hipSuccess : wait_prev(last_reader[t]);
    };
    if (pipe) {
        try {
            ov->recorded[fp].assign(n_layers, 0);
            ov->last_cur[fp].reserve(n_layers + 1);
        } catch (const std::bad_alloc&) {
            return DC_ERR_WORKSPACE;
        }
        ov->frame_recorded[fp] = false;
    }
    // Device workspace: [plans, frame parity 0][plans, parity 1][K-split scratch 0][scratch 1]
    unsigned char* plan_dev = nullptr;
    unsigned char* conv_scratch = nullptr;
    if (ws_dev && ws_dev_bytes >= 2 * kConvScratchBytes) {
        const size_t plan_half = (ws_dev_bytes - 2 * kConvScratchBytes) / 2 / 256 * 256;
        plan_dev = static_cast<unsigned char*>(ws_dev) + (size_t)fp * plan_half;
        conv_scratch = static_cast<unsigned char*>(ws_dev) + 2 * plan_half + (size_t)fp * kConvScratchBytes;
    }
    const int gh = H / block, gw = W / block;
    const size_t nb = (size_t)n_streams * gh * gw;

    dc_stack_stats local;
    std::memset(&local, 0, sizeof(local));
    if (stats) {
        local.layer_reused_px = stats->layer_reused_px;
        local.layer_issued_macs = stats->layer_issued_macs;
        local.profile = stats->profile;
        local.layer_kernel_id = stats->layer_kernel_id;
    }
    local.full = cached ? 0 : 1;
    local.n_blocks = (int32_t)nb;

    bool inplace = false;
    if (in_place) *in_place = 0;
    std::vector<std::vector<TensorRegions>> regs;  // [stream][tensor]
    unsigned char* hbase = static_cast<unsigned char*>(ws_host);

    // ---- planning on the GPU: no read-back of the mask, no host wait (when asked for and the kernels can take it) ----
    DevPlanLayout dl;
    bool devplan = false;
    PlanDev pd{};
    DevHostHeader* hdr = nullptr;
    std::vector<long> unit_hint;
    if (cached && match_options && match_options->device_plan && !in_place && gh >= 1 && gw >= 1 && gh <= 64 && gw <= 64 &&
        ws_host_bytes >= kDevHostRegion + 256 && ws_dev_bytes >= 2 * kConvScratchBytes) {
        try {
            device_plan_layout(layers, n_layers, hs, ws, n_streams, max_rects, dl, no_reuse);
            unit_hint.assign(dl.convs.size(), -1);
        } catch (const std::bad_alloc&) {
            return DC_ERR_WORKSPACE;
        }
        devplan = dl.ok && 3 * (align_up(dl.table_bytes, 256) + dl.frame_bytes) <= ws_dev_bytes - 2 * kConvScratchBytes &&
                  dl.table_bytes <= kDevHostRegion - 3 * kDevHostSlot;
    }
    if (torus && cached && !devplan) return DC_ERR_UNSUPPORTED;      // a torus frame is planned on the GPU or not at all
    if (torus && !cached && match_options->origins_dev_out) *match_options->origins_dev_out = nullptr;
    if (torus && !cached && ws_host && ws_host_bytes >= kDevHostRegion + 256) {
        // a full frame writes every tensor at its buffer's start: the next cached frame starts from origins (0, 0)
        DevHostHeader* h = reinterpret_cast<DevHostHeader*>(hbase + ((ws_host_bytes - kDevHostRegion) & ~(size_t)255));
        if (h->magic == kDevHostMagic) h->origin_area = -1;
    }
    if (devplan) {
        unsigned char* const region = hbase + ((ws_host_bytes - kDevHostRegion) & ~(size_t)255);
        hdr = reinterpret_cast<DevHostHeader*>(region);
        unsigned char* const slots = region + kDevHostSlot;
        unsigned char* const staging = region + 3 * kDevHostSlot;
        // The layer tables travel with every frame (a few KB, one small launch): what the device workspace holds
        // from earlier calls is never trusted.  The staging copy is rewritten only when it differs, and then nothing
        // may still be reading it.
        uint64_t sig = fnv1a(0xcbf29ce484222325ull, layers, (size_t)n_layers * sizeof(dc_layer));
        const int32_t shape[8] = {n_streams, H, W, C, block, dl.cap, dtype, n_layers};
        sig = fnv1a(sig, shape, sizeof(shape));
        try {
            std::vector<unsigned char> tables(dl.table_bytes, 0);
            std::memcpy(tables.data(), dl.layers.data(), dl.layers.size() * sizeof(PlanLayerDev));
            std::memcpy(tables.data() + dl.off_tensors, dl.tensors.data(), dl.tensors.size() * sizeof(PlanTensorDev));
            if (!dl.convs.empty()) std::memcpy(tables.data() + dl.off_convs, dl.convs.data(), dl.convs.size() * sizeof(PlanConvDev));
            if (std::memcmp(staging, tables.data(), dl.table_bytes) != 0) {
                if (ov) DC_TRY_HIP(hipStreamSynchronize(ov->aux));
                DC_TRY_HIP(hipStreamSynchronize(st));
                std::memcpy(staging, tables.data(), dl.table_bytes);
            }
        } catch (const std::bad_alloc&) {
            return DC_ERR_WORKSPACE;
        }
        if (hdr->magic != kDevHostMagic || hdr->signature != sig || hdr->ws_dev != ws_dev || (hdr->last_slot != 0 && hdr->last_slot != 1)) {
            std::memset(region, 0, 3 * kDevHostSlot);          // other stack or workspace: the counters start afresh
            hdr->last_slot = 1;
            hdr->origin_area = -1;
        }
        hdr->magic = kDevHostMagic; hdr->signature = sig; hdr->ws_dev = ws_dev;
        hdr->n_layers = n_layers; hdr->n_convs = (int32_t)dl.convs.size();
        for (size_t c = 0; c < dl.convs.size(); ++c) {
            const dc_layer& l = layers[dl.conv_layer[c]];
            hdr->conv[c] = DevHostConv{dl.conv_layer[c], (int32_t)(l.cout * dtype_size(dtype)), (int64_t)window_geom(l).kh * window_geom(l).kw * l.cin * l.cout,
                                       (int64_t)n_streams * dl.convs[c].Hout * dl.convs[c].Wout};
        }
        // With an overlap handle the matching and the planning run on the handle's stream, ahead of the layers: they
        // depend on the frames only, so they are done while the previous frame's layers still run, and the frame's
        // own stream only waits for the plan.  Three plan areas (tables included) take turns: two frames in flight
        // and the one being planned.
        const int area = ov ? ov->plan_counter % 3 : 0;
        hipStream_t pst = ov ? ov->aux : st;
        if (ov && ov->area_recorded[area]) DC_TRY_HIP(hipStreamWaitEvent(pst, ov->area_free[area], 0));
        const size_t table_slot = align_up(dl.table_bytes, 256);
        unsigned char* const table_dev = static_cast<unsigned char*>(ws_dev) + (size_t)area * (table_slot + dl.frame_bytes);
        DC_TRY_HIP(upload_plans(table_dev, staging, dl.table_bytes, ws_host, pst));
        // list lengths of the last frame whose counters have arrived: a guess of this frame's, for the launch shapes only
        {
            const PlanStatsConv* seen = reinterpret_cast<const PlanStatsConv*>(slots + (size_t)hdr->last_slot * kDevHostSlot + sizeof(PlanStatsHead));
            for (size_t c = 0; c < dl.convs.size(); ++c) {
                const int32_t v = *reinterpret_cast<const volatile int32_t*>(&seen[c].n_units);
                unit_hint[c] = v > 0 ? v : -1;
            }
        }
        const int slot = hdr->last_slot ^ 1;
        unsigned char* const frame = table_dev + table_slot;
        pd.layers = reinterpret_cast<const PlanLayerDev*>(table_dev);
        pd.tensors = reinterpret_cast<const PlanTensorDev*>(table_dev + dl.off_tensors);
        pd.convs = reinterpret_cast<const PlanConvDev*>(table_dev + dl.off_convs);
        pd.n_layers = n_layers; pd.n_convs = (int32_t)dl.convs.size(); pd.n_streams = n_streams; pd.cap = dl.cap;
        pd.rects = reinterpret_cast<dc_rect*>(frame);
        pd.nrect = reinterpret_cast<int32_t*>(frame + dl.off_nrect);
        pd.dxy = reinterpret_cast<int32_t*>(frame + dl.off_dxy);
        pd.stream_info = reinterpret_cast<int32_t*>(frame + dl.off_info);
        pd.n_units = reinterpret_cast<int32_t*>(frame + dl.off_nunits);
        pd.area = frame + dl.off_area;
        pd.bitmaps = reinterpret_cast<uint32_t*>(frame + dl.off_bitmaps);
        pd.bm_words = dl.bm_words;
        pd.origin = nullptr; pd.origin_prev = nullptr; pd.pool_torus = pool_torus ? 1 : 0;
        if (torus) {          // this frame's origins follow from the previous frame's, which its plan area still holds
            pd.origin = reinterpret_cast<int32_t*>(frame + dl.off_origin);
            if (hdr->origin_area >= 0 && hdr->origin_area < 3)
                pd.origin_prev = reinterpret_cast<const int32_t*>(static_cast<unsigned char*>(ws_dev) +
                                                                  (size_t)hdr->origin_area * (table_slot + dl.frame_bytes) + table_slot + dl.off_origin);
            hdr->origin_area = area;
        } else {
            hdr->origin_area = -1;
        }
        hdr->torus = torus ? 1 : 0;
        unsigned char* const slot_host = slots + (size_t)slot * kDevHostSlot;
        const unsigned char* alias = device_alias(ws_host);
        pd.stats = alias ? const_cast<unsigned char*>(alias) + (slot_host - static_cast<unsigned char*>(ws_host))
                         : frame + dl.off_stats;
        DC_TRY_HIP(wait_readers(0));
        DC_TRY_HIP(launch_frame_to_tensor(frames_cur, tensors_cur[0], (size_t)n_streams * H * W, C, c_tensor, dtype, st));
        // (the match buffers are shared by consecutive frames: their matching and planning kernels follow one another
        // on one stream)
        bool prefetched = false;
        if (ov) {
            prefetched = pf.valid && pf.cur == frames_cur && pf.prev == frames_prev && pf.mv == mv &&
                         pf.best_ssd == best_ssd && pf.gmv == global_mv && pf.n_pass == n_pass && pf.mask == block_mask &&
                         pf.ws_host == ws_host && pf.n_streams == n_streams && pf.H == H && pf.W == W && pf.C == C &&
                         pf.block == block && pf.radius == radius && pf.max_block_ssd == max_block_ssd &&
                         pf.method == match_options->method && pf.k_skip == match_options->k_skip;
        }
        if (!prefetched) {     // (a match started ahead of time is on the same stream: the plan follows it)
            rc = dc_match_blocks_opt(frames_cur, frames_prev, n_streams, H, W, C, block, radius, match_options,
                                     max_block_ssd, mv, best_ssd, global_mv, n_pass, block_mask, pst);
            if (rc) return rc;
        }
        if (match_options->exact_masks)
            DC_TRY_HIP(launch_plan_exact(pd, block_mask, global_mv, gh, gw, block, match_options->extend_borders, dl.max_chunks, true, pst));
        else
            DC_TRY_HIP(launch_plan(pd, block_mask, global_mv, gh, gw, block, match_options->extend_borders, dl.max_chunks, pst));
        if (!alias)
            DC_TRY_HIP(hipMemcpyAsync(slot_host, frame + dl.off_stats, sizeof(PlanStatsHead) + dl.convs.size() * sizeof(PlanStatsConv),
                                      hipMemcpyDeviceToHost, pst));
        if (ov) {
            DC_TRY_HIP(hipEventRecord(ov->plan_done[area], pst));
            DC_TRY_HIP(hipStreamWaitEvent(st, ov->plan_done[area], 0));
        }
        hdr->last_slot = slot;
        hdr->n_blocks = (int32_t)nb;
        if (torus && match_options->origins_dev_out) *match_options->origins_dev_out = pd.origin;
        if (torus && match_options->origins_out) {      // for inspection only: wait for the plan and read the origins back
            DC_TRY_HIP(hipStreamSynchronize(pst));
            DC_TRY_HIP(hipMemcpy(match_options->origins_out, pd.origin, (size_t)n_streams * (n_layers + 1) * 2 * sizeof(int32_t),
                                 hipMemcpyDeviceToHost));
        }
        if (regions_out) {      // for inspection only: wait for the lists and read them back
            const int nt = n_layers + 1;
            try {
                std::vector<int32_t> h_n((size_t)n_streams * nt), h_d((size_t)n_streams * nt * 2);
                std::vector<dc_rect> h_r((size_t)n_streams * nt * dl.cap);
                DC_TRY_HIP(hipStreamSynchronize(pst));
                DC_TRY_HIP(hipMemcpy(h_n.data(), pd.nrect, h_n.size() * sizeof(int32_t), hipMemcpyDeviceToHost));
                DC_TRY_HIP(hipMemcpy(h_d.data(), pd.dxy, h_d.size() * sizeof(int32_t), hipMemcpyDeviceToHost));
                DC_TRY_HIP(hipMemcpy(h_r.data(), pd.rects, h_r.size() * sizeof(dc_rect), hipMemcpyDeviceToHost));
                for (int s = 0; s < n_streams; ++s)
                    for (int t = 0; t < nt; ++t) {
                        dc_regions& r = regions_out[(size_t)s * nt + t];
                        const size_t at = (size_t)s * nt + t;
                        r.n = h_n[at]; r.dx = h_d[2 * at]; r.dy = h_d[2 * at + 1];
                        r.cum_stride = dl.tensors[t].cum_stride; r.h = hs[t]; r.w = ws[t];
                        if (r.n) std::memcpy(r.rects, h_r.data() + at * dl.cap, (size_t)r.n * sizeof(dc_rect));   // n <= cap <= capacity
                    }
            } catch (const std::bad_alloc&) {
                return DC_ERR_WORKSPACE;
            }
        }
    } else if (cached) {
        // With an overlap handle the matching runs on its own stream, next to whatever the main stream
        // still holds of the previous frame; only that stream is waited for.
        hipStream_t mst = ov ? ov->aux : st;
        uint8_t* h_mask = hbase;
        int32_t* h_gmv = reinterpret_cast<int32_t*>(hbase + align_up(nb, 256));
        // a match started ahead of time with exactly these arguments is on its way or done already
        bool prefetched = false;
        if (ov) {
            prefetched = pf.valid && pf.cur == frames_cur && pf.prev == frames_prev && pf.mv == mv &&
                         pf.best_ssd == best_ssd && pf.gmv == global_mv && pf.n_pass == n_pass && pf.mask == block_mask &&
                         pf.ws_host == ws_host && pf.n_streams == n_streams && pf.H == H && pf.W == W && pf.C == C &&
                         pf.block == block && pf.radius == radius && pf.max_block_ssd == max_block_ssd &&
                         pf.method == (match_options ? match_options->method : DC_MATCH_EXHAUSTIVE) &&
                         pf.k_skip == (match_options ? match_options->k_skip : 1);
            if (pf.valid && !prefetched) DC_TRY_HIP(hipStreamSynchronize(mst));   // let the stale match finish first
        }
        if (!prefetched) {
            rc = dc_match_blocks_opt(frames_cur, frames_prev, n_streams, H, W, C, block, radius, match_options,
                                     max_block_ssd, mv, best_ssd, global_mv, n_pass, block_mask, mst);
            if (rc) return rc;
            DC_TRY_HIP(hipMemcpyAsync(h_mask, block_mask, nb, hipMemcpyDeviceToHost, mst));
            DC_TRY_HIP(hipMemcpyAsync(h_gmv, global_mv, (size_t)n_streams * 2 * sizeof(int32_t), hipMemcpyDeviceToHost, mst));
        }
        // the network input does not depend on the match: its conversion overlaps the readback
        DC_TRY_HIP(wait_readers(0));
        DC_TRY_HIP(launch_frame_to_tensor(frames_cur, tensors_cur[0], (size_t)n_streams * H * W, C, c_tensor, dtype, st));
        if (ov) {
            if (!prefetched) DC_TRY_HIP(hipEventRecord(ov->match_done, mst));
            DC_TRY_HIP(spin_wait(ov->match_done));
        } else {
            DC_TRY_HIP(hipStreamSynchronize(mst));
        }
        if (in_place) {     // no stream moved: the previous frame's conv outputs can be updated where they are
            inplace = true;
            for (int s = 0; s < n_streams; ++s) inplace = inplace && h_gmv[2 * s] == 0 && h_gmv[2 * s + 1] == 0;
        }
        try {
            regs.resize(n_streams);
        } catch (const std::bad_alloc&) {
            return DC_ERR_WORKSPACE;
        }
        {   // per stream: count, merge (Step 5), propagate (Section 5); streams are independent
            std::vector<int> stream_rc(n_streams, DC_OK), stream_reusable(n_streams, 0), stream_over(n_streams, 0);
            parallel_for(n_streams, [&](int s) {
                try {
                    std::vector<dc_rect> rects0;
                    const uint8_t* m = h_mask + (size_t)s * gh * gw;
                    int cnt = 0;
                    for (int i = 0; i < gh * gw; ++i) cnt += m[i] ? 1 : 0;
                    stream_reusable[s] = cnt;
                    merge_blocks(m, gh, gw, block, rects0);
                    int r = propagate(layers, n_layers, H, W, rects0, h_gmv[2 * s], h_gmv[2 * s + 1], regs[s],
                                      match_options && match_options->extend_borders != 0);
                    // a list longer than the caller allows: the stream reuses nothing in this frame (always valid)
                    bool over = false;
                    for (int t = 0; r == DC_OK && t <= n_layers; ++t) over = over || (int)regs[s][t].rects.size() > max_rects;
                    if (over) {
                        for (int t = 0; t <= n_layers; ++t) regs[s][t].rects.clear();
                        stream_over[s] = 1;
                    }
                    stream_rc[s] = r;
                } catch (const std::bad_alloc&) {
                    stream_rc[s] = DC_ERR_WORKSPACE;
                }
            });
            for (int s = 0; s < n_streams; ++s) {
                if (stream_rc[s]) return stream_rc[s];
                local.n_reusable_blocks += stream_reusable[s];
                local.n_overflow_streams += stream_over[s];
            }
        }
        hbase += align_up(nb, 256) + align_up((size_t)n_streams * 3 * sizeof(int32_t), 256);
        if (ov) {
            // two staging halves: the upload of the frame before last must have left the half reused now
            const size_t half = (ws_host_bytes - kDevHostRegion - (size_t)(hbase - static_cast<unsigned char*>(ws_host))) / 2 / 256 * 256;
            hbase += (size_t)ov->parity * half;
            if (ov->pending[ov->parity]) {
                DC_TRY_HIP(spin_wait(ov->upload_done[ov->parity]));
                ov->pending[ov->parity] = false;
            }
        }
    } else {
        DC_TRY_HIP(wait_readers(0));
        DC_TRY_HIP(launch_frame_to_tensor(frames_cur, tensors_cur[0], (size_t)n_streams * H * W, C, c_tensor, dtype, st));
    }
    if (regions_out && !devplan) {
        for (int s = 0; s < n_streams; ++s)
            for (int t = 0; t <= n_layers; ++t) {
                dc_regions& r = regions_out[(size_t)s * (n_layers + 1) + t];
                if (cached) {
                    const TensorRegions& g = regs[s][t];
                    r.n = (int)g.rects.size(); r.dx = g.dx; r.dy = g.dy; r.cum_stride = g.cum_stride; r.h = g.h; r.w = g.w;
                    if (r.n) std::memcpy(r.rects, g.rects.data(), r.n * sizeof(dc_rect));     // n <= max_rects <= capacity
                } else {
                    r.n = 0; r.dx = r.dy = 0; r.cum_stride = 0; r.h = hs[t]; r.w = ws[t];
                }
            }
    }

    // ---- plans of all conv layers, one upload ----
    std::vector<LayerPlan> plans(n_layers);
    std::vector<PlanAddr> addrs(n_layers);
    std::vector<ConvTiling> tilings(n_layers);
    size_t off = 0;
    // The tiles of every (stream, conv layer) are classified in parallel over the streams into per-stream lists,
    // the per-layer offsets follow from their sizes, and the lists are then copied straight into the pinned
    // staging buffer, again in parallel (64 streams: 550 k tiles per frame).
    std::lock_guard<std::mutex> plan_guard(g_frame_plan_mutex);
    FramePlan& frame_plan = g_frame_plan;
    if (cached && !devplan) {
        int rc_plan = frame_plan.classify(layers, n_layers, n_streams, regs, hs, ws, no_reuse);
        if (rc_plan) return rc_plan;
    }

    try {
        for (int i = 0; i < n_layers; ++i) {
            const dc_layer& l = layers[i];
            if (l.type != DC_CONV) continue;
            tilings[i] = pick_tiling(l, hs[i + 1], ws[i + 1], n_streams, dtype);
            const int64_t px = (int64_t)hs[i + 1] * ws[i + 1] * n_streams;
            const int64_t mac_px = (int64_t)window_geom(l).kh * window_geom(l).kw * l.cin * l.cout;
            local.macs_full += px * mac_px;
            if (!cached) {
                local.macs_needed += px * mac_px;
                int64_t tiles = (int64_t)n_streams * ((hs[i + 1] + tilings[i].th - 1) / tilings[i].th) *
                                ((ws[i + 1] + tilings[i].tw - 1) / tilings[i].tw);
                int64_t issued = tiles * tilings[i].th * tilings[i].tw * mac_px;
                local.macs_issued += issued;
                if (local.layer_reused_px) local.layer_reused_px[i] = 0;
                if (local.layer_issued_macs) local.layer_issued_macs[i] = issued;
                continue;
            }
            if (devplan) continue;       // the counters of a frame planned on the GPU arrive with dc_stack_stats_fetch
            LayerPlan& plan = plans[i];
            addrs[i] = frame_plan.finish_layer(i, plan, hbase + off, plan_dev + off);
            off += addrs[i].bytes;
            int64_t issued = (int64_t)plan.n_tiles * tilings[i].th * tilings[i].tw * mac_px;
            local.macs_needed += (px - plan.reused_px) * mac_px;
            local.macs_issued += issued;
            if (!inplace) local.copy_bytes += 2 * plan.reused_px * l.cout * (int64_t)dtype_size(dtype);
            if (local.layer_reused_px) local.layer_reused_px[i] = plan.reused_px;
            if (local.layer_issued_macs) local.layer_issued_macs[i] = issued;
        }
    } catch (const std::bad_alloc&) {
        return DC_ERR_WORKSPACE;
    }
    if (cached && !devplan) frame_plan.copy_tiles();
    if (devplan) hdr->macs_full = local.macs_full;
    // ---- the shifted copies of all layers in one launch (16-byte vector path only); pipelined: one launch per
    // run of consecutive conv layers, issued when the previous frame has finished that run ----
    std::vector<char> copy_fused(n_layers, 0);
    struct CopyGroup { int first_layer, last_layer; size_t rect_begin, rect_end, max_vec; };
    std::vector<CopyGroup> groups;
    size_t all_rects_off = 0, copy_layers_off = 0, n_all_rects = 0;
    if (inplace)        // every reusable pixel already holds its value
        for (int i = 0; i < n_layers; ++i) copy_fused[i] = 1;
    // planned on the GPU: one per-unit copy launch per run of conv layers (maps of one size), from the unit masks
    struct DevCopyGroup { int first_layer, last_layer, vec_bytes; std::vector<CopyUnitsLayer> L; };
    std::vector<DevCopyGroup> dev_groups;
    if (devplan) {
        try {
            for (size_t c = 0; c < dl.convs.size(); ++c) {
                const int i = dl.conv_layer[c];
                copy_fused[i] = 1;
                if (no_reuse && no_reuse[i]) continue;          // nothing of this layer comes from the cache
                if (torus) continue;                            // the reusable pixels already lie where this frame looks for them
                const size_t px_bytes = (size_t)layers[i].cout * dtype_size(dtype);
                const bool vec16 = px_bytes % 16 == 0 && reinterpret_cast<uintptr_t>(tensors_prev[i + 1]) % 16 == 0 &&
                                   reinterpret_cast<uintptr_t>(tensors_cur[i + 1]) % 16 == 0;
                const int vb = vec16 ? 16 : (int)dtype_size(dtype);
                bool fresh_group = dev_groups.empty() || dev_groups.back().vec_bytes != vb;
                if (!fresh_group)
                    for (int j = dev_groups.back().last_layer + 1; j < i; ++j) fresh_group |= layers[j].type != DC_CONV;
                if (fresh_group) dev_groups.push_back(DevCopyGroup{i, i, vb, {}});
                DevCopyGroup& g = dev_groups.back();
                g.last_layer = i;
                const PlanConvDev& cv = dl.convs[c];
                g.L.push_back(CopyUnitsLayer{tensors_prev[i + 1], tensors_cur[i + 1],
                                             reinterpret_cast<const uint16_t*>(pd.area + cv.umask_off), cv.tensor, cv.Hout, cv.Wout,
                                             cv.units_x, cv.units_y, (int32_t)(px_bytes / vb), 0, 0});
            }
        } catch (const std::bad_alloc&) {
            return DC_ERR_WORKSPACE;
        }
    }
    if (cached && !inplace && !devplan) {
        try {
            std::vector<RectDev> all_rects;
            std::vector<CopyLayerDev> copy_layers;
            for (int i = 0; i < n_layers; ++i) {
                if (layers[i].type != DC_CONV || plans[i].rects.empty()) continue;
                const size_t px_bytes = (size_t)layers[i].cout * dtype_size(dtype);
                if (px_bytes % 16 || reinterpret_cast<uintptr_t>(tensors_prev[i + 1]) % 16 ||
                    reinterpret_cast<uintptr_t>(tensors_cur[i + 1]) % 16)
                    continue;
                copy_fused[i] = 1;
                const int pv = (int)(px_bytes / 16);
                // a new group starts at the first layer and, when pipelined, after every layer that is not a conv
                bool fresh = groups.empty();
                if (!fresh && pipe)
                    for (int j = groups.back().last_layer + 1; j < i; ++j) fresh |= layers[j].type != DC_CONV;
                if (fresh) groups.push_back(CopyGroup{i, i, all_rects.size(), all_rects.size(), 0});
                CopyGroup& g = groups.back();
                g.last_layer = i;
                for (RectDev r : plans[i].rects) {
                    r.pad = (int)copy_layers.size();
                    all_rects.push_back(r);
                    g.max_vec = std::max(g.max_vec, (size_t)r.w * r.h * pv);
                }
                g.rect_end = all_rects.size();
                copy_layers.push_back(CopyLayerDev{tensors_prev[i + 1], tensors_cur[i + 1], hs[i + 1], ws[i + 1], pv, 0});
            }
            n_all_rects = all_rects.size();
            if (n_all_rects) {
                all_rects_off = off;
                std::memcpy(hbase + off, all_rects.data(), n_all_rects * sizeof(RectDev));
                off += align_up(n_all_rects * sizeof(RectDev), 256);
                copy_layers_off = off;
                std::memcpy(hbase + off, copy_layers.data(), copy_layers.size() * sizeof(CopyLayerDev));
                off += align_up(copy_layers.size() * sizeof(CopyLayerDev), 256);
            }
        } catch (const std::bad_alloc&) {
            return DC_ERR_WORKSPACE;
        }
    }
    if (cached && off && !devplan) {
        DC_TRY_HIP(upload_plans(plan_dev, hbase, off, ws_host, st));
        if (ov) {
            DC_TRY_HIP(hipEventRecord(ov->upload_done[ov->parity], st));
            ov->pending[ov->parity] = true;
            ov->parity ^= 1;
        }
    }
    size_t next_group = 0;
    size_t next_dev_group = 0;
    auto launch_copy_group = [&](int layer) -> int {     // the group that starts at `layer`, if any
        if (devplan) {
            if (next_dev_group >= dev_groups.size() || dev_groups[next_dev_group].first_layer != layer) return DC_OK;
            const DevCopyGroup& g = dev_groups[next_dev_group++];
            DC_TRY_HIP(wait_prev(run_end[g.last_layer]));
            Bracket b(stats ? static_cast<Profile*>(stats->profile) : nullptr, n_layers + g.first_layer, st);
            DC_TRY_HIP(launch_shifted_copy_units(g.L.data(), (int)g.L.size(), pd.dxy, n_layers + 1, n_streams, g.vec_bytes, st));
            return DC_OK;
        }
        if (next_group >= groups.size() || groups[next_group].first_layer != layer) return DC_OK;
        const CopyGroup& g = groups[next_group++];
        DC_TRY_HIP(wait_prev(run_end[g.last_layer]));
        Bracket b(stats ? static_cast<Profile*>(stats->profile) : nullptr, n_layers + g.first_layer, st);
        DC_TRY_HIP(launch_shifted_copy_all(reinterpret_cast<const RectDev*>(plan_dev + all_rects_off) + g.rect_begin,
                                           (int)(g.rect_end - g.rect_begin),
                                           reinterpret_cast<const CopyLayerDev*>(plan_dev + copy_layers_off), g.max_vec, st));
        return DC_OK;
    };
    // Where each tensor of this frame lives: an in-place frame keeps the conv outputs in the previous frame's buffers.
    std::vector<void*> eff(n_layers + 1);
    for (int t = 0; t <= n_layers; ++t)
        eff[t] = (inplace && t > 0 && layers[t - 1].type == DC_CONV) ? tensors_prev[t] : tensors_cur[t];
    if (in_place) *in_place = inplace ? 1 : 0;
    // torus frames: where the origins of tensor t start (a stream's are 2 (n_layers + 1) ints apart); nullptr: the
    // tensor starts at its buffer's start (every tensor of a full frame, everything but conv outputs otherwise)
    auto origin_of = [&](int t) -> const int32_t* {
        return (devplan && on_torus(t)) ? pd.origin + 2 * t : nullptr;
    };
    // ---- layers ----
    int conv_seen = 0;
    for (int i = 0; i < n_layers; ++i) {
        const dc_layer& l = layers[i];
        const int a = l.in0, t = i + 1;
        switch (l.type) {
            case DC_CONV: {
                const int ci = conv_seen++;
                rc = launch_copy_group(i);
                if (rc) return rc;
                DC_TRY_HIP(wait_prev(run_end[i]));   // its cache: the previous frame's output of this layer (whole run)
                if (inplace || torus) DC_TRY_HIP(wait_prev(last_reader[t]));   // and the previous frame's readers of the buffer it updates
                rc = run_conv_planned(l, eff[a], weights[i], bias ? bias[i] : nullptr,
                                      cached ? tensors_prev[t] : nullptr, eff[t], n_streams, hs[a], ws[a], dtype,
                                      tilings[i], cached ? &plans[i] : nullptr, cached ? &addrs[i] : nullptr, st,
                                      stats ? static_cast<Profile*>(stats->profile) : nullptr, i, n_layers + i,
                                      local.layer_kernel_id ? &local.layer_kernel_id[i] : nullptr, copy_fused[i] != 0,
                                      conv_scratch, conv_scratch ? kConvScratchBytes : 0,
                                      packed_weights ? packed_weights[i] : nullptr,
                                      devplan ? reinterpret_cast<const TileDev*>(pd.area + dl.convs[ci].list_off) : nullptr,
                                      devplan ? n_streams * dl.convs[ci].units_x * dl.convs[ci].units_y : 0,
                                      devplan ? pd.n_units + ci : nullptr, devplan ? unit_hint[ci] : -1,
                                      origin_of(a), origin_of(t), 2 * (n_layers + 1));
                if (rc) return rc;
                break;
            }
            case DC_MAXPOOL:
                DC_TRY_HIP(wait_readers(t));
                if (origin_of(a)) {          // its input lies on a torus, and with the cache its output too
                    const CachedMap cm{pd.bitmaps, pd.bm_words, dl.tensors[t].bm_off, pd.dxy, n_layers + 1, t};
                    const bool through_cache = origin_of(t) && uses_cache(i);
                    if (through_cache) DC_TRY_HIP(wait_prev(i));     // its cache: the previous frame's output of this layer
                    DC_TRY_HIP(launch_maxpool2x2_torus(eff[a], eff[t], n_streams, hs[a], ws[a], cs[a], dtype, origin_of(a),
                                                       origin_of(t), 2 * (n_layers + 1), through_cache ? &cm : nullptr, st));
                    break;
                }
                if (devplan && uses_cache(i)) {
                    DC_TRY_HIP(wait_prev(i));                 // its cache: the previous frame's output of this layer
                    const CachedMap cm{pd.bitmaps, pd.bm_words, dl.tensors[t].bm_off, pd.dxy, n_layers + 1, t};
                    DC_TRY_HIP(launch_maxpool_cached(eff[a], tensors_prev[t], eff[t], n_streams, hs[a], ws[a], cs[a], l.k, l.s, l.p,
                                                     dtype, cm, st));
                    break;
                }
                DC_TRY_HIP(launch_maxpool(eff[a], eff[t], n_streams, hs[a], ws[a], cs[a], l.k, l.s, l.p,
                                          dtype, st));
                break;
            case DC_ADD:
                DC_TRY_HIP(wait_readers(t));
                if (devplan && uses_cache(i)) {
                    DC_TRY_HIP(wait_prev(i));
                    const CachedMap cm{pd.bitmaps, pd.bm_words, dl.tensors[t].bm_off, pd.dxy, n_layers + 1, t};
                    DC_TRY_HIP(launch_add_cached(eff[a], eff[l.in1], tensors_prev[t], eff[t], n_streams, hs[t], ws[t], cs[t], l.relu,
                                                 dtype, cm, st));
                    break;
                }
                DC_TRY_HIP(launch_add(eff[a], eff[l.in1], eff[t],
                                      (size_t)n_streams * hs[t] * ws[t] * cs[t], l.relu, dtype, st));
                break;
            case DC_AVGPOOL:
                DC_TRY_HIP(wait_readers(t));
                DC_TRY_HIP(launch_avgpool(eff[a], eff[t], n_streams, hs[a], ws[a], cs[a], l.k, l.s, l.p,
                                          dtype, st));
                break;
            case DC_LRN:
                DC_TRY_HIP(wait_readers(t));
                DC_TRY_HIP(launch_lrn(eff[a], eff[t], n_streams, hs[a], ws[a], cs[a], l.k, l.within,
                                      l.alpha, l.beta, l.kappa, dtype, st));
                break;
            case DC_CONCAT: {
                int ids[4], chans[4];
                const void* ins[4];
                const int m = concat_inputs(l, ids);
                for (int j = 0; j < m; ++j) { ins[j] = eff[ids[j]]; chans[j] = cs[ids[j]]; }
                DC_TRY_HIP(wait_readers(t));
                DC_TRY_HIP(launch_concat(ins, chans, m, eff[t], (size_t)n_streams * hs[t] * ws[t], dtype, st));
                break;
            }
            case DC_FC:
                DC_TRY_HIP(wait_readers(t));
                DC_TRY_HIP(launch_fc(eff[a], weights[i], bias ? bias[i] : nullptr, eff[t], n_streams,
                                     (size_t)hs[a] * ws[a] * cs[a], l.cout, l.relu, dtype, st));
                break;
            case DC_SOFTMAX:
                DC_TRY_HIP(wait_readers(t));
                DC_TRY_HIP(launch_softmax(eff[a], eff[t], (size_t)n_streams * hs[t] * ws[t], cs[t], dtype, st));
                break;
            default:
                DC_TRY_HIP(wait_readers(t));
                DC_TRY_HIP(launch_add(eff[a], nullptr, eff[t], (size_t)n_streams * hs[t] * ws[t] * cs[t],
                                      1, dtype, st));
                break;
        }
        if (pipe && is_target[i]) {
            DC_TRY_HIP(hipEventRecord(ov->layer_done[fp][i], st));
            ov->recorded[fp][i] = 1;
        }
    }
    if (devplan && ov) {      // the frame's layers are done with its plan area
        const int area = ov->plan_counter % 3;
        DC_TRY_HIP(hipEventRecord(ov->area_free[area], st));
        ov->area_recorded[area] = true;
        ov->plan_counter = (ov->plan_counter + 1) % 3;
    }
    if (pipe) {
        // the caller's stream sees the frame complete; the next frame goes to the other work stream
        DC_TRY_HIP(hipEventRecord(ov->frame_done[fp], st));
        ov->frame_recorded[fp] = true;
        ov->last_cur[fp].assign(tensors_cur, tensors_cur + n_layers + 1);   // capacity reserved above
        DC_TRY_HIP(hipStreamWaitEvent(caller_st, ov->frame_done[fp], 0));
        ov->frame_parity ^= 1;
    }
    if (stats) *stats = local;
    return DC_OK;
}

int32_t dc_propagate_masks_size(const dc_layer* layers, int32_t n_layers, int32_t H, int32_t W, int32_t C,
                                size_t* words_per_stream, int64_t* tensor_offset, size_t* ws_dev_bytes) {
    if (!layers || !words_per_stream || !ws_dev_bytes) return DC_ERR_NULL_PTR;
    if (n_layers < 1 || H < 1 || W < 1 || C < 1) return DC_ERR_INVALID_ARG;
    std::vector<int> hs, ws, cs;
    const int c_tensor = input_channels(layers, n_layers, C);
    if (c_tensor < C) return DC_ERR_BAD_SHAPE;
    int rc = validate_layers(layers, n_layers, H, W, c_tensor, &hs, &ws, &cs);
    if (rc) return rc;
    try {
        DevPlanLayout dl;
        device_plan_layout(layers, n_layers, hs, ws, 1, 1, dl);
        if (!dl.ok) return DC_ERR_UNSUPPORTED;
        *words_per_stream = (size_t)dl.bm_words;
        *ws_dev_bytes = dl.table_bytes + 256;
        if (tensor_offset)
            for (int t = 0; t <= n_layers; ++t) tensor_offset[t] = dl.tensors[t].bm_off;
    } catch (const std::bad_alloc&) {
        return DC_ERR_WORKSPACE;
    }
    return DC_OK;
}

int32_t dc_propagate_masks(const dc_layer* layers, int32_t n_layers, int32_t n_streams, int32_t H, int32_t W, int32_t C,
                           int32_t block, const uint8_t* block_mask, const int32_t* global_mv, int32_t extend_borders,
                           uint32_t* bitmaps, int32_t* dxy, void* ws_dev, size_t ws_dev_bytes, void* stream) {
    if (!layers || !block_mask || !global_mv || !bitmaps || !dxy || !ws_dev) return DC_ERR_NULL_PTR;
    if (n_layers < 1 || n_streams < 1 || H < 1 || W < 1 || C < 1 || block < 1) return DC_ERR_INVALID_ARG;
    if (block > H || block > W) return DC_ERR_BAD_SHAPE;
    std::vector<int> hs, ws, cs;
    const int c_tensor = input_channels(layers, n_layers, C);
    if (c_tensor < C) return DC_ERR_BAD_SHAPE;
    int rc = validate_layers(layers, n_layers, H, W, c_tensor, &hs, &ws, &cs);
    if (rc) return rc;
    hipStream_t st = as_stream(stream);
    try {
        DevPlanLayout dl;
        device_plan_layout(layers, n_layers, hs, ws, n_streams, 1, dl);
        if (!dl.ok) return DC_ERR_UNSUPPORTED;
        if (ws_dev_bytes < dl.table_bytes + 256) return DC_ERR_WORKSPACE;
        std::vector<unsigned char> tables(dl.table_bytes, 0);
        std::memcpy(tables.data(), dl.layers.data(), dl.layers.size() * sizeof(PlanLayerDev));
        std::memcpy(tables.data() + dl.off_tensors, dl.tensors.data(), dl.tensors.size() * sizeof(PlanTensorDev));
        unsigned char* const table_dev = static_cast<unsigned char*>(ws_dev);
        DC_TRY_HIP(hipMemcpyAsync(table_dev, tables.data(), dl.table_bytes, hipMemcpyHostToDevice, st));
        DC_TRY_HIP(hipStreamSynchronize(st));          // `tables` goes away with this scope
        PlanDev pd{};
        pd.layers = reinterpret_cast<const PlanLayerDev*>(table_dev);
        pd.tensors = reinterpret_cast<const PlanTensorDev*>(table_dev + dl.off_tensors);
        pd.n_layers = n_layers; pd.n_convs = 0; pd.n_streams = n_streams; pd.cap = 1;
        pd.dxy = dxy;
        // the kernel also leaves a block count and empty rectangle lists: into the tail of the workspace
        int32_t* tail = reinterpret_cast<int32_t*>(table_dev + dl.table_bytes);
        if (ws_dev_bytes < dl.table_bytes + 256 + (size_t)n_streams * (n_layers + 3) * sizeof(int32_t)) return DC_ERR_WORKSPACE;
        pd.stream_info = tail + 64;
        pd.nrect = tail + 64 + 2 * n_streams;
        pd.bitmaps = bitmaps; pd.bm_words = dl.bm_words;
        DC_TRY_HIP(launch_plan_exact(pd, block_mask, global_mv, H / block, W / block, block, extend_borders, 0, false, st));
    } catch (const std::bad_alloc&) {
        return DC_ERR_WORKSPACE;
    }
    return DC_OK;
}

int32_t dc_stack_stats_fetch(const void* ws_host, size_t ws_host_bytes, dc_stack_stats* stats) {
    if (!ws_host || !stats) return DC_ERR_NULL_PTR;
    if (ws_host_bytes < kDevHostRegion + 256) return DC_ERR_WORKSPACE;
    const unsigned char* region = static_cast<const unsigned char*>(ws_host) + ((ws_host_bytes - kDevHostRegion) & ~(size_t)255);
    const DevHostHeader* hdr = reinterpret_cast<const DevHostHeader*>(region);
    if (hdr->magic != kDevHostMagic || hdr->n_convs < 0 || hdr->n_convs > kPlanMaxConvs) return DC_ERR_INVALID_ARG;
    const unsigned char* slot = region + kDevHostSlot + (size_t)hdr->last_slot * kDevHostSlot;
    const PlanStatsHead* sh = reinterpret_cast<const PlanStatsHead*>(slot);
    const PlanStatsConv* sc = reinterpret_cast<const PlanStatsConv*>(slot + sizeof(PlanStatsHead));
    stats->full = 0;
    stats->n_blocks = hdr->n_blocks;
    stats->n_reusable_blocks = sh->n_reusable_blocks;
    stats->n_overflow_streams = sh->n_overflow_streams;
    stats->macs_full = hdr->macs_full;
    stats->macs_needed = 0; stats->macs_issued = 0; stats->copy_bytes = 0;
    for (int c = 0; c < hdr->n_convs; ++c) {
        const DevHostConv& hc = hdr->conv[c];
        const int64_t issued = (int64_t)sc[c].n_units * 16 * hc.mac_px;
        stats->macs_needed += (hc.px_total - sc[c].reused_px) * hc.mac_px;
        stats->macs_issued += issued;
        if (!hdr->torus) stats->copy_bytes += 2 * sc[c].reused_px * hc.cout_bytes;
        if (stats->layer_reused_px) stats->layer_reused_px[hc.layer] = sc[c].reused_px;
        if (stats->layer_issued_macs) stats->layer_issued_macs[hc.layer] = issued;
    }
    return DC_OK;
}

}  // extern "C"
