// Planning of a cached frame on the GPU: merging the reusable blocks into rectangles (Section 4, Step 5),
// propagating them through the layer table (Section 5 "Propagation", Table 2), and listing, per conv layer, the
// 4x4-pixel output units that hold a non-reusable pixel.  The host path (dc_regions.cpp) does the same after
// reading the block mask back; here nothing leaves the device, so the host never waits for the matching.
//
// The rules are those of the host path, and the results are the same lists in the same order:
//   merge      row-major scan; the first open block grows right over open blocks, then down while the whole run is
//              open; the blocks of the rectangle are closed
//   conv/pool  the largest output rectangle whose k x k windows lie inside the input rectangle:
//              first column ceil((x + p) / s), last column floor((x + w - k + p) / s)
//   LRN over pixels: x + r, y + r, w - 2r, h - 2r;  add / concat: pairwise overlaps;  FC / softmax: nothing
//   every tensor has one source offset round(M / cumulative stride); rectangles are clipped so that the source
//   stays inside the map
#include "dc_internal.h"

namespace dc {

namespace {

struct SpanD { int lo, hi; };   // half-open [lo, hi)

__device__ __forceinline__ int floor_div(int a, int b) {   // b > 0
    const int q = a / b, r = a % b;
    return r < 0 ? q - 1 : q;
}
__device__ __forceinline__ int ceil_div(int a, int b) { return floor_div(a + b - 1, b); }
__device__ __forceinline__ bool none(SpanD s) { return s.hi <= s.lo; }
__device__ __forceinline__ SpanD both(SpanD a, SpanD b) { return SpanD{a.lo > b.lo ? a.lo : b.lo, a.hi < b.hi ? a.hi : b.hi}; }
// outputs whose window [o s - p, o s - p + k) lies inside `in`
__device__ __forceinline__ SpanD windows_inside(SpanD in, int k, int s, int p) {
    return SpanD{ceil_div(in.lo + p, s), floor_div(in.hi - k + p, s) + 1};
}
// the same for a stream that did not move: taps in the zero padding read zeros in both frames, so a span that
// touches an end of the input axis keeps the outputs up to that end
__device__ __forceinline__ SpanD windows_inside_ext(SpanD in, int k, int s, int p, int size_in) {
    const int size_out = (size_in + 2 * p - k) / s + 1;
    const int lo = in.lo == 0 ? 0 : ceil_div(in.lo + p, s);
    int hi = floor_div(in.hi - k + p, s) + 1;
    hi = in.hi == size_in ? size_out : (hi < size_out ? hi : size_out);
    return SpanD{lo, hi};
}
// part of `cur` that lies in [0, size) and whose source cur + d does too
__device__ __forceinline__ SpanD source_inside(SpanD cur, int d, int size) {
    return both(both(cur, SpanD{0, size}), SpanD{-d, size - d});
}
__device__ __forceinline__ int round_half_away(int num, int den) {
    const long long mag = num < 0 ? -(long long)num : num;
    const long long q = (2 * mag + den) / (2 * (long long)den);
    return (int)(num < 0 ? -q : q);
}

// A rectangle another lane of this wavefront stored earlier in this kernel: read at device scope, past the CU's
// vector cache (the fence after every layer has made the stores visible there).
__device__ __forceinline__ dc_rect load_rect(const dc_rect* p) {
    const int* q = reinterpret_cast<const int*>(p);
    dc_rect r;
    r.x = __hip_atomic_load(q + 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    r.y = __hip_atomic_load(q + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    r.w = __hip_atomic_load(q + 2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    r.h = __hip_atomic_load(q + 3, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return r;
}

// Appends the rectangles (xs, ys) of the lanes with `ok` to `list` in lane order; returns the new length.
__device__ __forceinline__ int append(dc_rect* list, int n, int cap, bool ok, SpanD xs, SpanD ys, int lane, bool& over) {
    const unsigned long long b = __ballot(ok);
    const int pos = n + __popcll(b & ((1ull << lane) - 1ull));
    if (ok && pos < cap) list[pos] = dc_rect{xs.lo, ys.lo, xs.hi - xs.lo, ys.hi - ys.lo};
    n += __popcll(b);
    if (n > cap) { over = true; n = cap; }
    return n;
}

__global__ __launch_bounds__(64) void plan_regions_kernel(PlanDev P, const uint8_t* __restrict__ block_mask,
                                                          const int32_t* __restrict__ gmv, int gh, int gw, int B, int ext_opt) {
    const int stream = blockIdx.x, lane = threadIdx.x;
    const int nt = P.n_layers + 1, cap = P.cap;
    __shared__ int s_n[kPlanMaxTensors];
    __shared__ dc_rect s_acc[2][kPlanMaxRects];
    const int mx = gmv[2 * stream], my = gmv[2 * stream + 1];
    const bool ext = ext_opt != 0 && mx == 0 && my == 0;
    dc_rect* const lists = P.rects + (size_t)stream * nt * cap;
    int32_t* const dxy = P.dxy + (size_t)stream * nt * 2;
    bool over = false;

    // ---- Step 5: lane r holds row r of the block grid as a bit string (gh, gw <= 64) ----
    unsigned long long open = 0;
    if (lane < gh) {
        const uint8_t* m = block_mask + ((size_t)stream * gh + lane) * gw;
        for (int bx = 0; bx < gw; ++bx)
            if (m[bx]) open |= 1ull << bx;
    }
    int reusable = __popcll(open);
    for (int off = 32; off > 0; off >>= 1) reusable += __shfl_xor(reusable, off);
    const PlanTensorDev t0 = P.tensors[0];
    int n0 = 0;
    for (int by0 = 0; by0 < gh; ++by0) {
        const int by = __builtin_amdgcn_readfirstlane(by0);
        for (;;) {
            const unsigned lo = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)open, by);
            const unsigned hi = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)(open >> 32), by);
            const unsigned long long row = ((unsigned long long)hi << 32) | lo;
            if (!row) break;
            const int bx = __ffsll((long long)row) - 1;
            const unsigned long long rest = ~(row >> bx);            // first zero = end of the run (the shift fills with zeros)
            const int run = rest ? __ffsll((long long)rest) - 1 : 64 - bx;
            const unsigned long long m = (run >= 64 ? ~0ull : ((1ull << run) - 1ull)) << bx;
            // rows below that hold the whole run open, counted from by + 1 without a gap
            const unsigned long long whole = __ballot((open & m) == m);
            const unsigned long long below = by + 1 < 64 ? ~(whole >> (by + 1)) : ~0ull;
            const int down = below ? __ffsll((long long)below) - 1 : 64 - (by + 1);
            const int y1 = by + 1 + down;
            if (lane >= by && lane < y1) open &= ~m;
            const SpanD xs = source_inside(SpanD{bx * B, (bx + run) * B}, mx, t0.w);
            const SpanD ys = source_inside(SpanD{by * B, y1 * B}, my, t0.h);
            if (!none(xs) && !none(ys)) {
                if (n0 < cap) {
                    if (lane == 0) lists[n0] = dc_rect{xs.lo, ys.lo, xs.hi - xs.lo, ys.hi - ys.lo};
                    ++n0;
                } else {
                    over = true;
                }
            }
        }
    }
    if (lane == 0) { s_n[0] = n0; dxy[0] = mx; dxy[1] = my; }
    __threadfence();
    __syncthreads();

    // ---- Table 2, layer by layer ----
    for (int i = 0; i < P.n_layers; ++i) {
        const PlanLayerDev L = P.layers[i];
        const PlanTensorDev ta = P.tensors[L.in0], tt = P.tensors[i + 1];
        const int dx = round_half_away(mx, tt.cum_stride), dy = round_half_away(my, tt.cum_stride);
        const dc_rect* la = lists + (size_t)L.in0 * cap;
        dc_rect* lt = lists + (size_t)(i + 1) * cap;
        const int na = s_n[L.in0];
        int n_out = 0;
        const bool windowed = L.type == DC_CONV || L.type == DC_MAXPOOL || L.type == DC_AVGPOOL;
        if (L.type == DC_FC || L.type == DC_SOFTMAX) {
            // every output depends on every input: nothing is reusable from here on
        } else if (L.type == DC_ADD) {
            const dc_rect* lb = lists + (size_t)L.in1 * cap;
            const int nb = s_n[L.in1];
            for (int ia = 0; ia < na; ++ia) {
                const dc_rect ra = load_rect(la + ia);
                for (int base = 0; base < nb; base += 64) {
                    const int ib = base + lane;
                    bool ok = ib < nb;
                    const dc_rect rb = ok ? load_rect(lb + ib) : dc_rect{0, 0, 0, 0};
                    SpanD xs = both(SpanD{ra.x, ra.x + ra.w}, SpanD{rb.x, rb.x + rb.w});
                    SpanD ys = both(SpanD{ra.y, ra.y + ra.h}, SpanD{rb.y, rb.y + rb.h});
                    ok = ok && !none(xs) && !none(ys);
                    xs = source_inside(xs, dx, tt.w); ys = source_inside(ys, dy, tt.h);
                    ok = ok && !none(xs) && !none(ys);
                    n_out = append(lt, n_out, cap, ok, xs, ys, lane, over);
                }
            }
        } else if (L.type == DC_CONCAT) {
            // overlaps of the first two lists, then of those with the third, ...: the tuples (i0, i1, ..) with the
            // last index fastest; clipped at the end
            const int ids[4] = {L.in0, L.in1, L.in2, L.in3};
            int m = 2;
            while (m < 4 && ids[m] >= 0) ++m;
            int cur = 0, n_acc = na < kPlanMaxRects ? na : kPlanMaxRects;
            for (int j = lane; j < n_acc; j += 64) s_acc[0][j] = load_rect(la + j);
            __syncthreads();
            for (int j = 1; j < m; ++j) {
                const dc_rect* lb = lists + (size_t)ids[j] * cap;
                const int nb = s_n[ids[j]];
                int nn = 0;
                for (int ia = 0; ia < n_acc; ++ia) {
                    const dc_rect ra = s_acc[cur][ia];
                    for (int base = 0; base < nb; base += 64) {
                        const int ib = base + lane;
                        bool ok = ib < nb;
                        const dc_rect rb = ok ? load_rect(lb + ib) : dc_rect{0, 0, 0, 0};
                        const SpanD xs = both(SpanD{ra.x, ra.x + ra.w}, SpanD{rb.x, rb.x + rb.w});
                        const SpanD ys = both(SpanD{ra.y, ra.y + ra.h}, SpanD{rb.y, rb.y + rb.h});
                        ok = ok && !none(xs) && !none(ys);
                        nn = append(s_acc[cur ^ 1], nn, kPlanMaxRects, ok, xs, ys, lane, over);
                    }
                }
                __syncthreads();
                cur ^= 1;
                n_acc = nn;
            }
            for (int base = 0; base < n_acc; base += 64) {
                const int ia = base + lane;
                bool ok = ia < n_acc;
                const dc_rect r = ok ? s_acc[cur][ia] : dc_rect{0, 0, 0, 0};
                const SpanD xs = source_inside(SpanD{r.x, r.x + r.w}, dx, tt.w);
                const SpanD ys = source_inside(SpanD{r.y, r.y + r.h}, dy, tt.h);
                ok = ok && !none(xs) && !none(ys);
                n_out = append(lt, n_out, cap, ok, xs, ys, lane, over);
            }
        } else {
            const int radius = (L.k - 1) / 2;
            const bool lrn_px = L.type == DC_LRN && L.within != 0;
            for (int base = 0; base < na; base += 64) {
                const int ia = base + lane;
                bool ok = ia < na;
                const dc_rect r = ok ? load_rect(la + ia) : dc_rect{0, 0, 0, 0};
                SpanD xs{r.x, r.x + r.w}, ys{r.y, r.y + r.h};
                if (windowed) {
                    xs = ext ? windows_inside_ext(xs, L.k, L.s, L.p, ta.w) : windows_inside(xs, L.k, L.s, L.p);
                    ys = ext ? windows_inside_ext(ys, L.k, L.s, L.p, ta.h) : windows_inside(ys, L.k, L.s, L.p);
                } else if (lrn_px) {
                    if (ext) {
                        xs = windows_inside_ext(xs, L.k, 1, radius, ta.w);
                        ys = windows_inside_ext(ys, L.k, 1, radius, ta.h);
                    } else {
                        xs = SpanD{r.x + radius, r.x + r.w - radius};
                        ys = SpanD{r.y + radius, r.y + r.h - radius};
                    }
                }
                ok = ok && !none(xs) && !none(ys);
                xs = source_inside(xs, dx, tt.w); ys = source_inside(ys, dy, tt.h);
                ok = ok && !none(xs) && !none(ys);
                n_out = append(lt, n_out, cap, ok, xs, ys, lane, over);
            }
        }
        __threadfence();
        __syncthreads();
        if (lane == 0) { s_n[i + 1] = n_out; dxy[2 * (i + 1)] = dx; dxy[2 * (i + 1) + 1] = dy; }
        __syncthreads();
    }
    // a stream one of whose lists did not fit reuses nothing in this frame
    for (int t = lane; t < nt; t += 64) P.nrect[(size_t)stream * nt + t] = over ? 0 : s_n[t];
    if (lane == 0) { P.stream_info[2 * stream] = reusable; P.stream_info[2 * stream + 1] = over ? 1 : 0; }
}

// sums v over the workgroup (256 threads); the result is valid in every thread
__device__ __forceinline__ long long block_sum(long long v, long long* s_tmp) {
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) s_tmp[threadIdx.x >> 6] = v;
    __syncthreads();
    return s_tmp[0] + s_tmp[1] + s_tmp[2] + s_tmp[3];
}

__device__ __forceinline__ unsigned inside_mask(int Hout, int Wout, int ty, int tx) {
    const int hh = Hout - ty * 4 < 4 ? Hout - ty * 4 : 4, ww = Wout - tx * 4 < 4 ? Wout - tx * 4 : 4;
    const unsigned rows = 0x1111u & ((1u << (4 * hh)) - 1u);
    return rows * ((1u << ww) - 1u);
}

__global__ __launch_bounds__(kPlanChunk) void plan_masks_kernel(PlanDev P) {
    const int chunk = blockIdx.x, stream = blockIdx.y, c = blockIdx.z, tid = threadIdx.x;
    const PlanConvDev cv = P.convs[c];
    if (chunk >= cv.n_chunks) return;
    const int nt = P.n_layers + 1;
    __shared__ dc_rect s_r[kPlanMaxRects];
    __shared__ long long s_tmp[4];
    const int n = P.nrect[(size_t)stream * nt + cv.tensor];
    const dc_rect* list = P.rects + ((size_t)stream * nt + cv.tensor) * P.cap;
    for (int i = tid; i < n; i += kPlanChunk) s_r[i] = list[i];
    __syncthreads();
    const int units = cv.units_x * cv.units_y;
    const int u = chunk * kPlanChunk + tid;
    unsigned mask = 0;
    int dirty = 0;
    if (u < units) {
        const int ty = u / cv.units_x, tx = u - ty * cv.units_x;
        const int x0 = tx * 4, y0 = ty * 4;
        for (int r = 0; r < n; ++r) {
            const dc_rect q = s_r[r];
            const int xa = (q.x > x0 ? q.x : x0) - x0, xb = (q.x + q.w < x0 + 4 ? q.x + q.w : x0 + 4) - x0;
            const int ya = (q.y > y0 ? q.y : y0) - y0, yb = (q.y + q.h < y0 + 4 ? q.y + q.h : y0 + 4) - y0;
            if (xa < xb && ya < yb) {
                const unsigned cols = ((1u << xb) - 1u) & ~((1u << xa) - 1u);
                const unsigned rows = ((0x1111u << (4 * ya)) & 0xffffu) & ((1u << (4 * yb)) - 1u);
                mask |= rows * cols;
            }
        }
        const unsigned inside = inside_mask(cv.Hout, cv.Wout, ty, tx);
        dirty = (mask & inside) != inside ? 1 : 0;
        reinterpret_cast<uint16_t*>(P.area + cv.umask_off)[(size_t)stream * units + u] = (uint16_t)mask;
    }
    // (dirty units, reused pixels) of this chunk in one sum
    const long long both_sums = block_sum(((long long)dirty << 32) | (long long)__popc(mask), s_tmp);
    if (tid == 0) {
        int32_t* cnt = reinterpret_cast<int32_t*>(P.area + cv.count_off) + ((size_t)stream * cv.n_chunks + chunk) * 2;
        cnt[0] = (int32_t)(both_sums >> 32);
        cnt[1] = (int32_t)(both_sums & 0xffffffffll);
    }
}

__global__ __launch_bounds__(kPlanChunk) void plan_lists_kernel(PlanDev P) {
    const int chunk = blockIdx.x, stream = blockIdx.y, c = blockIdx.z, tid = threadIdx.x;
    const PlanConvDev cv = P.convs[c];
    if (chunk >= cv.n_chunks) return;
    __shared__ long long s_tmp[4];
    __shared__ int s_wave[4];
    const int32_t* cnt = reinterpret_cast<const int32_t*>(P.area + cv.count_off);
    const int me = stream * cv.n_chunks + chunk, all = P.n_streams * cv.n_chunks;
    const bool last = me == all - 1;
    // units listed before this chunk's (stream-major, then raster order); the last chunk also totals the layer
    long long before = 0, reused = 0;
    for (int i = tid; i < all; i += kPlanChunk) {
        if (i < me) before += cnt[2 * i];
        if (last) reused += cnt[2 * i + 1];
    }
    before = block_sum(before, s_tmp);
    if (last) reused = block_sum(reused, s_tmp);
    const int units = cv.units_x * cv.units_y;
    const int u = chunk * kPlanChunk + tid;
    unsigned mask = 0;
    bool dirty = false;
    int ty = 0, tx = 0;
    if (u < units) {
        ty = u / cv.units_x; tx = u - ty * cv.units_x;
        mask = reinterpret_cast<const uint16_t*>(P.area + cv.umask_off)[(size_t)stream * units + u];
        const unsigned inside = inside_mask(cv.Hout, cv.Wout, ty, tx);
        dirty = (mask & inside) != inside;
    }
    const unsigned long long b = __ballot(dirty);
    const int lane = tid & 63, wave = tid >> 6;
    if (lane == 0) s_wave[wave] = __popcll(b);
    __syncthreads();
    int pos = (int)before + __popcll(b & ((1ull << lane) - 1ull));
    for (int w = 0; w < wave; ++w) pos += s_wave[w];
    if (dirty) reinterpret_cast<TileDev*>(P.area + cv.list_off)[pos] = TileDev{stream, ty, tx, (int32_t)mask};
    if (last && tid == 0) {
        const int total = (int)before + s_wave[0] + s_wave[1] + s_wave[2] + s_wave[3];
        P.n_units[c] = total;
        PlanStatsConv* sc = reinterpret_cast<PlanStatsConv*>(static_cast<unsigned char*>(P.stats) + sizeof(PlanStatsHead)) + c;
        sc->reused_px = reused; sc->n_units = total; sc->pad = 0;
        if (c == 0) {
            int blocks = 0, overflow = 0;
            for (int s = 0; s < P.n_streams; ++s) { blocks += P.stream_info[2 * s]; overflow += P.stream_info[2 * s + 1]; }
            PlanStatsHead* sh = static_cast<PlanStatsHead*>(P.stats);
            sh->n_reusable_blocks = blocks; sh->n_overflow_streams = overflow; sh->pad0 = 0; sh->pad1 = 0;
        }
    }
}

struct CopyUnitsArgs {
    CopyUnitsLayer L[kCopyUnitsMaxLayers];
    const int32_t* dxy;
    int32_t n_tensors, pad;
};

// Section 5 "Reuse", step 1, from the unit masks: every pixel whose bit is set receives the previous frame's
// value at +(dx, dy).  A workgroup takes 16 units of one stream and layer; consecutive threads take consecutive
// vectors of a pixel, then the next pixel of the unit's row (contiguous in memory), four items per thread in flight.
template <typename V>
__global__ __launch_bounds__(256) void shifted_copy_units_kernel(CopyUnitsArgs A) {
    const CopyUnitsLayer& L = A.L[blockIdx.z];
    const int stream = blockIdx.y, tid = threadIdx.x;
    const int units = L.units_x * L.units_y, u0 = blockIdx.x * 16;
    if (u0 >= units) return;
    __shared__ unsigned short s_m[16];
    __shared__ int s_any;
    if (tid == 0) s_any = 0;
    __syncthreads();
    if (tid < 16) {
        const unsigned short m = u0 + tid < units ? L.umask[(size_t)stream * units + u0 + tid] : (unsigned short)0;
        s_m[tid] = m;
        if (m) s_any = 1;
    }
    __syncthreads();
    if (!s_any) return;
    const int dx = A.dxy[((size_t)stream * A.n_tensors + L.tensor) * 2], dy = A.dxy[((size_t)stream * A.n_tensors + L.tensor) * 2 + 1];
    const int pv = L.vec_per_px, per_unit = 16 * pv, total = 16 * per_unit;
    const V* __restrict__ prev = static_cast<const V*>(L.prev);
    V* __restrict__ out = static_cast<V*>(L.out);
    const size_t map = (size_t)stream * L.Hout * L.Wout;
    for (int i0 = tid; i0 < total; i0 += 4 * 256) {
        V val[4];
        size_t dst[4];
        bool on[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int i = i0 + j * 256;
            const int unit = i / per_unit, rem = i - unit * per_unit;
            const int px = rem / pv, v = rem - px * pv;
            on[j] = i < total && ((s_m[unit & 15] >> px) & 1);
            const int u = u0 + unit, ty = u / L.units_x, tx = u - ty * L.units_x;
            const int y = ty * 4 + (px >> 2), x = tx * 4 + (px & 3);
            dst[j] = (map + (size_t)y * L.Wout + x) * pv + v;
            if (on[j]) val[j] = prev[(map + (size_t)(y + dy) * L.Wout + (x + dx)) * pv + v];
        }
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (on[j]) out[dst[j]] = val[j];
    }
}

}  // namespace

hipError_t launch_plan(const PlanDev& P, const uint8_t* block_mask, const int32_t* gmv, int gh, int gw, int block,
                       int extend_borders, int max_chunks, hipStream_t st) {
    if (gh > 64 || gw > 64 || P.n_layers + 1 > kPlanMaxTensors || P.cap > kPlanMaxRects || P.cap < 1) return hipErrorInvalidValue;
    hipLaunchKernelGGL(plan_regions_kernel, dim3(P.n_streams), dim3(64), 0, st, P, block_mask, gmv, gh, gw, block, extend_borders);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || P.n_convs == 0) return e;
    const dim3 grid((unsigned)max_chunks, (unsigned)P.n_streams, (unsigned)P.n_convs);
    hipLaunchKernelGGL(plan_masks_kernel, grid, dim3(kPlanChunk), 0, st, P);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(plan_lists_kernel, grid, dim3(kPlanChunk), 0, st, P);
    return hipGetLastError();
}

hipError_t launch_shifted_copy_units(const CopyUnitsLayer* layers, int n_layers, const int32_t* dxy, int n_tensors,
                                     int n_streams, int vec_bytes, hipStream_t st) {
    for (int l0 = 0; l0 < n_layers; l0 += kCopyUnitsMaxLayers) {
        const int nl = n_layers - l0 < kCopyUnitsMaxLayers ? n_layers - l0 : kCopyUnitsMaxLayers;
        CopyUnitsArgs A{};
        int max_groups = 0;
        for (int i = 0; i < nl; ++i) {
            A.L[i] = layers[l0 + i];
            const int groups = (A.L[i].units_x * A.L[i].units_y + 15) / 16;
            max_groups = groups > max_groups ? groups : max_groups;
        }
        A.dxy = dxy; A.n_tensors = n_tensors;
        const dim3 grid((unsigned)max_groups, (unsigned)n_streams, (unsigned)nl);
        if (vec_bytes == 16) hipLaunchKernelGGL(shifted_copy_units_kernel<uint4>, grid, dim3(256), 0, st, A);
        else if (vec_bytes == 4) hipLaunchKernelGGL(shifted_copy_units_kernel<uint32_t>, grid, dim3(256), 0, st, A);
        else hipLaunchKernelGGL(shifted_copy_units_kernel<uint16_t>, grid, dim3(256), 0, st, A);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace dc
