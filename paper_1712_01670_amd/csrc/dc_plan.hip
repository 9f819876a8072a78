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
#include <atomic>

#include "dc_internal.h"

namespace dc {

namespace {

struct SpanD { int lo, hi; };   // half-open [lo, hi)

// floor(a / b), b > 0.  Strides are 1, 2 or 4 in every stack at hand: those divide by shifting (an arithmetic shift
// rounds towards minus infinity), which keeps the integer division out of the layer loop's dependency chain.
__device__ __forceinline__ int floor_div(int a, int b) {
    if (b == 1) return a;
    if ((b & (b - 1)) == 0) return a >> (__ffs(b) - 1);
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
// num / den rounded to nearest, halves away from zero (|num| and den are far below 2^30)
__device__ __forceinline__ int round_half_away(int num, int den) {
    const unsigned mag = (unsigned)(num < 0 ? -num : num);
    const unsigned q = (unsigned)floor_div((int)(2u * mag + (unsigned)den), 2 * den);
    return num < 0 ? -(int)q : (int)q;
}

// Whether tensor t (the output of a layer of this type) lies on a torus.
__device__ __forceinline__ bool torus_tensor(const PlanDev& P, int t, int producer_type) {
    return t > 0 && (producer_type == DC_CONV || (P.pool_torus && producer_type == DC_MAXPOOL));
}
// The torus origin of tensor t of a stream for this frame (see PlanDev): a tensor on a torus moves by its offset.
__device__ __forceinline__ void write_origin(const PlanDev& P, int stream, int nt, int t, bool conv_output, int dx, int dy, int w, int h) {
    const size_t at = ((size_t)stream * nt + t) * 2;
    int ox = 0, oy = 0;
    if (conv_output) {
        ox = ((P.origin_prev ? P.origin_prev[at] : 0) + dx) % w;
        oy = ((P.origin_prev ? P.origin_prev[at + 1] : 0) + dy) % h;
        if (ox < 0) ox += w;
        if (oy < 0) oy += h;
    }
    P.origin[at] = ox;
    P.origin[at + 1] = oy;
}

// Appends the rectangles (xs, ys) of the lanes with `ok` to `list` (LDS) in lane order; returns the new length.
// `room` is what the list may hold (the per-list bound, or what is left of the pool).
__device__ __forceinline__ int append(dc_rect* list, int n, int room, bool ok, SpanD xs, SpanD ys, int lane, bool& over) {
    const unsigned long long b = __ballot(ok);
    const int pos = n + __popcll(b & ((1ull << lane) - 1ull));
    if (ok && pos < room) list[pos] = dc_rect{xs.lo, ys.lo, xs.hi - xs.lo, ys.hi - ys.lo};
    n += __popcll(b);
    if (n > room) { over = true; n = room; }
    return n;
}

// One wavefront per stream.  All lists live in LDS while the stream is planned (a pool that the lists of the
// tensors share, filled front to back: a list is complete before the next one starts, and a layer only reads the
// lists of earlier tensors); every finished list is also written to its place in device memory for the kernels
// that follow.  A stream whose lists do not fit (one list beyond `cap`, or all of them beyond the pool) reuses
// nothing in this frame.
__global__ __launch_bounds__(64) void plan_regions_kernel(PlanDev P, const uint8_t* __restrict__ block_mask,
                                                          const int32_t* __restrict__ gmv, int gh, int gw, int B, int ext_opt,
                                                          int pool_rects) {
    const int stream = blockIdx.x, lane = threadIdx.x;
    const int nt = P.n_layers + 1, cap = P.cap;
    __shared__ int s_n[kPlanMaxTensors], s_off[kPlanMaxTensors], s_dxy[2 * kPlanMaxTensors];
    __shared__ unsigned long long s_flat[66];      // the block mask as one bit string, 64 blocks per word
    __shared__ dc_rect s_acc[2][kPlanMaxRects];
    // the layer and tensor tables, fetched once: read from memory inside the layer loop, every layer would wait for
    // two dependent loads
    __shared__ PlanLayerDev s_layers[kPlanMaxTensors];
    __shared__ PlanTensorDev s_tensors[kPlanMaxTensors];
    extern __shared__ __align__(16) unsigned char s_dyn[];
    dc_rect* const pool = reinterpret_cast<dc_rect*>(s_dyn);
    {
        const uint4* src = reinterpret_cast<const uint4*>(P.layers);
        uint4* dst = reinterpret_cast<uint4*>(s_layers);
        for (int j = lane; j < P.n_layers * 3; j += 64) dst[j] = src[j];          // 48 bytes per layer
        const uint4* tsrc = reinterpret_cast<const uint4*>(P.tensors);
        uint4* tdst = reinterpret_cast<uint4*>(s_tensors);
        for (int j = lane; j <= P.n_layers; j += 64) tdst[j] = tsrc[j];           // 16 bytes per tensor
    }
    const int mx = gmv[2 * stream], my = gmv[2 * stream + 1];
    const bool ext = ext_opt != 0 && mx == 0 && my == 0;
    bool over = false;
    int top = 0;                                   // rectangles of the pool in use (wavefront-uniform)

    // ---- Step 5: lane r holds row r of the block grid as a bit string (gh, gw <= 64) ----
    // (the mask bytes are read 64 at a time, one per lane, four loads in flight; lane r then cuts its gw bits out)
    unsigned long long open = 0;
    {
        const uint8_t* m = block_mask + (size_t)stream * gh * gw;
        const int nb = gh * gw;
        for (int j0 = 0; j0 < nb; j0 += 256) {
            uint8_t v[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int at = j0 + q * 64 + lane;
                v[q] = m[at < nb ? at : 0];
            }
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int at = j0 + q * 64 + lane;
                const unsigned long long bits = __ballot(at < nb && v[q] != 0);
                if (lane == 0 && j0 + q * 64 < nb + 64) s_flat[(j0 >> 6) + q] = bits;
            }
        }
        __syncthreads();
        if (lane < gh) {
            const int off = lane * gw, w = off >> 6, sh = off & 63;
            unsigned long long bits = s_flat[w] >> sh;
            if (sh) bits |= s_flat[w + 1] << (64 - sh);
            open = gw >= 64 ? bits : bits & ((1ull << gw) - 1ull);
        }
    }
    int reusable = __popcll(open);
    for (int off = 32; off > 0; off >>= 1) reusable += __shfl_xor(reusable, off);
    __syncthreads();
    const PlanTensorDev t0 = s_tensors[0];
    int n0 = 0;
    const int room0 = cap < pool_rects ? cap : pool_rects;
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
                if (n0 < room0) {
                    if (lane == 0) pool[n0] = dc_rect{xs.lo, ys.lo, xs.hi - xs.lo, ys.hi - ys.lo};
                    ++n0;
                } else {
                    over = true;
                }
            }
        }
    }
    if (lane == 0) { s_n[0] = n0; s_off[0] = 0; s_dxy[0] = mx; s_dxy[1] = my; }
    top = n0;
    __syncthreads();

    // ---- Table 2, layer by layer ----
    for (int i = 0; i < P.n_layers; ++i) {
        const PlanLayerDev L = s_layers[i];
        const PlanTensorDev ta = s_tensors[L.in0], tt = s_tensors[i + 1];
        const int dx = round_half_away(mx, tt.cum_stride), dy = round_half_away(my, tt.cum_stride);
        const dc_rect* la = pool + s_off[L.in0];
        dc_rect* lt = pool + top;
        const int room = cap < pool_rects - top ? cap : pool_rects - top;
        const int na = s_n[L.in0];
        int n_out = 0;
        const bool windowed = L.type == DC_CONV || L.type == DC_MAXPOOL || L.type == DC_AVGPOOL;
        if (L.type == DC_FC || L.type == DC_SOFTMAX) {
            // every output depends on every input: nothing is reusable from here on
        } else if (L.type == DC_ADD) {
            const dc_rect* lb = pool + s_off[L.in1];
            const int nb = s_n[L.in1];
            for (int ia = 0; ia < na; ++ia) {
                const dc_rect ra = la[ia];
                for (int base = 0; base < nb; base += 64) {
                    const int ib = base + lane;
                    bool ok = ib < nb;
                    const dc_rect rb = ok ? lb[ib] : dc_rect{0, 0, 0, 0};
                    SpanD xs = both(SpanD{ra.x, ra.x + ra.w}, SpanD{rb.x, rb.x + rb.w});
                    SpanD ys = both(SpanD{ra.y, ra.y + ra.h}, SpanD{rb.y, rb.y + rb.h});
                    ok = ok && !none(xs) && !none(ys);
                    xs = source_inside(xs, dx, tt.w); ys = source_inside(ys, dy, tt.h);
                    ok = ok && !none(xs) && !none(ys);
                    n_out = append(lt, n_out, room, ok, xs, ys, lane, over);
                }
            }
        } else if (L.type == DC_CONCAT) {
            // overlaps of the first two lists, then of those with the third, ...: the tuples (i0, i1, ..) with the
            // last index fastest; clipped at the end
            const int ids[4] = {L.in0, L.in1, L.in2, L.in3};
            int m = 2;
            while (m < 4 && ids[m] >= 0) ++m;
            int cur = 0, n_acc = na < kPlanMaxRects ? na : kPlanMaxRects;
            for (int j = lane; j < n_acc; j += 64) s_acc[0][j] = la[j];
            __syncthreads();
            for (int j = 1; j < m; ++j) {
                const dc_rect* lb = pool + s_off[ids[j]];
                const int nb = s_n[ids[j]];
                int nn = 0;
                for (int ia = 0; ia < n_acc; ++ia) {
                    const dc_rect ra = s_acc[cur][ia];
                    for (int base = 0; base < nb; base += 64) {
                        const int ib = base + lane;
                        bool ok = ib < nb;
                        const dc_rect rb = ok ? lb[ib] : dc_rect{0, 0, 0, 0};
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
                n_out = append(lt, n_out, room, ok, xs, ys, lane, over);
            }
        } else {
            const int radius = (L.k - 1) / 2;
            const bool lrn_px = L.type == DC_LRN && L.within != 0;
            for (int base = 0; base < na; base += 64) {
                const int ia = base + lane;
                bool ok = ia < na;
                const dc_rect r = ok ? la[ia] : dc_rect{0, 0, 0, 0};
                SpanD xs{r.x, r.x + r.w}, ys{r.y, r.y + r.h};
                if (windowed) {          // the kernel's span per axis (a conv kernel may be not square, or dilated)
                    const int ew = (L.kw - 1) * L.dil + 1, eh = (L.k - 1) * L.dil + 1;
                    xs = ext ? windows_inside_ext(xs, ew, L.s, L.pw, ta.w) : windows_inside(xs, ew, L.s, L.pw);
                    ys = ext ? windows_inside_ext(ys, eh, L.s, L.p, ta.h) : windows_inside(ys, eh, L.s, L.p);
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
                n_out = append(lt, n_out, room, ok, xs, ys, lane, over);
            }
        }
        if (lane == 0) { s_n[i + 1] = n_out; s_off[i + 1] = top; s_dxy[2 * (i + 1)] = dx; s_dxy[2 * (i + 1) + 1] = dy; }
        __syncthreads();                               // the list is complete in LDS: later layers read it
        top += n_out;
    }
    // Everything goes to device memory at the end, in one pass without a barrier (a store inside the layer loop would
    // be waited for at the next barrier).  A stream one of whose lists did not fit reuses nothing in this frame.
    dc_rect* const lists = P.rects + (size_t)stream * nt * cap;
    for (int t = 0; t < nt && !over; ++t) {
        const dc_rect* src = pool + s_off[t];
        dc_rect* out = lists + (size_t)t * cap;
        for (int j = lane; j < s_n[t]; j += 64) out[j] = src[j];
    }
    for (int t = lane; t < 2 * nt; t += 64) P.dxy[(size_t)stream * nt * 2 + t] = s_dxy[t];
    if (P.origin)
        for (int t = lane; t < nt; t += 64) write_origin(P, stream, nt, t, torus_tensor(P, t, t > 0 ? s_layers[t - 1].type : -1), s_dxy[2 * t], s_dxy[2 * t + 1],
                                                          s_tensors[t].w, s_tensors[t].h);
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

// ---- exact reuse maps -------------------------------------------------------------------------------------
constexpr int kErodeThreads = 1024;
constexpr int kErodeLdsWords = 32 * 1024;      // bitmaps of one stream up to this size (128 KB) stay in LDS

// word i of a bitmap row of w pixels; words outside the row, and bits beyond w, read as `outside`;
// row == nullptr: the whole row lies outside the map
__device__ __forceinline__ unsigned row_word(const uint32_t* row, int wpr, int w, int i, bool outside) {
    unsigned x = outside ? ~0u : 0u;
    if (row && i >= 0 && i < wpr) {
        x = row[i];
        const int valid = w - 32 * i;                      // bits of this word that lie inside the row
        if (outside && valid < 32) x |= ~0u << valid;
    }
    return x;
}
// even bits of x packed into the low half
__device__ __forceinline__ unsigned even_bits(unsigned long long x) {
    x &= 0x5555555555555555ull;
    x = (x | (x >> 1)) & 0x3333333333333333ull;
    x = (x | (x >> 2)) & 0x0f0f0f0f0f0f0f0full;
    x = (x | (x >> 4)) & 0x00ff00ff00ff00ffull;
    x = (x | (x >> 8)) & 0x0000ffff0000ffffull;
    x = (x | (x >> 16)) & 0x00000000ffffffffull;
    return (unsigned)x;
}
// bits [lo, hi) of a 32-bit word that starts at pixel column x0
__device__ __forceinline__ unsigned column_range(int x0, int lo, int hi) {
    const int a = lo - x0 < 0 ? 0 : lo - x0, b = hi - x0 > 32 ? 32 : hi - x0;
    if (b <= a) return 0u;
    const unsigned upto_b = b >= 32 ? ~0u : ((1u << b) - 1u);
    return upto_b & ~((1u << a) - 1u);
}

// The maps of one stream, tensor after tensor (a barrier in between: a layer reads the bitmaps of earlier tensors).
// Every thread computes whole 32-pixel words of the output bitmap:
//   windowed layers (conv, pooling, LRN over pixels)  AND over the k x k window, word-parallel for strides 1 and 2
//     (the k shifted copies of an input row are ANDed, for stride 2 every second bit is kept), bit by bit otherwise;
//     taps outside the map read 0, or 1 for a stream that did not move when the border case is on;
//   add / concat  AND of the inputs;   FC / softmax  nothing;   others  a copy;
// and every tensor is cut to the pixels whose source at +(dx, dy) lies inside the map.
// `maps` is the stream's bitmap area: LDS when it fits (a layer is a few LDS round trips then, not a few trips to
// the L2), the workspace otherwise.
__device__ __forceinline__ void erode_stream(uint32_t* maps, const PlanLayerDev* s_layers, const PlanTensorDev* s_tensors,
                                             int n_layers, int32_t* dxy, const uint8_t* m, int gh, int gw, int B, int mx, int my,
                                             bool ext, int tid) {
    {   // tensor 0: the pixels of the blocks that passed Step 4
        const PlanTensorDev t0 = s_tensors[0];
        const int wpr = (t0.w + 31) >> 5;
        const int col_lo = -mx < 0 ? 0 : -mx, col_hi = t0.w - mx < t0.w ? t0.w - mx : t0.w;
        for (int i = tid; i < t0.h * wpr; i += kErodeThreads) {
            const int y = i / wpr, x0 = (i - y * wpr) * 32;
            const int by = y / B;
            unsigned bits = 0;
            if (by < gh && y + my >= 0 && y + my < t0.h) {
                const int bx_hi = (x0 + 31) / B < gw - 1 ? (x0 + 31) / B : gw - 1;
                for (int bx = x0 / B; bx <= bx_hi; ++bx)
                    if (m[by * gw + bx]) bits |= column_range(x0, bx * B, bx * B + B);
            }
            maps[t0.bm_off + i] = bits & column_range(x0, col_lo, col_hi);
        }
    }
    __syncthreads();
    for (int li = 0; li < n_layers; ++li) {
        const PlanLayerDev L = s_layers[li];
        const PlanTensorDev ta = s_tensors[L.in0], tt = s_tensors[li + 1];
        const int dx = round_half_away(mx, tt.cum_stride), dy = round_half_away(my, tt.cum_stride);
        if (tid == 0) { dxy[2 * (li + 1)] = dx; dxy[2 * (li + 1) + 1] = dy; }
        const uint32_t* in = maps + ta.bm_off;
        uint32_t* out = maps + tt.bm_off;
        const int wpr_in = (ta.w + 31) >> 5, wpr = (tt.w + 31) >> 5;
        const bool windowed = L.type == DC_CONV || L.type == DC_MAXPOOL || L.type == DC_AVGPOOL;
        const bool lrn_px = L.type == DC_LRN && L.within != 0;
        // taps of the window: kh x kw, dil pixels apart, paddings ph / pw
        const int kh = (windowed || lrn_px) ? L.k : 1, kw = windowed ? L.kw : (lrn_px ? L.k : 1), dil = windowed ? L.dil : 1;
        const int s = windowed ? L.s : 1;
        const int ph = windowed ? L.p : (lrn_px ? (L.k - 1) / 2 : 0), pw = windowed ? L.pw : (lrn_px ? (L.k - 1) / 2 : 0);
        const int ew = (kw - 1) * dil + 1;
        const int col_lo = -dx < 0 ? 0 : -dx, col_hi = tt.w - dx < tt.w ? tt.w - dx : tt.w;
        for (int i = tid; i < tt.h * wpr; i += kErodeThreads) {
            const int y = i / wpr, x0 = (i - y * wpr) * 32;
            unsigned bits;
            if (L.type == DC_FC || L.type == DC_SOFTMAX) {
                bits = 0;
            } else if (L.type == DC_ADD) {
                bits = in[i] & maps[s_tensors[L.in1].bm_off + i];
            } else if (L.type == DC_CONCAT) {
                bits = in[i] & maps[s_tensors[L.in1].bm_off + i];
                if (L.in2 >= 0) bits &= maps[s_tensors[L.in2].bm_off + i];
                if (L.in2 >= 0 && L.in3 >= 0) bits &= maps[s_tensors[L.in3].bm_off + i];
            } else if (kh == 1 && kw == 1 && s == 1 && ph == 0 && pw == 0) {
                bits = in[i];
            } else if (s <= 2 && ew <= 32) {
                // bit b of acc: the whole window that starts at input column c0 + b.  Stride 1 needs 32 + k - 1 input
                // columns from c0 (three words), stride 2 needs 64 + k - 1 (four).
                unsigned long long acc = ~0ull;
                const int c0 = x0 * s - pw;
                const int w0 = c0 >> 5, sh = c0 & 31;           // arithmetic shift: floor for negative starts
                for (int ky = 0; ky < kh; ++ky) {
                    const int iy = y * s - ph + ky * dil;
                    const bool row_in = iy >= 0 && iy < ta.h;
                    if (!row_in && ext) continue;               // taps in the padding are ignored
                    const uint32_t* row = row_in ? in + (size_t)iy * wpr_in : nullptr;
                    const unsigned v0 = row_word(row, wpr_in, ta.w, w0, ext), v1 = row_word(row, wpr_in, ta.w, w0 + 1, ext);
                    const unsigned v2 = row_word(row, wpr_in, ta.w, w0 + 2, ext);
                    const unsigned v3 = s == 2 ? row_word(row, wpr_in, ta.w, w0 + 3, ext) : 0u;
                    const unsigned long long a = ((unsigned long long)v1 << 32) | v0, b = ((unsigned long long)v3 << 32) | v2;
                    const unsigned long long lo = sh ? (a >> sh) | (b << (64 - sh)) : a;    // columns c0 .. c0 + 63
                    const unsigned long long hi = b >> sh;                                  // columns c0 + 64 .. (at least 33 of them)
                    unsigned long long r = lo;
                    for (int kx = 1; kx < kw; ++kx) r &= (lo >> (kx * dil)) | (hi << (64 - kx * dil));
                    acc &= r;
                }
                bits = s == 1 ? (unsigned)acc : even_bits(acc);
            } else if (s <= 8 && ew <= 32) {
                // larger strides: the same AND of shifted rows for all 32 s start columns of the word (up to four
                // 64-column pieces), then every s-th bit is kept
                unsigned long long acc[4] = {~0ull, ~0ull, ~0ull, ~0ull};
                const int c0 = x0 * s - pw;
                const int pieces = (32 * s + 63) >> 6;
                for (int ky = 0; ky < kh; ++ky) {
                    const int iy = y * s - ph + ky * dil;
                    const bool row_in = iy >= 0 && iy < ta.h;
                    if (!row_in && ext) continue;
                    const uint32_t* row = row_in ? in + (size_t)iy * wpr_in : nullptr;
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        if (j >= pieces) continue;
                        const int c = c0 + 64 * j, w0 = c >> 5, sh = c & 31;
                        unsigned v[5];
#pragma unroll
                        for (int q = 0; q < 5; ++q) v[q] = row_word(row, wpr_in, ta.w, w0 + q, ext);
                        const unsigned long long a = ((unsigned long long)v[1] << 32) | v[0], b = ((unsigned long long)v[3] << 32) | v[2];
                        const unsigned long long lo = sh ? (a >> sh) | (b << (64 - sh)) : a;
                        const unsigned long long hi = sh ? (b >> sh) | ((unsigned long long)v[4] << (64 - sh)) : b;
                        unsigned long long r = lo;
                        for (int kx = 1; kx < kw; ++kx) r &= (lo >> (kx * dil)) | (hi << (64 - kx * dil));
                        acc[j] &= r;
                    }
                }
                bits = 0;
                for (int b = 0; b < 32; ++b) {
                    const int at = b * s, piece = at >> 6;
                    const unsigned long long word = piece == 0 ? acc[0] : (piece == 1 ? acc[1] : (piece == 2 ? acc[2] : acc[3]));
                    bits |= (unsigned)((word >> (at & 63)) & 1ull) << b;
                }
            } else {                                        // anything else: bit by bit
                bits = 0;
                for (int b = 0; b < 32 && x0 + b < tt.w; ++b) {
                    bool ok = true;
                    for (int ky = 0; ky < kh && ok; ++ky)
                        for (int kx = 0; kx < kw && ok; ++kx) {
                            const int iy = y * s - ph + ky * dil, ix = (x0 + b) * s - pw + kx * dil;
                            if (iy < 0 || iy >= ta.h || ix < 0 || ix >= ta.w) { ok = ext; continue; }
                            ok = (in[(size_t)iy * wpr_in + (ix >> 5)] >> (ix & 31)) & 1u;
                        }
                    if (ok) bits |= 1u << b;
                }
            }
            const bool row_ok = y + dy >= 0 && y + dy < tt.h;
            out[i] = row_ok ? (bits & column_range(x0, col_lo, col_hi)) : 0u;
        }
        __syncthreads();
    }
}

// One workgroup per stream.  IN_LDS: the stream's bitmaps are built in dynamic LDS (bm_words words) and written to
// the workspace in one pass at the end.
template <bool IN_LDS>
__global__ __launch_bounds__(kErodeThreads) void plan_erode_kernel(PlanDev P, const uint8_t* __restrict__ block_mask,
                                                                   const int32_t* __restrict__ gmv, int gh, int gw, int B, int ext_opt) {
    const int stream = blockIdx.x, tid = threadIdx.x;
    const int nt = P.n_layers + 1;
    __shared__ PlanLayerDev s_layers[kPlanMaxTensors];
    __shared__ PlanTensorDev s_tensors[kPlanMaxTensors];
    __shared__ int s_cnt[kErodeThreads / 64];
    extern __shared__ uint32_t s_maps[];
    {
        const uint4* src = reinterpret_cast<const uint4*>(P.layers);
        uint4* dst = reinterpret_cast<uint4*>(s_layers);
        for (int j = tid; j < P.n_layers * 3; j += kErodeThreads) dst[j] = src[j];
        const uint4* tsrc = reinterpret_cast<const uint4*>(P.tensors);
        uint4* tdst = reinterpret_cast<uint4*>(s_tensors);
        for (int j = tid; j < nt; j += kErodeThreads) tdst[j] = tsrc[j];
    }
    const int mx = gmv[2 * stream], my = gmv[2 * stream + 1];
    const bool ext = ext_opt != 0 && mx == 0 && my == 0;
    uint32_t* const g_maps = P.bitmaps + (size_t)stream * P.bm_words;
    int32_t* const dxy = P.dxy + (size_t)stream * nt * 2;
    const uint8_t* m = block_mask + (size_t)stream * gh * gw;
    {   // the stream's number of reusable blocks
        int reusable = 0;
        for (int j = tid; j < gh * gw; j += kErodeThreads) reusable += m[j] ? 1 : 0;
        for (int off = 32; off > 0; off >>= 1) reusable += __shfl_xor(reusable, off);
        if ((tid & 63) == 0) s_cnt[tid >> 6] = reusable;
    }
    __syncthreads();
    if (tid == 0) {
        int total = 0;
        for (int j = 0; j < kErodeThreads / 64; ++j) total += s_cnt[j];
        P.stream_info[2 * stream] = total; P.stream_info[2 * stream + 1] = 0; dxy[0] = mx; dxy[1] = my;
    }
    if (IN_LDS) {
        erode_stream(s_maps, s_layers, s_tensors, P.n_layers, dxy, m, gh, gw, B, mx, my, ext, tid);
        for (int64_t j = tid; j < P.bm_words; j += kErodeThreads) g_maps[j] = s_maps[j];
    } else {
        erode_stream(g_maps, s_layers, s_tensors, P.n_layers, dxy, m, gh, gw, B, mx, my, ext, tid);
    }
    for (int t = tid; t < nt; t += kErodeThreads) P.nrect[(size_t)stream * nt + t] = 0;      // no rectangles in this mode
    if (P.origin) {
        __syncthreads();          // the offsets of all tensors are written
        for (int t = tid; t < nt; t += kErodeThreads)
            write_origin(P, stream, nt, t, torus_tensor(P, t, t > 0 ? s_layers[t - 1].type : -1), dxy[2 * t], dxy[2 * t + 1], s_tensors[t].w, s_tensors[t].h);
    }
}

// The 16-bit unit masks of every conv layer cut out of the bitmaps (grid and outputs as plan_masks_kernel).
__global__ __launch_bounds__(kPlanChunk) void plan_masks_exact_kernel(PlanDev P) {
    const int chunk = blockIdx.x, stream = blockIdx.y, c = blockIdx.z, tid = threadIdx.x;
    const PlanConvDev cv = P.convs[c];
    if (chunk >= cv.n_chunks) return;
    __shared__ long long s_tmp[4];
    const PlanTensorDev tt = P.tensors[cv.tensor];
    const uint32_t* map = P.bitmaps + (size_t)stream * P.bm_words + tt.bm_off;
    const int wpr = (cv.Wout + 31) >> 5;
    const int units = cv.units_x * cv.units_y;
    const int u = chunk * kPlanChunk + tid;
    unsigned mask = 0;
    int dirty = 0;
    if (u < units) {
        const int ty = u / cv.units_x, tx = u - ty * cv.units_x;
        const int x0 = tx * 4;                               // a unit's four columns lie in one word
        for (int r = 0; r < 4; ++r) {
            const int y = ty * 4 + r;
            if (y < cv.Hout) mask |= ((map[(size_t)y * wpr + (x0 >> 5)] >> (x0 & 31)) & 0xfu) << (4 * r);
        }
        if (cv.no_reuse) mask = 0;                           // a layer that does not use the cache
        const unsigned inside = inside_mask(cv.Hout, cv.Wout, ty, tx);
        dirty = (mask & inside) != inside ? 1 : 0;
        reinterpret_cast<uint16_t*>(P.area + cv.umask_off)[(size_t)stream * units + u] = (uint16_t)mask;
    }
    const long long both_sums = block_sum(((long long)dirty << 32) | (long long)__popc(mask), s_tmp);
    if (tid == 0) {
        int32_t* cnt = reinterpret_cast<int32_t*>(P.area + cv.count_off) + ((size_t)stream * cv.n_chunks + chunk) * 2;
        cnt[0] = (int32_t)(both_sums >> 32);
        cnt[1] = (int32_t)(both_sums & 0xffffffffll);
    }
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
        if (cv.no_reuse) mask = 0;                           // a layer that does not use the cache
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

constexpr int kCopyUnitsPerGroup = 64;     // most units a workgroup of the per-unit copy takes (a power of two)
struct CopyUnitsArgs {
    CopyUnitsLayer L[kCopyUnitsMaxLayers];
    const int32_t* dxy;
    int32_t n_tensors, pad;
};

// Section 5 "Reuse", step 1, from the unit masks: every pixel whose bit is set receives the previous frame's
// value at +(dx, dy).  A workgroup takes UPB consecutive units of one stream and layer (UPB chosen by the launcher so
// that a thread has about four 16-byte items); consecutive threads take consecutive vectors of a pixel, then the
// next pixel of the unit's row (contiguous in memory); the four items of a thread are loaded before any is stored.
template <typename V>
__global__ __launch_bounds__(256) void shifted_copy_units_kernel(CopyUnitsArgs A) {
    const CopyUnitsLayer& L = A.L[blockIdx.z];
    const int stream = blockIdx.y, tid = threadIdx.x;
    const int units = L.units_x * L.units_y, upb = L.units_per_group, u0 = blockIdx.x * upb;
    if (u0 >= units) return;
    __shared__ unsigned short s_m[kCopyUnitsPerGroup];
    __shared__ int s_px0[kCopyUnitsPerGroup];          // pixel index (within the stream's map) of the unit's first pixel
    __shared__ int s_any;
    if (tid == 0) s_any = 0;
    __syncthreads();
    if (tid < upb) {
        const int u = u0 + tid;
        const unsigned short m = u < units ? L.umask[(size_t)stream * units + u] : (unsigned short)0;
        const int ty = u / L.units_x, tx = u - ty * L.units_x;
        s_m[tid] = m;
        s_px0[tid] = ty * 4 * L.Wout + tx * 4;
        if (m) s_any = 1;
    }
    __syncthreads();
    if (!s_any) return;
    const size_t at = ((size_t)stream * A.n_tensors + L.tensor) * 2;
    const int dx = A.dxy[at], dy = A.dxy[at + 1];
    const int pv = L.vec_per_px, sh = L.vec_shift, total = upb * 16 * pv;
    const V* __restrict__ prev = static_cast<const V*>(L.prev) + (size_t)stream * L.Hout * L.Wout * pv;
    V* __restrict__ out = static_cast<V*>(L.out) + (size_t)stream * L.Hout * L.Wout * pv;
    const int shift_px = dy * L.Wout + dx;
    // where item i goes (element index in `out`), whether it is copied at all, and where it comes from (element 0
    // for an item that is off, so that the load is unconditional and the four loads of a turn go out together)
    auto locate = [&](int i, int& dst, bool& on) -> size_t {
        int pxi, v;                                    // pixel index over the group's units, vector within the pixel
        if (sh >= 0) { pxi = i >> sh; v = i & (pv - 1); }
        else { pxi = i / pv; v = i - pxi * pv; }
        const int unit = (pxi >> 4) & (kCopyUnitsPerGroup - 1), px = pxi & 15;
        on = i < total && ((s_m[unit] >> px) & 1);
        const int pix = s_px0[unit] + (px >> 2) * L.Wout + (px & 3);
        dst = pix * pv + v;
        return on ? (size_t)(pix + shift_px) * pv + v : (size_t)0;
    };
    for (int i0 = tid; i0 < total; i0 += 4 * 256) {
        int d0, d1, d2, d3;
        bool on0, on1, on2, on3;
        const size_t s0 = locate(i0, d0, on0), s1 = locate(i0 + 256, d1, on1), s2 = locate(i0 + 512, d2, on2),
                     s3 = locate(i0 + 768, d3, on3);
        const V v0 = prev[s0], v1 = prev[s1], v2 = prev[s2], v3 = prev[s3];
        if (on0) out[d0] = v0;
        if (on1) out[d1] = v1;
        if (on2) out[d2] = v2;
        if (on3) out[d3] = v3;
    }
}

}  // namespace

hipError_t launch_plan(const PlanDev& P, const uint8_t* block_mask, const int32_t* gmv, int gh, int gw, int block,
                       int extend_borders, int max_chunks, hipStream_t st) {
    if (gh > 64 || gw > 64 || P.n_layers + 1 > kPlanMaxTensors || P.cap > kPlanMaxRects || P.cap < 1) return hipErrorInvalidValue;
    // LDS pool of the lists of one stream: 48 rectangles per tensor on average, 16 KiB .. 112 KiB
    int pool_rects = (P.n_layers + 1) * 48;
    pool_rects = pool_rects < 1024 ? 1024 : (pool_rects > 7168 ? 7168 : pool_rects);
    const size_t lds = (size_t)pool_rects * sizeof(dc_rect);
    static std::atomic<bool> raised{false};
    if (lds > 48 * 1024 && !raised.load()) {
        hipError_t a = hipFuncSetAttribute(reinterpret_cast<const void*>(plan_regions_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, 7168 * (int)sizeof(dc_rect));
        if (a != hipSuccess) return a;
        raised.store(true);
    }
    hipLaunchKernelGGL(plan_regions_kernel, dim3(P.n_streams), dim3(64), lds, st, P, block_mask, gmv, gh, gw, block, extend_borders, pool_rects);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || P.n_convs == 0) return e;
    const dim3 grid((unsigned)max_chunks, (unsigned)P.n_streams, (unsigned)P.n_convs);
    hipLaunchKernelGGL(plan_masks_kernel, grid, dim3(kPlanChunk), 0, st, P);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(plan_lists_kernel, grid, dim3(kPlanChunk), 0, st, P);
    return hipGetLastError();
}

namespace {
__global__ __launch_bounds__(256) void plan_args_kernel(PlanDev P, PlanConvDev conv, PlanArgRects R) {
    const int tid = threadIdx.x;
    if (tid == 0) const_cast<PlanConvDev*>(P.convs)[0] = conv;
    for (int s = tid; s < P.n_streams; s += 256) {
        P.nrect[s] = R.first[s + 1] - R.first[s];
        P.dxy[2 * s] = R.dxy[s][0]; P.dxy[2 * s + 1] = R.dxy[s][1];
        P.stream_info[2 * s] = 0; P.stream_info[2 * s + 1] = 0;
    }
    for (int s = 0; s < P.n_streams; ++s)
        for (int j = R.first[s] + tid; j < R.first[s + 1]; j += 256) P.rects[(size_t)s * P.cap + (j - R.first[s])] = R.r[j];
}
}  // namespace

hipError_t launch_plan_from_args(const PlanDev& P, const PlanConvDev& conv, const PlanArgRects& R, hipStream_t st) {
    if (P.n_layers != 0 || P.n_convs != 1 || P.n_streams < 1 || P.n_streams > kArgMaxStreams || P.cap < 1 || P.cap > kPlanMaxRects)
        return hipErrorInvalidValue;
    hipLaunchKernelGGL(plan_args_kernel, dim3(1), dim3(256), 0, st, P, conv, R);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const dim3 grid((unsigned)conv.n_chunks, (unsigned)P.n_streams, 1);
    hipLaunchKernelGGL(plan_masks_kernel, grid, dim3(kPlanChunk), 0, st, P);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(plan_lists_kernel, grid, dim3(kPlanChunk), 0, st, P);
    return hipGetLastError();
}

hipError_t launch_plan_exact(const PlanDev& P, const uint8_t* block_mask, const int32_t* gmv, int gh, int gw, int block,
                             int extend_borders, int max_chunks, bool with_lists, hipStream_t st) {
    if (P.n_layers + 1 > kPlanMaxTensors || !P.bitmaps || gh < 1 || gw < 1) return hipErrorInvalidValue;
    hipError_t e;
    if (P.bm_words <= kErodeLdsWords) {
        static std::atomic<bool> raised{false};       // more than 64 KB of dynamic LDS has to be asked for once
        if (!raised.load(std::memory_order_acquire)) {
            e = hipFuncSetAttribute(reinterpret_cast<const void*>(&plan_erode_kernel<true>), hipFuncAttributeMaxDynamicSharedMemorySize,
                                    kErodeLdsWords * (int)sizeof(uint32_t));
            if (e != hipSuccess) return e;
            raised.store(true, std::memory_order_release);
        }
        hipLaunchKernelGGL(plan_erode_kernel<true>, dim3(P.n_streams), dim3(kErodeThreads), (size_t)P.bm_words * sizeof(uint32_t), st,
                           P, block_mask, gmv, gh, gw, block, extend_borders);
    } else {
        hipLaunchKernelGGL(plan_erode_kernel<false>, dim3(P.n_streams), dim3(kErodeThreads), 0, st, P, block_mask, gmv, gh, gw, block,
                           extend_borders);
    }
    e = hipGetLastError();
    if (e != hipSuccess || !with_lists || P.n_convs == 0) return e;
    const dim3 grid((unsigned)max_chunks, (unsigned)P.n_streams, (unsigned)P.n_convs);
    hipLaunchKernelGGL(plan_masks_exact_kernel, grid, dim3(kPlanChunk), 0, st, P);
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
            // about sixteen items (vectors) per thread: 4096 per workgroup, 16 * vec_per_px per unit
            const int pv = A.L[i].vec_per_px;
            int upb = 256 / (pv > 0 ? pv : 1);
            upb = upb < 1 ? 1 : (upb > kCopyUnitsPerGroup ? kCopyUnitsPerGroup : upb);
            A.L[i].units_per_group = upb;
            A.L[i].vec_shift = (pv & (pv - 1)) == 0 ? __builtin_ctz((unsigned)pv) : -1;
            const int groups = (A.L[i].units_x * A.L[i].units_y + upb - 1) / upb;
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
