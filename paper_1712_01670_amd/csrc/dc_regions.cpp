// Host integer logic: merging matched blocks into rectangles (Section 4, Step 5),
// propagating rectangles through the layer table (Section 5, Table 2) and sorting the
// output tiles of a conv layer into clean / mixed / dirty for the GEMM tile list.
#include <algorithm>
#include <cstring>
#include <atomic>
#include <condition_variable>
#include <mutex>
#include <thread>

#include "dc_internal.h"

namespace dc {

namespace {

struct Span {  // half-open interval [lo, hi)
    int lo, hi;
    bool empty() const { return hi <= lo; }
};

inline int fdiv(int a, int b) {  // floor(a / b), b > 0
    int q = a / b, r = a % b;
    return (r < 0) ? q - 1 : q;
}
inline int cdiv(int a, int b) { return fdiv(a + b - 1, b); }

// Outputs whose window [o*s-p, o*s-p+k) lies inside `in` (one axis of Table 2's conv/pool row).
inline Span window_span(Span in, int k, int s, int p) {
    return Span{cdiv(in.lo + p, s), fdiv(in.hi - k + p, s) + 1};
}

// The same for a stream that did not move, with the border case: taps in the zero padding read zeros in both
// frames, so a span that touches an end of the input axis [0, size_in) reaches, for this rule, beyond that end.
inline Span window_span_ext(Span in, int k, int s, int p, int size_in) {
    const int size_out = (size_in + 2 * p - k) / s + 1;
    const int lo = in.lo == 0 ? 0 : cdiv(in.lo + p, s);
    const int hi = in.hi == size_in ? size_out : std::min(fdiv(in.hi - k + p, s) + 1, size_out);
    return Span{lo, hi};
}

inline Span intersect(Span a, Span b) { return Span{std::max(a.lo, b.lo), std::min(a.hi, b.hi)}; }

// Part of `cur` whose source cur+d lies inside [0, size).
inline Span keep_source_inside(Span cur, int d, int size) {
    return intersect(intersect(cur, Span{0, size}), Span{-d, size - d});
}

inline int round_half_away(long long num, long long den) {
    long long mag = num < 0 ? -num : num;
    long long q = (2 * mag + den) / (2 * den);
    return (int)(num < 0 ? -q : q);
}

inline void push_clipped(std::vector<dc_rect>& out, Span xs, Span ys, const TensorRegions& t) {
    xs = keep_source_inside(xs, t.dx, t.w);
    ys = keep_source_inside(ys, t.dy, t.h);
    if (xs.empty() || ys.empty()) return;
    out.push_back(dc_rect{xs.lo, ys.lo, xs.hi - xs.lo, ys.hi - ys.lo});
}

}  // namespace

void merge_blocks(const uint8_t* mask, int gh, int gw, int B, std::vector<dc_rect>& out) {
    out.clear();
    std::vector<uint8_t> open(mask, mask + (size_t)gh * gw);  // set and not yet claimed
    for (int by = 0; by < gh; ++by) {
        for (int bx = 0; bx < gw; ++bx) {
            if (!open[by * gw + bx]) continue;
            int x1 = bx;
            while (x1 < gw && open[by * gw + x1]) ++x1;
            int y1 = by + 1;
            while (y1 < gh && std::all_of(open.begin() + y1 * gw + bx, open.begin() + y1 * gw + x1,
                                          [](uint8_t v) { return v != 0; }))
                ++y1;
            for (int y = by; y < y1; ++y) std::fill(open.begin() + y * gw + bx, open.begin() + y * gw + x1, 0);
            out.push_back(dc_rect{bx * B, by * B, (x1 - bx) * B, (y1 - by) * B});
        }
    }
}

int concat_inputs(const dc_layer& l, int* ids) {
    // the first two producers always exist; the list ends at the first absent one after them
    const int32_t all[4] = {l.in0, l.in1, l.in2, l.in3};
    int n = 2;
    while (n < 4 && all[n] >= 0) ++n;
    std::copy(all, all + n, ids);
    return n;
}

int validate_layers(const dc_layer* L, int n_layers, int H, int W, int C, std::vector<int>* hs,
                    std::vector<int>* ws, std::vector<int>* cs) {
    std::vector<int> h(n_layers + 1), w(n_layers + 1), c(n_layers + 1);
    h[0] = H; w[0] = W; c[0] = C;
    for (int i = 0; i < n_layers; ++i) {
        const dc_layer& l = L[i];
        if (l.in0 < 0 || l.in0 > i) return DC_ERR_BAD_SHAPE;
        int a = l.in0;
        switch (l.type) {
            case DC_CONV:
            case DC_MAXPOOL:
            case DC_AVGPOOL:
            {
                const WindowGeom g = window_geom(l);
                if (g.kh < 1 || g.kw < 1 || l.s < 1 || g.ph < 0 || g.pw < 0 || g.ph >= g.eh || g.pw >= g.ew) return DC_ERR_INVALID_ARG;
                if (l.type == DC_CONV && (l.relu < 0 || l.relu > 2 || l.k2 < 0 || l.dil < 0 || l.dil > 64 || g.kh > 64 || g.kw > 64))
                    return DC_ERR_INVALID_ARG;
                if (l.cin != c[a] || l.cout < 1) return DC_ERR_BAD_SHAPE;
                if (l.type != DC_CONV && l.cout != l.cin) return DC_ERR_BAD_SHAPE;
                if (h[a] + 2 * g.ph < g.eh || w[a] + 2 * g.pw < g.ew) return DC_ERR_BAD_SHAPE;
                h[i + 1] = (h[a] + 2 * g.ph - g.eh) / l.s + 1;
                w[i + 1] = (w[a] + 2 * g.pw - g.ew) / l.s + 1;
                c[i + 1] = l.cout;
                break;
            }
            case DC_ADD:
                if (l.in1 < 0 || l.in1 > i) return DC_ERR_BAD_SHAPE;
                if (h[a] != h[l.in1] || w[a] != w[l.in1] || c[a] != c[l.in1] || l.cin != c[a] ||
                    l.cout != c[a])
                    return DC_ERR_BAD_SHAPE;
                h[i + 1] = h[a]; w[i + 1] = w[a]; c[i + 1] = c[a];
                break;
            case DC_LRN:
                if (l.k < 1 || l.k % 2 == 0) return DC_ERR_INVALID_ARG;
                // fall through
            case DC_SOFTMAX:
            case DC_RELU:
                if (l.cin != c[a] || l.cout != c[a]) return DC_ERR_BAD_SHAPE;
                h[i + 1] = h[a]; w[i + 1] = w[a]; c[i + 1] = c[a];
                break;
            case DC_CONCAT: {
                if (l.in1 < 0 || (l.in2 < 0 && l.in3 >= 0)) return DC_ERR_BAD_SHAPE;
                int ids[4];
                const int m = concat_inputs(l, ids);
                int sum = 0;
                for (int j = 0; j < m; ++j) {
                    if (ids[j] < 0 || ids[j] > i || h[ids[j]] != h[a] || w[ids[j]] != w[a]) return DC_ERR_BAD_SHAPE;
                    sum += c[ids[j]];
                }
                if (l.cout != sum || l.cin != sum) return DC_ERR_BAD_SHAPE;
                h[i + 1] = h[a]; w[i + 1] = w[a]; c[i + 1] = sum;
                break;
            }
            case DC_FC:
                if (l.cin != c[a] || l.cout < 1) return DC_ERR_BAD_SHAPE;
                h[i + 1] = 1; w[i + 1] = 1; c[i + 1] = l.cout;
                break;
            default:
                return DC_ERR_INVALID_ARG;
        }
    }
    if (hs) *hs = h;
    if (ws) *ws = w;
    if (cs) *cs = c;
    return DC_OK;
}

int propagate(const dc_layer* L, int n_layers, int H, int W, const std::vector<dc_rect>& rects0,
              int mx, int my, std::vector<TensorRegions>& out, bool extend_borders) {
    const bool ext = extend_borders && mx == 0 && my == 0;
    out.assign(n_layers + 1, TensorRegions());
    TensorRegions& t0 = out[0];
    t0.h = H; t0.w = W; t0.dx = mx; t0.dy = my; t0.cum_stride = 1;
    for (const dc_rect& r : rects0) push_clipped(t0.rects, Span{r.x, r.x + r.w}, Span{r.y, r.y + r.h}, t0);
    for (int i = 0; i < n_layers; ++i) {
        const dc_layer& l = L[i];
        const TensorRegions& a = out[l.in0];
        TensorRegions& t = out[i + 1];
        const bool windowed = (l.type == DC_CONV || l.type == DC_MAXPOOL || l.type == DC_AVGPOOL);
        const WindowGeom wg = window_geom(l);       // a conv kernel may span another extent per axis
        t.h = windowed ? (a.h + 2 * wg.ph - wg.eh) / l.s + 1 : (l.type == DC_FC ? 1 : a.h);
        t.w = windowed ? (a.w + 2 * wg.pw - wg.ew) / l.s + 1 : (l.type == DC_FC ? 1 : a.w);
        t.cum_stride = windowed ? a.cum_stride * l.s : a.cum_stride;
        t.dx = round_half_away(mx, t.cum_stride);
        t.dy = round_half_away(my, t.cum_stride);
        if (l.type == DC_FC || l.type == DC_SOFTMAX) {
            // every output depends on every input: nothing is reusable from here on
        } else if (l.type == DC_LRN && l.within) {
            const int r = (l.k - 1) / 2;
            for (const dc_rect& rc : a.rects) {
                Span xs{rc.x + r, rc.x + rc.w - r}, ys{rc.y + r, rc.y + rc.h - r};
                if (ext) {
                    xs = window_span_ext(Span{rc.x, rc.x + rc.w}, l.k, 1, r, a.w);
                    ys = window_span_ext(Span{rc.y, rc.y + rc.h}, l.k, 1, r, a.h);
                }
                if (xs.empty() || ys.empty()) continue;
                push_clipped(t.rects, xs, ys, t);
            }
        } else if (l.type == DC_CONCAT) {
            int ids[4];
            const int m = concat_inputs(l, ids);
            // overlaps of the first two lists, then of that with the third, ...: in the order of the tuples
            // (i0, i1, ..) with the last index fastest, which is the order a direct enumeration gives
            std::vector<std::pair<Span, Span>> acc, next;
            for (const dc_rect& r : a.rects) acc.push_back({Span{r.x, r.x + r.w}, Span{r.y, r.y + r.h}});
            for (int j = 1; j < m; ++j) {
                const TensorRegions& b = out[ids[j]];
                if (b.cum_stride != a.cum_stride) return DC_ERR_BAD_SHAPE;
                next.clear();
                for (const auto& ra : acc)
                    for (const dc_rect& rb : b.rects) {
                        Span xs = intersect(ra.first, Span{rb.x, rb.x + rb.w});
                        Span ys = intersect(ra.second, Span{rb.y, rb.y + rb.h});
                        if (xs.empty() || ys.empty()) continue;
                        next.push_back({xs, ys});
                    }
                acc.swap(next);
            }
            for (const auto& r : acc) push_clipped(t.rects, r.first, r.second, t);
        } else if (windowed) {
            for (const dc_rect& r : a.rects) {
                Span xs = ext ? window_span_ext(Span{r.x, r.x + r.w}, wg.ew, l.s, wg.pw, a.w) : window_span(Span{r.x, r.x + r.w}, wg.ew, l.s, wg.pw);
                Span ys = ext ? window_span_ext(Span{r.y, r.y + r.h}, wg.eh, l.s, wg.ph, a.h) : window_span(Span{r.y, r.y + r.h}, wg.eh, l.s, wg.ph);
                if (xs.empty() || ys.empty()) continue;
                push_clipped(t.rects, xs, ys, t);
            }
        } else if (l.type == DC_ADD) {
            const TensorRegions& b = out[l.in1];
            if (b.cum_stride != a.cum_stride) return DC_ERR_BAD_SHAPE;
            for (const dc_rect& ra : a.rects)
                for (const dc_rect& rb : b.rects) {
                    Span xs = intersect(Span{ra.x, ra.x + ra.w}, Span{rb.x, rb.x + rb.w});
                    Span ys = intersect(Span{ra.y, ra.y + ra.h}, Span{rb.y, rb.y + rb.h});
                    if (xs.empty() || ys.empty()) continue;
                    push_clipped(t.rects, xs, ys, t);
                }
        } else {
            for (const dc_rect& r : a.rects) push_clipped(t.rects, Span{r.x, r.x + r.w}, Span{r.y, r.y + r.h}, t);
        }
    }
    return DC_OK;
}

void plan_stream(const dc_rect* rects, int n, int dx, int dy, int stream, int Hout, int Wout, int th,
                 int tw, LayerPlan& plan) {
    // tiles are 4x4 pixels: the reusable pixels of a tile are one 16-bit mask (bit 4*row + column)
    (void)th; (void)tw;
    const int tiles_y = (Hout + 3) / 4, tiles_x = (Wout + 3) / 4;
    static thread_local std::vector<uint16_t> reuse;          // kept between calls: no allocation per layer and frame
    reuse.assign((size_t)tiles_y * tiles_x, 0);
    RangeDev range{(int)plan.rects.size(), 0};
    for (int i = 0; i < n; ++i) {
        const dc_rect& r = rects[i];
        if (r.w <= 0 || r.h <= 0) continue;
        plan.rects.push_back(RectDev{r.x, r.y, r.w, r.h, stream, dx, dy, 0});
        ++range.count;
        plan.reused_px += (int64_t)r.w * r.h;
        const int tx0 = r.x / 4, tx1 = (r.x + r.w - 1) / 4;
        const int fx0 = (r.x + 3) / 4, fx1 = (r.x + r.w) / 4;    // tile columns [fx0, fx1) lie wholly inside the rectangle
        for (int ty = r.y / 4; ty <= (r.y + r.h - 1) / 4; ++ty) {
            const int ya = std::max(r.y, ty * 4) - ty * 4, yb = std::min(r.y + r.h, ty * 4 + 4) - ty * 4;
            unsigned rows = 0;                                   // bit 4*y set for the covered rows
            for (int y = ya; y < yb; ++y) rows |= 1u << (4 * y);
            uint16_t* rowp = reuse.data() + (size_t)ty * tiles_x;
            auto partial = [&](int tx) {
                const int xa = std::max(r.x, tx * 4) - tx * 4, xb = std::min(r.x + r.w, tx * 4 + 4) - tx * 4;
                const unsigned cols = ((1u << xb) - 1u) & ~((1u << xa) - 1u);
                rowp[tx] |= (uint16_t)(rows * cols);
            };
            if (rows == 0x1111u && fx1 > fx0) {                  // the interior of the rectangle: whole tiles
                for (int tx = tx0; tx < fx0; ++tx) partial(tx);
                std::fill(rowp + fx0, rowp + fx1, (uint16_t)0xffff);
                for (int tx = fx1; tx <= tx1; ++tx) partial(tx);
            } else {
                for (int tx = tx0; tx <= tx1; ++tx) partial(tx);
            }
        }
    }
    plan.ranges.push_back(range);
    // a tile is listed unless every pixel of it that lies in the map is served by the copy
    const int full_cols = Wout / 4;                              // tile columns with all four pixel columns in the map
    for (int ty = 0; ty < tiles_y; ++ty) {
        const uint16_t* rowp = reuse.data() + (size_t)ty * tiles_x;
        const int hh = std::min(4, Hout - ty * 4);
        unsigned rows = 0;
        for (int y = 0; y < hh; ++y) rows |= 1u << (4 * y);
        const unsigned inside_full = rows * 0xfu;
        int tx = 0;
        if (inside_full == 0xffffu) {
            for (; tx + 4 <= full_cols; tx += 4) {               // four tiles at a time: the common case is "all reusable"
                uint64_t v;
                std::memcpy(&v, rowp + tx, sizeof(v));
                if (v == ~0ull) continue;
                for (int k = 0; k < 4; ++k)
                    if (rowp[tx + k] != 0xffffu) plan.tiles.push_back(TileDev{stream, ty, tx + k, (int32_t)rowp[tx + k]});
            }
        }
        for (; tx < full_cols; ++tx)
            if ((rowp[tx] & inside_full) != inside_full) plan.tiles.push_back(TileDev{stream, ty, tx, (int32_t)rowp[tx]});
        if (full_cols < tiles_x) {                               // the last column holds Wout % 4 pixel columns
            const unsigned inside = rows * ((1u << (Wout - full_cols * 4)) - 1u);
            if ((rowp[tx] & inside) != inside) plan.tiles.push_back(TileDev{stream, ty, tx, (int32_t)rowp[tx]});
        }
    }
}


// ---- host thread pool for the per-stream planning of many streams ----------------------------
namespace {
class Pool {
public:
    void run(int n, const std::function<void(int)>& fn) {
        std::lock_guard<std::mutex> serial(callers_);
        start_workers();
        unsigned long gen;
        {
            std::lock_guard<std::mutex> g(m_);
            gen = ++generation_;
            fn_ = &fn; n_ = n;
            pending_.store(n);
            ticket_.store((unsigned long long)gen << 32);      // (generation, next index): published last
        }
        work_.notify_all();
        drain(gen, &fn, n);                                    // the caller works too
        std::unique_lock<std::mutex> g(m_);
        done_.wait(g, [&] { return pending_.load() == 0; });
    }
    ~Pool() {
        {
            std::lock_guard<std::mutex> g(m_);
            stop_ = true;
        }
        work_.notify_all();
        for (std::thread& t : threads_) t.join();
    }

private:
    void start_workers() {
        if (!threads_.empty()) return;
        unsigned hw = std::thread::hardware_concurrency();
        int want = (int)(hw ? hw : 4);
        if (want > 16) want = 16;
        for (int i = 1; i < want; ++i) threads_.emplace_back([this] { worker(); });
    }
    // Takes indices of generation `gen` until none is left.  The ticket carries the generation, so a thread that
    // wakes up late (its generation is over, another one may have started) takes nothing and calls nothing.
    void drain(unsigned long gen, const std::function<void(int)>* fn, int n) {
        for (;;) {
            unsigned long long t = ticket_.load();
            if ((unsigned long)(t >> 32) != (gen & 0xfffffffful) || (int)(t & 0xffffffffull) >= n) return;
            if (!ticket_.compare_exchange_weak(t, t + 1)) continue;
            (*fn)((int)(t & 0xffffffffull));
            if (pending_.fetch_sub(1) == 1) {
                std::lock_guard<std::mutex> g(m_);
                done_.notify_all();
            }
        }
    }
    void worker() {
        unsigned long seen = 0;
        for (;;) {
            const std::function<void(int)>* fn;
            int n;
            {
                std::unique_lock<std::mutex> g(m_);
                work_.wait(g, [&] { return stop_ || generation_ != seen; });
                if (stop_) return;
                seen = generation_; fn = fn_; n = n_;
            }
            drain(seen, fn, n);
        }
    }
    std::mutex callers_, m_;
    std::condition_variable work_, done_;
    std::vector<std::thread> threads_;
    const std::function<void(int)>* fn_ = nullptr;
    int n_ = 0;
    std::atomic<unsigned long long> ticket_{0};
    std::atomic<int> pending_{0};
    unsigned long generation_ = 0;
    bool stop_ = false;
};
Pool g_pool;
}  // namespace

void parallel_for(int n, const std::function<void(int)>& fn) {
    if (n < 4) {
        for (int i = 0; i < n; ++i) fn(i);
        return;
    }
    g_pool.run(n, fn);
}

}  // namespace dc
