/*
 * CPU oracle for cache-aware CNN inference over a video stream (DeepCache).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is a plain, slow, obviously-correct
 * implementation used to check the HIP library and to report a CPU baseline.
 * It shares no code with the HIP path and nothing in the product path may
 * call it.  Every function follows the paper's steps in the paper's order.
 *
 * Floating point: feature maps are *stored* in the path's storage type
 * (fp32, or bf16 kept in a float whose low 16 bits are zero); every sum is
 * accumulated in fp64 and rounded once when stored.
 *
 * Conventions (readings of points the paper leaves open are marked "reading"):
 *  - frames: uint8 [H][W][C], interleaved channels, left-top origin;
 *  - feature maps: float [H][W][C] (channels last);
 *  - conv weights: float [cout][k][k][cin];
 *  - a motion vector (dx,dy) points from a block of the current frame to its
 *    match in the previous frame: source = current + (dx,dy)  (Section 4,
 *    Step 2: (x',y') is the position in the previous frame, Step 3 averages
 *    x'-x and y'-y).
 *
 * Pins (tests/test_oracle_*.py): the worked propagation example of Section 5
 * ((100,100,100,40) under conv k11 s2 p5 -> (53,53,45,15)), the erosion
 * arithmetic of Section 4 (two 5x5 -> 18 px, merged 5x10 -> 24 px), the 5x5
 * example of Section 2.2, brute-force window containment for the region rule,
 * closed-form matching results on constructed frame pairs, scipy's correlate
 * for the convolution, and the three invariants (zero reuse == full forward,
 * identical frames -> full reuse, exact shifted copy == full forward).
 * The diamond-search matcher (Step 2 as the paper runs it, plus k-skip) is
 * pinned by walks worked out by hand on small cost tables (moves, ties, range
 * and frame limits, a trap that separates it from the exhaustive search), by
 * the fixed-point property of the published algorithm checked against an
 * independent numpy cost table, by the closed form for content moved by a
 * point of the large pattern, and by the k-skip bookkeeping.
 * The remaining layer types (LRN, concat, fully-connected, softmax, average
 * pooling) are pinned by hand-computed values, the printed LRN row of Table 2
 * and brute-force window containment, pixel-wise AND for the concat row, and
 * the torch / scipy / numpy routines for the cases those implement.
 * The element-wise add and ReLU are pinned by hand values (exact binary
 * fractions, bf16 ties rounded once to even, negative zero) and numpy.
 * Unpinned by the paper (pinned only by hand cases of the stated reading):
 * the merge decomposition, the rounding of fractional motion, and the source
 * offset when the motion is not a multiple of the cumulative stride.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct { int32_t x, y, w, h; } oc_rect;

enum { OC_CONV = 0, OC_MAXPOOL = 1, OC_RELU = 2, OC_ADD = 3, OC_LRN = 4, OC_CONCAT = 5, OC_FC = 6, OC_SOFTMAX = 7,
       OC_AVGPOOL = 8 };

typedef struct {
    int32_t type;          /* OC_* */
    int32_t k, s, p;       /* kernel, stride, padding (conv, pool); k = window size of an LRN (odd) */
    int32_t cin, cout;
    int32_t relu;          /* fused ReLU after conv / add / fc */
    int32_t in0, in1;      /* producer tensor ids; tensor 0 = network input, tensor i+1 = layer i output */
    int32_t in2, in3;      /* further producers of a concat, -1: none */
    int32_t within;        /* LRN: 0 = window over channels at one pixel, 1 = k x k pixels of one channel */
    float alpha, beta, kappa;   /* LRN constants */
    /* conv layers only (Table 2's conv row speaks of a kernel of size k; these generalise it per axis):
     * k2 > 0: the kernel is k rows x k2 columns with padding p along y and p2 along x; k2 == 0: k x k, padding p.
     * dil > 1: taps are dil pixels apart, the kernel spans (k - 1) * dil + 1 pixels. */
    int32_t k2, p2, dil;
} oc_layer;

/* kernel rows / columns, padding along y / x, dilation, and the span of the kernel in pixels */
static int l_kh(const oc_layer* l) { return l->k; }
static int l_kw(const oc_layer* l) { return (l->type == OC_CONV && l->k2 > 0) ? l->k2 : l->k; }
static int l_ph(const oc_layer* l) { return l->p; }
static int l_pw(const oc_layer* l) { return (l->type == OC_CONV && l->k2 > 0) ? l->p2 : l->p; }
static int l_dil(const oc_layer* l) { return (l->type == OC_CONV && l->dil > 1) ? l->dil : 1; }
static int l_eh(const oc_layer* l) { return (l_kh(l) - 1) * l_dil(l) + 1; }
static int l_ew(const oc_layer* l) { return (l_kw(l) - 1) * l_dil(l) + 1; }

#define OC_MAX_CONCAT 4
/* producers of a concat layer, in channel order; returns their number */
static int concat_inputs(const oc_layer* l, int* ids)
{
    int n = 0;
    ids[n++] = l->in0;
    ids[n++] = l->in1;
    if (l->in2 >= 0) ids[n++] = l->in2;
    if (l->in2 >= 0 && l->in3 >= 0) ids[n++] = l->in3;
    return n;
}

/* ------------------------------------------------------------------ */
/* Section 4, Steps 1-4: block matching                               */
/* ------------------------------------------------------------------ */

/* Sum of squared differences between the BxB block of `cur` at (x,y) and the
 * BxB block of `prev` at (x+dx, y+dy), over all C channels.  PSNR of Section 4
 * is a decreasing function of this sum, so "PSNR > T" is "SSD <= bound"
 * (reading: the bound is passed as a per-block total). */
static uint32_t block_ssd(const uint8_t* cur, const uint8_t* prev, int W, int C,
                          int B, int x, int y, int dx, int dy)
{
    uint32_t s = 0;
    for (int r = 0; r < B; ++r)
        for (int c = 0; c < B; ++c)
            for (int ch = 0; ch < C; ++ch) {
                int a = cur[((size_t)(y + r) * W + (x + c)) * C + ch];
                int b = prev[((size_t)(y + dy + r) * W + (x + dx + c)) * C + ch];
                s += (uint32_t)((a - b) * (a - b));
            }
    return s;
}

static int iabs(int v) { return v < 0 ? -v : v; }

/* round(num/den) to nearest, halves away from zero; den > 0 (reading) */
static int32_t round_div(int64_t num, int64_t den)
{
    int64_t a = num < 0 ? -num : num;
    int64_t q = (2 * a + den) / (2 * den);
    return (int32_t)(num < 0 ? -q : q);
}

/*
 * Steps 1-4 for one frame pair.
 *   mv        [gh][gw][2]  best vector (dx,dy) per block (exhaustive search,
 *                          Section 7.6 "ES"), candidates |dx|,|dy|<=R whose
 *                          window lies inside the previous frame (reading);
 *                          ties: smallest (ssd, |dx|+|dy|, dy, dx) (reading)
 *   best_ssd  [gh][gw]
 *   gmv       [2]          Step 3 mean motion over blocks with best_ssd<=max_ssd
 *   n_pass    [1]          K of Step 3
 *   mask      [gh][gw]     Step 4: 1 iff block at +gmv is in-frame and SSD<=max_ssd
 * gh = H/B, gw = W/B (integer division; a remainder strip is never reusable).
 */
void oc_match_blocks(const uint8_t* cur, const uint8_t* prev, int H, int W, int C,
                     int B, int R, uint32_t max_ssd,
                     int16_t* mv, uint32_t* best_ssd, int32_t* gmv, int32_t* n_pass,
                     uint8_t* mask)
{
    int gh = H / B, gw = W / B;
#pragma omp parallel for collapse(2) schedule(dynamic)
    for (int by = 0; by < gh; ++by)
        for (int bx = 0; bx < gw; ++bx) {
            int x = bx * B, y = by * B;
            int have = 0, bdx = 0, bdy = 0;
            uint32_t bs = 0;
            for (int dy = -R; dy <= R; ++dy)
                for (int dx = -R; dx <= R; ++dx) {
                    if (x + dx < 0 || y + dy < 0 || x + dx + B > W || y + dy + B > H) continue;
                    uint32_t s = block_ssd(cur, prev, W, C, B, x, y, dx, dy);
                    int better;
                    if (!have) better = 1;
                    else if (s != bs) better = s < bs;
                    else if (iabs(dx) + iabs(dy) != iabs(bdx) + iabs(bdy))
                        better = iabs(dx) + iabs(dy) < iabs(bdx) + iabs(bdy);
                    else if (dy != bdy) better = dy < bdy;
                    else better = dx < bdx;
                    if (better) { have = 1; bs = s; bdx = dx; bdy = dy; }
                }
            mv[(by * gw + bx) * 2 + 0] = (int16_t)bdx;
            mv[(by * gw + bx) * 2 + 1] = (int16_t)bdy;
            best_ssd[by * gw + bx] = bs;
        }
    /* Step 3 */
    int64_t sx = 0, sy = 0;
    int K = 0;
    for (int i = 0; i < gh * gw; ++i)
        if (best_ssd[i] <= max_ssd) { sx += mv[2 * i]; sy += mv[2 * i + 1]; ++K; }
    *n_pass = K;
    if (K == 0) {                      /* nothing matched: no reuse in this frame */
        gmv[0] = gmv[1] = 0;
        memset(mask, 0, (size_t)gh * gw);
        return;
    }
    int mx = round_div(sx, K), my = round_div(sy, K);
    gmv[0] = mx; gmv[1] = my;
    /* Step 4 */
    for (int by = 0; by < gh; ++by)
        for (int bx = 0; bx < gw; ++bx) {
            int x = bx * B, y = by * B;
            int ok = !(x + mx < 0 || y + my < 0 || x + mx + B > W || y + my + B > H);
            if (ok) ok = block_ssd(cur, prev, W, C, B, x, y, mx, my) <= max_ssd;
            mask[by * gw + bx] = (uint8_t)ok;
        }
}

/*
 * Steps 1-4 with the exhaustive search and k-skip (Section 4, last part: the
 * acceleration skips blocks in Step 2 whatever the search is): as
 * oc_match_blocks, but only the blocks whose grid row and column are multiples
 * of k are searched; Step 3 averages over those that pass; Step 4 tests every
 * block.  Blocks that were not searched get mv = (0,0), best_ssd = UINT32_MAX.
 */
void oc_match_blocks_k(const uint8_t* cur, const uint8_t* prev, int H, int W, int C,
                       int B, int R, int k, uint32_t max_ssd,
                       int16_t* mv, uint32_t* best_ssd, int32_t* gmv, int32_t* n_pass,
                       uint8_t* mask)
{
    int gh = H / B, gw = W / B;
    int64_t sx = 0, sy = 0;
    int K = 0;
    for (int by = 0; by < gh; ++by)
        for (int bx = 0; bx < gw; ++bx) {
            int i = by * gw + bx;
            mv[2 * i] = mv[2 * i + 1] = 0;
            best_ssd[i] = UINT32_MAX;
            if (by % k != 0 || bx % k != 0) continue;
            int x = bx * B, y = by * B;
            int have = 0, bdx = 0, bdy = 0;
            uint32_t bs = 0;
            for (int dy = -R; dy <= R; ++dy)
                for (int dx = -R; dx <= R; ++dx) {
                    if (x + dx < 0 || y + dy < 0 || x + dx + B > W || y + dy + B > H) continue;
                    uint32_t s = block_ssd(cur, prev, W, C, B, x, y, dx, dy);
                    int better;
                    if (!have) better = 1;
                    else if (s != bs) better = s < bs;
                    else if (iabs(dx) + iabs(dy) != iabs(bdx) + iabs(bdy))
                        better = iabs(dx) + iabs(dy) < iabs(bdx) + iabs(bdy);
                    else if (dy != bdy) better = dy < bdy;
                    else better = dx < bdx;
                    if (better) { have = 1; bs = s; bdx = dx; bdy = dy; }
                }
            mv[2 * i] = (int16_t)bdx; mv[2 * i + 1] = (int16_t)bdy;
            best_ssd[i] = bs;
            if (bs <= max_ssd) { sx += bdx; sy += bdy; ++K; }
        }
    *n_pass = K;
    if (K == 0) {
        gmv[0] = gmv[1] = 0;
        memset(mask, 0, (size_t)gh * gw);
        return;
    }
    int mx = round_div(sx, K), my = round_div(sy, K);
    gmv[0] = mx; gmv[1] = my;
    for (int by = 0; by < gh; ++by)
        for (int bx = 0; bx < gw; ++bx) {
            int x = bx * B, y = by * B;
            int ok = !(x + mx < 0 || y + my < 0 || x + mx + B > W || y + my + B > H);
            if (ok) ok = block_ssd(cur, prev, W, C, B, x, y, mx, my) <= max_ssd;
            mask[by * gw + bx] = (uint8_t)ok;
        }
}

/* ------------------------------------------------------------------ */
/* Section 4, Step 2 with diamond search, k-skip (Section 4, last part) */
/* ------------------------------------------------------------------ */

/*
 * Diamond search (the block-matching algorithm Section 4 names for Step 2; the
 * paper cites it and does not restate it, so this is the published algorithm):
 *   large pattern: the centre and the eight points at (0,+-2), (+-2,0), (+-1,+-1);
 *   small pattern: the centre and the four points at (0,+-1), (+-1,0).
 *   1. centre = (0,0);
 *   2. evaluate the large pattern around the centre; if the best point is the
 *      centre go to 3, otherwise the best point becomes the centre, repeat 2;
 *   3. evaluate the small pattern around the centre; its best point is the result.
 * Readings: a candidate is valid iff |dx|,|dy| <= R and its window lies inside
 * the previous frame (as for the exhaustive search); the best point of a pattern
 * is the valid one with the smallest (cost, position in the pattern), the centre
 * being position 0 and the others following in raster order (dy, then dx), so
 * the centre only moves to a strictly smaller cost and the walk ends.
 * `cost` returns the block cost of a vector, `valid` whether it may be used.
 * rounds = number of times step 2 ran.
 */
typedef uint32_t (*ds_cost_fn)(void* ctx, int dx, int dy);
typedef int (*ds_valid_fn)(void* ctx, int dx, int dy);

static const int kLarge[9][2] = {{0, 0}, {0, -2}, {-1, -1}, {1, -1}, {-2, 0}, {2, 0}, {-1, 1}, {1, 1}, {0, 2}};
static const int kSmall[5][2] = {{0, 0}, {0, -1}, {-1, 0}, {1, 0}, {0, 1}};

static void diamond_search(ds_cost_fn cost, ds_valid_fn valid, void* ctx,
                           int* out_dx, int* out_dy, uint32_t* out_cost, int* out_rounds)
{
    int cx = 0, cy = 0, rounds = 0;
    uint32_t ccost = cost(ctx, 0, 0);          /* (0,0) is always valid: the block lies in both frames */
    for (;;) {
        int best = 0;
        uint32_t bcost = ccost;
        ++rounds;
        for (int i = 1; i < 9; ++i) {
            int dx = cx + kLarge[i][0], dy = cy + kLarge[i][1];
            if (!valid(ctx, dx, dy)) continue;
            uint32_t c = cost(ctx, dx, dy);
            if (c < bcost) { bcost = c; best = i; }
        }
        if (best == 0) break;
        cx += kLarge[best][0]; cy += kLarge[best][1]; ccost = bcost;
    }
    int best = 0;
    uint32_t bcost = ccost;
    for (int i = 1; i < 5; ++i) {
        int dx = cx + kSmall[i][0], dy = cy + kSmall[i][1];
        if (!valid(ctx, dx, dy)) continue;
        uint32_t c = cost(ctx, dx, dy);
        if (c < bcost) { bcost = c; best = i; }
    }
    *out_dx = cx + kSmall[best][0]; *out_dy = cy + kSmall[best][1];
    *out_cost = bcost; *out_rounds = rounds;
}

/* Diamond search over a given cost table: table[(dy+R)*(2R+1) + dx+R], entries
 * equal to UINT32_MAX are invalid vectors.  For tests of the search itself. */
typedef struct { const uint32_t* table; int R; } table_ctx;
static uint32_t table_cost(void* p, int dx, int dy)
{
    table_ctx* t = (table_ctx*)p;
    return t->table[(dy + t->R) * (2 * t->R + 1) + dx + t->R];
}
static int table_valid(void* p, int dx, int dy)
{
    table_ctx* t = (table_ctx*)p;
    if (iabs(dx) > t->R || iabs(dy) > t->R) return 0;
    return table_cost(p, dx, dy) != UINT32_MAX;
}
void oc_diamond_search_table(const uint32_t* table, int R, int32_t* best_dxdy, uint32_t* best, int32_t* rounds)
{
    table_ctx t = {table, R};
    int dx, dy, n;
    diamond_search(table_cost, table_valid, &t, &dx, &dy, best, &n);
    best_dxdy[0] = dx; best_dxdy[1] = dy; *rounds = n;
}

typedef struct { const uint8_t* cur; const uint8_t* prev; int H, W, C, B, R, x, y; } block_ctx;
static uint32_t block_cost(void* p, int dx, int dy)
{
    block_ctx* b = (block_ctx*)p;
    return block_ssd(b->cur, b->prev, b->W, b->C, b->B, b->x, b->y, dx, dy);
}
static int block_valid(void* p, int dx, int dy)
{
    block_ctx* b = (block_ctx*)p;
    if (iabs(dx) > b->R || iabs(dy) > b->R) return 0;
    return !(b->x + dx < 0 || b->y + dy < 0 || b->x + dx + b->B > b->W || b->y + dy + b->B > b->H);
}

/*
 * Steps 1-4 with the diamond search in Step 2 and k-skip: only the blocks whose
 * grid row and grid column are both multiples of k are searched (k = 1: all);
 * Step 3 averages over the searched blocks that pass; Step 4 tests every block.
 * Blocks that were not searched get mv = (0,0), best_ssd = UINT32_MAX, rounds = 0.
 * (Re-using Step 2's costs in Step 4 changes no result and is not modelled.)
 */
void oc_match_blocks_ds(const uint8_t* cur, const uint8_t* prev, int H, int W, int C,
                        int B, int R, int k, uint32_t max_ssd,
                        int16_t* mv, uint32_t* best_ssd, int32_t* gmv, int32_t* n_pass,
                        uint8_t* mask, int32_t* rounds)
{
    int gh = H / B, gw = W / B;
    int64_t sx = 0, sy = 0;
    int K = 0;
    for (int by = 0; by < gh; ++by)
        for (int bx = 0; bx < gw; ++bx) {
            int i = by * gw + bx;
            mv[2 * i] = mv[2 * i + 1] = 0;
            best_ssd[i] = UINT32_MAX;
            if (rounds) rounds[i] = 0;
            if (by % k != 0 || bx % k != 0) continue;
            block_ctx b = {cur, prev, H, W, C, B, R, bx * B, by * B};
            int dx, dy, n;
            uint32_t s;
            diamond_search(block_cost, block_valid, &b, &dx, &dy, &s, &n);
            mv[2 * i] = (int16_t)dx; mv[2 * i + 1] = (int16_t)dy;
            best_ssd[i] = s;
            if (rounds) rounds[i] = n;
            if (s <= max_ssd) { sx += dx; sy += dy; ++K; }      /* Step 3 */
        }
    *n_pass = K;
    if (K == 0) {
        gmv[0] = gmv[1] = 0;
        memset(mask, 0, (size_t)gh * gw);
        return;
    }
    int mx = round_div(sx, K), my = round_div(sy, K);
    gmv[0] = mx; gmv[1] = my;
    for (int by = 0; by < gh; ++by)                              /* Step 4 */
        for (int bx = 0; bx < gw; ++bx) {
            int x = bx * B, y = by * B;
            int ok = !(x + mx < 0 || y + my < 0 || x + mx + B > W || y + my + B > H);
            if (ok) ok = block_ssd(cur, prev, W, C, B, x, y, mx, my) <= max_ssd;
            mask[by * gw + bx] = (uint8_t)ok;
        }
}

/* ------------------------------------------------------------------ */
/* Section 4, Step 5: merge properly matched blocks into rectangles   */
/* ------------------------------------------------------------------ */

/* Reading: scan blocks row-major; at the first set, unclaimed block grow a
 * run to the right over set, unclaimed blocks, then grow the run downwards
 * while the whole run is set and unclaimed; emit it in pixel units.
 * Returns the number of rectangles (writes at most `cap`). */
int oc_merge_blocks(const uint8_t* mask, int gh, int gw, int B, oc_rect* out, int cap)
{
    uint8_t* used = (uint8_t*)calloc((size_t)gh * gw, 1);
    int n = 0;
    for (int by = 0; by < gh; ++by)
        for (int bx = 0; bx < gw; ++bx) {
            if (!mask[by * gw + bx] || used[by * gw + bx]) continue;
            int w = 0;
            while (bx + w < gw && mask[by * gw + bx + w] && !used[by * gw + bx + w]) ++w;
            int h = 1;
            for (;;) {
                if (by + h >= gh) break;
                int all = 1;
                for (int i = 0; i < w; ++i)
                    if (!mask[(by + h) * gw + bx + i] || used[(by + h) * gw + bx + i]) { all = 0; break; }
                if (!all) break;
                ++h;
            }
            for (int j = 0; j < h; ++j)
                for (int i = 0; i < w; ++i) used[(by + j) * gw + bx + i] = 1;
            if (n < cap) { out[n].x = bx * B; out[n].y = by * B; out[n].w = w * B; out[n].h = h * B; }
            ++n;
        }
    free(used);
    return n;
}

/* ------------------------------------------------------------------ */
/* Section 5, Table 2: region transformation D_t                      */
/* ------------------------------------------------------------------ */

static int floor_div(int a, int b) { int q = a / b; if ((a % b != 0) && ((a < 0) != (b < 0))) --q; return q; }
static int ceil_div(int a, int b) { return -floor_div(-a, b); }

/* Conv / pool row of Table 2.  The left-top corner is the table's
 * ceil((x+p)/s).  The size printed in the table disagrees with both worked
 * examples of the paper; the reading used here is the largest output
 * rectangle whose kxk windows lie wholly inside the input rectangle, which
 * reproduces both examples: last output column = floor((x+w-k+p)/s).
 * Returns 0 if nothing is left. */
int oc_dt_window2(oc_rect in, int ew, int eh, int s, int pw, int ph, oc_rect* out);
int oc_dt_window(oc_rect in, int k, int s, int p, oc_rect* out)
{
    return oc_dt_window2(in, k, k, s, p, p, out);
}
/* The same row for a window that spans ew columns and eh rows with paddings pw, ph (a kernel that is not square,
 * or dilated: its span is (k - 1) * dilation + 1; the whole span must lie inside the rectangle, which is what a
 * rectangle can guarantee for the taps). */
int oc_dt_window2(oc_rect in, int ew, int eh, int s, int pw, int ph, oc_rect* out)
{
    int x0 = ceil_div(in.x + pw, s), x1 = floor_div(in.x + in.w - ew + pw, s);
    int y0 = ceil_div(in.y + ph, s), y1 = floor_div(in.y + in.h - eh + ph, s);
    if (x1 < x0 || y1 < y0) return 0;
    out->x = x0; out->y = y0; out->w = x1 - x0 + 1; out->h = y1 - y0 + 1;
    return 1;
}

/* The same row with the border case that Table 2 leaves out, for a stream that did not move (offset zero in
 * every tensor): the taps of a window that fall into the zero padding read zeros in both frames, so only the
 * taps inside the map have to lie in the rectangle.  A rectangle that touches a side of the wa x ha input map
 * therefore extends, for this rule, beyond that side: the first output column is 0 if x == 0, the last one is
 * the last of the map if x + w == wa; likewise for rows.  (An optional extension beyond the paper; off = the
 * printed rule.) */
int oc_dt_window_ext2(oc_rect in, int ew, int eh, int s, int pw, int ph, int wa, int ha, oc_rect* out);
int oc_dt_window_ext(oc_rect in, int k, int s, int p, int wa, int ha, oc_rect* out)
{
    return oc_dt_window_ext2(in, k, k, s, p, p, wa, ha, out);
}
int oc_dt_window_ext2(oc_rect in, int ew, int eh, int s, int pw, int ph, int wa, int ha, oc_rect* out)
{
    int wo = (wa + 2 * pw - ew) / s + 1, ho = (ha + 2 * ph - eh) / s + 1;
    int x0 = in.x == 0 ? 0 : ceil_div(in.x + pw, s);
    int x1 = in.x + in.w == wa ? wo - 1 : floor_div(in.x + in.w - ew + pw, s);
    int y0 = in.y == 0 ? 0 : ceil_div(in.y + ph, s);
    int y1 = in.y + in.h == ha ? ho - 1 : floor_div(in.y + in.h - eh + ph, s);
    if (x1 > wo - 1) x1 = wo - 1;
    if (y1 > ho - 1) y1 = ho - 1;
    if (x1 < x0 || y1 < y0) return 0;
    out->x = x0; out->y = y0; out->w = x1 - x0 + 1; out->h = y1 - y0 + 1;
    return 1;
}

/* Concat row of Table 2, used for a residual add: overlap of two rectangles. */
int oc_dt_overlap(oc_rect a, oc_rect b, oc_rect* out)
{
    int x0 = a.x > b.x ? a.x : b.x, y0 = a.y > b.y ? a.y : b.y;
    int x1 = (a.x + a.w < b.x + b.w) ? a.x + a.w : b.x + b.w;
    int y1 = (a.y + a.h < b.y + b.h) ? a.y + a.h : b.y + b.h;
    if (x1 <= x0 || y1 <= y0) return 0;
    out->x = x0; out->y = y0; out->w = x1 - x0; out->h = y1 - y0;
    return 1;
}

/* LRN row of Table 2 for a window of radius r pixels: (x+r, y+r, w-2r, h-2r).  A window over channels only has
 * no spatial extent: its radius in the pixel grid is 0 and the row leaves the rectangle as it is (reading). */
int oc_dt_lrn(oc_rect in, int r, oc_rect* out)
{
    if (in.w - 2 * r <= 0 || in.h - 2 * r <= 0) return 0;
    out->x = in.x + r; out->y = in.y + r; out->w = in.w - 2 * r; out->h = in.h - 2 * r;
    return 1;
}

/* Keep the part of r whose source r+(dx,dy) lies inside a WxH map. */
static int clip_to_source(oc_rect r, int dx, int dy, int W, int H, oc_rect* out)
{
    int x0 = r.x, x1 = r.x + r.w, y0 = r.y, y1 = r.y + r.h;
    if (x0 < -dx) x0 = -dx;
    if (y0 < -dy) y0 = -dy;
    if (x1 > W - dx) x1 = W - dx;
    if (y1 > H - dy) y1 = H - dy;
    if (x0 < 0) x0 = 0;
    if (y0 < 0) y0 = 0;
    if (x1 > W) x1 = W;
    if (y1 > H) y1 = H;
    if (x1 <= x0 || y1 <= y0) return 0;
    out->x = x0; out->y = y0; out->w = x1 - x0; out->h = y1 - y0;
    return 1;
}

/*
 * Propagate the reusable rectangles of the input frame through the stack
 * (Section 5 "Propagation").  For tensor t (0 = input, i+1 = output of layer i):
 *   rects[t*cap .. t*cap+n_rects[t])  reusable rectangles in that tensor's pixels
 *   dxy[2t], dxy[2t+1]                source offset in that tensor's pixels
 *   cum_stride[t]                     product of the strides on the way there
 * Reading (paper silent when the motion is not a multiple of the stride): one
 * offset per tensor, round(M / cum_stride) halves away from zero; a rectangle
 * is clipped so that its source stays inside the map.
 * Returns 0, or -1 if some list overflowed `cap` (counts are still exact).
 */
int oc_propagate_ext(const oc_layer* L, int n_layers, int H, int W,
                     const oc_rect* rects0, int n0, int mx, int my, int extend_borders,
                     oc_rect* rects, int cap, int32_t* n_rects, int32_t* dxy,
                     int32_t* cum_stride, int32_t* hw /* [2*(n_layers+1)] heights, widths */)
{
    int overflow = 0;
    int ext = extend_borders && mx == 0 && my == 0;    /* border case of a stream that did not move */
    hw[0] = H; hw[1] = W; cum_stride[0] = 1; dxy[0] = mx; dxy[1] = my;
    int n = 0;
    for (int i = 0; i < n0; ++i) {
        oc_rect r;
        if (!clip_to_source(rects0[i], mx, my, W, H, &r)) continue;
        if (n < cap) rects[n] = r; else overflow = 1;
        ++n;
    }
    n_rects[0] = n;
    for (int li = 0; li < n_layers; ++li) {
        const oc_layer* l = &L[li];
        int t = li + 1, a = l->in0;
        int ha = hw[2 * a], wa = hw[2 * a + 1];
        int na = n_rects[a] < cap ? n_rects[a] : cap;
        const oc_rect* ra = rects + (size_t)a * cap;
        oc_rect* ro = rects + (size_t)t * cap;
        int ho = ha, wo = wa, S = cum_stride[a];
        int windowed = l->type == OC_CONV || l->type == OC_MAXPOOL || l->type == OC_AVGPOOL;
        if (windowed) {
            ho = (ha + 2 * l_ph(l) - l_eh(l)) / l->s + 1;
            wo = (wa + 2 * l_pw(l) - l_ew(l)) / l->s + 1;
            S *= l->s;
        }
        if (l->type == OC_FC) { ho = 1; wo = 1; }
        hw[2 * t] = ho; hw[2 * t + 1] = wo; cum_stride[t] = S;
        int dx = round_div(mx, S), dy = round_div(my, S);
        dxy[2 * t] = dx; dxy[2 * t + 1] = dy;
        n = 0;
        if (l->type == OC_FC || l->type == OC_SOFTMAX) {
            /* fully-connected / softmax row: (0,0,0,0), nothing is reusable from here on */
        } else if (l->type == OC_LRN && l->within) {
            for (int i = 0; i < na; ++i) {
                oc_rect r, c;
                if (!(ext ? oc_dt_window_ext(ra[i], l->k, 1, (l->k - 1) / 2, wa, ha, &r) : oc_dt_lrn(ra[i], (l->k - 1) / 2, &r))) continue;
                if (!clip_to_source(r, dx, dy, wo, ho, &c)) continue;
                if (n < cap) ro[n] = c; else overflow = 1;
                ++n;
            }
        } else if (l->type == OC_CONCAT) {
            /* overlapped region of the N inputs: every N-tuple of rectangles, one from each list */
            int ids[OC_MAX_CONCAT], m = concat_inputs(l, ids);
            int idx[OC_MAX_CONCAT] = {0, 0, 0, 0}, cnt[OC_MAX_CONCAT], empty = 0;
            for (int j = 0; j < m; ++j) { cnt[j] = n_rects[ids[j]] < cap ? n_rects[ids[j]] : cap; if (cnt[j] == 0) empty = 1; }
            while (!empty) {
                oc_rect r = rects[(size_t)ids[0] * cap + idx[0]], c;
                int ok = 1;
                for (int j = 1; j < m && ok; ++j) ok = oc_dt_overlap(r, rects[(size_t)ids[j] * cap + idx[j]], &r);
                if (ok && clip_to_source(r, dx, dy, wo, ho, &c)) {
                    if (n < cap) ro[n] = c; else overflow = 1;
                    ++n;
                }
                int j = m - 1;                 /* next tuple, last index fastest */
                while (j >= 0 && ++idx[j] == cnt[j]) idx[j--] = 0;
                if (j < 0) break;
            }
        } else if (windowed) {
            for (int i = 0; i < na; ++i) {
                oc_rect r, c;
                if (!(ext ? oc_dt_window_ext2(ra[i], l_ew(l), l_eh(l), l->s, l_pw(l), l_ph(l), wa, ha, &r)
                          : oc_dt_window2(ra[i], l_ew(l), l_eh(l), l->s, l_pw(l), l_ph(l), &r))) continue;
                if (!clip_to_source(r, dx, dy, wo, ho, &c)) continue;
                if (n < cap) ro[n] = c; else overflow = 1;
                ++n;
            }
        } else if (l->type == OC_ADD) {
            int b = l->in1;
            int nb = n_rects[b] < cap ? n_rects[b] : cap;
            const oc_rect* rb = rects + (size_t)b * cap;
            for (int i = 0; i < na; ++i)
                for (int j = 0; j < nb; ++j) {
                    oc_rect r, c;
                    if (!oc_dt_overlap(ra[i], rb[j], &r)) continue;
                    if (!clip_to_source(r, dx, dy, wo, ho, &c)) continue;
                    if (n < cap) ro[n] = c; else overflow = 1;
                    ++n;
                }
        } else {                       /* "Others" row: unchanged */
            for (int i = 0; i < na; ++i) {
                oc_rect c;
                if (!clip_to_source(ra[i], dx, dy, wo, ho, &c)) continue;
                if (n < cap) ro[n] = c; else overflow = 1;
                ++n;
            }
        }
        n_rects[t] = n;
    }
    return overflow ? -1 : 0;
}

/* Table 2 as printed (no border case). */
int oc_propagate(const oc_layer* L, int n_layers, int H, int W,
                 const oc_rect* rects0, int n0, int mx, int my,
                 oc_rect* rects, int cap, int32_t* n_rects, int32_t* dxy,
                 int32_t* cum_stride, int32_t* hw)
{
    return oc_propagate_ext(L, n_layers, H, W, rects0, n0, mx, my, 0, rects, cap, n_rects, dxy, cum_stride, hw);
}

/*
 * Exact reuse maps: Section 5's propagation applied to the set of reusable pixels itself instead of to the
 * rectangles Step 5 cut it into (Section 5 keeps a boolean map per layer anyway; Section 4 shows with its 18- against
 * 24-pixel example what every seam between two rectangles costs).  The rule per pixel is the rule Table 2 applies
 * per rectangle, a window must lie wholly inside what is reusable:
 *   tensor 0        a pixel is reusable iff its block passed Step 4 (pixels of the remainder strip never are);
 *   conv / pool     an output pixel is reusable iff every tap of its k x k window lies inside the map and is
 *                   reusable (reading: a tap in the zero padding makes it non-reusable, as a rectangle cannot reach
 *                   there; with extend_borders and zero motion such taps are ignored, as in oc_propagate_ext);
 *   LRN over pixels the same with the window of radius (k - 1) / 2; over channels: unchanged;
 *   add / concat    reusable in every input;   FC / softmax: nothing;   others: unchanged;
 * and in every tensor a pixel is only reusable if its source, the pixel at +(dx, dy) with the tensor's offset
 * (the same one offset per tensor as in oc_propagate_ext), lies inside the map.
 * masks[t] is tensor t's map [h][w] (1 = reusable), caller-allocated; dxy, cum_stride, hw as in oc_propagate_ext.
 * By construction the union of oc_propagate_ext's rectangles is a subset of these maps, with equality where
 * Step 5 yields a single rectangle.
 */
int oc_propagate_masks(const oc_layer* L, int n_layers, int H, int W, const uint8_t* block_mask, int gh, int gw,
                       int B, int mx, int my, int extend_borders, uint8_t* const* masks, int32_t* dxy,
                       int32_t* cum_stride, int32_t* hw)
{
    int ext = extend_borders && mx == 0 && my == 0;
    hw[0] = H; hw[1] = W; cum_stride[0] = 1; dxy[0] = mx; dxy[1] = my;
    for (int y = 0; y < H; ++y)
        for (int x = 0; x < W; ++x) {
            int by = y / B, bx = x / B;
            int in_grid = by < gh && bx < gw;
            int src_ok = x + mx >= 0 && x + mx < W && y + my >= 0 && y + my < H;
            masks[0][(size_t)y * W + x] = (uint8_t)(in_grid && block_mask[(size_t)by * gw + bx] && src_ok);
        }
    for (int i = 0; i < n_layers; ++i) {
        const oc_layer* l = &L[i];
        int t = i + 1, a = l->in0;
        int ha = hw[2 * a], wa = hw[2 * a + 1];
        int windowed = l->type == OC_CONV || l->type == OC_MAXPOOL || l->type == OC_AVGPOOL;
        int lrn_px = l->type == OC_LRN && l->within;
        /* taps of the window: kh x kw, dil pixels apart (a conv layer may have a kernel that is not square, or dilated) */
        int kh = windowed ? l_kh(l) : (lrn_px ? l->k : 1), kw = windowed ? l_kw(l) : (lrn_px ? l->k : 1);
        int dil = windowed ? l_dil(l) : 1;
        int s = windowed ? l->s : 1;
        int ph = windowed ? l_ph(l) : (lrn_px ? (l->k - 1) / 2 : 0), pw = windowed ? l_pw(l) : (lrn_px ? (l->k - 1) / 2 : 0);
        int ho = windowed ? (ha + 2 * l_ph(l) - l_eh(l)) / l->s + 1 : (l->type == OC_FC ? 1 : ha);
        int wo = windowed ? (wa + 2 * l_pw(l) - l_ew(l)) / l->s + 1 : (l->type == OC_FC ? 1 : wa);
        hw[2 * t] = ho; hw[2 * t + 1] = wo;
        cum_stride[t] = windowed ? cum_stride[a] * l->s : cum_stride[a];
        int dx = round_div(mx, cum_stride[t]), dy = round_div(my, cum_stride[t]);
        dxy[2 * t] = dx; dxy[2 * t + 1] = dy;
        const uint8_t* ma = masks[a];
        uint8_t* mt = masks[t];
        for (int y = 0; y < ho; ++y)
            for (int x = 0; x < wo; ++x) {
                int ok;
                if (l->type == OC_FC || l->type == OC_SOFTMAX) {
                    ok = 0;
                } else if (l->type == OC_ADD) {
                    ok = ma[(size_t)y * wa + x] && masks[l->in1][(size_t)y * wa + x];
                } else if (l->type == OC_CONCAT) {
                    int ids[OC_MAX_CONCAT], m = concat_inputs(l, ids);
                    ok = 1;
                    for (int j = 0; j < m; ++j) ok = ok && masks[ids[j]][(size_t)y * wa + x];
                } else {
                    ok = 1;
                    for (int ky = 0; ky < kh && ok; ++ky)
                        for (int kx = 0; kx < kw && ok; ++kx) {
                            int iy = y * s - ph + ky * dil, ix = x * s - pw + kx * dil;
                            if (iy < 0 || iy >= ha || ix < 0 || ix >= wa) { if (!ext) ok = 0; continue; }
                            ok = ma[(size_t)iy * wa + ix];
                        }
                }
                int src_ok = x + dx >= 0 && x + dx < wo && y + dy >= 0 && y + dy < ho;
                mt[(size_t)y * wo + x] = (uint8_t)(ok && src_ok);
            }
    }
    return 0;
}

/* Boolean map of Section 5 "Reuse", step 2: 1 where the pixel lies in a rectangle. */
void oc_rasterize(const oc_rect* rects, int n, int H, int W, uint8_t* mask)
{
    memset(mask, 0, (size_t)H * W);
    for (int i = 0; i < n; ++i)
        for (int y = rects[i].y; y < rects[i].y + rects[i].h; ++y)
            for (int x = rects[i].x; x < rects[i].x + rects[i].w; ++x)
                mask[(size_t)y * W + x] = 1;
}

/* ------------------------------------------------------------------ */
/* storage rounding                                                   */
/* ------------------------------------------------------------------ */

/* fp32 -> bf16 (round to nearest, ties to even), returned as a float whose low
 * 16 bits are zero.  Finite inputs only (NaN is passed through quietly). */
float oc_round_bf16(float v)
{
    uint32_t u;
    memcpy(&u, &v, 4);
    if ((u & 0x7f800000u) == 0x7f800000u) { u &= 0xffff0000u; if (v != v) u |= 0x00400000u; }
    else {
        uint32_t lsb = (u >> 16) & 1u;
        u += 0x7fffu + lsb;
        u &= 0xffff0000u;
    }
    float r;
    memcpy(&r, &u, 4);
    return r;
}

static float store_val(double acc, int bf16)
{
    float f = (float)acc;
    return bf16 ? oc_round_bf16(f) : f;
}

void oc_round_bf16_array(float* a, size_t n)
{
    for (size_t i = 0; i < n; ++i) a[i] = oc_round_bf16(a[i]);
}

/* network input: (u8 - 128) / 128, exact in fp32 and in bf16 */
void oc_frame_to_tensor(const uint8_t* frame, size_t n, float* out)
{
    for (size_t i = 0; i < n; ++i) out[i] = (float)((int)frame[i] - 128) / 128.0f;
}

/* ------------------------------------------------------------------ */
/* Section 5 "Reuse": cache-aware convolution                         */
/* ------------------------------------------------------------------ */

/*
 * out[y][x][:] = cache_prev[y+dy][x+dx][:]                 where mask[y][x] = 1   (step 1)
 *              = bias + sum_{ky,kx,ci} in * w  (+ReLU; relu == 2: leaky, v < 0 -> 0.1 v)  elsewhere   (step 3)
 * mask == NULL (or cache_prev == NULL) means: compute every pixel.
 * in [Hin][Win][cin], out [Hout][Wout][cout], w [cout][k][k][cin].
 */
void oc_conv_cached2(const float* in, int Hin, int Win, int cin,
                     const float* w, const float* bias, int cout, int kh, int kw, int s, int ph, int pw, int dil, int relu,
                     const float* cache_prev, const uint8_t* mask, int dx, int dy,
                     int bf16, float* out);
void oc_conv_cached(const float* in, int Hin, int Win, int cin,
                    const float* w, const float* bias, int cout, int k, int s, int p, int relu,
                    const float* cache_prev, const uint8_t* mask, int dx, int dy,
                    int bf16, float* out)
{
    oc_conv_cached2(in, Hin, Win, cin, w, bias, cout, k, k, s, p, p, 1, relu, cache_prev, mask, dx, dy, bf16, out);
}
/* The same with a kernel of kh rows x kw columns, paddings ph / pw and taps dil pixels apart: w [cout][kh][kw][cin],
 * out[y][x] = sum over (ky, kx) of in[y s - ph + ky dil][x s - pw + kx dil] * w[.][ky][kx]. */
void oc_conv_cached2(const float* in, int Hin, int Win, int cin,
                     const float* w, const float* bias, int cout, int kh, int kw, int s, int ph, int pw, int dil, int relu,
                     const float* cache_prev, const uint8_t* mask, int dx, int dy,
                     int bf16, float* out)
{
    int Hout = (Hin + 2 * ph - ((kh - 1) * dil + 1)) / s + 1, Wout = (Win + 2 * pw - ((kw - 1) * dil + 1)) / s + 1;
#pragma omp parallel for schedule(dynamic)
    for (int y = 0; y < Hout; ++y)
        for (int x = 0; x < Wout; ++x) {
            float* o = out + ((size_t)y * Wout + x) * cout;
            if (mask && cache_prev && mask[(size_t)y * Wout + x]) {
                const float* c = cache_prev + ((size_t)(y + dy) * Wout + (x + dx)) * cout;
                for (int co = 0; co < cout; ++co) o[co] = c[co];
                continue;
            }
            for (int co = 0; co < cout; ++co) {
                double acc = bias ? (double)bias[co] : 0.0;
                for (int ky = 0; ky < kh; ++ky) {
                    int iy = y * s - ph + ky * dil;
                    if (iy < 0 || iy >= Hin) continue;
                    for (int kx = 0; kx < kw; ++kx) {
                        int ix = x * s - pw + kx * dil;
                        if (ix < 0 || ix >= Win) continue;
                        const float* ip = in + ((size_t)iy * Win + ix) * cin;
                        const float* wp = w + (((size_t)co * kh + ky) * kw + kx) * cin;
                        for (int ci = 0; ci < cin; ++ci) acc += (double)ip[ci] * (double)wp[ci];
                    }
                }
                if (relu == 2) { if (acc < 0.0) acc *= 0.1; }      /* leaky ReLU, slope 0.1 (Darknet-style stacks) */
                else if (relu && acc < 0.0) acc = 0.0;
                o[co] = store_val(acc, bf16);
            }
        }
}

/* max pooling over the in-bounds part of each window (never cached: Section 5) */
void oc_maxpool(const float* in, int Hin, int Win, int C, int k, int s, int p, float* out)
{
    int Hout = (Hin + 2 * p - k) / s + 1, Wout = (Win + 2 * p - k) / s + 1;
#pragma omp parallel for schedule(static)
    for (int y = 0; y < Hout; ++y)
        for (int x = 0; x < Wout; ++x)
            for (int c = 0; c < C; ++c) {
                float m = -INFINITY;
                for (int ky = 0; ky < k; ++ky) {
                    int iy = y * s - p + ky;
                    if (iy < 0 || iy >= Hin) continue;
                    for (int kx = 0; kx < k; ++kx) {
                        int ix = x * s - p + kx;
                        if (ix < 0 || ix >= Win) continue;
                        float v = in[((size_t)iy * Win + ix) * C + c];
                        if (v > m) m = v;
                    }
                }
                out[((size_t)y * Wout + x) * C + c] = m;
            }
}

void oc_add(const float* a, const float* b, size_t n, int relu, int bf16, float* out)
{
    for (size_t i = 0; i < n; ++i) {
        double v = (double)a[i] + (double)b[i];
        if (relu && v < 0.0) v = 0.0;
        out[i] = store_val(v, bf16);
    }
}

void oc_relu(const float* a, size_t n, float* out)
{
    for (size_t i = 0; i < n; ++i) out[i] = a[i] > 0.0f ? a[i] : 0.0f;
}

/* Average pooling over the in-bounds part of each window (reading: the divisor counts the elements inside the
 * map; the models of Table 3 only average without padding, where every convention agrees). */
void oc_avgpool(const float* in, int Hin, int Win, int C, int k, int s, int p, int bf16, float* out)
{
    int Hout = (Hin + 2 * p - k) / s + 1, Wout = (Win + 2 * p - k) / s + 1;
#pragma omp parallel for schedule(static)
    for (int y = 0; y < Hout; ++y)
        for (int x = 0; x < Wout; ++x)
            for (int c = 0; c < C; ++c) {
                double sum = 0.0;
                int cnt = 0;
                for (int ky = 0; ky < k; ++ky) {
                    int iy = y * s - p + ky;
                    if (iy < 0 || iy >= Hin) continue;
                    for (int kx = 0; kx < k; ++kx) {
                        int ix = x * s - p + kx;
                        if (ix < 0 || ix >= Win) continue;
                        sum += (double)in[((size_t)iy * Win + ix) * C + c];
                        ++cnt;
                    }
                }
                out[((size_t)y * Wout + x) * C + c] = store_val(cnt ? sum / cnt : 0.0, bf16);
            }
}

/*
 * Local response normalisation (the layer of Table 2's LRN row; the paper gives no arithmetic, the reading is the
 * published definition of Krizhevsky et al. 2012 with the window average used by Caffe-style engines):
 *   out = in / (kappa + alpha / n * S)^beta
 * S = sum of squares over the window, zeros outside the tensor; window = `size` channels centred on the element's
 * channel at the same pixel (n = size), or size x size pixels centred on the element in its channel (n = size^2).
 */
void oc_lrn(const float* in, int H, int W, int C, int size, int within, double alpha, double beta, double kappa,
            int bf16, float* out)
{
    int r = (size - 1) / 2;
#pragma omp parallel for schedule(static)
    for (int y = 0; y < H; ++y)
        for (int x = 0; x < W; ++x)
            for (int c = 0; c < C; ++c) {
                double S = 0.0;
                if (within) {
                    for (int yy = y - r; yy <= y + r; ++yy)
                        for (int xx = x - r; xx <= x + r; ++xx) {
                            if (yy < 0 || yy >= H || xx < 0 || xx >= W) continue;
                            double v = in[((size_t)yy * W + xx) * C + c];
                            S += v * v;
                        }
                } else {
                    for (int cc = c - r; cc <= c + r; ++cc) {
                        if (cc < 0 || cc >= C) continue;
                        double v = in[((size_t)y * W + x) * C + cc];
                        S += v * v;
                    }
                }
                double n = within ? (double)size * size : (double)size;
                double v = (double)in[((size_t)y * W + x) * C + c] / pow(kappa + alpha / n * S, beta);
                out[((size_t)y * W + x) * C + c] = store_val(v, bf16);
            }
}

/* Concatenation along the channel axis: pixel by pixel, the channels of input 0, then of input 1, ... */
void oc_concat(const float* const* ins, const int32_t* cs, int n_in, size_t n_pixels, float* out)
{
    int ctot = 0;
    for (int j = 0; j < n_in; ++j) ctot += cs[j];
    for (size_t px = 0; px < n_pixels; ++px) {
        int off = 0;
        for (int j = 0; j < n_in; ++j) {
            for (int c = 0; c < cs[j]; ++c) out[px * ctot + off + c] = ins[j][px * cs[j] + c];
            off += cs[j];
        }
    }
}

/* Fully-connected layer over the whole input tensor, flattened in storage order (row, column, channel):
 * out[o] = bias[o] + sum_i w[o][i] in[i]. */
void oc_fc(const float* in, size_t K, const float* w, const float* bias, int cout, int relu, int bf16, float* out)
{
#pragma omp parallel for schedule(static)
    for (int o = 0; o < cout; ++o) {
        double acc = bias ? (double)bias[o] : 0.0;
        for (size_t i = 0; i < K; ++i) acc += (double)w[(size_t)o * K + i] * (double)in[i];
        if (relu && acc < 0.0) acc = 0.0;
        out[o] = store_val(acc, bf16);
    }
}

/* Softmax over the channels of each pixel: exp(v_c) / sum_j exp(v_j), evaluated after subtracting the largest
 * element (which leaves the quotient unchanged). */
void oc_softmax(const float* in, size_t n_pixels, int C, int bf16, float* out)
{
    for (size_t px = 0; px < n_pixels; ++px) {
        const float* v = in + px * C;
        double m = v[0], sum = 0.0;
        for (int c = 1; c < C; ++c) if (v[c] > m) m = v[c];
        for (int c = 0; c < C; ++c) sum += exp((double)v[c] - m);
        for (int c = 0; c < C; ++c) out[px * C + c] = store_val(exp((double)v[c] - m) / sum, bf16);
    }
}

/* ------------------------------------------------------------------ */
/* whole frame through the stack (Section 3 workflow)                 */
/* ------------------------------------------------------------------ */

/*
 * One frame of one stream.
 *   frame        uint8 [H][W][C]
 *   weights/bias per layer (NULL for layers without); weights already in the
 *                storage type (the caller rounds them for bf16)
 *   rects0,n0    reusable input rectangles (Step 5 output); n0 < 0: no cache
 *                (first frame, expiry, reset) -> every pixel is computed
 *   mx,my        global motion
 *   cur[t]       tensor t of this frame (written), t = 0..n_layers
 *   prev[t]      tensor t of the previous frame (read for conv outputs only)
 *   rects,cap,n_rects,dxy,cum_stride,hw: as oc_propagate (outputs)
 *   extend_borders  the border case of oc_dt_window_ext for a stream that did not move
 * Returns 0, -1 on rect overflow.
 */
int oc_run_stack(const oc_layer* L, int n_layers, const float* const* weights,
                 const float* const* bias, const uint8_t* frame, int H, int W, int C,
                 int bf16, const oc_rect* rects0, int n0, int mx, int my,
                 float* const* cur, const float* const* prev,
                 oc_rect* rects, int cap, int32_t* n_rects, int32_t* dxy,
                 int32_t* cum_stride, int32_t* hw, int extend_borders, const uint8_t* const* exact_masks,
                 int cache_pool_add, const uint8_t* no_reuse)
{
    /* exact_masks (optional): the maps of oc_propagate_masks for this frame; the conv layers then reuse exactly
     * those pixels instead of the rectangles'.
     * cache_pool_add (with exact_masks): max-pooling and add layers use the cache like the conv layers (Section 5
     * notes that the cache extends to other layer types): where the layer's map is set the output is the previous
     * frame's output of that layer at the tensor's offset, elsewhere it is computed.
     * no_reuse (optional, [n_layers]): Section 5 restricts the cache to the layer type where it pays (a trade-off of
     * latency against overhead) and Section 6 exposes cache parameters to the application; this setting carries that
     * choice down to single layers: a conv layer whose entry is non-zero is computed in full on every frame.
     * NULL: every conv layer uses the cache, as in Section 5.  The regions are propagated through such a
     * layer as through any other conv layer: they describe what could be reused, and the layers behind it still
     * reuse it from their own caches. */
    int cached = n0 >= 0;
    int rc = oc_propagate_ext(L, n_layers, H, W, rects0, cached ? n0 : 0, cached ? mx : 0,
                              cached ? my : 0, extend_borders, rects, cap, n_rects, dxy, cum_stride, hw);
    if (rc) return rc;
    oc_frame_to_tensor(frame, (size_t)H * W * C, cur[0]);
    for (int li = 0; li < n_layers; ++li) {
        const oc_layer* l = &L[li];
        int t = li + 1, a = l->in0;
        int ha = hw[2 * a], wa = hw[2 * a + 1], ho = hw[2 * t], wo = hw[2 * t + 1];
        if (l->type == OC_CONV) {
            uint8_t* mask = NULL;
            int uses_cache = cached && !(no_reuse && no_reuse[li]);
            if (!uses_cache) {
                /* computed in full */
            } else if (cached && exact_masks) {
                mask = (uint8_t*)malloc((size_t)ho * wo);
                memcpy(mask, exact_masks[t], (size_t)ho * wo);
            } else if (cached && n_rects[t] > 0) {
                mask = (uint8_t*)malloc((size_t)ho * wo);
                oc_rasterize(rects + (size_t)t * cap, n_rects[t], ho, wo, mask);
            }
            oc_conv_cached2(cur[a], ha, wa, l->cin, weights[li], bias ? bias[li] : NULL, l->cout,
                            l_kh(l), l_kw(l), l->s, l_ph(l), l_pw(l), l_dil(l), l->relu, mask ? prev[t] : NULL, mask,
                            dxy[2 * t], dxy[2 * t + 1], bf16, cur[t]);
            free(mask);
        } else if (l->type == OC_MAXPOOL) {
            oc_maxpool(cur[a], ha, wa, l->cin, l->k, l->s, l->p, cur[t]);
        } else if (l->type == OC_ADD) {
            oc_add(cur[a], cur[l->in1], (size_t)ho * wo * l->cout, l->relu, bf16, cur[t]);
        }
        if (cached && exact_masks && cache_pool_add && (l->type == OC_MAXPOOL || l->type == OC_ADD)) {
            int dx = dxy[2 * t], dy = dxy[2 * t + 1];
            for (int y = 0; y < ho; ++y)
                for (int x = 0; x < wo; ++x)
                    if (exact_masks[t][(size_t)y * wo + x])
                        memcpy(cur[t] + ((size_t)y * wo + x) * l->cout,
                               prev[t] + ((size_t)(y + dy) * wo + (x + dx)) * l->cout, (size_t)l->cout * sizeof(float));
        }
        if (l->type == OC_CONV || l->type == OC_MAXPOOL || l->type == OC_ADD) {
            /* done above */
        } else if (l->type == OC_AVGPOOL) {
            oc_avgpool(cur[a], ha, wa, l->cin, l->k, l->s, l->p, bf16, cur[t]);
        } else if (l->type == OC_LRN) {
            oc_lrn(cur[a], ha, wa, l->cin, l->k, l->within, l->alpha, l->beta, l->kappa, bf16, cur[t]);
        } else if (l->type == OC_CONCAT) {
            int ids[OC_MAX_CONCAT], m = concat_inputs(l, ids);
            const float* ins[OC_MAX_CONCAT];
            int32_t cs[OC_MAX_CONCAT];
            for (int j = 0; j < m; ++j) { ins[j] = cur[ids[j]]; cs[j] = ids[j] == 0 ? C : L[ids[j] - 1].cout; }
            oc_concat(ins, cs, m, (size_t)ho * wo, cur[t]);
        } else if (l->type == OC_FC) {
            oc_fc(cur[a], (size_t)ha * wa * l->cin, weights[li], bias ? bias[li] : NULL, l->cout, l->relu, bf16, cur[t]);
        } else if (l->type == OC_SOFTMAX) {
            oc_softmax(cur[a], (size_t)ho * wo, l->cout, bf16, cur[t]);
        } else {
            oc_relu(cur[a], (size_t)ho * wo * l->cout, cur[t]);
        }
    }
    return 0;
}

int oc_num_threads(void)
{
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    return omp_get_max_threads();
#else
    return 1;
#endif
}
