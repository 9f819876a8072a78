/*
 * deepcache.h -- C ABI of the MI355X (gfx950) library for cache-aware CNN
 * inference over a video stream (DeepCache, arXiv 1712.01670).
 *
 * Per frame the library (1) matches blocks of the new frame against the previous
 * frame (Section 4), (2) propagates the reusable rectangles through the layer stack
 * (Section 5, Table 2) and (3) runs every convolution only on the non-reusable
 * output pixels while the rest is copied from the previous frame's cached output
 * at the matched offset (Section 5, "Reuse").
 *
 * General rules
 *  - Every function returns a status: DC_OK (0) or a negative DC_ERR_*.  Nothing
 *    throws or aborts across this boundary.  Argument errors are detected before
 *    any kernel is launched.
 *  - "dev" pointers are device (HBM) addresses, "host" pointers are host memory.
 *    The caller owns all memory.  Apart from the handles it hands out (dc_profile_*,
 *    dc_overlap_*) and a pool of host threads, the library keeps no state between
 *    calls and allocates no device memory; scratch comes in as caller-provided
 *    workspaces.
 *  - All GPU work is enqueued on `stream` (a hipStream_t passed as void*; NULL is
 *    the default stream) and is asynchronous unless stated otherwise; with an overlap
 *    handle dc_run_stack also uses the handle's own streams and makes `stream` wait
 *    for them.
 *  - Frames are uint8 [n_streams][H][W][C] with interleaved channels, left-top
 *    origin.  Feature maps are [n_streams][H][W][C] channels-last in the storage
 *    type `dtype` (DC_F32 or DC_BF16; bf16 sums are accumulated in fp32 and rounded
 *    to nearest-even once when stored).  Convolution weights are
 *    [cout][k][k][cin] in the storage type, biases are fp32 [cout].
 *  - A motion vector (dx,dy) points from a block of the current frame to its match
 *    in the previous frame: source = current + (dx,dy)  (Section 4, Steps 2-4).
 */
#ifndef DEEPCACHE_H
#define DEEPCACHE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    DC_OK = 0,
    DC_ERR_INVALID_ARG = -1,   /* a scalar argument is out of range */
    DC_ERR_NULL_PTR = -2,      /* a required pointer is NULL */
    DC_ERR_BAD_SHAPE = -3,     /* shapes are inconsistent with each other or the layer table */
    DC_ERR_UNSUPPORTED = -4,   /* valid request the kernels do not implement */
    DC_ERR_WORKSPACE = -5,     /* a workspace is too small */
    DC_ERR_CAPACITY = -6,      /* a caller-provided list is too short (counts are still reported) */
    DC_ERR_HIP = -7            /* a HIP runtime call failed */
};

enum { DC_F32 = 0, DC_BF16 = 1 };
/* Layer types: the rows of Table 2.  Only DC_CONV is cached (Section 5); the others are computed in full. */
enum { DC_CONV = 0, DC_MAXPOOL = 1, DC_RELU = 2, DC_ADD = 3, DC_LRN = 4, DC_CONCAT = 5, DC_FC = 6, DC_SOFTMAX = 7,
       DC_AVGPOOL = 8 };

/* Rectangle in the pixel grid of one tensor, left-top origin (Section 3). */
typedef struct { int32_t x, y, w, h; } dc_rect;

/* One layer of the stack.  Tensor 0 is the network input (the frame mapped to
 * (u8-128)/128; it has the cin of the layers that read it, which may exceed the frame's
 * channel count: the extra channels are zero, so that a 3-channel frame can feed a first
 * layer whose weights are laid out with a 16-byte channel run); tensor i+1 is the output
 * of layer i.  in0 (and in1 for DC_ADD, in1..in3 for DC_CONCAT)
 * name producer tensors, so the table describes a DAG in topological order.
 *   DC_LRN      out = in / (kappa + alpha / n * S)^beta, S = sum of squares over a window centred on the element,
 *               zeros outside the tensor: k channels at the same pixel (within = 0, n = k) or k x k pixels of the
 *               same channel (within = 1, n = k * k); k odd, cin == cout.
 *   DC_CONCAT   channels of in0, then in1, then in2, in3 (each -1: absent; in3 needs in2) at every pixel;
 *               cout = sum of the producers' channels (cin repeats cout), equal spatial sizes.
 *   DC_FC       out[o] = bias[o] + sum_i w[o][i] in[i] over the whole producer tensor flattened in storage order
 *               (row, column, channel); weights [cout][H*W*cin], output tensor 1 x 1 x cout, optional fused ReLU.
 *   DC_SOFTMAX  over the channels of every pixel; cin == cout.
 *   DC_AVGPOOL  mean over the in-bounds part of each k x k window (stride s, padding p); cin == cout. */
typedef struct {
    int32_t type;          /* DC_CONV ... DC_AVGPOOL */
    int32_t k, s, p;       /* kernel size, stride, zero padding (conv, pool); k: window size of an LRN */
    int32_t cin, cout;
    int32_t relu;          /* fused ReLU after a conv, an add or a fully-connected layer; DC_CONV also takes 2:
                              leaky ReLU, v < 0 -> 0.1 v (Darknet-style stacks) */
    int32_t in0, in1;
    int32_t in2, in3;      /* DC_CONCAT: third and fourth producer, -1: none (other types ignore them) */
    int32_t within;        /* DC_LRN: 0 = window over channels, 1 = window over pixels */
    float alpha, beta, kappa;   /* DC_LRN */
    /* DC_CONV only (other types ignore them).  k2 > 0: the kernel has k rows and k2 columns, with padding p along y
     * and p2 along x (weights [cout][k][k2][cin]); k2 == 0: k x k with padding p on both axes.  dil > 1: the taps are
     * dil pixels apart (the kernel spans (k - 1) dil + 1 pixels).  Table 2's conv row applies with that span per axis;
     * the exact maps look at the taps themselves. */
    int32_t k2, p2, dil;
} dc_layer;

/* Reusable regions of one tensor of one stream (Section 5 "Propagation"):
 * pixels inside `rects` equal the previous frame's tensor at +(dx,dy). */
typedef struct {
    dc_rect* rects;        /* host, caller-provided storage */
    int32_t capacity;      /* length of `rects` */
    int32_t n;             /* out: number of rectangles (may exceed capacity on DC_ERR_CAPACITY) */
    int32_t dx, dy;        /* out: source offset in this tensor's pixels */
    int32_t cum_stride;    /* out: product of strides from the input to this tensor */
    int32_t h, w;          /* out: spatial size of this tensor */
} dc_regions;

/* Which search dc_run_stack uses in Step 2 of the matching (Section 4; Section 7.6 compares them). */
enum { DC_MATCH_EXHAUSTIVE = 0, DC_MATCH_DIAMOND = 1 };
typedef struct {
    int32_t method;        /* DC_MATCH_EXHAUSTIVE (dc_match_blocks) or DC_MATCH_DIAMOND (dc_match_blocks_ds) */
    int32_t k_skip;        /* >= 1: Step 2 runs only for blocks whose grid row and column are multiples of k */
    int32_t extend_borders;  /* dc_run_stack only; not a matching option.  0: Table 2 as printed.  1: for a stream
                              whose global motion is (0,0), the taps of a window that fall into the zero padding
                              need not lie in the rectangle (they read zeros in both frames), so a rectangle that
                              touches a side of the map keeps the outputs along that side: an extension beyond
                              the paper's table for static cameras (dc_propagate_regions_opt) */
    int32_t exact_masks;   /* dc_run_stack only, with device_plan (DC_ERR_UNSUPPORTED without).  0: reusable regions are
                              the rectangles of Step 5, propagated by Table 2.  1: the same rule per pixel (see
                              dc_propagate_masks): exact reuse maps, which lose nothing at the seams between
                              rectangles.  No rectangle lists exist then (regions_out reports empty lists). */
    int32_t cache_pool_add; /* dc_run_stack only, with exact_masks (DC_ERR_UNSUPPORTED without).  1: max-pooling and add layers
                              use the cache like the conv layers (Section 5: the cache extends to other layer types): where
                              the layer's map is set the output is the previous frame's output of that layer at the tensor's
                              offset, elsewhere it is computed.  tensors_prev must then hold those layers' previous outputs
                              (distinct buffers), and their channel runs must be whole 16-byte vectors. */
    const uint8_t* no_reuse; /* dc_run_stack only.  NULL, or host [n_layers]: a conv layer whose entry is non-zero does not use
                              the cache: it is computed in full on every frame (nothing copied, every unit listed).  The
                              regions are propagated through it as through any conv layer, and the layers behind it
                              still reuse from their own caches.  Section 5 restricts the cache to the layer type where
                              it pays; this carries that choice down to single layers (on this GPU a 1x1 layer or a
                              layer with few input channels costs less to compute than to copy). */
    int32_t torus;         /* dc_run_stack only, with device_plan.  1: the conv outputs are kept on a torus and never copied.
                              Every conv output is ONE buffer for all frames (tensors_prev[t] == tensors_cur[t]); pixel
                              (x, y) of stream s lies at ((x + ox) mod w, (y + oy) mod h) of it, and the origin (ox, oy)
                              moves with every cached frame by the tensor's offset (dx, dy), so that a reusable pixel
                              already lies where this frame looks for it: a cached frame writes its non-reusable
                              pixels only (Section 5 "Reuse" without step 1).  A full frame writes every tensor at
                              its buffer's start (origins (0, 0)).  The values are those of the copying path.  Only
                              stacks whose conv layers are 3x3 / stride 1 with whole 64-byte channel rows, 1x1 /
                              stride 1 with whole 16-byte channel rows and a multiple of 8 output channels (or a
                              first layer on a 16-byte pixel vector) and whose conv outputs are read by such layers or by
                              2x2 / stride-2 max-pooling qualify (DC_ERR_UNSUPPORTED otherwise); every other tensor
                              is stored as always.  Together with cache_pool_add the outputs of the max-pooling layers
                              (every one of them must then be such a 2x2 pooling of a conv output, read by conv layers
                              only; no add layers) are single buffers on a torus as well, and a pooled pixel whose map
                              bit is set is simply left alone.  A caller that reads a tensor kept on a torus (the stack's
                              output, if a conv layer ends it) goes through dc_torus_read (origins_dev_out) or
                              origins_out.  Calls on one workspace pair must not overlap: the next frame starts from
                              the origins this one leaves there. */
    int32_t* origins_out;  /* optional with torus: host [n_streams][n_layers + 1][2], receives (ox, oy) of every tensor
                              after a cached frame (for inspection: the call then waits for the planning) */
    const int32_t** origins_dev_out; /* optional with torus: host pointer that receives the DEVICE address of this frame's
                              origins, [n_streams][n_layers + 1][2] inside ws_dev (NULL after a full frame: every origin
                              is (0, 0)).  Nothing waits.  The array is written by the frame's planning, which precedes
                              its layers, and stays in place until the third dc_run_stack call from this one: pass
                              it (plus 2 * tensor) to dc_torus_read on the call's stream to get a tensor in its
                              logical layout. */
    int32_t device_plan;   /* dc_run_stack only.  0: the call waits for the matching, then merges, propagates and lists
                              the dirty units on the host.  1: three small kernels do that on the GPU from the block
                              mask in device memory (Section 4 Step 5, Section 5 "Propagation": the same rules, the
                              same lists), so that a cached frame needs no host wait; the convolutions are launched
                              for the longest possible list and read its length from memory.  Then
                               - a rectangle list may hold min(max_rects, 256) entries,
                               - the work counters of the frame arrive later: see dc_stack_stats_fetch,
                               - regions_out, if given, makes the call wait for the lists (inspection only),
                               - in_place frames are not available (the request is ignored when in_place is given),
                               - the tail of ws_host keeps the counters between the call and dc_stack_stats_fetch.
                              Grids of more than 64 x 64 blocks and stacks of more than 191 layers or 128
                              convolutions are planned on the host as with 0. */
} dc_match_options;

/* Work counters of one dc_run_stack call, summed over streams. */
typedef struct {
    int32_t full;               /* 1: every pixel was computed (no cache used) */
    int32_t n_blocks;           /* blocks in the grid, all streams */
    int32_t n_reusable_blocks;  /* blocks that passed Step 4 */
    int32_t n_overflow_streams; /* streams one of whose rectangle lists exceeded max_rects: they reuse nothing in this
                                   frame (every pixel computed, always valid), their lists are reported empty */
    int64_t macs_full;          /* conv multiply-adds of a full frame */
    int64_t macs_needed;        /* multiply-adds of the non-reusable output pixels */
    int64_t macs_issued;        /* multiply-adds of every pixel of every dirty tile (what ran) */
    int64_t copy_bytes;         /* bytes read plus bytes written by the shifted copies */
    int64_t* layer_reused_px;   /* optional host [n_layers]: reused output pixels per conv layer */
    int64_t* layer_issued_macs; /* optional host [n_layers] */
    int32_t* layer_kernel_id;   /* optional host [n_layers]: which GEMM instantiation ran (-1: none) */
    void* profile;              /* optional dc_profile handle with >= 2*n_layers slots: slot i brackets
                                   the GEMM kernel of conv layer i, slot n_layers+i its shifted copy; when the copies
                                   of all layers run as one launch, slot n_layers brackets that launch */
} dc_stack_stats;

const char* dc_status_string(int32_t status);

/*
 * Kernel timing with HIP events (measurement aid, not part of the method).  A profile
 * owns 2*n_slots events; a slot that brackets a kernel launch is recorded on the launch
 * stream.  dc_profile_elapsed_ms may be called after the stream has been synchronised;
 * it returns DC_ERR_INVALID_ARG for a slot that was not recorded since the last
 * dc_profile_reset.
 */
int32_t dc_profile_create(int32_t n_slots, void** profile);
int32_t dc_profile_destroy(void* profile);
int32_t dc_profile_reset(void* profile);
int32_t dc_profile_elapsed_ms(void* profile, int32_t slot, float* ms);

/*
 * Measurement aid: the bf16 matrix-core rate this GPU sustains (TFLOP/s) for the instruction stream of the
 * convolution kernels' inner loop, v_mfma_f32_16x16x32_bf16 on 4 x 4 tiles per wavefront, eight wavefronts on each
 * of 256 CUs, operands in registers (lds_reads = 0) or re-read from LDS every step as the kernels do (1).  Thirty
 * launches of about 0.3 ms run back to back and the last one is timed with HIP events, so the figure is the rate at
 * the clock the part settles at under its power limit, which is what a kernel can reach instead of the published
 * peak.  scratch_dev: at least 4 MiB of device memory (overwritten).  The call waits for the launches.
 */
int32_t dc_probe_mfma_rate(int32_t lds_reads, void* scratch_dev, size_t scratch_bytes, double* tflops, void* stream);

/*
 * Overlap handle (Section 7.6: matching and inference can run asynchronously): streams and
 * events owned by the library object.  Passed to dc_run_stack,
 *  - the matching of a frame runs on a stream of its own, next to whatever is still queued of
 *    the previous frame, and only the matching is waited for (without a handle the call waits
 *    for the caller's stream);
 *  - with dc_overlap_pipeline(handle, 2) two frames are in flight: consecutive calls enqueue
 *    their layers on two alternating internal streams, layer i of a frame waiting for layer i of
 *    the previous frame (its cache) and for the previous frame's readers of any tensor it
 *    overwrites.  The caller's stream is made to wait for the end of the frame, so synchronising
 *    it still yields the frame's results.  In this mode the inputs (frames, weights) must be
 *    complete in memory when the call is made, and the caller's own streams must be done with the
 *    tensors handed over; the device workspace holds two sets of plans and scratch.
 * Callers that may not create streams simply pass no handle.
 */
int32_t dc_overlap_create(void** overlap);
/*
 * Look-ahead matching (Section 7.6): starts Steps 1-4 for the NEXT frame on the handle's matching
 * stream and returns at once, so that the dc_run_stack call for that frame finds the mask and the
 * motion already in host memory instead of waiting for them.  Call it after the dc_run_stack call of
 * the current frame, with the arguments the next dc_run_stack call will pass (frames_next as its
 * frames_cur, frames_cur as its frames_prev, the same match buffers and host workspace): the very
 * next dc_run_stack call with the handle uses the result if every one of them is the same and
 * otherwise matches again itself; any later call ignores it.  Both frames must be complete in memory
 * and stay unchanged until that call; the match buffers and the head of ws_host are written from now
 * on (the previous frame's mv / mask are overwritten early).  Not needed before a frame that is
 * computed in full.  Errors as dc_match_blocks_opt; DC_ERR_WORKSPACE if ws_host is too small.
 */
int32_t dc_prefetch_match(void* overlap, const uint8_t* frames_next, const uint8_t* frames_cur,
                          int32_t n_streams, int32_t H, int32_t W, int32_t C, int32_t block, int32_t radius,
                          uint32_t max_block_ssd, const dc_match_options* match_options,
                          int16_t* mv, uint32_t* best_ssd, int32_t* global_mv, int32_t* n_pass,
                          uint8_t* block_mask, void* ws_host, size_t ws_host_bytes);
int32_t dc_overlap_destroy(void* overlap);
int32_t dc_overlap_pipeline(void* overlap, int32_t frames_in_flight /* 1 or 2 */);

/*
 * Overrides the launch heuristics of the 3x3 stride-1 GEMM kernels for the whole process (tests and
 * experiments; results do not depend on it beyond fp32 summation order): wavefront arrangement
 * (0: 64 channels per workgroup; bf16 only: 1: 128 channels, 2: 64 channels in two blocks per wavefront,
 * 3: the persistent kernel with the weights in registers, 64 input channels only, 4: 128 channels on twelve
 * wavefronts with 13..18 units per workgroup), units per workgroup
 * (1..18; for the 1x1 kernel 4 or 8 selects its 64 x 64 or 128 x 128 tile), number of workgroups that split K,
 * channel chunk index (0, 1).  A negative value leaves that choice to the library; values a layer cannot use are
 * ignored for that layer.
 */
int32_t dc_conv_tuning(int32_t arrangement, int32_t units_per_workgroup, int32_t k_split, int32_t chunk_index);

/* Name of a GEMM kernel instantiation (as a profiler prints it, without namespace and
 * argument list) for an id reported in dc_stack_stats.layer_kernel_id. */
int32_t dc_conv_kernel_name(int32_t kernel_id, char* buf, size_t n);

/* Granularity of the dirty-tile list of a conv layer: th x tw output pixels per list entry
 * (nt and cfg are informational). */
int32_t dc_conv_tile_shape(const dc_layer* layer, int32_t n_streams, int32_t Hin, int32_t Win,
                           int32_t dtype, int32_t* th, int32_t* tw, int32_t* nt, int32_t* cfg);

/*
 * Section 4, Steps 1-4 (block grid, exhaustive search of Section 7.6, mean motion,
 * re-test) for n_streams independent frame pairs.
 *   cur, prev      dev u8 [n_streams][H][W][C]
 *   block          block edge B in pixels; the grid is gh x gw = H/B x W/B (integer
 *                  division; a remainder strip is never reusable)
 *   radius         R: candidates |dx|,|dy| <= R whose window lies inside the previous frame
 *   max_block_ssd  a block matches iff its sum of squared differences over all
 *                  B*B*C samples is <= this bound (PSNR above a threshold, Section 4)
 *   mv             dev i16 [n_streams][gh][gw][2]  best (dx,dy); ties go to the smallest
 *                  (ssd, |dx|+|dy|, dy, dx)
 *   best_ssd       dev u32 [n_streams][gh][gw]
 *   global_mv      dev i32 [n_streams][2]  mean of the passing blocks' vectors per axis,
 *                  rounded to nearest, halves away from zero; (0,0) if none passes
 *   n_pass         dev i32 [n_streams]     number of passing blocks (K of Step 3)
 *   block_mask     dev u8  [n_streams][gh][gw]  1 iff the block at +global_mv is inside
 *                  the previous frame and within the bound (Step 4); all 0 if K = 0
 * Limits: B*C <= 256, R <= 127, (B+2R)*((B+2R)*C+16) <= 60 KiB.
 */
int32_t dc_match_blocks(const uint8_t* cur, const uint8_t* prev, int32_t n_streams,
                        int32_t H, int32_t W, int32_t C, int32_t block, int32_t radius,
                        uint32_t max_block_ssd, int16_t* mv, uint32_t* best_ssd,
                        int32_t* global_mv, int32_t* n_pass, uint8_t* block_mask,
                        void* stream);

/*
 * Section 4, Steps 1-4 with the search the paper runs in Step 2, the diamond search it cites,
 * and the k-skip acceleration of the same section.  Arguments as dc_match_blocks, plus
 *   k_skip   k >= 1: Step 2 runs only for the blocks whose grid row and grid column are both
 *            multiples of k; Step 3 averages over those; Step 4 still tests every block.
 *            A block that is not searched gets mv = (0,0) and best_ssd = 2^32 - 1.
 * The search: centre (0,0); evaluate the centre and the eight points at (0,+-2), (+-2,0),
 * (+-1,+-1) around it; if the centre is best evaluate the four points at (0,+-1), (+-1,0)
 * and take the best of the five, otherwise move the centre to the best point and repeat.
 * A point is usable iff |dx|,|dy| <= radius and its window lies inside the previous frame;
 * the best point is the one with the smallest (ssd, position in the pattern), the centre first
 * and the others in raster order (dy, then dx), so the centre moves only to a strictly smaller
 * sum.  The result is a local minimum and may differ from dc_match_blocks (Section 7.6 compares
 * the two).  Re-using Step 2's sums in Step 4 (same section) changes no result; Step 4 reads
 * 6 bytes per pixel here and is not worth a table.
 * Limits: radius <= 16383, block*block*C*255^2 < 2^32, block*W*C < 2^31.
 */
int32_t dc_match_blocks_ds(const uint8_t* cur, const uint8_t* prev, int32_t n_streams,
                           int32_t H, int32_t W, int32_t C, int32_t block, int32_t radius,
                           int32_t k_skip, uint32_t max_block_ssd, int16_t* mv,
                           uint32_t* best_ssd, int32_t* global_mv, int32_t* n_pass,
                           uint8_t* block_mask, void* stream);

/*
 * Steps 1-4 with the search and the k-skip of `options` (NULL: exhaustive search, every block):
 * dc_match_blocks and dc_match_blocks_ds in one call, plus k-skip for the exhaustive search (the
 * acceleration of Section 4 does not depend on the search in Step 2; skipped blocks report
 * mv = (0,0), best_ssd = 2^32 - 1 as in dc_match_blocks_ds).  Limits as for the chosen search.
 */
int32_t dc_match_blocks_opt(const uint8_t* cur, const uint8_t* prev, int32_t n_streams,
                            int32_t H, int32_t W, int32_t C, int32_t block, int32_t radius,
                            const dc_match_options* options, uint32_t max_block_ssd, int16_t* mv,
                            uint32_t* best_ssd, int32_t* global_mv, int32_t* n_pass,
                            uint8_t* block_mask, void* stream);

/*
 * Section 4 Step 5 and Section 5 "Propagation" for one stream; pure host integer code.
 *   block_mask     host u8 [gh][gw] (Step 4 result)
 *   mx, my         global motion of the stream
 *   regions        host [n_layers+1], one entry per tensor; `rects`/`capacity` are
 *                  inputs, the rest is written
 * Merge: row-major scan; at the first set unclaimed block grow right over set unclaimed
 * blocks, then down while the whole run is set and unclaimed.  Conv and pool map a
 * rectangle to the largest output rectangle whose k x k windows lie inside it
 * (Table 2; x' = ceil((x+p)/s), last column floor((x+w-k+p)/s)); DC_ADD takes pairwise
 * overlaps (Table 2, concat row) and DC_CONCAT the overlap of one rectangle from each of its
 * inputs; DC_LRN over pixels shrinks a rectangle by its radius on every side (Table 2, LRN row:
 * x+r, y+r, w-2r, h-2r), over channels it has no extent in the pixel grid and changes nothing;
 * DC_AVGPOOL follows the pooling row; after DC_FC or DC_SOFTMAX nothing is reusable (their row
 * is the empty rectangle); DC_RELU leaves rectangles unchanged.  Every tensor has
 * one source offset round(M / cum_stride) (halves away from zero) and rectangles are
 * clipped so that their source stays inside the map.
 * Returns DC_ERR_CAPACITY if a list overflowed (n is exact, stored rects are truncated).
 */
int32_t dc_propagate_regions(const dc_layer* layers, int32_t n_layers, int32_t H, int32_t W,
                             int32_t block, const uint8_t* block_mask, int32_t gh, int32_t gw,
                             int32_t mx, int32_t my, dc_regions* regions);
/* The same with the border case of dc_match_options.extend_borders (applied only when mx == my == 0). */
int32_t dc_propagate_regions_opt(const dc_layer* layers, int32_t n_layers, int32_t H, int32_t W,
                                 int32_t block, const uint8_t* block_mask, int32_t gh, int32_t gw,
                                 int32_t mx, int32_t my, int32_t extend_borders, dc_regions* regions);

/*
 * Packed weights (a layout choice of this library, not part of the method): the weights of a
 * 3x3 stride-1 layer with cout % 64 == 0 and cin * element size % 64 == 0, re-laid as
 * [cout/16][cin*es/64][3*3][16][64 bytes], so that the 64-byte channel runs the GEMM kernel
 * stages per load instruction are contiguous in memory and whole cache lines are used (the
 * strided runs of [cout][k][k][cin] use half of every line they touch).  The weights are constant
 * over a video, so they are packed once.
 *   dc_packed_weights_bytes  size of the packed copy; 0: the layer has no packed form
 *   dc_pack_conv_weights     weights dev [cout][3][3][cin] -> packed dev, both 16-byte aligned, distinct;
 *                            DC_ERR_BAD_SHAPE for a layer without a packed form
 * A packed copy passed to dc_cached_conv_layer / dc_run_stack next to the plain weights is used
 * where the kernel chosen for the layer reads it; results are identical bit for bit.
 */
int32_t dc_packed_weights_bytes(const dc_layer* layer, int32_t dtype, size_t* bytes);
int32_t dc_pack_conv_weights(const dc_layer* layer, const void* weights, int32_t dtype,
                             void* packed, void* stream);

/* Bytes of device / host workspace dc_cached_conv_layer needs for the given shape. */
int32_t dc_conv_workspace_bytes(const dc_layer* layer, int32_t n_streams, int32_t Hin,
                                int32_t Win, int32_t max_rects_per_stream,
                                size_t* dev_bytes, size_t* host_bytes);

/*
 * Section 5 "Reuse": cache-aware forward of one convolution layer (the paper's
 * c_forward(top, bottom, c_blob, c_regions)).
 *   in          dev [n_streams][Hin][Win][cin]       current input map (complete)
 *   weights     dev [cout][k][k][cin], bias dev fp32 [cout] or NULL
 *   packed_weights  dev, optional (NULL): the result of dc_pack_conv_weights for `weights`
 *   cache_prev  dev [n_streams][Hout][Wout][cout]    this layer's output for the previous frame
 *   out         dev [n_streams][Hout][Wout][cout]    written completely; must not alias cache_prev
 *   regions     host [n_streams]: reusable rectangles of the OUTPUT tensor and their source
 *               offset; NULL (or cache_prev NULL) computes every pixel
 * Pixels inside a rectangle receive cache_prev at +(dx,dy); every other pixel receives
 * conv(+bias)(+ReLU).  The GEMM runs over a compacted list of tiles that contain at
 * least one non-reusable pixel; reusable pixels inside such tiles still get the copy.
 *   ws_dev      dev workspace, ws_host host staging (pinned memory recommended); the
 *               staging must stay untouched until the stream has passed this call
 */
int32_t dc_cached_conv_layer(const dc_layer* layer, const void* in, const void* weights,
                             const void* packed_weights, const float* bias, const void* cache_prev, void* out,
                             int32_t n_streams, int32_t Hin, int32_t Win,
                             const dc_regions* regions, int32_t dtype,
                             void* ws_dev, size_t ws_dev_bytes,
                             void* ws_host, size_t ws_host_bytes, void* stream);

/*
 * dc_cached_conv_layer for callers that cannot allocate device memory or keep workspaces for the library: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments without the workspaces,
 * same result.  The call allocates nothing, on the device or the host: its scratch (the layer's plan and the partial
 * sums of a split K) is a 16 MiB array in device memory that belongs to the library on every GPU it runs on, until
 * the process ends; the rectangles travel as kernel arguments and the dirty-unit list is built on the GPU.  Limits
 * (errors before anything is launched): n_streams <= 32 and at most 128 rectangles over all streams
 * (DC_ERR_CAPACITY); a plan of at most 6 MiB, about 18 bytes per 4x4 output unit and stream, i.e. 340 k units
 * (DC_ERR_WORKSPACE).  Every call on a GPU uses that GPU's one array: calls that overlap in time on one GPU (two
 * streams, two threads) race on it; calls on one stream do not.
 */
int32_t dc_cached_conv_layer_noalloc(const dc_layer* layer, const void* in, const void* weights,
                                     const void* packed_weights, const float* bias, const void* cache_prev, void* out,
                                     int32_t n_streams, int32_t Hin, int32_t Win,
                                     const dc_regions* regions, int32_t dtype, void* stream);

/* Un-cached layers (Section 5: only convolutions use the cache), whole map every frame. */
/* out[pixel][c] = (frames[pixel][c] - 128) / 128 for c < c_frame, 0 for c_frame <= c < c_tensor. */
int32_t dc_frame_to_tensor(const uint8_t* frames, void* out, size_t n_pixels, int32_t c_frame,
                           int32_t c_tensor, int32_t dtype, void* stream);
/* A tensor kept on a torus (dc_match_options.torus) in its logical layout:
 * out[s][y][x][:] = in[s][(y + oy) mod H][(x + ox) mod W][:] with (ox, oy) = origins_dev[s * origin_stride + 0 / 1].
 * in, out: dev [n_streams][H][W][C] in `dtype`, distinct buffers; origins_dev: dev, or NULL for a plain copy (the
 * tensors of a full frame); origin_stride: ints between the entries of consecutive streams (2 * (n_layers + 1) for
 * the array dc_run_stack reports through origins_dev_out, offset by 2 * tensor).  n_streams * H <= 65535.
 * For the callers of dc_run_stack with torus: Section 5's cached feature maps stay where they are, this is the one
 * place where a reader gets them as the paper's layout has them. */
int32_t dc_torus_read(const void* in, void* out, const int32_t* origins_dev, int32_t origin_stride, int32_t n_streams,
                      int32_t H, int32_t W, int32_t C, int32_t dtype, void* stream);
int32_t dc_maxpool_layer(const void* in, void* out, int32_t n_streams, int32_t Hin, int32_t Win,
                         int32_t C, int32_t k, int32_t s, int32_t p, int32_t dtype, void* stream);
int32_t dc_add_layer(const void* a, const void* b, void* out, size_t n, int32_t relu,
                     int32_t dtype, void* stream);
/* The layer types of Table 2 besides convolution and pooling, and average pooling (arithmetic: see dc_layer).
 * All pointers dev; tensors [n_streams][H][W][C] in `dtype`; results are rounded once when stored.
 *   dc_lrn_layer      size odd >= 1
 *   dc_concat_layer   ins: host array of n_in (2..4) dev pointers, channels: host array of their channel counts;
 *                     out [n_pixels][sum of channels]; out must not alias an input
 *   dc_fc_layer       in [n_streams][K], weights [cout][K], bias fp32 [cout] or NULL, out [n_streams][cout]
 *   dc_softmax_layer  in, out [n_pixels][C] */
int32_t dc_avgpool_layer(const void* in, void* out, int32_t n_streams, int32_t Hin, int32_t Win,
                         int32_t C, int32_t k, int32_t s, int32_t p, int32_t dtype, void* stream);
int32_t dc_lrn_layer(const void* in, void* out, int32_t n_streams, int32_t H, int32_t W, int32_t C, int32_t size,
                     int32_t within, float alpha, float beta, float kappa, int32_t dtype, void* stream);
int32_t dc_concat_layer(const void* const* ins, const int32_t* channels, int32_t n_in, void* out, size_t n_pixels,
                        int32_t dtype, void* stream);
int32_t dc_fc_layer(const void* in, const void* weights, const float* bias, void* out, int32_t n_streams, size_t K,
                    int32_t cout, int32_t relu, int32_t dtype, void* stream);
int32_t dc_softmax_layer(const void* in, void* out, size_t n_pixels, int32_t C, int32_t dtype, void* stream);

/* Workspace sizes for dc_run_stack. */
int32_t dc_stack_workspace_bytes(const dc_layer* layers, int32_t n_layers, int32_t n_streams,
                                 int32_t H, int32_t W, int32_t C, int32_t block,
                                 int32_t max_rects_per_stream,
                                 size_t* dev_bytes, size_t* host_bytes);

/*
 * One frame of every stream through the whole path (Section 3 workflow): match,
 * merge, propagate, then per layer shifted copy + convolution of dirty tiles, with
 * pooling / add / ReLU layers computed in full.
 *   weights, bias   host arrays [n_layers] of dev pointers (NULL for non-conv layers)
 *   packed_weights  optional (NULL) host array [n_layers] of dev pointers: packed copies of the
 *                   weights (NULL entries for layers without one)
 *   frames_cur      dev u8 [n_streams][H][W][C]
 *   frames_prev     dev u8, previous frames (cache keys); ignored when force_full
 *   tensors_cur     host array [n_layers+1] of dev pointers, every tensor of this frame
 *                   (written).  Conv outputs are the cache values of the next frame.  The other
 *                   tensors may be the same buffers for every frame; with a pipelined overlap
 *                   handle a caller that alternates them between two sets as well saves the
 *                   library one cross-stream wait and one event per such tensor and frame.
 *   tensors_prev    host array [n_layers+1] of dev pointers: the previous frame's tensors;
 *                   only conv-layer outputs are read.  Must not alias tensors_cur for them.
 *                   Written only in an in-place frame (see in_place).
 *   match_options   optional (NULL: exhaustive search over every block)
 *   force_full      nonzero: first frame, cache expiry (Section 5) or reset: skip matching
 *                   and compute everything
 *   in_place        optional host (NULL: never).  When the global motion of every stream is (0,0)
 *                   (a static camera), every reusable pixel of every conv output already holds its
 *                   value in the previous frame's buffer, so the frame is computed in place: the
 *                   conv layers write their non-reusable pixels into the buffers of tensors_prev,
 *                   nothing is copied, and *in_place is set to 1.  The frame's conv outputs are then
 *                   the tensors_prev buffers (the other tensors are in tensors_cur as always), and
 *                   the caller passes the same two sets in the same roles for the next frame
 *                   instead of swapping them.  The values are the same as without it.  Otherwise 0.
 *   mv .. block_mask  dev buffers as in dc_match_blocks (written unless force_full)
 *   max_rects       most rectangles a tensor's list may hold; a stream one of whose lists would be longer reuses
 *                   nothing in this frame (every pixel of it is computed; counted in stats->n_overflow_streams)
 *   regions_out     optional host [n_streams][n_layers+1] with caller-provided rect storage of at least
 *                   max_rects entries each (DC_ERR_CAPACITY otherwise, before anything is launched); receives
 *                   every tensor's regions (for inspection); may be NULL
 *   ws_dev, ws_host workspaces of at least dc_stack_workspace_bytes; ws_host should be pinned
 *   stats           optional host; for a frame planned on the GPU (dc_match_options.device_plan) only full,
 *                   n_blocks, macs_full and layer_kernel_id are filled by the call itself
 *   overlap         optional dc_overlap handle; with it the frames must be visible to any stream
 *                   when the call is made (the matching does not wait for the main stream)
 * The call waits once for the matching (the region logic runs on the host): for the main
 * stream without an overlap handle, for the handle's stream with one; everything after that
 * is asynchronous.  With four or more streams the per-stream host work (merge, propagation,
 * tile classification) is spread over a pool of at most 16 host threads that the library
 * creates on first use and keeps; concurrent calls from several threads are serialised.
 */
int32_t dc_run_stack(const dc_layer* layers, int32_t n_layers,
                     const void* const* weights, const void* const* packed_weights,
                     const float* const* bias,
                     const uint8_t* frames_cur, const uint8_t* frames_prev,
                     void* const* tensors_cur, void* const* tensors_prev,
                     int32_t n_streams, int32_t H, int32_t W, int32_t C, int32_t dtype,
                     int32_t block, int32_t radius, uint32_t max_block_ssd,
                     const dc_match_options* match_options, int32_t force_full, int32_t* in_place,
                     int16_t* mv, uint32_t* best_ssd, int32_t* global_mv, int32_t* n_pass,
                     uint8_t* block_mask, int32_t max_rects, dc_regions* regions_out,
                     void* ws_dev, size_t ws_dev_bytes, void* ws_host, size_t ws_host_bytes,
                     dc_stack_stats* stats, void* overlap, void* stream);

/*
 * Section 5 "Propagation" per pixel: exact reuse maps of every tensor of the stack, on the GPU.  Table 2 maps a
 * reusable rectangle to the outputs whose windows lie wholly inside it; applied to the set of reusable pixels itself
 * (the union of the blocks that passed Step 4) the rule reads: an output pixel is reusable iff every tap of its
 * window lies inside the map and is reusable (taps in the zero padding are not; with extend_borders they are ignored
 * for a stream whose motion is (0,0)); add / concat: reusable in every input; LRN over pixels: its window; FC and
 * softmax: nothing; and in every tensor only pixels whose source at +(dx, dy) = round(M / cumulative stride) lies
 * inside the map.  The maps contain Step 5's propagated rectangles and lose nothing at the seams between them
 * (Section 4 counts 18 against 24 pixels for two 5x5 blocks under a 3x3 kernel).
 *   block_mask, global_mv   dev, as written by dc_match_blocks
 *   bitmaps    dev out [n_streams][words_per_stream]: tensor t of a stream starts at word tensor_offset[t]; row y is
 *              (w + 31) / 32 words, pixel x is bit x % 32 of word x / 32; bits beyond the row are 0
 *   dxy        dev out [n_streams][n_layers + 1][2]: source offset of every tensor
 *   ws_dev     at least ws_dev_bytes of dc_propagate_masks_size plus 4 * n_streams * (n_layers + 3) bytes
 * dc_propagate_masks_size: words of one stream's bitmaps, optionally every tensor's first word (host [n_layers + 1]),
 * and the workspace bytes.  The call waits once for its layer tables to be on the device (it is meant for
 * inspection and tests; dc_run_stack runs the same kernels without a wait when dc_match_options.exact_masks is set).
 */
int32_t dc_propagate_masks_size(const dc_layer* layers, int32_t n_layers, int32_t H, int32_t W, int32_t C,
                                size_t* words_per_stream, int64_t* tensor_offset, size_t* ws_dev_bytes);
int32_t dc_propagate_masks(const dc_layer* layers, int32_t n_layers, int32_t n_streams, int32_t H, int32_t W, int32_t C,
                           int32_t block, const uint8_t* block_mask, const int32_t* global_mv, int32_t extend_borders,
                           uint32_t* bitmaps, int32_t* dxy, void* ws_dev, size_t ws_dev_bytes, void* stream);

/*
 * Work counters of the most recent dc_run_stack call that planned its frame on the GPU with this host workspace
 * (Section 7.2 reports the saving per scenario; these are the quantities it depends on).  Call it after the stream
 * has been synchronised: the planning kernels write the counters into ws_host (directly if it is pinned memory,
 * else through a copy on the stream).  Fills every field of `stats` but `profile` and `layer_kernel_id`, and the
 * per-layer arrays if their pointers are set (same ws_host and ws_host_bytes as in that call).
 * DC_ERR_INVALID_ARG if the workspace holds no such frame.
 */
int32_t dc_stack_stats_fetch(const void* ws_host, size_t ws_host_bytes, dc_stack_stats* stats);

#ifdef __cplusplus
}
#endif
#endif /* DEEPCACHE_H */
