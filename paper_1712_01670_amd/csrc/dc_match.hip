// Block matching (Section 4, Steps 1-4) for gfx950.
//
// Kernel 1 (search): one workgroup per block of the grid.  The search window of the
// previous frame and the block of the current frame are staged in LDS with coalesced
// dword loads; every lane owns a few candidate vectors and evaluates
//     SSD = sum a^2 + sum b^2 - 2 sum a*b
// four samples per instruction with packed-u8 dot products; the arg-min key
// (ssd, |dx|+|dy|, dy, dx) is packed in 64 bits and reduced with wavefront shuffles.
// Kernel 2 (motion + re-test): every workgroup recomputes the stream's mean motion
// from the per-block results (a few hundred values) and re-tests its own block.
#include "dc_internal.h"

namespace dc {

namespace {

constexpr int kSearchThreads = 512;

__device__ __forceinline__ uint32_t udot4(uint32_t a, uint32_t b, uint32_t c) {
    return __builtin_amdgcn_udot4(a, b, c, false);
}

__device__ __forceinline__ unsigned long long wave_min_u64(unsigned long long v) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        unsigned long long o = __shfl_xor(v, off, 64);
        v = o < v ? o : v;
    }
    return v;
}

// LDS layout (bytes):
//   win : (B+2R) rows of `ws` bytes; row r holds previous-frame bytes
//         [a0, a0+ws) of frame row y0-R+r, a0 = 4-byte-aligned start at or below the
//         window's first byte; bytes outside the frame are zero
//   blk : B rows of `cs` bytes (cs = B*C rounded up to 4), zero padded
// CDW > 0: the block row is CDW dwords (compile-time, inner loop fully unrolled so that the LDS reads of a
// row are issued together); CDW == 0: any row length.
template <bool ALIGNED, int CDW>
__global__ __launch_bounds__(kSearchThreads) void match_search_kernel(
    const uint8_t* __restrict__ cur, const uint8_t* __restrict__ prev, int H, int W, int C, int B,
    int R, int gw, int gh, int ws, int cs, int16_t* __restrict__ mv, uint32_t* __restrict__ best_ssd) {
    extern __shared__ __align__(16) uint8_t lds[];
    const int tid = threadIdx.x;
    const int blk_id = blockIdx.x, stream = blockIdx.y;
    const int bx = blk_id % gw, by = blk_id / gw;
    const int x0 = bx * B, y0 = by * B;
    const int rows = B + 2 * R;
    const int row_bytes = W * C;
    const size_t frame_bytes = (size_t)H * row_bytes;
    const uint8_t* pf = prev + (size_t)stream * frame_bytes;
    const uint8_t* cf = cur + (size_t)stream * frame_bytes;
    uint8_t* win = lds;
    uint8_t* blk = lds + (size_t)rows * ws;
    __shared__ unsigned long long red[kSearchThreads / 64];

    const int gx0 = (x0 - R) * C;        // first window byte within the frame row (may be < 0)
    const int a0 = gx0 & ~3;             // aligned start (two's complement floor)
    const int skew = gx0 - a0;

    // ---- stage the search window ----
    const int wdw = ws / 4;
    for (int i = tid; i < rows * wdw; i += kSearchThreads) {
        int r = i / wdw, j = i - r * wdw;
        int y = y0 - R + r;
        int fb = a0 + 4 * j;
        uint32_t v = 0;
        if (y >= 0 && y < H) {
            const uint8_t* src = pf + (size_t)y * row_bytes;
            if (ALIGNED && fb >= 0 && fb + 3 < row_bytes) {
                v = *reinterpret_cast<const uint32_t*>(src + fb);
            } else {
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    int f = fb + b;
                    if (f >= 0 && f < row_bytes) v |= (uint32_t)src[f] << (8 * b);
                }
            }
        }
        reinterpret_cast<uint32_t*>(win)[i] = v;
    }
    // ---- stage the current block, zero padded to whole dwords ----
    const int cdw = CDW > 0 ? CDW : cs / 4;
    const int blk_bytes = B * C;
    for (int i = tid; i < B * cdw; i += kSearchThreads) {
        int r = i / cdw, j = i - r * cdw;
        const uint8_t* src = cf + (size_t)(y0 + r) * row_bytes + (size_t)x0 * C;
        uint32_t v = 0;
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            int f = 4 * j + b;
            if (f < blk_bytes) v |= (uint32_t)src[f] << (8 * b);
        }
        reinterpret_cast<uint32_t*>(blk)[i] = v;
    }
    __syncthreads();

    // sum a^2 (every lane computes it: B*cdw broadcast reads)
    uint32_t saa = 0;
    for (int i = 0; i < B * cdw; ++i) {
        uint32_t a = reinterpret_cast<const uint32_t*>(blk)[i];
        saa = udot4(a, a, saa);
    }
    const int tail = blk_bytes - 4 * (cdw - 1);                 // valid bytes of a row's last dword
    const uint32_t tail_mask = tail >= 4 ? 0xffffffffu : ((1u << (8 * tail)) - 1u);

    const int side = 2 * R + 1;
    unsigned long long best = ~0ull;
    for (int c = tid; c < side * side; c += kSearchThreads) {
        int dy = c / side - R, dx = c - (c / side) * side - R;
        if (x0 + dx < 0 || y0 + dy < 0 || x0 + dx + B > W || y0 + dy + B > H) continue;
        const int boff = skew + (dx + R) * C;   // byte offset of the candidate inside a window row
        const int sh = boff & 3;
        uint32_t sab = 0, sbb = 0;
        for (int r = 0; r < B; ++r) {
            const uint32_t* wrow = reinterpret_cast<const uint32_t*>(win + (size_t)(r + dy + R) * ws) + (boff >> 2);
            const uint32_t* arow = reinterpret_cast<const uint32_t*>(blk + (size_t)r * cs);
            if (CDW > 0) {
                uint32_t wv[CDW + 1], av[CDW > 0 ? CDW : 1];
#pragma unroll
                for (int j = 0; j <= CDW; ++j) wv[j] = wrow[j];
#pragma unroll
                for (int j = 0; j < CDW; ++j) av[j] = arow[j];
#pragma unroll
                for (int j = 0; j < CDW; ++j) {
                    uint32_t b = __builtin_amdgcn_alignbyte(wv[j + 1], wv[j], sh);
                    if (j == CDW - 1) b &= tail_mask;
                    sab = udot4(av[j], b, sab);
                    sbb = udot4(b, b, sbb);
                }
            } else {
                uint32_t lo = wrow[0];
                for (int j = 0; j < cdw; ++j) {
                    uint32_t hi = wrow[j + 1];
                    uint32_t b = __builtin_amdgcn_alignbyte(hi, lo, sh);
                    if (j == cdw - 1) b &= tail_mask;
                    uint32_t a = arow[j];
                    sab = udot4(a, b, sab);
                    sbb = udot4(b, b, sbb);
                    lo = hi;
                }
            }
        }
        uint32_t ssd = saa + sbb - 2u * sab;
        int ad = (dx < 0 ? -dx : dx) + (dy < 0 ? -dy : dy);
        unsigned long long key = ((unsigned long long)ssd << 32) | ((unsigned long long)ad << 16) |
                                 ((unsigned long long)(dy + R) << 8) | (unsigned long long)(dx + R);
        best = key < best ? key : best;
    }
    best = wave_min_u64(best);
    if ((tid & 63) == 0) red[tid >> 6] = best;
    __syncthreads();
    if (tid == 0) {
#pragma unroll
        for (int i = 1; i < kSearchThreads / 64; ++i) best = red[i] < best ? red[i] : best;
        size_t o = (size_t)stream * gh * gw + blk_id;
        mv[2 * o + 0] = (int16_t)((int)(best & 0xff) - R);
        mv[2 * o + 1] = (int16_t)((int)((best >> 8) & 0xff) - R);
        best_ssd[o] = (uint32_t)(best >> 32);
    }
}

__device__ __forceinline__ int wave_sum_i32(int v) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

__device__ __forceinline__ int round_half_away(int num, int den) {
    int mag = num < 0 ? -num : num;
    int q = (2 * mag + den) / (2 * den);
    return num < 0 ? -q : q;
}

// One wavefront per block: Step 3 (redundantly per workgroup) then Step 4 for this block.
__global__ __launch_bounds__(64) void motion_retest_kernel(
    const uint8_t* __restrict__ cur, const uint8_t* __restrict__ prev, int H, int W, int C, int B,
    int gw, int gh, uint32_t max_ssd, const int16_t* __restrict__ mv,
    const uint32_t* __restrict__ best_ssd, int32_t* __restrict__ gmv, int32_t* __restrict__ n_pass,
    uint8_t* __restrict__ mask) {
    const int lane = threadIdx.x;
    const int blk_id = blockIdx.x, stream = blockIdx.y;
    const int nb = gh * gw;
    const int16_t* smv = mv + (size_t)stream * nb * 2;
    const uint32_t* sbest = best_ssd + (size_t)stream * nb;
    int sx = 0, sy = 0, K = 0;
    for (int i = lane; i < nb; i += 64) {
        if (sbest[i] <= max_ssd) {
            sx += smv[2 * i];
            sy += smv[2 * i + 1];
            ++K;
        }
    }
    sx = wave_sum_i32(sx);
    sy = wave_sum_i32(sy);
    K = wave_sum_i32(K);
    int mx = 0, my = 0;
    if (K > 0) {
        mx = round_half_away(sx, K);
        my = round_half_away(sy, K);
    }
    if (blk_id == 0 && lane == 0) {
        gmv[2 * stream] = mx;
        gmv[2 * stream + 1] = my;
        n_pass[stream] = K;
    }
    const int bx = blk_id % gw, by = blk_id / gw;
    const int x0 = bx * B, y0 = by * B;
    bool inside = K > 0 && x0 + mx >= 0 && y0 + my >= 0 && x0 + mx + B <= W && y0 + my + B <= H;
    uint32_t ssd = 0;
    if (inside) {
        const size_t frame_bytes = (size_t)H * W * C;
        const uint8_t* cf = cur + stream * frame_bytes;
        const uint8_t* pf = prev + stream * frame_bytes;
        const int rb = B * C;
        for (int i = lane; i < B * rb; i += 64) {
            int r = i / rb, j = i - r * rb;
            int a = cf[((size_t)(y0 + r) * W + x0) * C + j];
            int b = pf[((size_t)(y0 + my + r) * W + x0 + mx) * C + j];
            ssd += (uint32_t)((a - b) * (a - b));
        }
        ssd = (uint32_t)wave_sum_i32((int)ssd);
    }
    if (lane == 0) mask[(size_t)stream * nb + blk_id] = (inside && ssd <= max_ssd) ? 1 : 0;
}

}  // namespace

hipError_t launch_match(const uint8_t* cur, const uint8_t* prev, int n_streams, int H, int W, int C,
                        int B, int R, uint32_t max_ssd, int16_t* mv, uint32_t* best_ssd,
                        int32_t* gmv, int32_t* n_pass, uint8_t* mask, hipStream_t st) {
    const int gh = H / B, gw = W / B;
    const int rows = B + 2 * R;
    const int ws = (int)align_up((size_t)rows * C + 3, 4) + 8;  // skew (<=3) + window + over-read of the last dword pair
    const int cs = (int)align_up((size_t)B * C, 4);
    const size_t lds = (size_t)rows * ws + (size_t)B * cs;
    const bool aligned = ((reinterpret_cast<uintptr_t>(prev) & 3) == 0) && ((W * C) % 4 == 0);
    dim3 grid(gh * gw, n_streams);
#define DC_MATCH_LAUNCH(AL, CD)                                                                                      \
    hipLaunchKernelGGL((match_search_kernel<AL, CD>), grid, dim3(kSearchThreads), lds, st, cur, prev, H, W, C, B, R, \
                       gw, gh, ws, cs, mv, best_ssd)
#define DC_MATCH_ALIGN(CD)             \
    do {                               \
        if (aligned) DC_MATCH_LAUNCH(true, CD); \
        else DC_MATCH_LAUNCH(false, CD);        \
    } while (0)
    switch (cs / 4) {
        case 6: DC_MATCH_ALIGN(6); break;     // 8x8x3
        case 8: DC_MATCH_ALIGN(8); break;     // 10x10x3, 8x8x4
        case 12: DC_MATCH_ALIGN(12); break;   // 16x16x3
        case 16: DC_MATCH_ALIGN(16); break;   // 16x16x4
        default: DC_MATCH_ALIGN(0); break;
    }
#undef DC_MATCH_ALIGN
#undef DC_MATCH_LAUNCH
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(motion_retest_kernel, grid, dim3(64), 0, st, cur, prev, H, W, C, B, gw, gh,
                       max_ssd, mv, best_ssd, gmv, n_pass, mask);
    return hipGetLastError();
}

}  // namespace dc
