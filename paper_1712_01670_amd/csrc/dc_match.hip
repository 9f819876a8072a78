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
#include <cstdlib>

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

// Sum over the 64 lanes, returned to every lane.  Data-parallel-primitive moves instead of LDS permutes (a
// dependent chain of six permutes costs more than a round of the diamond search should): within quads by
// quad permutation, within a row of 16 by row shifts, across rows by broadcasting lane 15 / lane 31 into
// the following rows; lanes without a source add zero.  The total ends up in lane 63.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ int dpp_add(int v) {
    return v + __builtin_amdgcn_update_dpp(0, v, CTRL, ROW_MASK, 0xf, false);
}
__device__ __forceinline__ int wave_sum_i32(int v) {
    v = dpp_add<0xb1, 0xf>(v);    // quad_perm [1,0,3,2]
    v = dpp_add<0x4e, 0xf>(v);    // quad_perm [2,3,0,1]
    v = dpp_add<0x114, 0xf>(v);   // row_shr:4
    v = dpp_add<0x118, 0xf>(v);   // row_shr:8
    v = dpp_add<0x142, 0xa>(v);   // row_bcast:15 into rows 1 and 3
    v = dpp_add<0x143, 0xc>(v);   // row_bcast:31 into rows 2 and 3
    return __builtin_amdgcn_readlane(v, 63);
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
    int R, int gw, int gh, int ws, int cs, int k_skip, int16_t* __restrict__ mv, uint32_t* __restrict__ best_ssd) {
    extern __shared__ __align__(16) uint8_t lds[];
    const int tid = threadIdx.x;
    // k-skip: the grid covers only the blocks on every k-th grid row and column
    const int lgw = (gw + k_skip - 1) / k_skip;
    const int bx = ((int)blockIdx.x % lgw) * k_skip, by = ((int)blockIdx.x / lgw) * k_skip;
    const int blk_id = by * gw + bx, stream = blockIdx.y;
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

// ---- search on the matrix cores ----------------------------------------------------------
// SSD = sum a'^2 + sum b'^2 - 2 sum a'b' with a' = a - 128, b' = b - 128 (signed bytes; the offset
// cancels in a - b).  The cross term of all candidates of a block is one integer GEMM per window row
// wr:  X[dx][dy] += A_wr[dx][k] * B_wr[k][dy],  k = byte within the block row,
//   A_wr[dx][k] = window row wr, byte C*dx + k          (the block-wide run that candidate dx sees)
//   B_wr[k][dy] = block row wr - dy, byte k              (zero if that is not a row of the block)
// (dx, dy count from -R), so that the sum over the window rows is the cross term of candidate
// (dx, dy).  v_mfma_i32_16x16x64_i8 covers 16 dx x 16 dy x 64 bytes; NT x NT tiles cover the
// (2R+1)^2 candidates, KS K-steps the block row.  sum b'^2 per candidate is a box sum of per-pixel
// sums.  The wavefronts split the window rows and add their partial tiles pairwise through LDS.  The arg-min
// key is the same as in the scalar kernel, so both give identical results.
typedef int intx4 __attribute__((ext_vector_type(4)));
constexpr int kMfmaWaves = 4;           // wavefronts per block: they split the window rows and the summing loops
constexpr int kMfmaThreads = 64 * kMfmaWaves;

// BT, CT: block edge and channel count when known at compile time (the summing loops are then unrolled and
// their LDS reads issued together), 0: taken from the arguments.
template <bool ALIGNED, int NT, int KS, int BT, int CT>
__global__ __launch_bounds__(kMfmaThreads, 7) void match_mfma_kernel(
    const uint8_t* __restrict__ cur, const uint8_t* __restrict__ prev, int H, int W, int C_rt, int B_rt,
    int R, int gw, int gh, int ws, int k_skip, int16_t* __restrict__ mv, uint32_t* __restrict__ best_ssd) {
    const int B = BT ? BT : B_rt, C = CT ? CT : C_rt;
    extern __shared__ __align__(16) uint8_t lds[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    // k-skip: the grid covers only the blocks on every k-th grid row and column
    const int lgw = (gw + k_skip - 1) / k_skip;
    const int bx = ((int)blockIdx.x % lgw) * k_skip, by = ((int)blockIdx.x / lgw) * k_skip;
    const int blk_id = by * gw + bx, stream = blockIdx.y;
    const int x0 = bx * B, y0 = by * B;
    const int rows = B + 2 * R, cols = rows, nd = 2 * R + 1;
    const int row_bytes = W * C;
    const size_t frame_bytes = (size_t)H * row_bytes;
    const uint8_t* pf = prev + (size_t)stream * frame_bytes;
    const uint8_t* cf = cur + (size_t)stream * frame_bytes;
    constexpr int BS = 64 * KS;                       // bytes of a staged block row
    // With the block shape known at compile time the row sums of squares are taken straight from the window bytes
    // and the per-pixel sums (p2) do not exist: one phase and 9 KB of LDS less (the kernel is bound by the latency of
    // its chain of phases, i.e. by how many workgroups a CU holds).
    constexpr bool kFused = BT > 0 && CT > 0 && CT <= 4 && (BT * CT) % 4 == 0;
    // LDS: [win rows*ws][blk B*BS][p2 rows*cols ints, unless kFused][h2 rows*nd ints][misc][v2 nd*nd ints]
    uint8_t* win = lds;
    uint8_t* blk = win + (size_t)rows * ws;
    int* p2 = reinterpret_cast<int*>(blk + (size_t)B * BS);
    const int n_p2 = kFused ? 0 : rows * cols;
    int* h2 = p2 + n_p2;
    int* misc = h2 + rows * nd + (4 - (n_p2 + rows * nd) % 4) % 4;   // 16-byte aligned
    // The summed tiles land at the start of LDS, over the window, the block and the sums, which are dead by then.
    int* tiles = reinterpret_cast<int*>(lds);
    unsigned long long* red = reinterpret_cast<unsigned long long*>(misc + kMfmaWaves);   // partial sums a'^2, then the arg-min keys
    int* v2 = misc + 3 * kMfmaWaves;

    const int gx0 = (x0 - R) * C;
    const int a0 = gx0 & ~3;
    const int skew = gx0 - a0;

    // ---- stage the window (signed bytes; out-of-frame bytes are never part of a valid candidate).  Only the
    // dwords that hold window bytes are fetched (the rest of a row is only read for candidates beyond the
    // search range); the loads of a thread are issued eight at a time before any of them is used ----
    // The block of the current frame is requested first and used after the window is in place, so that its load
    // travels together with the window's instead of after them (one memory latency less per block).  One dword per
    // thread; only when the block's rows are whole aligned dwords.
    const int blk_bytes = B * C;
    const bool blk_early = kFused && ALIGNED && BT * (BS / 4) <= kMfmaThreads && (reinterpret_cast<uintptr_t>(cf) & 3) == 0;
    uint32_t blk_raw = 0x80808080u;
    if (blk_early && tid < B * (BS / 4)) {
        const int r = tid / (BS / 4), j = tid - r * (BS / 4);
        if (4 * j < blk_bytes)
            blk_raw = *reinterpret_cast<const uint32_t*>(cf + (size_t)(y0 + r) * row_bytes + (size_t)x0 * C + 4 * j);
    }
    const int wdw = ws / 4;
    const int ldw = (skew + cols * C + 3) / 4;        // dwords per row that hold window bytes
    for (int base = 0; base < rows * ldw; base += 8 * kMfmaThreads) {
        uint32_t v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int i = base + u * kMfmaThreads + tid;
            const int r = i / ldw, j = i - r * ldw;
            const int y = y0 - R + r;
            const int fb = a0 + 4 * j;
            v[u] = 0x80808080u;
            if (i < rows * ldw && y >= 0 && y < H) {
                const uint8_t* src = pf + (size_t)y * row_bytes;
                if (ALIGNED && fb >= 0 && fb + 3 < row_bytes) {
                    v[u] = *reinterpret_cast<const uint32_t*>(src + fb);
                } else {
                    uint32_t t = 0;
#pragma unroll
                    for (int b = 0; b < 4; ++b) {
                        const int f = fb + b;
                        t |= (uint32_t)((f >= 0 && f < row_bytes) ? src[f] : 128) << (8 * b);
                    }
                    v[u] = t;
                }
            }
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int i = base + u * kMfmaThreads + tid;
            const int r = i / ldw, j = i - r * ldw;
            if (i < rows * ldw) reinterpret_cast<uint32_t*>(win)[r * wdw + j] = v[u] ^ 0x80808080u;
        }
    }
    for (int i = tid; i < rows * (wdw - ldw); i += kMfmaThreads) {   // the tail of every row: any defined value
        const int r = i / (wdw - ldw), j = ldw + (i - r * (wdw - ldw));
        reinterpret_cast<uint32_t*>(win)[r * wdw + j] = 0;
    }
    // ---- stage the block: signed bytes, true zeros behind the row so that the padding adds nothing ----
    int saa = 0;
    if (blk_early) {
        if (tid < B * (BS / 4)) {       // a dword outside the row arrives as 0x80808080: zeros once the offset is taken off
            const uint32_t v = blk_raw ^ 0x80808080u;
            saa = __builtin_amdgcn_sdot4((int)v, (int)v, 0, false);
            reinterpret_cast<uint32_t*>(blk)[tid] = v;
        }
    } else {
        for (int i = tid; i < B * (BS / 4); i += kMfmaThreads) {
            const int r = i / (BS / 4), j = i - r * (BS / 4);
            const uint8_t* src = cf + (size_t)(y0 + r) * row_bytes + (size_t)x0 * C;
            uint32_t v = 0;
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                const int f = 4 * j + b;
                if (f < blk_bytes) {
                    const int a = (int)src[f] - 128;
                    saa += a * a;
                    v |= (uint32_t)(a & 0xff) << (8 * b);
                }
            }
            reinterpret_cast<uint32_t*>(blk)[i] = v;
        }
    }
    saa = wave_sum_i32(saa);
    __syncthreads();
    if (lane == 0) misc[wave] = saa;

    // ---- box sums of squares over the block: B columns (h2), then B rows (v2) ----
    if constexpr (kFused) {
        // h2[r][d] = sum of squares of the BT * CT window bytes of row r that candidate d sees.  A thread takes four
        // neighbouring d: it aligns the bytes it needs once, sums the first run with byte dot products and slides it
        // three times by one pixel (CT bytes enter, CT leave).
        constexpr int NB = BT * CT;                                 // bytes of a block row
        constexpr int NA = (NB + 3 * CT + 3) / 4;                   // aligned dwords that hold NB + 3 CT bytes
        constexpr uint32_t kPix = CT == 4 ? 0xffffffffu : (1u << (8 * CT)) - 1u;
        const int ng = (nd + 3) / 4;
        for (int i = tid; i < rows * ng; i += kMfmaThreads) {
            const int r = i / ng, d0 = 4 * (i - r * ng);
            const int o0 = skew + CT * d0;
            const uint32_t* w32 = reinterpret_cast<const uint32_t*>(win + (size_t)r * ws) + (o0 >> 2);
            const int sh = o0 & 3;
            uint32_t raw[NA + 1], al[NA + 1];
#pragma unroll
            for (int k = 0; k <= NA; ++k) raw[k] = w32[k];
#pragma unroll
            for (int k = 0; k < NA; ++k) al[k] = __builtin_amdgcn_alignbyte(raw[k + 1], raw[k], sh);
            al[NA] = 0;
            int sq = 0;
#pragma unroll
            for (int k = 0; k < NB / 4; ++k) sq = __builtin_amdgcn_sdot4((int)al[k], (int)al[k], sq, false);
            h2[r * nd + d0] = sq;
#pragma unroll
            for (int q = 1; q < 4; ++q) {
                const int tin = NB + CT * (q - 1), tout = CT * (q - 1);       // first byte entering / leaving
                const uint32_t vin = __builtin_amdgcn_alignbyte(al[tin / 4 + 1], al[tin / 4], tin % 4) & kPix;
                const uint32_t vout = __builtin_amdgcn_alignbyte(al[tout / 4 + 1], al[tout / 4], tout % 4) & kPix;
                sq += __builtin_amdgcn_sdot4((int)vin, (int)vin, 0, false) - __builtin_amdgcn_sdot4((int)vout, (int)vout, 0, false);
                if (d0 + q < nd) h2[r * nd + d0 + q] = sq;
            }
        }
    } else {
        const int8_t* swin = reinterpret_cast<const int8_t*>(win);
        for (int i = tid; i < rows * cols; i += kMfmaThreads) {
            const int r = i / cols, x = i - r * cols;
            const int8_t* px = swin + (size_t)r * ws + skew + x * C;
            int s = 0;
#pragma unroll
            for (int c = 0; c < C; ++c) s += (int)px[c] * (int)px[c];
            p2[i] = s;
        }
        __syncthreads();
        for (int i = tid; i < rows * nd; i += kMfmaThreads) {
            const int r = i / nd, d = i - r * nd;
            int s = 0;
#pragma unroll
            for (int x = 0; x < B; ++x) s += p2[r * cols + d + x];
            h2[i] = s;
        }
    }
    __syncthreads();
    if constexpr (BT > 0) {
        // a thread takes eight candidates dy of one dx: the first sum over its B rows, then seven steps down the column
        // (one row enters, one leaves): 2 B - 2 + 16 reads for eight sums instead of 8 B
        const int nch = (nd + 7) / 8;
        for (int i = tid; i < nd * nch; i += kMfmaThreads) {
            const int ch = i / nd, dxi = i - ch * nd, dy0 = 8 * ch;
            int s = 0;
#pragma unroll
            for (int r = 0; r < BT; ++r) s += h2[(dy0 + r) * nd + dxi];
            v2[dy0 * nd + dxi] = s;
#pragma unroll
            for (int q = 1; q < 8; ++q) {
                if (dy0 + q >= nd) break;
                s += h2[(dy0 + q + BT - 1) * nd + dxi] - h2[(dy0 + q - 1) * nd + dxi];
                v2[(dy0 + q) * nd + dxi] = s;
            }
        }
    } else {
        for (int i = tid; i < nd * nd; i += kMfmaThreads) {
            const int dyi = i / nd, dxi = i - dyi * nd;
            int s = 0;
            for (int r = 0; r < B; ++r) s += h2[(dyi + r) * nd + dxi];
            v2[i] = s;
        }
    }

    // ---- cross terms: this wavefront's share of the window rows ----
    const int n = lane & 15, kq = lane >> 4;
    intx4 acc[NT][NT];
#pragma unroll
    for (int i = 0; i < NT; ++i)
#pragma unroll
        for (int j = 0; j < NT; ++j) acc[i][j] = intx4{0, 0, 0, 0};
    // Window row wr meets block rows only for the candidates dy with 0 <= wr - dy < B: a tile of 16 dy whose
    // block rows all fall outside is a product with zeros and is skipped (about half of the tiles).  The rows are
    // dealt round-robin so that every wavefront gets its share of the rows with one and with two live tiles.
    for (int wr = wave; wr < rows; wr += kMfmaWaves) {
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            intx4 af[NT], bf[NT];
#pragma unroll
            for (int i = 0; i < NT; ++i) {      // lane: candidate dx = 16 i + n, bytes [16 kq, 16 kq + 16) of its run
                const int o = skew + C * (16 * i + n) + 16 * kq + 64 * ks;
                const uint32_t* w32 = reinterpret_cast<const uint32_t*>(win + (size_t)wr * ws) + (o >> 2);
                const int sh = o & 3;
                uint32_t wv[5];
#pragma unroll
                for (int e = 0; e < 5; ++e) wv[e] = w32[e];
#pragma unroll
                for (int e = 0; e < 4; ++e) af[i][e] = (int)__builtin_amdgcn_alignbyte(wv[e + 1], wv[e], sh);
            }
#pragma unroll
            for (int j = 0; j < NT; ++j) {      // lane: candidate dy = 16 j + n, block row wr - dy
                const bool live = wr >= 16 * j && wr - 16 * j < B + 15;   // wavefront-uniform: some dy of the tile has a block row
                if (!live) continue;
                const int r = wr - (16 * j + n);
                const bool ok = r >= 0 && r < B;
                const intx4 v = *reinterpret_cast<const intx4*>(blk + (size_t)(ok ? r : 0) * BS + 64 * ks + 16 * kq);
                bf[j] = ok ? v : intx4{0, 0, 0, 0};
#pragma unroll
                for (int i = 0; i < NT; ++i)
                    acc[i][j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(af[i], bf[j], acc[i][j], 0, 0, 0);
            }
        }
    }
    // The four partial copies are added through one LDS buffer with plain 16-byte accesses (integer atomics, 36 per
    // lane, cost more): wavefront 3 stores its tiles, 2 adds them to its own and stores the sum, then 1, then 0, whose
    // sum the evaluation below reads.  A lane only ever touches its own slots, so a wavefront's reads and writes need
    // no barrier between them.  The buffer lies over the window, which is dead after the barrier (the launcher checks
    // that NT^2 KiB fit into what is dead by then).
    {
        intx4* buf = reinterpret_cast<intx4*>(tiles);
        __syncthreads();                       // every wavefront is done with the window, the block and the sums
#pragma unroll
        for (int w = kMfmaWaves - 1; w >= 0; --w) {
            if (wave == w) {
#pragma unroll
                for (int i = 0; i < NT; ++i)
#pragma unroll
                    for (int j = 0; j < NT; ++j) {
                        if (w < kMfmaWaves - 1) acc[i][j] += buf[(i * NT + j) * 64 + lane];
                        buf[(i * NT + j) * 64 + lane] = acc[i][j];
                    }
            }
            __syncthreads();
        }
    }

    // ---- SSD and arg-min: tile t is evaluated by wavefront t % kMfmaWaves; lane (n, kq) holds rows
    // dx = 16 i + 4 kq + e of column dy = 16 j + n ----
    int saa_all = 0;
#pragma unroll
    for (int w = 0; w < kMfmaWaves; ++w) saa_all += misc[w];
    unsigned long long best = ~0ull;
    for (int t = wave; t < NT * NT; t += kMfmaWaves) {
        const int i = t / NT, j = t - i * NT;
        const intx4 c = *reinterpret_cast<const intx4*>(tiles + (t * 64 + lane) * 4);
        const int dyi = 16 * j + n;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int dxi = 16 * i + 4 * kq + e;
            const int dx = dxi - R, dy = dyi - R;
            if (dxi >= nd || dyi >= nd || x0 + dx < 0 || y0 + dy < 0 || x0 + dx + B > W || y0 + dy + B > H) continue;
            const uint32_t ssd = (uint32_t)(saa_all + v2[dyi * nd + dxi] - 2 * c[e]);
            const int ad = (dx < 0 ? -dx : dx) + (dy < 0 ? -dy : dy);
            const unsigned long long key = ((unsigned long long)ssd << 32) | ((unsigned long long)ad << 16) |
                                           ((unsigned long long)dyi << 8) | (unsigned long long)dxi;
            best = key < best ? key : best;
        }
    }
    best = wave_min_u64(best);
    if (lane == 0) red[wave] = best;
    __syncthreads();
    if (tid == 0) {
#pragma unroll
        for (int w = 1; w < kMfmaWaves; ++w) best = red[w] < best ? red[w] : best;
        const size_t o = (size_t)stream * gh * gw + blk_id;
        mv[2 * o + 0] = (int16_t)((int)(best & 0xff) - R);
        mv[2 * o + 1] = (int16_t)((int)((best >> 8) & 0xff) - R);
        best_ssd[o] = (uint32_t)(best >> 32);
    }
}

__device__ __forceinline__ int round_half_away(int num, int den) {
    int mag = num < 0 ? -num : num;
    int q = (2 * mag + den) / (2 * den);
    return num < 0 ? -q : q;
}

// One wavefront per block: Step 3 (redundantly per workgroup) then Step 4 for this block.
__global__ __launch_bounds__(64) void motion_retest_kernel(
    const uint8_t* __restrict__ cur, const uint8_t* __restrict__ prev, int H, int W, int C, int B,
    int gw, int gh, uint32_t max_ssd, int16_t* mv, uint32_t* best_ssd, int32_t* __restrict__ gmv,
    int32_t* __restrict__ n_pass, uint8_t* __restrict__ mask, int k_skip) {
    const int lane = threadIdx.x;
    const int blk_id = blockIdx.x, stream = blockIdx.y;
    const int nb = gh * gw;
    int16_t* smv = mv + (size_t)stream * nb * 2;
    uint32_t* sbest = best_ssd + (size_t)stream * nb;
    int sx = 0, sy = 0, K = 0;
    for (int base = 0; base < nb; base += 4 * 64) {     // four independent loads per lane at a time
        uint32_t bs[4];
        int vx[4], vy[4];
        bool has[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int i = base + u * 64 + lane;
            // with k-skip only the blocks on every k-th grid row and column carry a vector; the entries of the others
            // are written further down by their own workgroups and are not read here
            const bool in = i < nb && (k_skip == 1 || ((i / gw) % k_skip == 0 && (i % gw) % k_skip == 0));
            has[u] = in;
            bs[u] = in ? sbest[i] : 0xffffffffu;
            vx[u] = in ? smv[2 * i] : 0;
            vy[u] = in ? smv[2 * i + 1] : 0;
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const bool pass = has[u] && bs[u] <= max_ssd;
            sx += pass ? vx[u] : 0;
            sy += pass ? vy[u] : 0;
            K += pass ? 1 : 0;
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
    if (k_skip > 1 && (bx % k_skip != 0 || by % k_skip != 0) && lane == 0) {
        // not searched: no vector (no workgroup reads these entries: the mean above leaves them out)
        smv[2 * blk_id] = 0; smv[2 * blk_id + 1] = 0;
        sbest[blk_id] = 0xffffffffu;
    }
    const int x0 = bx * B, y0 = by * B;
    bool inside = K > 0 && x0 + mx >= 0 && y0 + my >= 0 && x0 + mx + B <= W && y0 + my + B <= H;
    uint32_t ssd = 0;
    if (inside) {
        const size_t frame_bytes = (size_t)H * W * C;
        const uint8_t* cf = cur + stream * frame_bytes;
        const uint8_t* pf = prev + stream * frame_bytes;
        const int rb = B * C;
        for (int base = 0; base < B * rb; base += 8 * 64) {   // eight independent byte pairs per lane at a time
            int a[8], b[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int i = base + u * 64 + lane;
                const int r = i / rb, j = i - r * rb;
                const bool in = i < B * rb;
                a[u] = in ? cf[((size_t)(y0 + r) * W + x0) * C + j] : 0;
                b[u] = in ? pf[((size_t)(y0 + my + r) * W + x0 + mx) * C + j] : 0;
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) ssd += (uint32_t)((a[u] - b[u]) * (a[u] - b[u]));
        }
        ssd = (uint32_t)wave_sum_i32((int)ssd);
    }
    if (lane == 0) mask[(size_t)stream * nb + blk_id] = (inside && ssd <= max_ssd) ? 1 : 0;
}


// ---- diamond search (Section 4, Step 2 as the paper runs it) with k-skip ----------------------
// One wavefront per block of the grid.  The walk is sequential, so what counts is the latency of a round:
// the wavefront first copies its search window of the previous frame ((B+2R)^2 pixels) and its block into
// LDS (one pass of independent loads), then every round reads LDS only.  The lanes share the block's
// samples (sample i goes to lane i % 64), the eight new points of the large pattern are evaluated
// together, and every decision is taken on wavefront-uniform values.  Windows too large for LDS are read
// from memory instead (WIN = false).
//   large pattern: centre, (0,-2), (-1,-1), (1,-1), (-2,0), (2,0), (-1,1), (1,1), (0,2)
//   small pattern: centre, (0,-1), (-1,0), (1,0), (0,1)
// The best point of a pattern is the valid one with the smallest (cost, position in the list above); the
// centre is position 0, so it moves only to a strictly smaller cost and the walk ends; max_rounds (the
// number of vectors in the search range) bounds it independently of the data.
// Blocks off the k-skip lattice get mv = (0,0) and best_ssd = 2^32 - 1.
__constant__ const signed char kLargeDx[8] = {0, -1, 1, -2, 2, -1, 1, 0};
__constant__ const signed char kLargeDy[8] = {-2, -1, -1, 0, 0, 1, 1, 2};
__constant__ const signed char kSmallDx[4] = {0, -1, 1, 0};
__constant__ const signed char kSmallDy[4] = {-1, 0, 0, 1};

struct DiamondBlock {
    const uint8_t* cblk;   // the block: memory (pitch W*C) or LDS (pitch B*C)
    const uint8_t* pwin;   // WIN: LDS window whose origin is the frame position (x0-R, y0-R); else the previous frame
    int H, W, C, B, R, x0, y0;
    uint32_t rb_magic;     // ceil(2^32 / (B*C)): sample index -> block row by one multiplication (exact for B^3 C^2 < 2^32)
};

// Costs of NP points around (cx, cy): cost[p] = SSD of the block against the previous frame at
// (cx + pdx[p], cy + pdy[p]), or 2^32 - 1 for a point outside the range or the frame.
template <int NP, bool WIN>
__device__ __forceinline__ void diamond_costs(const DiamondBlock& k, int cx, int cy, const signed char* pdx,
                                              const signed char* pdy, int lane, uint32_t (&cost)[NP]) {
    const int rb = k.B * k.C, n_elem = k.B * rb;
    const int cpitch = WIN ? rb : k.W * k.C;                    // block rows
    const int ppitch = WIN ? (k.B + 2 * k.R) * k.C : k.W * k.C; // previous-frame rows
    const uint8_t* src[NP];
    bool ok[NP];
    uint32_t s[NP];
#pragma unroll
    for (int p = 0; p < NP; ++p) {
        const int dx = cx + pdx[p], dy = cy + pdy[p];
        ok[p] = dx >= -k.R && dx <= k.R && dy >= -k.R && dy <= k.R && k.x0 + dx >= 0 && k.y0 + dy >= 0 &&
                k.x0 + dx + k.B <= k.W && k.y0 + dy + k.B <= k.H;
        const int ex = ok[p] ? dx : 0, ey = ok[p] ? dy : 0;       // a point that is not usable is never read
        src[p] = WIN ? k.pwin + (size_t)(k.R + ey) * ppitch + (k.R + ex) * k.C
                     : k.pwin + ((size_t)(k.y0 + ey) * k.W + k.x0 + ex) * k.C;
        s[p] = 0;
    }
    // Straight-line code: every read is unconditional, so that the reads of a batch are issued together instead
    // of one latency after the other.  A sample beyond the block reads the block's first byte on both sides
    // (difference zero); a point that is not usable reads the centre's samples and is discarded below.
    for (int base = 0; base < n_elem; base += 4 * 64) {       // four samples per lane at a time
        int a[4], off[4];
        bool in[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int i = base + u * 64 + lane;
            in[u] = i < n_elem;
            const int r = rb == 1 ? i : (int)__umulhi((uint32_t)i, k.rb_magic), j = i - r * rb;
            off[u] = r * ppitch + j;
            const uint8_t* pa = in[u] ? k.cblk + (r * cpitch + j) : k.cblk;
            a[u] = *pa;
        }
#pragma unroll
        for (int p = 0; p < NP; ++p) {
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const uint8_t* pb = in[u] ? src[p] + off[u] : k.cblk;
                const int d = a[u] - (int)*pb;
                s[p] += (uint32_t)(d * d);
            }
        }
    }
#pragma unroll
    for (int p = 0; p < NP; ++p) cost[p] = ok[p] ? (uint32_t)wave_sum_i32((int)s[p]) : 0xffffffffu;
}

template <bool WIN>
__global__ __launch_bounds__(256) void match_diamond_kernel(
    const uint8_t* __restrict__ cur, const uint8_t* __restrict__ prev, int H, int W, int C, int B, int R, int gw,
    int gh, int k_skip, int max_rounds, int region_bytes, uint32_t rb_magic, int16_t* __restrict__ mv,
    uint32_t* __restrict__ best_ssd) {
    extern __shared__ __align__(16) unsigned char dsm[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, waves = blockDim.x >> 6;
    const int nb = gh * gw;
    const int blk_id = blockIdx.x * waves + wave, stream = blockIdx.y;
    const int bx = blk_id % gw, by = blk_id / gw;
    const bool searched = blk_id < nb && bx % k_skip == 0 && by % k_skip == 0;
    const size_t frame_bytes = (size_t)H * W * C;
    const uint8_t* pf = prev + stream * frame_bytes;
    const int x0 = bx * B, y0 = by * B;
    const int rb = B * C, side = B + 2 * R;
    DiamondBlock k{cur + stream * frame_bytes + ((size_t)y0 * W + x0) * C, pf, H, W, C, B, R, x0, y0, rb_magic};
    if (WIN) {
        unsigned char* win = dsm + (size_t)wave * region_bytes;   // side rows of side*C bytes, then the block
        unsigned char* lblk = win + (size_t)side * side * C;
        if (searched) {
            // Row by row, the lanes across a row's bytes; four rows at a time, so that a pass issues 4 * ceil(wb/64)
            // independent loads per lane and the copy costs a few memory latencies, not one per byte.
            const int wb = side * C, per_row = (wb + 63) / 64;
            const int fb0 = (x0 - R) * C;
            for (int r0 = 0; r0 < side; r0 += 4) {
                for (int q = 0; q < per_row; ++q) {
                    const int j = q * 64 + lane, fb = fb0 + j;
                    unsigned char v[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u) {             // bytes outside the frame are never used: zero
                        const int r = r0 + u, fy = y0 - R + r;
                        const bool in = r < side && j < wb && fy >= 0 && fy < H && fb >= 0 && fb < W * C;
                        const unsigned char g = pf[in ? (size_t)fy * W * C + fb : 0];   // unconditional: the loads overlap
                        v[u] = in ? g : 0;
                    }
#pragma unroll
                    for (int u = 0; u < 4; ++u)
                        if (r0 + u < side && j < wb) win[(r0 + u) * wb + j] = v[u];
                }
            }
            for (int r0 = 0; r0 < B; r0 += 8) {
                for (int q = 0; q < (rb + 63) / 64; ++q) {
                    const int j = q * 64 + lane;
                    unsigned char v[8];
#pragma unroll
                    for (int u = 0; u < 8; ++u) v[u] = k.cblk[(r0 + u < B && j < rb) ? (size_t)(r0 + u) * W * C + j : 0];
#pragma unroll
                    for (int u = 0; u < 8; ++u)
                        if (r0 + u < B && j < rb) lblk[(r0 + u) * rb + j] = v[u];
                }
            }
        }
        __syncthreads();     // every wavefront of the workgroup arrives here, searched block or not
        k.cblk = lblk;
        k.pwin = win;
    }
    if (blk_id >= nb) return;
    int16_t* out_mv = mv + ((size_t)stream * nb + blk_id) * 2;
    uint32_t* out_ssd = best_ssd + (size_t)stream * nb + blk_id;
    if (!searched) {
        if (lane == 0) { out_mv[0] = 0; out_mv[1] = 0; *out_ssd = 0xffffffffu; }
        return;
    }
    const signed char zero = 0;
    uint32_t c0[1];
    diamond_costs<1, WIN>(k, 0, 0, &zero, &zero, lane, c0);
    int cx = 0, cy = 0;
    uint32_t ccost = c0[0];
    for (int round = 0; round < max_rounds; ++round) {
        uint32_t c[8];
        diamond_costs<8, WIN>(k, cx, cy, kLargeDx, kLargeDy, lane, c);
        int best = -1;
        uint32_t bcost = ccost;
#pragma unroll
        for (int p = 0; p < 8; ++p)
            if (c[p] < bcost) { bcost = c[p]; best = p; }
        if (best < 0) break;
        cx += kLargeDx[best]; cy += kLargeDy[best]; ccost = bcost;
    }
    uint32_t c[4];
    diamond_costs<4, WIN>(k, cx, cy, kSmallDx, kSmallDy, lane, c);
    int best = -1;
    uint32_t bcost = ccost;
#pragma unroll
    for (int p = 0; p < 4; ++p)
        if (c[p] < bcost) { bcost = c[p]; best = p; }
    if (best >= 0) { cx += kSmallDx[best]; cy += kSmallDy[best]; }
    if (lane == 0) { out_mv[0] = (int16_t)cx; out_mv[1] = (int16_t)cy; *out_ssd = bcost; }
}

}  // namespace

hipError_t launch_match(const uint8_t* cur, const uint8_t* prev, int n_streams, int H, int W, int C,
                        int B, int R, int k_skip, uint32_t max_ssd, int16_t* mv, uint32_t* best_ssd,
                        int32_t* gmv, int32_t* n_pass, uint8_t* mask, hipStream_t st) {
    const int gh = H / B, gw = W / B;
    const int rows = B + 2 * R;
    const bool aligned = ((reinterpret_cast<uintptr_t>(prev) & 3) == 0) && ((W * C) % 4 == 0);
    dim3 grid(((gw + k_skip - 1) / k_skip) * ((gh + k_skip - 1) / k_skip), n_streams);   // the searched blocks
    constexpr bool use_mfma = true;
    const int nt = (2 * R + 1 + 15) / 16, ksteps = (B * C + 63) / 64;
    bool done = false;
    if (use_mfma && nt <= 3 && ksteps <= 2 && B + 2 * R <= 255) {
        const int nd = 2 * R + 1;
        const int need = 3 + C * (16 * nt - 1) + 64 * ksteps + 4, real = 3 + rows * C + 4;
        const int wsm = (int)align_up((size_t)(need > real ? need : real), 16);
        // the instantiations below that know the block shape take their row sums from the window bytes: no per-pixel sums
        const bool fused = (nt == 3 && B == 16 && C == 3) || (nt == 2 && B == 8 && C == 3);
        const size_t dead = (size_t)rows * wsm + (size_t)B * 64 * ksteps + (size_t)((fused ? 0 : rows * rows) + rows * nd) * 4;
        const size_t ldsm = dead + 16 + (size_t)(3 * kMfmaWaves + nd * nd) * 4;
        if (ldsm <= 64 * 1024 && (size_t)nt * nt * 1024 <= dead) {   // the tile buffer of the final sum fits over the dead part
#define DC_MFMA_LAUNCH(AL, NTT, KSS, BT, CT)                                                                          \
    hipLaunchKernelGGL((match_mfma_kernel<AL, NTT, KSS, BT, CT>), grid, dim3(kMfmaThreads), ldsm, st, cur, prev, H, W, C, \
                       B, R, gw, gh, wsm, k_skip, mv, best_ssd)
#define DC_MFMA_KS(AL, NTT)                            \
    do {                                               \
        if (ksteps == 1) DC_MFMA_LAUNCH(AL, NTT, 1, 0, 0); \
        else DC_MFMA_LAUNCH(AL, NTT, 2, 0, 0);             \
    } while (0)
#define DC_MFMA_NT(AL)                                                     \
    do {                                                                   \
        if (nt == 3 && B == 16 && C == 3) DC_MFMA_LAUNCH(AL, 3, 1, 16, 3); \
        else if (nt == 2 && B == 8 && C == 3) DC_MFMA_LAUNCH(AL, 2, 1, 8, 3); \
        else if (nt == 1) DC_MFMA_KS(AL, 1);                               \
        else if (nt == 2) DC_MFMA_KS(AL, 2);                               \
        else DC_MFMA_KS(AL, 3);                                            \
    } while (0)
            if (aligned) DC_MFMA_NT(true);
            else DC_MFMA_NT(false);
#undef DC_MFMA_NT
#undef DC_MFMA_KS
#undef DC_MFMA_LAUNCH
            done = true;
        }
    }
    const int ws = (int)align_up((size_t)rows * C + 3, 4) + 8;  // skew (<=3) + window + over-read of the last dword pair
    const int cs = (int)align_up((size_t)B * C, 4);
    const size_t lds = (size_t)rows * ws + (size_t)B * cs;
#define DC_MATCH_LAUNCH(AL, CD)                                                                                      \
    hipLaunchKernelGGL((match_search_kernel<AL, CD>), grid, dim3(kSearchThreads), lds, st, cur, prev, H, W, C, B, R, \
                       gw, gh, ws, cs, k_skip, mv, best_ssd)
#define DC_MATCH_ALIGN(CD)             \
    do {                               \
        if (aligned) DC_MATCH_LAUNCH(true, CD); \
        else DC_MATCH_LAUNCH(false, CD);        \
    } while (0)
    if (!done) switch (cs / 4) {
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
    hipLaunchKernelGGL(motion_retest_kernel, dim3(gh * gw, n_streams), dim3(64), 0, st, cur, prev, H, W, C, B, gw, gh,
                       max_ssd, mv, best_ssd, gmv, n_pass, mask, k_skip);
    return hipGetLastError();
}

hipError_t launch_match_diamond(const uint8_t* cur, const uint8_t* prev, int n_streams, int H, int W, int C, int B,
                                int R, int k_skip, uint32_t max_ssd, int16_t* mv, uint32_t* best_ssd, int32_t* gmv,
                                int32_t* n_pass, uint8_t* mask, hipStream_t st) {
    const int gh = H / B, gw = W / B;
    const unsigned long long nvec = (2ull * R + 1) * (2ull * R + 1);
    const int cap = (int)(nvec < 0x7fffffffull ? nvec : 0x7fffffffull);
    const uint32_t rb_magic = (uint32_t)((0x100000000ull + (uint64_t)(B * C) - 1) / (uint64_t)(B * C));
    // LDS per wavefront: the search window and the block; as many wavefronts per workgroup as fit into 64 KiB
    const size_t side = (size_t)B + 2 * (size_t)R;
    const size_t region = align_up(side * side * C + (size_t)B * B * C, 16);
    const int waves = region <= 16 * 1024 ? 4 : (region <= 32 * 1024 ? 2 : 1);
    if (region <= 64 * 1024)
        hipLaunchKernelGGL(match_diamond_kernel<true>, dim3((gh * gw + waves - 1) / waves, n_streams), dim3(waves * 64),
                           region * waves, st, cur, prev, H, W, C, B, R, gw, gh, k_skip, cap, (int)region, rb_magic, mv, best_ssd);
    else
        hipLaunchKernelGGL(match_diamond_kernel<false>, dim3((gh * gw + 3) / 4, n_streams), dim3(256), 0, st, cur, prev,
                           H, W, C, B, R, gw, gh, k_skip, cap, 0, rb_magic, mv, best_ssd);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(motion_retest_kernel, dim3(gh * gw, n_streams), dim3(64), 0, st, cur, prev, H, W, C, B, gw, gh,
                       max_ssd, mv, best_ssd, gmv, n_pass, mask, k_skip);
    return hipGetLastError();
}

}  // namespace dc
