// Cache-aware convolution (Section 5 "Reuse", steps 2-3) as an implicit GEMM on the
// gfx950 matrix cores, over a compacted list of output tiles that hold at least one
// non-reusable pixel.
//
//   M = TH x TW output pixels of one tile, N = NT output channels, K = k*k*cin.
// Per workgroup (WM x WN wavefronts): the input patch of the tile
// ((TH-1)s+k) x ((TW-1)s+k) pixels x KC channels is staged in LDS once per channel
// chunk and re-read for all k*k taps; the weight slice [NT][KC] of one tap is staged
// per tap.  Lanes 0-31 of a wavefront hold the first half of each K group, lanes
// 32-63 the second half, for both operands, so one 16-byte LDS read per operand feeds
// four fp32 MFMAs (32x32x2) or one bf16 MFMA (32x32x16).
// Epilogue: bias, ReLU, rounding to the storage type, and a per-pixel predicate: a
// pixel that lies in a reusable rectangle keeps the value the shifted copy wrote.
#include <hip/hip_bf16.h>

#include "dc_internal.h"

namespace dc {

namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

struct ConvParams {
    const void* in;
    const void* w;
    const float* bias;
    void* out;
    int n_streams, Hin, Win, Cin, Hout, Wout, Cout, k, s, p, relu;
    const TileDev* tiles;
    const RectDev* rects;
    const RangeDev* ranges;
    int tiles_x, tiles_y;
    int ph, pw;      // patch rows / columns
    int vec_in;      // 1: cin run is 16-byte aligned (vector loads allowed)
};

template <typename T>
struct Frag;
template <>
struct Frag<float> {
    typedef floatx4 vec;
    static constexpr int VE = 4;  // elements per 16-byte vector
    static __device__ __forceinline__ void mma(const vec& a, const vec& b, floatx16& c) {
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(a[0], b[0], c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(a[1], b[1], c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(a[2], b[2], c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(a[3], b[3], c, 0, 0, 0);
    }
    static __device__ __forceinline__ float load(const float* p) { return *p; }
    static __device__ __forceinline__ void store(float* p, float v) { *p = v; }
};
template <>
struct Frag<__hip_bfloat16> {
    typedef bf16x8 vec;
    static constexpr int VE = 8;
    static __device__ __forceinline__ void mma(const vec& a, const vec& b, floatx16& c) {
        c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
    }
    static __device__ __forceinline__ void store(__hip_bfloat16* p, float v) { *p = __float2bfloat16(v); }
};

template <typename T, int TH, int TW, int NT, int WM, int WN, int KC>
__global__ __launch_bounds__(WM* WN * 64) void conv_tiles_kernel(ConvParams P) {
    typedef Frag<T> F;
    typedef typename F::vec vec;
    constexpr int VE = F::VE;
    constexpr int KG = 2 * VE;                 // K elements consumed per fragment pair
    constexpr int MT = TH * TW;
    constexpr int NTHREADS = WM * WN * 64;
    constexpr int MB = MT / WM / 32;           // 32-row blocks per wavefront
    constexpr int NB = NT / WN / 32;           // 32-column blocks per wavefront
    constexpr int KCP = KC + VE;               // padded channel run (elements)
    constexpr int NVEC = KC / VE;              // 16-byte vectors per pixel per chunk
    static_assert(MT % (WM * 32) == 0 && NT % (WN * 32) == 0 && KC % KG == 0, "tile shape");

    extern __shared__ __align__(16) unsigned char smem[];
    T* patch = reinterpret_cast<T*>(smem);
    T* wt = patch + (size_t)P.ph * P.pw * KCP;
    unsigned char* tmask = reinterpret_cast<unsigned char*>(wt + (size_t)NT * KCP);

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wave_m = wave % WM, wave_n = wave / WM;
    const int l32 = lane & 31, half = lane >> 5;

    int stream, ty, tx, mixed;
    if (P.tiles) {
        TileDev t = P.tiles[blockIdx.x];
        stream = t.stream; ty = t.ty; tx = t.tx; mixed = t.mixed;
    } else {
        int per = P.tiles_x * P.tiles_y;
        stream = blockIdx.x / per;
        int r = blockIdx.x - stream * per;
        ty = r / P.tiles_x; tx = r - ty * P.tiles_x; mixed = 0;
    }
    const int oy0 = ty * TH, ox0 = tx * TW;
    const int n0 = blockIdx.y * NT;
    const int iy0 = oy0 * P.s - P.p, ix0 = ox0 * P.s - P.p;
    const T* in = reinterpret_cast<const T*>(P.in) + (size_t)stream * P.Hin * P.Win * P.Cin;
    const T* w = reinterpret_cast<const T*>(P.w);
    const int kk = P.k * P.k;

    if (mixed) {
        RangeDev rg = P.ranges[stream];
        for (int m = tid; m < MT; m += NTHREADS) {
            int y = oy0 + m / TW, x = ox0 + m % TW;
            unsigned char hit = 0;
            for (int i = 0; i < rg.count; ++i) {
                RectDev r = P.rects[rg.begin + i];
                hit |= (x >= r.x && x < r.x + r.w && y >= r.y && y < r.y + r.h) ? 1 : 0;
            }
            tmask[m] = hit;
        }
    }

    // per-lane fragment offsets (elements)
    int aoff[MB], boff[NB];
#pragma unroll
    for (int b = 0; b < MB; ++b) {
        int m = (wave_m * MB + b) * 32 + l32;
        aoff[b] = ((m / TW) * P.s * P.pw + (m % TW) * P.s) * KCP + half * VE;
    }
#pragma unroll
    for (int j = 0; j < NB; ++j) boff[j] = ((wave_n * NB + j) * 32 + l32) * KCP + half * VE;

    floatx16 acc[MB][NB];
#pragma unroll
    for (int b = 0; b < MB; ++b)
#pragma unroll
        for (int j = 0; j < NB; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[b][j][r] = 0.f;

    const int npix = P.ph * P.pw;
    for (int c0 = 0; c0 < P.Cin; c0 += KC) {
        __syncthreads();  // previous chunk fully consumed
        // ---- stage the input patch for channels [c0, c0+KC) ----
        for (int i = tid; i < npix * NVEC; i += NTHREADS) {
            int pix = i / NVEC, v = i - pix * NVEC;
            int py = pix / P.pw, px = pix - py * P.pw;
            int iy = iy0 + py, ix = ix0 + px, c = c0 + v * VE;
            vec val;
#pragma unroll
            for (int e = 0; e < VE; ++e) val[e] = 0;
            if (iy >= 0 && iy < P.Hin && ix >= 0 && ix < P.Win && c < P.Cin) {
                const T* src = in + ((size_t)iy * P.Win + ix) * P.Cin + c;
                if (P.vec_in && c + VE <= P.Cin) {
                    val = *reinterpret_cast<const vec*>(src);
                } else {
                    T tmp[VE];
#pragma unroll
                    for (int e = 0; e < VE; ++e) tmp[e] = (c + e < P.Cin) ? src[e] : T(0.f);
                    val = *reinterpret_cast<const vec*>(tmp);
                }
            }
            *reinterpret_cast<vec*>(patch + (size_t)pix * KCP + v * VE) = val;
        }
        for (int tap = 0; tap < kk; ++tap) {
            if (tap) __syncthreads();  // previous tap's weights consumed
            // ---- stage the weight slice [NT][KC] of this tap ----
            for (int i = tid; i < NT * NVEC; i += NTHREADS) {
                int n = i / NVEC, v = i - n * NVEC;
                int co = n0 + n, c = c0 + v * VE;
                vec val;
#pragma unroll
                for (int e = 0; e < VE; ++e) val[e] = 0;
                if (co < P.Cout && c < P.Cin) {
                    const T* src = w + ((size_t)co * kk + tap) * P.Cin + c;
                    if (P.vec_in && c + VE <= P.Cin) {
                        val = *reinterpret_cast<const vec*>(src);
                    } else {
                        T tmp[VE];
#pragma unroll
                        for (int e = 0; e < VE; ++e) tmp[e] = (c + e < P.Cin) ? src[e] : T(0.f);
                        val = *reinterpret_cast<const vec*>(tmp);
                    }
                }
                *reinterpret_cast<vec*>(wt + (size_t)n * KCP + v * VE) = val;
            }
            __syncthreads();
            const int ky = tap / P.k, kx = tap - ky * P.k;
            const int toff = (ky * P.pw + kx) * KCP;
#pragma unroll
            for (int g = 0; g < KC / KG; ++g) {
                vec a[MB], bq[NB];
#pragma unroll
                for (int b = 0; b < MB; ++b) a[b] = *reinterpret_cast<const vec*>(patch + aoff[b] + toff + g * KG);
#pragma unroll
                for (int j = 0; j < NB; ++j) bq[j] = *reinterpret_cast<const vec*>(wt + boff[j] + g * KG);
#pragma unroll
                for (int b = 0; b < MB; ++b)
#pragma unroll
                    for (int j = 0; j < NB; ++j) F::mma(a[b], bq[j], acc[b][j]);
            }
        }
    }

    // ---- epilogue ----
    T* out = reinterpret_cast<T*>(P.out) + (size_t)stream * P.Hout * P.Wout * P.Cout;
#pragma unroll
    for (int j = 0; j < NB; ++j) {
        const int co = n0 + (wave_n * NB + j) * 32 + l32;
        if (co >= P.Cout) continue;
        const float bv = P.bias ? P.bias[co] : 0.f;
#pragma unroll
        for (int b = 0; b < MB; ++b) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                int m = (wave_m * MB + b) * 32 + (r >> 2) * 8 + half * 4 + (r & 3);
                int y = oy0 + m / TW, x = ox0 + m % TW;
                if (y >= P.Hout || x >= P.Wout) continue;
                if (mixed && tmask[m]) continue;
                float v = acc[b][j][r] + bv;
                if (P.relu) v = v > 0.f ? v : 0.f;
                F::store(out + ((size_t)y * P.Wout + x) * P.Cout + co, v);
            }
        }
    }
}

struct KernelEntry {
    int th, tw, nt, kc_f32, kc_bf16, threads;
    void (*f32)(ConvParams);
    void (*bf16)(ConvParams);
};

#define DC_ENTRY(TH, TW, NT, WM, WN, KF, KB)                                        \
    {TH, TW, NT, KF, KB, WM * WN * 64, conv_tiles_kernel<float, TH, TW, NT, WM, WN, KF>, \
     conv_tiles_kernel<__hip_bfloat16, TH, TW, NT, WM, WN, KB>}

// cfg 0-3: deep channel chunks; cfg 4-7: the same tiles with a shallow chunk for cin < 16
const KernelEntry kTable[] = {
    DC_ENTRY(8, 16, 128, 2, 2, 32, 64),  // 0: large maps, cout >= 128
    DC_ENTRY(8, 16, 64, 2, 2, 32, 64),   // 1: large maps, cout 64
    DC_ENTRY(8, 8, 64, 2, 2, 32, 64),    // 2: small maps
    DC_ENTRY(8, 16, 32, 4, 1, 32, 64),   // 3: cout <= 32
    DC_ENTRY(8, 16, 128, 2, 2, 8, 16),   // 4
    DC_ENTRY(8, 16, 64, 2, 2, 8, 16),    // 5
    DC_ENTRY(8, 8, 64, 2, 2, 8, 16),     // 6
    DC_ENTRY(8, 16, 32, 4, 1, 8, 16),    // 7
};

}  // namespace

ConvTiling pick_tiling(const dc_layer& L, int Hout, int Wout, int n_streams, int dtype) {
    (void)dtype;
    int cfg;
    if (L.cout <= 32) {
        cfg = 3;
    } else {
        long tiles128 = (long)n_streams * ((Hout + 7) / 8) * ((Wout + 15) / 16);
        if (L.cout >= 128 && tiles128 * ((L.cout + 127) / 128) >= 512) cfg = 0;
        else if (tiles128 * ((L.cout + 63) / 64) >= 512) cfg = 1;
        else cfg = 2;
    }
    if (L.cin < 16) cfg += 4;
    return ConvTiling{cfg, kTable[cfg].th, kTable[cfg].tw, kTable[cfg].nt};
}

hipError_t launch_conv(const ConvLaunch& c, hipStream_t st) {
    const KernelEntry& e = kTable[c.tiling.cfg];
    ConvParams P;
    P.in = c.in; P.w = c.w; P.bias = c.bias; P.out = c.out;
    P.n_streams = c.n_streams; P.Hin = c.Hin; P.Win = c.Win; P.Cin = c.Cin;
    P.Hout = c.Hout; P.Wout = c.Wout; P.Cout = c.Cout; P.k = c.k; P.s = c.s; P.p = c.p; P.relu = c.relu;
    P.tiles = c.tiles; P.rects = c.rects; P.ranges = c.ranges;
    P.tiles_y = (c.Hout + e.th - 1) / e.th;
    P.tiles_x = (c.Wout + e.tw - 1) / e.tw;
    P.ph = (e.th - 1) * c.s + c.k;
    P.pw = (e.tw - 1) * c.s + c.k;
    const size_t esz = dtype_size(c.dtype);
    const int ve = (int)(16 / esz);
    P.vec_in = ((size_t)c.Cin * esz) % 16 == 0 && reinterpret_cast<uintptr_t>(c.in) % 16 == 0 &&
               reinterpret_cast<uintptr_t>(c.w) % 16 == 0;
    const int kc = c.dtype == DC_BF16 ? e.kc_bf16 : e.kc_f32;
    const size_t kcp = kc + ve;
    size_t lds = ((size_t)P.ph * P.pw * kcp + (size_t)e.nt * kcp) * esz + (size_t)e.th * e.tw;
    if (lds > 160 * 1024) return hipErrorInvalidValue;
    const int n_tiles = c.tiles ? c.n_tiles : c.n_streams * P.tiles_x * P.tiles_y;
    if (n_tiles <= 0) return hipSuccess;
    void (*fn)(ConvParams) = c.dtype == DC_BF16 ? e.bf16 : e.f32;
    if (lds > 64 * 1024) {
        hipError_t a = hipFuncSetAttribute(reinterpret_cast<const void*>(fn),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (a != hipSuccess) return a;
    }
    dim3 grid(n_tiles, (c.Cout + e.nt - 1) / e.nt);
    hipLaunchKernelGGL(fn, grid, dim3(e.threads), lds, st, P);
    return hipGetLastError();
}

}  // namespace dc
