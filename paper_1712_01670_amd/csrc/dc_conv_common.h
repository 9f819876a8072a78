// Pieces shared by the convolution kernels: operand fragments, the LDS header with the unit table,
// workgroup and unit decoding, and the epilogue.
#pragma once
#include <hip/hip_bf16.h>

#include "dc_internal.h"

namespace dc {
namespace {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned int uintx4 __attribute__((ext_vector_type(4)));
typedef unsigned int uintx2 __attribute__((ext_vector_type(2)));

constexpr int PVMAX = 8;               // staged kernel: patch vectors per thread per stage
constexpr int WVMAX = 9;               // staged kernel: weight vectors per thread per stage
constexpr int DPMAX = 6;               // direct kernel: patch load instructions per wavefront per stage
constexpr int DWMAX = 12;              // direct kernel: weight load instructions per wavefront per stage
constexpr int kMaxK = 15;              // largest kernel edge
constexpr int kHeaderBytes = 1024;     // unit info and reuse mask at the start of LDS
constexpr uint32_t kOob = 0x80000000u; // byte offset beyond any tensor: buffer loads return zero
constexpr int kBufferFlags = 0x00020000;
constexpr int kMaxLdsBytes = 160 * 1024;   // LDS of one CU: the most a workgroup can ask for

struct ConvParams {
    const void* in;
    const void* w;
    const float* bias;
    void* out;
    int Hin, Win, Cin, Hout, Wout, Cout, k, s, p, relu;
    const int32_t* in_origin;    // tensors on a torus (3x3 stride-1 and first-layer kernels only): (ox, oy) of stream s at
    const int32_t* out_origin;   // origin[s * origin_stride + 0 / 1]; nullptr: the tensor starts at its buffer's start
    int origin_stride;
    int n_streams;               // conv_regw_kernel and the first-layer kernels on a torus: entries of their LDS table of origins (0: none)
    int kx, px, dil;        // general kernels: kernel columns (k: rows), padding along x (p: along y), distance between taps
    const TileDev* units;   // nullptr: every unit of every stream in raster order
    int n_units;            // length of the unit list; with n_units_dev the most it can be (the launch is sized for it)
    const int* n_units_dev; // optional, device: the length of a list that was built on the GPU
    const RectDev* rects;
    const RangeDev* ranges;
    int units_x, units_y;
    int ph, pw;             // patch rows / columns of one unit
    uint32_t npix_magic, pw_magic;   // ceil(2^32 / d) for the two runtime divisors of the slot decode
    int tg;                 // taps per stage
    int n_tapgroups, n_chunks;
    int R;                  // number of NT-wide channel tiles
    int pv, wv;             // load slots per thread (staged) or per wavefront (direct) per stage
    int p_instr, w_instr;   // direct kernel: 1 KiB load instructions per stage for the patches / the weights
    int patch_bytes;        // LDS bytes of one patch buffer (whole slots)
    int weight_bytes;       // LDS bytes of one weight buffer (whole slots)
    int dump_off;           // staged kernel: byte offset (after the header) of the per-thread dump slots
    uint32_t in_bytes, w_bytes;
    int g_rt;               // units per workgroup actually used (<= G)
    int chan_tail;          // 1: Cin is not a multiple of the channel chunk (per-slot channel check needed)
    int tap_tail;           // 1: k*k is not a multiple of TG (per-slot tap check needed)
    int out_vec;            // 1: four consecutive output channels can be stored (and the bias read) as one vector
    int ks;                 // workgroups that share one output tile, each with its own range of channel chunks
    int chunks_per_split;
    float* partial;         // ks > 1: [ks][n_units][16 pixels][Cout] partial sums
    int w_packed;           // 1: w is the packed layout [Cout/16][Cin*es/64][k*k][16][64 bytes]
    int n_wg_tiles, tiles_per_xcd;   // 1x1 kernel: (unit group, channel tile) pairs in all, and per XCD
};

template <typename T>
struct Frag;
template <>
struct Frag<float> {
    typedef floatx4 vec;
    static constexpr int VE = 4;
    // acc[channel][pixel] += W[channel][k] * X[pixel][k]
    static __device__ __forceinline__ void mma(const vec& wv, const vec& xv, floatx4& c) {
        c = __builtin_amdgcn_mfma_f32_16x16x4f32(wv[0], xv[0], c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_16x16x4f32(wv[1], xv[1], c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_16x16x4f32(wv[2], xv[2], c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_16x16x4f32(wv[3], xv[3], c, 0, 0, 0);
    }
    static constexpr int NE = 4;   // MFMAs per fragment pair
    static __device__ __forceinline__ void mma1(const vec& wv, const vec& xv, floatx4& c, int e) {
        c = __builtin_amdgcn_mfma_f32_16x16x4f32(wv[e], xv[e], c, 0, 0, 0);
    }
    static __device__ __forceinline__ void store4(float* p, const floatx4& v) { *reinterpret_cast<floatx4*>(p) = v; }
    static __device__ __forceinline__ void store1(float* p, float v) { *p = v; }
    static __device__ __forceinline__ float elem(__amdgpu_buffer_rsrc_t r, uint32_t off) {
        return __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(r, off, 0, 0));
    }
};
template <>
struct Frag<__hip_bfloat16> {
    typedef bf16x8 vec;
    static constexpr int VE = 8;
    static __device__ __forceinline__ void mma(const vec& wv, const vec& xv, floatx4& c) {
        c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wv, xv, c, 0, 0, 0);
    }
    static constexpr int NE = 1;
    static __device__ __forceinline__ void mma1(const vec& wv, const vec& xv, floatx4& c, int) {
        c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wv, xv, c, 0, 0, 0);
    }
    static __device__ __forceinline__ unsigned short bits(float v) {
        return __builtin_bit_cast(unsigned short, __float2bfloat16(v));
    }
    static __device__ __forceinline__ void store4(__hip_bfloat16* p, const floatx4& v) {
        uintx2 u;
        u[0] = (uint32_t)bits(v[0]) | ((uint32_t)bits(v[1]) << 16);
        u[1] = (uint32_t)bits(v[2]) | ((uint32_t)bits(v[3]) << 16);
        *reinterpret_cast<uintx2*>(p) = u;
    }
    static __device__ __forceinline__ void store1(__hip_bfloat16* p, float v) { *p = __float2bfloat16(v); }
    static __device__ __forceinline__ __bf16 elem(__amdgpu_buffer_rsrc_t r, uint32_t off) {
        return __builtin_bit_cast(__bf16, (unsigned short)__builtin_amdgcn_raw_buffer_load_b16(r, off, 0, 0));
    }
};

// Makes a wavefront-uniform value opaque to the optimiser, so that it is kept in scalar registers
// instead of being re-loaded from the kernel arguments inside the main loop (a scalar load there
// costs a full lgkmcnt(0) wait, which also drains the LDS reads in flight).
template <typename V>
__device__ __forceinline__ V keep_scalar(V v) {
    asm volatile("" : "+s"(v));
    return v;
}

// Activation fused into a convolution's epilogue: 1 = ReLU, 2 = leaky ReLU with slope 0.1 (Darknet-style stacks).
__device__ __forceinline__ float activate(float v, int mode) {
    return mode == 2 ? (v > 0.f ? v : 0.1f * v) : fmaxf(v, 0.f);
}
__device__ __forceinline__ void activate4(floatx4& v, int mode) {
    v[0] = activate(v[0], mode); v[1] = activate(v[1], mode); v[2] = activate(v[2], mode); v[3] = activate(v[3], mode);
}

__device__ __forceinline__ int fast_div(int n, uint32_t magic) { return (int)__umulhi((uint32_t)n, magic); }
// floor(n / d) for any 0 <= n < 2^31 with magic = ceil(2^32 / d): the product above is exact while n d < 2^32 and one
// too large at most beyond that (the stream of a raster position in a large batch).
__device__ __forceinline__ int fast_div_any(int n, uint32_t magic, int d) {
    const uint32_t q = __umulhi((uint32_t)n, magic);
    return (int)(q * (uint32_t)d > (uint32_t)n ? q - 1 : q);
}

// Number of units this launch works on: the host's count, or the one the planning kernels left in memory.
__device__ __forceinline__ int unit_count(const ConvParams& P) {
    return P.n_units_dev ? __builtin_amdgcn_readfirstlane(*P.n_units_dev) : P.n_units;
}

// ---- pieces shared by both kernels ------------------------------------------------

// LDS header: uinfo[G][4] = {valid, stream, oy0, ox0}, tmask[G*16], umask[G] (reusable pixels of the unit)
template <int G>
struct Header {
    int* uinfo;
    unsigned char* tmask;
    unsigned short* umask;
    __device__ __forceinline__ explicit Header(unsigned char* smem)
        : uinfo(reinterpret_cast<int*>(smem)),
          tmask(reinterpret_cast<unsigned char*>(smem) + 16 * G),
          umask(reinterpret_cast<unsigned short*>(smem + 32 * G)) {}
};

// workgroup -> (unit group, channel tile); channel tiles spread over the 8 XCDs so that each
// XCD's L2 holds only its share of the weights
__device__ __forceinline__ void decode_workgroup(int R, int& ug, int& ntile) {
    const int id = blockIdx.x;
    if ((R & 7) == 0) {
        const int r8 = R >> 3, j = id >> 3;
        ntile = (id & 7) + 8 * (j % r8);
        ug = j / r8;
    } else {
        ntile = id % R;
        ug = id / R;
    }
}

template <int G, int NTHREADS>
__device__ __forceinline__ void decode_units(const ConvParams& P, const Header<G>& H, int ug, int tid, int n_units) {
    if (tid < G) {
        const int u = ug * P.g_rt + tid;
        int valid = tid < P.g_rt && u < n_units, stream = 0, uy = 0, ux = 0, mixed = 0;
        if (valid) {
            if (P.units) {
                const TileDev t = P.units[u];
                stream = t.stream; uy = t.ty; ux = t.tx; mixed = t.reuse_mask;
            } else {
                const int per = P.units_x * P.units_y;
                stream = u / per;
                const int r = u - stream * per;
                uy = r / P.units_x; ux = r - uy * P.units_x;
            }
        }
        H.uinfo[4 * tid + 0] = valid; H.uinfo[4 * tid + 1] = stream;
        H.uinfo[4 * tid + 2] = uy * 4; H.uinfo[4 * tid + 3] = ux * 4;
        H.umask[tid] = (unsigned short)mixed;
    }
    __syncthreads();
    for (int m = tid; m < G * 16; m += NTHREADS) {   // per-pixel reuse flags
        const unsigned char hit = (unsigned char)((H.umask[m >> 4] >> (m & 15)) & 1);
        H.tmask[m] = hit;
    }
}

// Byte offset in the input tensor of patch pixel `prow` (row index over all units of the
// workgroup), or kOob if the pixel is padding or belongs to a missing unit.
template <int G, int ES>
__device__ __forceinline__ uint32_t patch_pixel_offset(const ConvParams& P, const Header<G>& H, int prow, int npix) {
    if (prow >= G * npix) return kOob;
    const int g = fast_div(prow, P.npix_magic), pix = prow - g * npix;
    const int py = fast_div(pix, P.pw_magic), px = pix - py * P.pw;
    const int iy = H.uinfo[4 * g + 2] * P.s - P.p + py, ix = H.uinfo[4 * g + 3] * P.s - P.px + px;
    if (!H.uinfo[4 * g] || iy < 0 || iy >= P.Hin || ix < 0 || ix >= P.Win) return kOob;
    return (uint32_t)(((H.uinfo[4 * g + 1] * P.Hin + iy) * P.Win + ix) * P.Cin) * ES;
}

// Adds the accumulators of the K-split wavefronts through LDS; returns false for wavefronts
// that have nothing left to do.
template <int WM, int WN, int WK, int UPW, int NBW>
__device__ __forceinline__ bool reduce_k_split(floatx4 (&acc)[UPW][NBW], unsigned char* scratch, int wave, int lane) {
    if (WK == 1) return true;
    const int wave_k = wave % WK, grp = wave / WK;
    float* red = reinterpret_cast<float*>(scratch);   // [(WK-1)][WM*WN][UPW*NBW][64 lanes][4]
    __syncthreads();
    if (wave_k > 0) {
#pragma unroll
        for (int u = 0; u < UPW; ++u)
#pragma unroll
            for (int j = 0; j < NBW; ++j)
                *reinterpret_cast<floatx4*>(red + ((((size_t)(wave_k - 1) * (WM * WN) + grp) * (UPW * NBW) + u * NBW + j) * 64 + lane) * 4) = acc[u][j];
    }
    __syncthreads();
    if (wave_k != 0) return false;
#pragma unroll
    for (int kq = 1; kq < WK; ++kq)
#pragma unroll
        for (int u = 0; u < UPW; ++u)
#pragma unroll
            for (int j = 0; j < NBW; ++j)
                acc[u][j] += *reinterpret_cast<const floatx4*>(red + ((((size_t)(kq - 1) * (WM * WN) + grp) * (UPW * NBW) + u * NBW + j) * 64 + lane) * 4);
    return true;
}

// lane (l16, q): pixel l16 of the unit, channels 4q..4q+3 of each 16-channel block
// wavefront-local unit u is unit u * unit_stride + unit0 of the workgroup
template <typename T, int G, int UPW, int NBW>
__device__ __forceinline__ void epilogue(const ConvParams& P, const Header<G>& H, const floatx4 (&acc)[UPW][NBW],
                                         int unit0, int unit_stride, int chan0, int l16, int q) {
    typedef Frag<T> F;
    T* out = reinterpret_cast<T*>(P.out);
    const bool vec_ok = P.out_vec != 0;
#pragma unroll
    for (int u = 0; u < UPW; ++u) {
        const int g = unit0 + u * unit_stride;
        if (!H.uinfo[4 * g]) continue;
        const int y = H.uinfo[4 * g + 2] + (l16 >> 2), x = H.uinfo[4 * g + 3] + (l16 & 3);
        if (y >= P.Hout || x >= P.Wout || H.tmask[g * 16 + l16]) continue;
        T* px = out + (((size_t)H.uinfo[4 * g + 1] * P.Hout + y) * P.Wout + x) * P.Cout;
#pragma unroll
        for (int j = 0; j < NBW; ++j) {
            const int co = chan0 + j * 16 + 4 * q;
            if (co >= P.Cout) continue;
            floatx4 v = acc[u][j];
            if (vec_ok) {   // co + 3 < Cout because both are multiples of 4
                if (P.bias) v += *reinterpret_cast<const floatx4*>(P.bias + co);
                if (P.relu) activate4(v, P.relu);
                F::store4(px + co, v);
            } else {
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    if (co + r >= P.Cout) continue;
                    float s = v[r] + (P.bias ? P.bias[co + r] : 0.f);
                    if (P.relu) s = activate(s, P.relu);
                    F::store1(px + co + r, s);
                }
            }
        }
    }
}

}  // namespace
}  // namespace dc
