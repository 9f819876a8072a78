// Cache-aware convolution (Section 5 "Reuse", steps 2-3) as an implicit GEMM on the
// gfx950 matrix cores over a compacted list of 4x4-pixel output units that hold at
// least one non-reusable pixel.
//
//   M = G units x 16 pixels, N = NT output channels, K = k*k*cin.
//
// A workgroup takes G consecutive units of the list (any positions, any streams) and
// NT output channels.  K is walked in stages of (TG taps) x (KC channels): the input
// patch of every unit ((3s+k)^2 pixels x KC channels) is staged in LDS once per channel
// chunk, the weight slices [TG][NT][KC] once per stage.  Global loads of stage i+1 are
// issued into registers before the MFMAs of stage i and written to LDS afterwards, so
// HBM/L2 latency overlaps the matrix work.
//
// MFMA 16x16: lane l holds row/column l%16 and the K elements [VE*(l/16), VE*(l/16)+VE)
// of each K group for both operands, so one 16-byte LDS read per operand feeds four
// fp32 MFMAs (16x16x4) or one bf16 MFMA (16x16x32).  The accumulator register j of lane l
// is output pixel (row l/16, column j) of the unit and channel l%16 of the block.
//
// WK > 1: the wavefronts of a workgroup split the K steps of every stage among
// themselves and add their accumulators through LDS in a fixed order (deterministic).
//
// Epilogue: bias, ReLU, rounding to the storage type, and a per-pixel predicate: a pixel
// inside a reusable rectangle keeps the value the shifted copy wrote.
#include <hip/hip_bf16.h>

#include <cstdio>

#include "dc_internal.h"

namespace dc {

namespace {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

constexpr int PVMAX = 8;   // patch vectors per thread per stage (upper bound)
constexpr int WVMAX = 9;   // weight vectors per thread per stage (upper bound)
constexpr int kMaxTaps = 128;
constexpr int kHeaderBytes = 1024;   // tap offsets, unit info and reuse mask at the start of LDS

struct ConvParams {
    const void* in;
    const void* w;
    const float* bias;
    void* out;
    int Hin, Win, Cin, Hout, Wout, Cout, k, s, p, relu;
    const TileDev* units;   // nullptr: every unit of every stream in raster order
    int n_units;
    const RectDev* rects;
    const RangeDev* ranges;
    int units_x, units_y;
    int ph, pw;             // patch rows / columns of one unit
    int tg;                 // taps per stage
    int n_tapgroups, n_chunks;
    int R;                  // number of NT-wide channel tiles
};

template <typename T>
struct Frag;
template <>
struct Frag<float> {
    typedef floatx4 vec;
    static constexpr int VE = 4;
    static __device__ __forceinline__ void mma(const vec& a, const vec& b, floatx4& c) {
        c = __builtin_amdgcn_mfma_f32_16x16x4f32(a[0], b[0], c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_16x16x4f32(a[1], b[1], c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_16x16x4f32(a[2], b[2], c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_16x16x4f32(a[3], b[3], c, 0, 0, 0);
    }
    static __device__ __forceinline__ void store(float* p, float v) { *p = v; }
};
template <>
struct Frag<__hip_bfloat16> {
    typedef bf16x8 vec;
    static constexpr int VE = 8;
    static __device__ __forceinline__ void mma(const vec& a, const vec& b, floatx4& c) {
        c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
    }
    static __device__ __forceinline__ void store(__hip_bfloat16* p, float v) { *p = __float2bfloat16(v); }
};

__device__ __forceinline__ float elem_load(const float* p) { return *p; }
__device__ __forceinline__ __bf16 elem_load(const __hip_bfloat16* p) {
    return __builtin_bit_cast(__bf16, *reinterpret_cast<const unsigned short*>(p));
}

// slot descriptor: bits 0..19 LDS element offset, 20..27 channel offset in the chunk,
// 28..31 tap index inside the stage (weights only)
__device__ __forceinline__ uint32_t pack_slot(int lds_off, int ch, int tl) {
    return (uint32_t)lds_off | ((uint32_t)ch << 20) | ((uint32_t)tl << 28);
}

template <typename T, int G, int NT, int WM, int WN, int WK, int KC, bool VEC>
__global__ __launch_bounds__(WM* WN* WK * 64) void conv_units_kernel(ConvParams P) {
    typedef Frag<T> F;
    typedef typename F::vec vec;
    constexpr int VE = F::VE;
    constexpr int KG = 4 * VE;                 // K elements per MFMA group
    constexpr int NTHREADS = WM * WN * WK * 64;
    constexpr int UPW = G / WM;                // units per wavefront
    constexpr int NBW = NT / WN / 16;          // 16-channel blocks per wavefront
    constexpr int KCP = KC + VE;               // padded channel run (elements)
    constexpr int GPC = KC / KG;               // K groups per chunk
    constexpr int NVEC = KC / VE;              // 16-byte vectors per pixel per chunk
    static_assert(G % WM == 0 && NT % (WN * 16) == 0 && KC % KG == 0, "tile shape");

    extern __shared__ __align__(16) unsigned char smem[];
    const int npix = P.ph * P.pw;
    int* tapoff = reinterpret_cast<int*>(smem);                               // [kMaxTaps]
    int* uinfo = tapoff + kMaxTaps;                                           // [G][4]: valid, stream, oy0, ox0
    unsigned char* tmask = reinterpret_cast<unsigned char*>(uinfo + 4 * G);   // [G*16]
    unsigned char* umixed = tmask + G * 16;                                   // [G]
    T* patch = reinterpret_cast<T*>(smem + kHeaderBytes);
    T* wt = patch + (size_t)G * npix * KCP;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wave_k = wave % WK, wave_n = (wave / WK) % WN, wave_m = wave / (WK * WN);
    const int l16 = lane & 15, q = lane >> 4;
    const int kk = P.k * P.k;

    // ---- workgroup -> (unit group, channel tile); channel tiles spread over the 8 XCDs ----
    int ug, ntile;
    {
        const int id = blockIdx.x, R = P.R;
        if ((R & 7) == 0) {
            const int r8 = R >> 3, j = id >> 3;
            ntile = (id & 7) + 8 * (j % r8);
            ug = j / r8;
        } else {
            ntile = id % R;
            ug = id / R;
        }
    }
    const int n0 = ntile * NT;

    if (tid < G) {
        const int u = ug * G + tid;
        int valid = u < P.n_units, stream = 0, uy = 0, ux = 0, mixed = 0;
        if (valid) {
            if (P.units) {
                TileDev t = P.units[u];
                stream = t.stream; uy = t.ty; ux = t.tx; mixed = t.mixed;
            } else {
                const int per = P.units_x * P.units_y;
                stream = u / per;
                const int r = u - stream * per;
                uy = r / P.units_x; ux = r - uy * P.units_x;
            }
        }
        uinfo[4 * tid + 0] = valid; uinfo[4 * tid + 1] = stream;
        uinfo[4 * tid + 2] = uy * 4; uinfo[4 * tid + 3] = ux * 4;
        umixed[tid] = (unsigned char)mixed;
    }
    for (int t = tid; t < kk; t += NTHREADS) tapoff[t] = ((t / P.k) * P.pw + (t % P.k)) * KCP;
    __syncthreads();

    // per-pixel reuse mask of mixed units
    for (int m = tid; m < G * 16; m += NTHREADS) {
        const int g = m >> 4;
        unsigned char hit = 0;
        if (umixed[g]) {
            const int y = uinfo[4 * g + 2] + ((m >> 2) & 3), x = uinfo[4 * g + 3] + (m & 3);
            const RangeDev rg = P.ranges[uinfo[4 * g + 1]];
            for (int i = 0; i < rg.count; ++i) {
                const RectDev r = P.rects[rg.begin + i];
                hit |= (x >= r.x && x < r.x + r.w && y >= r.y && y < r.y + r.h) ? 1 : 0;
            }
        }
        tmask[m] = hit;
    }

    // ---- per-thread load slots ----
    const T* in = reinterpret_cast<const T*>(P.in);
    const T* w = reinterpret_cast<const T*>(P.w);
    int pg[PVMAX];        // global element offset of the slot at chunk 0, or -1 (zero fill)
    uint32_t pl[PVMAX];   // packed LDS offset / channel offset
    const int ptotal = G * npix * NVEC;
#pragma unroll
    for (int i = 0; i < PVMAX; ++i) {
        const int idx = tid + i * NTHREADS;
        pg[i] = -1; pl[i] = 0xffffffffu;
        if (idx < ptotal) {
            const int g = idx / (npix * NVEC), rem = idx - g * (npix * NVEC);
            const int pix = rem / NVEC, v = rem - pix * NVEC;
            const int py = pix / P.pw, px = pix - py * P.pw;
            const int iy = uinfo[4 * g + 2] * P.s - P.p + py, ix = uinfo[4 * g + 3] * P.s - P.p + px;
            pl[i] = pack_slot((g * npix + pix) * KCP + v * VE, v * VE, 0);
            if (uinfo[4 * g] && iy >= 0 && iy < P.Hin && ix >= 0 && ix < P.Win)
                pg[i] = (((uinfo[4 * g + 1] * P.Hin + iy) * P.Win) + ix) * P.Cin + v * VE;
        }
    }
    int wg[WVMAX];
    uint32_t wl[WVMAX];
    const int wtotal = P.tg * NT * NVEC;
#pragma unroll
    for (int i = 0; i < WVMAX; ++i) {
        const int idx = tid + i * NTHREADS;
        wg[i] = -1; wl[i] = 0xffffffffu;
        if (idx < wtotal) {
            const int tl = idx / (NT * NVEC), rem = idx - tl * (NT * NVEC);
            const int n = rem / NVEC, v = rem - n * NVEC;
            wl[i] = pack_slot((tl * NT + n) * KCP + v * VE, v * VE, tl);
            if (n0 + n < P.Cout) wg[i] = ((n0 + n) * kk + tl) * P.Cin + v * VE;
        }
    }

    // ---- per-lane fragment bases (elements) ----
    int abase[UPW], bbase[NBW];
    // lane l16 is pixel (row l16/4, column l16%4) of the unit for the A operand
#pragma unroll
    for (int u = 0; u < UPW; ++u)
        abase[u] = ((wave_m * UPW + u) * npix + ((l16 >> 2) * P.s) * P.pw + (l16 & 3) * P.s) * KCP + q * VE;
#pragma unroll
    for (int j = 0; j < NBW; ++j) bbase[j] = ((wave_n * NBW + j) * 16 + l16) * KCP + q * VE;

    floatx4 acc[UPW][NBW];
#pragma unroll
    for (int u = 0; u < UPW; ++u)
#pragma unroll
        for (int j = 0; j < NBW; ++j) acc[u][j] = floatx4{0.f, 0.f, 0.f, 0.f};

    vec pr[PVMAX], wr[WVMAX];
    const vec zero = vec{};

    auto load_stage = [&](int chunk, int tgi) {
        const int c0 = chunk * KC;
        if (tgi == 0) {
#pragma unroll
            for (int i = 0; i < PVMAX; ++i) {
                pr[i] = zero;
                const int ch = c0 + (int)((pl[i] >> 20) & 0xff);
                if (pg[i] >= 0 && ch < P.Cin) {
                    const T* src = in + (size_t)(uint32_t)pg[i] + c0;
                    if (VEC) {
                        pr[i] = *reinterpret_cast<const vec*>(src);
                    } else {
#pragma unroll
                        for (int e = 0; e < VE; ++e)
                            if (ch + e < P.Cin) pr[i][e] = elem_load(src + e);
                    }
                }
            }
        }
        const int tap0 = tgi * P.tg;
#pragma unroll
        for (int i = 0; i < WVMAX; ++i) {
            wr[i] = zero;
            const int ch = c0 + (int)((wl[i] >> 20) & 0xff);
            const int tl = (int)(wl[i] >> 28);
            if (wg[i] >= 0 && ch < P.Cin && tap0 + tl < kk) {
                const T* src = w + (size_t)(uint32_t)wg[i] + (size_t)tap0 * P.Cin + c0;
                if (VEC) {
                    wr[i] = *reinterpret_cast<const vec*>(src);
                } else {
#pragma unroll
                    for (int e = 0; e < VE; ++e)
                        if (ch + e < P.Cin) wr[i][e] = elem_load(src + e);
                }
            }
        }
    };
    auto store_stage = [&](int tgi) {
        if (tgi == 0) {
#pragma unroll
            for (int i = 0; i < PVMAX; ++i)
                if (pl[i] != 0xffffffffu) *reinterpret_cast<vec*>(patch + (pl[i] & 0xfffff)) = pr[i];
        }
#pragma unroll
        for (int i = 0; i < WVMAX; ++i)
            if (wl[i] != 0xffffffffu) *reinterpret_cast<vec*>(wt + (wl[i] & 0xfffff)) = wr[i];
    };

    const int n_stages = P.n_chunks * P.n_tapgroups;
    load_stage(0, 0);
    int chunk = 0, tgi = 0;
    for (int st = 0; st < n_stages; ++st) {
        __syncthreads();           // every wavefront is done with the previous stage's LDS
        store_stage(tgi);
        __syncthreads();
        int nchunk = chunk, ntgi = tgi + 1;
        if (ntgi == P.n_tapgroups) { ntgi = 0; ++nchunk; }
        if (st + 1 < n_stages) load_stage(nchunk, ntgi);   // in flight during the MFMAs below

        const int tap0 = tgi * P.tg;
        const int ntap = (kk - tap0) < P.tg ? (kk - tap0) : P.tg;
        const int steps = ntap * GPC;
        for (int sidx = wave_k; sidx < steps; sidx += WK) {
            const int tl = sidx / GPC, g = sidx - tl * GPC;
            const int aoff = tapoff[tap0 + tl] + g * KG;
            const int boff = tl * NT * KCP + g * KG;
            vec a[UPW], b[NBW];
#pragma unroll
            for (int u = 0; u < UPW; ++u) a[u] = *reinterpret_cast<const vec*>(patch + abase[u] + aoff);
#pragma unroll
            for (int j = 0; j < NBW; ++j) b[j] = *reinterpret_cast<const vec*>(wt + bbase[j] + boff);
#pragma unroll
            for (int u = 0; u < UPW; ++u)
#pragma unroll
                for (int j = 0; j < NBW; ++j) F::mma(a[u], b[j], acc[u][j]);
        }
        chunk = nchunk; tgi = ntgi;
    }

    // ---- add the accumulators of the K-split wavefronts (fixed order) ----
    if (WK > 1) {
        __syncthreads();
        float* red = reinterpret_cast<float*>(smem + kHeaderBytes);   // [(WK-1)][WM*WN][UPW*NBW][64 lanes][4]
        const int grp = wave / WK;                      // (wave_m, wave_n) pair
        if (wave_k > 0) {
#pragma unroll
            for (int u = 0; u < UPW; ++u)
#pragma unroll
                for (int j = 0; j < NBW; ++j)
                    *reinterpret_cast<floatx4*>(red + ((((size_t)(wave_k - 1) * (WM * WN) + grp) * (UPW * NBW) + u * NBW + j) * 64 + lane) * 4) = acc[u][j];
        }
        __syncthreads();
        if (wave_k == 0) {
#pragma unroll
            for (int kq = 1; kq < WK; ++kq)
#pragma unroll
                for (int u = 0; u < UPW; ++u)
#pragma unroll
                    for (int j = 0; j < NBW; ++j)
                        acc[u][j] += *reinterpret_cast<const floatx4*>(red + ((((size_t)(kq - 1) * (WM * WN) + grp) * (UPW * NBW) + u * NBW + j) * 64 + lane) * 4);
        }
    }
    if (wave_k != 0) return;

    // ---- epilogue: lane group q is row q of the unit, register j is column j ----
    T* out = reinterpret_cast<T*>(P.out);
#pragma unroll
    for (int u = 0; u < UPW; ++u) {
        const int g = wave_m * UPW + u;
        if (!uinfo[4 * g]) continue;
        const int y = uinfo[4 * g + 2] + q;
        if (y >= P.Hout) continue;
        const size_t row = ((size_t)uinfo[4 * g + 1] * P.Hout + y) * P.Wout;
#pragma unroll
        for (int j = 0; j < NBW; ++j) {
            const int co = n0 + (wave_n * NBW + j) * 16 + l16;
            if (co >= P.Cout) continue;
            const float bv = P.bias ? P.bias[co] : 0.f;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int x = uinfo[4 * g + 3] + r;
                if (x >= P.Wout) continue;
                if (tmask[g * 16 + q * 4 + r]) continue;
                float v = acc[u][j][r] + bv;
                if (P.relu) v = v > 0.f ? v : 0.f;
                F::store(out + (row + x) * P.Cout + co, v);
            }
        }
    }
}

// ---- kernel table ---------------------------------------------------------------
struct Shape { int g, nt, wm, wn, wk; };
constexpr Shape kShapes[3] = {
    {4, 64, 2, 2, 1},   // 0: plenty of units
    {2, 32, 1, 2, 2},   // 1: medium
    {1, 32, 1, 1, 4},   // 2: few units, deep K (small maps)
};

typedef void (*KernelFn)(ConvParams);
struct KernelEntry { KernelFn fn[2][4]; };   // [dtype][KC index 0..2 vector loads, 3 = scalar loads at the smallest KC]

#define DC_K(T, S, KC, VEC) conv_units_kernel<T, kShapes[S].g, kShapes[S].nt, kShapes[S].wm, kShapes[S].wn, kShapes[S].wk, KC, VEC>
#define DC_ENTRY(S)                                                                                  \
    {{{DC_K(float, S, 16, true), DC_K(float, S, 32, true), DC_K(float, S, 64, true), DC_K(float, S, 16, false)}, \
      {DC_K(__hip_bfloat16, S, 32, true), DC_K(__hip_bfloat16, S, 64, true), DC_K(__hip_bfloat16, S, 128, true), \
       DC_K(__hip_bfloat16, S, 32, false)}}}
const KernelEntry kTable[3] = {DC_ENTRY(0), DC_ENTRY(1), DC_ENTRY(2)};

struct Choice { int shape, kci, kc, tg, ph, pw; size_t lds; bool ok; };

// Pick the channel chunk KC and taps per stage TG for a shape: the deepest stage
// (TG*KC) whose register-staged loads and LDS footprint fit.
Choice choose_stage(int shape, const ConvLaunch& c) {
    const Shape& S = kShapes[shape];
    const int nth = S.wm * S.wn * S.wk * 64;
    const size_t esz = dtype_size(c.dtype);
    const int ve = (int)(16 / esz), kg = 4 * ve;
    const int kk = c.k * c.k;
    const int ph = 3 * c.s + c.k, pw = ph;
    const bool vec_ok = (c.Cin % ve) == 0 && reinterpret_cast<uintptr_t>(c.in) % 16 == 0 &&
                        reinterpret_cast<uintptr_t>(c.w) % 16 == 0;
    Choice best{shape, 0, 0, 0, ph, pw, 0, false};
    long best_score = -1;
    for (int kci = 0; kci < 3; ++kci) {
        const int kc = kg << kci;
        if (!vec_ok && kci > 0) break;
        if (kci > 0 && kc / 2 >= c.Cin) break;   // a deeper chunk would be mostly padding
        const int nvec = kc / ve;
        const int pv = (S.g * ph * pw * nvec + nth - 1) / nth;
        if (pv > PVMAX) continue;
        int tg = (WVMAX * nth) / (S.nt * nvec);
        if (tg < 1) continue;
        if (tg > kk) tg = kk;
        if (tg > 15) tg = 15;
        const size_t kcp = kc + ve;
        auto lds_of = [&](int t) {
            return ((size_t)S.g * ph * pw * kcp + (size_t)t * S.nt * kcp) * esz + kHeaderBytes;
        };
        while (tg > 1 && lds_of(tg) > 64 * 1024) --tg;
        size_t lds = lds_of(tg);
        const size_t red = (size_t)(S.wk - 1) * S.wm * S.wn * (S.g / S.wm) * (S.nt / S.wn / 16) * 64 * 16;
        if (red + kHeaderBytes > lds) lds = red + kHeaderBytes;
        if (lds > 150 * 1024) continue;
        long score = (long)tg * (kc < c.Cin ? kc : c.Cin);   // useful K per stage
        if (score > best_score) {
            best_score = score;
            best = Choice{shape, vec_ok ? kci : 3, kc, tg, ph, pw, lds, true};
        }
    }
    return best;
}

}  // namespace

ConvTiling pick_tiling(const dc_layer&, int, int, int, int) { return ConvTiling{0, 4, 4, 64}; }

// Name of a kernel instantiation as a profiler prints it (without namespaces and arguments).
void conv_kernel_name(int id, char* buf, size_t n) {
    if (id < 0 || id >= 24) { snprintf(buf, n, "?"); return; }
    const int kci = id & 3, shape = (id >> 2) % 3, bf16 = (id >> 2) / 3;
    const Shape& S = kShapes[shape];
    const int kg = bf16 ? 32 : 16;
    const int kc = kci == 3 ? kg : (kg << kci);
    snprintf(buf, n, "conv_units_kernel<%s, %d, %d, %d, %d, %d, %d, %s>", bf16 ? "__hip_bfloat16" : "float", S.g, S.nt,
             S.wm, S.wn, S.wk, kc, kci == 3 ? "false" : "true");
}

hipError_t launch_conv(const ConvLaunch& c, hipStream_t st) {
    const int units_y = (c.Hout + 3) / 4, units_x = (c.Wout + 3) / 4;
    const long n_units = c.tiles ? c.n_tiles : (long)c.n_streams * units_x * units_y;
    if (n_units <= 0) return hipSuccess;
    if (c.k * c.k > kMaxTaps) return hipErrorInvalidValue;
    // 32-bit element offsets inside the kernel
    if ((double)c.n_streams * c.Hin * c.Win * c.Cin >= 2147483648.0 ||
        (double)c.Cout * c.k * c.k * c.Cin >= 2147483648.0)
        return hipErrorInvalidValue;
    // shape by the amount of work: largest tile that still fills the chip
    int shape;
    {
        const long r64 = (c.Cout + 63) / 64, r32 = (c.Cout + 31) / 32;
        if (c.Cout > 32 && ((n_units + 3) / 4) * r64 >= 384) shape = 0;
        else if (((n_units + 1) / 2) * r32 >= 256) shape = 1;
        else shape = 2;
    }
    Choice ch = choose_stage(shape, c);
    for (int s2 = shape + 1; !ch.ok && s2 < 3; ++s2) ch = choose_stage(s2, c);
    if (!ch.ok) return hipErrorInvalidValue;
    const Shape& S = kShapes[ch.shape];

    ConvParams P;
    P.in = c.in; P.w = c.w; P.bias = c.bias; P.out = c.out;
    P.Hin = c.Hin; P.Win = c.Win; P.Cin = c.Cin; P.Hout = c.Hout; P.Wout = c.Wout; P.Cout = c.Cout;
    P.k = c.k; P.s = c.s; P.p = c.p; P.relu = c.relu;
    P.units = c.tiles; P.n_units = (int)n_units; P.rects = c.rects; P.ranges = c.ranges;
    P.units_x = units_x; P.units_y = units_y;
    P.ph = ch.ph; P.pw = ch.pw; P.tg = ch.tg;
    P.n_tapgroups = (c.k * c.k + ch.tg - 1) / ch.tg;
    P.n_chunks = (c.Cin + ch.kc - 1) / ch.kc;
    P.R = (c.Cout + S.nt - 1) / S.nt;
    KernelFn fn = kTable[ch.shape].fn[c.dtype == DC_BF16 ? 1 : 0][ch.kci];
    if (c.kernel_id) *c.kernel_id = ((c.dtype == DC_BF16 ? 1 : 0) * 3 + ch.shape) * 4 + ch.kci;
    if (ch.lds > 64 * 1024) {
        hipError_t a = hipFuncSetAttribute(reinterpret_cast<const void*>(fn),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)ch.lds);
        if (a != hipSuccess) return a;
    }
    const long groups = (n_units + S.g - 1) / S.g;
    const long wgs = groups * P.R;
    if (wgs > 2147483647L) return hipErrorInvalidValue;
    hipLaunchKernelGGL(fn, dim3((unsigned)wgs), dim3(S.wm * S.wn * S.wk * 64), ch.lds, st, P);
    return hipGetLastError();
}

}  // namespace dc
