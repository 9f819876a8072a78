// Cache-aware convolution (Section 5 "Reuse", steps 2-3) as an implicit GEMM on the
// gfx950 matrix cores over a compacted list of 4x4-pixel output units that hold at
// least one non-reusable pixel.
//
//   M = G units x 16 pixels, N = NT output channels, K = k*k*cin.
//
// A workgroup takes G consecutive units of the list (any positions, any streams) and
// NT output channels.  K is walked in stages of (TG taps) x (KC channels): the input
// patch of every unit ((3s+k)^2 pixels x KC channels) is staged in LDS once per channel
// chunk, the weight slices [TG][NT][KC] once per stage.
//
// Two kernels share the unit decoding, the MFMA loop structure and the epilogue:
//  - conv_direct_kernel (channel runs that are whole 16-byte vectors): the stage is loaded
//    with buffer_load ... lds (memory -> LDS without passing registers) into one of two LDS
//    buffers while the matrix cores work on the other; one barrier per stage.  LDS rows are
//    unpadded (a load instruction fills 1 KiB of consecutive LDS), so the 16-byte chunks of
//    a row are XOR-swizzled by the row index to keep fragment reads spread over the banks;
//    the swizzle is applied on the global-address side of the load.
//  - conv_staged_kernel (any channel count): element-wise buffer loads into registers,
//    written to padded LDS rows after the MFMAs of the previous stage.
// Out-of-range pixels (zero padding), channels, taps and units are loaded from a buffer
// offset beyond the tensor, for which the hardware returns zeros.
//
// MFMA 16x16: the weights are the A operand (rows = channels), the pixels the B operand
// (columns = pixels of a unit); lane l holds row/column l%16 and the K elements
// [VE*(l/16), VE*(l/16)+VE) of each K group for both operands, so one 16-byte LDS read per
// operand feeds four fp32 MFMAs (16x16x4) or one bf16 MFMA (16x16x32).  Accumulator
// register r of lane l is channel 4*(l/16)+r of the block at pixel l%16 of the unit, so
// the epilogue stores four consecutive channels per lane.
//
// WK > 1: the wavefronts of a workgroup split the K steps of every stage among
// themselves and add their accumulators through LDS in a fixed order (deterministic).
//
// Epilogue: bias, ReLU, rounding to the storage type, and a per-pixel predicate: a pixel
// inside a reusable rectangle keeps the value the shifted copy wrote.
#include <hip/hip_bf16.h>

#include <cstdio>
#include <cstdlib>

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

__device__ __forceinline__ int fast_div(int n, uint32_t magic) { return (int)__umulhi((uint32_t)n, magic); }

// ---- pieces shared by both kernels ------------------------------------------------

// LDS header: uinfo[G][4] = {valid, stream, oy0, ox0}, tmask[G*16], umixed[G]
template <int G>
struct Header {
    int* uinfo;
    unsigned char* tmask;
    unsigned char* umixed;
    __device__ __forceinline__ explicit Header(unsigned char* smem)
        : uinfo(reinterpret_cast<int*>(smem)),
          tmask(reinterpret_cast<unsigned char*>(smem) + 16 * G),
          umixed(reinterpret_cast<unsigned char*>(smem) + 32 * G) {}
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
__device__ __forceinline__ void decode_units(const ConvParams& P, const Header<G>& H, int ug, int tid) {
    if (tid < G) {
        const int u = ug * P.g_rt + tid;
        int valid = tid < P.g_rt && u < P.n_units, stream = 0, uy = 0, ux = 0, mixed = 0;
        if (valid) {
            if (P.units) {
                const TileDev t = P.units[u];
                stream = t.stream; uy = t.ty; ux = t.tx; mixed = t.mixed;
            } else {
                const int per = P.units_x * P.units_y;
                stream = u / per;
                const int r = u - stream * per;
                uy = r / P.units_x; ux = r - uy * P.units_x;
            }
        }
        H.uinfo[4 * tid + 0] = valid; H.uinfo[4 * tid + 1] = stream;
        H.uinfo[4 * tid + 2] = uy * 4; H.uinfo[4 * tid + 3] = ux * 4;
        H.umixed[tid] = (unsigned char)mixed;
    }
    __syncthreads();
    for (int m = tid; m < G * 16; m += NTHREADS) {   // per-pixel reuse mask of mixed units
        const int g = m >> 4;
        unsigned char hit = 0;
        if (H.umixed[g]) {
            const int y = H.uinfo[4 * g + 2] + ((m >> 2) & 3), x = H.uinfo[4 * g + 3] + (m & 3);
            const RangeDev rg = P.ranges[H.uinfo[4 * g + 1]];
            for (int i = 0; i < rg.count; ++i) {
                const RectDev r = P.rects[rg.begin + i];
                hit |= (x >= r.x && x < r.x + r.w && y >= r.y && y < r.y + r.h) ? 1 : 0;
            }
        }
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
    const int iy = H.uinfo[4 * g + 2] * P.s - P.p + py, ix = H.uinfo[4 * g + 3] * P.s - P.p + px;
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
                if (P.relu) { v[0] = fmaxf(v[0], 0.f); v[1] = fmaxf(v[1], 0.f); v[2] = fmaxf(v[2], 0.f); v[3] = fmaxf(v[3], 0.f); }
                F::store4(px + co, v);
            } else {
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    if (co + r >= P.Cout) continue;
                    float s = v[r] + (P.bias ? P.bias[co + r] : 0.f);
                    if (P.relu) s = fmaxf(s, 0.f);
                    F::store1(px + co + r, s);
                }
            }
        }
    }
}

// ---- direct-to-LDS kernel ------------------------------------------------------------
//
// LDS rows are RB = KC*sizeof(T) bytes (64, 128 or 256) without padding.  RPC = 256/RB rows
// share one pass over the 64 banks; chunk c (16 bytes) of row r is stored at chunk position
// c ^ ((r / RPC) % NVEC), which makes any 16 consecutive rows conflict-free for a fixed c.
template <typename T, int G, int NT, int WM, int WN, int WK, int KC>
__global__ __launch_bounds__(WM* WN* WK * 64) void conv_direct_kernel(ConvParams P) {
    typedef Frag<T> F;
    typedef typename F::vec vec;
    constexpr int VE = F::VE;
    constexpr int ES = (int)sizeof(T);
    constexpr int KG = 4 * VE;                 // K elements per MFMA group
    constexpr int NWAVES = WM * WN * WK;
    constexpr int NTHREADS = NWAVES * 64;
    constexpr int UPW = G / WM;                // units per wavefront
    constexpr int NBW = NT / WN / 16;          // 16-channel blocks per wavefront
    constexpr int GPC = KC / KG;               // K groups per chunk
    constexpr int NVEC = KC / VE;              // 16-byte chunks per row
    constexpr int RB = KC * ES;                // row bytes
    constexpr int RPC = 256 / RB;              // rows per pass over the banks
    constexpr int RPI = 64 / NVEC;             // rows filled by one load instruction (1 KiB)
    constexpr int UC = UPW >= 2 ? 2 : 1;       // units per compute group
    static_assert(G % WM == 0 && NT % (WN * 16) == 0 && KC % KG == 0 && RB <= 256, "tile shape");

    extern __shared__ __align__(16) unsigned char smem[];
    const Header<G> H(smem);
    unsigned char* const stage0 = smem + kHeaderBytes;
    // [patch 0][patch 1][weights 0][weights 1]
    const int npix = P.ph * P.pw;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave id in a scalar register
    const int wave_k = wave % WK, wave_n = (wave / WK) % WN, wave_m = wave / (WK * WN);
    const int l16 = lane & 15, q = lane >> 4;
    const int kk = P.k * P.k;

    int ug, ntile;
    decode_workgroup(P.R, ug, ntile);
    const int n0 = ntile * NT;
    decode_units<G, NTHREADS>(P, H, ug, tid);

    const __amdgpu_buffer_rsrc_t in_rsrc = __builtin_amdgcn_make_buffer_rsrc(
        reinterpret_cast<void*>(keep_scalar(reinterpret_cast<uintptr_t>(P.in))), 0, keep_scalar(P.in_bytes), kBufferFlags);
    const __amdgpu_buffer_rsrc_t w_rsrc = __builtin_amdgcn_make_buffer_rsrc(
        reinterpret_cast<void*>(keep_scalar(reinterpret_cast<uintptr_t>(P.w))), 0, keep_scalar(P.w_bytes), kBufferFlags);

    // ---- load slots: instruction j of a buffer fills LDS bytes [1024 j, 1024 j + 1024); this
    // wavefront issues instructions wave, wave + NWAVES, ...; lane fills chunk position lane % NVEC
    // of row j * RPI + lane / NVEC and therefore fetches logical chunk pos ^ swizzle(row).
    const int lrow = lane / NVEC, lpos = lane % NVEC;
    uint32_t pgo[DPMAX];   // byte offset at chunk 0 | logical chunk index in the low 4 bits
#pragma unroll
    for (int i = 0; i < DPMAX; ++i) {
        const int row = (wave + i * NWAVES) * RPI + lrow;
        const int c = lpos ^ ((row / RPC) % NVEC);
        const uint32_t base = patch_pixel_offset<G, ES>(P, H, row, npix);
        pgo[i] = base == kOob ? kOob : (base + c * 16) | (uint32_t)c;
    }
    uint32_t wgo[DWMAX];   // byte offset at chunk 0, tap 0 of the stage | logical chunk index
    int wtl[DWMAX];        // tap of the slot inside the stage
#pragma unroll
    for (int i = 0; i < DWMAX; ++i) {
        const int row = (wave + i * NWAVES) * RPI + lrow;   // tl * NT + n
        const int c = lpos ^ ((row / RPC) % NVEC);
        const int tl = row / NT, n = row - tl * NT;
        wtl[i] = tl;
        wgo[i] = (tl < P.tg && n0 + n < P.Cout) ? ((uint32_t)(((n0 + n) * kk + tl) * P.Cin) * ES + c * 16) | (uint32_t)c : kOob;
    }

    // loop-invariant scalars, pinned in SGPRs
    const int Cin = keep_scalar(P.Cin), kdim = keep_scalar(P.k), pwid = keep_scalar(P.pw), tgs = keep_scalar(P.tg);
    const int n_tapgroups = keep_scalar(P.n_tapgroups), patch_bytes = keep_scalar(P.patch_bytes);
    const int weight_bytes = keep_scalar(P.weight_bytes);
    const int np_slots = keep_scalar((P.p_instr - wave + NWAVES - 1) / NWAVES);   // load instructions of this wavefront
    const int nw_slots = keep_scalar((P.w_instr - wave + NWAVES - 1) / NWAVES);
    const int tails = keep_scalar(P.chan_tail | P.tap_tail);

    auto issue_stage = [&](int chunk, int tgi, int pbuf, int wbuf) {
        const int c0 = chunk * KC;
        if (tgi == 0) {
            unsigned char* dst = stage0 + pbuf * patch_bytes + wave * 1024;
#pragma unroll
            for (int i = 0; i < DPMAX; ++i) {
                if (i < np_slots) {
                    uint32_t off = pgo[i] + (uint32_t)c0 * ES;   // kOob stays out of range; the low 4 bits are ignored below
                    if (tails) off = (pgo[i] != kOob && c0 + (int)(pgo[i] & 15) * VE < Cin) ? off : kOob;
                    off &= ~15u;
                    __builtin_amdgcn_raw_ptr_buffer_load_lds(in_rsrc, (__attribute__((address_space(3))) void*)(dst + i * (NWAVES * 1024)),
                                                             16, off, 0, 0, 0);
                }
            }
        }
        const int tap0 = tgi * tgs;
        unsigned char* dst = stage0 + 2 * patch_bytes + wbuf * weight_bytes + wave * 1024;
        const uint32_t stage_off = (uint32_t)(tap0 * Cin + c0) * ES;
#pragma unroll
        for (int i = 0; i < DWMAX; ++i) {
            if (i < nw_slots) {
                uint32_t off = wgo[i] + stage_off;
                if (tails)
                    off = (wgo[i] != kOob && tap0 + wtl[i] < kk && c0 + (int)(wgo[i] & 15) * VE < Cin) ? off : kOob;
                off &= ~15u;
                __builtin_amdgcn_raw_ptr_buffer_load_lds(w_rsrc, (__attribute__((address_space(3))) void*)(dst + i * (NWAVES * 1024)),
                                                         16, off, 0, 0, 0);
            }
        }
    };

    // ---- per-lane fragment rows ----
    int xrow[UPW];   // patch row of this lane's pixel at tap (0,0)
#pragma unroll
    for (int u = 0; u < UPW; ++u) xrow[u] = (u * WM + wave_m) * npix + ((l16 >> 2) * P.s) * P.pw + (l16 & 3) * P.s;
    const int n_u = keep_scalar((P.g_rt - wave_m + WM - 1) / WM);   // units of this wavefront: wave_m, wave_m + WM, ...
    int wbase[NBW];  // byte offset of this lane's weight row at tap 0 of the stage
#pragma unroll
    for (int j = 0; j < NBW; ++j) wbase[j] = ((wave_n * NBW + j) * 16 + l16) * RB;
    const int wswz = (l16 / RPC) % NVEC;   // rows tl*NT + 16 m + l16 all share this swizzle

    floatx4 acc[UPW][NBW];
#pragma unroll
    for (int u = 0; u < UPW; ++u)
#pragma unroll
        for (int j = 0; j < NBW; ++j) acc[u][j] = floatx4{0.f, 0.f, 0.f, 0.f};

    const int n_stages = keep_scalar(P.n_chunks * P.n_tapgroups);
    issue_stage(0, 0, 0, 0);
    int chunk = 0, tgi = 0;
    for (int st = 0; st < n_stages; ++st) {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // this wavefront's loads of stage st are in LDS
        __syncthreads();                                   // ... and everybody's; stage st-1 is fully consumed
        int nchunk = chunk, ntgi = tgi + 1;
        if (ntgi == n_tapgroups) { ntgi = 0; ++nchunk; }
        if (st + 1 < n_stages) issue_stage(nchunk, ntgi, nchunk & 1, (st + 1) & 1);   // fills the other buffers

        const unsigned char* patch = stage0 + (chunk & 1) * patch_bytes;
        const unsigned char* wt = stage0 + 2 * patch_bytes + (st & 1) * weight_bytes;
        const int tap0 = tgi * tgs;
        const int ntap = (kk - tap0) < tgs ? (kk - tap0) : tgs;
        const int steps = ntap * GPC;
        int sidx = wave_k;
        if (sidx < steps) {
            int tl = sidx / GPC, g = sidx - tl * GPC;
            int ky = (tap0 + tl) / kdim, kx = (tap0 + tl) - ky * kdim;
            vec x0[UPW], w0[NBW], x1[UPW], w1[NBW];
            auto frag = [&](vec (&xv)[UPW], vec (&wv)[NBW]) {
                const int trow = ky * pwid + kx, c = g * 4 + q;
#pragma unroll
                for (int u0 = 0; u0 < UPW; u0 += UC) {
                    if (u0 < n_u) {     // units are handled in groups of UC: one uniform branch per group
#pragma unroll
                        for (int u = u0; u < u0 + UC; ++u) {
                            const uint32_t row = (uint32_t)(xrow[u] + trow);
                            xv[u] = *reinterpret_cast<const vec*>(patch + row * RB + (((uint32_t)c ^ ((row / RPC) % NVEC)) << 4));
                        }
                    }
                }
                const int woff = tl * (NT * RB) + ((c ^ wswz) << 4);
#pragma unroll
                for (int j = 0; j < NBW; ++j) wv[j] = *reinterpret_cast<const vec*>(wt + wbase[j] + woff);
            };
            auto advance = [&]() {   // move (tl, g, ky, kx) forward by WK steps
                g += WK;
                while (g >= GPC) {
                    g -= GPC; ++tl; ++kx;
                    if (kx == kdim) { kx = 0; ++ky; }
                }
            };
            auto mma = [&](const vec (&xv)[UPW], const vec (&wv)[NBW]) {
#pragma unroll
                for (int u0 = 0; u0 < UPW; u0 += UC) {
                    if (u0 < n_u) {     // UC * NBW independent accumulator chains are interleaved
#pragma unroll
                        for (int e = 0; e < F::NE; ++e)
#pragma unroll
                            for (int u = u0; u < u0 + UC; ++u)
#pragma unroll
                                for (int j = 0; j < NBW; ++j) F::mma1(wv[j], xv[u], acc[u][j], e);
                    }
                }
            };
            frag(x0, w0);
            for (;;) {
                sidx += WK;
                if (sidx < steps) { advance(); frag(x1, w1); }
                mma(x0, w0);
                if (sidx >= steps) break;
                sidx += WK;
                if (sidx < steps) { advance(); frag(x0, w0); }
                mma(x1, w1);
                if (sidx >= steps) break;
            }
        }
        chunk = nchunk; tgi = ntgi;
    }

    if (!reduce_k_split<WM, WN, WK, UPW, NBW>(acc, stage0, wave, lane)) return;
    epilogue<T, G, UPW, NBW>(P, H, acc, wave_m, WM, n0 + wave_n * NBW * 16, l16, q);
}

// ---- register-staged kernel (any channel count) -----------------------------------------
template <typename T, int G, int NT, int WM, int WN, int WK, int KC>
__global__ __launch_bounds__(WM* WN* WK * 64) void conv_staged_kernel(ConvParams P) {
    typedef Frag<T> F;
    typedef typename F::vec vec;
    constexpr int VE = F::VE;
    constexpr int ES = (int)sizeof(T);
    constexpr int KG = 4 * VE;
    constexpr int NTHREADS = WM * WN * WK * 64;
    constexpr int UPW = G / WM;
    constexpr int NBW = NT / WN / 16;
    constexpr int KCP = KC + VE;               // padded channel run (elements)
    constexpr int GPC = KC / KG;
    constexpr int NVEC = KC / VE;
    constexpr int RS = NTHREADS / NVEC;        // LDS rows covered per slot step
    static_assert(G % WM == 0 && NT % (WN * 16) == 0 && KC % KG == 0 && NTHREADS % NVEC == 0, "tile shape");

    extern __shared__ __align__(16) unsigned char smem[];
    const Header<G> H(smem);
    const int npix = P.ph * P.pw;
    T* patch = reinterpret_cast<T*>(smem + kHeaderBytes);
    T* wt = reinterpret_cast<T*>(smem + kHeaderBytes + P.patch_bytes);
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wave_k = wave % WK, wave_n = (wave / WK) % WN, wave_m = wave / (WK * WN);
    const int l16 = lane & 15, q = lane >> 4;
    const int kk = P.k * P.k;

    int ug, ntile;
    decode_workgroup(P.R, ug, ntile);
    const int n0 = ntile * NT;
    decode_units<G, NTHREADS>(P, H, ug, tid);

    const __amdgpu_buffer_rsrc_t in_rsrc = __builtin_amdgcn_make_buffer_rsrc(
        reinterpret_cast<void*>(keep_scalar(reinterpret_cast<uintptr_t>(P.in))), 0, keep_scalar(P.in_bytes), kBufferFlags);
    const __amdgpu_buffer_rsrc_t w_rsrc = __builtin_amdgcn_make_buffer_rsrc(
        reinterpret_cast<void*>(keep_scalar(reinterpret_cast<uintptr_t>(P.w))), 0, keep_scalar(P.w_bytes), kBufferFlags);

    // slot i of a thread covers LDS row (tid / NVEC) + i * RS, vector tid % NVEC
    const int row0 = tid / NVEC, chv = (tid % NVEC) * VE;
    const int lds0 = row0 * KCP + chv;
    uint32_t pgo[PVMAX];
#pragma unroll
    for (int i = 0; i < PVMAX; ++i) {
        const uint32_t base = patch_pixel_offset<G, ES>(P, H, row0 + i * RS, npix);
        pgo[i] = base == kOob ? kOob : base + chv * ES;
    }
    uint32_t wgo[WVMAX];
    int wtl[WVMAX];
#pragma unroll
    for (int i = 0; i < WVMAX; ++i) {
        const int wrow = row0 + i * RS;        // tl * NT + n
        const int tl = wrow / NT, n = wrow - tl * NT;
        wtl[i] = tl;
        wgo[i] = (tl < P.tg && n0 + n < P.Cout) ? (uint32_t)(((n0 + n) * kk + tl) * P.Cin + chv) * ES : kOob;
    }

    int xbase[UPW], wbase[NBW];
#pragma unroll
    for (int u = 0; u < UPW; ++u)
        xbase[u] = ((wave_m * UPW + u) * npix + ((l16 >> 2) * P.s) * P.pw + (l16 & 3) * P.s) * KCP + q * VE;
#pragma unroll
    for (int j = 0; j < NBW; ++j) wbase[j] = ((wave_n * NBW + j) * 16 + l16) * KCP + q * VE;

    floatx4 acc[UPW][NBW];
#pragma unroll
    for (int u = 0; u < UPW; ++u)
#pragma unroll
        for (int j = 0; j < NBW; ++j) acc[u][j] = floatx4{0.f, 0.f, 0.f, 0.f};

    vec pr[PVMAX], wr[WVMAX];
    // Straight-line code: every slot is always loaded; a slot that is unused, out of range or beyond
    // the last stage reads offset kOob and receives zeros.
    auto load_stage = [&](int chunk, int tgi, bool live) {
        const int c0 = chunk * KC;
        const bool p_live = live && tgi == 0;
#pragma unroll
        for (int i = 0; i < PVMAX; ++i)
#pragma unroll
            for (int e = 0; e < VE; ++e) {
                const bool ok = p_live && pgo[i] != kOob && c0 + chv + e < P.Cin;
                pr[i][e] = F::elem(in_rsrc, ok ? pgo[i] + (uint32_t)(c0 + e) * ES : kOob);
            }
        const int tap0 = tgi * P.tg;
#pragma unroll
        for (int i = 0; i < WVMAX; ++i)
#pragma unroll
            for (int e = 0; e < VE; ++e) {
                const bool ok = live && wgo[i] != kOob && tap0 + wtl[i] < kk && c0 + chv + e < P.Cin;
                wr[i][e] = F::elem(w_rsrc, ok ? wgo[i] + (uint32_t)(tap0 * P.Cin + c0 + e) * ES : kOob);
            }
    };
    // unused slots go to a per-thread dump slot
    T* dump = reinterpret_cast<T*>(smem + kHeaderBytes + P.dump_off) + tid * VE;
    auto store_stage = [&](int tgi) {
#pragma unroll
        for (int i = 0; i < PVMAX; ++i) {
            T* dst = (i < P.pv && tgi == 0) ? patch + lds0 + i * (RS * KCP) : dump;
            *reinterpret_cast<vec*>(dst) = pr[i];
        }
#pragma unroll
        for (int i = 0; i < WVMAX; ++i) {
            T* dst = (i < P.wv) ? wt + lds0 + i * (RS * KCP) : dump;
            *reinterpret_cast<vec*>(dst) = wr[i];
        }
    };

    const int n_stages = P.n_chunks * P.n_tapgroups;
    load_stage(0, 0, true);
    int chunk = 0, tgi = 0;
    for (int st = 0; st < n_stages; ++st) {
        __syncthreads();           // every wavefront is done with the previous stage's LDS
        store_stage(tgi);
        __syncthreads();
        int nchunk = chunk, ntgi = tgi + 1;
        if (ntgi == P.n_tapgroups) { ntgi = 0; ++nchunk; }
        load_stage(nchunk, ntgi, st + 1 < n_stages);   // in flight during the MFMAs below

        const int tap0 = tgi * P.tg;
        const int ntap = (kk - tap0) < P.tg ? (kk - tap0) : P.tg;
        const int steps = ntap * GPC;
        for (int sidx = wave_k; sidx < steps; sidx += WK) {
            const int tl = sidx / GPC, g = sidx - tl * GPC;
            const int ky = (tap0 + tl) / P.k, kx = (tap0 + tl) - ky * P.k;
            const int xoff = (ky * P.pw + kx) * KCP + g * KG;
            const int woff = tl * (NT * KCP) + g * KG;
            vec xv[UPW], wv[NBW];
#pragma unroll
            for (int u = 0; u < UPW; ++u) xv[u] = *reinterpret_cast<const vec*>(patch + xbase[u] + xoff);
#pragma unroll
            for (int j = 0; j < NBW; ++j) wv[j] = *reinterpret_cast<const vec*>(wt + wbase[j] + woff);
#pragma unroll
            for (int u = 0; u < UPW; ++u)
#pragma unroll
                for (int j = 0; j < NBW; ++j) F::mma(wv[j], xv[u], acc[u][j]);
        }
        chunk = nchunk; tgi = ntgi;
    }

    if (!reduce_k_split<WM, WN, WK, UPW, NBW>(acc, smem + kHeaderBytes, wave, lane)) return;
    epilogue<T, G, UPW, NBW>(P, H, acc, wave_m * UPW, 1, n0 + wave_n * NBW * 16, l16, q);
}

// ---- kernel table ---------------------------------------------------------------
struct Shape { int g, nt, wm, wn, wk; };
// Eight wavefronts per workgroup: two per SIMD, so that one issues MFMAs while the other computes
// addresses and waits for LDS.
constexpr int kNumShapes = 4;
constexpr Shape kShapes[kNumShapes] = {
    {4, 64, 2, 2, 2},   // 0: plenty of units
    {2, 32, 1, 2, 4},   // 1: medium
    {1, 32, 1, 1, 8},   // 2: few units, deep K (small maps)
    {16, 64, 2, 4, 1},  // 3: up to 16 units per workgroup (the count is a launch parameter): large maps
};

typedef void (*KernelFn)(ConvParams);
// [dtype][0..2: direct kernel with KC = KG, 2 KG, 4 KG; 3: staged kernel with KC = KG]
struct KernelEntry { KernelFn fn[2][4]; };

#define DC_D(T, S, KC) conv_direct_kernel<T, kShapes[S].g, kShapes[S].nt, kShapes[S].wm, kShapes[S].wn, kShapes[S].wk, KC>
#define DC_S(T, S, KC) conv_staged_kernel<T, kShapes[S].g, kShapes[S].nt, kShapes[S].wm, kShapes[S].wn, kShapes[S].wk, KC>
#define DC_ENTRY(S)                                                                       \
    {{{DC_D(float, S, 16), DC_D(float, S, 32), DC_D(float, S, 64), DC_S(float, S, 16)},   \
      {DC_D(__hip_bfloat16, S, 32), DC_D(__hip_bfloat16, S, 64), DC_D(__hip_bfloat16, S, 128), DC_S(__hip_bfloat16, S, 32)}}}
const KernelEntry kTable[kNumShapes] = {DC_ENTRY(0), DC_ENTRY(1), DC_ENTRY(2), DC_ENTRY(3)};

struct Choice { int shape, kci, kc, tg, pv, wv, patch_bytes, weight_bytes, dump_off; size_t lds; bool ok; int p_instr, w_instr; };
bool tune_override(int& kci, int& tg);

size_t reduce_bytes(const Shape& S) {
    return (size_t)(S.wk - 1) * S.wm * S.wn * (S.g / S.wm) * (S.nt / S.wn / 16) * 64 * 16;
}

// Direct kernel: pick the channel chunk KC and taps per stage TG with the deepest stage
// (TG*KC useful K) whose two LDS buffers fit.
Choice choose_direct(int shape, const ConvLaunch& c, int ph, int pw) {
    const Shape& S = kShapes[shape];
    const int nwaves = S.wm * S.wn * S.wk;
    const size_t esz = dtype_size(c.dtype);
    const int ve = (int)(16 / esz), kg = 4 * ve;
    const int kk = c.k * c.k;
    Choice best{shape, 0, 0, 0, 0, 0, 0, 0, 0, 0, false, 0, 0};
    long best_score = -1;
    int f_kci = -1, f_tg = 0;
    const bool forced = tune_override(f_kci, f_tg);
    for (int kci = 0; kci < 3; ++kci) {
        const int kc = kg << kci;
        if (kci > 0 && kc / 2 >= c.Cin) break;   // a deeper chunk would be mostly padding
        if (forced && kci != f_kci && f_kci >= 0 && f_kci < 3 && (kg << f_kci) / 2 < c.Cin) continue;
        const int rb = kc * (int)esz, rpi = 1024 / rb;           // rows per load instruction
        const int p_instr = (S.g * ph * pw + rpi - 1) / rpi;
        const int pv = (p_instr + nwaves - 1) / nwaves;
        if (pv > DPMAX) continue;
        const size_t patch_bytes = (size_t)p_instr * 1024;
        // taps per stage: balanced splits of the k*k taps only (ceil(kk/m)), so that no stage is much shorter
        // than the loads it has to hide
        for (int m = 1; m <= kk; ++m) {
            int tg = (kk + m - 1) / m;
            if (m > 1 && tg == (kk + m - 2) / (m - 1)) continue;
            if (forced && f_tg >= 1 && f_tg <= kk) { if (m > 1) break; tg = f_tg; }
            const int w_instr = (tg * S.nt + rpi - 1) / rpi;
            const int wv = (w_instr + nwaves - 1) / nwaves;
            if (wv > DWMAX) continue;
            const size_t weight_bytes = (size_t)w_instr * 1024;
            size_t body = 2 * patch_bytes + 2 * weight_bytes;
            if (body < reduce_bytes(S)) body = reduce_bytes(S);
            const size_t lds = kHeaderBytes + body;
            if (lds > 160 * 1024) continue;
            // useful K per stage; prefer stages that keep two workgroups per CU when the gain is small
            long score = (long)tg * (kc < c.Cin ? kc : c.Cin);
            if (lds > 80 * 1024) score = score * 3 / 4;
            if (score > best_score) {
                best_score = score;
                best = Choice{shape, kci, kc, tg, pv, wv, (int)patch_bytes, (int)weight_bytes, 0, lds, true, p_instr, w_instr};
            }
            break;   // smaller tg only lowers the score for this kc (unless LDS-limited: handled by continue)
        }
    }
    return best;
}

Choice choose_staged(int shape, const ConvLaunch& c, int ph, int pw) {
    const Shape& S = kShapes[shape];
    const int nth = S.wm * S.wn * S.wk * 64;
    const size_t esz = dtype_size(c.dtype);
    const int ve = (int)(16 / esz), kc = 4 * ve;
    const int kk = c.k * c.k;
    const int nvec = kc / ve, rs = nth / nvec, kcp = kc + ve;
    Choice ch{shape, 3, kc, 0, 0, 0, 0, 0, 0, 0, false, 0, 0};
    const int pv = (S.g * ph * pw + rs - 1) / rs;
    if (pv > PVMAX) return ch;
    int tg = (WVMAX * rs) / S.nt;
    if (tg < 1) return ch;
    if (tg > kk) tg = kk;
    const size_t patch_bytes = (size_t)pv * rs * kcp * esz;
    auto wv_of = [&](int t) { return (t * S.nt + rs - 1) / rs; };
    auto body_of = [&](int t) { return patch_bytes + (size_t)wv_of(t) * rs * kcp * esz; };
    while (tg > 1 && body_of(tg) > 56 * 1024) --tg;
    size_t body = body_of(tg);
    const int dump_off = (int)body;
    body += (size_t)nth * 16;
    if (body < reduce_bytes(S)) body = reduce_bytes(S);
    ch.tg = tg; ch.pv = pv; ch.wv = wv_of(tg); ch.patch_bytes = (int)patch_bytes;
    ch.weight_bytes = (int)(body_of(tg) - patch_bytes); ch.dump_off = dump_off;
    ch.lds = kHeaderBytes + body; ch.ok = ch.lds <= 150 * 1024;
    return ch;
}

// Optional override for experiments: DC_CONV_TUNE="kci,tg" forces the channel-chunk index and the
// taps per stage of the direct kernel (ignored when the combination does not fit).
bool tune_override(int& kci, int& tg) {
    static int cached = -1, o_kci = 0, o_tg = 0;
    if (cached < 0) {
        const char* e = getenv("DC_CONV_TUNE");
        cached = (e && sscanf(e, "%d,%d", &o_kci, &o_tg) == 2) ? 1 : 0;
    }
    if (cached == 1) { kci = o_kci; tg = o_tg; }
    return cached == 1;
}

uint32_t magic_of(int d) { return (uint32_t)((0x100000000ull + (uint64_t)d - 1) / (uint64_t)d); }

}  // namespace

ConvTiling pick_tiling(const dc_layer&, int, int, int, int) { return ConvTiling{0, 4, 4, 64}; }

// Name of a kernel instantiation as a profiler prints it (without namespaces and arguments).
void conv_kernel_name(int id, char* buf, size_t n) {
    if (id < 0 || id >= 8 * kNumShapes) { snprintf(buf, n, "?"); return; }
    const int kci = id & 3, shape = (id >> 2) % kNumShapes, bf16 = (id >> 2) / kNumShapes;
    const Shape& S = kShapes[shape];
    const int kg = bf16 ? 32 : 16;
    const int kc = kci == 3 ? kg : (kg << kci);
    snprintf(buf, n, "%s<%s, %d, %d, %d, %d, %d, %d>", kci == 3 ? "conv_staged_kernel" : "conv_direct_kernel",
             bf16 ? "__hip_bfloat16" : "float", S.g, S.nt, S.wm, S.wn, S.wk, kc);
}

hipError_t launch_conv(const ConvLaunch& c, hipStream_t st) {
    const int units_y = (c.Hout + 3) / 4, units_x = (c.Wout + 3) / 4;
    const long n_units = c.tiles ? c.n_tiles : (long)c.n_streams * units_x * units_y;
    if (n_units <= 0) return hipSuccess;
    if (c.k > kMaxK) return hipErrorInvalidValue;
    // buffer loads address each tensor with 31-bit byte offsets
    if ((double)c.n_streams * c.Hin * c.Win * c.Cin * dtype_size(c.dtype) >= 2147483648.0 ||
        (double)c.Cout * c.k * c.k * c.Cin * dtype_size(c.dtype) >= 2147483648.0)
        return hipErrorInvalidValue;
    // Shape by the amount of work.  With enough units a workgroup takes g of them (up to 16) and 64
    // channels, g chosen so that the launch fills the 256 CUs in whole rounds; with few units the
    // smaller shapes split K among the wavefronts instead.
    int shape, g_rt;
    {
        static int t1 = -1, xl_min = -1;
        if (t1 < 0) {
            const char* e1 = getenv("DC_CONV_T1");
            const char* e2 = getenv("DC_CONV_XLMIN");
            t1 = e1 ? atoi(e1) : 160;
            xl_min = e2 ? atoi(e2) : 8;
        }
        const long r64 = (c.Cout + 63) / 64, r32 = (c.Cout + 31) / 32;
        const long rounds = (n_units * r64 + 256 * 16 - 1) / (256 * 16);
        const long g = (n_units * r64 + 256 * rounds - 1) / (256 * rounds);
        if (c.Cout > 32 && g >= xl_min) { shape = 3; g_rt = (int)(g > 16 ? 16 : g); }
        else if (c.Cout > 32 && ((n_units + 3) / 4) * r64 >= 160) { shape = 0; g_rt = 4; }
        else if (((n_units + 1) / 2) * r32 >= t1) { shape = 1; g_rt = 2; }
        else { shape = 2; g_rt = 1; }
    }
    const int ph = 3 * c.s + c.k, pw = ph;
    const size_t esz = dtype_size(c.dtype);
    const bool vec_ok = (c.Cin % (16 / esz)) == 0 && reinterpret_cast<uintptr_t>(c.in) % 16 == 0 &&
                        reinterpret_cast<uintptr_t>(c.w) % 16 == 0;
    Choice ch{};
    for (int s2 = shape; s2 < 4; s2 = (s2 == 3 ? 0 : (s2 == 2 ? 4 : s2 + 1))) {   // 3 -> 0 -> 1 -> 2
        ch = vec_ok ? choose_direct(s2, c, ph, pw) : Choice{};
        if (!ch.ok) { ch = choose_staged(s2, c, ph, pw); if (ch.ok) g_rt = kShapes[s2].g; }
        else if (s2 != shape) g_rt = kShapes[s2].g;
        if (ch.ok) break;
    }
    if (!ch.ok) return hipErrorInvalidValue;
    const Shape& S = kShapes[ch.shape];

    ConvParams P;
    P.in = c.in; P.w = c.w; P.bias = c.bias; P.out = c.out;
    P.Hin = c.Hin; P.Win = c.Win; P.Cin = c.Cin; P.Hout = c.Hout; P.Wout = c.Wout; P.Cout = c.Cout;
    P.k = c.k; P.s = c.s; P.p = c.p; P.relu = c.relu;
    P.units = c.tiles; P.n_units = (int)n_units; P.rects = c.rects; P.ranges = c.ranges;
    P.units_x = units_x; P.units_y = units_y;
    P.ph = ph; P.pw = pw; P.npix_magic = magic_of(ph * pw); P.pw_magic = magic_of(pw);
    P.tg = ch.tg; P.pv = ch.pv; P.wv = ch.wv; P.g_rt = g_rt; P.p_instr = ch.p_instr; P.w_instr = ch.w_instr;
    P.chan_tail = (c.Cin % ch.kc) != 0; P.tap_tail = ((c.k * c.k) % ch.tg) != 0;
    P.patch_bytes = ch.patch_bytes; P.weight_bytes = ch.weight_bytes; P.dump_off = ch.dump_off;
    P.in_bytes = (uint32_t)((size_t)c.n_streams * c.Hin * c.Win * c.Cin * esz);
    P.w_bytes = (uint32_t)((size_t)c.Cout * c.k * c.k * c.Cin * esz);
    P.out_vec = (c.Cout % 4 == 0) && reinterpret_cast<uintptr_t>(c.out) % 16 == 0 &&
                (!c.bias || reinterpret_cast<uintptr_t>(c.bias) % 16 == 0);
    P.n_tapgroups = (c.k * c.k + ch.tg - 1) / ch.tg;
    P.n_chunks = (c.Cin + ch.kc - 1) / ch.kc;
    P.R = (c.Cout + S.nt - 1) / S.nt;
    KernelFn fn = kTable[ch.shape].fn[c.dtype == DC_BF16 ? 1 : 0][ch.kci];
    if (c.kernel_id) *c.kernel_id = ((c.dtype == DC_BF16 ? 1 : 0) * kNumShapes + ch.shape) * 4 + ch.kci;
    if (ch.lds > 64 * 1024) {
        hipError_t a = hipFuncSetAttribute(reinterpret_cast<const void*>(fn),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)ch.lds);
        if (a != hipSuccess) return a;
    }
    const long groups = (n_units + g_rt - 1) / g_rt;
    const long wgs = groups * P.R;
    if (wgs > 2147483647L) return hipErrorInvalidValue;
    hipLaunchKernelGGL(fn, dim3((unsigned)wgs), dim3(S.wm * S.wn * S.wk * 64), ch.lds, st, P);
    return hipGetLastError();
}

}  // namespace dc
