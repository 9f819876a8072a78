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
#include <algorithm>
#include <cstdio>
#include <cstdlib>

#include "dc_conv_common.h"

namespace dc {

namespace {


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
    const int kk = P.k * P.kx;

    int ug, ntile;
    decode_workgroup(P.R, ug, ntile);
    const int n0 = ntile * NT;
    const int n_units = unit_count(P);
    if (ug * P.g_rt >= n_units) return;     // the launch is sized for the longest possible list (whole workgroup, before any barrier)
    decode_units<G, NTHREADS>(P, H, ug, tid, n_units);

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
    const int Cin = keep_scalar(P.Cin), kdim = keep_scalar(P.kx), pwid = keep_scalar(P.pw), tgs = keep_scalar(P.tg);
    const int dil = keep_scalar(P.dil);
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
                const int trow = (ky * pwid + kx) * dil, c = g * 4 + q;
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
    const int kk = P.k * P.kx;

    int ug, ntile;
    decode_workgroup(P.R, ug, ntile);
    const int n0 = ntile * NT;
    const int n_units = unit_count(P);
    if (ug * P.g_rt >= n_units) return;     // the launch is sized for the longest possible list (whole workgroup, before any barrier)
    decode_units<G, NTHREADS>(P, H, ug, tid, n_units);

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
            const int ky = (tap0 + tl) / P.kx, kx = (tap0 + tl) - ky * P.kx;
            const int xoff = (ky * P.pw + kx) * P.dil * KCP + g * KG;
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

size_t reduce_bytes(const Shape& S) {
    return (size_t)(S.wk - 1) * S.wm * S.wn * (S.g / S.wm) * (S.nt / S.wn / 16) * 64 * 16;
}

// Direct kernel: pick the channel chunk KC and taps per stage TG.  With `f_tg` > 0 only that stage shape
// (chunk index f_kci, f_tg taps) is considered; otherwise the deepest stage (TG*KC useful K) whose two LDS
// buffers fit wins.
// kernel columns and taps of a launch (c.k rows; c.kw > 0: that many columns)
inline int tap_cols(const ConvLaunch& c) { return c.kw > 0 ? c.kw : c.k; }
inline int tap_count(const ConvLaunch& c) { return c.k * tap_cols(c); }

Choice choose_direct_from(int shape, const ConvLaunch& c, int ph, int pw, bool forced, int f_kci, int f_tg) {
    const Shape& S = kShapes[shape];
    const int nwaves = S.wm * S.wn * S.wk;
    const size_t esz = dtype_size(c.dtype);
    const int ve = (int)(16 / esz), kg = 4 * ve;
    const int kk = tap_count(c);
    Choice best{shape, 0, 0, 0, 0, 0, 0, 0, 0, 0, false, 0, 0};
    long best_score = -1;
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

// A deep stage hides the load latency of a workgroup that has its CU to itself.  Once a launch puts
// three workgroups on every two CUs or more, co-resident workgroups hide it for each other, and short
// stages with the narrowest channel chunk (less LDS per workgroup, hence more of them per CU) measure
// 15-25 % faster: one kernel row of taps per stage where at most two wavefronts share a stage's K, about a
// dozen taps where four do.  `wgs` is the number of workgroups the launch would have with this shape.
Choice choose_direct(int shape, const ConvLaunch& c, int ph, int pw, long wgs) {
    const int kk = tap_count(c);
    if (wgs >= 384 && kk > 1) {
        int tg = tap_cols(c) > 1 ? tap_cols(c) : c.k;      // one kernel row of taps (the column of a k x 1 kernel)
        if (kShapes[shape].wk > 2) { const int m = (kk + 12) / 13; tg = (kk + m - 1) / m; }
        Choice ch = choose_direct_from(shape, c, ph, pw, true, 0, tg);
        if (ch.ok) return ch;
    }
    return choose_direct_from(shape, c, ph, pw, false, -1, 0);
}

Choice choose_staged(int shape, const ConvLaunch& c, int ph, int pw) {
    const Shape& S = kShapes[shape];
    const int nth = S.wm * S.wn * S.wk * 64;
    const size_t esz = dtype_size(c.dtype);
    const int ve = (int)(16 / esz), kc = 4 * ve;
    const int kk = tap_count(c);
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

uint32_t magic_of(int d) { return (uint32_t)((0x100000000ull + (uint64_t)d - 1) / (uint64_t)d); }

}  // namespace

ConvTiling pick_tiling(const dc_layer&, int, int, int, int) { return ConvTiling{0, 4, 4, 64}; }

// Name of a kernel instantiation as a profiler prints it (without namespaces and arguments).
void conv_kernel_name(int id, char* buf, size_t n) {
    if (id >= 64) { conv_fast_kernel_name(id, buf, n); return; }
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
    const long n_hint = (c.tiles && c.n_tiles_dev && c.n_tiles_hint >= 0) ? std::max(1L, std::min(c.n_tiles_hint, n_units)) : n_units;
    const int kh = c.k, kw = tap_cols(c), dil = c.dil > 1 ? c.dil : 1;
    if (kh > kMaxK || kw > kMaxK) return hipErrorInvalidValue;
    // buffer loads address each tensor with 31-bit byte offsets
    if ((double)c.n_streams * c.Hin * c.Win * c.Cin * dtype_size(c.dtype) >= 2147483648.0 ||
        (double)c.Cout * kh * kw * c.Cin * dtype_size(c.dtype) >= 2147483648.0)
        return hipErrorInvalidValue;
    if (c.kw == 0 && dil == 1) {      // the kernels for the common shapes take square kernels without dilation
        hipError_t fe = hipSuccess;
        if (launch_conv_fast(c, n_units, n_hint, st, &fe)) return fe;
    }
    if (c.in_origin || c.out_origin) return hipErrorInvalidValue;      // only those kernels address a torus
    // Shape by the amount of work.  With enough units a workgroup takes g of them (up to 16) and 64
    // channels, g chosen so that the launch fills the 256 CUs in whole rounds; with few units the
    // smaller shapes split K among the wavefronts instead.
    int shape, g_rt;
    {
        constexpr int t1 = 160, xl_min = 8;
        const long r64 = (c.Cout + 63) / 64, r32 = (c.Cout + 31) / 32;
        const long rounds = (n_hint * r64 + 256 * 16 - 1) / (256 * 16);
        const long g = (n_hint * r64 + 256 * rounds - 1) / (256 * rounds);
        if (c.Cout > 32 && g >= xl_min) { shape = 3; g_rt = (int)(g > 16 ? 16 : g); }
        else if (c.Cout > 32 && ((n_hint + 3) / 4) * r64 >= 160) { shape = 0; g_rt = 4; }
        else if (((n_hint + 1) / 2) * r32 >= t1) { shape = 1; g_rt = 2; }
        else { shape = 2; g_rt = 1; }
    }
    // patch of a unit: its 4 x 4 outputs see 3 s + (kernel span) input rows and columns
    const int ph = 3 * c.s + (kh - 1) * dil + 1, pw = 3 * c.s + (kw - 1) * dil + 1;
    const size_t esz = dtype_size(c.dtype);
    const bool vec_ok = (c.Cin % (16 / esz)) == 0 && reinterpret_cast<uintptr_t>(c.in) % 16 == 0 &&
                        reinterpret_cast<uintptr_t>(c.w) % 16 == 0;
    // A smaller shape of the direct kernel (loads straight into LDS) beats any shape of the staged one (element
    // loads through registers): the staged kernel is only for channel counts that are not whole vectors, or for
    // patches that fit no direct shape (large strided kernels).
    Choice ch{};
    for (int pass = 0; pass < 2 && !ch.ok; ++pass)
        for (int s2 = shape; s2 < 4; s2 = (s2 == 3 ? 0 : (s2 == 2 ? 4 : s2 + 1))) {   // 3 -> 0 -> 1 -> 2
            if (pass == 0 && !vec_ok) break;
            const long g2 = s2 == shape ? g_rt : kShapes[s2].g;
            const long wgs2 = ((n_hint + g2 - 1) / g2) * ((c.Cout + kShapes[s2].nt - 1) / kShapes[s2].nt);
            ch = pass == 0 ? choose_direct(s2, c, ph, pw, wgs2) : choose_staged(s2, c, ph, pw);
            if (ch.ok && (s2 != shape || pass == 1)) g_rt = kShapes[s2].g;
            if (ch.ok) break;
        }
    if (!ch.ok) return hipErrorInvalidValue;
    const Shape& S = kShapes[ch.shape];

    ConvParams P;
    P.in = c.in; P.w = c.w; P.bias = c.bias; P.out = c.out;
    P.Hin = c.Hin; P.Win = c.Win; P.Cin = c.Cin; P.Hout = c.Hout; P.Wout = c.Wout; P.Cout = c.Cout;
    P.k = c.k; P.s = c.s; P.p = c.p; P.relu = c.relu;
    P.kx = kw; P.px = c.kw > 0 ? c.pw : c.p; P.dil = dil;
    P.units = c.tiles; P.n_units = (int)n_units; P.n_units_dev = c.tiles ? c.n_tiles_dev : nullptr; P.rects = c.rects; P.ranges = c.ranges;
    P.units_x = units_x; P.units_y = units_y;
    P.ph = ph; P.pw = pw; P.npix_magic = magic_of(ph * pw); P.pw_magic = magic_of(pw);
    P.tg = ch.tg; P.pv = ch.pv; P.wv = ch.wv; P.g_rt = g_rt; P.p_instr = ch.p_instr; P.w_instr = ch.w_instr;
    P.chan_tail = (c.Cin % ch.kc) != 0; P.tap_tail = ((kh * kw) % ch.tg) != 0;
    P.patch_bytes = ch.patch_bytes; P.weight_bytes = ch.weight_bytes; P.dump_off = ch.dump_off;
    P.in_bytes = (uint32_t)((size_t)c.n_streams * c.Hin * c.Win * c.Cin * esz);
    P.w_bytes = (uint32_t)((size_t)c.Cout * kh * kw * c.Cin * esz);
    P.out_vec = (c.Cout % 4 == 0) && reinterpret_cast<uintptr_t>(c.out) % 16 == 0 &&
                (!c.bias || reinterpret_cast<uintptr_t>(c.bias) % 16 == 0);
    P.ks = 1; P.chunks_per_split = 0; P.partial = nullptr;
    P.n_tapgroups = (kh * kw + ch.tg - 1) / ch.tg;
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
