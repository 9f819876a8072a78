// HBM-bound kernels: the shifted copy that serves reusable pixels from the previous
// frame's cached feature map (Section 5 "Reuse", step 1) and the layers that are never
// cached (Section 5: pooling, add, the input conversion; the layer types of Table 2 other
// than convolution: LRN, concat, fully-connected, softmax).  All channels-last, 16-byte
// vector accesses whenever the channel run allows it.
#include <hip/hip_bf16.h>

#include "dc_internal.h"

namespace dc {

namespace {

constexpr int kThreads = 256;

// out[s][y][x][:] = prev[s][y+dy][x+dx][:] for every pixel of every rectangle.
// grid.y = rectangle, grid.x = chunks of the rectangle's vectors (grid-stride).
template <typename V>
__global__ __launch_bounds__(kThreads) void shifted_copy_kernel(const RectDev* __restrict__ rects,
                                                                const V* __restrict__ prev,
                                                                V* __restrict__ out, int Hout, int Wout,
                                                                int pv /* vectors per pixel */) {
    const RectDev r = rects[blockIdx.y];
    const int row_v = r.w * pv;
    const int total = r.h * row_v;
    const size_t map = (size_t)r.stream * Hout * Wout;
    for (int i = blockIdx.x * kThreads + threadIdx.x; i < total; i += gridDim.x * kThreads) {
        int row = i / row_v, col = i - row * row_v;
        size_t dst = (map + (size_t)(r.y + row) * Wout + r.x) * pv + col;
        size_t src = (map + (size_t)(r.y + r.dy + row) * Wout + (r.x + r.dx)) * pv + col;
        out[dst] = prev[src];
    }
}

// The same for the rectangles of every conv layer of a frame in one launch: the copies only depend
// on the previous frame's maps, so they can all run before the first layer.
__global__ __launch_bounds__(kThreads) void shifted_copy_all_kernel(const RectDev* __restrict__ rects,
                                                                    const CopyLayerDev* __restrict__ layers) {
    const RectDev r = rects[blockIdx.y];
    const CopyLayerDev L = layers[r.pad];
    const uint4* __restrict__ prev = static_cast<const uint4*>(L.prev);
    uint4* __restrict__ out = static_cast<uint4*>(L.out);
    const int row_v = r.w * L.pv;
    const int total = r.h * row_v;
    const size_t map = (size_t)r.stream * L.Hout * L.Wout;
    for (int i = blockIdx.x * kThreads + threadIdx.x; i < total; i += gridDim.x * kThreads) {
        int row = i / row_v, col = i - row * row_v;
        size_t dst = (map + (size_t)(r.y + row) * L.Wout + r.x) * L.pv + col;
        size_t src = (map + (size_t)(r.y + r.dy + row) * L.Wout + (r.x + r.dx)) * L.pv + col;
        out[dst] = prev[src];
    }
}

template <typename T>
__device__ __forceinline__ T from_float(float v);
template <>
__device__ __forceinline__ float from_float<float>(float v) { return v; }
template <>
__device__ __forceinline__ __hip_bfloat16 from_float<__hip_bfloat16>(float v) { return __float2bfloat16(v); }
__device__ __forceinline__ float to_float(float v) { return v; }
__device__ __forceinline__ float to_float(__hip_bfloat16 v) { return __bfloat162float(v); }

// out[pixel][c] = (frame[pixel][c] - 128) / 128 for c < cf, 0 for the padding channels cf <= c < ct
template <typename T>
__global__ __launch_bounds__(kThreads) void frame_to_tensor_kernel(const uint8_t* __restrict__ f,
                                                                   T* __restrict__ out, size_t n_out, int cf, int ct) {
    size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * kThreads;
    for (; i < n_out; i += stride) {
        const size_t px = i / ct;
        const int c = (int)(i - px * ct);
        out[i] = from_float<T>(c < cf ? (float)((int)f[px * cf + c] - 128) * (1.0f / 128.0f) : 0.f);
    }
}

// Max or average pooling (mean over the in-bounds part of the window) for channel counts that are not whole 16-byte
// vectors: one thread per (output pixel, channel); consecutive threads walk the channels.
template <typename T, bool AVG>
__global__ __launch_bounds__(kThreads) void pool_kernel(const T* __restrict__ in, T* __restrict__ out,
                                                        int n_streams, int Hin, int Win, int C, int Hout,
                                                        int Wout, int k, int s, int p) {
    const size_t total = (size_t)n_streams * Hout * Wout * C;
    size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * kThreads;
    for (; i < total; i += stride) {
        int c = (int)(i % C);
        size_t pix = i / C;
        int x = (int)(pix % Wout);
        size_t t = pix / Wout;
        int y = (int)(t % Hout);
        int st = (int)(t / Hout);
        float acc = AVG ? 0.f : -INFINITY;
        int cnt = 0;
        for (int ky = 0; ky < k; ++ky) {
            int iy = y * s - p + ky;
            if (iy < 0 || iy >= Hin) continue;
            for (int kx = 0; kx < k; ++kx) {
                int ix = x * s - p + kx;
                if (ix < 0 || ix >= Win) continue;
                float v = to_float(in[(((size_t)st * Hin + iy) * Win + ix) * C + c]);
                acc = AVG ? acc + v : (v > acc ? v : acc);
                ++cnt;
            }
        }
        out[i] = from_float<T>(AVG ? (cnt ? acc / (float)cnt : 0.f) : acc);
    }
}

template <typename T>
__global__ __launch_bounds__(kThreads) void add_kernel(const T* __restrict__ a, const T* __restrict__ b,
                                                       T* __restrict__ out, size_t n, int relu) {
    size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * kThreads;
    for (; i < n; i += stride) {
        float v = to_float(a[i]) + (b ? to_float(b[i]) : 0.f);  // b == nullptr: plain ReLU layer
        if (relu) v = v > 0.f ? v : 0.f;
        out[i] = from_float<T>(v);
    }
}

// Local response normalisation, out = in / (kappa + alpha_n * S)^beta with S the sum of squares over the window
// (zeros outside the tensor) and alpha_n = alpha / window elements: `size` channels around the element's channel
// at the same pixel, or size x size pixels around the element in its channel.  One thread per element; the
// neighbours are re-read through the vector cache.
template <typename T>
__global__ __launch_bounds__(kThreads) void lrn_kernel(const T* __restrict__ in, T* __restrict__ out, int n_streams,
                                                       int H, int W, int C, int r, int within, float alpha_n,
                                                       float beta, float kappa) {
    const size_t total = (size_t)n_streams * H * W * C;
    size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * kThreads;
    for (; i < total; i += stride) {
        const int c = (int)(i % C);
        float S = 0.f;
        if (within) {
            const size_t pix = i / C;
            const int x = (int)(pix % W);
            const size_t t = pix / W;
            const int y = (int)(t % H);
            const size_t map = (t / H) * H;
            for (int yy = y - r; yy <= y + r; ++yy) {
                if (yy < 0 || yy >= H) continue;
                for (int xx = x - r; xx <= x + r; ++xx) {
                    if (xx < 0 || xx >= W) continue;
                    const float v = to_float(in[((map + yy) * W + xx) * C + c]);
                    S += v * v;
                }
            }
        } else {
            const size_t base = i - c;
            const int c0 = c - r < 0 ? 0 : c - r, c1 = c + r >= C ? C - 1 : c + r;
            for (int cc = c0; cc <= c1; ++cc) {
                const float v = to_float(in[base + cc]);
                S += v * v;
            }
        }
        out[i] = from_float<T>(to_float(in[i]) * powf(kappa + alpha_n * S, -beta));
    }
}

__device__ __forceinline__ float wave_sum_f32(float v) {
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, 64);
    return v;
}
__device__ __forceinline__ float wave_max_f32(float v) {
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) v = fmaxf(v, __shfl_xor(v, m, 64));
    return v;
}

// Softmax over the channels of a pixel; one wavefront per pixel, the largest element subtracted first.  Up to 1024
// channels are read once and kept in registers (a pixel of a classifier's output is read from cold memory, and each
// pass over it would pay that latency again).
template <typename T>
__global__ __launch_bounds__(kThreads) void softmax_kernel(const T* __restrict__ in, T* __restrict__ out, size_t n_pixels,
                                                           int C) {
    const int lane = threadIdx.x & 63;
    const size_t px = (size_t)blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6);
    if (px >= n_pixels) return;                   // whole wavefronts leave
    const T* v = in + px * C;
    if (C <= 1024) {
        float r[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) r[i] = lane + 64 * i < C ? to_float(v[lane + 64 * i]) : -INFINITY;
        float m = r[0];
#pragma unroll
        for (int i = 1; i < 16; ++i) m = fmaxf(m, r[i]);
        m = wave_max_f32(m);
        float sum = 0.f;
#pragma unroll
        for (int i = 0; i < 16; ++i) { r[i] = expf(r[i] - m); sum += r[i]; }    // exp(-inf) = 0 for the padding
        sum = wave_sum_f32(sum);
        const float inv = 1.0f / sum;
#pragma unroll
        for (int i = 0; i < 16; ++i)
            if (lane + 64 * i < C) out[px * C + lane + 64 * i] = from_float<T>(r[i] * inv);
        return;
    }
    float m = -INFINITY;
    for (int c = lane; c < C; c += 64) m = fmaxf(m, to_float(v[c]));
    m = wave_max_f32(m);
    float sum = 0.f;
    for (int c = lane; c < C; c += 64) sum += expf(to_float(v[c]) - m);
    sum = wave_sum_f32(sum);
    const float inv = 1.0f / sum;
    for (int c = lane; c < C; c += 64) out[px * C + c] = from_float<T>(expf(to_float(v[c]) - m) * inv);
}

// Fully-connected layer: out[s][o] = bias[o] + sum_i w[o][i] x[s][i].  The weights are the large operand (each is
// used once per stream), so a wavefront takes one output neuron, streams its weight row once and multiplies it with
// the inputs of NS streams, which come from the caches; per-lane partial sums are added across the wavefront at the
// end.  VE elements per load: a 16-byte vector, or 1 when K or an address is not a multiple of that.
template <typename T, int VE>
__device__ __forceinline__ void fc_load(const T* p, float (&f)[VE]) {
    if constexpr (VE == 1) {
        f[0] = to_float(*p);
    } else if constexpr (sizeof(T) == 4) {
        const float4 v = *reinterpret_cast<const float4*>(p);
        f[0] = v.x; f[1] = v.y; f[2] = v.z; f[3] = v.w;
    } else {                                      // eight bf16: the value is the upper half of the fp32 pattern
        const uint4 v = *reinterpret_cast<const uint4*>(p);
        const uint32_t u[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            f[2 * e] = __uint_as_float(u[e] << 16);
            f[2 * e + 1] = __uint_as_float(u[e] & 0xffff0000u);
        }
    }
}
template <typename T, int NS, int VE, int NO>
__global__ __launch_bounds__(kThreads) void fc_kernel(const T* __restrict__ x, const T* __restrict__ w,
                                                      const float* __restrict__ bias, T* __restrict__ out, int n_streams,
                                                      size_t K, int cout, int relu) {
    // NO output neurons per wavefront: with many streams the inputs (read again for every neuron) are the larger
    // traffic, and one input vector then serves NO weight rows.
    const int lane = threadIdx.x & 63;
    const int o0 = (blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6)) * NO;
    const int s0 = blockIdx.y * NS;
    if (o0 >= cout) return;                       // whole wavefronts leave
    float acc[NO][NS];
#pragma unroll
    for (int j = 0; j < NO; ++j)
#pragma unroll
        for (int s = 0; s < NS; ++s) acc[j][s] = 0.f;
    for (size_t k = (size_t)lane * VE; k < K; k += 64 * VE) {
        float wf[NO][VE];
#pragma unroll
        for (int j = 0; j < NO; ++j) {
            const int o = o0 + j < cout ? o0 + j : cout - 1;      // a row past the end repeats the last one (not stored)
            fc_load<T, VE>(w + (size_t)o * K + k, wf[j]);
        }
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            if (s0 + s < n_streams) {             // uniform over the wavefront
                float xf[VE];
                fc_load<T, VE>(x + (size_t)(s0 + s) * K + k, xf);
#pragma unroll
                for (int j = 0; j < NO; ++j)
#pragma unroll
                    for (int e = 0; e < VE; ++e) acc[j][s] = fmaf(wf[j][e], xf[e], acc[j][s]);
            }
        }
    }
#pragma unroll
    for (int j = 0; j < NO; ++j) {
        if (o0 + j >= cout) break;                // uniform
        const float b = bias ? bias[o0 + j] : 0.f;
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            float v = wave_sum_f32(acc[j][s]) + b;
            if (relu) v = v > 0.f ? v : 0.f;
            if (lane == 0 && s0 + s < n_streams) out[(size_t)(s0 + s) * cout + o0 + j] = from_float<T>(v);
        }
    }
}

// ---- 16-byte vector forms: one thread per (pixel, vector of 4 fp32 / 8 bf16 channels) --------------------------
template <typename T>
struct Vec16 {
    static constexpr int VE = 16 / sizeof(T);
    static __device__ __forceinline__ void load(const uint4* p, float (&f)[VE]) {
        const uint4 v = *p;
        const uint32_t u[4] = {v.x, v.y, v.z, v.w};
        if constexpr (sizeof(T) == 4) {
#pragma unroll
            for (int e = 0; e < 4; ++e) f[e] = __uint_as_float(u[e]);
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                f[2 * e] = __uint_as_float(u[e] << 16);
                f[2 * e + 1] = __uint_as_float(u[e] & 0xffff0000u);
            }
        }
    }
    static __device__ __forceinline__ void store(uint4* p, const float (&f)[VE]) {
        uint32_t u[4];
        if constexpr (sizeof(T) == 4) {
#pragma unroll
            for (int e = 0; e < 4; ++e) u[e] = __float_as_uint(f[e]);
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const __hip_bfloat16 lo = __float2bfloat16(f[2 * e]), hi = __float2bfloat16(f[2 * e + 1]);
                u[e] = (uint32_t)__builtin_bit_cast(uint16_t, lo) | ((uint32_t)__builtin_bit_cast(uint16_t, hi) << 16);
            }
        }
        *p = uint4{u[0], u[1], u[2], u[3]};
    }
};

// Max or average pooling, CV vectors per pixel.
template <typename T, bool AVG>
__global__ __launch_bounds__(kThreads) void pool_vec_kernel(const uint4* __restrict__ in, uint4* __restrict__ out,
                                                            int n_streams, int Hin, int Win, int CV, int Hout, int Wout,
                                                            int k, int s, int p) {
    constexpr int VE = Vec16<T>::VE;
    const size_t total = (size_t)n_streams * Hout * Wout * CV;
    size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * kThreads;
    for (; i < total; i += stride) {
        const int cv = (int)(i % CV);
        const size_t pix = i / CV;
        const int x = (int)(pix % Wout);
        const size_t t = pix / Wout;
        const int y = (int)(t % Hout);
        const size_t map = (t / Hout) * Hin;
        float acc[VE];
#pragma unroll
        for (int e = 0; e < VE; ++e) acc[e] = AVG ? 0.f : -INFINITY;
        const int y0 = max(y * s - p, 0), y1 = min(y * s - p + k, Hin), x0 = max(x * s - p, 0), x1 = min(x * s - p + k, Win);
        for (int iy = y0; iy < y1; ++iy)
            for (int ix = x0; ix < x1; ++ix) {
                float f[VE];
                Vec16<T>::load(in + ((map + iy) * Win + ix) * CV + cv, f);
#pragma unroll
                for (int e = 0; e < VE; ++e) acc[e] = AVG ? acc[e] + f[e] : fmaxf(acc[e], f[e]);
            }
        if (AVG) {
            const int cnt = (y1 - y0) * (x1 - x0);
#pragma unroll
            for (int e = 0; e < VE; ++e) acc[e] = cnt > 0 ? acc[e] / (float)cnt : 0.f;
        }
        Vec16<T>::store(out + i, acc);
    }
}

// The pooling of the VGG- and Darknet-style stacks, 2x2 windows with stride 2 and no padding: every window lies
// inside the map, so a thread's four loads have fixed offsets and go out together (two outputs per thread: eight
// loads in flight).  grid.y = (stream, output row), grid.x covers the Wout * CV vectors of the row.
template <typename T>
__global__ __launch_bounds__(kThreads) void maxpool2x2_vec_kernel(const uint4* __restrict__ in, uint4* __restrict__ out,
                                                                  int Hin, int Win, int CV, int Hout, int Wout) {
    constexpr int VE = Vec16<T>::VE;
    const int row = blockIdx.y;                     // stream * Hout + y
    const int stream = row / Hout, y = row - stream * Hout;
    const int row_vecs = Wout * CV;
    const uint4* __restrict__ r0 = in + ((size_t)stream * Hin + 2 * y) * Win * CV;
    const uint4* __restrict__ r1 = r0 + (size_t)Win * CV;
    uint4* __restrict__ o = out + (size_t)row * row_vecs;
    const int j0 = (int)blockIdx.x * (2 * kThreads) + (int)threadIdx.x, j1 = j0 + kThreads;
    float a[2][4][VE];
    bool on[2];
#pragma unroll
    for (int q = 0; q < 2; ++q) {
        const int j = q ? j1 : j0;
        on[q] = j < row_vecs;
        const int x = on[q] ? j / CV : 0, cv = on[q] ? j - x * CV : 0;
        const int at = 2 * x * CV + cv;
        Vec16<T>::load(r0 + at, a[q][0]);
        Vec16<T>::load(r0 + at + CV, a[q][1]);
        Vec16<T>::load(r1 + at, a[q][2]);
        Vec16<T>::load(r1 + at + CV, a[q][3]);
    }
#pragma unroll
    for (int q = 0; q < 2; ++q) {
        if (!on[q]) continue;
        float m[VE];
#pragma unroll
        for (int e = 0; e < VE; ++e) m[e] = fmaxf(fmaxf(a[q][0][e], a[q][1][e]), fmaxf(a[q][2][e], a[q][3][e]));
        Vec16<T>::store(o + (q ? j1 : j0), m);
    }
}

// The same pooling of a conv output that lies on a torus: pixel (x, y) of stream s is stored at
// ((x + ox) mod Win, (y + oy) mod Hin) with (ox, oy) = origin[s * origin_stride + 0 / 1]; the output has an origin of
// its own or none.  CACHED: the output is a cache value as well, and a pixel whose bit is set in its reuse bitmap
// keeps what the buffer holds (the previous frame's value, which the moved origin has put in its place).
template <typename T, bool CACHED>
__global__ __launch_bounds__(kThreads) void maxpool2x2_torus_kernel(const uint4* __restrict__ in, uint4* __restrict__ out,
                                                                    int Hin, int Win, int CV, int Hout, int Wout,
                                                                    const int32_t* __restrict__ origin,
                                                                    const int32_t* __restrict__ out_origin, int origin_stride,
                                                                    CachedMap M) {
    constexpr int VE = Vec16<T>::VE;
    const int row = blockIdx.y;                     // stream * Hout + y
    const int stream = row / Hout, y = row - stream * Hout;
    const int ox = origin[(size_t)stream * origin_stride], oy = origin[(size_t)stream * origin_stride + 1];
    const int j = (int)blockIdx.x * kThreads + (int)threadIdx.x;
    if (j >= Wout * CV) return;
    const int x = j / CV, cv = j - x * CV;
    if (CACHED) {
        const uint32_t* bits = M.bitmaps + (size_t)stream * M.bm_words + M.bm_off + (size_t)y * ((Wout + 31) >> 5);
        if ((bits[x >> 5] >> (x & 31)) & 1u) return;
    }
    const uint4* __restrict__ base = in + (size_t)stream * Hin * Win * CV + cv;
    const size_t r0 = (size_t)torus_wrap(2 * y, oy, Hin) * Win, r1 = (size_t)torus_wrap(2 * y + 1, oy, Hin) * Win;
    const int c0 = torus_wrap(2 * x, ox, Win), c1 = torus_wrap(2 * x + 1, ox, Win);
    float a[4][VE], m[VE];
    Vec16<T>::load(base + (r0 + c0) * CV, a[0]);
    Vec16<T>::load(base + (r0 + c1) * CV, a[1]);
    Vec16<T>::load(base + (r1 + c0) * CV, a[2]);
    Vec16<T>::load(base + (r1 + c1) * CV, a[3]);
#pragma unroll
    for (int e = 0; e < VE; ++e) m[e] = fmaxf(fmaxf(a[0][e], a[1][e]), fmaxf(a[2][e], a[3][e]));
    size_t at = (size_t)row * Wout * CV + j;
    if (out_origin) {
        const int xo = torus_wrap(x, out_origin[(size_t)stream * origin_stride], Wout);
        const int yo = torus_wrap(y, out_origin[(size_t)stream * origin_stride + 1], Hout);
        at = (((size_t)stream * Hout + yo) * Wout + xo) * CV + cv;
    }
    Vec16<T>::store(out + at, m);
}

// Max-pooling and add with the cache: grid.y = (stream, output row), a thread takes one 16-byte vector of one pixel;
// a pixel whose bit is set in the tensor's reuse bitmap receives the previous frame's output at the tensor's offset.
template <typename T>
__global__ __launch_bounds__(kThreads) void maxpool_cached_kernel(const uint4* __restrict__ in, const uint4* __restrict__ prev,
                                                                  uint4* __restrict__ out, int Hin, int Win, int CV, int Hout,
                                                                  int Wout, int k, int s, int p, CachedMap M) {
    constexpr int VE = Vec16<T>::VE;
    const int row = blockIdx.y, stream = row / Hout, y = row - stream * Hout;
    const int j = (int)blockIdx.x * kThreads + (int)threadIdx.x;
    if (j >= Wout * CV) return;
    const int x = j / CV, cv = j - x * CV;
    const uint32_t* bits = M.bitmaps + (size_t)stream * M.bm_words + M.bm_off + (size_t)y * ((Wout + 31) >> 5);
    uint4* o = out + (size_t)row * Wout * CV + j;
    if ((bits[x >> 5] >> (x & 31)) & 1u) {
        const size_t at = ((size_t)stream * M.n_tensors + M.tensor) * 2;
        const int dx = M.dxy[at], dy = M.dxy[at + 1];
        *o = prev[(((size_t)stream * Hout + (y + dy)) * Wout + (x + dx)) * CV + cv];
        return;
    }
    float acc[VE];
#pragma unroll
    for (int e = 0; e < VE; ++e) acc[e] = -INFINITY;
    const int y0 = max(y * s - p, 0), y1 = min(y * s - p + k, Hin), x0 = max(x * s - p, 0), x1 = min(x * s - p + k, Win);
    for (int iy = y0; iy < y1; ++iy)
        for (int ix = x0; ix < x1; ++ix) {
            float f[VE];
            Vec16<T>::load(in + (((size_t)stream * Hin + iy) * Win + ix) * CV + cv, f);
#pragma unroll
            for (int e = 0; e < VE; ++e) acc[e] = fmaxf(acc[e], f[e]);
        }
    Vec16<T>::store(o, acc);
}

template <typename T>
__global__ __launch_bounds__(kThreads) void add_cached_kernel(const uint4* __restrict__ a, const uint4* __restrict__ b,
                                                              const uint4* __restrict__ prev, uint4* __restrict__ out, int H, int W,
                                                              int CV, int relu, CachedMap M) {
    constexpr int VE = Vec16<T>::VE;
    const int row = blockIdx.y, stream = row / H, y = row - stream * H;
    const int j = (int)blockIdx.x * kThreads + (int)threadIdx.x;
    if (j >= W * CV) return;
    const int x = j / CV, cv = j - x * CV;
    const uint32_t* bits = M.bitmaps + (size_t)stream * M.bm_words + M.bm_off + (size_t)y * ((W + 31) >> 5);
    const size_t i = (size_t)row * W * CV + j;
    if ((bits[x >> 5] >> (x & 31)) & 1u) {
        const size_t at = ((size_t)stream * M.n_tensors + M.tensor) * 2;
        const int dx = M.dxy[at], dy = M.dxy[at + 1];
        out[i] = prev[(((size_t)stream * H + (y + dy)) * W + (x + dx)) * CV + cv];
        return;
    }
    float u[VE], v[VE];
    Vec16<T>::load(a + i, u);
    Vec16<T>::load(b + i, v);
#pragma unroll
    for (int e = 0; e < VE; ++e) { u[e] += v[e]; if (relu) u[e] = u[e] > 0.f ? u[e] : 0.f; }
    Vec16<T>::store(out + i, u);
}

// out = a + b (b == nullptr: out = a), optional ReLU, 16 bytes per thread.
template <typename T>
__global__ __launch_bounds__(kThreads) void add_vec_kernel(const uint4* __restrict__ a, const uint4* __restrict__ b,
                                                           uint4* __restrict__ out, size_t n_vec, int relu) {
    constexpr int VE = Vec16<T>::VE;
    size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * kThreads;
    for (; i < n_vec; i += stride) {
        float x[VE], y[VE];
        Vec16<T>::load(a + i, x);
        if (b) {
            Vec16<T>::load(b + i, y);
#pragma unroll
            for (int e = 0; e < VE; ++e) x[e] += y[e];
        }
        if (relu) {
#pragma unroll
            for (int e = 0; e < VE; ++e) x[e] = x[e] > 0.f ? x[e] : 0.f;
        }
        Vec16<T>::store(out + i, x);
    }
}

// The input conversion for a tensor pixel of exactly 16 bytes (the padded first layer): one thread per pixel.
template <typename T>
__global__ __launch_bounds__(kThreads) void frame_to_tensor_px_kernel(const uint8_t* __restrict__ f, uint4* __restrict__ out,
                                                                      size_t n_pixels, int cf) {
    constexpr int VE = Vec16<T>::VE;
    size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * kThreads;
    for (; i < n_pixels; i += stride) {
        float v[VE];
#pragma unroll
        for (int e = 0; e < VE; ++e) v[e] = e < cf ? (float)((int)f[i * cf + e] - 128) * (1.0f / 128.0f) : 0.f;
        Vec16<T>::store(out + i, v);
    }
}

// LRN over channels with radius R <= VE: the thread's vector and its two neighbours hold every channel of the window.
template <typename T, int R>
__global__ __launch_bounds__(kThreads) void lrn_vec_kernel(const uint4* __restrict__ in, uint4* __restrict__ out,
                                                           size_t n_pixels, int CV, float alpha_n, float beta, float kappa) {
    constexpr int VE = Vec16<T>::VE;
    static_assert(R <= VE, "window inside the neighbouring vectors");
    const size_t total = n_pixels * CV;
    size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * kThreads;
    for (; i < total; i += stride) {
        const int cv = (int)(i % CV);
        float f[3][VE];
        Vec16<T>::load(in + i, f[1]);
        if (cv > 0) Vec16<T>::load(in + i - 1, f[0]);
        if (cv + 1 < CV) Vec16<T>::load(in + i + 1, f[2]);
        float sq[3 * VE];
#pragma unroll
        for (int e = 0; e < VE; ++e) {
            sq[e] = cv > 0 ? f[0][e] * f[0][e] : 0.f;
            sq[VE + e] = f[1][e] * f[1][e];
            sq[2 * VE + e] = cv + 1 < CV ? f[2][e] * f[2][e] : 0.f;
        }
        float o[VE];
#pragma unroll
        for (int e = 0; e < VE; ++e) {
            float S = 0.f;
#pragma unroll
            for (int d = -R; d <= R; ++d) S += sq[VE + e + d];
            o[e] = f[1][e] * __powf(kappa + alpha_n * S, -beta);
        }
        Vec16<T>::store(out + i, o);
    }
}

// All inputs of a concatenation in one launch: a thread moves one unit of V of the output and finds the input it
// comes from by its channel offset.
struct ConcatArgs {
    const void* in[4];
    int c[4], off[4];     // channel count and first output channel of each input, in units of V
    int n, ctot;
};
template <typename V>
__global__ __launch_bounds__(kThreads) void concat_all_kernel(ConcatArgs a, V* __restrict__ out, size_t n_pixels) {
    const size_t total = n_pixels * a.ctot;
    size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * kThreads;
    for (; i < total; i += stride) {
        const size_t px = i / a.ctot;
        const int c = (int)(i - px * a.ctot);
        int j = 0;
        if (a.n > 1 && c >= a.off[1]) j = 1;
        if (a.n > 2 && c >= a.off[2]) j = 2;
        if (a.n > 3 && c >= a.off[3]) j = 3;
        out[i] = static_cast<const V*>(a.in[j])[px * a.c[j] + (c - a.off[j])];
    }
}

inline int grid_for(size_t n, int cap = 256 * 16) {
    size_t g = (n + kThreads - 1) / kThreads;
    return (int)(g < 1 ? 1 : (g > (size_t)cap ? cap : g));
}

}  // namespace

hipError_t launch_shifted_copy(const RectDev* rects_dev, int n_rects, int max_rect_w, int max_rect_h,
                               const void* prev, void* out, int Hout, int Wout, int Cout, int dtype,
                               hipStream_t st) {
    if (n_rects <= 0) return hipSuccess;
    const size_t px_bytes = (size_t)Cout * dtype_size(dtype);
    const bool aligned16 = (reinterpret_cast<uintptr_t>(prev) % 16 == 0) && (reinterpret_cast<uintptr_t>(out) % 16 == 0);
    // at most 65535 rectangles per launch in grid.y
    for (int r0 = 0; r0 < n_rects; r0 += 65535) {
        int nr = n_rects - r0 < 65535 ? n_rects - r0 : 65535;
        if (px_bytes % 16 == 0 && aligned16) {
            int pv = (int)(px_bytes / 16);
            size_t vec = (size_t)max_rect_w * max_rect_h * pv;
            dim3 grid(grid_for((vec + 3) / 4, 1024), nr);
            hipLaunchKernelGGL(shifted_copy_kernel<uint4>, grid, dim3(kThreads), 0, st, rects_dev + r0,
                               (const uint4*)prev, (uint4*)out, Hout, Wout, pv);
        } else if (dtype == DC_F32) {
            size_t vec = (size_t)max_rect_w * max_rect_h * Cout;
            dim3 grid(grid_for((vec + 3) / 4, 1024), nr);
            hipLaunchKernelGGL(shifted_copy_kernel<uint32_t>, grid, dim3(kThreads), 0, st, rects_dev + r0,
                               (const uint32_t*)prev, (uint32_t*)out, Hout, Wout, Cout);
        } else {
            size_t vec = (size_t)max_rect_w * max_rect_h * Cout;
            dim3 grid(grid_for((vec + 3) / 4, 1024), nr);
            hipLaunchKernelGGL(shifted_copy_kernel<uint16_t>, grid, dim3(kThreads), 0, st, rects_dev + r0,
                               (const uint16_t*)prev, (uint16_t*)out, Hout, Wout, Cout);
        }
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

hipError_t launch_shifted_copy_all(const RectDev* rects_dev, int n_rects, const CopyLayerDev* layers_dev,
                                   size_t max_vec_per_rect, hipStream_t st) {
    for (int r0 = 0; r0 < n_rects; r0 += 65535) {
        const int nr = n_rects - r0 < 65535 ? n_rects - r0 : 65535;
        dim3 grid(grid_for((max_vec_per_rect + 3) / 4, 1024), nr);
        hipLaunchKernelGGL(shifted_copy_all_kernel, grid, dim3(kThreads), 0, st, rects_dev + r0, layers_dev);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

// A tensor that lies on a torus, written out from its origin: out[s][y][x] = in[s][(y + oy) mod H][(x + ox) mod W].
// A thread moves one vector of V bytes; grid.y = (stream, row).
template <typename V>
__global__ __launch_bounds__(kThreads) void torus_read_kernel(const V* __restrict__ in, V* __restrict__ out, int H, int W, int PV,
                                                              const int32_t* __restrict__ origin, int origin_stride) {
    const int row = blockIdx.y, stream = row / H, y = row - stream * H;
    const int j = (int)blockIdx.x * kThreads + (int)threadIdx.x;
    if (j >= W * PV) return;
    const int x = j / PV, v = j - x * PV;
    const int ox = origin ? origin[(size_t)stream * origin_stride] : 0, oy = origin ? origin[(size_t)stream * origin_stride + 1] : 0;
    out[(size_t)row * W * PV + j] = in[(((size_t)stream * H + torus_wrap(y, oy, H)) * W + torus_wrap(x, ox, W)) * PV + v];
}

hipError_t launch_torus_read(const void* in, void* out, int n_streams, int H, int W, size_t pixel_bytes,
                             const int32_t* origin, int origin_stride, hipStream_t st) {
    if ((size_t)n_streams * H > 65535) return hipErrorInvalidValue;
    const bool v16 = pixel_bytes % 16 == 0 && reinterpret_cast<uintptr_t>(in) % 16 == 0 && reinterpret_cast<uintptr_t>(out) % 16 == 0;
    const bool v4 = pixel_bytes % 4 == 0 && reinterpret_cast<uintptr_t>(in) % 4 == 0 && reinterpret_cast<uintptr_t>(out) % 4 == 0;
    const int vb = v16 ? 16 : (v4 ? 4 : 1);
    const int pv = (int)(pixel_bytes / vb);
    const dim3 grid((unsigned)(((size_t)W * pv + kThreads - 1) / kThreads), (unsigned)(n_streams * H));
    if (v16)
        hipLaunchKernelGGL(torus_read_kernel<uint4>, grid, dim3(kThreads), 0, st, (const uint4*)in, (uint4*)out, H, W, pv, origin, origin_stride);
    else if (v4)
        hipLaunchKernelGGL(torus_read_kernel<uint32_t>, grid, dim3(kThreads), 0, st, (const uint32_t*)in, (uint32_t*)out, H, W, pv, origin, origin_stride);
    else
        hipLaunchKernelGGL(torus_read_kernel<uint8_t>, grid, dim3(kThreads), 0, st, (const uint8_t*)in, (uint8_t*)out, H, W, pv, origin, origin_stride);
    return hipGetLastError();
}

hipError_t launch_frame_to_tensor(const uint8_t* f, void* out, size_t n_pixels, int cf, int ct, int dtype,
                                  hipStream_t st) {
    const size_t n = n_pixels * ct;
    if (n == 0) return hipSuccess;
    if (ct * dtype_size(dtype) == 16 && reinterpret_cast<uintptr_t>(out) % 16 == 0) {
        if (dtype == DC_BF16)
            hipLaunchKernelGGL(frame_to_tensor_px_kernel<__hip_bfloat16>, dim3(grid_for(n_pixels)), dim3(kThreads), 0, st, f,
                               (uint4*)out, n_pixels, cf);
        else
            hipLaunchKernelGGL(frame_to_tensor_px_kernel<float>, dim3(grid_for(n_pixels)), dim3(kThreads), 0, st, f,
                               (uint4*)out, n_pixels, cf);
        return hipGetLastError();
    }
    if (dtype == DC_BF16)
        hipLaunchKernelGGL(frame_to_tensor_kernel<__hip_bfloat16>, dim3(grid_for(n)), dim3(kThreads), 0, st, f,
                           (__hip_bfloat16*)out, n, cf, ct);
    else
        hipLaunchKernelGGL(frame_to_tensor_kernel<float>, dim3(grid_for(n)), dim3(kThreads), 0, st, f,
                           (float*)out, n, cf, ct);
    return hipGetLastError();
}

namespace {
template <bool AVG>
hipError_t launch_pool(const void* in, void* out, int n_streams, int Hin, int Win, int C, int k, int s, int p, int dtype,
                       hipStream_t st) {
    const int Hout = (Hin + 2 * p - k) / s + 1, Wout = (Win + 2 * p - k) / s + 1;
    const size_t n = (size_t)n_streams * Hout * Wout * C;
    if (n == 0) return hipSuccess;
    if ((C * dtype_size(dtype)) % 16 == 0 && reinterpret_cast<uintptr_t>(in) % 16 == 0 && reinterpret_cast<uintptr_t>(out) % 16 == 0) {
        const int cv = (int)(C * dtype_size(dtype) / 16);
        const size_t nv = (size_t)n_streams * Hout * Wout * cv;
        if (!AVG && k == 2 && s == 2 && p == 0 && (size_t)n_streams * Hout <= 65535 && (size_t)Hin * Win * cv < 0x7fffffffull) {
            const dim3 grid((unsigned)((Wout * cv + 2 * kThreads - 1) / (2 * kThreads)), (unsigned)(n_streams * Hout));
            if (dtype == DC_BF16)
                hipLaunchKernelGGL(maxpool2x2_vec_kernel<__hip_bfloat16>, grid, dim3(kThreads), 0, st, (const uint4*)in, (uint4*)out,
                                   Hin, Win, cv, Hout, Wout);
            else
                hipLaunchKernelGGL(maxpool2x2_vec_kernel<float>, grid, dim3(kThreads), 0, st, (const uint4*)in, (uint4*)out, Hin,
                                   Win, cv, Hout, Wout);
            return hipGetLastError();
        }
        if (dtype == DC_BF16)
            hipLaunchKernelGGL((pool_vec_kernel<__hip_bfloat16, AVG>), dim3(grid_for(nv)), dim3(kThreads), 0, st,
                               (const uint4*)in, (uint4*)out, n_streams, Hin, Win, cv, Hout, Wout, k, s, p);
        else
            hipLaunchKernelGGL((pool_vec_kernel<float, AVG>), dim3(grid_for(nv)), dim3(kThreads), 0, st, (const uint4*)in,
                               (uint4*)out, n_streams, Hin, Win, cv, Hout, Wout, k, s, p);
        return hipGetLastError();
    }
    if (dtype == DC_BF16)
        hipLaunchKernelGGL((pool_kernel<__hip_bfloat16, AVG>), dim3(grid_for(n)), dim3(kThreads), 0, st,
                           (const __hip_bfloat16*)in, (__hip_bfloat16*)out, n_streams, Hin, Win, C, Hout, Wout, k, s, p);
    else
        hipLaunchKernelGGL((pool_kernel<float, AVG>), dim3(grid_for(n)), dim3(kThreads), 0, st, (const float*)in,
                           (float*)out, n_streams, Hin, Win, C, Hout, Wout, k, s, p);
    return hipGetLastError();
}
}  // namespace

hipError_t launch_maxpool(const void* in, void* out, int n_streams, int Hin, int Win, int C, int k, int s,
                          int p, int dtype, hipStream_t st) {
    return launch_pool<false>(in, out, n_streams, Hin, Win, C, k, s, p, dtype, st);
}

template <typename T>
static void maxpool2x2_torus_go(dim3 grid, hipStream_t st, const void* in, void* out, int Hin, int Win, int cv, int Hout, int Wout,
                                const int32_t* origin, const int32_t* out_origin, int origin_stride, const CachedMap* M) {
    if (M)
        hipLaunchKernelGGL((maxpool2x2_torus_kernel<T, true>), grid, dim3(kThreads), 0, st, (const uint4*)in, (uint4*)out, Hin, Win,
                           cv, Hout, Wout, origin, out_origin, origin_stride, *M);
    else
        hipLaunchKernelGGL((maxpool2x2_torus_kernel<T, false>), grid, dim3(kThreads), 0, st, (const uint4*)in, (uint4*)out, Hin, Win,
                           cv, Hout, Wout, origin, out_origin, origin_stride, CachedMap{});
}

hipError_t launch_maxpool2x2_torus(const void* in, void* out, int n_streams, int Hin, int Win, int C, int dtype,
                                   const int32_t* origin, const int32_t* out_origin, int origin_stride, const CachedMap* M,
                                   hipStream_t st) {
    const int Hout = Hin / 2, Wout = Win / 2;
    if ((C * dtype_size(dtype)) % 16 || (size_t)n_streams * Hout > 65535 || !origin || Hout < 1 || Wout < 1) return hipErrorInvalidValue;
    if (M && (!M->bitmaps || !out_origin)) return hipErrorInvalidValue;     // a cached pooling output lies on a torus
    const int cv = (int)(C * dtype_size(dtype) / 16);
    const dim3 grid((unsigned)((Wout * cv + kThreads - 1) / kThreads), (unsigned)(n_streams * Hout));
    if (dtype == DC_BF16)
        maxpool2x2_torus_go<__hip_bfloat16>(grid, st, in, out, Hin, Win, cv, Hout, Wout, origin, out_origin, origin_stride, M);
    else
        maxpool2x2_torus_go<float>(grid, st, in, out, Hin, Win, cv, Hout, Wout, origin, out_origin, origin_stride, M);
    return hipGetLastError();
}

hipError_t launch_maxpool_cached(const void* in, const void* prev, void* out, int n_streams, int Hin, int Win, int C, int k,
                                 int s, int p, int dtype, const CachedMap& M, hipStream_t st) {
    const int Hout = (Hin + 2 * p - k) / s + 1, Wout = (Win + 2 * p - k) / s + 1;
    if ((C * dtype_size(dtype)) % 16 || (size_t)n_streams * Hout > 65535) return hipErrorInvalidValue;
    const int cv = (int)(C * dtype_size(dtype) / 16);
    const dim3 grid((unsigned)((Wout * cv + kThreads - 1) / kThreads), (unsigned)(n_streams * Hout));
    if (dtype == DC_BF16)
        hipLaunchKernelGGL(maxpool_cached_kernel<__hip_bfloat16>, grid, dim3(kThreads), 0, st, (const uint4*)in, (const uint4*)prev,
                           (uint4*)out, Hin, Win, cv, Hout, Wout, k, s, p, M);
    else
        hipLaunchKernelGGL(maxpool_cached_kernel<float>, grid, dim3(kThreads), 0, st, (const uint4*)in, (const uint4*)prev,
                           (uint4*)out, Hin, Win, cv, Hout, Wout, k, s, p, M);
    return hipGetLastError();
}

hipError_t launch_add_cached(const void* a, const void* b, const void* prev, void* out, int n_streams, int H, int W, int C,
                             int relu, int dtype, const CachedMap& M, hipStream_t st) {
    if ((C * dtype_size(dtype)) % 16 || (size_t)n_streams * H > 65535) return hipErrorInvalidValue;
    const int cv = (int)(C * dtype_size(dtype) / 16);
    const dim3 grid((unsigned)((W * cv + kThreads - 1) / kThreads), (unsigned)(n_streams * H));
    if (dtype == DC_BF16)
        hipLaunchKernelGGL(add_cached_kernel<__hip_bfloat16>, grid, dim3(kThreads), 0, st, (const uint4*)a, (const uint4*)b,
                           (const uint4*)prev, (uint4*)out, H, W, cv, relu, M);
    else
        hipLaunchKernelGGL(add_cached_kernel<float>, grid, dim3(kThreads), 0, st, (const uint4*)a, (const uint4*)b,
                           (const uint4*)prev, (uint4*)out, H, W, cv, relu, M);
    return hipGetLastError();
}

hipError_t launch_avgpool(const void* in, void* out, int n_streams, int Hin, int Win, int C, int k, int s,
                          int p, int dtype, hipStream_t st) {
    return launch_pool<true>(in, out, n_streams, Hin, Win, C, k, s, p, dtype, st);
}

hipError_t launch_lrn(const void* in, void* out, int n_streams, int H, int W, int C, int size, int within,
                      float alpha, float beta, float kappa, int dtype, hipStream_t st) {
    const size_t n = (size_t)n_streams * H * W * C;
    if (n == 0) return hipSuccess;
    const int r = (size - 1) / 2;
    const float alpha_n = alpha / (within ? (float)size * (float)size : (float)size);
    if (!within && (r == 1 || r == 2) && (C * dtype_size(dtype)) % 16 == 0 && reinterpret_cast<uintptr_t>(in) % 16 == 0 &&
        reinterpret_cast<uintptr_t>(out) % 16 == 0) {
        const int cv = (int)(C * dtype_size(dtype) / 16);
        const size_t px = (size_t)n_streams * H * W;
        const dim3 grid(grid_for(px * cv));
#define DC_LRN_VEC(T, R) hipLaunchKernelGGL((lrn_vec_kernel<T, R>), grid, dim3(kThreads), 0, st, (const uint4*)in, \
                                            (uint4*)out, px, cv, alpha_n, beta, kappa)
        if (dtype == DC_BF16) { if (r == 1) DC_LRN_VEC(__hip_bfloat16, 1); else DC_LRN_VEC(__hip_bfloat16, 2); }
        else { if (r == 1) DC_LRN_VEC(float, 1); else DC_LRN_VEC(float, 2); }
#undef DC_LRN_VEC
        return hipGetLastError();
    }
    if (dtype == DC_BF16)
        hipLaunchKernelGGL(lrn_kernel<__hip_bfloat16>, dim3(grid_for(n)), dim3(kThreads), 0, st,
                           (const __hip_bfloat16*)in, (__hip_bfloat16*)out, n_streams, H, W, C, r, within, alpha_n, beta,
                           kappa);
    else
        hipLaunchKernelGGL(lrn_kernel<float>, dim3(grid_for(n)), dim3(kThreads), 0, st, (const float*)in, (float*)out,
                           n_streams, H, W, C, r, within, alpha_n, beta, kappa);
    return hipGetLastError();
}

hipError_t launch_concat(const void* const* ins, const int* cs, int n_in, void* out, size_t n_pixels, int dtype,
                         hipStream_t st) {
    const size_t es = dtype_size(dtype);
    int ctot = 0;
    bool vec = reinterpret_cast<uintptr_t>(out) % 16 == 0;
    for (int j = 0; j < n_in; ++j) {
        ctot += cs[j];
        vec = vec && (cs[j] * es) % 16 == 0 && reinterpret_cast<uintptr_t>(ins[j]) % 16 == 0;
    }
    if (n_pixels == 0) return hipSuccess;
    const int unit = vec ? (int)(16 / es) : 1;        // elements per moved unit
    ConcatArgs a{};
    a.n = n_in; a.ctot = ctot / unit;
    int off = 0;
    for (int j = 0; j < n_in; ++j) {
        a.in[j] = ins[j]; a.c[j] = cs[j] / unit; a.off[j] = off / unit;
        off += cs[j];
    }
    const dim3 grid(grid_for(n_pixels * a.ctot));
    if (vec) hipLaunchKernelGGL(concat_all_kernel<uint4>, grid, dim3(kThreads), 0, st, a, (uint4*)out, n_pixels);
    else if (dtype == DC_BF16) hipLaunchKernelGGL(concat_all_kernel<uint16_t>, grid, dim3(kThreads), 0, st, a, (uint16_t*)out, n_pixels);
    else hipLaunchKernelGGL(concat_all_kernel<uint32_t>, grid, dim3(kThreads), 0, st, a, (uint32_t*)out, n_pixels);
    return hipGetLastError();
}

hipError_t launch_softmax(const void* in, void* out, size_t n_pixels, int C, int dtype, hipStream_t st) {
    if (n_pixels == 0 || C == 0) return hipSuccess;
    const size_t wgs = (n_pixels + kThreads / 64 - 1) / (kThreads / 64);
    if (wgs > 2147483647u) return hipErrorInvalidValue;
    if (dtype == DC_BF16)
        hipLaunchKernelGGL(softmax_kernel<__hip_bfloat16>, dim3((unsigned)wgs), dim3(kThreads), 0, st,
                           (const __hip_bfloat16*)in, (__hip_bfloat16*)out, n_pixels, C);
    else
        hipLaunchKernelGGL(softmax_kernel<float>, dim3((unsigned)wgs), dim3(kThreads), 0, st, (const float*)in,
                           (float*)out, n_pixels, C);
    return hipGetLastError();
}

namespace {
template <typename T, int VE>
hipError_t fc_launch(const void* x, const void* w, const float* bias, void* out, int n_streams, size_t K, int cout,
                     int relu, hipStream_t st) {
    const T* xp = (const T*)x;
    const T* wp = (const T*)w;
    T* op = (T*)out;
    constexpr int WPB = kThreads / 64;
    // streams per pass over the weights: the partial sums of a pass live in registers
    if (n_streams == 1) {
        const unsigned gx = (unsigned)((cout + WPB - 1) / WPB);
        hipLaunchKernelGGL((fc_kernel<T, 1, VE, 1>), dim3(gx, 1), dim3(kThreads), 0, st, xp, wp, bias, op, n_streams, K, cout, relu);
    } else if (n_streams <= 4) {
        const unsigned gx = (unsigned)((cout + WPB - 1) / WPB);
        hipLaunchKernelGGL((fc_kernel<T, 4, VE, 1>), dim3(gx, 1), dim3(kThreads), 0, st, xp, wp, bias, op, n_streams, K, cout, relu);
    } else if (n_streams <= 16) {     // one pass: bound by streaming the weights, as many wavefronts as possible
        const unsigned gx = (unsigned)((cout + WPB - 1) / WPB);
        hipLaunchKernelGGL((fc_kernel<T, 16, VE, 1>), dim3(gx, 1), dim3(kThreads), 0, st, xp, wp, bias, op, n_streams, K, cout, relu);
    } else {                          // several passes: four neurons per wavefront share every input vector
        const unsigned gx = (unsigned)((cout + 4 * WPB - 1) / (4 * WPB));
        hipLaunchKernelGGL((fc_kernel<T, 16, VE, 4>), dim3(gx, (unsigned)((n_streams + 15) / 16)), dim3(kThreads), 0, st, xp, wp,
                           bias, op, n_streams, K, cout, relu);
    }
    return hipGetLastError();
}
}  // namespace

hipError_t launch_fc(const void* x, const void* w, const float* bias, void* out, int n_streams, size_t K, int cout,
                     int relu, int dtype, hipStream_t st) {
    if (n_streams == 0 || cout == 0) return hipSuccess;
    if ((n_streams + 15) / 16 > 65535) return hipErrorInvalidValue;
    const size_t es = dtype_size(dtype);
    const bool vec = (K * es) % 16 == 0 && reinterpret_cast<uintptr_t>(x) % 16 == 0 && reinterpret_cast<uintptr_t>(w) % 16 == 0;
    if (dtype == DC_BF16)
        return vec ? fc_launch<__hip_bfloat16, 8>(x, w, bias, out, n_streams, K, cout, relu, st)
                   : fc_launch<__hip_bfloat16, 1>(x, w, bias, out, n_streams, K, cout, relu, st);
    return vec ? fc_launch<float, 4>(x, w, bias, out, n_streams, K, cout, relu, st)
               : fc_launch<float, 1>(x, w, bias, out, n_streams, K, cout, relu, st);
}

hipError_t launch_add(const void* a, const void* b, void* out, size_t n, int relu, int dtype, hipStream_t st) {
    if (n == 0) return hipSuccess;
    if ((n * dtype_size(dtype)) % 16 == 0 && reinterpret_cast<uintptr_t>(a) % 16 == 0 && reinterpret_cast<uintptr_t>(b) % 16 == 0 &&
        reinterpret_cast<uintptr_t>(out) % 16 == 0) {
        const size_t nv = n * dtype_size(dtype) / 16;
        if (dtype == DC_BF16)
            hipLaunchKernelGGL(add_vec_kernel<__hip_bfloat16>, dim3(grid_for(nv)), dim3(kThreads), 0, st, (const uint4*)a,
                               (const uint4*)b, (uint4*)out, nv, relu);
        else
            hipLaunchKernelGGL(add_vec_kernel<float>, dim3(grid_for(nv)), dim3(kThreads), 0, st, (const uint4*)a, (const uint4*)b,
                               (uint4*)out, nv, relu);
        return hipGetLastError();
    }
    if (dtype == DC_BF16)
        hipLaunchKernelGGL(add_kernel<__hip_bfloat16>, dim3(grid_for(n)), dim3(kThreads), 0, st,
                           (const __hip_bfloat16*)a, (const __hip_bfloat16*)b, (__hip_bfloat16*)out, n, relu);
    else
        hipLaunchKernelGGL(add_kernel<float>, dim3(grid_for(n)), dim3(kThreads), 0, st, (const float*)a,
                           (const float*)b, (float*)out, n, relu);
    return hipGetLastError();
}

}  // namespace dc
