// HBM-bound kernels: the shifted copy that serves reusable pixels from the previous
// frame's cached feature map (Section 5 "Reuse", step 1) and the layers that are never
// cached (Section 5: pooling, add, the input conversion).  All channels-last, 16-byte
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

// One thread per (output pixel, channel); consecutive threads walk the channels.
template <typename T>
__global__ __launch_bounds__(kThreads) void maxpool_kernel(const T* __restrict__ in, T* __restrict__ out,
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
        float m = -INFINITY;
        for (int ky = 0; ky < k; ++ky) {
            int iy = y * s - p + ky;
            if (iy < 0 || iy >= Hin) continue;
            for (int kx = 0; kx < k; ++kx) {
                int ix = x * s - p + kx;
                if (ix < 0 || ix >= Win) continue;
                float v = to_float(in[(((size_t)st * Hin + iy) * Win + ix) * C + c]);
                m = v > m ? v : m;
            }
        }
        out[i] = from_float<T>(m);
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

hipError_t launch_frame_to_tensor(const uint8_t* f, void* out, size_t n_pixels, int cf, int ct, int dtype,
                                  hipStream_t st) {
    const size_t n = n_pixels * ct;
    if (n == 0) return hipSuccess;
    if (dtype == DC_BF16)
        hipLaunchKernelGGL(frame_to_tensor_kernel<__hip_bfloat16>, dim3(grid_for(n)), dim3(kThreads), 0, st, f,
                           (__hip_bfloat16*)out, n, cf, ct);
    else
        hipLaunchKernelGGL(frame_to_tensor_kernel<float>, dim3(grid_for(n)), dim3(kThreads), 0, st, f,
                           (float*)out, n, cf, ct);
    return hipGetLastError();
}

hipError_t launch_maxpool(const void* in, void* out, int n_streams, int Hin, int Win, int C, int k, int s,
                          int p, int dtype, hipStream_t st) {
    const int Hout = (Hin + 2 * p - k) / s + 1, Wout = (Win + 2 * p - k) / s + 1;
    const size_t n = (size_t)n_streams * Hout * Wout * C;
    if (n == 0) return hipSuccess;
    if (dtype == DC_BF16)
        hipLaunchKernelGGL(maxpool_kernel<__hip_bfloat16>, dim3(grid_for(n)), dim3(kThreads), 0, st,
                           (const __hip_bfloat16*)in, (__hip_bfloat16*)out, n_streams, Hin, Win, C, Hout, Wout,
                           k, s, p);
    else
        hipLaunchKernelGGL(maxpool_kernel<float>, dim3(grid_for(n)), dim3(kThreads), 0, st, (const float*)in,
                           (float*)out, n_streams, Hin, Win, C, Hout, Wout, k, s, p);
    return hipGetLastError();
}

hipError_t launch_add(const void* a, const void* b, void* out, size_t n, int relu, int dtype, hipStream_t st) {
    if (n == 0) return hipSuccess;
    if (dtype == DC_BF16)
        hipLaunchKernelGGL(add_kernel<__hip_bfloat16>, dim3(grid_for(n)), dim3(kThreads), 0, st,
                           (const __hip_bfloat16*)a, (const __hip_bfloat16*)b, (__hip_bfloat16*)out, n, relu);
    else
        hipLaunchKernelGGL(add_kernel<float>, dim3(grid_for(n)), dim3(kThreads), 0, st, (const float*)a,
                           (const float*)b, (float*)out, n, relu);
    return hipGetLastError();
}

}  // namespace dc
