// Measurement aid: the rate the matrix cores sustain on this GPU for the instruction stream of the bf16 convolution
// kernels' inner loop (v_mfma_f32_16x16x32_bf16, 4 x 4 tiles per wavefront, eight wavefronts per CU), with the
// operands in registers or re-read from LDS every step as the kernels do (4 + 4 fragments of 16 bytes per lane for 16
// MFMAs).  Under load the part lowers its clock to stay inside its power limit, so the rate a kernel can reach is
// below the published peak; the bench reports this figure next to the peak.
#include <type_traits>

#include "dc_conv_common.h"

namespace dc {
namespace {

template <int LDSR>
__global__ __launch_bounds__(512) void probe_mfma_kernel(const uint4* __restrict__ src, float* __restrict__ out, int steps) {
    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x;
    for (int i = tid; i < 8192; i += 512) reinterpret_cast<uint4*>(smem)[i] = src[(blockIdx.x * 8192 + i) & 0xffff];
    __syncthreads();
    bf16x8 x[2][4], w[2][4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        x[0][u] = x[1][u] = __builtin_bit_cast(bf16x8, src[(tid + u * 512) & 0xffff]);
        w[0][u] = w[1][u] = __builtin_bit_cast(bf16x8, src[(tid * 3 + u * 512 + 77) & 0xffff]);
    }
    floatx4 acc[4][4];
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[u][j] = floatx4{0.f, 0.f, 0.f, 0.f};
    const int addr = tid * 16;
    auto step = [&](int s, auto btag) {
        constexpr int b = decltype(btag)::value;
        if (LDSR) {
#pragma unroll
            for (int u = 0; u < 4; ++u) x[b ^ 1][u] = *reinterpret_cast<const bf16x8*>(smem + ((addr + u * 8192 + s * 1024) & 0x1fff0));
#pragma unroll
            for (int j = 0; j < 4; ++j) w[b ^ 1][j] = *reinterpret_cast<const bf16x8*>(smem + ((addr + j * 8192 + 4096 + s * 1024) & 0x1fff0));
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int j = 0; j < 4; ++j) acc[u][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w[b][j], x[b][u], acc[u][j], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
    };
    for (int s = 0; s < steps; s += 2) {
        step(s, std::integral_constant<int, 0>());
        step(s + 1, std::integral_constant<int, 1>());
    }
    floatx4 sum{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int j = 0; j < 4; ++j) sum += acc[u][j];
    out[(size_t)blockIdx.x * 512 + tid] = sum[0] + sum[1] + sum[2] + sum[3];
}

__global__ void probe_fill_kernel(uint32_t* p, size_t n) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) {
        // two bf16 values of moderate size per word (sign, exponent 126 / 127, varying mantissa)
        uint32_t h = (uint32_t)i * 2654435761u;
        const uint32_t lo = ((h >> 3) & 0x807fu) | 0x3f00u, hi = ((h >> 17) & 0x807fu) | 0x3f80u;
        p[i] = lo | (hi << 16);
    }
}

}  // namespace

hipError_t probe_mfma_rate(int lds_reads, void* scratch, int wgs, int steps, int launches, float* last_ms, hipStream_t st) {
    uint4* src = static_cast<uint4*>(scratch);
    float* out = reinterpret_cast<float*>(static_cast<unsigned char*>(scratch) + (1 << 20));
    hipLaunchKernelGGL(probe_fill_kernel, dim3(256), dim3(256), 0, st, static_cast<uint32_t*>(scratch), (size_t)(1 << 18));
    const size_t lds = 128 * 1024;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(probe_mfma_kernel<0>), hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLdsBytes);
    if (e == hipSuccess) e = hipFuncSetAttribute(reinterpret_cast<const void*>(probe_mfma_kernel<1>), hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLdsBytes);
    if (e != hipSuccess) return e;
    hipEvent_t e0, e1;
    if ((e = hipEventCreate(&e0)) != hipSuccess) return e;
    if ((e = hipEventCreate(&e1)) != hipSuccess) { (void)hipEventDestroy(e0); return e; }
    for (int i = 0; i < launches; ++i) {      // back to back: the last launch runs at the sustained clock
        if (i == launches - 1) (void)hipEventRecord(e0, st);
        if (lds_reads) hipLaunchKernelGGL(probe_mfma_kernel<1>, dim3(wgs), dim3(512), lds, st, src, out, steps);
        else hipLaunchKernelGGL(probe_mfma_kernel<0>, dim3(wgs), dim3(512), lds, st, src, out, steps);
    }
    (void)hipEventRecord(e1, st);
    e = hipEventSynchronize(e1);
    if (e == hipSuccess) e = hipEventElapsedTime(last_ms, e0, e1);
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    return e == hipSuccess ? hipGetLastError() : e;
}

}  // namespace dc
