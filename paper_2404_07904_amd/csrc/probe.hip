// Two probes of what the machine sustains, timed by the benchmark next to the kernels of the
// method: a plain device-to-device copy (the practical ceiling of a bandwidth-bound kernel here)
// and a loop of nothing but bf16 matrix instructions (the practical ceiling of the contractions).
#include "../../include/hgrn2.h"
#include "common.hpp"

namespace hgrn2 {

__global__ __launch_bounds__(256) void probe_copy_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n16)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

constexpr int kProbeChains = 4;      // independent accumulators per wave: covers the latency of the matrix pipeline

__global__ __launch_bounds__(256) void probe_mfma_kernel(int iters, float* out)
{
    typedef Mma<__bf16> M;
    M::frag a, b;
#pragma unroll
    for (int s = 0; s < 8; ++s) { a[s] = (__bf16)(0.001f * (float)((threadIdx.x + s) & 7)); b[s] = (__bf16)(0.002f * (float)((threadIdx.x + 3 * s) & 7)); }
    f32x16 acc[kProbeChains];
#pragma unroll
    for (int c = 0; c < kProbeChains; ++c)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[c][v] = 0.0f;
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int c = 0; c < kProbeChains; ++c) M::mma(acc[c], a, b);
    }
    float s = 0.0f;
#pragma unroll
    for (int c = 0; c < kProbeChains; ++c)
#pragma unroll
        for (int v = 0; v < 16; ++v) s += acc[c][v];
    out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;     // keeps the loop alive
}

}   // namespace hgrn2

extern "C" {

int hgrn2_probe_copy(void* dst, const void* src, size_t bytes, void* hip_stream)
{
    if (bytes == 0) return HGRN2_OK;
    if (!dst || !src) return HGRN2_ERR_NULL;
    if ((bytes & 15) || ((uintptr_t)dst & 15) || ((uintptr_t)src & 15)) return HGRN2_ERR_SHAPE;
    hipLaunchKernelGGL(hgrn2::probe_copy_kernel, dim3(256 * 8), dim3(256), 0, static_cast<hipStream_t>(hip_stream),
                       static_cast<const uint4*>(src), static_cast<uint4*>(dst), bytes / 16);
    return hipGetLastError() == hipSuccess ? HGRN2_OK : HGRN2_ERR_HIP;
}

size_t hgrn2_probe_mfma_out_floats(void) { return (size_t)256 * 8 * 256; }

int hgrn2_probe_mfma(int32_t iters, float* out, double* flops, void* hip_stream)
{
    if (iters < 0) return HGRN2_ERR_SHAPE;
    if (!out) return HGRN2_ERR_NULL;
    const int blocks = 256 * 8;          // eight workgroups of four waves per compute unit
    hipLaunchKernelGGL(hgrn2::probe_mfma_kernel, dim3(blocks), dim3(256), 0, static_cast<hipStream_t>(hip_stream), iters, out);
    if (flops) *flops = (double)blocks * 4.0 * (double)iters * hgrn2::kProbeChains * 2.0 * 32.0 * 32.0 * 16.0;
    return hipGetLastError() == hipSuccess ? HGRN2_OK : HGRN2_ERR_HIP;
}

}   // extern "C"
