// Single-token decode step (paper Section 3.2, Eq. 3, applied once per (batch, head)):
//     S <- Diag(f) S + (1 - f)^T v   in place,     o = q S   (from the updated state).
// Pure streaming read-modify-write of the fp32 state: one workgroup per (batch, head), each
// thread owns 16-byte column groups of several state rows, rows are fully coalesced, and the
// read-out is a per-thread partial dot product reduced across the row groups through LDS.
#include "common.hpp"
#include "kernels.hpp"

namespace hgrn2 {

template <typename T, int DK, int DV>
__global__ __launch_bounds__(kThreads) void step_kernel(const T* __restrict__ q, const void* __restrict__ f,
                                                        const T* __restrict__ v, float* __restrict__ state,
                                                        T* __restrict__ o, int gate_bf16,
                                                        const float* __restrict__ beta, int H)
{
    constexpr int CG = DV / 4;               // 16-byte column groups per row
    constexpr int RG = kThreads / CG;        // row groups
    constexpr int RPT = DK / RG;             // rows per thread
    __shared__ float sq[DK], sf[DK];
    __shared__ float part[RG][DV];

    const int bh = blockIdx.x, tid = threadIdx.x;
    if (tid < DK / 2) {
        const f32x2 qq = load_pair_t<T>(q, (size_t)bh * DK + 2 * tid);
        f32x2 ff = load_pair(f, (size_t)bh * DK + 2 * tid, gate_bf16 != 0);
        if (beta) {      // the gate tensor holds the pre-activation: f = beta + (1 - beta) sigmoid(z), Eq. 2
            const f32x2 bb = *reinterpret_cast<const f32x2*>(beta + (size_t)(bh % H) * DK + 2 * tid);
            ff = f32x2{lower_bounded_gate(ff.x, bb.x), lower_bounded_gate(ff.y, bb.y)};
        }
        sq[2 * tid] = qq.x; sq[2 * tid + 1] = qq.y;
        sf[2 * tid] = ff.x; sf[2 * tid + 1] = ff.y;
    }
    const int cg = tid % CG, rg = tid / CG;
    const f32x2 v01 = load_pair_t<T>(v, (size_t)bh * DV + 4 * cg);
    const f32x2 v23 = load_pair_t<T>(v, (size_t)bh * DV + 4 * cg + 2);
    float* S = state + (size_t)bh * DK * DV + 4 * cg;
    f32x4 s[RPT];
#pragma unroll
    for (int i = 0; i < RPT; ++i) s[i] = *reinterpret_cast<const f32x4*>(S + (size_t)(rg * RPT + i) * DV);
    __syncthreads();
    f32x4 acc; acc.x = 0.f; acc.y = 0.f; acc.z = 0.f; acc.w = 0.f;
#pragma unroll
    for (int i = 0; i < RPT; ++i) {
        const int a = rg * RPT + i;
        const float fa = sf[a], ka = 1.0f - fa, qa = sq[a];
        f32x4 x = s[i];
        x.x = fa * x.x + ka * v01.x;
        x.y = fa * x.y + ka * v01.y;
        x.z = fa * x.z + ka * v23.x;
        x.w = fa * x.w + ka * v23.y;
        *reinterpret_cast<f32x4*>(S + (size_t)a * DV) = x;
        acc.x += qa * x.x; acc.y += qa * x.y; acc.z += qa * x.z; acc.w += qa * x.w;
    }
    *reinterpret_cast<f32x4*>(&part[rg][4 * cg]) = acc;
    __syncthreads();
    if (tid < DV / 2) {
        float s0 = 0.f, s1 = 0.f;
#pragma unroll
        for (int r = 0; r < RG; ++r) { s0 += part[r][2 * tid]; s1 += part[r][2 * tid + 1]; }
        store_pair_t<T>(o, (size_t)bh * DV + 2 * tid, s0, s1);
    }
}

template <typename T>
static hipError_t launch_t(int BH, int dk, int dv, bool gate_bf16, const void* q, const void* f, const void* v,
                           float* state, void* o, const float* beta, int H, hipStream_t stream)
{
    const T* qq = static_cast<const T*>(q);
    const T* vv = static_cast<const T*>(v);
    T* oo = static_cast<T*>(o);
    const int gb = gate_bf16 ? 1 : 0;
    if (dk == 128 && dv == 128)
        hipLaunchKernelGGL((step_kernel<T, 128, 128>), dim3(BH), dim3(kThreads), 0, stream, qq, f, vv, state, oo, gb, beta, H);
    else if (dk == 64 && dv == 64)
        hipLaunchKernelGGL((step_kernel<T, 64, 64>), dim3(BH), dim3(kThreads), 0, stream, qq, f, vv, state, oo, gb, beta, H);
    else if (dk == 128 && dv == 64)
        hipLaunchKernelGGL((step_kernel<T, 128, 64>), dim3(BH), dim3(kThreads), 0, stream, qq, f, vv, state, oo, gb, beta, H);
    else if (dk == 64 && dv == 128)
        hipLaunchKernelGGL((step_kernel<T, 64, 128>), dim3(BH), dim3(kThreads), 0, stream, qq, f, vv, state, oo, gb, beta, H);
    else
        return hipErrorInvalidValue;
    return hipGetLastError();
}

hipError_t launch_step(int BH, int dk, int dv, bool io_bf16, bool gate_bf16, const void* q, const void* f,
                       const void* v, float* state, void* o, const float* beta, int H, hipStream_t stream)
{
    if (BH == 0) return hipSuccess;
    return io_bf16 ? launch_t<__bf16>(BH, dk, dv, gate_bf16, q, f, v, state, o, beta, H, stream)
                   : launch_t<float>(BH, dk, dv, gate_bf16, q, f, v, state, o, beta, H, stream);
}

}   // namespace hgrn2
