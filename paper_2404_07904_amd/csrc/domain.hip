// Gate-domain probe.  The chunkwise kernels place one reference row in the middle of every
// 64-token chunk and divide by the gate product between a row and that reference; they are exact
// (up to rounding) while the product of the gates of each half chunk of each channel stays above
// 2^-100.  This kernel reads the gates once and returns the smallest such half-chunk product of
// the whole call, so that a caller can check its inputs against that bound:
//     min over (b, h, chunk n, half s, channel a) of  prod_{t in half s of chunk n} f[b, h, t, a]
// (with reference rows every 16 tokens the windows are 8 tokens long instead of 32).
// One wave per (sequence, window): a channel pair per lane, coalesced rows, a butterfly
// minimum over the lanes, one atomic minimum per wave (non-negative floats order like their bit
// patterns, so the integer atomic serves).
#include "common.hpp"
#include "kernels.hpp"

namespace hgrn2 {

struct DomainParams {
    const void* f;
    const float* beta;
    float* out;
    int BH, N, n_win, window, dk, gate_bf16, H;
    TokenLayout lay;
};

__global__ void domain_init_kernel(float* out) { *out = 1.0f; }

__global__ __launch_bounds__(256) void domain_min_kernel(DomainParams p)
{
    const int lane = threadIdx.x & 63;
    const long long wave = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);      // (sequence, window)
    const long long n_waves = (long long)p.BH * p.n_win;
    if (wave >= n_waves) return;
    const int bh = (int)(wave / p.n_win), hc = (int)(wave % p.n_win);
    const int row0 = hc * p.window;
    const bool active = 2 * lane < p.dk;
    const int col = active ? 2 * lane : 0;
    const size_t seq = p.lay.off_k(bh);
    f32x2 b = {0.0f, 0.0f};
    if (p.beta) b = *reinterpret_cast<const f32x2*>(p.beta + (size_t)(bh % p.H) * p.dk + col);
    float p0 = 1.0f, p1 = 1.0f;
    for (int i = 0; i < p.window; ++i) {
        const int row = row0 + i;
        if (row >= p.N) break;                                  // uniform over the wave
        f32x2 g = load_pair(p.f, seq + (size_t)row * p.lay.sn_k + col, p.gate_bf16 != 0);
        if (p.beta) g = f32x2{lower_bounded_gate(g.x, b.x), lower_bounded_gate(g.y, b.y)};
        p0 *= g.x; p1 *= g.y;
    }
    float m = active ? fminf(p0, p1) : 1.0f;
    m = fmaxf(m, 0.0f);                                         // a negative "gate" is outside any domain: report 0
#pragma unroll
    for (int s = 32; s >= 1; s >>= 1) m = fminf(m, __shfl_xor(m, s, 64));
    if (lane == 0) atomicMin(reinterpret_cast<int*>(p.out), __float_as_int(m));
}

hipError_t launch_min_gate_product(const SeqDims& d, int window, const void* f, float* out, hipStream_t stream)
{
    hipLaunchKernelGGL(domain_init_kernel, dim3(1), dim3(1), 0, stream, out);
    const int n_win = (d.N + window - 1) / window;
    const long long n_waves = (long long)d.BH * n_win;
    if (n_waves > 0) {
        DomainParams p;
        p.f = f; p.beta = d.beta; p.out = out; p.BH = d.BH; p.N = d.N; p.n_win = n_win; p.window = window; p.dk = d.dk;
        p.gate_bf16 = d.gate_bf16 ? 1 : 0; p.H = d.H; p.lay = d.lay;
        hipLaunchKernelGGL(domain_min_kernel, dim3((unsigned)((n_waves + 3) / 4)), dim3(256), 0, stream, p);
    }
    return hipGetLastError();
}

}   // namespace hgrn2
