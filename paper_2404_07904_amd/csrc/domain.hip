// Gate-domain probe.  The chunkwise kernels place one reference row in the middle of every
// 64-token chunk and divide by the gate product between a row and that reference; they are exact
// (up to rounding) while the product of the gates of each half chunk of each channel stays above
// 2^-100.  This kernel reads the gates once and returns the smallest such half-chunk product of
// the whole call, so that a caller can check its inputs against that bound:
//     min over (b, h, chunk n, half s, channel a) of  prod_{t in half s of chunk n} f[b, h, t, a]
// (with reference rows every 16 tokens the windows are 8 tokens long instead of 32).
// In a packed batch the windows start anew with every sequence, as the chunks do.
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
    long long n_waves;
    TokenLayout lay;
};

__global__ void domain_init_kernel(float* out) { *out = 1.0f; }

__global__ __launch_bounds__(256) void domain_min_kernel(DomainParams p)
{
    const int lane = threadIdx.x & 63;
    const long long wave = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);      // (sequence, window)
    if (wave >= p.n_waves) return;
    int bh, row0, n_rows = p.N;
    size_t seq;
    if (p.lay.vl) {
        // packed batch: windows are numbered chunk by chunk through the batch's sequence table
        const int per_chunk = kChunk / p.window;
        int n;
        if (!locate_chunk<false>(p.lay, 0, 0, (int)(wave / per_chunk), bh, n)) return;
        const SeqView sv = seq_view<false, 0, 0>(p.lay, 0, 0, bh);
        row0 = n * kChunk + (int)(wave % per_chunk) * p.window;
        n_rows = sv.N;
        seq = sv.off_k;
    } else {
        bh = (int)(wave / p.n_win);
        row0 = (int)(wave % p.n_win) * p.window;
        seq = p.lay.off_k(bh);
    }
    const bool active = 2 * lane < p.dk;
    const int col = active ? 2 * lane : 0;
    f32x2 b = {0.0f, 0.0f};
    if (p.beta) b = *reinterpret_cast<const f32x2*>(p.beta + (size_t)(bh % p.H) * p.dk + col);
    float p0 = 1.0f, p1 = 1.0f;
    for (int i = 0; i < p.window; ++i) {
        const int row = row0 + i;
        if (row >= n_rows) break;                               // uniform over the wave
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
    // packed batch: a bound on the windows of all sequences, a chunk's worth at a time (d.NC bounds the chunks)
    const int n_win = d.packed ? d.NC * (kChunk / window) : (d.N + window - 1) / window;
    const long long n_waves = d.packed ? (long long)d.H * n_win : (long long)d.BH * n_win;
    if (n_waves > 0) {
        DomainParams p;
        p.f = f; p.beta = d.beta; p.out = out; p.BH = d.BH; p.N = d.N; p.n_win = n_win; p.window = window; p.dk = d.dk; p.n_waves = n_waves;
        p.gate_bf16 = d.gate_bf16 ? 1 : 0; p.H = d.H; p.lay = d.lay;
        hipLaunchKernelGGL(domain_min_kernel, dim3((unsigned)((n_waves + 3) / 4)), dim3(256), 0, stream, p);
    }
    return hipGetLastError();
}

}   // namespace hgrn2
