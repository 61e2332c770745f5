// HGRN1: the element-wise gated linear recurrence the paper starts from (Section 2, Eq. 1, with
// the forget gate f of Eq. 2 given),
//
//     h_t = f_t * h_{t-1} + (1 - f_t) * i_t,      y_t = h_t * o_t        per channel,
//
// and its reverse mode.  Five flops per 8 bytes: the kernels are bound by HBM bandwidth, so they
// are organised around coalesced streaming and enough independent work to keep the memory system
// busy.  The recurrence is affine in h, so a segment of T consecutive tokens acts on its incoming
// state as h_out = A h_in + H with A = prod f and H the segment's result from a zero state:
//
//   pass 1 (summaries)  every wave takes one (batch, segment, 128 channels), walks its T tokens
//                       (one coalesced 256-byte row of each tensor per token, a channel pair per
//                       lane) and stores A and H (backward: also the reverse counterpart Q);
//   pass 2 (apply)      every wave composes the summaries of the segments before its own (after
//                       it, for the reverse direction) into its incoming state -- a few dozen
//                       fused multiply-adds on L2-resident data -- and walks its tokens again,
//                       now producing the outputs.
//
// Nothing waits on another workgroup, B * N/T * d/128 waves are independent, and the gates and
// inputs are read twice (the second time mostly from the 256 MB last-level cache).
// Tensors are [B][N][d] (token-major, d a multiple of 128), states [B][d] fp32.
#include "common.hpp"
#include "kernels.hpp"

namespace hgrn2 {

constexpr int kH1Threads = 256;          // four independent waves per workgroup
constexpr int kH1Chan = 128;             // channels per wave: a pair per lane
constexpr int kH1SegFwd = 64;            // tokens per segment, forward
constexpr int kH1SegBwd = 32;            // backward: the wave keeps h_{t-1} of its segment in registers

struct H1Params {
    const void* f;
    const void* i;
    const void* o;
    const void* dy;
    const float* h0;
    const float* dhN;
    void* y;          // forward: y; backward: unused
    void* df;
    void* di;
    void* dout;
    float* hN;
    float* dh0;
    float* sumA;      // [B][NS][d]
    float* sumH;      // [B][NS][d]
    float* sumQ;      // [B][NS][d]  (backward)
    int B, N, d, NS, NCB;
};

template <bool BF16>
__device__ __forceinline__ f32x2 h1_load(const void* base, size_t elem)
{
    return load_pair(base, elem, BF16);
}

// wave -> (batch, segment, channel block); waves next to each other share token rows
__device__ __forceinline__ bool h1_map(const H1Params& p, int& b, int& seg, int& c0)
{
    const long long gw = (long long)blockIdx.x * (kH1Threads / 64) + (threadIdx.x >> 6);
    if (gw >= (long long)p.B * p.NS * p.NCB) return false;
    const int cb = (int)(gw % p.NCB);
    seg = (int)((gw / p.NCB) % p.NS);
    b = (int)(gw / ((long long)p.NCB * p.NS));
    c0 = cb * kH1Chan + 2 * (threadIdx.x & 63);
    return true;
}

// ---- pass 1: segment summaries --------------------------------------------------------------------
template <bool GATE_BF16, int TS, bool BACKWARD>
__global__ __launch_bounds__(kH1Threads) void hgrn1_summaries_kernel(H1Params p)
{
    int b, seg, c0;
    if (!h1_map(p, b, seg, c0)) return;
    const int t0 = seg * TS, nt = min(TS, p.N - t0);
    const size_t base = ((size_t)b * p.N + t0) * p.d + c0;
    float a0 = 1.0f, a1 = 1.0f, h0 = 0.0f, h1 = 0.0f;
#pragma unroll 8
    for (int t = 0; t < nt; ++t) {
        const f32x2 f = h1_load<GATE_BF16>(p.f, base + (size_t)t * p.d);
        const f32x2 x = h1_load<true>(p.i, base + (size_t)t * p.d);
        a0 *= f.x; a1 *= f.y;
        h0 = fmaf(f.x, h0 - x.x, x.x); h1 = fmaf(f.y, h1 - x.y, x.y);        // f h + (1 - f) x
    }
    const size_t so = ((size_t)b * p.NS + seg) * p.d + c0;
    *reinterpret_cast<f32x2*>(p.sumA + so) = f32x2{a0, a1};
    *reinterpret_cast<f32x2*>(p.sumH + so) = f32x2{h0, h1};
    if (BACKWARD) {
        // reverse direction: r_t = dy_t o_t + c_t, c_{t-1} = f_t r_t, from c = 0 at the segment's end
        float c0r = 0.0f, c1r = 0.0f;
#pragma unroll 8
        for (int t = nt - 1; t >= 0; --t) {
            const f32x2 f = h1_load<GATE_BF16>(p.f, base + (size_t)t * p.d);
            const f32x2 g = h1_load<true>(p.dy, base + (size_t)t * p.d);
            const f32x2 og = h1_load<true>(p.o, base + (size_t)t * p.d);
            c0r = f.x * fmaf(g.x, og.x, c0r); c1r = f.y * fmaf(g.y, og.y, c1r);
        }
        *reinterpret_cast<f32x2*>(p.sumQ + so) = f32x2{c0r, c1r};
    }
}

// ---- pass 2, forward -----------------------------------------------------------------------------
template <bool GATE_BF16, int TS>
__global__ __launch_bounds__(kH1Threads) void hgrn1_fwd_apply_kernel(H1Params p)
{
    int b, seg, c0;
    if (!h1_map(p, b, seg, c0)) return;
    f32x2 h = p.h0 ? *reinterpret_cast<const f32x2*>(p.h0 + (size_t)b * p.d + c0) : f32x2{0.0f, 0.0f};
    {
        const float* sa = p.sumA + (size_t)b * p.NS * p.d + c0;
        const float* sh = p.sumH + (size_t)b * p.NS * p.d + c0;
#pragma unroll 4
        for (int j = 0; j < seg; ++j) {
            const f32x2 A = *reinterpret_cast<const f32x2*>(sa + (size_t)j * p.d);
            const f32x2 H = *reinterpret_cast<const f32x2*>(sh + (size_t)j * p.d);
            h.x = fmaf(A.x, h.x, H.x); h.y = fmaf(A.y, h.y, H.y);
        }
    }
    const int t0 = seg * TS, nt = min(TS, p.N - t0);
    const size_t base = ((size_t)b * p.N + t0) * p.d + c0;
    __bf16* yg = static_cast<__bf16*>(p.y);
#pragma unroll 8
    for (int t = 0; t < nt; ++t) {
        const f32x2 f = h1_load<GATE_BF16>(p.f, base + (size_t)t * p.d);
        const f32x2 x = h1_load<true>(p.i, base + (size_t)t * p.d);
        const f32x2 og = h1_load<true>(p.o, base + (size_t)t * p.d);
        h.x = fmaf(f.x, h.x - x.x, x.x); h.y = fmaf(f.y, h.y - x.y, x.y);
        store_pair_t<__bf16>(yg, base + (size_t)t * p.d, h.x * og.x, h.y * og.y);
    }
    if (p.hN && seg == p.NS - 1) *reinterpret_cast<f32x2*>(p.hN + (size_t)b * p.d + c0) = h;
}

// ---- pass 2, backward ----------------------------------------------------------------------------
//   dL/dh_t = r_t = dy_t o_t + c_t,  c_{t-1} = f_t r_t  (c_N = grad_hN)
//   do_t = dy_t h_t,   df_t = r_t (h_{t-1} - i_t),   di_t = r_t (1 - f_t),   dh0 = c_0
template <bool GATE_BF16, int TS>
__global__ __launch_bounds__(kH1Threads) void hgrn1_bwd_apply_kernel(H1Params p)
{
    int b, seg, c0;
    if (!h1_map(p, b, seg, c0)) return;
    const float* sa = p.sumA + (size_t)b * p.NS * p.d + c0;
    f32x2 h = p.h0 ? *reinterpret_cast<const f32x2*>(p.h0 + (size_t)b * p.d + c0) : f32x2{0.0f, 0.0f};
    {
        const float* sh = p.sumH + (size_t)b * p.NS * p.d + c0;
#pragma unroll 4
        for (int j = 0; j < seg; ++j) {
            const f32x2 A = *reinterpret_cast<const f32x2*>(sa + (size_t)j * p.d);
            const f32x2 H = *reinterpret_cast<const f32x2*>(sh + (size_t)j * p.d);
            h.x = fmaf(A.x, h.x, H.x); h.y = fmaf(A.y, h.y, H.y);
        }
    }
    f32x2 c = p.dhN ? *reinterpret_cast<const f32x2*>(p.dhN + (size_t)b * p.d + c0) : f32x2{0.0f, 0.0f};
    {
        const float* sq = p.sumQ + (size_t)b * p.NS * p.d + c0;
#pragma unroll 4
        for (int j = p.NS - 1; j > seg; --j) {
            const f32x2 A = *reinterpret_cast<const f32x2*>(sa + (size_t)j * p.d);
            const f32x2 Q = *reinterpret_cast<const f32x2*>(sq + (size_t)j * p.d);
            c.x = fmaf(A.x, c.x, Q.x); c.y = fmaf(A.y, c.y, Q.y);
        }
    }
    const int t0 = seg * TS, nt = min(TS, p.N - t0);
    const size_t base = ((size_t)b * p.N + t0) * p.d + c0;
    // forward walk: keep f, i and the state BEFORE every token
    f32x2 fr[TS], xr[TS], hp[TS];
#pragma unroll
    for (int t = 0; t < TS; ++t) {
        const size_t e = base + (size_t)min(t, nt - 1) * p.d;      // rows past the end re-read the last one, unused
        fr[t] = h1_load<GATE_BF16>(p.f, e);
        xr[t] = h1_load<true>(p.i, e);
    }
#pragma unroll
    for (int t = 0; t < TS; ++t) {
        hp[t] = h;
        if (t < nt) { h.x = fmaf(fr[t].x, h.x - xr[t].x, xr[t].x); h.y = fmaf(fr[t].y, h.y - xr[t].y, xr[t].y); }
    }
    __bf16* dfg = static_cast<__bf16*>(p.df);
    __bf16* dig = static_cast<__bf16*>(p.di);
    __bf16* dog = static_cast<__bf16*>(p.dout);
#pragma unroll
    for (int t = TS - 1; t >= 0; --t) {
        if (t < nt) {
            const size_t e = base + (size_t)t * p.d;
            const f32x2 g = h1_load<true>(p.dy, e);
            const f32x2 og = h1_load<true>(p.o, e);
            const float ht0 = fmaf(fr[t].x, hp[t].x - xr[t].x, xr[t].x), ht1 = fmaf(fr[t].y, hp[t].y - xr[t].y, xr[t].y);
            const float r0 = fmaf(g.x, og.x, c.x), r1 = fmaf(g.y, og.y, c.y);
            store_pair_t<__bf16>(dog, e, g.x * ht0, g.y * ht1);
            store_pair_t<__bf16>(dfg, e, r0 * (hp[t].x - xr[t].x), r1 * (hp[t].y - xr[t].y));
            store_pair_t<__bf16>(dig, e, r0 * (1.0f - fr[t].x), r1 * (1.0f - fr[t].y));
            c.x = fr[t].x * r0; c.y = fr[t].y * r1;
        }
    }
    if (p.dh0 && seg == 0) *reinterpret_cast<f32x2*>(p.dh0 + (size_t)b * p.d + c0) = c;
}

// N = 0: the final state is the initial one (and the gradient of the initial state that of the final one)
__global__ void hgrn1_copy_state_kernel(const float* src, float* dst, size_t n)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = src ? src[i] : 0.0f;
}

// ---- host side -----------------------------------------------------------------------------------
size_t hgrn1_ws_bytes(int B, int N, int d)
{
    const size_t ns = ((size_t)N + kH1SegBwd - 1) / kH1SegBwd;
    return 3 * (size_t)B * ns * d * sizeof(float);
}

static void h1_fill(H1Params& p, int B, int N, int d, int TS, void* ws)
{
    p.B = B; p.N = N; p.d = d; p.NS = (N + TS - 1) / TS; p.NCB = d / kH1Chan;
    const size_t one = (size_t)B * p.NS * d;
    p.sumA = static_cast<float*>(ws); p.sumH = p.sumA + one; p.sumQ = p.sumH + one;
}

static unsigned h1_grid(const H1Params& p)
{
    const long long waves = (long long)p.B * p.NS * p.NCB;
    return (unsigned)((waves + kH1Threads / 64 - 1) / (kH1Threads / 64));
}

hipError_t launch_hgrn1_fwd(int B, int N, int d, bool gate_bf16, const void* f, const void* i, const void* o,
                            const float* h0, void* y, float* hN, void* ws, hipStream_t stream)
{
    if ((size_t)B * d == 0) return hipSuccess;
    if (N == 0) {
        if (hN) hipLaunchKernelGGL(hgrn1_copy_state_kernel, dim3((unsigned)(((size_t)B * d + 255) / 256)), dim3(256), 0,
                                   stream, h0, hN, (size_t)B * d);
        return hipGetLastError();
    }
    H1Params p = {};
    p.f = f; p.i = i; p.o = o; p.h0 = h0; p.y = y; p.hN = hN;
    h1_fill(p, B, N, d, kH1SegFwd, ws);
    const unsigned grid = h1_grid(p);
    if (gate_bf16) {
        hipLaunchKernelGGL((hgrn1_summaries_kernel<true, kH1SegFwd, false>), dim3(grid), dim3(kH1Threads), 0, stream, p);
        hipLaunchKernelGGL((hgrn1_fwd_apply_kernel<true, kH1SegFwd>), dim3(grid), dim3(kH1Threads), 0, stream, p);
    } else {
        hipLaunchKernelGGL((hgrn1_summaries_kernel<false, kH1SegFwd, false>), dim3(grid), dim3(kH1Threads), 0, stream, p);
        hipLaunchKernelGGL((hgrn1_fwd_apply_kernel<false, kH1SegFwd>), dim3(grid), dim3(kH1Threads), 0, stream, p);
    }
    return hipGetLastError();
}

hipError_t launch_hgrn1_bwd(int B, int N, int d, bool gate_bf16, const void* f, const void* i, const void* o,
                            const float* h0, const void* dy, const float* dhN, void* df, void* di, void* dout,
                            float* dh0, void* ws, hipStream_t stream)
{
    if ((size_t)B * d == 0) return hipSuccess;
    if (N == 0) {
        if (dh0) hipLaunchKernelGGL(hgrn1_copy_state_kernel, dim3((unsigned)(((size_t)B * d + 255) / 256)), dim3(256), 0,
                                    stream, dhN, dh0, (size_t)B * d);
        return hipGetLastError();
    }
    H1Params p = {};
    p.f = f; p.i = i; p.o = o; p.dy = dy; p.h0 = h0; p.dhN = dhN; p.df = df; p.di = di; p.dout = dout; p.dh0 = dh0;
    h1_fill(p, B, N, d, kH1SegBwd, ws);
    const unsigned grid = h1_grid(p);
    if (gate_bf16) {
        hipLaunchKernelGGL((hgrn1_summaries_kernel<true, kH1SegBwd, true>), dim3(grid), dim3(kH1Threads), 0, stream, p);
        hipLaunchKernelGGL((hgrn1_bwd_apply_kernel<true, kH1SegBwd>), dim3(grid), dim3(kH1Threads), 0, stream, p);
    } else {
        hipLaunchKernelGGL((hgrn1_summaries_kernel<false, kH1SegBwd, true>), dim3(grid), dim3(kH1Threads), 0, stream, p);
        hipLaunchKernelGGL((hgrn1_bwd_apply_kernel<false, kH1SegBwd>), dim3(grid), dim3(kH1Threads), 0, stream, p);
    }
    return hipGetLastError();
}

}   // namespace hgrn2
