// HGRN1: the element-wise gated linear recurrence the paper starts from (Section 2, Eq. 1, with
// the forget gate f of Eq. 2 given),
//
//     h_t = f_t * h_{t-1} + (1 - f_t) * i_t,      y_t = h_t * o_t        per channel,
//
// and its reverse mode.  Five flops per 8 bytes: the kernels are bound by HBM bandwidth, so they
// are organised to read every input once (the backward: the gates and inputs twice) with long
// coalesced streams in flight.  The recurrence is affine in h, so a segment of T consecutive
// tokens acts on its incoming state as h_out = A h_in + H with A = prod f and H the segment's
// result from a zero state.
//
// A workgroup of eight waves owns 64 channels of one sequence and walks it in blocks of sixteen
// segments.  Every half-wave takes one segment of the block (16 or 32 tokens, a channel pair per
// lane, so a load instruction of a wave fetches one 128-byte row piece for each of its two
// segments); with 64 channels per workgroup a [8][2048][2048] problem already gives one workgroup
// to each of the 256 compute units.  Per block:
//   1. the half-wave walks its segment from a zero state out of registers that were filled one
//      block ahead, and publishes (A, H) in LDS;
//   2. after one barrier every lane chains the sixteen summaries (32 fused multiply-adds) into
//      the state entering its own segment and the state leaving the block;
//   3. it walks the same registers again from the true state and writes its outputs.
// The forward keeps two register sets and requests a whole block ahead in one burst; the backward,
// which holds more per token, refills every register row with the next block's token as soon as
// the row is consumed.
// The backward first runs steps 1-2 over the whole sequence to record the state entering every
// segment (a few MB), then walks the blocks from the last to the first with the same scheme for
// the reverse recurrence  r_t = dy_t o_t + c_t,  c_{t-1} = f_t r_t.
// Tensors are [B][N][d] (token-major, d a multiple of 64), states [B][d] fp32.
//
// The "act" forms take the three pre-activations of Eq. 1 instead (the outputs of the layer's
// projections) and the layer's lower bounds of Eq. 2, and form
//     f = beta + (1 - beta) sigmoid(zf),   i = SiLU(zi),   o = sigmoid(zo)
// when a register row is first used: the layer never writes f, i or o to memory.
#include <type_traits>

#include "common.hpp"
#include "kernels.hpp"

namespace hgrn2 {


constexpr int kH1Waves = 8;                       // waves per workgroup
constexpr int kH1Threads = 64 * kH1Waves;
constexpr int kH1Chan = 64;                       // channels per workgroup: a pair per lane of a half-wave
constexpr int kH1Segs = 2 * kH1Waves;             // segments per block: one per half-wave
constexpr int kH1SegLong = 32;                    // tokens per segment
constexpr int kH1SegShort = 16;                   // ... of the backward with activations (it holds more per token)

struct H1Params {
    const void* f;        // gates, or their pre-activations zf
    const void* i;        // inputs, or zi
    const void* o;        // output gates, or zo
    const void* dy;
    const float* h0;
    const float* dhN;
    const float* beta;    // [d] lower bounds (act forms)
    void* y;
    void* df;
    void* di;
    void* dout;
    float* hN;
    float* dh0;
    float* carry;         // [B][NBLK * kH1Segs][d]: state entering every segment (backward)
    float* dbeta_part;    // [B][d]: every sequence's share of the gradient of beta (act backward)
    int B, N, d, NBLK, NCB;
    int NBLK16;           // blocks of 16-token segments: the granularity at which the forward pass leaves the states in `carry`
};

// A channel pair as it sits in memory: packed bf16 (one register) or two floats.
template <bool BF16> struct H1Raw {
    typedef uint32_t type;
    static __device__ __forceinline__ type one() { return 0x3f803f80u; }
};
template <> struct H1Raw<false> {
    typedef f32x2 type;
    static __device__ __forceinline__ type one() { return f32x2{1.0f, 1.0f}; }
};

// Token rows are addressed through buffer descriptors: one per tensor, covering the tokens from
// the start of a block to the end of the sequence.  The whole address of an access is the scalar
// descriptor plus a 32-bit per-lane byte offset, a read past the last token returns 0 and a write
// past it is dropped, so the ragged last block needs no clamped addresses and no branches.
typedef __amdgpu_buffer_rsrc_t H1Rsrc;

__device__ __forceinline__ H1Rsrc h1_rows_from(const void* tensor, size_t seq_elem, int tok0, int N, int d, int esize)
{
    const int first = min((unsigned)tok0, (unsigned)N);        // a negative tok0 gives an empty range
    const unsigned long long bytes = (unsigned long long)(N - first) * d * esize;
    const char* base = static_cast<const char*>(tensor) + (seq_elem + (size_t)first * d) * esize;
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(base), 0, (int)(unsigned)min(bytes, 0xfffffff8ull), 0x00020000);
}

template <bool BF16>
__device__ __forceinline__ typename H1Raw<BF16>::type h1_ld(H1Rsrc r, unsigned byte_off)
{
    if constexpr (BF16) {
        return __builtin_amdgcn_raw_buffer_load_b32(r, byte_off, 0, 0);
    } else {
        const auto v = __builtin_amdgcn_raw_buffer_load_b64(r, byte_off, 0, 0);
        return f32x2{__uint_as_float(v[0]), __uint_as_float(v[1])};
    }
}
__device__ __forceinline__ uint32_t h1_pack(float a, float b)
{
    bf16x2 h;
    h.x = (__bf16)a;
    h.y = (__bf16)b;
    return __builtin_bit_cast(uint32_t, h);
}
__device__ __forceinline__ void h1_st(H1Rsrc r, unsigned byte_off, float a, float b)
{
    __builtin_amdgcn_raw_buffer_store_b32(h1_pack(a, b), r, byte_off, 0, 0);
}
__device__ __forceinline__ f32x2 h1_cvt(uint32_t u)
{
    return f32x2{__uint_as_float(u << 16), __uint_as_float(u & 0xffff0000u)};
}
__device__ __forceinline__ f32x2 h1_cvt(f32x2 v) { return v; }

__device__ __forceinline__ float h1_sigmoid(float z) { return fast_rcp(1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * z)); }
__device__ __forceinline__ f32x2 h1_sigmoid(f32x2 z) { return f32x2{h1_sigmoid(z.x), h1_sigmoid(z.y)}; }
__device__ __forceinline__ f32x2 h1_silu(f32x2 z) { return f32x2{z.x * h1_sigmoid(z.x), z.y * h1_sigmoid(z.y)}; }

// At the top of a row's work in a second or third walk over the same registers: makes the compiler
// convert the packed values again there, instead of keeping a segment of converted floats alive or
// moving the row's arithmetic away from its place between the scheduling fences.
__device__ __forceinline__ void h1_forget(uint32_t& u) { asm volatile("" : "+v"(u)); }
__device__ __forceinline__ void h1_forget(f32x2& v) { asm volatile("" : "+v"(v.x), "+v"(v.y)); }
// The row pitch as a value the compiler recomputes offsets from (instead of keeping one per row).
__device__ __forceinline__ unsigned h1_pitch(int d) { unsigned x = 2u * (unsigned)d; asm volatile("" : "+s"(x)); return x; }

// chain the published summaries in ascending (forward) or descending (reverse) segment order:
// `mine` = state entering segment `vs` (this half-wave's), return value = state leaving the block
template <bool ASCENDING>
__device__ __forceinline__ f32x2 h1_chain(const f32x2 (*sA)[32], const f32x2 (*sX)[32], int vs, int cp, f32x2 c, f32x2& mine)
{
    mine = c;
#pragma unroll
    for (int k = 0; k < kH1Segs; ++k) {
        const int j = ASCENDING ? k : kH1Segs - 1 - k;
        if (j == vs) mine = c;
        const f32x2 A = sA[j][cp], X = sX[j][cp];
        c = f32x2{fmaf(A.x, c.x, X.x), fmaf(A.y, c.y, X.y)};
    }
    return c;
}

// The forget gate of a register row when it is first used: the stored gate, or Eq. 2 on its
// pre-activation; a row past the end of the sequence gets exactly 1 (its input reads as 0).
template <bool GATE_BF16, bool ACT>
__device__ __forceinline__ f32x2 h1_first_gate(typename H1Raw<GATE_BF16>::type raw, f32x2 beta, bool valid)
{
    f32x2 f = h1_cvt(raw);
    if constexpr (ACT) f = f32x2{lower_bounded_gate(f.x, beta.x), lower_bounded_gate(f.y, beta.y)};
    return valid ? f : f32x2{1.0f, 1.0f};
}

// Register rows of the gate: fr holds what was loaded (the next block's, from the moment the row
// is refilled).  Stored bf16 gates are used straight from it (one register per channel pair,
// converted at every use); fp32 gates and gates formed from pre-activations are kept as two
// floats in fa once the row has been used for the first time.
template <bool GATE_BF16, bool ACT, typename RAW>
__device__ __forceinline__ void h1_touch_gate(RAW& raw, f32x2& kept, f32x2 beta, bool valid)
{
    if constexpr (GATE_BF16 && !ACT) raw = valid ? raw : H1Raw<true>::one();
    else kept = h1_first_gate<GATE_BF16, ACT>(raw, beta, valid);
}
template <bool GATE_BF16, bool ACT, typename RAW>
__device__ __forceinline__ f32x2 h1_gate(RAW& raw, const f32x2& kept, bool again)
{
    if constexpr (GATE_BF16 && !ACT) {
        if (again) h1_forget(raw);
        return h1_cvt(raw);
    } else {
        return kept;
    }
}

// ---- forward -------------------------------------------------------------------------------------
// Two register sets: while one block is worked on out of one set, the loads of the next block,
// issued in one burst before that work starts, fill the other.  (A wave can wait for "all but the
// n youngest" of its loads only for n < 64, so a set is kept to 48 loads: 16-token segments.)
template <bool GATE_BF16, bool ACT>
__global__ __launch_bounds__(kH1Threads) void hgrn1_fwd_kernel(H1Params p)
{
    constexpr int TS = kH1SegShort, BLOCK = kH1Segs * TS;
    constexpr int GS = GATE_BF16 ? 1 : 2;         // gate bytes per bf16 byte
    __shared__ f32x2 sA[2][kH1Segs][32], sH[2][kH1Segs][32];
    const int cp = threadIdx.x & 31;                             // channel pair of the workgroup's 64 channels
    const int vs = threadIdx.x >> 5;                             // segment of the block: each half-wave walks its own
    const int b = blockIdx.x / p.NCB, cb = blockIdx.x % p.NCB;
    const size_t c0 = (size_t)cb * kH1Chan + 2 * cp;
    const size_t seq = (size_t)b * p.N * p.d;
    const unsigned lane_b = 2u * (unsigned)c0;                   // byte offset of this lane's pair in a bf16 row
    const f32x2 beta = ACT ? *reinterpret_cast<const f32x2*>(p.beta + c0) : f32x2{0.0f, 0.0f};

    struct Rows {
        typename H1Raw<GATE_BF16>::type fr[TS];
        uint32_t xr[TS], orw[TS];
    };
    f32x2 fa[TS];
    // all rows of a block; a block past the end of the sequence is an empty range and moves no data
    auto load_block = [&](Rows& s, int blk) {
        const H1Rsrc rf = h1_rows_from(p.f, seq, blk * BLOCK, p.N, p.d, 2 * GS),
                     ri = h1_rows_from(p.i, seq, blk * BLOCK, p.N, p.d, 2), ro = h1_rows_from(p.o, seq, blk * BLOCK, p.N, p.d, 2);
        const unsigned pitch = h1_pitch(p.d);
#pragma unroll
        for (int t = 0; t < TS; ++t) {
            const unsigned off = lane_b + (unsigned)(vs * TS + t) * pitch;
            s.fr[t] = h1_ld<GATE_BF16>(rf, off * GS);
            s.xr[t] = h1_ld<true>(ri, off);
            s.orw[t] = h1_ld<true>(ro, off);
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    f32x2 carry = p.h0 ? *reinterpret_cast<const f32x2*>(p.h0 + (size_t)b * p.d + c0) : f32x2{0.0f, 0.0f};
    // one block out of one register set (a block past the end: every row neutral, every store dropped)
    auto work = [&](Rows& s, int blk) {
        const int t0 = blk * BLOCK + vs * TS;
        const int par = blk & 1;
        // 1. segment summary from a zero state
        f32x2 a = {1.0f, 1.0f}, h = {0.0f, 0.0f};
#pragma unroll
        for (int t = 0; t < TS; ++t) {
            h1_touch_gate<GATE_BF16, ACT>(s.fr[t], fa[t], beta, t0 + t < p.N);
            if constexpr (ACT) { const f32x2 x = h1_silu(h1_cvt(s.xr[t])); s.xr[t] = h1_pack(x.x, x.y); }
            const f32x2 f = h1_gate<GATE_BF16, ACT>(s.fr[t], fa[t], false), x = h1_cvt(s.xr[t]);
            a = f32x2{a.x * f.x, a.y * f.y};
            h = f32x2{fmaf(f.x, h.x - x.x, x.x), fmaf(f.y, h.y - x.y, x.y)};      // f h + (1 - f) x
            __builtin_amdgcn_sched_barrier(0);
        }
        sA[par][vs][cp] = a;
        sH[par][vs][cp] = h;
        __syncthreads();
        // 2. state entering this half-wave's segment, state leaving the block
        f32x2 mine;
        carry = h1_chain<true>(sA[par], sH[par], vs, cp, carry, mine);
        // kept for a backward pass of the same step (hgrn1_bwd_saved): 8 bytes per lane and block
        if (p.carry && blk < p.NBLK)
            *reinterpret_cast<f32x2*>(p.carry + ((size_t)b * p.NBLK * kH1Segs + (size_t)blk * kH1Segs + vs) * p.d + c0) = mine;
        // 3. outputs
        const H1Rsrc ry = h1_rows_from(p.y, seq, blk * BLOCK, p.N, p.d, 2);
        const unsigned pitch = h1_pitch(p.d);
        h = mine;
#pragma unroll
        for (int t = 0; t < TS; ++t) {
            h1_forget(s.xr[t]);
            const f32x2 f = h1_gate<GATE_BF16, ACT>(s.fr[t], fa[t], true), x = h1_cvt(s.xr[t]);
            f32x2 og = h1_cvt(s.orw[t]);
            if constexpr (ACT) og = h1_sigmoid(og);
            h = f32x2{fmaf(f.x, h.x - x.x, x.x), fmaf(f.y, h.y - x.y, x.y)};
            h1_st(ry, lane_b + (unsigned)(vs * TS + t) * pitch, h.x * og.x, h.y * og.y);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    Rows even, odd;
    load_block(even, 0);
    for (int blk = 0; blk < p.NBLK; blk += 2) {      // always whole pairs: the pass after the last block works on an empty one
        load_block(odd, blk + 1);
        work(even, blk);
        load_block(even, blk + 2);
        work(odd, blk + 1);
    }
    if (p.hN && vs == 0) *reinterpret_cast<f32x2*>(p.hN + (size_t)b * p.d + c0) = carry;
}

// ---- backward ------------------------------------------------------------------------------------
//   dL/dh_t = r_t = dy_t o_t + c_t,  c_{t-1} = f_t r_t  (c_N = grad_hN)
//   do_t = dy_t h_t,   df_t = r_t (h_{t-1} - i_t),   di_t = r_t (1 - f_t),   dh0 = c_0
// act forms, through the activations (s = sigmoid):
//   dzo = do o (1 - o),   dzi = di s(zi) (1 + zi (1 - s(zi))),
//   dzf = df (f - beta)(1 - f) / (1 - beta),   dbeta = sum over batch and time of df (1 - f) / (1 - beta)
// SAVED: the forward pass of the same step has left the state entering every 16-token segment in
// `carry`; the forward phase below (a second pass over f and i) is then left out.
template <bool GATE_BF16, bool ACT, bool SAVED>
__global__ __launch_bounds__(kH1Threads) void hgrn1_bwd_kernel(H1Params p)
{
    constexpr int TS = ACT ? kH1SegShort : kH1SegLong, BLOCK = kH1Segs * TS;
    constexpr int GS = GATE_BF16 ? 1 : 2;
    __shared__ f32x2 sA[2][kH1Segs][32], sX[2][kH1Segs][32];      // sX: forward H, later the reverse summary
    const int cp = threadIdx.x & 31;
    const int vs = threadIdx.x >> 5;
    const int b = blockIdx.x / p.NCB, cb = blockIdx.x % p.NCB;
    const size_t c0 = (size_t)cb * kH1Chan + 2 * cp;
    const size_t seq = (size_t)b * p.N * p.d;
    const unsigned lane_b = 2u * (unsigned)c0;
    const int last_blk = p.NBLK - 1;
    const f32x2 beta = ACT ? *reinterpret_cast<const f32x2*>(p.beta + c0) : f32x2{0.0f, 0.0f};
    const f32x2 inv1mb = {1.0f / (1.0f - beta.x), 1.0f / (1.0f - beta.y)};
    // this thread's own slots of the saved states: written in the forward phase, read back in the reverse one
    float* my_carry = p.carry + ((size_t)b * p.NBLK * kH1Segs + vs) * p.d + c0;
    const size_t carry_blk = (size_t)kH1Segs * p.d;

    typename H1Raw<GATE_BF16>::type fr[TS];
    f32x2 fa[TS];
    uint32_t xr[TS], orw[TS], gr[TS];
    // the input of a row as the recurrence uses it (act: its pre-activation stays in the register,
    // the reverse walk needs it for the derivative)
    auto input_of = [&](uint32_t raw) {
        const f32x2 z = h1_cvt(raw);
        if constexpr (ACT) return h1_silu(z);
        else return z;
    };
    {
        // first rows: of block 0 for the forward phase, of the last block when the states are given
        const int first_tok = SAVED ? last_blk * BLOCK : 0;
        const H1Rsrc rf = h1_rows_from(p.f, seq, first_tok, p.N, p.d, 2 * GS), ri = h1_rows_from(p.i, seq, first_tok, p.N, p.d, 2);
        const unsigned pitch = h1_pitch(p.d);
#pragma unroll
        for (int t = 0; t < TS; ++t) {
            const unsigned off = lane_b + (unsigned)(vs * TS + t) * pitch;
            fr[t] = h1_ld<GATE_BF16>(rf, off * GS);
            xr[t] = h1_ld<true>(ri, off);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    int it = 0;       // LDS buffer parity runs over both phases

    // ---- forward phase: the state entering every segment ----
    // The last block is not followed by a refill: its gates and inputs stay in their registers,
    // which is where the reverse phase starts.
    f32x2 carry = p.h0 ? *reinterpret_cast<const f32x2*>(p.h0 + (size_t)b * p.d + c0) : f32x2{0.0f, 0.0f};
    auto forward_block = [&](int blk, auto refill_tag) {
        constexpr bool REFILL = decltype(refill_tag)::value;
        const int t0 = blk * BLOCK + vs * TS;
        const int par = it & 1;
        const H1Rsrc rf = h1_rows_from(p.f, seq, (blk + 1) * BLOCK, p.N, p.d, 2 * GS),
                     ri = h1_rows_from(p.i, seq, (blk + 1) * BLOCK, p.N, p.d, 2);
        const unsigned pitch = h1_pitch(p.d);
        f32x2 a = {1.0f, 1.0f}, h = {0.0f, 0.0f};
#pragma unroll
        for (int t = 0; t < TS; ++t) {
            const f32x2 f = h1_first_gate<GATE_BF16, ACT>(fr[t], beta, t0 + t < p.N), x = input_of(xr[t]);
            a = f32x2{a.x * f.x, a.y * f.y};
            h = f32x2{fmaf(f.x, h.x - x.x, x.x), fmaf(f.y, h.y - x.y, x.y)};
            if constexpr (REFILL) {
                const unsigned off = lane_b + (unsigned)(vs * TS + t) * pitch;
                fr[t] = h1_ld<GATE_BF16>(rf, off * GS);
                xr[t] = h1_ld<true>(ri, off);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        sA[par][vs][cp] = a;
        sX[par][vs][cp] = h;
        __syncthreads();
        f32x2 mine;
        carry = h1_chain<true>(sA[par], sX[par], vs, cp, carry, mine);
        *reinterpret_cast<f32x2*>(my_carry + blk * carry_blk) = mine;
        ++it;
    };
    if constexpr (!SAVED) {
        for (int blk = 0; blk < last_blk; ++blk) forward_block(blk, std::true_type{});
        forward_block(last_blk, std::false_type{});
    }

    // ---- reverse phase ----
    {
        // o and dy of the last block; f and i of it are in place
        const H1Rsrc rg = h1_rows_from(p.dy, seq, last_blk * BLOCK, p.N, p.d, 2),
                     ro = h1_rows_from(p.o, seq, last_blk * BLOCK, p.N, p.d, 2);
        const unsigned pitch = h1_pitch(p.d);
#pragma unroll
        for (int t = TS - 1; t >= 0; --t) {
            const unsigned off = lane_b + (unsigned)(vs * TS + t) * pitch;
            gr[t] = h1_ld<true>(rg, off);
            orw[t] = h1_ld<true>(ro, off);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    f32x2 cr = p.dhN ? *reinterpret_cast<const f32x2*>(p.dhN + (size_t)b * p.d + c0) : f32x2{0.0f, 0.0f};
    f32x2 dbeta = {0.0f, 0.0f};
    for (int blk = last_blk; blk >= 0; --blk, ++it) {
        const int t0 = blk * BLOCK + vs * TS;
        const int par = it & 1;
        f32x2 h_in;
        if constexpr (SAVED) {
            // the forward pass's slot of the 16-token segment this one starts with (a segment that lies
            // wholly past the end has none: any slot will do, its value reaches no result)
            const int seg16 = min((blk * kH1Segs + vs) * (TS / kH1SegShort), p.NBLK16 * kH1Segs - 1);
            h_in = *reinterpret_cast<const f32x2*>(p.carry + ((size_t)b * p.NBLK16 * kH1Segs + seg16) * p.d + c0);
        } else {
            h_in = *reinterpret_cast<const f32x2*>(my_carry + blk * carry_blk);
        }
        // reverse summary of the segment from c = 0 at its end (rows past the end: f = 1, dy was read as 0)
        f32x2 a = {1.0f, 1.0f}, q = {0.0f, 0.0f};
#pragma unroll
        for (int t = TS - 1; t >= 0; --t) {
            h1_touch_gate<GATE_BF16, ACT>(fr[t], fa[t], beta, t0 + t < p.N);
            if constexpr (ACT) { const f32x2 s = h1_sigmoid(h1_cvt(orw[t])); orw[t] = h1_pack(s.x, s.y); }
            const f32x2 f = h1_gate<GATE_BF16, ACT>(fr[t], fa[t], false), g = h1_cvt(gr[t]), og = h1_cvt(orw[t]);
            a = f32x2{a.x * f.x, a.y * f.y};
            q = f32x2{f.x * fmaf(g.x, og.x, q.x), f.y * fmaf(g.y, og.y, q.y)};
            __builtin_amdgcn_sched_barrier(0);
        }
        sA[par][vs][cp] = a;
        sX[par][vs][cp] = q;
        __syncthreads();
        f32x2 c;
        cr = h1_chain<false>(sA[par], sX[par], vs, cp, cr, c);
        // the state before every token of the segment
        f32x2 hp[TS];
        {
            f32x2 h = h_in;
#pragma unroll
            for (int t = 0; t < TS; ++t) {
                h1_forget(xr[t]);
                const f32x2 f = h1_gate<GATE_BF16, ACT>(fr[t], fa[t], true), x = input_of(xr[t]);
                hp[t] = h;
                h = f32x2{fmaf(f.x, h.x - x.x, x.x), fmaf(f.y, h.y - x.y, x.y)};
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        // gradients, last token first; every row is refilled with the previous block's token once consumed
        // block 0 has nothing before it: a negative first token makes its refills address an empty range
        const int pb = (blk - 1) * BLOCK, cb0 = blk * BLOCK;
        const H1Rsrc rdo = h1_rows_from(p.dout, seq, cb0, p.N, p.d, 2), rdf = h1_rows_from(p.df, seq, cb0, p.N, p.d, 2),
                     rdi = h1_rows_from(p.di, seq, cb0, p.N, p.d, 2);
        const H1Rsrc rf = h1_rows_from(p.f, seq, pb, p.N, p.d, 2 * GS), ri = h1_rows_from(p.i, seq, pb, p.N, p.d, 2),
                     rg = h1_rows_from(p.dy, seq, pb, p.N, p.d, 2), ro = h1_rows_from(p.o, seq, pb, p.N, p.d, 2);
        const unsigned pitch = h1_pitch(p.d);
#pragma unroll
        for (int t = TS - 1; t >= 0; --t) {
            h1_forget(xr[t]);
            h1_forget(gr[t]);
            h1_forget(orw[t]);
            const f32x2 f = h1_gate<GATE_BF16, ACT>(fr[t], fa[t], true), z = h1_cvt(xr[t]), g = h1_cvt(gr[t]), og = h1_cvt(orw[t]);
            f32x2 x = z, sx = {0.0f, 0.0f};
            if constexpr (ACT) { sx = h1_sigmoid(z); x = f32x2{z.x * sx.x, z.y * sx.y}; }
            const f32x2 e = {hp[t].x - x.x, hp[t].y - x.y};
            const f32x2 ht = {fmaf(f.x, e.x, x.x), fmaf(f.y, e.y, x.y)};
            const f32x2 r = {fmaf(g.x, og.x, c.x), fmaf(g.y, og.y, c.y)};
            f32x2 go = {g.x * ht.x, g.y * ht.y}, gf = {r.x * e.x, r.y * e.y};
            f32x2 gi = {r.x * (1.0f - f.x), r.y * (1.0f - f.y)};
            if constexpr (ACT) {
                go = f32x2{go.x * og.x * (1.0f - og.x), go.y * og.y * (1.0f - og.y)};
                gi = f32x2{gi.x * sx.x * fmaf(z.x, 1.0f - sx.x, 1.0f), gi.y * sx.y * fmaf(z.y, 1.0f - sx.y, 1.0f)};
                const f32x2 u = {gf.x * (1.0f - f.x) * inv1mb.x, gf.y * (1.0f - f.y) * inv1mb.y};      // df (1 - g)
                dbeta = f32x2{dbeta.x + u.x, dbeta.y + u.y};              // rows past the end add r e = c (h - 0) times 1 - f = 0
                gf = f32x2{u.x * (f.x - beta.x), u.y * (f.y - beta.y)};
            }
            const unsigned off = lane_b + (unsigned)(vs * TS + t) * pitch;
            h1_st(rdo, off, go.x, go.y);
            h1_st(rdf, off, gf.x, gf.y);
            h1_st(rdi, off, gi.x, gi.y);
            c = f32x2{f.x * r.x, f.y * r.y};
            fr[t] = h1_ld<GATE_BF16>(rf, off * GS);
            xr[t] = h1_ld<true>(ri, off);
            gr[t] = h1_ld<true>(rg, off);
            orw[t] = h1_ld<true>(ro, off);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    if (p.dh0 && vs == 0) *reinterpret_cast<f32x2*>(p.dh0 + (size_t)b * p.d + c0) = cr;
    if constexpr (ACT) {
        // this sequence's share of the gradient of beta: the sixteen segments' sums, added in order
        __syncthreads();
        sX[0][vs][cp] = dbeta;
        __syncthreads();
        if (vs == 0) {
            f32x2 t = {0.0f, 0.0f};
#pragma unroll
            for (int j = 0; j < kH1Segs; ++j) { const f32x2 u = sX[0][j][cp]; t = f32x2{t.x + u.x, t.y + u.y}; }
            *reinterpret_cast<f32x2*>(p.dbeta_part + (size_t)b * p.d + c0) = t;
        }
    }
}

// grad_beta[c] = sum over the batch of the sequences' shares, in index order
__global__ void hgrn1_reduce_beta_kernel(const float* part, float* grad_beta, int B, int d)
{
    const int c = blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= d) return;
    float s = 0.0f;
    for (int b = 0; b < B; ++b) s += part[(size_t)b * d + c];
    grad_beta[c] = s;
}

// N = 0: the final state is the initial one (and the gradient of the initial state that of the final one)
__global__ void hgrn1_copy_state_kernel(const float* src, float* dst, size_t n)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = src ? src[i] : 0.0f;
}

// ---- host side -----------------------------------------------------------------------------------
static int h1_blocks(int N, int seg) { return (N + kH1Segs * seg - 1) / (kH1Segs * seg); }

// saved segment states of the backward (sized for its shorter segments) and the per-sequence shares of grad_beta
static size_t h1_carry_floats(int B, int N, int d) { return (size_t)B * h1_blocks(N, kH1SegShort) * kH1Segs * d; }
size_t hgrn1_ws_bytes(int B, int N, int d)
{
    return (h1_carry_floats(B, N, d) + (size_t)B * d) * sizeof(float);
}

static H1Params h1_params(int B, int N, int d, int seg, void* ws)
{
    H1Params p = {};
    p.B = B; p.N = N; p.d = d; p.NBLK = h1_blocks(N, seg); p.NCB = d / kH1Chan;
    p.NBLK16 = h1_blocks(N, kH1SegShort);
    p.carry = static_cast<float*>(ws);
    p.dbeta_part = p.carry + h1_carry_floats(B, N, d);
    return p;
}

hipError_t launch_hgrn1_fwd(int B, int N, int d, bool gate_bf16, const void* f, const void* i, const void* o,
                            const float* beta, const float* h0, void* y, float* hN, void* ws, hipStream_t stream)
{
    if ((size_t)B * d == 0) return hipSuccess;
    if (N == 0) {
        if (hN) hipLaunchKernelGGL(hgrn1_copy_state_kernel, dim3((unsigned)(((size_t)B * d + 255) / 256)), dim3(256), 0,
                                   stream, h0, hN, (size_t)B * d);
        return hipGetLastError();
    }
    H1Params p = h1_params(B, N, d, kH1SegShort, ws);
    p.f = f; p.i = i; p.o = o; p.beta = beta; p.h0 = h0; p.y = y; p.hN = hN;
    const dim3 grid((unsigned)(B * p.NCB));
    auto kern = beta ? (gate_bf16 ? hgrn1_fwd_kernel<true, true> : hgrn1_fwd_kernel<false, true>)
                     : (gate_bf16 ? hgrn1_fwd_kernel<true, false> : hgrn1_fwd_kernel<false, false>);
    hipLaunchKernelGGL(kern, grid, dim3(kH1Threads), 0, stream, p);
    return hipGetLastError();
}

hipError_t launch_hgrn1_bwd(int B, int N, int d, bool gate_bf16, const void* f, const void* i, const void* o,
                            const float* beta, const float* h0, const void* dy, const float* dhN, void* df, void* di,
                            void* dout, float* dbeta, float* dh0, void* ws, bool states_saved, hipStream_t stream)
{
    if ((size_t)B * d == 0) return hipSuccess;
    if (N == 0) {
        if (dh0) hipLaunchKernelGGL(hgrn1_copy_state_kernel, dim3((unsigned)(((size_t)B * d + 255) / 256)), dim3(256), 0,
                                    stream, dhN, dh0, (size_t)B * d);
        if (beta && dbeta) hipLaunchKernelGGL(hgrn1_reduce_beta_kernel, dim3((d + 255) / 256), dim3(256), 0, stream,
                                              static_cast<const float*>(nullptr), dbeta, 0, d);
        return hipGetLastError();
    }
    H1Params p = h1_params(B, N, d, beta ? kH1SegShort : kH1SegLong, ws);
    p.f = f; p.i = i; p.o = o; p.beta = beta; p.dy = dy; p.h0 = h0; p.dhN = dhN; p.df = df; p.di = di; p.dout = dout; p.dh0 = dh0;
    const dim3 grid((unsigned)(B * p.NCB));
    auto kern = states_saved
                    ? (beta ? (gate_bf16 ? hgrn1_bwd_kernel<true, true, true> : hgrn1_bwd_kernel<false, true, true>)
                            : (gate_bf16 ? hgrn1_bwd_kernel<true, false, true> : hgrn1_bwd_kernel<false, false, true>))
                    : (beta ? (gate_bf16 ? hgrn1_bwd_kernel<true, true, false> : hgrn1_bwd_kernel<false, true, false>)
                            : (gate_bf16 ? hgrn1_bwd_kernel<true, false, false> : hgrn1_bwd_kernel<false, false, false>));
    hipLaunchKernelGGL(kern, grid, dim3(kH1Threads), 0, stream, p);
    if (beta && dbeta)
        hipLaunchKernelGGL(hgrn1_reduce_beta_kernel, dim3((d + 255) / 256), dim3(256), 0, stream, p.dbeta_part, dbeta, B, d);
    return hipGetLastError();
}

}   // namespace hgrn2
