// Small gates.  The chunkwise kernels divide by the gate product between a row and the reference
// row in the middle of its 64-token chunk, which limits them to gates whose product over a half
// chunk stays above 2^-100.  A caller whose gates can be smaller asks for reference rows every 32
// or 16 tokens (hgrn2_shape::chunk = 32, 16).  Those modes are built from the same kernels: every
// block of 32 (16) tokens is spread into a chunk of its own, at rows 16 .. 47 (24 .. 39) around
// the chunk's reference row, and the other rows are filled with tokens that change nothing (f = 1, hence k = 0; q = 0;
// v = 0; grad_o = 0; where the kernels form f = beta + (1 - beta) sigmoid(z) themselves, z = +inf,
// for which that expression is exactly 1 in fp32).  Eq. 3 over the spread sequence is the recurrence over the original one with
// identity steps in between, so outputs, gradients and states of the real tokens are the same,
// while no quotient spans more than 16 (8) real tokens.  It costs two (four) times the work and
// the memory of the spread tensors: a path for inputs outside the normal domain, not a fast one.
#include "common.hpp"
#include "kernels.hpp"

namespace hgrn2 {

namespace {

typedef uint32_t raw16 __attribute__((ext_vector_type(4)));    // 16 bytes of a row

struct SpreadParams {
    const char* src;
    char* dst;
    long long rows;          // BH * Np (spread) or BH * N (gather)
    int N, Np, H, d;
    int block;               // real tokens per chunk of the spread sequence, centred on its reference row
    long long sb, sh, sn;    // element strides of the caller's tensor: batch, head, token
    uint32_t fill;           // bit pattern of the filler, two bf16 or one float
};

// token t of a sequence sits at this row of the spread sequence
__device__ __forceinline__ long long spread_row(int t, int block)
{
    return (long long)(t / block) * kChunk + (kChunk - block) / 2 + t % block;
}

// One thread per 16 bytes of a spread row: the token's bytes, or the filler.
template <int ES>
__global__ __launch_bounds__(256) void spread_kernel(SpreadParams p)
{
    const int vecs = p.d * ES / 16;
    const long long gid = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    const long long row = gid / vecs;
    if (row >= p.rows) return;
    const int vi = (int)(gid - row * vecs);
    const int bh = (int)(row / p.Np), pos = (int)(row - (long long)bh * p.Np);
    const int first = (kChunk - p.block) / 2;
    const int w = pos % kChunk, t = (pos / kChunk) * p.block + w - first;
    raw16 val = {p.fill, p.fill, p.fill, p.fill};
    if (w >= first && w < first + p.block && t < p.N) {
        const long long e = (long long)(bh / p.H) * p.sb + (long long)(bh % p.H) * p.sh + (long long)t * p.sn;
        val = *reinterpret_cast<const raw16*>(p.src + e * ES + vi * 16);
    }
    *reinterpret_cast<raw16*>(p.dst + row * p.d * ES + vi * 16) = val;
}

// The reverse: one thread per 16 bytes of a row of the caller's tensor.
template <int ES>
__global__ __launch_bounds__(256) void gather_kernel(SpreadParams p)
{
    const int vecs = p.d * ES / 16;
    const long long gid = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    const long long row = gid / vecs;
    if (row >= p.rows) return;
    const int vi = (int)(gid - row * vecs);
    const int bh = (int)(row / p.N), t = (int)(row - (long long)bh * p.N);
    const long long from = (long long)bh * p.Np + spread_row(t, p.block);
    const long long e = (long long)(bh / p.H) * p.sb + (long long)(bh % p.H) * p.sh + (long long)t * p.sn;
    *reinterpret_cast<raw16*>(p.dst + e * ES + vi * 16) = *reinterpret_cast<const raw16*>(p.src + from * p.d * ES + vi * 16);
}

SpreadParams make_params(const SeqDims& d, int block, bool key_side, const void* src, void* dst, bool to_spread)
{
    SpreadParams p;
    p.src = static_cast<const char*>(src);
    p.dst = static_cast<char*>(dst);
    p.N = d.N;
    p.block = block;
    p.Np = spread_tokens(d.N, block);
    p.rows = (long long)d.BH * (to_spread ? p.Np : p.N);
    p.H = d.H;
    p.d = key_side ? d.dk : d.dv;
    p.sb = key_side ? d.lay.sb_k : d.lay.sb_v;
    p.sh = key_side ? d.lay.sh_k : d.lay.sh_v;
    p.sn = key_side ? d.lay.sn_k : d.lay.sn_v;
    p.fill = 0;
    return p;
}

template <typename K>
hipError_t launch_rows(K kern, const SpreadParams& p, int elem_size, hipStream_t stream)
{
    if (p.rows == 0) return hipSuccess;
    const long long threads = p.rows * (p.d * elem_size / 16);
    hipLaunchKernelGGL(kern, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, stream, p);
    return hipGetLastError();
}

}   // namespace

int spread_tokens(int N, int block) { return (N + block - 1) / block * kChunk; }

hipError_t launch_spread(const SeqDims& d, int block, bool key_side, bool bf16, SpreadFill fill, const void* src, void* dst,
                         hipStream_t stream)
{
    SpreadParams p = make_params(d, block, key_side, src, dst, true);
    if (fill == kFillOne) p.fill = bf16 ? 0x3f803f80u : 0x3f800000u;
    if (fill == kFillPlusInf) p.fill = bf16 ? 0x7f807f80u : 0x7f800000u;
    return bf16 ? launch_rows(spread_kernel<2>, p, 2, stream) : launch_rows(spread_kernel<4>, p, 4, stream);
}

hipError_t launch_gather(const SeqDims& d, int block, bool key_side, bool bf16, const void* src, void* dst, hipStream_t stream)
{
    const SpreadParams p = make_params(d, block, key_side, src, dst, false);
    return bf16 ? launch_rows(gather_kernel<2>, p, 2, stream) : launch_rows(gather_kernel<4>, p, 4, stream);
}

}   // namespace hgrn2
