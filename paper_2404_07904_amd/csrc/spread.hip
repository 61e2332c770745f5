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

// ---- packed batches: every sequence is spread on its own -----------------------------------------
struct PackedSpreadParams {
    const char* src;
    char* dst;
    const int* seq_tab;      // the batch's sequence table: first token and length of every sequence
    const int* cu_spread;    // [B + 1] first row of every sequence in the spread batch
    int B, block, row_bytes;
    long long rows;          // spread rows (spread) or tokens (gather)
    uint32_t fill;
};

// largest b < B with first[b] <= x (first is non-decreasing; 0 if there is none)
__device__ __forceinline__ int sequence_at(const int* first, int B, long long x)
{
    int lo = 0, hi = B;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (first[mid] <= x) lo = mid; else hi = mid;
    }
    return lo;
}

__global__ __launch_bounds__(256) void spread_packed_kernel(PackedSpreadParams p)
{
    const int vecs = p.row_bytes / 16;
    const long long gid = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    const long long row = gid / vecs;
    if (row >= p.rows) return;
    const int vi = (int)(gid - row * vecs);
    raw16 val = {p.fill, p.fill, p.fill, p.fill};
    if (p.B > 0 && row < p.cu_spread[p.B]) {
        const int b = sequence_at(p.cu_spread, p.B, row);
        const int pos = (int)(row - p.cu_spread[b]), first = (kChunk - p.block) / 2;
        const int w = pos % kChunk, t = (pos / kChunk) * p.block + w - first;
        if (w >= first && w < first + p.block && t < p.seq_tab[p.B + 1 + b])
            val = *reinterpret_cast<const raw16*>(p.src + (long long)(p.seq_tab[b] + t) * p.row_bytes + vi * 16);
    }
    *reinterpret_cast<raw16*>(p.dst + row * p.row_bytes + vi * 16) = val;
}

__global__ __launch_bounds__(256) void gather_packed_kernel(PackedSpreadParams p)
{
    const int vecs = p.row_bytes / 16;
    const long long gid = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    const long long row = gid / vecs;
    if (row >= p.rows || p.B == 0) return;
    const int vi = (int)(gid - row * vecs);
    const int b = sequence_at(p.seq_tab, p.B, row);
    const long long t = row - p.seq_tab[b];
    if (t < 0 || t >= p.seq_tab[p.B + 1 + b]) return;          // a token of no sequence: left as it is
    const long long from = p.cu_spread[b] + spread_row((int)t, p.block);
    *reinterpret_cast<raw16*>(p.dst + row * p.row_bytes + vi * 16) =
        *reinterpret_cast<const raw16*>(p.src + from * p.row_bytes + vi * 16);
}

// cu_spread[b] = rows of the spread sequences before b (one workgroup, slices of the batch per thread)
__global__ __launch_bounds__(256) void spread_offsets_kernel(const int* seq_tab, int B, int block, int* cu_spread)
{
    __shared__ int part[256];
    const int n = B + 1, tid = threadIdx.x;
    const int per = (n + 255) / 256;
    const int lo = min(tid * per, n), hi = min(lo + per, n);
    auto rows_of = [&](int b) { return b < B ? (seq_tab[n + b] + block - 1) / block * kChunk : 0; };
    int c = 0;
    for (int b = lo; b < hi; ++b) c += rows_of(b);
    part[tid] = c;
    __syncthreads();
    int run = 0;
    for (int j = 0; j < tid; ++j) run += part[j];
    for (int b = lo; b < hi; ++b) { cu_spread[b] = run; run += rows_of(b); }
}

}   // namespace

int spread_tokens_packed(int T, int B, int block) { return (T / block + B) * kChunk; }

hipError_t launch_spread_offsets(const int* seq_table, int B, int block, int* cu_spread, hipStream_t stream)
{
    hipLaunchKernelGGL(spread_offsets_kernel, dim3(1), dim3(256), 0, stream, seq_table, B, block, cu_spread);
    return hipGetLastError();
}

hipError_t launch_spread_packed(int T, int B, int block, int row_bytes, SpreadFill fill, bool bf16, const int* seq_table,
                                const int* cu_spread, const void* src, void* dst, bool to_spread, hipStream_t stream)
{
    PackedSpreadParams p;
    p.src = static_cast<const char*>(src);
    p.dst = static_cast<char*>(dst);
    p.seq_tab = seq_table; p.cu_spread = cu_spread; p.B = B; p.block = block; p.row_bytes = row_bytes;
    p.rows = to_spread ? spread_tokens_packed(T, B, block) : T;
    p.fill = 0;
    if (fill == kFillOne) p.fill = bf16 ? 0x3f803f80u : 0x3f800000u;
    if (fill == kFillPlusInf) p.fill = bf16 ? 0x7f807f80u : 0x7f800000u;
    if (p.rows == 0) return hipSuccess;
    const long long threads = p.rows * (row_bytes / 16);
    if (to_spread) hipLaunchKernelGGL(spread_packed_kernel, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, stream, p);
    else           hipLaunchKernelGGL(gather_packed_kernel, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, stream, p);
    return hipGetLastError();
}

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
