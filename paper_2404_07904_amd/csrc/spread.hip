// Small gates in packed batches.  The chunkwise kernels divide by the gate product between a row and
// the reference row in the middle of its 64-token chunk, which limits them to gates whose product
// over a half chunk stays above 2^-100.  A caller whose gates can be smaller asks for reference rows
// every 32 or 16 tokens (hgrn2_shape::chunk = 32, 16): a chunk then holds only that many tokens, in
// its rows 16 .. 47 (24 .. 39) around the reference row, and its other rows stand for tokens that
// change nothing (f = 1, hence k = 0; q = 0; v = 0; grad_o = 0), so that no quotient spans more than
// 16 (8) real tokens.  For equal-length batches the kernels map chunk rows to tokens that way
// themselves (ChunkRows in common.hpp).  For packed batches the mode is built here from copies: every
// sequence is spread, block by block, into the middle rows of chunks of its own in a second packed
// batch whose other rows hold such filler tokens (where the kernels form f = beta + (1 - beta)
// sigmoid(z) themselves, z = +inf, for which that expression is exactly 1 in fp32); the spread batch
// goes through the ordinary packed entry point and the rows of the real tokens are copied back.
#include "common.hpp"
#include "kernels.hpp"

namespace hgrn2 {

namespace {

typedef uint32_t raw16 __attribute__((ext_vector_type(4)));    // 16 bytes of a row

// token t of a sequence sits at this row of the spread sequence
__device__ __forceinline__ long long spread_row(int t, int block)
{
    return (long long)(t / block) * kChunk + (kChunk - block) / 2 + t % block;
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

}   // namespace hgrn2
