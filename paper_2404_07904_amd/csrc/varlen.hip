// Variable-length batches: B sequences packed back to back along the token axis.  The kernels
// find a sequence's tokens and its slots in the per-chunk workspaces through a small device table
// (TokenLayout::vl) that this kernel builds from the caller's cumulative sequence lengths:
//
//   table[0 .. B]            first token of sequence b            (entry B: end of the last one)
//   table[B+1 .. 2B+1]       length of sequence b                 (entry B: 0)
//   table[2B+2 .. 3B+2]      chunks of the sequences before b     (entry B: chunks of all)
//   table[3B+3 .. 4B+3]      the sequences ordered by falling length (entry B unused)
// The last array is for the kernels that give a whole sequence to one workgroup: workgroups start
// in index order, so handing out the longest sequences first keeps the longest one from being the
// last to start (for more than kSortMax sequences the order is left as it is).
//
// The offsets are clamped to [0, T] and replaced by their running maximum, so the table always
// describes disjoint, ordered pieces of the T tokens, whatever the caller's array holds: a wrong
// array gives wrong results, never an access outside the tensors or the workspaces.
#include "common.hpp"
#include "kernels.hpp"

namespace hgrn2 {

constexpr int kTabThreads = 256;
constexpr int kSortMax = 8192;
constexpr int kSortLds = 2048;
typedef int i32x4 __attribute__((ext_vector_type(4)));

// Group g of G starts at the first entry e whose chunks-before count reaches g / G of all chunks
// (bisection over the table's non-decreasing third array); the last group ends at the last entry,
// so that empty entries at the end belong to a group too.  Behind the G + 1 group starts: the choice
// between the two backward passes, then, for each of the G equal spans of chunks the reverse walk
// takes, the entry the span ends in.
// (Called by all threads of a one-workgroup kernel, after a barrier that follows the table's writes.)
__device__ __forceinline__ void build_groups(const int* tab, int n_entries, int G, int* groups)
{
    const int* before = tab + 2 * (n_entries + 1);
    const long long total = before[n_entries];
    for (int grp = threadIdx.x; grp <= G; grp += kTabThreads) {
        int first = n_entries;
        if (grp < G) {
            int lo = -1, hi = n_entries;                 // invariant: before[lo] G < grp total <= before[hi] G
            const long long want = (long long)grp * total;
            while (hi - lo > 1) {
                const int mid = (lo + hi) >> 1;
                if ((long long)before[mid] * G >= want) hi = mid; else lo = mid;
            }
            first = hi;
        }
        groups[grp] = first;
    }
    __syncthreads();
    // Which backward pass.  The reverse walk gives every workgroup a span of total / G chunks of a
    // head (about 10 us a chunk) and has it first walk, at a sixth of that cost, the chunks between
    // the end of its span and the end of the sequence the span ends in; the other pass (two sweeps,
    // as long as the longest sequence at about 4.6 us a chunk, then the per-chunk kernel at 11 us per
    // chunk of a compute unit's share) wins only when one sequence is several times longer than a
    // span: the walk is chosen while the longest such tail is at most four spans long.
    __shared__ int longest[kTabThreads];
    int mine = 0;
    for (int s = threadIdx.x; s < G; s += kTabThreads) {
        const long long p0 = (long long)s * total / G, p1 = (long long)(s + 1) * total / G;
        if (p1 <= p0) { groups[G + 2 + s] = 0; continue; }
        int lo = 0, hi = n_entries;                      // invariant: before[lo] <= p1 - 1 < before[hi]
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (before[mid] <= p1 - 1) lo = mid; else hi = mid;
        }
        groups[G + 2 + s] = lo;                          // the sequence span s ends in
        mine = max(mine, (int)(before[lo + 1] - p1));    // chunks of sequence `lo` after the span's last one
    }
    longest[threadIdx.x] = mine;
    __syncthreads();
    if (threadIdx.x == 0) {
        int m = 0;
        for (int j = 0; j < kTabThreads; ++j) m = max(m, longest[j]);
        const long long share = (total + G - 1) / G;
        groups[G + 1] = (m <= 4 * share) ? 1 : 0;
    }
}

__global__ __launch_bounds__(kTabThreads) void varlen_groups_kernel(const int* tab, int n_entries, int G, int* groups,
                                                                    const int* choice, int path)
{
    if (choice && table_read(choice, 0) != path) return;        // one of several alternatives, and not the one called for
    build_groups(tab, n_entries, G, groups);
}

// Exclusive prefix (sum, or running maximum of non-negative values) of one value per thread over the
// workgroup: inside a wave by shuffles, across the waves through `wave_tot` (one int per wave).
template <bool MAX>
__device__ __forceinline__ int block_prefix(int v, int* wave_tot)
{
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    int inc = v;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const int o = __shfl_up(inc, d, 64);
        if (lane >= d) inc = MAX ? max(inc, o) : inc + o;
    }
    __syncthreads();                    // (the previous use of wave_tot is over)
    if (lane == 63) wave_tot[w] = inc;
    __syncthreads();
    int before = 0;
    for (int j = 0; j < w; ++j) before = MAX ? max(before, wave_tot[j]) : before + wave_tot[j];
    int exc = __shfl_up(inc, 1, 64);
    if (lane == 0) exc = 0;
    return MAX ? max(before, exc) : before + exc;
}

// With `groups` (null: none) the group array of the table is built in the same launch.
__global__ __launch_bounds__(kTabThreads) void varlen_table_kernel(const int* cu, int B, int T, int* tab, int G, int* groups, int sub,
                                                                   const int* choice, int path)
{
    if (choice && table_read(choice, 0) != path) return;        // one of several alternatives, and not the one called for
    const int shift = 31 - __builtin_clz((unsigned)sub);         // sub is a power of two
    __shared__ int wave_tot[kTabThreads / 64];
    const int n = B + 1, tid = threadIdx.x;
    const int per = (n + kTabThreads - 1) / kTabThreads;
    const int lo = min(tid * per, n), hi = min(lo + per, n);      // this thread's entries
    auto clamped = [&](int i) { return min(max(cu[i], 0), T); };

    // starts: running maximum of the clamped offsets
    int m = 0;
    for (int i = lo; i < hi; ++i) m = max(m, clamped(i));
    int run = block_prefix<true>(m, wave_tot);
    for (int i = lo; i < hi; ++i) { run = max(run, clamped(i)); tab[i] = run; }
    __syncthreads();                                              // starts of the neighbouring slices are visible

    // lengths, and the chunk counts before every sequence
    int c = 0;
    for (int i = lo; i < hi; ++i) {
        const int len = i < B ? tab[i + 1] - tab[i] : 0;
        tab[n + i] = len;
        c += (len + sub - 1) >> shift;
    }
    run = block_prefix<false>(c, wave_tot);
    for (int i = lo; i < hi; ++i) {
        tab[2 * n + i] = run;
        run += (tab[n + i] + sub - 1) >> shift;
    }
    __syncthreads();                                              // all lengths are visible

    // order by falling length: the rank of sequence b is the number of sequences that come before
    // it (longer, or as long with a smaller index), counted directly
    const int* len = tab + n;
    int* order = tab + 3 * n;
    // (up to kSortLds sequences the lengths are compared out of LDS, four at a time)
    __shared__ int slen[kSortLds];
    const bool in_lds = B <= kSortLds;
    if (in_lds) {
        for (int j = tid; j < kSortLds; j += kTabThreads) slen[j] = j < B ? len[j] : -1;     // padding never counts
        __syncthreads();
    }
    for (int b = tid; b < B; b += kTabThreads) {
        int rank = b;
        if (in_lds) {
            rank = 0;
            const int mine = slen[b];
            for (int j = 0; j < ((B + 3) & ~3); j += 4) {
                const i32x4 l = *reinterpret_cast<const i32x4*>(slen + j);
#pragma unroll
                for (int e = 0; e < 4; ++e) rank += (l[e] > mine || (l[e] == mine && j + e < b)) ? 1 : 0;
            }
        } else if (B <= kSortMax) {
            rank = 0;
            const int mine = len[b];
            for (int j = 0; j < B; ++j) rank += (len[j] > mine || (len[j] == mine && j < b)) ? 1 : 0;
        }
        order[rank] = b;
    }
    if (groups) {
        __syncthreads();
        build_groups(tab, B, G, groups);
    }
}

// Long sequences of a packed batch are walked in runs of at most `run_chunks` chunks: the kernels
// then get a table whose entries are the runs (same four arrays, R entries, those past the last
// run empty), in which a run is a sequence like any other; only the carried states know which
// runs make up a sequence, through first_run[b] = number of runs of the sequences before b
// (B + 1 entries).  Runs are whole chunks, so the chunk counts of the run table add up as those of
// the sequence table do.  The runs keep their order (no sorting by length: none is long).
__global__ __launch_bounds__(kTabThreads) void varlen_run_table_kernel(const int* seq_tab, int B, int T, int run_chunks,
                                                                       int R, int* run_tab, int* first_run, int sub,
                                                                       const int* choice, int path)
{
    if (choice && table_read(choice, 0) != path) return;
    const int shift = 31 - __builtin_clz((unsigned)sub);         // sub is a power of two
    __shared__ int part[kTabThreads];
    const int n = B + 1, tid = threadIdx.x;
    const int per = (n + kTabThreads - 1) / kTabThreads;
    const int lo = min(tid * per, n), hi = min(lo + per, n);
    const int* start = seq_tab;
    const int* len = seq_tab + n;
    const int* before = seq_tab + 2 * n;
    auto runs_of = [&](int b) {
        const int nc = b < B ? (len[b] + sub - 1) >> shift : 0;
        return (nc + run_chunks - 1) / run_chunks;
    };
    int c = 0;
    for (int b = lo; b < hi; ++b) c += runs_of(b);
    part[tid] = c;
    __syncthreads();
    int first = 0;
    for (int j = 0; j < tid; ++j) first += part[j];
    const int m = R + 1, run_tokens = run_chunks * sub;
    for (int b = lo; b < hi; ++b) {
        first_run[b] = first;
        const int nr = runs_of(b);
        for (int k = 0; k < nr && first + k < R; ++k) {           // R bounds the runs of any batch of T tokens
            const int r = first + k;
            run_tab[r] = start[b] + k * run_tokens;
            run_tab[m + r] = min(run_tokens, len[b] - k * run_tokens);
            run_tab[2 * m + r] = before[b] + k * run_chunks;
            run_tab[3 * m + r] = r;
        }
        first += nr;
    }
    __syncthreads();
    const int used = min(first_run[B], R);
    for (int r = used + tid; r <= R; r += kTabThreads) {           // empty entries, and entry R of every array
        run_tab[r] = T;
        run_tab[m + r] = 0;
        run_tab[2 * m + r] = before[B];
        run_tab[3 * m + r] = r;
    }
}

// Zero fill as a kernel: a caller may have the stream under graph capture, where a memset node is
// not an option.
__global__ void zero_floats_kernel(float* dst, size_t n)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = 0.0f;
}

hipError_t launch_zero_floats(float* dst, size_t n, hipStream_t stream)
{
    if (n == 0) return hipSuccess;
    hipLaunchKernelGGL(zero_floats_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, dst, n);
    return hipGetLastError();
}

// *out = src[0] + ... + src[n - 1] (a few ints)
__global__ void sum_ints_kernel(const int* src, int n, int* out)
{
    int t = 0;
    for (int i = 0; i < n; ++i) t += src[i];
    *out = t;
}

hipError_t launch_sum_ints(const int* src, int n, int* out, hipStream_t stream)
{
    hipLaunchKernelGGL(sum_ints_kernel, dim3(1), dim3(1), 0, stream, src, n, out);
    return hipGetLastError();
}

size_t varlen_table_bytes(int B) { return 4 * ((size_t)B + 1) * sizeof(int); }

hipError_t launch_varlen_table(const int* cu_seqlens, int B, int T, int* table, hipStream_t stream, int G, int* groups, int sub,
                               const int* choice, int path)
{
    hipLaunchKernelGGL(varlen_table_kernel, dim3(1), dim3(kTabThreads), 0, stream, cu_seqlens, B, T, table, G, groups, sub, choice, path);
    return hipGetLastError();
}

size_t varlen_groups_bytes(int G) { return (2 * (size_t)G + 2) * sizeof(int); }

hipError_t launch_varlen_groups(const int* table, int n_entries, int G, int* groups, hipStream_t stream, const int* choice, int path)
{
    hipLaunchKernelGGL(varlen_groups_kernel, dim3(1), dim3(kTabThreads), 0, stream, table, n_entries, G, groups, choice, path);
    return hipGetLastError();
}

size_t varlen_run_table_bytes(int B, int R) { return varlen_table_bytes(R) + ((size_t)B + 1) * sizeof(int); }

hipError_t launch_varlen_run_table(const int* seq_table, int B, int T, int run_chunks, int R, int* run_table,
                                   int* first_run, hipStream_t stream, int sub, const int* choice, int path)
{
    hipLaunchKernelGGL(varlen_run_table_kernel, dim3(1), dim3(kTabThreads), 0, stream, seq_table, B, T, run_chunks, R,
                       run_table, first_run, sub, choice, path);
    return hipGetLastError();
}

}   // namespace hgrn2
