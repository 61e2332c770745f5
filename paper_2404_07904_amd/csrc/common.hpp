// Shared device-side building blocks for the gfx950 HGRN2 kernels.
//
// Notation (paper Section 3.2, Eq. 3 and Table 4): q = output gate (query), f = forget gate,
// k = 1 - f = input gate (key), v = input vector (value), S = dk x dv state.  Within one chunk
// of C tokens, G_r = prod_{s<=r} f_s is the cumulative gate product from the chunk start and
// g = G_C the whole-chunk decay.
//
// Thread layout used for all element-wise ("prep") work on a [C x D] tile: a workgroup has four
// wave64s; wave w owns the RW = C/4 consecutive rows (tokens) RW*w .. RW*w+RW-1 and lane l owns the
// channel pair (2l, 2l+1).  A global row is then one fully coalesced wave-wide load, the
// cumulative products along time run serially in registers, and because a thread holds RW
// consecutive tokens of a channel it can also write the tile TRANSPOSED (token-contiguous) to
// LDS with 16-byte vectors, which is the layout an MFMA operand needs when the contraction runs
// over time.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kernels.hpp"

namespace hgrn2 {

typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;
constexpr int kWaves = 4;
constexpr float kTinyProduct = 7.888609052210118e-31f;   // 2^-100: floor under a reciprocal

// LDS row padding (in elements) that keeps rows 16-byte aligned and staggers banks.
template <typename T> __host__ __device__ constexpr int pad_elems() { return 16 / (int)sizeof(T); }

__device__ __forceinline__ float fast_rcp(float x) { return __builtin_amdgcn_rcpf(x); }

// Entry i of one of the small device tables (sequence table, groups).  An earlier kernel wrote
// them and they are constant while a kernel of the passes runs, which the constant address space
// tells the compiler: a wave-uniform read then becomes a scalar load, which neither waits for nor
// is counted with the vector loads and stores a kernel has in flight.
__device__ __forceinline__ int table_read(const int* table, int i)
{
    typedef const __attribute__((address_space(4))) int* const_ptr;
    return ((const_ptr)table)[i];
}

// A launch may be one of several alternatives, of which an int that an earlier kernel wrote picks
// one (TokenLayout::choice, ::path): the workgroups of the others return at once.
__device__ __forceinline__ bool not_chosen(const TokenLayout& lay)
{
    return (lay.choice && table_read(lay.choice, 0) != lay.path) || (lay.alt && table_read(lay.alt, 0) != lay.alt_path);
}

// ---- which tokens a sequence (b, h) owns --------------------------------------------------------
// N tokens, NC chunks, element offsets of its first token in q / f (off_k) and v / o (off_v), and
// the index of its first chunk in the per-chunk workspaces.  `bh` must be uniform over the wave.
struct SeqView {
    size_t off_k, off_v, chunk0;
    int N, NC;
};

// Which tokens the C rows of chunk n of a sequence of N tokens stand for.  Ordinarily row r is token
// n C + r.  In the small-gate modes (TokenLayout::sub = 16 or 32) a chunk holds only `sub` tokens,
// n sub .. (n + 1) sub - 1, in its middle rows (C - sub) / 2 .. (C + sub) / 2 - 1: the mid-chunk
// reference row then has at most sub / 2 tokens on either side, which is all a quotient of gate
// products ever spans.  The other rows stand for no token and behave like the rows past the end of a
// sequence (f = 1, q = 0, whatever finite values for v and grad_o; nothing stored), which leaves
// Eq. 3 unchanged.  Row r stands for token tok0 + r iff first <= tok0 + r < end.
struct ChunkRows {
    int tok0, first, end;
    __device__ __forceinline__ bool holds(int row) const { return tok0 + row >= first && tok0 + row < end; }
};
__device__ __forceinline__ ChunkRows chunk_rows(int sub, int n, int N)
{
    ChunkRows c;
    c.tok0 = n * sub - (kChunk - sub) / 2;
    c.first = max(n * sub, 0);
    c.end = min(N, (n + 1) * sub);
    return c;
}

// RUNS: the caller is one of the kernels that walk a sequence and may be handed the runs of
// segmented sequences (TokenLayout::seg); the per-chunk kernels never are.
template <bool DENSE, int DK, int DV, bool RUNS = false>
__device__ __forceinline__ SeqView seq_view(const TokenLayout& lay, int N, int NC, int bh)
{
    SeqView s;
    if (RUNS && lay.seg > 1) {
        // run r of sequence bh / seg: N tokens (NC chunks) unless it is the last, shorter one
        const int whole = bh / lay.seg, r = bh - whole * lay.seg;
        const int nc_all = lay.chunks_of(lay.n_tokens);
        s.N = min(N, lay.n_tokens - r * N);
        s.NC = min(NC, nc_all - r * NC);
        s.chunk0 = (size_t)whole * nc_all + (size_t)r * NC;
        if constexpr (DENSE) {
            s.off_k = ((size_t)whole * lay.n_tokens + (size_t)r * N) * DK;
            s.off_v = ((size_t)whole * lay.n_tokens + (size_t)r * N) * DV;
        } else {
            s.off_k = lay.off_k(whole) + (size_t)r * N * lay.sn_k;
            s.off_v = lay.off_v(whole) + (size_t)r * N * lay.sn_v;
        }
        return s;
    }
    if constexpr (DENSE) {
        s.N = N; s.NC = NC;
        s.off_k = (size_t)bh * N * DK; s.off_v = (size_t)bh * N * DV;
        s.chunk0 = (size_t)bh * NC;
    } else {
        if (lay.vl) {
            const int b = bh / lay.H, h = bh - b * lay.H;
            const int start = table_read(lay.vl, b);
            s.N = table_read(lay.vl, lay.B + 1 + b);
            s.NC = lay.chunks_of(s.N);
            s.off_k = (size_t)start * lay.sn_k + (size_t)h * lay.sh_k;
            s.off_v = (size_t)start * lay.sn_v + (size_t)h * lay.sh_v;
            s.chunk0 = (size_t)table_read(lay.vl, 2 * (lay.B + 1) + b) * lay.H + (size_t)h * s.NC;
        } else {
            s.N = N; s.NC = NC;
            s.off_k = lay.off_k(bh); s.off_v = lay.off_v(bh);
            s.chunk0 = (size_t)bh * NC;
        }
    }
    return s;
}

// Kernels that give a whole sequence to one workgroup: which (b, h) the workgroup numbered `id`
// takes.  Workgroups start in index order, so variable-length batches hand out their sequences
// longest first.
template <bool DENSE>
__device__ __forceinline__ int sequence_of_workgroup(const TokenLayout& lay, int id)
{
    if constexpr (!DENSE) {
        if (lay.vl) {
            const int slot = id / lay.H, h = id - slot * lay.H;
            return table_read(lay.vl, 3 * (lay.B + 1) + slot) * lay.H + h;
        }
    }
    return id;
}

// Global chunk index -> (sequence, chunk within it).  Chunk indices run over the sequences in
// order, each sequence's NC chunks per head together.  With variable lengths the batch entry is
// found in the table's chunk counts: by bisection, or, for a caller that asks for non-decreasing
// chunk indices, by walking forward from the entry of its previous question (`hint`, start at 0).
// Returns false past the last chunk.
template <bool DENSE>
__device__ __forceinline__ bool locate_chunk(const TokenLayout& lay, int BH, int NC, int chunk, int& bh, int& n,
                                             int* hint = nullptr)
{
    if constexpr (!DENSE) {
        if (lay.vl) {
            const int* cb = lay.vl + 2 * (lay.B + 1);
            if (chunk >= cb[lay.B] * lay.H) return false;
            int lo;
            if (hint) {
                lo = *hint;                            // cb[lo] * H <= chunk holds from the previous question
                while (cb[lo + 1] * lay.H <= chunk) ++lo;
                *hint = lo;
            } else {
                lo = 0;
                int hi = lay.B;                        // invariant: cb[lo] * H <= chunk < cb[hi] * H
                while (hi - lo > 1) {
                    const int mid = (lo + hi) >> 1;
                    if (cb[mid] * lay.H <= chunk) lo = mid; else hi = mid;
                }
            }
            const int nc = lay.chunks_of(lay.vl[lay.B + 1 + lo]);               // > 0: the range is not empty
            const int rem = chunk - cb[lo] * lay.H;
            const int h = rem / nc;
            bh = lo * lay.H + h;
            n = rem - h * nc;
            return true;
        }
    }
    if (chunk >= BH * NC) return false;
    bh = chunk / NC;
    n = chunk - bh * NC;
    return true;
}

// ---- global memory access of element pairs, storage type chosen at run time -------------------
__device__ __forceinline__ f32x2 load_pair(const void* base, size_t idx, bool is_bf16)
{
    if (is_bf16) {
        const uint32_t u = *reinterpret_cast<const uint32_t*>(static_cast<const char*>(base) + idx * 2);
        f32x2 r;
        r.x = __uint_as_float(u << 16);
        r.y = __uint_as_float(u & 0xffff0000u);
        return r;
    }
    return *reinterpret_cast<const f32x2*>(static_cast<const char*>(base) + idx * 4);
}

template <typename T> __device__ __forceinline__ f32x2 load_pair_t(const T* base, size_t idx);
template <> __device__ __forceinline__ f32x2 load_pair_t<__bf16>(const __bf16* base, size_t idx)
{
    return load_pair(base, idx, true);
}
template <> __device__ __forceinline__ f32x2 load_pair_t<float>(const float* base, size_t idx)
{
    return load_pair(base, idx, false);
}

template <typename T> __device__ __forceinline__ void store_pair_t(T* base, size_t idx, float a, float b);
template <> __device__ __forceinline__ void store_pair_t<__bf16>(__bf16* base, size_t idx, float a, float b)
{
    bf16x2 h;
    h.x = (__bf16)a;
    h.y = (__bf16)b;
    *reinterpret_cast<bf16x2*>(base + idx) = h;
}
template <> __device__ __forceinline__ void store_pair_t<float>(float* base, size_t idx, float a, float b)
{
    f32x2 h;
    h.x = a;
    h.y = b;
    *reinterpret_cast<f32x2*>(base + idx) = h;
}

// ---- batched row loads ---------------------------------------------------------------------------
// RW consecutive rows of one channel pair, kept RAW (bf16 pairs as a 32-bit pattern in .x) so
// that all loads of a batch are issued back to back and converted only when first used.  Row
// indices are clamped into [0, n_rows) and the column is the caller's (already valid) one, so
// every address is in bounds and no load sits behind a branch; out-of-range rows are replaced
// by `fill` at conversion time.  (`row0` may be negative or past the end: the first rows of a chunk
// of a small-gate mode stand for no token, see ChunkRows.)
template <int RW> struct RawRows { f32x2 r[RW]; };

template <int RW>
__device__ __forceinline__ void load_rows(RawRows<RW>& out, const void* base, size_t seq_off, int row_stride,
                                          int col, int row0, int n_rows, bool is_bf16)
{
    // A block that lies fully inside the sequence (every block but possibly the last) needs one
    // address; its rows are compile-time offsets from it.  Only a ragged block clamps per row.
    const bool full = row0 >= 0 && row0 + RW <= n_rows;
    if (is_bf16) {
        const char* b = static_cast<const char*>(base) + (seq_off + col) * 2;
        if (full) {
            const char* b0 = b + (size_t)row0 * row_stride * 2;
#pragma unroll
            for (int i = 0; i < RW; ++i)
                out.r[i].x = __uint_as_float(*reinterpret_cast<const uint32_t*>(b0 + i * row_stride * 2));
        } else {
#pragma unroll
            for (int i = 0; i < RW; ++i) {
                const int rc = min(max(row0 + i, 0), n_rows - 1);
                out.r[i].x = __uint_as_float(*reinterpret_cast<const uint32_t*>(b + (size_t)rc * row_stride * 2));
            }
        }
    } else {
        const char* b = static_cast<const char*>(base) + (seq_off + col) * 4;
        if (full) {
            const char* b0 = b + (size_t)row0 * row_stride * 4;
#pragma unroll
            for (int i = 0; i < RW; ++i) out.r[i] = *reinterpret_cast<const f32x2*>(b0 + i * row_stride * 4);
        } else {
#pragma unroll
            for (int i = 0; i < RW; ++i) {
                const int rc = min(max(row0 + i, 0), n_rows - 1);
                out.r[i] = *reinterpret_cast<const f32x2*>(b + (size_t)rc * row_stride * 4);
            }
        }
    }
}

// The same without any branch: rows past `last_row` re-read that row (conversion replaces them
// by the fill value).  `seq_base` (start of the sequence, in bytes) and `row0` must be
// wave-uniform, so that the row addresses live in scalar registers and the lane only adds its
// byte offset; every load is issued unconditionally, which lets the compiler count outstanding
// loads exactly instead of draining them all.
template <int RW, bool IS_BF16>
__device__ __forceinline__ void load_rows_clamped(RawRows<RW>& out, const char* seq_base, int row0, int last_row,
                                                  int row_elems, int lane_col)
{
    constexpr int ES = IS_BF16 ? 2 : 4;
    if (row0 >= 0 && row0 + RW - 1 <= last_row) {      // whole block inside the sequence: one address, constant offsets
        const char* rp = seq_base + (size_t)row0 * (row_elems * ES) + lane_col * ES;
#pragma unroll
        for (int i = 0; i < RW; ++i) {
            if (IS_BF16) out.r[i].x = __uint_as_float(*reinterpret_cast<const uint32_t*>(rp + i * row_elems * ES));
            else out.r[i] = *reinterpret_cast<const f32x2*>(rp + i * row_elems * ES);
        }
    } else {
#pragma unroll
        for (int i = 0; i < RW; ++i) {
            const char* rp = seq_base + (size_t)min(max(row0 + i, 0), last_row) * (row_elems * ES);
            if (IS_BF16) out.r[i].x = __uint_as_float(*reinterpret_cast<const uint32_t*>(rp + lane_col * ES));
            else out.r[i] = *reinterpret_cast<const f32x2*>(rp + lane_col * ES);
        }
    }
}

// Rows row0 + i outside [first_row, n_rows) are replaced by `fill`.
template <int RW>
__device__ __forceinline__ void convert_rows(f32x2 (&dst)[RW], const RawRows<RW>& raw, int row0, int n_rows,
                                             bool lane_active, bool is_bf16, float fill, int first_row = 0)
{
    const bool all_rows = row0 >= first_row && row0 + RW <= n_rows;      // wave-uniform
#pragma unroll
    for (int i = 0; i < RW; ++i) {
        f32x2 x = raw.r[i];
        if (is_bf16) {
            const uint32_t u = __float_as_uint(raw.r[i].x);
            x.x = __uint_as_float(u << 16);
            x.y = __uint_as_float(u & 0xffff0000u);
        }
        dst[i] = x;
    }
    if (!all_rows || !lane_active) {
#pragma unroll
        for (int i = 0; i < RW; ++i) {
            const bool ok = lane_active && (row0 + i >= first_row) && (row0 + i < n_rows);
            dst[i].x = ok ? dst[i].x : fill;
            dst[i].y = ok ? dst[i].y : fill;
        }
    }
}

template <typename T> __host__ __device__ constexpr bool is_bf16_type() { return sizeof(T) == 2; }

// ---- lower-bounded forget gate (paper Section 2, Eq. 2) -------------------------------------------
// The gate tensor may hold the pre-activation z of the gate instead of the gate itself; the gate
// is then formed on the fly as f = beta + (1 - beta) * sigmoid(z), with one lower bound beta per
// channel of the layer ([H][dk], shared by batch and time).  Rows past the end of the sequence
// must read as f = 1 exactly, so the fill is applied after the transformation.
__device__ __forceinline__ float lower_bounded_gate(float z, float beta)
{
    const float s = fast_rcp(1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * z));
    return fmaf(1.0f - beta, s, beta);
}

template <int RW>
__device__ __forceinline__ void gate_rows(f32x2 (&rf)[RW], const float* beta_head, int col, bool lane_active,
                                          int row0, int n_rows, int first_row = 0)
{
    const f32x2 b = *reinterpret_cast<const f32x2*>(beta_head + col);
#pragma unroll
    for (int i = 0; i < RW; ++i) {
        const bool ok = lane_active && (row0 + i >= first_row) && (row0 + i < n_rows);
        rf[i].x = ok ? lower_bounded_gate(rf[i].x, b.x) : 1.0f;
        rf[i].y = ok ? lower_bounded_gate(rf[i].y, b.y) : 1.0f;
    }
}

// ---- matrix-core policy -------------------------------------------------------------------------
// One "k-step" contracts 16 values.  A fragment holds the 8 values one lane contributes to it:
// lane (r = lane % 32, g = lane / 32) supplies row r of A (or column r of B) at k-slots 8g..8g+7.
// Which physical k index a slot denotes is the caller's choice as long as A and B agree.
// Accumulator layout of a 32x32 tile (both MFMA flavours): register v of lane (c = lane % 32,
// g = lane / 32) is element [row 8*(v/4) + 4*g + v%4][column c].
template <typename T> struct Mma;

template <> struct Mma<__bf16> {
    typedef bf16x8 frag;
    static __device__ __forceinline__ frag load(const __bf16* p) { return *reinterpret_cast<const bf16x8*>(p); }
    // two separate runs of 4 consecutive values
    static __device__ __forceinline__ frag load2(const __bf16* p0, const __bf16* p1)
    {
        const bf16x4 lo = *reinterpret_cast<const bf16x4*>(p0);
        const bf16x4 hi = *reinterpret_cast<const bf16x4*>(p1);
        return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    }
    // 8 values `stride` elements apart (an operand whose k index is the slow axis of the tile)
    static __device__ __forceinline__ frag gather(const __bf16* p, int stride)
    {
        frag r;
#pragma unroll
        for (int s = 0; s < 8; ++s) r[s] = p[s * stride];
        return r;
    }
    // Operand whose k index is the SLOW axis of a row-major LDS tile (element (k, x) at
    // tile[k * pitch + x]): lane (x0 + lane % 32, g) receives k = k0 + 8g .. k0 + 8g + 7 through
    // two LDS transpose reads.  In a transpose read the 16 lanes of a group each fetch 4
    // consecutive 16-bit values (4 lanes per k row, 16 columns) and lane i gets back column i
    // of the 4 x 16 block, i.e. 4 consecutive k of one x.
    static __device__ __forceinline__ frag load_kmajor(const __bf16* tile, int pitch, int k0, int x0, int lane)
    {
        typedef __attribute__((address_space(3))) bf16x4 lds_bf16x4;
        const int i16 = lane & 15;
        const __bf16* p = tile + (k0 + 8 * (lane >> 5) + (i16 >> 2)) * pitch + x0 + (lane & 16) + 4 * (i16 & 3);
        const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)(p));
        const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)(p + 4 * pitch));
        return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    }
    // The same for a tile whose columns are stored, inside every group of 16, in the order the state
    // fragments keep their contraction index (column c at position c with bits 2 and 3 swapped):
    // lane x0 + lane % 32 receives the TRUE column x0 + lane % 32.  Only the quad of columns a
    // source lane supplies changes (quads 1 and 2 trade places).
    static __device__ __forceinline__ frag load_kmajor_swapped(const __bf16* tile, int pitch, int k0, int x0, int lane)
    {
        typedef __attribute__((address_space(3))) bf16x4 lds_bf16x4;
        const int i16 = lane & 15;
        const int quad = ((i16 & 1) << 1) | ((i16 & 2) >> 1);
        const __bf16* p = tile + (k0 + 8 * (lane >> 5) + (i16 >> 2)) * pitch + x0 + (lane & 16) + 4 * quad;
        const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)(p));
        const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)(p + 4 * pitch));
        return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    }
    static __device__ __forceinline__ frag pack(const float* x)
    {
        frag r;
#pragma unroll
        for (int s = 0; s < 8; ++s) r[s] = (__bf16)x[s];
        return r;
    }
    static __device__ __forceinline__ float get(const frag& a, int s) { return (float)a[s]; }
    static __device__ __forceinline__ void mma(f32x16& acc, const frag& a, const frag& b)
    {
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc, 0, 0, 0);
    }
};

template <> struct Mma<float> {
    struct frag { float v[8]; };
    static __device__ __forceinline__ frag load(const float* p)
    {
        frag r;
        const f32x4 lo = *reinterpret_cast<const f32x4*>(p);
        const f32x4 hi = *reinterpret_cast<const f32x4*>(p + 4);
#pragma unroll
        for (int s = 0; s < 4; ++s) { r.v[s] = lo[s]; r.v[4 + s] = hi[s]; }
        return r;
    }
    static __device__ __forceinline__ frag load2(const float* p0, const float* p1)
    {
        frag r;
        const f32x4 lo = *reinterpret_cast<const f32x4*>(p0);
        const f32x4 hi = *reinterpret_cast<const f32x4*>(p1);
#pragma unroll
        for (int s = 0; s < 4; ++s) { r.v[s] = lo[s]; r.v[4 + s] = hi[s]; }
        return r;
    }
    static __device__ __forceinline__ frag gather(const float* p, int stride)
    {
        frag r;
#pragma unroll
        for (int s = 0; s < 8; ++s) r.v[s] = p[s * stride];
        return r;
    }
    static __device__ __forceinline__ frag load_kmajor(const float* tile, int pitch, int k0, int x0, int lane)
    {
        return gather(tile + (k0 + 8 * (lane >> 5)) * pitch + x0 + (lane & 31), pitch);
    }
    // columns stored with bits 2 and 3 of their index swapped: lane x0 + lane % 32 receives the true column
    static __device__ __forceinline__ frag load_kmajor_swapped(const float* tile, int pitch, int k0, int x0, int lane)
    {
        const int c = lane & 31, pos = (c & ~12) | ((c & 4) << 1) | ((c & 8) >> 1);
        return gather(tile + (k0 + 8 * (lane >> 5)) * pitch + x0 + pos, pitch);
    }
    static __device__ __forceinline__ frag pack(const float* x)
    {
        frag r;
#pragma unroll
        for (int s = 0; s < 8; ++s) r.v[s] = x[s];
        return r;
    }
    static __device__ __forceinline__ float get(const frag& a, int s) { return a.v[s]; }
    // the fp32 MFMA contracts 2 values per instruction: lane group g supplies k = g
    static __device__ __forceinline__ void mma(f32x16& acc, const frag& a, const frag& b)
    {
#pragma unroll
        for (int s = 0; s < 8; ++s) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.v[s], b.v[s], acc, 0, 0, 0);
    }
};

// 16 consecutive columns of one row as raw bits, on their way from global memory to an LDS tile
// whose columns are kept, inside every group of 16, in the order the state fragments hold their
// contraction index: the four quads of columns land in the order (0, 2, 1, 3).
template <typename T> struct Raw16;
template <> struct Raw16<__bf16> {
    u32x4 v[2];
    __device__ __forceinline__ void load(const __bf16* p)
    {
        v[0] = *reinterpret_cast<const u32x4*>(p);
        v[1] = *reinterpret_cast<const u32x4*>(p + 8);
    }
    __device__ __forceinline__ void store_swapped(__bf16* dst) const
    {
        *reinterpret_cast<u32x4*>(dst) = u32x4{v[0][0], v[0][1], v[1][0], v[1][1]};
        *reinterpret_cast<u32x4*>(dst + 8) = u32x4{v[0][2], v[0][3], v[1][2], v[1][3]};
    }
};
template <> struct Raw16<float> {
    u32x4 v[4];
    __device__ __forceinline__ void load(const float* p)
    {
#pragma unroll
        for (int i = 0; i < 4; ++i) v[i] = *reinterpret_cast<const u32x4*>(p + 4 * i);
    }
    __device__ __forceinline__ void store_swapped(float* dst) const
    {
        *reinterpret_cast<u32x4*>(dst) = v[0];
        *reinterpret_cast<u32x4*>(dst + 4) = v[2];
        *reinterpret_cast<u32x4*>(dst + 8) = v[1];
        *reinterpret_cast<u32x4*>(dst + 12) = v[3];
    }
};

__device__ __forceinline__ int acc_row(int v, int lane) { return 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3); }

// Fragment order of a dk x dv state tile in the workspace: the 32x32 accumulator tile (ta, tb)
// is stored as two k-step fragments; fragment `half` of lane `lane` holds accumulator registers
// 8*half .. 8*half+7, i.e. rows 16*half + 8*(s/4) + 4*(lane/32) + s%4 (s = 0..7) of column
// lane%32.  A consumer reads the same 8 values back as one MFMA operand fragment.
__device__ __forceinline__ size_t state_frag_offset(int ta, int tb, int n_tb, int half, int lane)
{
    return ((size_t)((ta * n_tb + tb) * 2 + half) * 64 + lane) * 8;
}

// ---- per-thread gate products of one RW-token block ---------------------------------------------
template <int RW> struct GateBlock {
    float f[RW][2];   // gate values, channel pair
    float a[RW][2];   // inclusive product from the block start:  prod_{s<=i} f_s
    float z[RW][2];   // exclusive product to the block end:      prod_{s>i}  f_s
};

template <int RW> __device__ __forceinline__ void gate_products(GateBlock<RW>& gb)
{
#pragma unroll
    for (int c = 0; c < 2; ++c) {
        float run = 1.0f;
#pragma unroll
        for (int i = 0; i < RW; ++i) { run *= gb.f[i][c]; gb.a[i][c] = run; }
        run = 1.0f;
#pragma unroll
        for (int i = RW - 1; i >= 0; --i) { gb.z[i][c] = run; run *= gb.f[i][c]; }
    }
}

// Block totals of the four waves -> decay from the chunk start to this block's start (pre),
// from this block's end to the chunk end (post), and the extra factor that links this block to
// the mid-chunk reference row C/2 (mid): for the two blocks after the reference it is the
// product of the blocks between the reference and this block, likewise before it.
struct BlockDecay { float pre, post, mid, all; };

__device__ __forceinline__ BlockDecay block_decay(const float* tot, int D, int w, int ch)
{
    const float t0 = tot[0 * D + ch], t1 = tot[1 * D + ch], t2 = tot[2 * D + ch], t3 = tot[3 * D + ch];
    BlockDecay r;
    r.pre = (w == 0) ? 1.0f : (w == 1) ? t0 : (w == 2) ? t0 * t1 : t0 * t1 * t2;
    r.post = (w == 3) ? 1.0f : (w == 2) ? t3 : (w == 1) ? t2 * t3 : t1 * t2 * t3;
    r.mid = (w == 0) ? t1 : (w == 3) ? t2 : 1.0f;
    r.all = (t0 * t1) * (t2 * t3);
    return r;
}

// The same for NW row blocks (one per wave): products of the block totals before / after block w,
// between block w and the mid-chunk reference row, and over the whole chunk.
template <int NW> __device__ __forceinline__ BlockDecay block_decay_n(const float* tot, int D, int w, int ch)
{
    BlockDecay r;
    r.pre = 1.0f; r.post = 1.0f; r.mid = 1.0f; r.all = 1.0f;
#pragma unroll
    for (int i = 0; i < NW; ++i) {
        const float t = tot[i * D + ch];
        r.all *= t;
        r.pre *= (i < w) ? t : 1.0f;
        r.post *= (i > w) ? t : 1.0f;
        const bool between = (w >= NW / 2) ? (i >= NW / 2 && i < w) : (i > w && i < NW / 2);
        r.mid *= between ? t : 1.0f;
    }
    return r;
}

// Write RW consecutive values (one channel, tokens RW*w..) as 16-byte vectors to a transposed tile.
template <typename T, int RW> __device__ __forceinline__ void store_run(T* dst, const float* x);
template <> __device__ __forceinline__ void store_run<__bf16, 16>(__bf16* dst, const float* x)
{
    *reinterpret_cast<bf16x8*>(dst) = Mma<__bf16>::pack(x);
    *reinterpret_cast<bf16x8*>(dst + 8) = Mma<__bf16>::pack(x + 8);
}
template <> __device__ __forceinline__ void store_run<float, 16>(float* dst, const float* x)
{
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        f32x4 t;
        t.x = x[4 * j]; t.y = x[4 * j + 1]; t.z = x[4 * j + 2]; t.w = x[4 * j + 3];
        *reinterpret_cast<f32x4*>(dst + 4 * j) = t;
    }
}

// XCD-aware decomposition of a linear workgroup id into (sequence, tile): consecutive ids are
// dealt round-robin to the 8 XCDs, so all tiles of one sequence (which read the same q/f rows)
// are placed on the same XCD and share its L2.  The grid must be seq_padded * n_tile with
// seq_padded a multiple of 8; ids whose sequence is out of range exit.
__device__ __forceinline__ void xcd_map(int id, int n_tile, int& seq, int& tile)
{
    const int x = id & 7;
    const int r = id >> 3;
    tile = r % n_tile;
    seq = (r / n_tile) * 8 + x;
}

}   // namespace hgrn2
