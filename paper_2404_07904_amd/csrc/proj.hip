// Input side of the HGRU2 token mixer (paper Section 2, Eq. 1): the three projections of the layer
// input and their activations,
//
//     z = U x + b_u   (pre-activation of the forget gate; Eq. 2 turns sigmoid(z) into f inside
//                      the recurrence kernels),
//     v = SiLU(V x + b_v)   (the paper's input vector i),
//     q = sigmoid(W x + b_w)   (the paper's output gate o),
//
// as ONE bf16 matrix product [M, d] x [d, 3d] on the matrix cores with bias and activation applied
// to the fp32 accumulators, written token-major ([B][N][H][dh] = [M][d]), which is the layout the
// recurrence takes with HGRN2_LAYOUT_BNHD: neither the pre-activations of q nor the gate ever
// reach memory.  The reverse mode is two more products, dx = dA W3 and dW3 = dA^T x, on the same
// kernel, after one element-wise pass that forms dA = (dz, dv SiLU'(a_v), dq q (1 - q)) and the
// bias gradients.
//
// Two matrix kernels, both with a 256 x 256 tile of the result per workgroup and the accumulators
// kept transposed (result column in the register index), so that four consecutive result columns of
// a row leave a lane together:
//   gemm_dl_kernel  both operands k-contiguous (x W3^T; dA W3 with W3 transposed beforehand): four
//                   waves of 128 x 128 or eight of 128 x 64, LDS stages filled by direct
//                   global -> LDS loads (see there);
//   gemm_kernel     an operand whose contraction index is the slow axis of its array (both operands
//                   of dW3 = dA^T x) keeps its natural orientation in LDS and is read with LDS
//                   transpose loads: eight waves (2 x 4, each 128 x 64), K in steps of 64 through
//                   double-buffered LDS tiles filled from registers loaded two steps ahead.
#include "../../include/hgrn2.h"
#include "common.hpp"
#include "kernels.hpp"
#include <type_traits>

namespace hgrn2 {

constexpr int kGemmThreads = 512;
constexpr int BM = 256, BN = 256, BK = 64;
constexpr int PKT = BK + 8;        // pitch of a tile kept [row][k]
constexpr int PXT = 256 + 32;      // pitch of a tile kept [k][row]: a transpose read takes 4 rows x 64 bytes per half wave, so rows 16 banks apart
constexpr int kTileElems = (BM * PKT > BK * PXT) ? BM * PKT : BK * PXT;
constexpr int kXcds = 8;         // accelerator dies; consecutive workgroup ids land on consecutive dies
constexpr int kBandRows = 4;     // row blocks per band of the workgroup -> tile order
constexpr int PST = BN + 8;        // pitch of the bf16 staging tile of the epilogue

enum GemmEpilogue { kEpiProj = 0, kEpiPlain = 1, kEpiFloat = 2 };

struct GemmParams {
    const __bf16* A;      // [M][K] (lda = K stride) or, A_KM, [K][M]
    const __bf16* B;      // [N][K] or, B_KM, [K][N]
    long long lda, ldb;
    int M, N, K;
    // outputs
    __bf16* C;            // kEpiPlain: [M][N] bf16, row stride ldc
    float* Cf;            // kEpiFloat: [M][N] fp32, row stride ldc
    long long ldc;
    // kEpiProj: N = 3 d; columns [0, d) -> z, [d, 2d) -> v (and a_v), [2d, 3d) -> q, each [M][d]
    const float* bias;
    __bf16 *z, *v, *q, *av;
    int d;
};

template <bool KM, int TR = 256>
__device__ __forceinline__ void tile_load(u32x4 (&r)[4], const __bf16* src, long long ld, int row0, int k0, int n_rows, int n_k, int tid)
{
    // TR x 64 elements = TR * 8 vectors of 16 bytes: four per thread (TR = 256) or three (192)
#pragma unroll
    for (int j = 0; j < TR / 64; ++j) {
        const int vi = tid + kGemmThreads * j;
        if constexpr (!KM) {
            const int row = vi >> 3, kc = (vi & 7) * 8;
            const int rc = min(row0 + row, n_rows - 1);          // rows past the end re-read the last one (never stored)
            r[j] = *reinterpret_cast<const u32x4*>(src + (size_t)rc * ld + k0 + kc);
        } else {
            const int kr = vi / (TR / 8), xc = (vi % (TR / 8)) * 8;
            const int kk = min(k0 + kr, n_k - 1);
            const int xr = min(row0 + xc, n_rows - 8);           // whole vectors stay inside the row (n_rows is a multiple of 8)
            u32x4 x = *reinterpret_cast<const u32x4*>(src + (size_t)kk * ld + xr);
            if (k0 + kr >= n_k) x = u32x4{0u, 0u, 0u, 0u};     // a contraction index past the end contributes nothing
            r[j] = x;
        }
    }
}

template <bool KM, int TR = 256>
__device__ __forceinline__ void tile_store(__bf16* tile, const u32x4 (&r)[4], int tid)
{
#pragma unroll
    for (int j = 0; j < TR / 64; ++j) {
        const int vi = tid + kGemmThreads * j;
        if constexpr (!KM) *reinterpret_cast<u32x4*>(tile + (size_t)(vi >> 3) * PKT + (vi & 7) * 8) = r[j];
        else               *reinterpret_cast<u32x4*>(tile + (size_t)(vi / (TR / 8)) * PXT + (vi % (TR / 8)) * 8) = r[j];
    }
}

template <bool KM>
__device__ __forceinline__ bf16x8 tile_frag(const __bf16* tile, int x0, int ks, int lane)
{
    if constexpr (!KM) return Mma<__bf16>::load(tile + (size_t)(x0 + (lane & 31)) * PKT + 16 * ks + 8 * (lane >> 5));
    else               return Mma<__bf16>::load_kmajor(tile, PXT, 16 * ks, x0, lane);
}

// TBM: rows of the tile, 256 or 192 (wave tiles of 128 or 96 rows).  The narrower tile is for
// products whose tile count would otherwise leave compute units idle (dW3 at width 2048: 24 x 8
// tiles of 256 rows on 256 units, but 32 x 8 of 192 rows).
template <bool A_KM, bool B_KM, int EPI, int TBM = 256>
__global__ __launch_bounds__(kGemmThreads) void gemm_kernel(GemmParams p)
{
    static_assert(TBM == 256 || (TBM == 192 && EPI == kEpiFloat), "the staged epilogues assume 256 rows");
    constexpr int NI = TBM / 64;                                    // 32-row MFMA tiles per wave
    typedef Mma<__bf16> M;
    extern __shared__ __align__(16) char smem[];
    __bf16* At = reinterpret_cast<__bf16*>(smem);                   // [2][tile]
    __bf16* Bt = At + 2 * kTileElems;                               // [2][tile]

    const int tid = threadIdx.x, lane = tid & 63, r32 = lane & 31, g = lane >> 5;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = w >> 2, wn = w & 3;                              // wave tile: rows (TBM / 2) wm .., columns 64 wn ..
    // Workgroup -> tile.  Workgroup ids go round the eight XCDs (id % 8), each with an L2 of its
    // own, so the ids are first renumbered so that an XCD holds a contiguous range, and the range is
    // laid over the tile grid in bands of kBandRows row blocks walked column by column: the 32
    // workgroups an XCD runs together then cover about 4 x 8 tiles and share their operand panels
    // in that XCD's L2 instead of each XCD streaming whole panels of its own.
    const int n_bn = p.N / BN, n_bm = (p.M + TBM - 1) / TBM;
    int bm, bn;
    {
        const int grid = (int)gridDim.x, id = (int)blockIdx.x;
        const int per = grid / kXcds, rem = grid - per * kXcds, x = id % kXcds;
        const int t = x * per + min(x, rem) + id / kXcds;             // position in the XCD-contiguous order
        const int band_tiles = kBandRows * n_bn, band = t / band_tiles, in_band = t - band * band_tiles;
        const int rows = min(kBandRows, n_bm - band * kBandRows);     // the last band may be shorter
        bn = in_band / rows;
        bm = band * kBandRows + in_band - bn * rows;
    }
    const int m0 = bm * TBM, n0 = bn * BN;

    // accumulators, transposed: acc[i][j][v] = C[m0 + (TBM / 2) wm + 32 i + lane % 32][n0 + 64 wn + 32 j + 8 (v/4) + 4 g + v%4]
    f32x16 acc[NI][2];
#pragma unroll
    for (int i = 0; i < NI; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    // Tiles travel global memory -> registers -> LDS.  The registers are loaded TWO steps ahead (two
    // register sets, the loop unrolled by two so that each set is a fixed group of registers): one
    // step of matrix work is shorter than a trip to memory.  Loads are unconditional (steps past
    // the end fetch the last one again and are never stored).
    u32x4 ra[2][4], rb[2][4];
    const int nk = (p.K + BK - 1) / BK;
    auto fetch = [&](int set, int kb) {
        const int k0 = min(kb, nk - 1) * BK;
        tile_load<A_KM, TBM>(ra[set], p.A, p.lda, m0, k0, p.M, p.K, tid);
        tile_load<B_KM>(rb[set], p.B, p.ldb, n0, k0, p.N, p.K, tid);
    };
    auto stash = [&](int set, int buf) {
        tile_store<A_KM, TBM>(At + (size_t)buf * kTileElems, ra[set], tid);
        tile_store<B_KM>(Bt + (size_t)buf * kTileElems, rb[set], tid);
    };
    auto multiply = [&](int buf) {
        const __bf16* Ac = At + (size_t)buf * kTileElems;
        const __bf16* Bc = Bt + (size_t)buf * kTileElems;
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            bf16x8 fa[NI], fb[2];
#pragma unroll
            for (int i = 0; i < NI; ++i) fa[i] = tile_frag<A_KM>(Ac, (TBM / 2) * wm + 32 * i, ks, lane);
#pragma unroll
            for (int j = 0; j < 2; ++j) fb[j] = tile_frag<B_KM>(Bc, 64 * wn + 32 * j, ks, lane);
#pragma unroll
            for (int i = 0; i < NI; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j) M::mma(acc[i][j], fb[j], fa[i]);       // rows = result columns
        }
    };
    fetch(0, 0);
    stash(0, 0);
    fetch(0, 1);
    fetch(1, 2);
    __syncthreads();
    for (int kb = 0; kb < nk; kb += 2) {
        multiply(0);                      // step kb
        stash(0, 1);                      // step kb + 1 (fetched two steps ago)
        fetch(0, kb + 3);
        __syncthreads();
        if (kb + 1 < nk) multiply(1);     // step kb + 1
        stash(1, 0);                      // step kb + 2
        fetch(1, kb + 4);
        __syncthreads();
    }

    // ---------------- epilogue ----------------
    if constexpr (EPI == kEpiFloat) {
        // fp32 result: four consecutive columns of a row per store
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const int row = m0 + (TBM / 2) * wm + 32 * i + r32;
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const int col = n0 + 64 * wn + 32 * j + 8 * c + 4 * g;
                    if (row < p.M)
                        *reinterpret_cast<f32x4*>(p.Cf + (size_t)row * p.ldc + col) =
                            f32x4{acc[i][j][4 * c], acc[i][j][4 * c + 1], acc[i][j][4 * c + 2], acc[i][j][4 * c + 3]};
                }
        }
        return;
    } else {
        // bf16 result(s): bias and activation on the accumulators, then through an LDS tile [256][256]
        // so that rows leave as whole 16-byte vectors.  A column block lies inside one of z, v, q.
        // A second pass does the same for the pre-activation of v when the caller keeps it.
        __bf16* St = reinterpret_cast<__bf16*>(smem);               // the operand tiles are free now (barrier above)
        int which = 0;
        if constexpr (EPI == kEpiProj) which = n0 / p.d;
        const int n_pass = (EPI == kEpiProj && which == 1 && p.av != nullptr) ? 2 : 1;
        for (int pass = 0; pass < n_pass; ++pass) {
#pragma unroll
            for (int i = 0; i < NI; ++i) {
                const int row = 128 * wm + 32 * i + r32;
#pragma unroll
                for (int j = 0; j < 2; ++j)
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        const int col = 64 * wn + 32 * j + 8 * c + 4 * g;
                        float x[4];
#pragma unroll
                        for (int e = 0; e < 4; ++e) x[e] = acc[i][j][4 * c + e];
                        if constexpr (EPI == kEpiProj) {
                            const f32x4 b = *reinterpret_cast<const f32x4*>(p.bias + n0 + col);
#pragma unroll
                            for (int e = 0; e < 4; ++e) {
                                const float a = x[e] + b[e];
                                const float sg = fast_rcp(1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * a));
                                x[e] = (pass == 1 || which == 0) ? a : (which == 1) ? a * sg : sg;
                            }
                        }
                        bf16x4 pk;
#pragma unroll
                        for (int e = 0; e < 4; ++e) pk[e] = (__bf16)x[e];
                        *reinterpret_cast<bf16x4*>(St + (size_t)row * PST + col) = pk;
                    }
            }
            __syncthreads();
            __bf16* out;
            long long ld;
            int c0;
            if constexpr (EPI == kEpiProj) {
                out = (pass == 1) ? p.av : (which == 0) ? p.z : (which == 1) ? p.v : p.q;
                ld = p.d;
                c0 = n0 - which * p.d;
            } else {
                out = p.C; ld = p.ldc; c0 = n0;
            }
            for (int vi = tid; vi < BM * (BN / 8); vi += kGemmThreads) {       // 256 rows x 32 vectors
                const int row = vi >> 5, vc = (vi & 31) * 8;
                if (m0 + row < p.M)
                    *reinterpret_cast<u32x4*>(out + (size_t)(m0 + row) * ld + c0 + vc) =
                        *reinterpret_cast<const u32x4*>(St + (size_t)row * PST + vc);
            }
            __syncthreads();
        }
    }
}

constexpr size_t kGemmLds = (size_t)4 * kTileElems * sizeof(__bf16);
static_assert(kGemmLds <= 160 * 1024, "LDS budget");
static_assert((size_t)BM * PST * sizeof(__bf16) <= kGemmLds, "the staging tile of the epilogue aliases the operand tiles");

template <bool A_KM, bool B_KM, int EPI, int TBM = 256>
static hipError_t launch_gemm(const GemmParams& p, hipStream_t stream)
{
    auto kern = gemm_kernel<A_KM, B_KM, EPI, TBM>;
    hipError_t e = allow_dynamic_lds(reinterpret_cast<const void*>(kern), (int)kGemmLds);
    if (e != hipSuccess) return e;
    const unsigned grid = (unsigned)(((p.M + TBM - 1) / TBM) * (p.N / BN));
    hipLaunchKernelGGL(kern, dim3(grid), dim3(kGemmThreads), kGemmLds, stream, p);
    return hipGetLastError();
}

// ---- the same product for operands that are both k-contiguous, fed by direct global -> LDS loads ----
// (x W3^T of the forward pass; dA W3 of the reverse pass once W3 has been transposed.)  Four waves
// (2 x 2), each owning 128 x 128 of the 256 x 256 tile as 4 x 4 MFMA tiles (an operand fragment read
// from LDS feeds four MFMAs; the accumulators fill the 256 accumulation registers, the wave is
// alone on its SIMD and overlaps its own LDS reads, loads and MFMAs), or eight waves (2 x 4) of
// 128 x 64, two per SIMD (half again as many fragment reads, but a wave's waits and its epilogue
// are covered by its neighbour: the projection with its activation epilogue is 5% faster this way,
// the plain product 4% slower).  K advances in steps of 32
// through FIVE LDS stages that are filled by `global_load_lds` (16 bytes per lane, no registers in
// between) four steps ahead.  Such a load writes the 64 lanes' vectors to consecutive LDS
// addresses, so a tile row is 64 bytes with no padding; bank conflicts are avoided by a swizzle
// instead: the 16-byte piece c of row r is kept at position c ^ ((r >> 2) & 3), which the loading
// lane realises by fetching the piece that belongs at its position, and 16 consecutive rows then
// cover all 64 banks for any piece.  One barrier per step: it ends the reads of the stage that
// is refilled next and publishes the stage that is read next (each wave has waited for its own
// loads of that stage; loads are counted by hand, the compiler does not track them).

constexpr int DBK = 32;                                  // k per stage
constexpr int kDlStages = 5;                            // 5 x 32 KB: all of a compute unit's LDS
constexpr int kDlTileBytes = 256 * DBK * 2;              // one operand's tile of one stage
constexpr int kDlStageBytes = 2 * kDlTileBytes;
constexpr size_t kDlLds = ((size_t)kDlStages * kDlStageBytes > (size_t)BM * PST * sizeof(__bf16))
                              ? (size_t)kDlStages * kDlStageBytes : (size_t)BM * PST * sizeof(__bf16);
static_assert(kDlLds <= 160 * 1024, "LDS budget");
// s_waitcnt with only the vector-memory counter set (gfx9 encoding: vmcnt in bits 3:0 and 15:14)
constexpr int vmcnt_only(int n) { return (n & 15) | ((n >> 4) << 14) | 0x0f70; }

// NWV waves: 4 (2 x 2, each 128 x 128, alone on its SIMD) or 8 (2 x 4, each 128 x 64, two per SIMD,
// which can fill each other's waits).
template <int EPI, int NWV>
__global__ __launch_bounds__(64 * NWV) void gemm_dl_kernel(GemmParams p)
{
    static_assert(NWV == 4 || NWV == 8, "wave layouts: 2 x 2 or 2 x 4");
    constexpr int THREADS = 64 * NWV;
    constexpr int WNG = NWV / 2;                 // waves side by side
    constexpr int TN = BN / WNG, NJ = TN / 32;   // columns of a wave's tile; its 32-column MFMA tiles
    constexpr int LP = 16 / NWV;                 // load pairs (one instruction of A, one of B) per wave and stage
    constexpr int WROWS = 256 / NWV;             // tile rows a wave loads
    typedef Mma<__bf16> M;
    typedef __attribute__((address_space(3))) void* lds_ptr;
    typedef const __attribute__((address_space(1))) void* global_ptr;
    extern __shared__ __align__(16) char smem[];
    const int tid = threadIdx.x, lane = tid & 63, r32 = lane & 31, g = lane >> 5;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = w / WNG, wn = w % WNG;                           // wave tile: rows 128 wm .., columns TN wn ..
    const int n_bn = p.N / BN, n_bm = (p.M + BM - 1) / BM;
    int bm, bn;
    {   // workgroup -> tile, as in gemm_kernel
        const int grid = (int)gridDim.x, id = (int)blockIdx.x;
        const int per = grid / kXcds, rem = grid - per * kXcds, x = id % kXcds;
        const int t = x * per + min(x, rem) + id / kXcds;
        const int band_tiles = kBandRows * n_bn, band = t / band_tiles, in_band = t - band * band_tiles;
        const int rows = min(kBandRows, n_bm - band * kBandRows);
        bn = in_band / rows;
        bm = band * kBandRows + in_band - bn * rows;
    }
    const int m0 = bm * BM, n0 = bn * BN;

    // accumulators, transposed: acc[i][j][v] = C[m0 + 128 wm + 32 i + lane % 32][n0 + TN wn + 32 j + 8 (v/4) + 4 g + v%4]
    f32x16 acc[4][NJ];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    // Loads: instruction j of wave w fills rows WROWS w + 16 j .. + 15 of a tile (1 KB); lane l sits at
    // row l / 4, position l % 4 and fetches piece (l % 4) ^ ((row >> 2) & 3) = (l & 3) ^ ((l >> 4) & 3).
    // Rows past the end of A re-read its last row (never stored).
    const int piece = (lane & 3) ^ ((lane >> 4) & 3);
    const char* ga[LP];
    const char* gb[LP];
#pragma unroll
    for (int j = 0; j < LP; ++j) {
        const int ra = min(m0 + WROWS * w + 16 * j + (lane >> 2), p.M - 1);
        const int rb = n0 + WROWS * w + 16 * j + (lane >> 2);
        ga[j] = reinterpret_cast<const char*>(p.A) + ((size_t)ra * p.lda) * 2 + piece * 16;
        gb[j] = reinterpret_cast<const char*>(p.B) + ((size_t)rb * p.ldb) * 2 + piece * 16;
    }
    const int nk = p.K / DBK;
    // loads j (one of A, one of B) of this wave for stage `stage`, k-step kb
    auto issue_pair = [&](int stage, int kb, int j) {
        const size_t ko = (size_t)min(kb, nk - 1) * (DBK * 2);       // steps past the end fetch the last one again (never read)
        char* sa = smem + stage * kDlStageBytes + w * (WROWS * DBK * 2);
        __builtin_amdgcn_global_load_lds((global_ptr)(ga[j] + ko), (lds_ptr)(sa + j * 1024), 16, 0, 0);
        __builtin_amdgcn_global_load_lds((global_ptr)(gb[j] + ko), (lds_ptr)(sa + kDlTileBytes + j * 1024), 16, 0, 0);
    };
    auto issue = [&](int stage, int kb) {
#pragma unroll
        for (int j = 0; j < LP; ++j) issue_pair(stage, kb, j);
    };
    // fragment of 32 rows x 16 k: lane (r32, g) reads piece 2 kk + g of its row
    const int frag_off0 = r32 * 64 + ((0 + g) ^ ((r32 >> 2) & 3)) * 16;
    const int frag_off1 = r32 * 64 + ((2 + g) ^ ((r32 >> 2) & 3)) * 16;
    // Fragments of k-half kk (16 of the stage's 32 k) of a stage: four of A, NJ of B.
    auto read_frags = [&](bf16x8 (&fa)[4], bf16x8 (&fb)[NJ], int stage, int kk) {
        const char* sa = smem + stage * kDlStageBytes + (128 * wm) * 64 + (kk ? frag_off1 : frag_off0);
        const char* sb = smem + stage * kDlStageBytes + kDlTileBytes + (TN * wn) * 64 + (kk ? frag_off1 : frag_off0);
#pragma unroll
        for (int i = 0; i < 4; ++i) fa[i] = *reinterpret_cast<const bf16x8*>(sa + 32 * i * 64);
#pragma unroll
        for (int j = 0; j < NJ; ++j) fb[j] = *reinterpret_cast<const bf16x8*>(sb + 32 * j * 64);
    };
    // the NM MFMAs of one k-half, in parts: the first kHead of them, then HP segments, each followed
    // by one pair of the stage refill's loads
    constexpr int NM = 4 * NJ, kHead = 2, HP = LP / 2, SEG = (NM - kHead) / HP;
    auto multiply = [&](const bf16x8 (&fa)[4], const bf16x8 (&fb)[NJ], int from, int to) {
#pragma unroll
        for (int t = 0; t < NM; ++t)
            if (t >= from && t < to) M::mma(acc[t / NJ][t % NJ], fb[t % NJ], fa[t / NJ]);   // rows = result columns
    };
    // the rest of a half-step after its first MFMAs: segments of MFMAs, each followed by load pair
    // pair0 + h of stage `stage`, k-step kf
    auto rest_and_refill = [&](const bf16x8 (&fa)[4], const bf16x8 (&fb)[NJ], int stage, int kf, int pair0) {
#pragma unroll
        for (int h = 0; h < HP; ++h) {
            multiply(fa, fb, kHead + h * SEG, h + 1 == HP ? NM : kHead + (h + 1) * SEG);
            __builtin_amdgcn_sched_barrier(0);
            issue_pair(stage, kf, pair0 + h);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // The loop is software-pipelined by hand (the scheduling barriers keep the order).  The compiler
    // waits for ALL outstanding LDS reads before an MFMA that needs any of them (the direct loads
    // make it give up counting), so fragments are requested right after the first MFMAs of the
    // previous batch have been issued: by the time the next batch needs them, the remaining MFMAs of
    // this one have covered the LDS latency, and nothing else is outstanding when the wait comes.
    //   second-half fragments of stage kb   <- during the MFMAs of its first half
    //   first-half fragments of stage kb+1  <- during the MFMAs of the second half of stage kb
    // In between: this wave's loads of stage kb+1 have landed (those of the stages after may be in
    // flight), a barrier publishes stage kb+1 and retires stage kb-1, whose buffer is refilled.
    bf16x8 fa0[4], fb0[NJ], fa1[4], fb1[NJ];
    constexpr int S = kDlStages;
#pragma unroll
    for (int st = 0; st < S - 1; ++st) issue(st, st);
    __builtin_amdgcn_s_waitcnt(vmcnt_only(2 * LP * (S - 2)));    // stage 0 (each stage: 2 LP loads per lane)
    __builtin_amdgcn_s_barrier();
    read_frags(fa0, fb0, 0, 0);
    int s_cur = 0;                                               // kb % S
    for (int kb = 0; kb < nk; ++kb) {
        const int s_next = s_cur + 1 == S ? 0 : s_cur + 1;
        const int s_fill = s_cur == 0 ? S - 1 : s_cur - 1;       // (kb + S - 1) % S: the stage read before this one
        // The refill of a retired stage goes out a pair of loads at a time between the MFMAs, spread
        // over the two half-steps that follow the barrier (a wave that issues its loads in one burst
        // stalls on the full memory queue, and its MFMAs with it): the first half of the pairs behind
        // the barrier of this step, the second half in the first half of the next one.
        multiply(fa0, fb0, 0, kHead);
        __builtin_amdgcn_sched_barrier(0);
        read_frags(fa1, fb1, s_cur, 1);
        __builtin_amdgcn_sched_barrier(0);
        {
            // second half of the refill begun in the step before (first step: stage S - 2 once more)
            const int s_prev = s_fill == 0 ? S - 1 : s_fill - 1, k_prev = kb + S - 2;
            rest_and_refill(fa0, fb0, s_prev, k_prev, HP);
        }
        __builtin_amdgcn_s_waitcnt(vmcnt_only(2 * LP * (S - 3)));   // stage kb + 1 (the S - 3 younger ones may be in flight)
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
        multiply(fa1, fb1, 0, kHead);
        __builtin_amdgcn_sched_barrier(0);
        read_frags(fa0, fb0, s_next, 0);                         // (after the last step: unused)
        __builtin_amdgcn_sched_barrier(0);
        rest_and_refill(fa1, fb1, s_fill, kb + S - 1, 0);
        s_cur = s_next;
    }
    __builtin_amdgcn_s_waitcnt(vmcnt_only(0));           // no load may land in what the epilogue reuses
    __builtin_amdgcn_s_barrier();

    // ---------------- epilogue: as in gemm_kernel, for this wave layout ----------------
    // With one wave per SIMD (NWV = 4) nothing hides the latency of this part, so it does no more than it
    // must: the activation is chosen by a wave-uniform branch around the loops (the gate's block
    // needs none, the second pass of v's block only the bias), and the copy from the staging tile to
    // global memory moves eight vectors per thread at a time.
    __bf16* St = reinterpret_cast<__bf16*>(smem);
    int which = 0;
    if constexpr (EPI == kEpiProj) which = n0 / p.d;
    const int n_pass = (EPI == kEpiProj && which == 1 && p.av != nullptr) ? 2 : 1;
    for (int pass = 0; pass < n_pass; ++pass) {
        // 0: the sum itself (plus bias in the projections); 1: SiLU; 2: sigmoid
        const int mode = (EPI != kEpiProj || pass == 1 || which == 0) ? 0 : which;
        auto stage_tile = [&](auto MODE) {
            constexpr int md = decltype(MODE)::value;
#pragma unroll
            for (int j = 0; j < NJ; ++j)
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const int col = TN * wn + 32 * j + 8 * c + 4 * g;
                    f32x4 b = {0.0f, 0.0f, 0.0f, 0.0f};
                    if constexpr (EPI == kEpiProj) b = *reinterpret_cast<const f32x4*>(p.bias + n0 + col);
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const int row = 128 * wm + 32 * i + r32;
                        bf16x4 pk;
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const float a = acc[i][j][4 * c + e] + b[e];
                            float y = a;
                            if constexpr (md != 0) {
                                const float sg = fast_rcp(1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * a));
                                y = (md == 1) ? a * sg : sg;
                            }
                            pk[e] = (__bf16)y;
                        }
                        *reinterpret_cast<bf16x4*>(St + (size_t)row * PST + col) = pk;
                    }
                }
        };
        if (mode == 0)      stage_tile(std::integral_constant<int, 0>());
        else if (mode == 1) stage_tile(std::integral_constant<int, 1>());
        else                stage_tile(std::integral_constant<int, 2>());
        __syncthreads();
        __bf16* out;
        long long ld;
        int c0;
        if constexpr (EPI == kEpiProj) {
            out = (pass == 1) ? p.av : (which == 0) ? p.z : (which == 1) ? p.v : p.q;
            ld = p.d;
            c0 = n0 - which * p.d;
        } else {
            out = p.C; ld = p.ldc; c0 = n0;
        }
        // 256 rows x 32 vectors of 16 bytes; a wave's 64 lanes cover two whole rows (1 KB contiguous in all)
        constexpr int kBatch = 8;
        for (int v0 = tid; v0 < BM * (BN / 8); v0 += THREADS * kBatch) {
            u32x4 buf[kBatch];
#pragma unroll
            for (int k = 0; k < kBatch; ++k) {
                const int vi = v0 + k * THREADS;
                buf[k] = *reinterpret_cast<const u32x4*>(St + (size_t)(vi >> 5) * PST + (vi & 31) * 8);
            }
#pragma unroll
            for (int k = 0; k < kBatch; ++k) {
                const int vi = v0 + k * THREADS, row = vi >> 5;
                if (m0 + row < p.M) *reinterpret_cast<u32x4*>(out + (size_t)(m0 + row) * ld + c0 + (vi & 31) * 8) = buf[k];
            }
        }
        __syncthreads();
    }
}

template <int EPI, int NWV>
static hipError_t launch_gemm_dl(const GemmParams& p, hipStream_t stream)
{
    auto kern = gemm_dl_kernel<EPI, NWV>;
    hipError_t e = allow_dynamic_lds(reinterpret_cast<const void*>(kern), (int)kDlLds);
    if (e != hipSuccess) return e;
    const unsigned grid = (unsigned)(((p.M + BM - 1) / BM) * (p.N / BN));
    hipLaunchKernelGGL(kern, dim3(grid), dim3(64 * NWV), kDlLds, stream, p);
    return hipGetLastError();
}

// ---- element-wise pass of the reverse mode -------------------------------------------------------
// dA[t][0:d] = dz, dA[t][d:2d] = dv * SiLU'(a_v), dA[t][2d:3d] = dq * q (1 - q); and per block of 128
// rows the column sums of dA (the bias gradients are their sum over the row blocks, in order).
constexpr int kActRows = 128;

__global__ __launch_bounds__(256) void proj_dact_kernel(const __bf16* dz, const __bf16* dv, const __bf16* dq, const __bf16* q,
                                                         const __bf16* av, __bf16* dA, float* partial, int M, int d)
{
    const int col = ((int)blockIdx.x * 256 + (int)threadIdx.x) * 2;       // column pair of [0, 3d)
    if (col >= 3 * d) return;
    const int which = col / d, c = col - which * d;
    const int r0 = (int)blockIdx.y * kActRows, r1 = min(M, r0 + kActRows);
    float s0 = 0.0f, s1 = 0.0f;
    for (int r = r0; r < r1; ++r) {
        const size_t e = (size_t)r * d + c;
        f32x2 g;
        if (which == 0) {
            g = load_pair_t<__bf16>(dz, e);
        } else if (which == 1) {
            const f32x2 u = load_pair_t<__bf16>(dv, e), a = load_pair_t<__bf16>(av, e);
            const float sx = fast_rcp(1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * a.x));
            const float sy = fast_rcp(1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * a.y));
            g.x = u.x * sx * (1.0f + a.x * (1.0f - sx));
            g.y = u.y * sy * (1.0f + a.y * (1.0f - sy));
        } else {
            const f32x2 u = load_pair_t<__bf16>(dq, e), o = load_pair_t<__bf16>(q, e);
            g.x = u.x * o.x * (1.0f - o.x);
            g.y = u.y * o.y * (1.0f - o.y);
        }
        // the sums take the values the products will see (rounded to bf16)
        bf16x2 h;
        h.x = (__bf16)g.x; h.y = (__bf16)g.y;
        *reinterpret_cast<bf16x2*>(dA + (size_t)r * 3 * d + col) = h;
        s0 += (float)h.x; s1 += (float)h.y;
    }
    *reinterpret_cast<f32x2*>(partial + (size_t)blockIdx.y * 3 * d + col) = f32x2{s0, s1};
}

// dst [cols][rows] = src [rows][cols]^T (bf16), 64 x 64 tiles through LDS; rows and cols multiples of 64.
__global__ __launch_bounds__(256) void proj_transpose_kernel(const __bf16* src, __bf16* dst, int rows, int cols)
{
    __shared__ __bf16 tile[64][64 + 2];
    const int r0 = (int)blockIdx.y * 64, c0 = (int)blockIdx.x * 64;
    const int tx = (int)threadIdx.x & 63, ty = (int)threadIdx.x >> 6;
    for (int r = ty; r < 64; r += 4) tile[r][tx] = src[(size_t)(r0 + r) * cols + c0 + tx];
    __syncthreads();
    for (int c = ty; c < 64; c += 4) dst[(size_t)(c0 + c) * rows + r0 + tx] = tile[tx][c];
}

// db[c] = sum over the row blocks of partial[block][c], in a fixed order: 32 columns per workgroup,
// the blocks in eight consecutive slices (one per 32 threads) that are then added in order.
constexpr int kBiasCols = 32, kBiasSlices = 8;

__global__ __launch_bounds__(kBiasCols * kBiasSlices) void proj_bias_grad_kernel(const float* partial, float* db, int n_blocks, int n)
{
    __shared__ float part[kBiasSlices][kBiasCols];
    const int tx = (int)threadIdx.x % kBiasCols, ty = (int)threadIdx.x / kBiasCols;
    const int c = (int)blockIdx.x * kBiasCols + tx;
    const int per = (n_blocks + kBiasSlices - 1) / kBiasSlices;
    const int b0 = ty * per, b1 = min(n_blocks, b0 + per);
    float s = 0.0f;
    if (c < n)
        for (int b = b0; b < b1; ++b) s += partial[(size_t)b * n + c];
    part[ty][tx] = s;
    __syncthreads();
    if (ty == 0 && c < n) {
        float t = 0.0f;
#pragma unroll
        for (int k = 0; k < kBiasSlices; ++k) t += part[k][tx];
        db[c] = t;
    }
}

}   // namespace hgrn2

using namespace hgrn2;

namespace {
int proj_check(int32_t M, int32_t d)
{
    if (M < 0 || d < 0) return HGRN2_ERR_SHAPE;
    if ((long long)M * 3 * d > (long long)INT32_MAX * 8) return HGRN2_ERR_SHAPE;
    if (d % 256 != 0) return HGRN2_ERR_UNSUPPORTED;        // a 256-column block of the product lies inside one of z, v, q
    return HGRN2_OK;
}
size_t round256p(size_t x) { return (x + 255) & ~(size_t)255; }
}   // namespace

extern "C" {

size_t hgru2_proj_bwd_workspace_bytes(int32_t M, int32_t d)
{
    if (proj_check(M, d) != HGRN2_OK) return 0;
    const size_t blocks = ((size_t)M + kActRows - 1) / kActRows;
    return round256p((size_t)M * 3 * d * sizeof(__bf16)) + round256p(blocks * 3 * d * sizeof(float)) +
           round256p((size_t)3 * d * d * sizeof(__bf16));           // dA, row-block sums of dA, W3 transposed
}

int hgru2_proj_fwd(int32_t M, int32_t d, const void* x, const void* w3, const float* b3, void* z, void* v, void* q,
                   void* av, void* hip_stream)
{
    const int rc = proj_check(M, d);
    if (rc != HGRN2_OK) return rc;
    if ((size_t)M * d == 0) return HGRN2_OK;
    if (!x || !w3 || !b3 || !z || !v || !q) return HGRN2_ERR_NULL;
    GemmParams p = {};
    p.A = static_cast<const __bf16*>(x); p.lda = d;
    p.B = static_cast<const __bf16*>(w3); p.ldb = d;
    p.M = M; p.N = 3 * d; p.K = d;
    p.bias = b3; p.z = static_cast<__bf16*>(z); p.v = static_cast<__bf16*>(v); p.q = static_cast<__bf16*>(q);
    p.av = static_cast<__bf16*>(av); p.d = d;
    return launch_gemm_dl<kEpiProj, 8>(p, static_cast<hipStream_t>(hip_stream)) == hipSuccess ? HGRN2_OK : HGRN2_ERR_HIP;
}

int hgru2_proj_bwd(int32_t M, int32_t d, const void* x, const void* w3, const void* q, const void* av, const void* grad_z,
                   const void* grad_v, const void* grad_q, void* grad_x, float* grad_w3, float* grad_b3, void* workspace,
                   size_t workspace_bytes, void* hip_stream)
{
    const int rc = proj_check(M, d);
    if (rc != HGRN2_OK) return rc;
    if (d == 0) return HGRN2_OK;
    if (!grad_w3 || !grad_b3) return HGRN2_ERR_NULL;
    if (M > 0 && (!x || !w3 || !q || !av || !grad_z || !grad_v || !grad_q || !grad_x)) return HGRN2_ERR_NULL;
    const size_t need = hgru2_proj_bwd_workspace_bytes(M, d);
    if (need > 0 && (!workspace || workspace_bytes < need || ((uintptr_t)workspace & 255))) return HGRN2_ERR_WORKSPACE;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if (M == 0) {       // nothing contributes
        if (launch_zero_floats(grad_w3, (size_t)3 * d * d, stream) != hipSuccess ||
            launch_zero_floats(grad_b3, (size_t)3 * d, stream) != hipSuccess)
            return HGRN2_ERR_HIP;
        return HGRN2_OK;
    }
    __bf16* dA = static_cast<__bf16*>(workspace);
    float* partial = reinterpret_cast<float*>(static_cast<char*>(workspace) + round256p((size_t)M * 3 * d * sizeof(__bf16)));
    const int blocks = (M + kActRows - 1) / kActRows;
    hipLaunchKernelGGL(proj_dact_kernel, dim3((3 * d / 2 + 255) / 256, blocks), dim3(256), 0, stream,
                       static_cast<const __bf16*>(grad_z), static_cast<const __bf16*>(grad_v), static_cast<const __bf16*>(grad_q),
                       static_cast<const __bf16*>(q), static_cast<const __bf16*>(av), dA, partial, M, d);
    hipLaunchKernelGGL(proj_bias_grad_kernel, dim3((3 * d + kBiasCols - 1) / kBiasCols), dim3(kBiasCols * kBiasSlices), 0, stream, partial, grad_b3,
                       blocks, 3 * d);
    if (hipGetLastError() != hipSuccess) return HGRN2_ERR_HIP;
    // dx [M][d] = dA [M][3d] . W3 [3d][d]: W3's contraction index is its slow axis, so it is transposed
    // first (25 MB at width 2048, a few microseconds) and the product takes the kernel for k-contiguous operands
    __bf16* w3t = reinterpret_cast<__bf16*>(reinterpret_cast<char*>(partial) + round256p((size_t)blocks * 3 * d * sizeof(float)));
    hipLaunchKernelGGL(proj_transpose_kernel, dim3(d / 64, 3 * d / 64), dim3(256), 0, stream,
                       static_cast<const __bf16*>(w3), w3t, 3 * d, d);
    if (hipGetLastError() != hipSuccess) return HGRN2_ERR_HIP;
    GemmParams px = {};
    px.A = dA; px.lda = 3 * d;
    px.B = w3t; px.ldb = 3 * d;
    px.M = M; px.N = d; px.K = 3 * d;
    px.C = static_cast<__bf16*>(grad_x); px.ldc = d;
    if (launch_gemm_dl<kEpiPlain, 4>(px, stream) != hipSuccess) return HGRN2_ERR_HIP;
    // dW3 [3d][d] = dA^T [3d][M] . x [M][d]: the token index is the slow axis of both
    GemmParams pw = {};
    pw.A = dA; pw.lda = 3 * d;
    pw.B = static_cast<const __bf16*>(x); pw.ldb = d;
    pw.M = 3 * d; pw.N = d; pw.K = M;
    pw.Cf = grad_w3; pw.ldc = d;
    // tile height by the time it implies: rounds of 256 workgroups times the rows of a tile
    const long long t256 = ((3LL * d / 256) * (d / 256) + 255) / 256 * 256, t192 = ((3LL * d / 192) * (d / 256) + 255) / 256 * 192;
    if ((t192 < t256 ? launch_gemm<true, true, kEpiFloat, 192>(pw, stream) : launch_gemm<true, true, kEpiFloat, 256>(pw, stream)) != hipSuccess)
        return HGRN2_ERR_HIP;
    return HGRN2_OK;
}

}   // extern "C"
