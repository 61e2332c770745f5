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
// The matrix kernel: a 256 x 256 tile of the result per workgroup of eight waves (2 x 4, each
// 128 x 64 = 4 x 2 MFMA tiles of 32 x 32), K in steps of 64 through double-buffered LDS tiles
// filled from registers that were loaded two steps ahead.  An operand whose contraction index is
// the slow axis of its array (W3 in dx; both operands in dW3) keeps its natural orientation in LDS
// and is read with LDS transpose loads.  The accumulators are kept transposed (result column in
// the register index), so that four consecutive result columns of a row leave a lane together.
#include "../../include/hgrn2.h"
#include "common.hpp"
#include "kernels.hpp"

namespace hgrn2 {

constexpr int kGemmThreads = 512;
constexpr int BM = 256, BN = 256, BK = 64;
constexpr int PKT = BK + 8;        // pitch of a tile kept [row][k]
constexpr int PXT = 256 + 24;      // pitch of a tile kept [k][row]: transpose reads want rows 12 banks apart
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

template <bool KM>
__device__ __forceinline__ void tile_load(u32x4 (&r)[4], const __bf16* src, long long ld, int row0, int k0, int n_rows, int n_k, int tid)
{
    // 256 x 64 elements = 2048 vectors of 16 bytes, four per thread
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int vi = tid + kGemmThreads * j;
        if constexpr (!KM) {
            const int row = vi >> 3, kc = (vi & 7) * 8;
            const int rc = min(row0 + row, n_rows - 1);          // rows past the end re-read the last one (never stored)
            r[j] = *reinterpret_cast<const u32x4*>(src + (size_t)rc * ld + k0 + kc);
        } else {
            const int kr = vi >> 5, xc = (vi & 31) * 8;
            const int kk = min(k0 + kr, n_k - 1);
            const int xr = min(row0 + xc, n_rows - 8);           // whole vectors stay inside the row (n_rows is a multiple of 8)
            u32x4 x = *reinterpret_cast<const u32x4*>(src + (size_t)kk * ld + xr);
            if (k0 + kr >= n_k) x = u32x4{0u, 0u, 0u, 0u};     // a contraction index past the end contributes nothing
            r[j] = x;
        }
    }
}

template <bool KM>
__device__ __forceinline__ void tile_store(__bf16* tile, const u32x4 (&r)[4], int tid)
{
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int vi = tid + kGemmThreads * j;
        if constexpr (!KM) *reinterpret_cast<u32x4*>(tile + (size_t)(vi >> 3) * PKT + (vi & 7) * 8) = r[j];
        else               *reinterpret_cast<u32x4*>(tile + (size_t)(vi >> 5) * PXT + (vi & 31) * 8) = r[j];
    }
}

template <bool KM>
__device__ __forceinline__ bf16x8 tile_frag(const __bf16* tile, int x0, int ks, int lane)
{
    if constexpr (!KM) return Mma<__bf16>::load(tile + (size_t)(x0 + (lane & 31)) * PKT + 16 * ks + 8 * (lane >> 5));
    else               return Mma<__bf16>::load_kmajor(tile, PXT, 16 * ks, x0, lane);
}

template <bool A_KM, bool B_KM, int EPI>
__global__ __launch_bounds__(kGemmThreads) void gemm_kernel(GemmParams p)
{
    typedef Mma<__bf16> M;
    extern __shared__ __align__(16) char smem[];
    __bf16* At = reinterpret_cast<__bf16*>(smem);                   // [2][tile]
    __bf16* Bt = At + 2 * kTileElems;                               // [2][tile]

    const int tid = threadIdx.x, lane = tid & 63, r32 = lane & 31, g = lane >> 5;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = w >> 2, wn = w & 3;                              // wave tile: rows 128 wm .., columns 64 wn ..
    // Workgroup -> tile.  Workgroup ids go round the eight XCDs (id % 8), each with an L2 of its
    // own, so the ids are first renumbered so that an XCD holds a contiguous range, and the range is
    // laid over the tile grid in bands of kBandRows row blocks walked column by column: the 32
    // workgroups an XCD runs together then cover about 4 x 8 tiles and share their operand panels
    // in that XCD's L2 instead of each XCD streaming whole panels of its own.
    const int n_bn = p.N / BN, n_bm = (p.M + BM - 1) / BM;
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
    const int m0 = bm * BM, n0 = bn * BN;

    // accumulators, transposed: acc[i][j][v] = C[m0 + 128 wm + 32 i + lane % 32][n0 + 64 wn + 32 j + 8 (v/4) + 4 g + v%4]
    f32x16 acc[4][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
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
        tile_load<A_KM>(ra[set], p.A, p.lda, m0, k0, p.M, p.K, tid);
        tile_load<B_KM>(rb[set], p.B, p.ldb, n0, k0, p.N, p.K, tid);
    };
    auto stash = [&](int set, int buf) {
        tile_store<A_KM>(At + (size_t)buf * kTileElems, ra[set], tid);
        tile_store<B_KM>(Bt + (size_t)buf * kTileElems, rb[set], tid);
    };
    auto multiply = [&](int buf) {
        const __bf16* Ac = At + (size_t)buf * kTileElems;
        const __bf16* Bc = Bt + (size_t)buf * kTileElems;
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            bf16x8 fa[4], fb[2];
#pragma unroll
            for (int i = 0; i < 4; ++i) fa[i] = tile_frag<A_KM>(Ac, 128 * wm + 32 * i, ks, lane);
#pragma unroll
            for (int j = 0; j < 2; ++j) fb[j] = tile_frag<B_KM>(Bc, 64 * wn + 32 * j, ks, lane);
#pragma unroll
            for (int i = 0; i < 4; ++i)
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
        for (int i = 0; i < 4; ++i) {
            const int row = m0 + 128 * wm + 32 * i + r32;
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
            for (int i = 0; i < 4; ++i) {
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

template <bool A_KM, bool B_KM, int EPI>
static hipError_t launch_gemm(const GemmParams& p, hipStream_t stream)
{
    auto kern = gemm_kernel<A_KM, B_KM, EPI>;
    hipError_t e = allow_dynamic_lds(reinterpret_cast<const void*>(kern), (int)kGemmLds);
    if (e != hipSuccess) return e;
    const unsigned grid = (unsigned)(((p.M + BM - 1) / BM) * (p.N / BN));
    hipLaunchKernelGGL(kern, dim3(grid), dim3(kGemmThreads), kGemmLds, stream, p);
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

__global__ void proj_bias_grad_kernel(const float* partial, float* db, int n_blocks, int n)
{
    const int c = (int)blockIdx.x * (int)blockDim.x + (int)threadIdx.x;
    if (c >= n) return;
    float s = 0.0f;
    for (int b = 0; b < n_blocks; ++b) s += partial[(size_t)b * n + c];
    db[c] = s;
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
    return round256p((size_t)M * 3 * d * sizeof(__bf16)) + round256p(blocks * 3 * d * sizeof(float));
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
    return launch_gemm<false, false, kEpiProj>(p, static_cast<hipStream_t>(hip_stream)) == hipSuccess ? HGRN2_OK : HGRN2_ERR_HIP;
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
    hipLaunchKernelGGL(proj_bias_grad_kernel, dim3((3 * d + 255) / 256), dim3(256), 0, stream, partial, grad_b3, blocks, 3 * d);
    if (hipGetLastError() != hipSuccess) return HGRN2_ERR_HIP;
    // dx [M][d] = dA [M][3d] . W3 [3d][d]: W3's contraction index is its slow axis
    GemmParams px = {};
    px.A = dA; px.lda = 3 * d;
    px.B = static_cast<const __bf16*>(w3); px.ldb = d;
    px.M = M; px.N = d; px.K = 3 * d;
    px.C = static_cast<__bf16*>(grad_x); px.ldc = d;
    if (launch_gemm<false, true, kEpiPlain>(px, stream) != hipSuccess) return HGRN2_ERR_HIP;
    // dW3 [3d][d] = dA^T [3d][M] . x [M][d]: the token index is the slow axis of both
    GemmParams pw = {};
    pw.A = dA; pw.lda = 3 * d;
    pw.B = static_cast<const __bf16*>(x); pw.ldb = d;
    pw.M = 3 * d; pw.N = d; pw.K = M;
    pw.Cf = grad_w3; pw.ldc = d;
    if (launch_gemm<true, true, kEpiFloat>(pw, stream) != hipSuccess) return HGRN2_ERR_HIP;
    return HGRN2_OK;
}

}   // extern "C"
