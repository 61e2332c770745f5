// Per-chunk gradients of the chunkwise HGRN2 recurrence (reverse mode of paper Section 3.2,
// Eq. 3; the paper gives no backward algorithm).  For one chunk of C tokens with incoming state
// S_n and outgoing state gradient dS_{n+1} (both produced by the state sweeps), and with
// P = tril(Q~ K~^T), dP = tril(dO V^T) (diagonal kept, decays factored around the row C/2):
//
//   dq_i = sq_i * ( dP K~           + G_m  * dO S_n^T    )_i       sq = Q~/q
//   dk_j = sk_j * ( dP^T Q~         + H_m  * V dS_{n+1}^T )_j       sk = K~/k,  H_m = g / G_m
//   dv_j =        ( P^T dO          + K~ (H_m * dS_{n+1}) )_j       since k g/G = K~ H_m
//   dL_i = q_i dq_i - k_i dk_i                                      gradient w.r.t. log G_i
//   dg_s = sum_{i>=s in chunk} dL_i + R ,   R = rowsum(dS_{n+1} * S_{n+1})   (chunk-local form)
//   df_s = dg_s / f_s - dk_s                                        tied gate k = 1 - f
//
// G_m is the gate product of the first half of the chunk and g of the whole chunk.  In exact
// arithmetic every pair (i, j) with both tokens at or after s drops out of dg_s, and what is
// left carries a factor f_s; a small gate would otherwise amplify the rounding noise of the
// cancelled pairs by 1/f_s.  dg_s is therefore assembled as
//   dg_s = sum_{i>=s} ( Q~_i (dP K~)_i - K~_i (dP^T Q~)_i )      pair terms, with the SAME rounded
//                                                                  operands the MFMAs consumed, so
//                                                                  that they cancel to fp32 accuracy
//        + sum_{i>=s} q_i G_i (dO S_n^T)_i                        read-out of the incoming state
//        + sum_{j<s}  k_j (g/G_j) (V dS_{n+1}^T)_j                (R minus the suffix of the same terms)
//        + g * rowsum(dS_{n+1} * S_n)
// in which no term cancels against another.
//
// One workgroup of eight wave64s per chunk (two waves per SIMD, so that LDS and MFMA latencies of
// one wave are covered by the other).  Wave w owns rows 8w..8w+7 of the chunk for the
// element-wise stages, the 32x32 tile (row tile w / NAT, channel tile w % NAT) of the 64 x dk
// gradients -- the contraction over dv is complete inside the wave and the states arrive
// straight from global memory as operand fragments -- and one 32x32 tile of dv.  Operands whose
// contraction index is the slow axis of their LDS tile are fetched with LDS transpose reads.
// The final element-wise stage runs in the row-block / channel-pair layout after the
// accumulators have been staged through LDS.
#include "common.hpp"
#include "kernels.hpp"

namespace hgrn2 {

constexpr int kBwdWaves = 8;
constexpr int kBwdThreads = 64 * kBwdWaves;

struct BwdGradParams {
    const void* q;
    const void* f;
    const void* v;
    const void* dO;
    const void* ws_s;
    const void* ws_ds;
    void* dq;
    void* df;
    void* dv;
    int BH, N, NC, gate_bf16;
#ifdef HGRN2_PHASE_TIMING
    long long* dbg;      // [workgroup][wave][24] clock ticks per phase (diagnostic builds only)
#endif
};

#ifdef HGRN2_PHASE_TIMING
#define HGRN2_STAMP(k) do { const long long t_now = wall_clock64(); ph[k] = t_now - t_prev; t_prev = t_now; } while (0)
#else
#define HGRN2_STAMP(k) do { } while (0)
#endif

template <typename T, int DK, int DV> struct BwdGradLds {
    static constexpr int C = kChunk;
    // Tiles that are also read with LDS transpose loads (Q~, K~, dO, dS) take a pitch of D + 24
    // elements: row-major 16-byte reads stay conflict-free and the transpose reads run at twice
    // the rate they reach at D + 8.  V and the dv staging tile are only read row-major.
    static constexpr int PK = DK + 3 * pad_elems<T>();  // pitch of the Q~, K~ tiles [C][DK]
    static constexpr int PV = DV + 3 * pad_elems<T>();  // pitch of the dO tile [C][DV] and of dS [DK][DV]
    static constexpr int PVR = DV + pad_elems<T>();     // pitch of the V tile and of the dv staging tile
    static constexpr int PC = C + pad_elems<T>();       // pitch of [C][C] tiles
    static constexpr int PF = DK + 4;                   // pitch of fp32 staging [C][DK]
    // phase 1: operand tiles
    static constexpr size_t qm = 0;                                         // Q~   [C][PK]
    static constexpr size_t km = qm + (size_t)C * PK * sizeof(T);           // K~   [C][PK]
    static constexpr size_t vm = km + (size_t)C * PK * sizeof(T);           // V    [C][PVR]
    static constexpr size_t dom = vm + (size_t)C * PVR * sizeof(T);         // dO   [C][PV]
    static constexpr size_t dsm = dom + (size_t)C * PV * sizeof(T);         // H_m * dS  [DK][PV]
    static constexpr size_t pt = dsm + (size_t)DK * PV * sizeof(T);         // P^T  [C][PC]  ([j][i])
    static constexpr size_t dpt = pt + (size_t)C * PC * sizeof(T);          // dP^T [C][PC]
    static constexpr size_t tot = dpt + (size_t)C * PC * sizeof(T);         // [8][DK] fp32 block products
    static constexpr size_t rp = tot + (size_t)kBwdWaves * DK * sizeof(float);   // [DK] fp32  g * rowsum(dS * S_n)
    static constexpr size_t blk = rp + (size_t)DK * sizeof(float);               // [8][DK] fp32 block sums of e
    static constexpr size_t ys = blk + (size_t)kBwdWaves * DK * sizeof(float);   // [2][DK] fp32 column sums per row tile
    static constexpr size_t dvs = ys + (size_t)2 * DK * sizeof(float);           // dv staging [C][PV]
    static constexpr size_t total = dvs + (size_t)C * PVR * sizeof(T);
    static_assert(total <= 160 * 1024, "LDS budget of one workgroup");
    // phase 2 (aliases the operand tiles): fp32 staging of X and Y
    static constexpr size_t cq = 0;                                         // [C][PF] fp32
    static constexpr size_t ck = cq + (size_t)C * PF * sizeof(float);       // [C][PF] fp32
    static_assert(ck + (size_t)C * PF * sizeof(float) <= tot, "staging must fit in the operand and P tiles");
};

template <typename T, int DK, int DV>
__global__ __launch_bounds__(kBwdThreads) void bwd_grad_kernel(BwdGradParams p)
{
    constexpr int C = kChunk, NW = kBwdWaves, RW = C / NW;
    typedef BwdGradLds<T, DK, DV> L;
    constexpr int PK = L::PK, PV = L::PV, PVR = L::PVR, PC = L::PC, PF = L::PF;
    constexpr int NRT = C / 32, NAT = DK / 32, NBT = DV / 32;
    static_assert(NRT == 2 && NRT * NAT <= NW && NRT * NBT <= NW, "one tile per wave");
    typedef Mma<T> M;
    typedef typename M::frag frag;

    extern __shared__ __align__(16) char smem[];
    T* Qm = reinterpret_cast<T*>(smem + L::qm);
    T* Km = reinterpret_cast<T*>(smem + L::km);
    T* Vm = reinterpret_cast<T*>(smem + L::vm);
    T* dOm = reinterpret_cast<T*>(smem + L::dom);
    T* dSm = reinterpret_cast<T*>(smem + L::dsm);
    T* Pt = reinterpret_cast<T*>(smem + L::pt);
    T* dPt = reinterpret_cast<T*>(smem + L::dpt);
    float* tot = reinterpret_cast<float*>(smem + L::tot);
    float* Rp = reinterpret_cast<float*>(smem + L::rp);
    float* blkE = reinterpret_cast<float*>(smem + L::blk);     // [8][DK] block sums of e
    float* Ys = reinterpret_cast<float*>(smem + L::ys);       // [2][DK]
    float* cQ = reinterpret_cast<float*>(smem + L::cq);
    float* cK = reinterpret_cast<float*>(smem + L::ck);
    T* dVs = reinterpret_cast<T*>(smem + L::dvs);

    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, r32 = lane & 31, g = lane >> 5;
    const bool k_act = 2 * lane < DK, v_act = 2 * lane < DV;
    const bool gate_bf16 = p.gate_bf16 != 0;
    const T* qg = static_cast<const T*>(p.q);
    const T* vg = static_cast<const T*>(p.v);
    const T* dog = static_cast<const T*>(p.dO);
    const int col_k = k_act ? 2 * lane : 0, col_v = v_act ? 2 * lane : 0;

    // tile ownership (a wave without a tile of a kind skips that work)
    const bool has_a = w < NRT * NAT, has_b = w < NRT * NBT;
    const int rt_a = has_a ? w / NAT : 0, at = w % NAT;     // (row tile, channel tile) of dq / dk
    const int rt_b = has_b ? w / NBT : 0, bt = w % NBT;     // (row tile, column tile) of dv

    // Everything one chunk needs from global memory: the raw rows of f, q, v, dO of this wave's row
    // block and the state fragments of channel tile `at` (operand B[k = dv index][n = channel]).
    // The workgroup is persistent: it walks the chunks blockIdx.x, blockIdx.x + gridDim.x, ... and
    // issues the row loads of its next chunk as soon as the matrix stage of the current one is
    // done, so that they fly during the element-wise epilogue; the state fragments are requested
    // at the top of a chunk and are not needed before its own element-wise stage is over.
    auto load_chunk_rows = [&](RawRows<RW>& cf, RawRows<RW>& cq, RawRows<RW>& cv, RawRows<RW>& cdo, int chunk) {
        const int cn = chunk % p.NC, cbh = chunk / p.NC;
        const size_t sk_ = (size_t)cbh * p.N * DK, sv_ = (size_t)cbh * p.N * DV;
        const int r0 = cn * C + RW * w;
        load_rows<RW>(cf, p.f, sk_, DK, col_k, r0, p.N, gate_bf16);
        load_rows<RW>(cq, qg, sk_, DK, col_k, r0, p.N, is_bf16_type<T>());
        load_rows<RW>(cv, vg, sv_, DV, col_v, r0, p.N, is_bf16_type<T>());
        load_rows<RW>(cdo, dog, sv_, DV, col_v, r0, p.N, is_bf16_type<T>());
    };
    auto load_chunk_states = [&](frag (&cS)[2 * NBT], frag (&cD)[2 * NBT], int chunk) {
        const size_t slot = (size_t)chunk * DK * DV;
        const T* wsS = static_cast<const T*>(p.ws_s) + slot;
        const T* wsD = static_cast<const T*>(p.ws_ds) + slot;
#pragma unroll
        for (int kk = 0; kk < 2 * NBT; ++kk) {
            cS[kk] = *reinterpret_cast<const frag*>(wsS + state_frag_offset(at, kk >> 1, NBT, kk & 1, lane));
            cD[kk] = *reinterpret_cast<const frag*>(wsD + state_frag_offset(at, kk >> 1, NBT, kk & 1, lane));
        }
    };

    const int n_chunks = p.BH * p.NC;
    RawRows<RW> raw_f, raw_q, raw_v, raw_d;
    frag sS[2 * NBT], sD[2 * NBT];
    if ((int)blockIdx.x < n_chunks) load_chunk_rows(raw_f, raw_q, raw_v, raw_d, blockIdx.x);

  for (int chunk = blockIdx.x; chunk < n_chunks; chunk += gridDim.x) {
    // Re-derive the lane-dependent indices inside the loop from a value the compiler cannot see
    // through: otherwise it hoists dozens of loop-invariant LDS addresses out of the loop, keeps
    // them in registers across the whole body and spills.
    int lane_opaque = threadIdx.x & 63;
    asm volatile("" : "+v"(lane_opaque));
    const int lane = lane_opaque, r32 = lane & 31, g = lane >> 5;
    const int n = chunk % p.NC, bh = chunk / p.NC;
    const size_t seq_k = (size_t)bh * p.N * DK, seq_v = (size_t)bh * p.N * DV;
    load_chunk_states(sS, sD, chunk);      // first needed two barriers from here; covered by the element-wise stage

#ifdef HGRN2_PHASE_TIMING
    long long ph[24] = {0};
    long long t_prev = wall_clock64();
#endif
    // rf/rq are re-derived from the raw rows in the epilogue (the raw bf16 pairs cost half the registers)
    const int row0 = n * C + RW * w;
    f32x2 rf[RW], rq[RW];
    {
        f32x2 rv[RW], rd[RW];
        convert_rows<RW>(rf, raw_f, row0, p.N, k_act, gate_bf16, 1.0f);
        convert_rows<RW>(rq, raw_q, row0, p.N, k_act, is_bf16_type<T>(), 0.0f);
        convert_rows<RW>(rv, raw_v, row0, p.N, v_act, is_bf16_type<T>(), 0.0f);
        convert_rows<RW>(rd, raw_d, row0, p.N, v_act, is_bf16_type<T>(), 0.0f);
        if (v_act) {
#pragma unroll
            for (int i = 0; i < RW; ++i) {
                store_pair_t<T>(Vm, (size_t)(RW * w + i) * PVR + 2 * lane, rv[i].x, rv[i].y);
                store_pair_t<T>(dOm, (size_t)(RW * w + i) * PV + 2 * lane, rd[i].x, rd[i].y);
            }
        }
    }

    // ---------------- gate products; scaled operand tiles ----------------
    // pr = product of the gates between each row and the block edge that faces the reference row
    // (rows after the reference: from the block start up to the row; rows before: after the row
    // up to the block end); sq/sk are kept for the epilogue: dq = sq * (...), dk = sk * (...)
    float mm0[RW], mm1[RW];
    // sq = Q~/q and sk = K~/k from m: rows after the reference carry m on the q side, rows before on the k side
    auto scales = [&](float m0, float m1, float& sq0, float& sq1, float& sk0, float& sk1) {
        const float i0 = fast_rcp(fmaxf(m0, kTinyProduct)), i1 = fast_rcp(fmaxf(m1, kTinyProduct));
        if (w >= NW / 2) { sq0 = m0; sq1 = m1; sk0 = i0; sk1 = i1; }
        else             { sk0 = m0; sk1 = m1; sq0 = i0; sq1 = i1; }
    };
    {
        float pr0[RW], pr1[RW], t0 = 1.0f, t1 = 1.0f;
        if (w >= NW / 2) {
#pragma unroll
            for (int i = 0; i < RW; ++i) { t0 *= rf[i].x; t1 *= rf[i].y; pr0[i] = t0; pr1[i] = t1; }
        } else {
#pragma unroll
            for (int i = RW - 1; i >= 0; --i) { pr0[i] = t0; pr1[i] = t1; t0 *= rf[i].x; t1 *= rf[i].y; }
        }
        if (k_act) {
            tot[w * DK + 2 * lane] = t0;
            tot[w * DK + 2 * lane + 1] = t1;
        }
        HGRN2_STAMP(0);
        __syncthreads();
        HGRN2_STAMP(1);
        if (k_act) {
            // product of the block totals between this block and the reference row
            float mid0 = 1.0f, mid1 = 1.0f;
#pragma unroll
            for (int i = 0; i < NW; ++i) {
                const bool between = (w >= NW / 2) ? (i >= NW / 2 && i < w) : (i > w && i < NW / 2);
                mid0 *= between ? tot[i * DK + 2 * lane] : 1.0f;
                mid1 *= between ? tot[i * DK + 2 * lane + 1] : 1.0f;
            }
#pragma unroll
            for (int i = 0; i < RW; ++i) {
                const int row = RW * w + i;
                mm0[i] = mid0 * pr0[i]; mm1[i] = mid1 * pr1[i];
                float sq0, sq1, sk0, sk1;
                scales(mm0[i], mm1[i], sq0, sq1, sk0, sk1);
                store_pair_t<T>(Qm, (size_t)row * PK + 2 * lane, rq[i].x * sq0, rq[i].y * sq1);
                store_pair_t<T>(Km, (size_t)row * PK + 2 * lane, (1.0f - rf[i].x) * sk0, (1.0f - rf[i].y) * sk1);
            }
        } else {
#pragma unroll
            for (int i = 0; i < RW; ++i) { mm0[i] = 1.0f; mm1[i] = 1.0f; }
        }
    }
    // H_m * dS_{n+1} of channel tile `at` -> LDS, row-major [channel][dv index] (the fragments hold
    // it already scaled and rounded: their bits go to LDS as they are), and
    // R = rowsum((H_m dS) * (G_m S_n)) = g * rowsum(dS * S_n).  Once per channel tile (row tile 0).
    if (w < NAT) {
        const int ch = 32 * at + r32;
        float rs = 0.0f;
#pragma unroll
        for (int kk = 0; kk < 2 * NBT; ++kk) {
            T* row = dSm + (size_t)ch * PV + 16 * kk + 4 * g;
#pragma unroll
            for (int s = 0; s < 8; ++s) rs += M::get(sS[kk], s) * M::get(sD[kk], s);
            float x[8];
#pragma unroll
            for (int s = 0; s < 8; ++s) x[s] = M::get(sD[kk], s);
            store_pair_t<T>(row, 0, x[0], x[1]);
            store_pair_t<T>(row, 2, x[2], x[3]);
            store_pair_t<T>(row, 8, x[4], x[5]);
            store_pair_t<T>(row, 10, x[6], x[7]);
        }
        rs += __shfl_xor(rs, 32);
        if (g == 0) Rp[ch] = rs;
    }
    HGRN2_STAMP(2);
    __syncthreads();
    HGRN2_STAMP(3);

    // ---------------- P^T and dP^T blocks ----------------
    // waves 0..2: P blocks (I,J) = (0,0), (1,0), (1,1); waves 3..5: the same for dP; waves 6, 7 zero
    // the never-computed block (rows j >= 32, columns i < 32) so that every later contraction can
    // run over the full chunk without reading stale data.
    if (w < 6) {
        const bool is_dp = w >= 3;
        const int b = is_dp ? w - 3 : w;
        const int I = (b == 0) ? 0 : 1, J = (b == 2) ? 1 : 0;
        f32x16 acc0, acc1;
#pragma unroll
        for (int v = 0; v < 16; ++v) { acc0[v] = 0.0f; acc1[v] = 0.0f; }
        if (is_dp) {
#pragma unroll
            for (int ks = 0; ks < DV / 16; ks += 2) {
                M::mma(acc0, M::load(dOm + (32 * I + r32) * PV + 16 * ks + 8 * g),
                       M::load(Vm + (32 * J + r32) * PVR + 16 * ks + 8 * g));
                M::mma(acc1, M::load(dOm + (32 * I + r32) * PV + 16 * (ks + 1) + 8 * g),
                       M::load(Vm + (32 * J + r32) * PVR + 16 * (ks + 1) + 8 * g));
            }
        } else {
#pragma unroll
            for (int ks = 0; ks < DK / 16; ks += 2) {
                M::mma(acc0, M::load(Qm + (32 * I + r32) * PK + 16 * ks + 8 * g),
                       M::load(Km + (32 * J + r32) * PK + 16 * ks + 8 * g));
                M::mma(acc1, M::load(Qm + (32 * I + r32) * PK + 16 * (ks + 1) + 8 * g),
                       M::load(Km + (32 * J + r32) * PK + 16 * (ks + 1) + 8 * g));
            }
        }
        // acc[row i][col j]; keep j <= i; store transposed: dst[j][i .. i+3]
        T* dst = is_dp ? dPt : Pt;
        const int j_glob = 32 * J + r32;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int i0 = 32 * I + 8 * c + 4 * g;
            float x[4];
#pragma unroll
            for (int ii = 0; ii < 4; ++ii) x[ii] = (j_glob <= i0 + ii) ? acc0[4 * c + ii] + acc1[4 * c + ii] : 0.0f;
            store_pair_t<T>(dst, (size_t)j_glob * PC + i0, x[0], x[1]);
            store_pair_t<T>(dst, (size_t)j_glob * PC + i0 + 2, x[2], x[3]);
        }
    } else {
        T* dst = (w == 6) ? Pt : dPt;
#pragma unroll
        for (int c = 0; c < 8; ++c)      // rows 32..63, columns 0..31: 32 x 32 values, 16 per lane
            store_pair_t<T>(dst, (size_t)(32 + (lane >> 1)) * PC + 16 * (lane & 1) + 2 * c, 0.0f, 0.0f);
    }
    HGRN2_STAMP(4);
    __syncthreads();
    HGRN2_STAMP(5);

    // ---------------- main contractions ----------------
    // dv tile (rt_b, bt) first: P^T dO over the chunk and K~ (H_m dS) over the channels (the masked
    // halves of P^T / dP^T are zero, so every contraction runs over the full chunk with no
    // branches).  It goes to its staging area at once, which frees its registers.
    if (has_b) {
        f32x16 aV, aV2;
#pragma unroll
        for (int v = 0; v < 16; ++v) { aV[v] = 0.0f; aV2[v] = 0.0f; }
#pragma unroll
        for (int ks = 0; ks < 2 * NRT; ++ks)
            M::mma(aV2, M::load(Pt + (32 * rt_b + r32) * PC + 16 * ks + 8 * g), M::load_kmajor(dOm, PV, 16 * ks, 32 * bt, lane));
#pragma unroll
        for (int ks = 0; ks < DK / 16; ++ks)
            M::mma(aV, M::load(Km + (32 * rt_b + r32) * PK + 16 * ks + 8 * g), M::load_kmajor(dSm, PV, 16 * ks, 32 * bt, lane));
#pragma unroll
        for (int v = 0; v < 16; ++v)
            dVs[(size_t)(32 * rt_b + acc_row(v, lane)) * PVR + 32 * bt + r32] = (T)(aV[v] + aV2[v]);
    }
    // tile (rt_a, at):  X = dP K~ + dO (G_m S_n)^T,  Y = dP^T Q~ + V (H_m dS)^T.  The second part of Y
    // is accumulated on its own first, because sum_j K~_j * (V (H_m dS)^T)_j over ALL rows of the chunk
    // (the R-like term of the gate gradient, see the epilogue) is taken from it.
    f32x16 aX, aY;
#pragma unroll
    for (int v = 0; v < 16; ++v) { aX[v] = 0.0f; aY[v] = 0.0f; }
    if (has_a) {
        f32x16 aKs;
#pragma unroll
        for (int v = 0; v < 16; ++v) aKs[v] = 0.0f;
#pragma unroll
        for (int kk = 0; kk < 2 * NBT; ++kk) {
            const T* drow = dOm + (32 * rt_a + r32) * PV + 16 * kk + 4 * g;
            const T* vrow = Vm + (32 * rt_a + r32) * PVR + 16 * kk + 4 * g;
            M::mma(aX, M::load2(drow, drow + 8), sS[kk]);
            M::mma(aKs, M::load2(vrow, vrow + 8), sD[kk]);
        }
        float ys = 0.0f;
#pragma unroll
        for (int v = 0; v < 16; ++v)
            ys += (float)Km[(size_t)(32 * rt_a + acc_row(v, lane)) * PK + 32 * at + r32] * aKs[v];
        ys += __shfl_xor(ys, 32);
        if (g == 0) Ys[rt_a * DK + 32 * at + r32] = ys;
#pragma unroll
        for (int ks = 0; ks < 2 * NRT; ++ks) {
            M::mma(aX, M::load_kmajor(dPt, PC, 16 * ks, 32 * rt_a, lane), M::load_kmajor(Km, PK, 16 * ks, 32 * at, lane));
            M::mma(aY, M::load(dPt + (32 * rt_a + r32) * PC + 16 * ks + 8 * g), M::load_kmajor(Qm, PK, 16 * ks, 32 * at, lane));
        }
#pragma unroll
        for (int v = 0; v < 16; ++v) aY[v] += aKs[v];
    }
    // next chunk of this workgroup: its row loads are in flight during the staging / epilogue below
    // (and this chunk's own f, q rows again, for the epilogue: re-reading 8 cached rows is cheaper
    // than holding them in registers across the matrix stage)
    RawRows<RW> nxt_f, nxt_q;
    const bool has_next = chunk + (int)gridDim.x < n_chunks;
    load_rows<RW>(raw_f, p.f, seq_k, DK, col_k, row0, p.N, gate_bf16);
    load_rows<RW>(raw_q, qg, seq_k, DK, col_k, row0, p.N, is_bf16_type<T>());
    if (has_next) load_chunk_rows(nxt_f, nxt_q, raw_v, raw_d, chunk + gridDim.x);   // v, dO of this chunk are dead
    HGRN2_STAMP(6);
    __syncthreads();     // every wave is done with the operand tiles
    HGRN2_STAMP(7);

    // ---------------- staging: X, Y as [row][channel] fp32 ----------------
    if (has_a) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const size_t o = (size_t)(32 * rt_a + acc_row(v, lane)) * PF + 32 * at + r32;
            cQ[o] = aX[v];
            cK[o] = aY[v];
        }
    }
    HGRN2_STAMP(8);
    __syncthreads();
    HGRN2_STAMP(9);

    // ---------------- element-wise epilogue in the row-block / channel-pair layout ----------------
    //   dq = sq X,  dk = sk Y,  e = bf16(Q~) X - bf16(K~) Y   (with the values the MFMAs consumed)
    //   dg_s = sum_{i >= s in chunk} e_i + sum_{all j in chunk} K~_j (V (H_m dS)^T)_j + R
    // In e the pair terms of X and Y cancel to fp32 accuracy; the outgoing-state part of Y that e
    // subtracts for rows >= s is added back for ALL rows from the very same products, so what remains
    // of it is the exact prefix over j < s (see the header comment).
    float e0[RW], e1[RW], dk0[RW], dk1[RW];
    T* dqg = static_cast<T*>(p.dq);
    T* dfg = static_cast<T*>(p.df);
    convert_rows<RW>(rf, raw_f, row0, p.N, k_act, gate_bf16, 1.0f);
    convert_rows<RW>(rq, raw_q, row0, p.N, k_act, is_bf16_type<T>(), 0.0f);
    if (k_act) {
        float se0 = 0.0f, se1 = 0.0f;
#pragma unroll
        for (int i = RW - 1; i >= 0; --i) {
            const int row = RW * w + i;
            const f32x2 xq = *reinterpret_cast<const f32x2*>(cQ + (size_t)row * PF + 2 * lane);
            const f32x2 xk = *reinterpret_cast<const f32x2*>(cK + (size_t)row * PF + 2 * lane);
            float sq0, sq1, sk0, sk1;
            scales(mm0[i], mm1[i], sq0, sq1, sk0, sk1);
            const float qs0 = rq[i].x * sq0, qs1 = rq[i].y * sq1;                       // exactly what went into Q~
            const float ks0 = (1.0f - rf[i].x) * sk0, ks1 = (1.0f - rf[i].y) * sk1;     // ... and into K~
            dk0[i] = sk0 * xk.x; dk1[i] = sk1 * xk.y;
            se0 += (float)(T)qs0 * xq.x - (float)(T)ks0 * xk.x;
            se1 += (float)(T)qs1 * xq.y - (float)(T)ks1 * xk.y;
            e0[i] = se0; e1[i] = se1;                                                   // inclusive suffix inside the block
            const int grow = n * C + row;
            if (grow < p.N) store_pair_t<T>(dqg, seq_k + (size_t)grow * DK + 2 * lane, sq0 * xq.x, sq1 * xq.y);
        }
        blkE[w * DK + 2 * lane] = se0; blkE[w * DK + 2 * lane + 1] = se1;
    }
    // coalesced store of dv
    {
        constexpr int VEC = 16 / (int)sizeof(T);
        constexpr int VPR = DV / VEC;
        T* dvg = static_cast<T*>(p.dv);
        for (int idx = tid; idx < C * VPR; idx += kBwdThreads) {
            const int row = idx / VPR, cv = idx % VPR;
            const int grow = n * C + row;
            if (grow < p.N) {
                const uint4 val = *reinterpret_cast<const uint4*>(dVs + (size_t)row * PVR + cv * VEC);
                *reinterpret_cast<uint4*>(dvg + seq_v + (size_t)grow * DV + cv * VEC) = val;
            }
        }
    }
    HGRN2_STAMP(10);
    __syncthreads();
    HGRN2_STAMP(12);
    if (k_act) {
        const int c0 = 2 * lane, c1 = 2 * lane + 1;
        float add0 = Rp[c0] + Ys[c0] + Ys[DK + c0], add1 = Rp[c1] + Ys[c1] + Ys[DK + c1];
#pragma unroll
        for (int ww = 0; ww < NW; ++ww) {
            add0 += (ww > w) ? blkE[ww * DK + c0] : 0.0f;
            add1 += (ww > w) ? blkE[ww * DK + c1] : 0.0f;
        }
#pragma unroll
        for (int i = 0; i < RW; ++i) {
            const int grow = n * C + RW * w + i;
            if (grow < p.N) {
                const float df0 = (e0[i] + add0) * fast_rcp(fmaxf(rf[i].x, 1e-30f)) - dk0[i];
                const float df1 = (e1[i] + add1) * fast_rcp(fmaxf(rf[i].y, 1e-30f)) - dk1[i];
                store_pair_t<T>(dfg, seq_k + (size_t)grow * DK + 2 * lane, df0, df1);
            }
        }
    }
#ifdef HGRN2_PHASE_TIMING
    HGRN2_STAMP(17);
    if (lane == 0 && p.dbg)
        for (int k = 0; k < 24; ++k) p.dbg[((size_t)chunk * NW + w) * 24 + k] = ph[k];
#endif
    raw_f = nxt_f;
    raw_q = nxt_q;
    __syncthreads();     // the staging areas alias the operand tiles the next chunk is about to write
  }
}

template <typename T, int DK, int DV>
static hipError_t launch_one(const SeqDims& d, const BwdGradParams& p, hipStream_t stream)
{
    typedef BwdGradLds<T, DK, DV> L;
    auto kern = bwd_grad_kernel<T, DK, DV>;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)L::total);
    if (e != hipSuccess) return e;
    // one persistent workgroup per CU (the LDS footprint admits no more), each walking its share of chunks
    const size_t n_chunks = (size_t)d.BH * d.NC;
    const unsigned grid = (unsigned)(n_chunks < 256 ? n_chunks : 256);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(kBwdThreads), L::total, stream, p);
    return hipGetLastError();
}

hipError_t launch_bwd_grad(const SeqDims& d, const void* q, const void* f, const void* v, const void* grad_o,
                           const void* ws_state, const void* ws_dstate, void* grad_q, void* grad_f,
                           void* grad_v, hipStream_t stream)
{
    if ((size_t)d.BH * d.NC == 0) return hipSuccess;
    if (!d.io_bf16) return hipErrorInvalidValue;
    BwdGradParams p;
    p.q = q; p.f = f; p.v = v; p.dO = grad_o; p.ws_s = ws_state; p.ws_ds = ws_dstate;
    p.dq = grad_q; p.df = grad_f; p.dv = grad_v;
    p.BH = d.BH; p.N = d.N; p.NC = d.NC; p.gate_bf16 = d.gate_bf16 ? 1 : 0;
#ifdef HGRN2_PHASE_TIMING
    p.dbg = nullptr;
#endif
    if (d.dk == 128 && d.dv == 128) return launch_one<__bf16, 128, 128>(d, p, stream);
    if (d.dk == 64 && d.dv == 64) return launch_one<__bf16, 64, 64>(d, p, stream);
    if (d.dk == 128 && d.dv == 64) return launch_one<__bf16, 128, 64>(d, p, stream);
    if (d.dk == 64 && d.dv == 128) return launch_one<__bf16, 64, 128>(d, p, stream);
    return hipErrorInvalidValue;
}

}   // namespace hgrn2
