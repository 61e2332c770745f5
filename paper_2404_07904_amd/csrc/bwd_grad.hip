// Per-chunk gradients of the chunkwise HGRN2 recurrence (reverse mode of paper Section 3.2,
// Eq. 3; the paper gives no backward algorithm).  For one chunk of C tokens with incoming state
// S_n and outgoing state gradient dS_{n+1} (both produced by the state sweeps), and with
// P = tril(Q~ K~^T), dP = tril(dO V^T) (diagonal kept, decays factored around the row C/2):
//
//   dq_i = sq_i * ( dP K~           + G_m  * dO S_n^T    )_i       sq = Q~/q
//   dk_j = sk_j * ( dP^T Q~         + H_m  * V dS_{n+1}^T )_j       sk = K~/k,  H_m = g / G_m
//   dv_j =        ( P^T dO          + K^ dS_{n+1}         )_j       K^ = k * g / G
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
// One workgroup per chunk.  The 64 x dk gradients are produced by waves that own a 32-channel
// slice (so the contraction over dv is complete inside a wave and the states arrive straight
// from global memory as operand fragments); dv is produced by waves that own a 32-column slice.
// Operands whose contraction index is the slow axis of their LDS tile are fetched with LDS
// transpose reads.  The final element-wise stage runs in the row-block / channel-pair thread
// layout of common.hpp after the accumulators have been staged through LDS.
#include "common.hpp"
#include "kernels.hpp"

namespace hgrn2 {

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
};

template <typename T, int DK, int DV> struct BwdGradLds {
    static constexpr int C = kChunk;
    static constexpr int PK = DK + pad_elems<T>();      // pitch of [C][DK] tiles
    static constexpr int PV = DV + pad_elems<T>();      // pitch of [C][DV] tiles and of dS [DK][DV]
    static constexpr int PC = C + pad_elems<T>();       // pitch of [C][C] tiles
    static constexpr int PF = DK + 4;                   // pitch of fp32 staging [C][DK]
    // phase 1: operand tiles
    static constexpr size_t qm = 0;                                         // Q~   [C][PK]
    static constexpr size_t km = qm + (size_t)C * PK * sizeof(T);           // K~   [C][PK]
    static constexpr size_t kh = km + (size_t)C * PK * sizeof(T);           // K^   [C][PK]
    static constexpr size_t vm = kh + (size_t)C * PK * sizeof(T);           // V    [C][PV]
    static constexpr size_t dom = vm + (size_t)C * PV * sizeof(T);          // dO   [C][PV]
    static constexpr size_t dsm = dom + (size_t)C * PV * sizeof(T);         // dS   [DK][PV]
    static constexpr size_t pt = dsm + (size_t)DK * PV * sizeof(T);         // P^T  [C][PC]  ([j][i])
    static constexpr size_t dpt = pt + (size_t)C * PC * sizeof(T);          // dP^T [C][PC]
    static constexpr size_t tot = dpt + (size_t)C * PC * sizeof(T);         // [4][DK] fp32
    static constexpr size_t rp = tot + (size_t)kWaves * DK * sizeof(float); // [4][32] fp32 partial R
    static constexpr size_t blk = rp + (size_t)kWaves * 32 * sizeof(float); // [2][4][DK] fp32 block sums
    static constexpr size_t total = blk + (size_t)2 * kWaves * DK * sizeof(float);
    // phase 2 (aliases the operand tiles): fp32 staging of two accumulator sets at a time
    static constexpr size_t cq = 0;                                         // [C][PF] fp32
    static constexpr size_t ck = cq + (size_t)C * PF * sizeof(float);       // [C][PF] fp32
    static constexpr size_t dvs = dsm;                                      // dv  [C][PV]
    static_assert(ck + (size_t)C * PF * sizeof(float) <= dsm, "fp32 staging must fit below the dS tile");
    static_assert((size_t)C * PV <= (size_t)DK * PV, "dv staging must fit in the dS tile");
};

template <typename T, int DK, int DV>
__global__ __launch_bounds__(kThreads) void bwd_grad_kernel(BwdGradParams p)
{
    constexpr int C = kChunk, RW = C / kWaves;
    typedef BwdGradLds<T, DK, DV> L;
    constexpr int PK = L::PK, PV = L::PV, PC = L::PC, PF = L::PF;
    constexpr int NRT = C / 32, NAT = DK / 32, NBT = DV / 32;
    constexpr int TA = NRT * NAT / kWaves;      // (row tile, channel tile) accumulators per wave
    constexpr int TB = NRT * NBT / kWaves;      // (row tile, column tile) accumulators per wave
    static_assert(kWaves % NAT == 0 && kWaves % NBT == 0 && TA >= 1 && TB >= 1, "tile/wave mapping");
    typedef Mma<T> M;
    typedef typename M::frag frag;

    extern __shared__ __align__(16) char smem[];
    T* Qm = reinterpret_cast<T*>(smem + L::qm);
    T* Km = reinterpret_cast<T*>(smem + L::km);
    T* Kh = reinterpret_cast<T*>(smem + L::kh);
    T* Vm = reinterpret_cast<T*>(smem + L::vm);
    T* dOm = reinterpret_cast<T*>(smem + L::dom);
    T* dSm = reinterpret_cast<T*>(smem + L::dsm);
    T* Pt = reinterpret_cast<T*>(smem + L::pt);
    T* dPt = reinterpret_cast<T*>(smem + L::dpt);
    float* tot = reinterpret_cast<float*>(smem + L::tot);
    float* Rp = reinterpret_cast<float*>(smem + L::rp);
    float* blk = reinterpret_cast<float*>(smem + L::blk);
    float* cQ = reinterpret_cast<float*>(smem + L::cq);
    float* cK = reinterpret_cast<float*>(smem + L::ck);
    T* dVs = reinterpret_cast<T*>(smem + L::dvs);

    const int n = blockIdx.x % p.NC, bh = blockIdx.x / p.NC;
    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, r32 = lane & 31, g = lane >> 5;
    const bool k_act = 2 * lane < DK, v_act = 2 * lane < DV;
    const size_t seq_k = (size_t)bh * p.N * DK, seq_v = (size_t)bh * p.N * DV;
    const bool gate_bf16 = p.gate_bf16 != 0;
    const T* qg = static_cast<const T*>(p.q);
    const T* vg = static_cast<const T*>(p.v);
    const T* dog = static_cast<const T*>(p.dO);
    const size_t slot = ((size_t)bh * p.NC + n) * DK * DV;
    const T* wsS = static_cast<const T*>(p.ws_s) + slot;
    const T* wsD = static_cast<const T*>(p.ws_ds) + slot;

    const int at = w % NAT;     // channel tile of every (row, channel) accumulator of this wave
    const int bt = w % NBT;     // column tile of every dv accumulator of this wave

    // ---------------- loads ----------------
    // state fragments of channel tile `at`: operand B[k = dv index][n = channel], 2*NBT k-steps
    frag sS[2 * NBT], sD[2 * NBT];
#pragma unroll
    for (int kk = 0; kk < 2 * NBT; ++kk) {
        sS[kk] = *reinterpret_cast<const frag*>(wsS + state_frag_offset(at, kk >> 1, NBT, kk & 1, lane));
        sD[kk] = *reinterpret_cast<const frag*>(wsD + state_frag_offset(at, kk >> 1, NBT, kk & 1, lane));
    }
    f32x2 rf[RW], rq[RW];
    {
        f32x2 rv[RW], rd[RW];
        RawRows<RW> raw_f, raw_q, raw_v, raw_d;
        const int row0 = n * C + RW * w;
        const int col_k = k_act ? 2 * lane : 0, col_v = v_act ? 2 * lane : 0;
        load_rows<RW>(raw_f, p.f, seq_k, DK, col_k, row0, p.N, gate_bf16);
        load_rows<RW>(raw_q, qg, seq_k, DK, col_k, row0, p.N, is_bf16_type<T>());
        load_rows<RW>(raw_v, vg, seq_v, DV, col_v, row0, p.N, is_bf16_type<T>());
        load_rows<RW>(raw_d, dog, seq_v, DV, col_v, row0, p.N, is_bf16_type<T>());
        convert_rows<RW>(rf, raw_f, row0, p.N, k_act, gate_bf16, 1.0f);
        convert_rows<RW>(rq, raw_q, row0, p.N, k_act, is_bf16_type<T>(), 0.0f);
        convert_rows<RW>(rv, raw_v, row0, p.N, v_act, is_bf16_type<T>(), 0.0f);
        convert_rows<RW>(rd, raw_d, row0, p.N, v_act, is_bf16_type<T>(), 0.0f);
        if (v_act) {
#pragma unroll
            for (int i = 0; i < RW; ++i) {
                store_pair_t<T>(Vm, (size_t)(RW * w + i) * PV + 2 * lane, rv[i].x, rv[i].y);
                store_pair_t<T>(dOm, (size_t)(RW * w + i) * PV + 2 * lane, rd[i].x, rd[i].y);
            }
        }
    }

    // ---------------- gate products; scaled operand tiles ----------------
    // sq/sk are kept for the epilogue: dq = sq * (...), dk = sk * (...)
    float sq0[RW], sq1[RW], sk0[RW], sk1[RW];
    float gall = 1.0f;   // whole-chunk decay of channel 32*at + r32 (set below)
    {
        float a0[RW], a1[RW], z0[RW], z1[RW];
        float run0 = 1.0f, run1 = 1.0f;
#pragma unroll
        for (int i = 0; i < RW; ++i) { run0 *= rf[i].x; run1 *= rf[i].y; a0[i] = run0; a1[i] = run1; }
        run0 = 1.0f; run1 = 1.0f;
#pragma unroll
        for (int i = RW - 1; i >= 0; --i) { z0[i] = run0; z1[i] = run1; run0 *= rf[i].x; run1 *= rf[i].y; }
        if (k_act) {
            tot[w * DK + 2 * lane] = a0[RW - 1];
            tot[w * DK + 2 * lane + 1] = a1[RW - 1];
        }
        __syncthreads();
        if (k_act) {
            const BlockDecay d0 = block_decay(tot, DK, w, 2 * lane);
            const BlockDecay d1 = block_decay(tot, DK, w, 2 * lane + 1);
#pragma unroll
            for (int i = 0; i < RW; ++i) {
                const int row = RW * w + i;
                float m0, m1;
                if (w >= 2) {
                    m0 = d0.mid * a0[i]; m1 = d1.mid * a1[i];
                    sq0[i] = m0; sq1[i] = m1;
                    sk0[i] = fast_rcp(fmaxf(m0, kTinyProduct)); sk1[i] = fast_rcp(fmaxf(m1, kTinyProduct));
                } else {
                    m0 = d0.mid * z0[i]; m1 = d1.mid * z1[i];
                    sk0[i] = m0; sk1[i] = m1;
                    sq0[i] = fast_rcp(fmaxf(m0, kTinyProduct)); sq1[i] = fast_rcp(fmaxf(m1, kTinyProduct));
                }
                const float k0 = 1.0f - rf[i].x, k1 = 1.0f - rf[i].y;
                store_pair_t<T>(Qm, (size_t)row * PK + 2 * lane, rq[i].x * sq0[i], rq[i].y * sq1[i]);
                store_pair_t<T>(Km, (size_t)row * PK + 2 * lane, k0 * sk0[i], k1 * sk1[i]);
                store_pair_t<T>(Kh, (size_t)row * PK + 2 * lane, k0 * (z0[i] * d0.post), k1 * (z1[i] * d1.post));
            }
        } else {
#pragma unroll
            for (int i = 0; i < RW; ++i) { sq0[i] = sq1[i] = sk0[i] = sk1[i] = 0.0f; }
        }
        {
            const int ch = 32 * at + r32;
            gall = (tot[0 * DK + ch] * tot[1 * DK + ch]) * (tot[2 * DK + ch] * tot[3 * DK + ch]);
        }
    }
    // outgoing state gradient of channel tile `at` -> LDS, row-major [channel][dv index]
    if (w < NAT) {
#pragma unroll
        for (int kk = 0; kk < 2 * NBT; ++kk) {
            T* row = dSm + (size_t)(32 * at + r32) * PV + 16 * kk + 4 * g;
            float x[8];
#pragma unroll
            for (int s = 0; s < 8; ++s) x[s] = M::get(sD[kk], s);
            store_pair_t<T>(row, 0, x[0], x[1]);
            store_pair_t<T>(row, 2, x[2], x[3]);
            store_pair_t<T>(row, 8, x[4], x[5]);
            store_pair_t<T>(row, 10, x[6], x[7]);
        }
    }
    __syncthreads();

    // ---------------- P^T and dP^T blocks (I >= J): items 0..NB-1 are P, NB..2NB-1 are dP ----------------
    {
        constexpr int NB = NRT * (NRT + 1) / 2;
        for (int item = w; item < 2 * NB; item += kWaves) {
            const bool is_dp = item >= NB;
            const int b = is_dp ? item - NB : item;
            int I = 0, J = 0, cnt = 0;
            for (int ii = 0; ii < NRT; ++ii)
                for (int jj = 0; jj <= ii; ++jj) { if (cnt == b) { I = ii; J = jj; } ++cnt; }
            f32x16 acc;
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[v] = 0.0f;
            if (is_dp) {
#pragma unroll
                for (int ks = 0; ks < DV / 16; ++ks)
                    M::mma(acc, M::load(dOm + (32 * I + r32) * PV + 16 * ks + 8 * g),
                           M::load(Vm + (32 * J + r32) * PV + 16 * ks + 8 * g));
            } else {
#pragma unroll
                for (int ks = 0; ks < DK / 16; ++ks)
                    M::mma(acc, M::load(Qm + (32 * I + r32) * PK + 16 * ks + 8 * g),
                           M::load(Km + (32 * J + r32) * PK + 16 * ks + 8 * g));
            }
            // acc[row i][col j]; keep j <= i; store transposed: dst[j][i .. i+3]
            T* dst = is_dp ? dPt : Pt;
            const int j_glob = 32 * J + r32;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const int i0 = 32 * I + 8 * c + 4 * g;
                float x[4];
#pragma unroll
                for (int ii = 0; ii < 4; ++ii) x[ii] = (j_glob <= i0 + ii) ? acc[4 * c + ii] : 0.0f;
                store_pair_t<T>(dst, (size_t)j_glob * PC + i0, x[0], x[1]);
                store_pair_t<T>(dst, (size_t)j_glob * PC + i0 + 2, x[2], x[3]);
            }
        }
    }
    __syncthreads();

    // ---------------- main contractions ----------------
    // aQ = dP K~, aQs = dO S_n^T, aK = dP^T Q~, aKs = V dS^T for the (row, channel) tiles of this wave
    f32x16 aQ[TA], aQs[TA], aK[TA], aKs[TA], accV[TB];
#pragma unroll
    for (int t = 0; t < TA; ++t) {
        const int rt = (w + kWaves * t) / NAT;
#pragma unroll
        for (int v = 0; v < 16; ++v) { aQ[t][v] = 0.0f; aQs[t][v] = 0.0f; aK[t][v] = 0.0f; aKs[t][v] = 0.0f; }
        // dP K~ : rows i of tile rt, contraction over j <= i  (k-steps 0 .. 2*rt+1)
        for (int ks = 0; ks < 2 * (rt + 1); ++ks)
            M::mma(aQ[t], M::load_kmajor(dPt, PC, 16 * ks, 32 * rt, lane), M::load_kmajor(Km, PK, 16 * ks, 32 * at, lane));
        // dP^T Q~ : rows j of tile rt, contraction over i >= j  (k-steps 2*rt .. 2*NRT-1)
        for (int ks = 2 * rt; ks < 2 * NRT; ++ks)
            M::mma(aK[t], M::load(dPt + (32 * rt + r32) * PC + 16 * ks + 8 * g), M::load_kmajor(Qm, PK, 16 * ks, 32 * at, lane));
        // dO S_n^T and V dS^T : contraction over the dv index, state fragments from registers
#pragma unroll
        for (int kk = 0; kk < 2 * NBT; ++kk) {
            const T* drow = dOm + (32 * rt + r32) * PV + 16 * kk + 4 * g;
            const T* vrow = Vm + (32 * rt + r32) * PV + 16 * kk + 4 * g;
            M::mma(aQs[t], M::load2(drow, drow + 8), sS[kk]);
            M::mma(aKs[t], M::load2(vrow, vrow + 8), sD[kk]);
        }
    }
    // g * rowsum(dS * S_n), once per channel tile
    if (w < NAT) {
        float rs = 0.0f;
#pragma unroll
        for (int kk = 0; kk < 2 * NBT; ++kk)
#pragma unroll
            for (int s = 0; s < 8; ++s) rs += M::get(sS[kk], s) * M::get(sD[kk], s);
        rs += __shfl_xor(rs, 32);
        if (g == 0) Rp[w * 32 + r32] = gall * rs;
    }

#pragma unroll
    for (int t = 0; t < TB; ++t) {
        const int rt = (w + kWaves * t) / NBT;
        f32x16 aV;
#pragma unroll
        for (int v = 0; v < 16; ++v) aV[v] = 0.0f;
        // P^T dO : rows j of tile rt, contraction over i >= j
        for (int ks = 2 * rt; ks < 2 * NRT; ++ks)
            M::mma(aV, M::load(Pt + (32 * rt + r32) * PC + 16 * ks + 8 * g), M::load_kmajor(dOm, PV, 16 * ks, 32 * bt, lane));
        // K^ dS : contraction over the channels
#pragma unroll
        for (int ks = 0; ks < DK / 16; ++ks)
            M::mma(aV, M::load(Kh + (32 * rt + r32) * PK + 16 * ks + 8 * g), M::load_kmajor(dSm, PV, 16 * ks, 32 * bt, lane));
        accV[t] = aV;
    }
    __syncthreads();     // every wave is done with the operand tiles

    // ---------------- round 1 staging: aQ, aQs as [row][channel] fp32; dv as T ----------------
#pragma unroll
    for (int t = 0; t < TA; ++t) {
        const int rt = (w + kWaves * t) / NAT;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const size_t o = (size_t)(32 * rt + acc_row(v, lane)) * PF + 32 * at + r32;
            cQ[o] = aQ[t][v];
            cK[o] = aQs[t][v];
        }
    }
#pragma unroll
    for (int t = 0; t < TB; ++t) {
        const int rt = (w + kWaves * t) / NBT;
#pragma unroll
        for (int v = 0; v < 16; ++v)
            dVs[(size_t)(32 * rt + acc_row(v, lane)) * PV + 32 * bt + r32] = (T)accV[t][v];
    }
    __syncthreads();

    // ---------------- element-wise epilogue in the row-block / channel-pair layout ----------------
    // e = pair terms + incoming-state term of dL (summed as a suffix), y = outgoing-state term
    // (summed as an exclusive prefix); see the header comment.
    float e0[RW], e1[RW], dk0[RW], dk1[RW];
    float hp0 = 0.0f, hp1 = 0.0f, hq0 = 0.0f, hq1 = 0.0f;
    T* dqg = static_cast<T*>(p.dq);
    T* dfg = static_cast<T*>(p.df);
    if (k_act) {
        hp0 = tot[0 * DK + 2 * lane] * tot[1 * DK + 2 * lane];           // G_m
        hp1 = tot[0 * DK + 2 * lane + 1] * tot[1 * DK + 2 * lane + 1];
        hq0 = tot[2 * DK + 2 * lane] * tot[3 * DK + 2 * lane];           // g / G_m
        hq1 = tot[2 * DK + 2 * lane + 1] * tot[3 * DK + 2 * lane + 1];
#pragma unroll
        for (int i = 0; i < RW; ++i) {
            const int row = RW * w + i;
            const f32x2 xq = *reinterpret_cast<const f32x2*>(cQ + (size_t)row * PF + 2 * lane);
            const f32x2 xs = *reinterpret_cast<const f32x2*>(cK + (size_t)row * PF + 2 * lane);
            const float qs0 = rq[i].x * sq0[i], qs1 = rq[i].y * sq1[i];   // exactly what went into Q~
            const float dq0 = sq0[i] * (xq.x + hp0 * xs.x), dq1 = sq1[i] * (xq.y + hp1 * xs.y);
            e0[i] = (float)(T)qs0 * xq.x + qs0 * (hp0 * xs.x);
            e1[i] = (float)(T)qs1 * xq.y + qs1 * (hp1 * xs.y);
            const int grow = n * C + row;
            if (grow < p.N) store_pair_t<T>(dqg, seq_k + (size_t)grow * DK + 2 * lane, dq0, dq1);
        }
    }
    __syncthreads();     // everyone has read round 1

    // ---------------- round 2 staging: aK, aKs ----------------
#pragma unroll
    for (int t = 0; t < TA; ++t) {
        const int rt = (w + kWaves * t) / NAT;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const size_t o = (size_t)(32 * rt + acc_row(v, lane)) * PF + 32 * at + r32;
            cQ[o] = aK[t][v];
            cK[o] = aKs[t][v];
        }
    }
    __syncthreads();
    float* blkE = blk;                    // [4][DK] block sums of e
    float* blkY = blk + kWaves * DK;      // [4][DK] block sums of y
    float y0[RW], y1[RW];
    if (k_act) {
        float se0 = 0.0f, se1 = 0.0f, sy0 = 0.0f, sy1 = 0.0f;
#pragma unroll
        for (int i = 0; i < RW; ++i) {
            const int row = RW * w + i;
            const f32x2 xk = *reinterpret_cast<const f32x2*>(cQ + (size_t)row * PF + 2 * lane);
            const f32x2 xs = *reinterpret_cast<const f32x2*>(cK + (size_t)row * PF + 2 * lane);
            const float ks0 = (1.0f - rf[i].x) * sk0[i], ks1 = (1.0f - rf[i].y) * sk1[i];   // what went into K~
            dk0[i] = sk0[i] * (xk.x + hq0 * xs.x);
            dk1[i] = sk1[i] * (xk.y + hq1 * xs.y);
            e0[i] -= (float)(T)ks0 * xk.x;
            e1[i] -= (float)(T)ks1 * xk.y;
            y0[i] = sy0; y1[i] = sy1;                         // exclusive prefix inside the block
            sy0 += ks0 * (hq0 * xs.x);
            sy1 += ks1 * (hq1 * xs.y);
        }
#pragma unroll
        for (int i = RW - 1; i >= 0; --i) { se0 += e0[i]; se1 += e1[i]; e0[i] = se0; e1[i] = se1; }   // inclusive suffix
        blkE[w * DK + 2 * lane] = se0; blkE[w * DK + 2 * lane + 1] = se1;
        blkY[w * DK + 2 * lane] = sy0; blkY[w * DK + 2 * lane + 1] = sy1;
    }
    __syncthreads();
    if (k_act) {
        const int c0 = 2 * lane, c1 = 2 * lane + 1;
        float add0 = Rp[(c0 >> 5) * 32 + (c0 & 31)], add1 = Rp[(c1 >> 5) * 32 + (c1 & 31)];
        for (int ww = kWaves - 1; ww > w; --ww) { add0 += blkE[ww * DK + c0]; add1 += blkE[ww * DK + c1]; }
        for (int ww = 0; ww < w; ++ww) { add0 += blkY[ww * DK + c0]; add1 += blkY[ww * DK + c1]; }
#pragma unroll
        for (int i = 0; i < RW; ++i) {
            const int grow = n * C + RW * w + i;
            if (grow < p.N) {
                const float df0 = (e0[i] + y0[i] + add0) * fast_rcp(fmaxf(rf[i].x, 1e-30f)) - dk0[i];
                const float df1 = (e1[i] + y1[i] + add1) * fast_rcp(fmaxf(rf[i].y, 1e-30f)) - dk1[i];
                store_pair_t<T>(dfg, seq_k + (size_t)grow * DK + 2 * lane, df0, df1);
            }
        }
    }
    // ---------------- coalesced store of dv ----------------
    {
        constexpr int VEC = 16 / (int)sizeof(T);
        constexpr int VPR = DV / VEC;
        T* dvg = static_cast<T*>(p.dv);
        for (int idx = tid; idx < C * VPR; idx += kThreads) {
            const int row = idx / VPR, cv = idx % VPR;
            const int grow = n * C + row;
            if (grow < p.N) {
                const uint4 val = *reinterpret_cast<const uint4*>(dVs + (size_t)row * PV + cv * VEC);
                *reinterpret_cast<uint4*>(dvg + seq_v + (size_t)grow * DV + cv * VEC) = val;
            }
        }
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
    hipLaunchKernelGGL(kern, dim3((unsigned)((size_t)d.BH * d.NC)), dim3(kThreads), L::total, stream, p);
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
    if (d.dk == 128 && d.dv == 128) return launch_one<__bf16, 128, 128>(d, p, stream);
    if (d.dk == 64 && d.dv == 64) return launch_one<__bf16, 64, 64>(d, p, stream);
    if (d.dk == 128 && d.dv == 64) return launch_one<__bf16, 128, 64>(d, p, stream);
    if (d.dk == 64 && d.dv == 128) return launch_one<__bf16, 64, 128>(d, p, stream);
    return hipErrorInvalidValue;
}

}   // namespace hgrn2
