// Per-chunk forward read-out of the chunkwise HGRN2 algorithm (paper Section 3.2, Eq. 3,
// unrolled inside one chunk of C tokens whose incoming state is S_n):
//
//     o_i = sum_{j<=i} ( sum_a q_i[a] k_j[a] prod_{j<s<=i} f_s[a] ) v_j  +  (q_i * G_i) S_n
//
// (q_i * G_i) S_n is evaluated as Q~_i (G_m * S_n): the state sweep stores G_m * S_n.
//
// The decay between two tokens is factored around the reference row m = C/2:
//     prod_{j<s<=i} f_s = (G_i / G_m) (G_m / G_j)  ->  P = tril(Q~ K~^T),  Q~ = q G/G_m,  K~ = k G_m/G
// so every cumulative product spans at most C/2 tokens, and the one that appears as a divisor is
// the product BETWEEN the row and the reference, formed directly by multiplication (no logs).
// One workgroup handles one chunk of one (batch, head); all chunks are independent because the
// state sweep has already written every S_n.  P is built transposed so that the accumulator
// registers already hold 4 consecutive j per lane and go to LDS as 8-byte vectors.
#include "common.hpp"
#include "kernels.hpp"

namespace hgrn2 {

struct FwdOutParams {
    const void* q;
    const void* f;
    const void* v;
    const void* ws;
    void* o;
    int BH, N, NC, gate_bf16;
    const float* beta;   // [H][dk] lower bounds, or null: the gate tensor holds f itself
    int H;
    TokenLayout lay;     // used when dense == 0
    int dense;           // sequence tensors are [B][H][N][d]
    int* flag;           // null, or set to 1 when a gate product falls below the floor of the reciprocals
};

template <typename T, int DK, int DV> struct FwdOutLds {
    static constexpr int C = kChunk;
    static constexpr int PK = DK + pad_elems<T>();
    static constexpr int PC = C + pad_elems<T>();
    static constexpr int PO = DV + pad_elems<T>();
    static constexpr size_t qm = 0;                                   // [C][PK]  Q~
    static constexpr size_t km = qm + (size_t)C * PK * sizeof(T);     // [C][PK]  K~, later [C][PO] output staging
    static constexpr size_t ost = km;
    static constexpr size_t vt = km + (size_t)C * (PK > PO ? PK : PO) * sizeof(T);   // [DV][PC] V transposed
    static constexpr size_t pm = vt + (size_t)DV * PC * sizeof(T);    // [C][PC]  P
    static constexpr size_t tot = pm + (size_t)C * PC * sizeof(T);    // [4][DK] fp32
    static constexpr size_t total = tot + (size_t)kWaves * DK * sizeof(float);
};

template <typename T, int DK, int DV, bool DENSE>
__device__ __forceinline__ void fwd_out_body(const FwdOutParams& p)
{
    constexpr int C = kChunk, RW = C / kWaves;
    typedef FwdOutLds<T, DK, DV> L;
    constexpr int PK = L::PK, PC = L::PC, PO = L::PO;
    constexpr int NRT = C / 32, NBT = DV / 32, NKS = DK / 16;
    typedef Mma<T> M;

    extern __shared__ __align__(16) char smem[];
    T* Qm = reinterpret_cast<T*>(smem + L::qm);
    T* Km = reinterpret_cast<T*>(smem + L::km);
    T* Vt = reinterpret_cast<T*>(smem + L::vt);
    T* Pm = reinterpret_cast<T*>(smem + L::pm);
    float* tot = reinterpret_cast<float*>(smem + L::tot);
    T* Ost = reinterpret_cast<T*>(smem + L::ost);   // output staging aliases K~ once P has been formed

    if (not_chosen(p.lay)) return;       // one of several chunk lengths, and not the one called for
    int n, bh;
    if (!locate_chunk<DENSE>(p.lay, p.BH, p.NC, blockIdx.x, bh, n)) return;
    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, r32 = lane & 31, g = lane >> 5;
    const bool k_act = 2 * lane < DK, v_act = 2 * lane < DV;
    const SeqView sv = seq_view<DENSE, DK, DV>(p.lay, p.N, p.NC, bh);
    const size_t seq_k = sv.off_k, seq_v = sv.off_v;
    const int N = sv.N;
    const ChunkRows cr = chunk_rows(p.lay.sub, n, N);        // which tokens the chunk's rows stand for
    const int ld_k = DENSE ? DK : (int)p.lay.sn_k, ld_v = DENSE ? DV : (int)p.lay.sn_v;   // token stride, elements
    const bool gate_bf16 = p.gate_bf16 != 0;
    const T* qg = static_cast<const T*>(p.q);
    const T* vg = static_cast<const T*>(p.v);
    const T* wsn = static_cast<const T*>(p.ws) + (size_t)blockIdx.x * DK * DV;      // chunk indices are the workspace order

    // ---------------- loads ----------------
    // incoming state S_n, column block bt of this wave, as B-operand fragments (k runs over dk)
    static_assert(kWaves % NBT == 0 && (NRT * NBT) % kWaves == 0, "tile/wave mapping");
    const int bt = w % NBT;
    typename M::frag sfrag[NKS];
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks)
        sfrag[ks] = *reinterpret_cast<const typename M::frag*>(
            wsn + state_frag_offset(ks >> 1, bt, NBT, ks & 1, lane));
    f32x2 rf[RW], rq[RW], rv[RW];
    {
        RawRows<RW> raw_f, raw_q, raw_v;
        const int row0 = cr.tok0 + RW * w;
        const int col_k = k_act ? 2 * lane : 0, col_v = v_act ? 2 * lane : 0;
        load_rows<RW>(raw_f, p.f, seq_k, ld_k, col_k, row0, N, gate_bf16);
        load_rows<RW>(raw_q, qg, seq_k, ld_k, col_k, row0, N, is_bf16_type<T>());
        load_rows<RW>(raw_v, vg, seq_v, ld_v, col_v, row0, N, is_bf16_type<T>());
        convert_rows<RW>(rf, raw_f, row0, cr.end, k_act, gate_bf16, 1.0f, cr.first);
        if (p.beta) gate_rows<RW>(rf, p.beta + (size_t)(bh % p.H) * DK, col_k, k_act, row0, cr.end, cr.first);
        convert_rows<RW>(rq, raw_q, row0, cr.end, k_act, is_bf16_type<T>(), 0.0f, cr.first);
        convert_rows<RW>(rv, raw_v, row0, cr.end, v_act, is_bf16_type<T>(), 0.0f, cr.first);
    }

    // ---------------- gate products and scaled operands ----------------
    float a0[RW], a1[RW], z0[RW], z1[RW];
    {
        float run0 = 1.0f, run1 = 1.0f;
#pragma unroll
        for (int i = 0; i < RW; ++i) { run0 *= rf[i].x; run1 *= rf[i].y; a0[i] = run0; a1[i] = run1; }
        run0 = 1.0f; run1 = 1.0f;
#pragma unroll
        for (int i = RW - 1; i >= 0; --i) { z0[i] = run0; z1[i] = run1; run0 *= rf[i].x; run1 *= rf[i].y; }
    }
    if (k_act) {
        tot[w * DK + 2 * lane] = a0[RW - 1];
        tot[w * DK + 2 * lane + 1] = a1[RW - 1];
    }
    __syncthreads();
    if (k_act) {
        const BlockDecay d0 = block_decay(tot, DK, w, 2 * lane);
        const BlockDecay d1 = block_decay(tot, DK, w, 2 * lane + 1);
        {   // the smallest product this thread takes a reciprocal of: its first row after the reference, its last before
            const float s0 = d0.mid * (w >= 2 ? a0[RW - 1] : z0[0]), s1 = d1.mid * (w >= 2 ? a1[RW - 1] : z1[0]);
            if (p.flag && fminf(s0, s1) < kTinyProduct) *p.flag = 1;
        }
#pragma unroll
        for (int i = 0; i < RW; ++i) {
            const int row = RW * w + i;
            // m = product of the gates strictly between this row and the reference row C/2
            float m0, m1, qs0, qs1, ks0, ks1;
            if (w >= 2) {          // rows after the reference: G_i/G_m = m <= 1
                m0 = d0.mid * a0[i]; m1 = d1.mid * a1[i];
                const float i0 = fast_rcp(fmaxf(m0, kTinyProduct)), i1 = fast_rcp(fmaxf(m1, kTinyProduct));
                qs0 = rq[i].x * m0; qs1 = rq[i].y * m1;
                ks0 = (1.0f - rf[i].x) * i0; ks1 = (1.0f - rf[i].y) * i1;
            } else {               // rows up to the reference: G_m/G_j = m <= 1
                m0 = d0.mid * z0[i]; m1 = d1.mid * z1[i];
                const float i0 = fast_rcp(fmaxf(m0, kTinyProduct)), i1 = fast_rcp(fmaxf(m1, kTinyProduct));
                qs0 = rq[i].x * i0; qs1 = rq[i].y * i1;
                ks0 = (1.0f - rf[i].x) * m0; ks1 = (1.0f - rf[i].y) * m1;
            }
            store_pair_t<T>(Qm, (size_t)row * PK + 2 * lane, qs0, qs1);
            store_pair_t<T>(Km, (size_t)row * PK + 2 * lane, ks0, ks1);
        }
    }
    if (v_act) {
        float x0[RW], x1[RW];
#pragma unroll
        for (int i = 0; i < RW; ++i) { x0[i] = rv[i].x; x1[i] = rv[i].y; }
        store_run<T, RW>(Vt + (2 * lane) * PC + RW * w, x0);
        store_run<T, RW>(Vt + (2 * lane + 1) * PC + RW * w, x1);
    }
    __syncthreads();

    // ---------------- P^T blocks: (J, I) with J <= I; wave w takes block w ----------------
    {
        constexpr int NBLK = NRT * (NRT + 1) / 2;
        for (int blk = w; blk < NBLK; blk += kWaves) {
            // enumerate (J, I): 0 -> (0,0), 1 -> (0,1), 2 -> (1,1)
            int I = 0, J = 0, cnt = 0;
            for (int ii = 0; ii < NRT; ++ii)
                for (int jj = 0; jj <= ii; ++jj) { if (cnt == blk) { I = ii; J = jj; } ++cnt; }
            f32x16 acc;
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[v] = 0.0f;
#pragma unroll
            for (int ks = 0; ks < NKS; ++ks) {
                const typename M::frag fa = M::load(Km + (32 * J + r32) * PK + 16 * ks + 8 * g);
                const typename M::frag fb = M::load(Qm + (32 * I + r32) * PK + 16 * ks + 8 * g);
                M::mma(acc, fa, fb);    // acc[row j][col i]
            }
            const int i_glob = 32 * I + r32;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const int j0 = 32 * J + 8 * c + 4 * g;
                float x[4];
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) x[jj] = (j0 + jj <= i_glob) ? acc[4 * c + jj] : 0.0f;
                store_pair_t<T>(Pm, (size_t)i_glob * PC + j0, x[0], x[1]);
                store_pair_t<T>(Pm, (size_t)i_glob * PC + j0 + 2, x[2], x[3]);
            }
        }
    }
    __syncthreads();

    // ---------------- O tiles: P V + (q G) S_n ----------------
    // (NRT * NBT is a multiple of the wave count and NBT divides it, so every tile of a wave
    // shares the column block bt and the state fragments loaded at the top are reused.)
    for (int tix = w; tix < NRT * NBT; tix += kWaves) {
        const int rt = tix / NBT;
        f32x16 acc;
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[v] = 0.0f;
        for (int ks = 0; ks < 2 * (rt + 1); ++ks) {
            const typename M::frag fa = M::load(Pm + (32 * rt + r32) * PC + 16 * ks + 8 * g);
            const typename M::frag fb = M::load(Vt + (32 * bt + r32) * PC + 16 * ks + 8 * g);
            M::mma(acc, fa, fb);
        }
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) {
            // k-slot order of the state fragments: rows 16ks + {4g..4g+3, 8+4g..8+4g+3}
            const T* qrow = Qm + (32 * rt + r32) * PK + 16 * ks + 4 * g;
            const typename M::frag fa = M::load2(qrow, qrow + 8);
            M::mma(acc, fa, sfrag[ks]);
        }
#pragma unroll
        for (int v = 0; v < 16; ++v)
            Ost[(size_t)(32 * rt + acc_row(v, lane)) * PO + 32 * bt + r32] = (T)acc[v];
    }
    __syncthreads();

    // ---------------- coalesced store of the [C][DV] tile ----------------
    {
        constexpr int VEC = 16 / (int)sizeof(T);         // elements per 16-byte vector
        constexpr int VPR = DV / VEC;                     // vectors per row
        T* og = static_cast<T*>(p.o);
        for (int idx = tid; idx < C * VPR; idx += kThreads) {
            const int row = idx / VPR, cv = idx % VPR;
            const int grow = cr.tok0 + row;
            if (cr.holds(row)) {
                const uint4 val = *reinterpret_cast<const uint4*>(Ost + (size_t)row * PO + cv * VEC);
                *reinterpret_cast<uint4*>(og + seq_v + (size_t)grow * ld_v + cv * VEC) = val;
            }
        }
    }
}

template <typename T, int DK, int DV>
__global__ __launch_bounds__(kThreads) void fwd_out_kernel(FwdOutParams p)
{
    if (p.dense) fwd_out_body<T, DK, DV, true>(p);
    else         fwd_out_body<T, DK, DV, false>(p);
}

template <typename T, int DK, int DV>
static hipError_t launch_one(const SeqDims& d, const FwdOutParams& p, hipStream_t stream)
{
    typedef FwdOutLds<T, DK, DV> L;
    auto kern = fwd_out_kernel<T, DK, DV>;
    hipError_t e = allow_dynamic_lds(reinterpret_cast<const void*>(kern), (int)L::total);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3((unsigned)d.total_chunks()), dim3(kThreads), L::total, stream, p);
    return hipGetLastError();
}

template <typename T>
static hipError_t launch_dims(const SeqDims& d, const FwdOutParams& p, hipStream_t stream)
{
    if (d.dk == 128 && d.dv == 128) return launch_one<T, 128, 128>(d, p, stream);
    if (d.dk == 64 && d.dv == 64) return launch_one<T, 64, 64>(d, p, stream);
    if (d.dk == 128 && d.dv == 64) return launch_one<T, 128, 64>(d, p, stream);
    if (d.dk == 64 && d.dv == 128) return launch_one<T, 64, 128>(d, p, stream);
    return hipErrorInvalidValue;
}

hipError_t launch_fwd_out(const SeqDims& d, const void* q, const void* f, const void* v, const void* ws_state,
                          void* o, hipStream_t stream)
{
    if (d.total_chunks() == 0) return hipSuccess;
    FwdOutParams p;
    p.q = q; p.f = f; p.v = v; p.ws = ws_state; p.o = o;
    p.BH = d.BH; p.N = d.N; p.NC = d.NC; p.gate_bf16 = d.gate_bf16 ? 1 : 0;
    p.beta = d.beta; p.H = d.H; p.lay = d.lay; p.dense = d.dense() ? 1 : 0; p.flag = d.domain_flag;
    return d.io_bf16 ? launch_dims<__bf16>(d, p, stream) : launch_dims<float>(d, p, stream);
}

}   // namespace hgrn2
