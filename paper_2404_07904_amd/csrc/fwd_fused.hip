// Fused forward pass of the chunkwise HGRN2 algorithm (paper Section 3.2, Eq. 3): the
// chunk-to-chunk state recurrence and the per-chunk read-out in ONE pass over q, f, v,
//
//     O_n     = tril(Q~ K~^T) V + (q G) S_n
//     S_{n+1} = Diag(g) S_n + K^^T V
//
// so that the per-chunk states never travel through HBM (the two-kernel path writes and re-reads
// 2*dk*dv bytes per chunk, as much again as the chunk's own q, f, v, o).  One workgroup of eight
// wave64s owns a whole (batch, head) and walks its chunks in order:
//   * the dk x dv state lives in fp32 MFMA accumulators, two 32x32 tiles per wave; after every
//     update each wave drops a bf16 copy of its tiles into LDS in MFMA-fragment order, from where
//     all waves read the operand of (q G) S_n;
//   * wave w owns rows 8w..8w+7 of the chunk for the element-wise work (gate products along time
//     serially in registers, channel pair per lane), and the 32x32 output tile (w/4, w%4);
//   * the next chunk's rows are loaded into registers while the current chunk is computed.
// Used for bf16 storage with dk = dv = 128 when there are enough sequences to fill the chip;
// other cases take the sweep + read-out path.
#include "common.hpp"
#include "kernels.hpp"

namespace hgrn2 {

constexpr int kFusedWaves = 8;
constexpr int kFusedThreads = 64 * kFusedWaves;

struct FwdFusedParams {
    const void* q;
    const void* f;
    const void* v;
    const float* h0;
    void* o;
    float* hT;
    int N, NC, gate_bf16;
#ifdef HGRN2_PHASE_TIMING
    long long* dbg;      // [workgroup][wave][16] accumulated clock ticks per phase (diagnostic builds only)
#endif
};

#ifdef HGRN2_PHASE_TIMING
#define HGRN2_STAMP(k) do { const long long t_now = wall_clock64(); ph[k] += t_now - t_prev; t_prev = t_now; } while (0)
#else
#define HGRN2_STAMP(k) do { } while (0)
#endif

template <int DK, int DV> struct FwdFusedLds {
    typedef __bf16 T;
    static constexpr int C = kChunk;
    static constexpr int PK = DK + 8, PC = C + 8, PO = DV + 8;
    static constexpr size_t qm = 0;                                     // Q~   [C][PK]
    static constexpr size_t km = qm + (size_t)C * PK * 2;               // K~   [C][PK]
    static constexpr size_t qf = km + (size_t)C * PK * 2;               // q G  [C][PK]
    static constexpr size_t vt = qf + (size_t)C * PK * 2;               // V^T  [DV][PC]
    static constexpr size_t kt = vt + (size_t)DV * PC * 2;              // K^^T [DK][PC]
    static constexpr size_t pm = kt + (size_t)DK * PC * 2;              // P    [C][PC]
    static constexpr size_t sb = pm + (size_t)C * PC * 2;               // state, bf16, fragment order
    static constexpr size_t gam = sb + (size_t)DK * DV * 2;             // [DK] fp32
    static constexpr size_t tot = gam + (size_t)DK * 4;                 // [8][DK] fp32
    static constexpr size_t total = tot + (size_t)kFusedWaves * DK * 4;
    static_assert(2 * C * PK >= C * PO, "output staging must fit in the Q~/K~ tiles");
};

template <int DK, int DV>
__global__ __launch_bounds__(kFusedThreads) void fwd_fused_kernel(FwdFusedParams p)
{
    typedef __bf16 T;
    typedef Mma<T> M;
    typedef typename M::frag frag;
    typedef FwdFusedLds<DK, DV> L;
    constexpr int C = kChunk, NW = kFusedWaves, RW = C / NW;
    constexpr int PK = L::PK, PC = L::PC, PO = L::PO;
    constexpr int NRT = C / 32, NAT = DK / 32, NBT = DV / 32, NKS = DK / 16;
    static_assert(DK == 128 && DV == 128 && NRT * NBT == NW && NAT * NBT == 2 * NW, "tile/wave mapping");

    extern __shared__ __align__(16) char smem[];
    T* Qm = reinterpret_cast<T*>(smem + L::qm);
    T* Km = reinterpret_cast<T*>(smem + L::km);
    T* Qf = reinterpret_cast<T*>(smem + L::qf);
    T* Vt = reinterpret_cast<T*>(smem + L::vt);
    T* Kt = reinterpret_cast<T*>(smem + L::kt);
    T* Pm = reinterpret_cast<T*>(smem + L::pm);
    T* Sb = reinterpret_cast<T*>(smem + L::sb);
    float* gam = reinterpret_cast<float*>(smem + L::gam);
    float* tot = reinterpret_cast<float*>(smem + L::tot);
    T* Ost = Qm;

    const int bh = blockIdx.x;
    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, r32 = lane & 31, g = lane >> 5;
    const size_t seq_k = (size_t)bh * p.N * DK, seq_v = (size_t)bh * p.N * DV;
    const bool gate_bf16 = p.gate_bf16 != 0;
    const T* qg = static_cast<const T*>(p.q);
    const T* vg = static_cast<const T*>(p.v);
    T* og = static_cast<T*>(p.o);

    const int rt = w / NBT, bt = w % NBT;    // output tile of this wave
    const int at0 = 2 * rt;                  // its two state tiles: (at0, bt), (at0 + 1, bt)

    // ---- state: fp32 accumulators + bf16 fragment copy in LDS ----
    f32x16 accS[2];
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v)
            accS[j][v] = p.h0 ? p.h0[(size_t)bh * DK * DV + (size_t)(32 * (at0 + j) + acc_row(v, lane)) * DV + 32 * bt + r32]
                              : 0.0f;
    auto publish_state = [&]() {
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                float x[8];
#pragma unroll
                for (int s = 0; s < 8; ++s) x[s] = accS[j][8 * half + s];
                *reinterpret_cast<frag*>(Sb + state_frag_offset(at0 + j, bt, NBT, half, lane)) = M::pack(x);
            }
    };
    publish_state();

    RawRows<RW> raw_f, raw_q, raw_v;
    auto load_chunk = [&](int n) {
        const int row0 = n * C + RW * w;
        load_rows<RW>(raw_f, p.f, seq_k, DK, 2 * lane, row0, p.N, gate_bf16);
        load_rows<RW>(raw_q, qg, seq_k, DK, 2 * lane, row0, p.N, true);
        load_rows<RW>(raw_v, vg, seq_v, DV, 2 * lane, row0, p.N, true);
    };
    if (p.NC > 0) load_chunk(0);

#ifdef HGRN2_PHASE_TIMING
    long long ph[16] = {0};
    long long t_prev = wall_clock64();
#endif
    for (int n = 0; n < p.NC; ++n) {
        // ---------------- element-wise stage ----------------
        f32x2 rf[RW], rq[RW], rv[RW];
        {
            const int row0 = n * C + RW * w;
            convert_rows<RW>(rf, raw_f, row0, p.N, true, gate_bf16, 1.0f);
            convert_rows<RW>(rq, raw_q, row0, p.N, true, true, 0.0f);
            convert_rows<RW>(rv, raw_v, row0, p.N, true, true, 0.0f);
        }
        float a0[RW], a1[RW], z0[RW], z1[RW];
        {
            float run0 = 1.0f, run1 = 1.0f;
#pragma unroll
            for (int i = 0; i < RW; ++i) { run0 *= rf[i].x; run1 *= rf[i].y; a0[i] = run0; a1[i] = run1; }
            run0 = 1.0f; run1 = 1.0f;
#pragma unroll
            for (int i = RW - 1; i >= 0; --i) { z0[i] = run0; z1[i] = run1; run0 *= rf[i].x; run1 *= rf[i].y; }
        }
        tot[w * DK + 2 * lane] = a0[RW - 1];
        tot[w * DK + 2 * lane + 1] = a1[RW - 1];
        HGRN2_STAMP(0);
        __syncthreads();                                   // B1 (also: previous chunk's staging has been read)
        HGRN2_STAMP(1);
        {
            const BlockDecay d0 = block_decay_n<NW>(tot, DK, w, 2 * lane);
            const BlockDecay d1 = block_decay_n<NW>(tot, DK, w, 2 * lane + 1);
            float kh0[RW], kh1[RW], v0[RW], v1[RW];
#pragma unroll
            for (int i = 0; i < RW; ++i) {
                const int row = RW * w + i;
                float m0, m1, qs0, qs1, ks0, ks1;
                const float k0 = 1.0f - rf[i].x, k1 = 1.0f - rf[i].y;
                if (w >= NW / 2) {
                    m0 = d0.mid * a0[i]; m1 = d1.mid * a1[i];
                    qs0 = rq[i].x * m0; qs1 = rq[i].y * m1;
                    ks0 = k0 * fast_rcp(fmaxf(m0, kTinyProduct)); ks1 = k1 * fast_rcp(fmaxf(m1, kTinyProduct));
                } else {
                    m0 = d0.mid * z0[i]; m1 = d1.mid * z1[i];
                    qs0 = rq[i].x * fast_rcp(fmaxf(m0, kTinyProduct)); qs1 = rq[i].y * fast_rcp(fmaxf(m1, kTinyProduct));
                    ks0 = k0 * m0; ks1 = k1 * m1;
                }
                store_pair_t<T>(Qm, (size_t)row * PK + 2 * lane, qs0, qs1);
                store_pair_t<T>(Km, (size_t)row * PK + 2 * lane, ks0, ks1);
                store_pair_t<T>(Qf, (size_t)row * PK + 2 * lane, rq[i].x * (d0.pre * a0[i]), rq[i].y * (d1.pre * a1[i]));
                kh0[i] = k0 * (z0[i] * d0.post); kh1[i] = k1 * (z1[i] * d1.post);
                v0[i] = rv[i].x; v1[i] = rv[i].y;
            }
            *reinterpret_cast<frag*>(Kt + (2 * lane) * PC + RW * w) = M::pack(kh0);
            *reinterpret_cast<frag*>(Kt + (2 * lane + 1) * PC + RW * w) = M::pack(kh1);
            *reinterpret_cast<frag*>(Vt + (2 * lane) * PC + RW * w) = M::pack(v0);
            *reinterpret_cast<frag*>(Vt + (2 * lane + 1) * PC + RW * w) = M::pack(v1);
            if (w == 0) { gam[2 * lane] = d0.all; gam[2 * lane + 1] = d1.all; }
        }
        if (n + 1 < p.NC) load_chunk(n + 1);              // in flight during the matrix stages
        HGRN2_STAMP(2);
        __syncthreads();                                   // B2
        HGRN2_STAMP(3);

        // ---------------- P^T blocks (J <= I), one per wave ----------------
        if (w < NRT * (NRT + 1) / 2) {
            const int I = (w == 0) ? 0 : 1, J = (w == 2) ? 1 : 0;     // 0:(0,0) 1:(0,1) 2:(1,1) as (J,I)
            f32x16 acc;
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[v] = 0.0f;
#pragma unroll
            for (int ks = 0; ks < NKS; ++ks)
                M::mma(acc, M::load(Km + (32 * J + r32) * PK + 16 * ks + 8 * g),
                       M::load(Qm + (32 * I + r32) * PK + 16 * ks + 8 * g));     // acc[row j][col i]
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
        HGRN2_STAMP(4);
        __syncthreads();                                   // B3
        HGRN2_STAMP(5);

        // ---------------- output tile (rt, bt): P V + (q G) S_n ----------------
        {
            f32x16 acc;
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[v] = 0.0f;
            for (int ks = 0; ks < 2 * (rt + 1); ++ks)
                M::mma(acc, M::load(Pm + (32 * rt + r32) * PC + 16 * ks + 8 * g),
                       M::load(Vt + (32 * bt + r32) * PC + 16 * ks + 8 * g));
#pragma unroll
            for (int ks = 0; ks < NKS; ++ks) {
                const T* qrow = Qf + (32 * rt + r32) * PK + 16 * ks + 4 * g;
                M::mma(acc, M::load2(qrow, qrow + 8),
                       *reinterpret_cast<const frag*>(Sb + state_frag_offset(ks >> 1, bt, NBT, ks & 1, lane)));
            }
#pragma unroll
            for (int v = 0; v < 16; ++v)
                Ost[(size_t)(32 * rt + acc_row(v, lane)) * PO + 32 * bt + r32] = (T)acc[v];
        }
        HGRN2_STAMP(6);
        // ---------------- state tiles (at0, bt), (at0+1, bt): Diag(g) S + K^^T V ----------------
#pragma unroll
        for (int j = 0; j < 2; ++j) {
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const f32x4 gm = *reinterpret_cast<const f32x4*>(gam + 32 * (at0 + j) + 8 * c + 4 * g);
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) accS[j][4 * c + jj] *= gm[jj];
            }
#pragma unroll
            for (int ks = 0; ks < C / 16; ++ks)
                M::mma(accS[j], M::load(Kt + (32 * (at0 + j) + r32) * PC + 16 * ks + 8 * g),
                       M::load(Vt + (32 * bt + r32) * PC + 16 * ks + 8 * g));
        }
        HGRN2_STAMP(7);
        __syncthreads();                                   // B4: S_n and the operand tiles are no longer read
        HGRN2_STAMP(8);

        publish_state();
        {
            constexpr int VPR = DV / 8;
            for (int idx = tid; idx < C * VPR; idx += kFusedThreads) {
                const int row = idx / VPR, cv = idx % VPR;
                const int grow = n * C + row;
                if (grow < p.N)
                    *reinterpret_cast<uint4*>(og + seq_v + (size_t)grow * DV + cv * 8) =
                        *reinterpret_cast<const uint4*>(Ost + (size_t)row * PO + cv * 8);
            }
        }
    }

#ifdef HGRN2_PHASE_TIMING
    HGRN2_STAMP(9);
    if (lane == 0 && p.dbg)
        for (int k = 0; k < 16; ++k) p.dbg[((size_t)bh * NW + w) * 16 + k] = ph[k];
#endif
    if (p.hT) {
        float* s1 = p.hT + (size_t)bh * DK * DV;
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v)
                s1[(size_t)(32 * (at0 + j) + acc_row(v, lane)) * DV + 32 * bt + r32] = accS[j][v];
    }
}

bool fwd_fused_supported(const SeqDims& d)
{
    return d.io_bf16 && d.dk == 128 && d.dv == 128 && d.BH >= 64;
}

hipError_t launch_fwd_fused(const SeqDims& d, const void* q, const void* f, const void* v, const float* h0,
                            void* o, float* hT, hipStream_t stream)
{
    if (d.BH == 0) return hipSuccess;
    typedef FwdFusedLds<128, 128> L;
    FwdFusedParams p;
    p.q = q; p.f = f; p.v = v; p.h0 = h0; p.o = o; p.hT = hT;
    p.N = d.N; p.NC = d.NC; p.gate_bf16 = d.gate_bf16 ? 1 : 0;
    auto kern = fwd_fused_kernel<128, 128>;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)L::total);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3(d.BH), dim3(kFusedThreads), L::total, stream, p);
    return hipGetLastError();
}

}   // namespace hgrn2
