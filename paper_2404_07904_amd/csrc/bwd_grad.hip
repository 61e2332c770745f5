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
// in which no term cancels against another.  The first two lines are the suffix sum of
// e'_i = Q~_i X_i - K~_i Y1_i with X = dP K~ + dO (G_m S_n)^T and Y1 = dP^T Q~, the third the
// exclusive prefix sum of K~_j Ks_j with Ks = V (H_m dS)^T, the fourth is R.
//
// LDS instructions cost about the same whatever their width, so the kernel is laid out to need
// few of them: V and dO travel from global memory to their LDS tiles as raw 16-byte vectors,
// with the columns inside every group of 16 stored in the order the state fragments keep their
// contraction index (bits 2 and 3 of the index swapped), so that the matching MFMA operand is
// one 16-byte read; the accumulators of the 64 x dk results are kept transposed (channel in the
// register index), so that they reach their fp32 staging tiles as 16-byte vectors.
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

constexpr int kMaxLightRuns = 4;
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
    int BH, N, NC;
    const float* beta;       // [H][dk] lower bounds, or null: the gate tensor holds f itself
    float* beta_partials;    // [B*H*NC][8][dk] per-wave partial sums of the gradient w.r.t. beta
    int H;
    TokenLayout lay;         // used when dense == 0
    int dense;               // sequence tensors are [B][H][N][d]
    // Fused reverse walk (see bwd_grad_body<..., FUSED>): the state gradient is carried in registers
    // instead of being read from ws_ds.  Every sequence is cut into R runs of rc chunks, one
    // workgroup each; a run starts from grad_hT (the last one), from bound0[bh] (run 0) or from
    // run_state[bh * seg_tail + r * s_sub - 1] (the state gradient at the end of run r, which a
    // zero-start sweep over the later tokens and its carry have left there); run 0 leaves grad_h0.
    // With few runs (`light`), no boundary states are needed: a workgroup first walks the chunks
    // after its run, from grad_hT, doing nothing but the state-gradient recurrence (a fraction of a
    // chunk's full work), and the runs are cut at bnd[0] = 0 < bnd[1] < ... < bnd[R] = NC so that
    // all workgroups finish together.
    const float* dhT;
    float* dh0;
    const float* bound0;
    const float* run_state;
    int R, rc, s_sub, seg_tail;
    int light;
    int bnd[kMaxLightRuns + 1];
    int* flag;               // null, or set to 1 when a gate product falls below the floor of the reciprocals
};


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
    static constexpr size_t cmax(size_t a, size_t b) { return a > b ? a : b; }
    // phase 1: operand tiles
    static constexpr size_t qm = 0;                                         // Q~   [C][PK]
    static constexpr size_t km = qm + (size_t)C * PK * sizeof(T);           // K~   [C][PK]
    static constexpr size_t vm = km + (size_t)C * PK * sizeof(T);           // V    [C][PVR]  (columns permuted)
    static constexpr size_t dom = vm + (size_t)C * PVR * sizeof(T);         // dO   [C][PV]   (columns permuted)
    static constexpr size_t dsm = dom + (size_t)C * PV * sizeof(T);         // H_m * dS  [DK][PV] (columns permuted)
    static constexpr size_t pt = dsm + (size_t)DK * PV * sizeof(T);         // P^T  [C][PC]  ([j][i])
    static constexpr size_t dpt = pt + (size_t)C * PC * sizeof(T);          // dP^T [C][PC]
    static constexpr size_t tot = dpt + (size_t)C * PC * sizeof(T);         // [8][DK] fp32 block products
    static constexpr size_t p1_end = tot + (size_t)kBwdWaves * DK * sizeof(float);
    // phase 2 (aliases phase 1): fp32 staging of X, Y1, Ks and the block sums of the epilogue
    static constexpr size_t cx = 0;                                         // [C][PF] fp32
    static constexpr size_t cy = cx + (size_t)C * PF * sizeof(float);
    static constexpr size_t cks = cy + (size_t)C * PF * sizeof(float);
    static constexpr size_t blke = cks + (size_t)C * PF * sizeof(float);    // [8][DK] fp32 block sums of e'
    static constexpr size_t blkk = blke + (size_t)kBwdWaves * DK * sizeof(float);   // [8][DK] block sums of K~ Ks
    static constexpr size_t p2_end = blkk + (size_t)kBwdWaves * DK * sizeof(float);
    // The next chunk's first stage writes the V, dO tiles and the block products while the last
    // stage of this one may still read the block sums; where those overlap, a barrier ends the chunk.
    static constexpr bool end_barrier = !(blke >= dsm && p2_end <= tot);
    // both phases
    static constexpr size_t rp = cmax(p1_end, p2_end);                      // [DK] fp32  g * rowsum(dS * S_n)
    static constexpr size_t dvs = rp + (size_t)DK * sizeof(float);          // dv staging [C][PVR]
    static constexpr size_t one = dvs + (size_t)C * PVR * sizeof(T);        // [DK] fp32, all 1.0 (neutral factor)
    static constexpr size_t zero = one + (size_t)DK * sizeof(float);        // [DK] fp32, all 0.0 (neutral term)
    static constexpr size_t total = zero + (size_t)DK * sizeof(float);
    static_assert(total <= 160 * 1024, "LDS budget of one workgroup");
};

// FUSED: the workgroup owns run `r` of sequence `bh` and walks its chunks from the last to the
// first with the state gradient in fp32 MFMA accumulators, oriented [dv][channel]:
//     E_n = D'_n + Q~_n^T dO_n ,   D'_n = (g_n / G_m,n) dS_{n+1} ,   dS_n = G_m,n E_n
// so that before each chunk the accumulators are scaled by (second-half gate product of this
// chunk) x (first-half gate product of the chunk just done), published to the LDS tile the
// contractions read D' from, and after the chunk's contractions receive Q~^T dO.  Only the forward
// states S_n come from the workspace.
// GROUPED (a FUSED walk over a packed batch): the chunks of one head, sequence after sequence, are
// cut into `spans` equal pieces and the workgroup owns one, which may start and end inside a
// sequence.  It walks its chunks from the last to the first: the state gradient starts from a
// sequence's grad_hT (or zero) at its last chunk and leaves as its grad_h0 after its first, and the
// rows of the next chunk of the walk -- be it of the sequence before -- are always in flight during
// the epilogue of the current one.  A span that ends inside a sequence first takes the light walk
// over the chunks between its end and the sequence's, which yields the state gradient it starts from.
template <typename T, int DK, int DV, bool GATE_BF16, bool DENSE, bool FUSED, bool GROUPED = false>
__device__ __forceinline__ void bwd_grad_body(const BwdGradParams& p)
{
    static_assert(!GROUPED || (FUSED && !DENSE), "groups: fused walk over a packed batch");
    constexpr int C = kChunk, NW = kBwdWaves, RW = C / NW;
    typedef BwdGradLds<T, DK, DV> L;
    constexpr int PK = L::PK, PV = L::PV, PVR = L::PVR, PC = L::PC, PF = L::PF;
    constexpr int NRT = C / 32, NAT = DK / 32, NBT = DV / 32;
    static_assert(NRT == 2 && NRT * NAT <= NW && NRT * NBT <= NW, "one tile per wave");
    typedef Mma<T> M;
    typedef typename M::frag frag;
    typedef T tx2 __attribute__((ext_vector_type(2)));
    typedef T tx4 __attribute__((ext_vector_type(4)));
    constexpr bool io_bf16 = is_bf16_type<T>();
    constexpr int VEC = 16 / (int)sizeof(T);            // elements per 16-byte vector

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
    float* cX = reinterpret_cast<float*>(smem + L::cx);
    float* cY = reinterpret_cast<float*>(smem + L::cy);
    float* cKs = reinterpret_cast<float*>(smem + L::cks);
    float* blkE = reinterpret_cast<float*>(smem + L::blke);
    float* blkK = reinterpret_cast<float*>(smem + L::blkk);
    T* dVs = reinterpret_cast<T*>(smem + L::dvs);
    float* ones = reinterpret_cast<float*>(smem + L::one);
    float* zeros = reinterpret_cast<float*>(smem + L::zero);

    if (not_chosen(p.lay)) return;       // (a packed batch whose table chose the other backward pass; a chunk length not called for)
    const int tid = threadIdx.x;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);      // wave index, in a scalar register
    constexpr bool gate_bf16 = GATE_BF16;
    constexpr int GES = GATE_BF16 ? 2 : 4;
    const T* qg = static_cast<const T*>(p.q);
    const T* vg = static_cast<const T*>(p.v);
    const T* dog = static_cast<const T*>(p.dO);

    // tile ownership (a wave without a tile of a kind skips that work)
    const bool has_a = (NRT * NAT == NW) || w < NRT * NAT, has_b = (NRT * NBT == NW) || w < NRT * NBT;
    const bool after = w >= NW / 2;          // rows of this wave lie after the mid-chunk reference
    const int rt_a = has_a ? w / NAT : 0, at = w % NAT;     // (row tile, channel tile) of dq / dk
    const int rt_b = has_b ? w / NBT : 0, bt = w % NBT;     // (row tile, column tile) of dv

    // V and dO tiles: one (row, 16-column group) per thread, 32 bytes
    constexpr int GPR = DV / 16;
    const bool vd_act = tid < C * GPR;
    const int vd_row = vd_act ? tid / GPR : 0, vd_grp = tid % GPR;

    // Everything one chunk needs from global memory: the raw rows of f, q of this wave's row block,
    // this thread's 32 bytes of V and dO, and the state fragments of channel tile `at` (operand
    // B[k = dv index][n = channel]).  The workgroup is persistent: it walks the chunks blockIdx.x,
    // blockIdx.x + gridDim.x, ... and issues the row loads of its next chunk as soon as the matrix
    // stage of the current one is done, so that they fly during the element-wise epilogue; the
    // state fragments are requested at the top of a chunk and are not needed before its own
    // element-wise stage is over.  Rows past the end of a sequence re-read its last row: their
    // gates are replaced by one and their q by zero, which makes whatever finite values stand in
    // for V and dO there drop out of every stored result.
    // chunk index -> sequence and chunk within it (every chunk index handed in is a valid one)
    // chunk index -> sequence and chunk within it (every chunk index handed in is a valid one);
    // found once per chunk, when its rows are requested, and kept for the chunk's own pass
    struct ChunkAt { SeqView sv; int bh, n; };
    int seq_hint = 0;         // the workgroup asks for chunk indices in non-decreasing order
    auto where = [&](int chunk) {
        ChunkAt c;
        locate_chunk<DENSE>(p.lay, p.BH, p.NC, chunk, c.bh, c.n, &seq_hint);
        c.sv = seq_view<DENSE, DK, DV>(p.lay, p.N, p.NC, c.bh);
        return c;
    };
    // the token whose V / dO row this thread copies into row vd_row of the tiles (a row that stands for
    // no token re-reads a neighbouring one: what it holds drops out of every stored result)
    auto tile_token = [&](const ChunkAt& c) {
        return min(max(chunk_rows(p.lay.sub, c.n, c.sv.N).tok0 + vd_row, 0), c.sv.N - 1);
    };
    auto load_fq_rows = [&](RawRows<RW>& cf, RawRows<RW>& cq, const ChunkAt& c, int lane) {
        const int col_k = (2 * lane < DK) ? 2 * lane : 0;
        const int r0 = chunk_rows(p.lay.sub, c.n, c.sv.N).tok0 + RW * w;
        load_rows_clamped<RW, GATE_BF16>(cf, static_cast<const char*>(p.f) + c.sv.off_k * GES, r0, c.sv.N - 1, DENSE ? DK : (int)p.lay.sn_k, col_k);
        load_rows_clamped<RW, io_bf16>(cq, reinterpret_cast<const char*>(qg + c.sv.off_k), r0, c.sv.N - 1, DENSE ? DK : (int)p.lay.sn_k, col_k);
    };
    auto load_chunk_rows = [&](RawRows<RW>& cf, RawRows<RW>& cq, Raw16<T>& cv, Raw16<T>& cd, const ChunkAt& c, int lane) {
        load_fq_rows(cf, cq, c, lane);
        const size_t vo = c.sv.off_v + (size_t)tile_token(c) * (DENSE ? (size_t)DV : (size_t)p.lay.sn_v) + 16 * vd_grp;
        cv.load(vg + vo);
        cd.load(dog + vo);
    };
    auto load_chunk_states = [&](frag (&cS)[2 * NBT], frag (&cD)[2 * NBT], int chunk, int lane) {
        const size_t slot = (size_t)chunk * DK * DV;
        const T* wsS = static_cast<const T*>(p.ws_s) + slot;
        const T* wsD = static_cast<const T*>(p.ws_ds) + slot;
#pragma unroll
        for (int kk = 0; kk < 2 * NBT; ++kk) {
            cS[kk] = *reinterpret_cast<const frag*>(wsS + state_frag_offset(at, kk >> 1, NBT, kk & 1, lane));
            if constexpr (!FUSED) cD[kk] = *reinterpret_cast<const frag*>(wsD + state_frag_offset(at, kk >> 1, NBT, kk & 1, lane));
        }
    };

    int n_chunks = p.BH * p.NC;
    if constexpr (!DENSE) {
        if (p.lay.vl) n_chunks = table_read(p.lay.vl, 2 * (p.lay.B + 1) + p.lay.B) * p.lay.H;      // the table's total, not the host's bound
    }
    // GROUPED: a span of the chunks of head g_head; chunk (e, n) of the walk as a ChunkAt
    int g_head = 0;
    auto chunk_en = [&](int e, int n) {
        ChunkAt c;
        c.bh = e * p.lay.H + g_head;
        c.n = n;
        c.sv = seq_view<DENSE, DK, DV>(p.lay, p.N, p.NC, c.bh);
        return c;
    };
    // the chunk the walk visits after c: the one before it in its sequence, else the last chunk of
    // the nearest earlier sequence of the group that has tokens; after the very last one, c again
    auto walk_next = [&](const ChunkAt& c) {
        if (c.n > 0) { ChunkAt r = c; r.n = c.n - 1; return r; }
        for (int e = c.bh / p.lay.H - 1; e >= 0; --e) {
            const int len = table_read(p.lay.vl, p.lay.B + 1 + e);
            if (len > 0) return chunk_en(e, p.lay.chunks_of(len) - 1);
        }
        return c;
    };
    RawRows<RW> raw_f, raw_q;
    Raw16<T> raw_v, raw_d;
    frag sS[2 * NBT], sD[2 * NBT];
    // chunks of this workgroup: every gridDim.x-th one, or (FUSED) those of its run, last to first
    int n_iter, f_bh = 0, f_run = 0, f_first = 0, f_last = 0;
    int span_end = 0;                     // GROUPED: one past the last chunk of the span, counted over the head's chunks
    if constexpr (GROUPED) {
        if ((int)blockIdx.x >= p.lay.spans * p.lay.H) return;
        const int grp = (int)blockIdx.x / p.lay.H;
        g_head = (int)blockIdx.x - grp * p.lay.H;
        const int total = table_read(p.lay.vl, 2 * (p.lay.B + 1) + p.lay.B);       // chunks of one head
        const int span_start = (int)((long long)grp * total / p.lay.spans);
        span_end = (int)((long long)(grp + 1) * total / p.lay.spans);
        n_iter = span_end - span_start;
        // a sequence without tokens hands the gradient of its final state on to its initial state
        // (such sequences lie in no span: they are dealt out by their number)
        if (p.dh0)
            for (int e = grp; e < p.lay.B; e += p.lay.spans)
                if (table_read(p.lay.vl, p.lay.B + 1 + e) == 0)
                    for (int i = tid; i < DK * DV; i += kBwdThreads) {
                        const size_t x = (size_t)(e * p.lay.H + g_head) * DK * DV + i;
                        p.dh0[x] = p.dhT ? p.dhT[x] : 0.0f;
                    }
    } else if constexpr (FUSED) {
        f_bh = (int)blockIdx.x / p.R;
        f_run = (int)blockIdx.x - f_bh * p.R;
        if (f_bh >= p.BH) return;
        if (p.light) {
            f_first = p.bnd[f_run];
            f_last = p.bnd[f_run + 1] - 1;
        } else {
            f_first = f_run * p.rc;
            f_last = min(p.NC, f_first + p.rc) - 1;
        }
        n_iter = f_last - f_first + 1;
    } else {
        if ((int)blockIdx.x >= n_chunks) return;
        n_iter = (n_chunks - (int)blockIdx.x + (int)gridDim.x - 1) / (int)gridDim.x;
    }
    auto chunk_of = [&](int it) {         // global chunk index of iteration `it`, clamped to the workgroup's last one
        if constexpr (FUSED) return f_bh * p.NC + max(f_last - it, f_first);
        else return min((int)blockIdx.x + it * (int)gridDim.x, n_chunks - 1);
    };

    // FUSED: accumulator tiles of the state gradient owned by this wave, tile id w + 8 j -> (channel
    // tile id % NAT, which is this wave's `at`; dv tile id / NAT), as [dv][channel]
    constexpr int NDT = NAT * NBT, TPW = (NDT + NW - 1) / NW;
    const bool has_d = FUSED && ((NDT % NW == 0) || w < NDT);
    f32x16 accD[FUSED ? TPW : 1];
    float gm_prev = 1.0f;                 // first-half gate product of the chunk done before, channel 32 at + lane % 32
    // Element (tile j, register v) of this lane in a [dk][dv] fp32 state: a wave-uniform address
    // (sequence, dv tile, group of four registers) plus one per-lane 32-bit byte offset plus a small
    // constant, so that no access needs an address register of its own (GROUPED walks read and write
    // such states in the middle of the chunk loop, where registers are scarce).
    const uint32_t st_lane = (uint32_t)((32 * at + (tid & 31)) * DV + 4 * ((tid >> 5) & 1)) * 4u;
    auto state_cols = [&](const float* base, int seq, int j, int c) {
        return reinterpret_cast<const char*>(base) + ((size_t)seq * DK * DV + (size_t)(32 * ((w + NW * j) / NAT) + 8 * c)) * 4;
    };
    if constexpr (FUSED && !GROUPED) {
        const int r32i = tid & 31, gi = (tid >> 5) & 1;
        const float* init = (f_run == p.R - 1 || p.light) ? p.dhT : (f_run == 0) ? p.bound0 : p.run_state;
        if (init) {
            if (f_run == p.R - 1 || f_run == 0 || p.light) init += (size_t)f_bh * DK * DV;
            else init += ((size_t)f_bh * p.seg_tail + (size_t)f_run * p.s_sub - 1) * DK * DV;
        }
#pragma unroll
        for (int j = 0; j < TPW; ++j) {
            const int btj = (w + NW * j) / NAT;
#pragma unroll
            for (int v = 0; v < 16; ++v)
                accD[j][v] = (init && has_d) ? init[(size_t)(32 * at + r32i) * DV + 32 * btj + 8 * (v >> 2) + 4 * gi + (v & 3)] : 0.0f;
        }
    }
    // FUSED walks over one run add up their partial sums of the gradient w.r.t. beta chunk after chunk
    // (a fixed order) and leave one row per wave and run, in the slot of chunk `run` of the sequence.
    constexpr bool RUN_BETA = FUSED && !GROUPED;
    float run_b0 = 0.0f, run_b1 = 0.0f;
    auto store_run_beta = [&]() {
        const int lane = threadIdx.x & 63;
        if (RUN_BETA && p.beta && 2 * lane < DK)
            *reinterpret_cast<f32x2*>(p.beta_partials + ((size_t)(f_bh * p.NC + f_run) * NW + w) * DK + 2 * lane) = f32x2{run_b0, run_b1};
    };
    if (n_iter <= 0) {                    // (FUSED) a sequence without tokens: the host routes those elsewhere
        store_run_beta();
        return;
    }
    for (int i = tid; i < DK; i += kBwdThreads) { ones[i] = 1.0f; zeros[i] = 0.0f; }    // first read after a barrier
    ChunkAt cur;
    bool rows_loaded = false;
    float below_floor = 1.0f;             // smallest product a reciprocal was taken of (reported once, at the end)
    if constexpr (FUSED) {
        int n_light = 0;
        if constexpr (GROUPED) {
            // the sequence the span ends in (found by the table kernel): the last one whose chunks
            // start at or before the span's last chunk
            const int* before = p.lay.vl + 2 * (p.lay.B + 1);
            const int lo = min(max(table_read(p.lay.span_seq, (int)blockIdx.x / p.lay.H), 0), p.lay.B - 1);
            const int nc_e = table_read(before, lo + 1) - table_read(before, lo);
            cur = chunk_en(lo, nc_e - 1);                          // that sequence's last chunk
            n_light = table_read(before, lo + 1) - span_end;       // its chunks after the span
            if (n_light > 0) {
                // the light walk starts from the sequence's grad_hT (the chunk loop does that itself
                // for every sequence whose last chunk lies in the span)
#pragma unroll
                for (int j = 0; j < TPW; ++j)
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        const char* cols = state_cols(p.dhT, cur.bh, j, c);
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            accD[j][4 * c + e] = (p.dhT && has_d) ? *reinterpret_cast<const float*>(cols + st_lane + 4 * e) : 0.0f;
                    }
            }
        } else {
            n_light = p.light ? p.NC - 1 - f_last : 0;
            if (n_light > 0) cur = where(f_bh * p.NC + p.NC - 1);
        }
        if (n_light > 0) {
            // ---- light walk over the chunks after this run: dS_n = Diag(g_n) dS_{n+1} + Q^_n^T dO_n with
            // Q^ = q G (G the gate product from the chunk start: no quotient), true state gradient in
            // the accumulators.  Three barriers per chunk; the Q~ and dO tiles and the block totals are reused.
            auto load_light = [&](RawRows<RW>& cf, RawRows<RW>& cq, Raw16<T>& cd, const ChunkAt& c, int lane) {
                load_fq_rows(cf, cq, c, lane);
                const size_t vo = c.sv.off_v + (size_t)tile_token(c) * (DENSE ? (size_t)DV : (size_t)p.lay.sn_v) + 16 * vd_grp;
                cd.load(dog + vo);
            };
            load_light(raw_f, raw_q, raw_d, cur, tid & 63);
            for (int li = 0; li < n_light; ++li) {
                int lane_opaque = threadIdx.x & 63;
                asm volatile("" : "+v"(lane_opaque));
                const int lane = lane_opaque, r32 = lane & 31;
                const bool k_act = 2 * lane < DK;
                if (vd_act) raw_d.store_swapped(dOm + (size_t)vd_row * PV + 16 * vd_grp);
                const ChunkRows lr = chunk_rows(p.lay.sub, cur.n, cur.sv.N);
                const int row0 = lr.tok0 + RW * w;
                f32x2 rf[RW], rq[RW];
                convert_rows<RW>(rf, raw_f, row0, lr.end, k_act, gate_bf16, 1.0f, lr.first);
                if (p.beta) gate_rows<RW>(rf, p.beta + (size_t)(cur.bh % p.H) * DK, k_act ? 2 * lane : 0, k_act, row0, lr.end, lr.first);
                convert_rows<RW>(rq, raw_q, row0, lr.end, k_act, io_bf16, 0.0f, lr.first);
                float a0[RW], a1[RW], t0 = 1.0f, t1 = 1.0f;
#pragma unroll
                for (int i = 0; i < RW; ++i) { t0 *= rf[i].x; t1 *= rf[i].y; a0[i] = t0; a1[i] = t1; }
                if (k_act) *reinterpret_cast<f32x2*>(tot + w * DK + 2 * lane) = f32x2{t0, t1};
                __syncthreads();
                // rows of the next chunk of the walk (after the last light chunk: the run's own last chunk)
                RawRows<RW> nxt_f, nxt_q;
                ChunkAt nxt = cur;            // the chunk before, in the same sequence
                nxt.n = cur.n - 1;
                load_light(nxt_f, nxt_q, raw_d, nxt, lane);
                if (k_act) {
                    float pre0 = 1.0f, pre1 = 1.0f;
#pragma unroll
                    for (int i = 0; i < NW - 1; ++i) {
                        const float* src = (i < w) ? tot + i * DK : ones;       // wave-uniform row address
                        const f32x2 t = *reinterpret_cast<const f32x2*>(src + 2 * lane);
                        pre0 *= t.x; pre1 *= t.y;
                    }
#pragma unroll
                    for (int i = 0; i < RW; ++i) {
                        tx2 x;
                        x.x = (T)(rq[i].x * (pre0 * a0[i])); x.y = (T)(rq[i].y * (pre1 * a1[i]));
                        *reinterpret_cast<tx2*>(Qm + (size_t)(RW * w + i) * PK + 2 * lane) = x;
                    }
                }
                float g_all = 1.0f;
                if (has_d) {
#pragma unroll
                    for (int i = 0; i < NW; ++i) g_all *= tot[i * DK + 32 * at + r32];
                }
                __syncthreads();
                if (has_d) {
#pragma unroll
                    for (int j = 0; j < TPW; ++j)
#pragma unroll
                        for (int v = 0; v < 16; ++v) accD[j][v] *= g_all;
#pragma unroll
                    for (int ks = 0; ks < 2 * NRT; ++ks) {
                        const frag qf = M::load_kmajor(Qm, PK, 16 * ks, 32 * at, lane);
#pragma unroll
                        for (int j = 0; j < TPW; ++j)
                            M::mma(accD[j], M::load_kmajor_swapped(dOm, PV, 16 * ks, 32 * ((w + NW * j) / NAT), lane), qf);
                    }
                }
                raw_f = nxt_f;
                raw_q = nxt_q;
                cur = nxt;
                __syncthreads();          // the tiles and totals are free for the next chunk
            }
            // what the full pass over the run's last chunk needs on top: its V rows
            const size_t vo = cur.sv.off_v + (size_t)tile_token(cur) * (DENSE ? (size_t)DV : (size_t)p.lay.sn_v) + 16 * vd_grp;
            raw_v.load(vg + vo);
            rows_loaded = true;
        }
    }
    if constexpr (GROUPED) {
        // Keeps the compiler from computing the chunk loop's lane-dependent values ahead of the light
        // walk and carrying them through it in registers (which made the loop spill, and a reload in
        // the loop waits for every load in flight, the next chunk's rows included).
        int opaque = threadIdx.x & 63;
        asm volatile("" : "+v"(opaque));
    }
    if (!rows_loaded) {
        if constexpr (!GROUPED) cur = where(chunk_of(0));     // (a span: its last chunk, found above)
        load_chunk_rows(raw_f, raw_q, raw_v, raw_d, cur, tid & 63);
    }

  for (int it = 0; it < n_iter; ++it) {
    const int chunk = GROUPED ? (int)cur.sv.chunk0 + cur.n : chunk_of(it);
    // Re-derive the lane-dependent indices inside the loop from a value the compiler cannot see
    // through: otherwise it hoists dozens of loop-invariant LDS addresses out of the loop, keeps
    // them in registers across the whole body and spills.
    int lane_opaque = threadIdx.x & 63;
    asm volatile("" : "+v"(lane_opaque));
    const int lane = lane_opaque, r32 = lane & 31, g = lane >> 5;
    const bool k_act = 2 * lane < DK;
    const int n = cur.n, bh = cur.bh;
    const size_t seq_k = cur.sv.off_k, seq_v = cur.sv.off_v;
    const int N = cur.sv.N;
    const size_t ld_k = DENSE ? (size_t)DK : (size_t)p.lay.sn_k, ld_v = DENSE ? (size_t)DV : (size_t)p.lay.sn_v;
    load_chunk_states(sS, sD, chunk, lane);      // first needed two barriers from here; covered by the element-wise stage

    // V, dO tiles: raw bits, the four 4-column quads of a 16-column group stored in the order
    // (0, 2, 1, 3), i.e. column b at position b with bits 2 and 3 swapped
    if (vd_act) {
        raw_v.store_swapped(Vm + (size_t)vd_row * PVR + 16 * vd_grp);
        raw_d.store_swapped(dOm + (size_t)vd_row * PV + 16 * vd_grp);
    }
    // rf is re-derived from the raw rows in the epilogue (the raw bf16 pairs cost half the registers)
    const ChunkRows cr = chunk_rows(p.lay.sub, n, N);     // which tokens the chunk's rows stand for
    const int row0 = cr.tok0 + RW * w;
    f32x2 rf[RW], rq[RW];
    convert_rows<RW>(rf, raw_f, row0, cr.end, k_act, gate_bf16, 1.0f, cr.first);
    if (p.beta) gate_rows<RW>(rf, p.beta + (size_t)(bh % p.H) * DK, k_act ? 2 * lane : 0, k_act, row0, cr.end, cr.first);
    convert_rows<RW>(rq, raw_q, row0, cr.end, k_act, io_bf16, 0.0f, cr.first);

    // ---------------- gate products; scaled operand tiles ----------------
    // With a = inclusive gate product from the start of this wave's 8-row block, z = exclusive
    // product to its end, t = a z the block total, mid = product of the blocks between this block
    // and the mid-chunk reference row, and m = product of the gates between the reference row and
    // this row:
    //   rows after the reference:  Q~ = q m,   K~ = k / m,   m = mid a,  1/m = z / (mid t)
    //   rows before it:            Q~ = q / m, K~ = k m,     m = mid z,  1/m = a / (mid t)
    // so sq = Q~/q = s_a a and sk = K~/k = s_z z with per-channel block factors s_a, s_z in
    // {mid, 1/(mid t)}: one reciprocal per channel and block, with a floor added under it so that
    // it stays finite outside the supported gate range.  a, z, s_a, s_z are kept for the
    // epilogue (dq = sq * (...), dk = sk * (...)).
    float a0[RW], a1[RW], z0[RW], z1[RW], sa0 = 1.0f, sa1 = 1.0f, sz0 = 1.0f, sz1 = 1.0f;
    tx2 qb[RW], kb[RW];         // Q~, K~ of this thread's elements exactly as rounded for the MFMAs (epilogue)
    {
        float t0 = 1.0f, t1 = 1.0f;
#pragma unroll
        for (int i = 0; i < RW; ++i) { t0 *= rf[i].x; t1 *= rf[i].y; a0[i] = t0; a1[i] = t1; }
        float u0 = 1.0f, u1 = 1.0f;
#pragma unroll
        for (int i = RW - 1; i >= 0; --i) { z0[i] = u0; z1[i] = u1; u0 *= rf[i].x; u1 *= rf[i].y; }
        if (k_act) *reinterpret_cast<f32x2*>(tot + w * DK + 2 * lane) = f32x2{t0, t1};
        __syncthreads();
        if (k_act) {
            // product of the (at most three) block totals between this block and the reference
            // row; the row addresses are wave-uniform, an absent factor reads the row of ones
            const float* r1 = after ? (w > 4 ? tot + 4 * DK : ones) : (w < 3 ? tot + 3 * DK : ones);
            const float* r2 = after ? (w > 5 ? tot + 5 * DK : ones) : (w < 2 ? tot + 2 * DK : ones);
            const float* r3 = after ? (w > 6 ? tot + 6 * DK : ones) : (w < 1 ? tot + 1 * DK : ones);
            const f32x2 m1 = *reinterpret_cast<const f32x2*>(r1 + 2 * lane);
            const f32x2 m2 = *reinterpret_cast<const f32x2*>(r2 + 2 * lane);
            const f32x2 m3 = *reinterpret_cast<const f32x2*>(r3 + 2 * lane);
            const float mid0 = m1.x * m2.x * m3.x, mid1 = m1.y * m2.y * m3.y;
            const float R0 = fast_rcp(fmaxf(mid0 * t0, kTinyProduct)), R1 = fast_rcp(fmaxf(mid1 * t1, kTinyProduct));
            below_floor = fminf(below_floor, fminf(mid0 * t0, mid1 * t1));
            sa0 = after ? mid0 : R0; sa1 = after ? mid1 : R1;
            sz0 = after ? R0 : mid0; sz1 = after ? R1 : mid1;
#pragma unroll
            for (int i = 0; i < RW; ++i) {
                const int row = RW * w + i;
                qb[i].x = (T)(rq[i].x * (sa0 * a0[i])); qb[i].y = (T)(rq[i].y * (sa1 * a1[i]));
                kb[i].x = (T)((1.0f - rf[i].x) * (sz0 * z0[i])); kb[i].y = (T)((1.0f - rf[i].y) * (sz1 * z1[i]));
                *reinterpret_cast<tx2*>(Qm + (size_t)row * PK + 2 * lane) = qb[i];
                *reinterpret_cast<tx2*>(Km + (size_t)row * PK + 2 * lane) = kb[i];
            }
        } else {
#pragma unroll
            for (int i = 0; i < RW; ++i) { qb[i] = tx2{(T)0.0f, (T)0.0f}; kb[i] = qb[i]; }
        }
    }
    // H_m * dS_{n+1} of channel tile `at` -> LDS, row-major [channel][dv position] (the fragments hold
    // it already scaled and rounded, and in position order: their bits go to LDS as they are), and
    // R = rowsum((H_m dS) * (G_m S_n)) = g * rowsum(dS * S_n).  Once per channel tile (row tile 0).
    if constexpr (GROUPED) {
        // the walk enters a sequence at its last chunk: the state gradient starts from its grad_hT
        if (cur.n == cur.sv.NC - 1) {
            gm_prev = 1.0f;
#pragma unroll
            for (int j = 0; j < TPW; ++j)
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const char* cols = state_cols(p.dhT, cur.bh, j, c);
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        accD[j][4 * c + e] = (p.dhT && has_d) ? *reinterpret_cast<const float*>(cols + st_lane + 4 * e) : 0.0f;
                }
        }
    }
    if constexpr (FUSED) {
        // scale the carried state gradient to D'_n and publish it as the bf16 tile the contractions read
        if (has_d) {
            const int ch = 32 * at + r32;
            const float hn = (tot[4 * DK + ch] * tot[5 * DK + ch]) * (tot[6 * DK + ch] * tot[7 * DK + ch]);
            const float gm = (tot[0 * DK + ch] * tot[1 * DK + ch]) * (tot[2 * DK + ch] * tot[3 * DK + ch]);
            const float c = hn * gm_prev;
            gm_prev = gm;
#pragma unroll
            for (int j = 0; j < TPW; ++j) {
                const int btj = (w + NW * j) / NAT;
#pragma unroll
                for (int v = 0; v < 16; ++v) accD[j][v] *= c;
#pragma unroll
                for (int half = 0; half < 2; ++half) {
                    float x[8];
#pragma unroll
                    for (int e = 0; e < 8; ++e) x[e] = accD[j][8 * half + e];
                    *reinterpret_cast<frag*>(dSm + (size_t)ch * PV + 32 * btj + 16 * half + 8 * g) = M::pack(x);
                }
            }
        }
    }
    if (!FUSED && w < NAT) {
        const int ch = 32 * at + r32;
        f32x16 accR;
#pragma unroll
        for (int v = 0; v < 16; ++v) accR[v] = 0.0f;
#pragma unroll
        for (int kk = 0; kk < 2 * NBT; ++kk) {
            M::mma(accR, sS[kk], sD[kk]);          // [channel a][channel a'] = sum_b S'[a][b] D'[a'][b]; R is its diagonal
            *reinterpret_cast<frag*>(dSm + (size_t)ch * PV + 16 * kk + 8 * g) = sD[kk];
        }
        // diagonal element of column r32: accumulator register 4 (r32 / 8) + r32 % 4 of the lane group (r32 / 4) % 2
        const int vsel = 4 * (r32 >> 3) + (r32 & 3);
        float rs = 0.0f;
#pragma unroll
        for (int v = 0; v < 16; ++v) rs = (v == vsel) ? accR[v] : rs;
        if (g == ((r32 >> 2) & 1)) Rp[ch] = rs;
    }
    __syncthreads();

    if constexpr (FUSED) {
        // R on the last NAT waves, D'_n of their channel tile read back from the tile as operand fragments
        if (w >= NW - NAT) {
            f32x16 accR;
#pragma unroll
            for (int v = 0; v < 16; ++v) accR[v] = 0.0f;
#pragma unroll
            for (int kk = 0; kk < 2 * NBT; ++kk)
                M::mma(accR, sS[kk], *reinterpret_cast<const frag*>(dSm + (size_t)(32 * at + r32) * PV + 16 * kk + 8 * g));
            const int vsel = 4 * (r32 >> 3) + (r32 & 3);
            float rs = 0.0f;
#pragma unroll
            for (int v = 0; v < 16; ++v) rs = (v == vsel) ? accR[v] : rs;
            if (g == ((r32 >> 2) & 1)) Rp[32 * at + r32] = rs;
        }
    }

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
            tx4 pk;
#pragma unroll
            for (int ii = 0; ii < 4; ++ii) pk[ii] = (T)((j_glob <= i0 + ii) ? acc0[4 * c + ii] + acc1[4 * c + ii] : 0.0f);
            *reinterpret_cast<tx4*>(dst + (size_t)j_glob * PC + i0) = pk;
        }
    } else {
        T* dst = (w == 6) ? Pt : dPt;    // rows 32..63, columns 0..31: 32 x 32 values, 16 per lane
        const u32x4 z = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int k = 0; k < 16 / VEC; ++k)
            *reinterpret_cast<u32x4*>(dst + (size_t)(32 + (lane >> 1)) * PC + 16 * (lane & 1) + VEC * k) = z;
    }
    __syncthreads();

    // ---------------- main contractions ----------------
    // dv tile (rt_b, bt) first: P^T dO over the chunk and K~ (H_m dS) over the channels (the masked
    // halves of P^T / dP^T are zero, so every contraction runs over the full chunk with no
    // branches).  It goes to its staging area at once, which frees its registers.  Its columns
    // come out in the position order of the dO and dS tiles and are put back here.
    if (has_b) {
        f32x16 aV, aV2;
#pragma unroll
        for (int v = 0; v < 16; ++v) { aV[v] = 0.0f; aV2[v] = 0.0f; }
#pragma unroll
        for (int ks = 0; ks < 2 * NRT; ++ks)
            M::mma(aV2, M::load_kmajor(dOm, PV, 16 * ks, 32 * bt, lane), M::load(Pt + (32 * rt_b + r32) * PC + 16 * ks + 8 * g));
#pragma unroll
        for (int ks = 0; ks < DK / 16; ++ks)
            M::mma(aV, M::load_kmajor(dSm, PV, 16 * ks, 32 * bt, lane), M::load(Km + (32 * rt_b + r32) * PK + 16 * ks + 8 * g));
        // The tile is held transposed (accumulator row = dv position 8 c + 4 g + jj, column = token), so
        // that four registers are four neighbouring dv columns of one token: position -> column swaps
        // bits 2 and 3, which sends them to columns 16 (c / 2) + 8 g + 4 (c % 2) + jj.
        T* dst = dVs + (size_t)(32 * rt_b + r32) * PVR + 32 * bt + 8 * g;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            tx4 pk;
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) pk[jj] = (T)(aV[4 * c + jj] + aV2[4 * c + jj]);
            *reinterpret_cast<tx4*>(dst + 16 * (c >> 1) + 4 * (c & 1)) = pk;
        }
    }
    // tile (rt_a, at), transposed (channel = accumulator row):
    //   X^T = K~^T dP^T + (G_m S_n) dO^T,   Y1^T = Q~^T dP,   Ks^T = (H_m dS) V^T
    f32x16 aX, aY, aKs;
#pragma unroll
    for (int v = 0; v < 16; ++v) { aX[v] = 0.0f; aY[v] = 0.0f; aKs[v] = 0.0f; }
    if (has_a) {
#pragma unroll
        for (int kk = 0; kk < 2 * NBT; ++kk) {
            M::mma(aX, sS[kk], M::load(dOm + (32 * rt_a + r32) * PV + 16 * kk + 8 * g));
            if constexpr (FUSED)
                M::mma(aKs, *reinterpret_cast<const frag*>(dSm + (size_t)(32 * at + r32) * PV + 16 * kk + 8 * g),
                       M::load(Vm + (32 * rt_a + r32) * PVR + 16 * kk + 8 * g));
            else
                M::mma(aKs, sD[kk], M::load(Vm + (32 * rt_a + r32) * PVR + 16 * kk + 8 * g));
        }
#pragma unroll
        for (int ks = 0; ks < 2 * NRT; ++ks) {
            M::mma(aX, M::load_kmajor(Km, PK, 16 * ks, 32 * at, lane), M::load_kmajor(dPt, PC, 16 * ks, 32 * rt_a, lane));
            M::mma(aY, M::load_kmajor(Qm, PK, 16 * ks, 32 * at, lane), M::load(dPt + (32 * rt_a + r32) * PC + 16 * ks + 8 * g));
        }
    }
    // next chunk of this workgroup: its row loads are in flight during the staging / epilogue below
    // Every load is unconditional (the last chunk of a workgroup fetches itself again), which
    // keeps the count of outstanding loads exact, so that nothing below waits for these.
    if constexpr (FUSED) {
        // E_n = D'_n + Q~^T dO: rows = dv (true column order), columns = channels
        if (has_d) {
#pragma unroll
            for (int ks = 0; ks < 2 * NRT; ++ks) {
                const frag qf = M::load_kmajor(Qm, PK, 16 * ks, 32 * at, lane);
#pragma unroll
                for (int j = 0; j < TPW; ++j)
                    M::mma(accD[j], M::load_kmajor_swapped(dOm, PV, 16 * ks, 32 * ((w + NW * j) / NAT), lane), qf);
            }
        }
    }
    if constexpr (GROUPED) {
        // the walk leaves a sequence after its first chunk: dS_0 = G_m E is its grad_h0 (formed in
        // place: the next chunk of the walk starts from its own sequence's grad_hT)
        if (cur.n == 0 && p.dh0 && has_d) {
#pragma unroll
            for (int j = 0; j < TPW; ++j)
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    char* cols = const_cast<char*>(state_cols(p.dh0, cur.bh, j, c));
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        accD[j][4 * c + e] *= gm_prev;
                        *reinterpret_cast<float*>(cols + st_lane + 4 * e) = accD[j][4 * c + e];
                    }
                }
        }
    }
    RawRows<RW> nxt_f, nxt_q;
    ChunkAt nxt;
    if constexpr (GROUPED) nxt = walk_next(cur);
    else nxt = where(chunk_of(it + 1));
    load_chunk_rows(nxt_f, nxt_q, raw_v, raw_d, nxt, lane);   // v, dO of this chunk are dead
    __syncthreads();     // every wave is done with the operand tiles

    // ---------------- staging: X, Y1, Ks as [row][channel] fp32, 16 bytes per store ----------------
    if (has_a) {
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const size_t o = (size_t)(32 * rt_a + r32) * PF + 32 * at + 8 * c + 4 * g;
            *reinterpret_cast<f32x4*>(cX + o) = f32x4{aX[4 * c], aX[4 * c + 1], aX[4 * c + 2], aX[4 * c + 3]};
            *reinterpret_cast<f32x4*>(cY + o) = f32x4{aY[4 * c], aY[4 * c + 1], aY[4 * c + 2], aY[4 * c + 3]};
            *reinterpret_cast<f32x4*>(cKs + o) = f32x4{aKs[4 * c], aKs[4 * c + 1], aKs[4 * c + 2], aKs[4 * c + 3]};
        }
    }
    __syncthreads();

    // ---------------- element-wise epilogue in the row-block / channel-pair layout ----------------
    //   dq = sq X,  dk = sk (Y1 + Ks),  e' = bf16(Q~) X - bf16(K~) Y1,  kk = bf16(K~) Ks
    //   dg_s = sum_{i >= s in chunk} e'_i + sum_{j < s in chunk} kk_j + R
    // (bf16(.) are the values the MFMAs consumed, so that the pair terms inside e' cancel to fp32
    // accuracy).  Here: suffix / prefix inside the wave's row block, and the block sums to LDS.
    float gs0[RW], gs1[RW], dk0[RW], dk1[RW];
    T* dqg = static_cast<T*>(p.dq);
    T* dfg = static_cast<T*>(p.df);
    // (gates formed from pre-activations are kept instead: a second round of exponentials and reciprocals costs more than 16 registers)
    if (!p.beta) convert_rows<RW>(rf, raw_f, row0, cr.end, k_act, gate_bf16, 1.0f, cr.first);
    if constexpr (FUSED) {
        // the gate products again (32 multiplications) rather than 32 registers kept through the contractions
        asm volatile("" : "+v"(rf[0].x), "+v"(rf[0].y));
        float t0 = 1.0f, t1 = 1.0f;
#pragma unroll
        for (int i = 0; i < RW; ++i) { t0 *= rf[i].x; t1 *= rf[i].y; a0[i] = t0; a1[i] = t1; }
        float u0 = 1.0f, u1 = 1.0f;
#pragma unroll
        for (int i = RW - 1; i >= 0; --i) { z0[i] = u0; z1[i] = u1; u0 *= rf[i].x; u1 *= rf[i].y; }
    }
    // rows of this wave's block to global memory: one address and constant offsets when the
    // whole block lies inside the sequence, row by row otherwise
    auto store_block = [&](T* dst, const float (&x0)[RW], const float (&x1)[RW]) {
        T* bp = dst + seq_k + (ptrdiff_t)row0 * (ptrdiff_t)ld_k + 2 * lane;
        if (row0 >= cr.first && row0 + RW <= cr.end) {
#pragma unroll
            for (int i = 0; i < RW; ++i) store_pair_t<T>(bp, (size_t)i * ld_k, x0[i], x1[i]);
        } else {
#pragma unroll
            for (int i = 0; i < RW; ++i)
                if (cr.holds(RW * w + i)) store_pair_t<T>(bp, (size_t)i * ld_k, x0[i], x1[i]);
        }
    };
    if (k_act) {
        float kk0[RW], kk1[RW], dq0[RW], dq1[RW];
        float se0 = 0.0f, se1 = 0.0f;
#pragma unroll
        for (int i = RW - 1; i >= 0; --i) {
            const int row = RW * w + i;
            const f32x2 xq = *reinterpret_cast<const f32x2*>(cX + (size_t)row * PF + 2 * lane);
            const f32x2 xy = *reinterpret_cast<const f32x2*>(cY + (size_t)row * PF + 2 * lane);
            const f32x2 xs = *reinterpret_cast<const f32x2*>(cKs + (size_t)row * PF + 2 * lane);
            const float qb0 = (float)qb[i].x, qb1 = (float)qb[i].y, kb0 = (float)kb[i].x, kb1 = (float)kb[i].y;
            dk0[i] = (sz0 * z0[i]) * (xy.x + xs.x); dk1[i] = (sz1 * z1[i]) * (xy.y + xs.y);
            se0 = fmaf(qb0, xq.x, se0); se0 = fmaf(-kb0, xy.x, se0);
            se1 = fmaf(qb1, xq.y, se1); se1 = fmaf(-kb1, xy.y, se1);
            gs0[i] = se0; gs1[i] = se1;                                                 // inclusive suffix inside the block
            kk0[i] = kb0 * xs.x; kk1[i] = kb1 * xs.y;
            dq0[i] = (sa0 * a0[i]) * xq.x; dq1[i] = (sa1 * a1[i]) * xq.y;
        }
        store_block(dqg, dq0, dq1);
        float pk0 = 0.0f, pk1 = 0.0f;
#pragma unroll
        for (int i = 0; i < RW; ++i) { gs0[i] += pk0; gs1[i] += pk1; pk0 += kk0[i]; pk1 += kk1[i]; }   // exclusive prefix inside the block
        *reinterpret_cast<f32x2*>(blkE + w * DK + 2 * lane) = f32x2{se0, se1};
        *reinterpret_cast<f32x2*>(blkK + w * DK + 2 * lane) = f32x2{pk0, pk1};
    }
    // coalesced store of dv
    {
        constexpr int VPR = DV / VEC;
        T* dvg = static_cast<T*>(p.dv);
        for (int idx = tid; idx < C * VPR; idx += kBwdThreads) {
            const int row = idx / VPR, cv = idx % VPR;
            const int grow = cr.tok0 + row;
            if (cr.holds(row))
                *reinterpret_cast<u32x4*>(dvg + seq_v + (size_t)grow * ld_v + cv * VEC) =
                    *reinterpret_cast<const u32x4*>(dVs + (size_t)row * PVR + cv * VEC);
        }
    }
    __syncthreads();
    if (k_act) {
        // R + block sums of e' of the later blocks + block sums of K~ Ks of the earlier ones (row
        // addresses are wave-uniform; this block's own slot reads the row of zeros)
        f32x2 add = *reinterpret_cast<const f32x2*>(Rp + 2 * lane);
#pragma unroll
        for (int ww = 0; ww < NW; ++ww) {
            const float* src = (ww > w) ? blkE + ww * DK : (ww < w) ? blkK + ww * DK : zeros;
            const f32x2 b = *reinterpret_cast<const f32x2*>(src + 2 * lane);
            add.x += b.x; add.y += b.y;
        }
#pragma unroll
        for (int i = 0; i < RW; ++i) {
            gs0[i] = (gs0[i] + add.x) * fast_rcp(rf[i].x + 1e-30f) - dk0[i];
            gs1[i] = (gs1[i] + add.y) * fast_rcp(rf[i].y + 1e-30f) - dk1[i];
        }
        if (p.beta) {
            // gate formed from its pre-activation z (paper Eq. 2): with g = sigmoid(z) = (f - beta)/(1 - beta),
            //   dL/dz = df (1 - beta) g (1 - g) = df (f - beta)(1 - f)/(1 - beta),   dL/dbeta = sum df (1 - g)
            // (rows past the end of the sequence have f = 1 and drop out of the sum by themselves)
            const f32x2 b = *reinterpret_cast<const f32x2*>(p.beta + (size_t)(bh % p.H) * DK + 2 * lane);
            const float inv0 = fast_rcp(1.0f - b.x), inv1 = fast_rcp(1.0f - b.y);
            float sb0 = 0.0f, sb1 = 0.0f;
#pragma unroll
            for (int i = 0; i < RW; ++i) {
                const float u0 = gs0[i] * (1.0f - rf[i].x) * inv0, u1 = gs1[i] * (1.0f - rf[i].y) * inv1;
                sb0 += u0; sb1 += u1;
                gs0[i] = u0 * (rf[i].x - b.x); gs1[i] = u1 * (rf[i].y - b.y);
            }
            if constexpr (RUN_BETA) { run_b0 += sb0; run_b1 += sb1; }
            else *reinterpret_cast<f32x2*>(p.beta_partials + ((size_t)chunk * NW + w) * DK + 2 * lane) = f32x2{sb0, sb1};
        }
        store_block(dfg, gs0, gs1);
    }
    raw_f = nxt_f;
    raw_q = nxt_q;
    cur = nxt;
    if (L::end_barrier) __syncthreads();     // the block sums alias tiles the next chunk is about to write
  }
    if (p.flag && below_floor < kTinyProduct) *p.flag = 1;
    store_run_beta();
    if constexpr (FUSED && !GROUPED) {
        // run 0 ends at the start of the sequence: dS_0 = G_m E of its first chunk is grad_h0
        if (f_run == 0 && p.dh0 && has_d) {
            const int r32i = tid & 31, gi = (tid >> 5) & 1;
            float* out = p.dh0 + (size_t)f_bh * DK * DV;
#pragma unroll
            for (int j = 0; j < TPW; ++j) {
                const int btj = (w + NW * j) / NAT;
#pragma unroll
                for (int v = 0; v < 16; ++v)
                    out[(size_t)(32 * at + r32i) * DV + 32 * btj + 8 * (v >> 2) + 4 * gi + (v & 3)] = accD[j][v] * gm_prev;
            }
        }
    }
}

template <typename T, int DK, int DV, bool GATE_BF16>
__global__ __launch_bounds__(kBwdThreads) void bwd_grad_kernel(BwdGradParams p)
{
    if (p.dense) bwd_grad_body<T, DK, DV, GATE_BF16, true, false>(p);
    else         bwd_grad_body<T, DK, DV, GATE_BF16, false, false>(p);
}

template <typename T, int DK, int DV, bool GATE_BF16>
__global__ __launch_bounds__(kBwdThreads) void bwd_fused_kernel(BwdGradParams p)
{
    if (p.dense) bwd_grad_body<T, DK, DV, GATE_BF16, true, true>(p);
    else         bwd_grad_body<T, DK, DV, GATE_BF16, false, true>(p);
}

// The fused reverse walk over groups of a packed batch's sequences (a kernel of its own).
template <typename T, int DK, int DV, bool GATE_BF16>
__global__ __launch_bounds__(kBwdThreads) void bwd_fused_grouped_kernel(BwdGradParams p)
{
    bwd_grad_body<T, DK, DV, GATE_BF16, false, true, true>(p);
}

template <typename T, int DK, int DV>
static hipError_t launch_one(const SeqDims& d, const BwdGradParams& p, hipStream_t stream)
{
    typedef BwdGradLds<T, DK, DV> L;
    auto kern = d.gate_bf16 ? bwd_grad_kernel<T, DK, DV, true> : bwd_grad_kernel<T, DK, DV, false>;
    hipError_t e = allow_dynamic_lds(reinterpret_cast<const void*>(kern), (int)L::total);
    if (e != hipSuccess) return e;
    // one persistent workgroup per CU (the LDS footprint admits no more), each walking its share of chunks
    const size_t n_chunks = d.total_chunks();
    const unsigned grid = (unsigned)(n_chunks < 256 ? n_chunks : 256);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(kBwdThreads), L::total, stream, p);
    return hipGetLastError();
}

hipError_t launch_bwd_grad(const SeqDims& d, const void* q, const void* f, const void* v, const void* grad_o,
                           const void* ws_state, const void* ws_dstate, void* grad_q, void* grad_f,
                           void* grad_v, float* beta_partials, hipStream_t stream)
{
    if (d.total_chunks() == 0) return hipSuccess;
    if (!d.io_bf16) return hipErrorInvalidValue;
    BwdGradParams p;
    p.q = q; p.f = f; p.v = v; p.dO = grad_o; p.ws_s = ws_state; p.ws_ds = ws_dstate;
    p.dq = grad_q; p.df = grad_f; p.dv = grad_v;
    p.BH = d.BH; p.N = d.N; p.NC = d.NC;
    p.beta = d.beta; p.beta_partials = beta_partials; p.H = d.H; p.lay = d.lay; p.dense = d.dense() ? 1 : 0;
    p.dhT = nullptr; p.dh0 = nullptr; p.bound0 = nullptr; p.run_state = nullptr; p.R = 1; p.rc = d.NC; p.s_sub = 1; p.seg_tail = 0;
    p.light = 0;
    for (int i = 0; i <= kMaxLightRuns; ++i) p.bnd[i] = 0;
    p.flag = d.domain_flag;
    if (d.beta && !beta_partials) return hipErrorInvalidValue;
    if (d.dk == 128 && d.dv == 128) return launch_one<__bf16, 128, 128>(d, p, stream);
    if (d.dk == 64 && d.dv == 64) return launch_one<__bf16, 64, 64>(d, p, stream);
    if (d.dk == 128 && d.dv == 64) return launch_one<__bf16, 128, 64>(d, p, stream);
    if (d.dk == 64 && d.dv == 128) return launch_one<__bf16, 64, 128>(d, p, stream);
    return hipErrorInvalidValue;
}

template <typename T, int DK, int DV>
static hipError_t launch_fused_one(const SeqDims& d, const BwdGradParams& p, hipStream_t stream)
{
    typedef BwdGradLds<T, DK, DV> L;
    auto kern = d.gate_bf16 ? bwd_fused_kernel<T, DK, DV, true> : bwd_fused_kernel<T, DK, DV, false>;
    hipError_t e = allow_dynamic_lds(reinterpret_cast<const void*>(kern), (int)L::total);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3((unsigned)(d.BH * p.R)), dim3(kBwdThreads), L::total, stream, p);
    return hipGetLastError();
}

BwdFusedPlan plan_bwd_fused(const SeqDims& d)
{
    // One workgroup per run and one run per compute unit at a time: as many runs per sequence as it
    // takes to fill the chip, but at least four chunks each.  The zero-start sweep that supplies the
    // state gradient at the run boundaries walks sub-runs of about eight chunks.
    BwdFusedPlan pl;
    pl.light = 0;
    for (int i = 0; i <= kMaxLightRuns; ++i) pl.bnd[i] = 0;
    int R = d.BH > 0 ? 256 / d.BH : 1;
    if (R > d.NC / 4) R = d.NC / 4;
    if (R < 1) R = 1;
    if (R >= 2 && R <= kMaxLightRuns) {
        // Few runs: each workgroup walks the chunks after its run itself, at `rho` of a chunk's full
        // cost, and the cuts are placed so that all runs take the same time T:
        // len_r = T - rho (NC - end_r), from the last run (len = T) backwards; T by bisection.
        // rho is set by the balance that measures best (128 sequences of 32 chunks in two runs: 14 + 18
        // chunks 180 us, 15 + 17 185 us, 13 + 19 187 us; a light chunk alone costs 0.16 of a full one,
        // but the light walks run while the memory system is busiest).
        const double rho = 0.24;
        double lo = 0.0, hi = (double)d.NC;
        for (int iter = 0; iter < 50; ++iter) {
            const double T = 0.5 * (lo + hi);
            double end = (double)d.NC;
            for (int r = R - 1; r >= 0; --r) end -= T - rho * ((double)d.NC - end);
            if (end > 0.0) lo = T; else hi = T;        // runs too short: raise T
        }
        double end = (double)d.NC;
        pl.bnd[R] = d.NC;
        for (int r = R - 1; r >= 1; --r) {
            end -= hi - rho * ((double)d.NC - end);
            int b = (int)(end + 0.5);
            if (b < r) b = r;                          // every run keeps at least one chunk
            if (b > pl.bnd[r + 1] - 1) b = pl.bnd[r + 1] - 1;
            pl.bnd[r] = b;
        }
        pl.bnd[0] = 0;
        pl.light = 1;
        pl.R = R; pl.rc = 0; pl.s_sub = 1; pl.sub_chunks = 0; pl.seg_tail = 0;
        return pl;
    }
    int rc = (d.NC + R - 1) / R;
    int s = rc / 8;                               // sub-runs of about eight chunks: fewer, longer walks and fewer states to carry
    if (s < 1) s = 1;
    if (R > 1) rc = (rc + s - 1) / s * s;         // whole sub-runs per run
    pl.rc = rc;
    pl.R = rc > 0 ? (d.NC + rc - 1) / rc : 1;
    if (pl.R < 1) pl.R = 1;
    pl.s_sub = s;
    pl.sub_chunks = rc / s;
    pl.seg_tail = pl.R > 1 ? (d.NC - rc + pl.sub_chunks - 1) / pl.sub_chunks : 0;
    return pl;
}

hipError_t launch_bwd_fused(const SeqDims& d, const BwdFusedPlan& pl, const void* q, const void* f, const void* v,
                            const void* grad_o, const void* ws_state, const float* grad_hT, float* grad_h0,
                            const float* bound0, const float* run_state, void* grad_q, void* grad_f, void* grad_v,
                            float* beta_partials, hipStream_t stream)
{
    if (d.total_chunks() == 0) return hipSuccess;
    if (d.packed || d.lay.vl) return hipErrorInvalidValue;
    if (!d.io_bf16 && !(d.dk == 64 && d.dv == 64)) return hipErrorInvalidValue;    // fp32 tiles of wider heads exceed the LDS
    if (d.beta && !beta_partials) return hipErrorInvalidValue;
    BwdGradParams p;
    p.q = q; p.f = f; p.v = v; p.dO = grad_o; p.ws_s = ws_state; p.ws_ds = nullptr;
    p.dq = grad_q; p.df = grad_f; p.dv = grad_v;
    p.BH = d.BH; p.N = d.N; p.NC = d.NC;
    p.beta = d.beta; p.beta_partials = beta_partials; p.H = d.H; p.lay = d.lay; p.dense = d.dense() ? 1 : 0;
    p.dhT = grad_hT; p.dh0 = grad_h0; p.bound0 = bound0; p.run_state = run_state;
    p.R = pl.R; p.rc = pl.rc; p.s_sub = pl.s_sub; p.seg_tail = pl.seg_tail;
    p.light = pl.light;
    for (int i = 0; i <= kMaxLightRuns; ++i) p.bnd[i] = pl.bnd[i];
    p.flag = d.domain_flag;
    if (!d.io_bf16) return launch_fused_one<float, 64, 64>(d, p, stream);
    if (d.dk == 128 && d.dv == 128) return launch_fused_one<__bf16, 128, 128>(d, p, stream);
    if (d.dk == 64 && d.dv == 64) return launch_fused_one<__bf16, 64, 64>(d, p, stream);
    if (d.dk == 128 && d.dv == 64) return launch_fused_one<__bf16, 128, 64>(d, p, stream);
    if (d.dk == 64 && d.dv == 128) return launch_fused_one<__bf16, 64, 128>(d, p, stream);
    return hipErrorInvalidValue;
}

template <int DK, int DV>
static hipError_t launch_grouped_one(const SeqDims& d, const BwdGradParams& p, hipStream_t stream)
{
    typedef BwdGradLds<__bf16, DK, DV> L;
    auto kern = d.gate_bf16 ? bwd_fused_grouped_kernel<__bf16, DK, DV, true> : bwd_fused_grouped_kernel<__bf16, DK, DV, false>;
    hipError_t e = allow_dynamic_lds(reinterpret_cast<const void*>(kern), (int)L::total);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3((unsigned)(d.lay.spans * d.lay.H)), dim3(kBwdThreads), L::total, stream, p);
    return hipGetLastError();
}

hipError_t launch_bwd_fused_grouped(const SeqDims& d, const void* q, const void* f, const void* v, const void* grad_o,
                                    const void* ws_state, const float* grad_hT, float* grad_h0, void* grad_q,
                                    void* grad_f, void* grad_v, float* beta_partials, hipStream_t stream)
{
    if (d.total_chunks() == 0) return hipSuccess;
    if (!d.lay.vl || d.lay.spans <= 0 || !d.lay.span_seq || !d.io_bf16) return hipErrorInvalidValue;
    if (d.beta && !beta_partials) return hipErrorInvalidValue;
    BwdGradParams p;
    p.q = q; p.f = f; p.v = v; p.dO = grad_o; p.ws_s = ws_state; p.ws_ds = nullptr;
    p.dq = grad_q; p.df = grad_f; p.dv = grad_v;
    p.BH = d.BH; p.N = d.N; p.NC = d.NC;
    p.beta = d.beta; p.beta_partials = beta_partials; p.H = d.H; p.lay = d.lay; p.dense = 0;
    p.dhT = grad_hT; p.dh0 = grad_h0; p.bound0 = nullptr; p.run_state = nullptr;
    p.R = 1; p.rc = d.NC; p.s_sub = 1; p.seg_tail = 0; p.light = 0;
    for (int i = 0; i <= kMaxLightRuns; ++i) p.bnd[i] = 0;
    p.flag = d.domain_flag;
    if (d.dk == 128 && d.dv == 128) return launch_grouped_one<128, 128>(d, p, stream);
    if (d.dk == 64 && d.dv == 64) return launch_grouped_one<64, 64>(d, p, stream);
    if (d.dk == 128 && d.dv == 64) return launch_grouped_one<128, 64>(d, p, stream);
    if (d.dk == 64 && d.dv == 128) return launch_grouped_one<64, 128>(d, p, stream);
    return hipErrorInvalidValue;
}

constexpr int kRedGroups = 16;      // groups of 64 threads per workgroup, each adding every 16th row of its share
constexpr int kRedSlices = 8;       // workgroups that share the rows of one (head, 64 channels)

size_t beta_partials_bytes(const SeqDims& d)
{
    // the per-wave rows of every chunk slot, then the sums of the slices
    if (d.total_chunks() == 0) return 0;
    return (d.total_chunks() * kBwdWaves + (size_t)kRedSlices * d.H) * d.dk * sizeof(float);
}

// grad_beta[h][a] = sum over batch, chunks and waves of the partial sums, in a fixed order.  First
// pass: workgroup (head, 64 channels, slice) adds its share of the partial rows (the groups of 16
// consecutive rows numbered slice, slice + 8, ... of every sequence; 16 groups of 64 threads take a
// row each, coalesced across the channels, and the 16 group sums are added in order).  Second
// pass: the slice sums are added in order.
__global__ __launch_bounds__(64 * kRedGroups) void reduce_beta_kernel(const float* partials, float* slice_sums, int B,
                                                                      int H, int NC, int used, int dk, const int* vl,
                                                                      const int* choice, int path, int sub)
{
    if (choice && table_read(choice, 0) != path) return;        // one of several alternatives, and not the one called for
    __shared__ float part[kRedGroups][64];
    const int h = blockIdx.x / (dk / 64), a = 64 * (blockIdx.x % (dk / 64)) + (threadIdx.x & 63);
    const int grp = threadIdx.x >> 6, slice = blockIdx.y;
    float s = 0.0f;
    for (int b = 0; b < B; ++b) {
        // partial rows of (batch, head): kBwdWaves per chunk, the chunks of a sequence and head together
        // (of which the first `used` hold rows: one per chunk, or one per run of a reverse walk)
        size_t first = (size_t)(b * H + h) * NC;
        int nc = used;
        if (vl) {
            nc = (vl[B + 1 + b] + sub - 1) >> (31 - __builtin_clz((unsigned)sub));
            first = (size_t)vl[2 * (B + 1) + b] * H + (size_t)h * nc;
        }
        const int rows = nc * kBwdWaves;
        const float* pp = partials + first * kBwdWaves * dk + a;
#pragma unroll 4
        for (int i = grp + kRedGroups * slice; i < rows; i += kRedGroups * kRedSlices) s += pp[(size_t)i * dk];
    }
    part[grp][threadIdx.x & 63] = s;
    __syncthreads();
    if (grp == 0) {
        float t = 0.0f;
#pragma unroll
        for (int j = 0; j < kRedGroups; ++j) t += part[j][threadIdx.x];
        slice_sums[((size_t)slice * H + h) * dk + a] = t;
    }
}

__global__ void reduce_beta_slices_kernel(const float* slice_sums, float* grad_beta, int n, const int* choice, int path)
{
    if (choice && table_read(choice, 0) != path) return;
    const int c = blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= n) return;
    float t = 0.0f;
#pragma unroll
    for (int j = 0; j < kRedSlices; ++j) t += slice_sums[(size_t)j * n + c];
    grad_beta[c] = t;
}

hipError_t reduce_beta_partials(const SeqDims& d, float* beta_partials, float* grad_beta, hipStream_t stream, int runs)
{
    if (d.H * d.dk == 0) return hipSuccess;
    const int B = d.BH / d.H, n = d.H * d.dk;
    if (d.total_chunks() == 0) return launch_zero_floats(grad_beta, (size_t)n, stream);      // nothing contributes
    float* slice_sums = beta_partials + d.total_chunks() * kBwdWaves * d.dk;
    hipLaunchKernelGGL(reduce_beta_kernel, dim3(d.H * (d.dk / 64), kRedSlices), dim3(64 * kRedGroups), 0, stream,
                       beta_partials, slice_sums, B, d.H, d.NC, runs > 0 ? runs : d.NC, d.dk, d.lay.vl,
                       d.packed ? d.lay.alt : d.lay.choice, d.packed ? d.lay.alt_path : d.lay.path, d.lay.sub);
    hipLaunchKernelGGL(reduce_beta_slices_kernel, dim3((n + 255) / 256), dim3(256), 0, stream, slice_sums, grad_beta, n,
                       d.packed ? d.lay.alt : d.lay.choice, d.packed ? d.lay.alt_path : d.lay.path);
    return hipGetLastError();
}

// beta[l][c] = cumsum_l(softmax_l(gamma[:, c])) - its first row; one thread per channel, the
// layer axis walked serially (L is a few dozen).
__global__ void cumax_kernel(const float* gamma, float* beta, int L, int d)
{
    const int c = blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= d) return;
    float m = -3.0e38f;
    for (int l = 0; l < L; ++l) m = fmaxf(m, gamma[(size_t)l * d + c]);
    float z = 0.0f;
    for (int l = 0; l < L; ++l) z += expf(gamma[(size_t)l * d + c] - m);
    const float inv = 1.0f / z;
    float run = 0.0f;
    for (int l = 0; l < L; ++l) {
        beta[(size_t)l * d + c] = run;          // cumulative sum up to layer l, minus the first layer's share
        if (l + 1 < L) run += expf(gamma[(size_t)(l + 1) * d + c] - m) * inv;
    }
}

hipError_t launch_cumax(int L, int d, const float* gamma, float* beta, hipStream_t stream)
{
    if (L <= 0 || d <= 0) return hipSuccess;
    hipLaunchKernelGGL(cumax_kernel, dim3((d + 127) / 128), dim3(128), 0, stream, gamma, beta, L, d);
    return hipGetLastError();
}

}   // namespace hgrn2
