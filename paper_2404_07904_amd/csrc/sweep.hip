// Chunk-to-chunk state recurrence of the chunkwise HGRN2 algorithm (paper Section 3.2, Eq. 3,
// regrouped per chunk of C tokens):
//
//   forward state     S_{n+1} = Diag(g_n) S_n + K^_n^T V_n ,       K^_j = k_j * prod_{s>j in chunk} f_s
//   state gradient    dS_n    = Diag(g_n) dS_{n+1} + Q^_n^T dO_n , Q^_i = q_i * prod_{s<=i in chunk} f_s
//
// with g_n the product of all gates of chunk n.  One workgroup owns a [dk x TV] column slab of
// the state of one (batch, head) and walks the chunks in order (reverse order for the gradient),
// keeping the slab in fp32 MFMA accumulators.  Before each update it writes the slab, scaled by
// the half-chunk gate product its consumer would apply anyway (G_m of chunk n for S_n, g/G_m for
// dS_{n+1}) and rounded to the operand type, to the workspace in MFMA-fragment order so that the
// per-chunk kernels can load it straight into operand registers.  The contraction runs over time,
// so both operands are staged in LDS token-contiguous (see common.hpp for the thread layout that
// makes this free).
//
// A batch of few, long sequences would leave most of the chip idle in such a walk.  The recurrence
// is linear in the state, so a sequence can be cut into runs of whole chunks: a walk per run from
// a zero state (no workspace writes) gives the run's own contribution A_r and the product D_r of
// its gates, the short recurrence  S <- Diag(D_r) S + A_r  over the runs (run_carry_kernel) gives
// the state entering every run, and the walk proper then starts run by run, all runs at once.
#include "common.hpp"
#include "kernels.hpp"

namespace hgrn2 {

// Workgroups (per column slab) a sweep needs: one per sequence, or one per group of a packed
// batch's sequences (the walks from zero, ENDS, always take one per sequence).
template <bool ENDS> static int sweep_walkers(const SeqDims& d)
{
    return (!ENDS && d.lay.vl && d.lay.groups) ? d.lay.G * d.lay.H : d.BH;
}

struct SweepParams {
    const void* q;
    const void* f;
    const void* bsrc;
    const float* init;
    float* fin;
    void* ws;
    float* decay;        // set: walk from zero, nothing per chunk; receives the per-channel product of all gates of the sequence, [BH][dk], or null
    int BH, N, NC, n_tile, gate_bf16;
    const float* beta;   // [H][dk] lower bounds, or null: the gate tensor holds f itself
    int H;
    TokenLayout lay;     // used when dense == 0
    int dense;           // sequence tensors are [B][H][N][d]: token strides are the compile-time dk, dv
};


template <typename T, int DK, int DV, int TV, int MODE, bool DENSE, bool ENDS>
__device__ __forceinline__ void sweep_body(const SweepParams& p, int block_id)
{
    constexpr int C = kChunk, RW = C / kWaves;
    constexpr int PC = C + pad_elems<T>();
    constexpr int NAT = DK / 32, NBT = TV / 32, NT = NAT * NBT, TPW = NT / kWaves;
    static_assert(NT % kWaves == 0 && TPW >= 1, "tile count must be a multiple of the wave count");
    constexpr bool TRANS = MODE != kSweepStateFwd;
    constexpr bool REVERSE = MODE == kSweepGrad;
    typedef Mma<T> M;

    extern __shared__ __align__(16) char smem[];
    T* AT = reinterpret_cast<T*>(smem);          // [DK][PC]  a-side operand, token-contiguous
    T* BT = AT + DK * PC;                        // [TV][PC]  b-side operand, token-contiguous
    float* gam = reinterpret_cast<float*>(BT + TV * PC);   // [DK] whole-chunk decay
    float* tot = gam + DK;                       // [4][DK] per-wave block products
    float* hsc = tot + kWaves * DK;              // [DK] half-chunk decay folded into the stored fragments

    // ENDS: the walk starts from a zero slab and hands nothing to the workspace; what it leaves is
    // the slab after the last chunk and the product of all gates it passed, per channel.
    //
    // Which sequences this workgroup walks: one, or -- a packed batch with a group table -- the
    // sequences [groups[g], groups[g + 1]) of one head, one after the other (each from its own initial
    // slab to its own final one), with the first rows of the next sequence already in flight during
    // the last chunk of the current one: a batch of many short sequences then costs a workgroup's
    // start-up and a trip to memory once per group, not once per sequence.
    if (not_chosen(p.lay)) return;       // (a packed batch whose table chose the other backward pass; a chunk length not called for)
    int id, tile;
    xcd_map(block_id, p.n_tile, id, tile);
    int bh_first, bh_end, bh_step;
    bool grouped = false;
    if constexpr (!DENSE && !ENDS) grouped = p.lay.vl != nullptr && p.lay.groups != nullptr;
    if (grouped) {
        if (id >= p.lay.G * p.lay.H) return;
        const int grp = id / p.lay.H, head = id - grp * p.lay.H;
        bh_step = p.lay.H;
        bh_first = table_read(p.lay.groups, grp) * p.lay.H + head;
        bh_end = table_read(p.lay.groups, grp + 1) * p.lay.H + head;
    } else {
        if (id >= p.BH) return;
        bh_first = sequence_of_workgroup<DENSE>(p.lay, id);
        bh_step = 1;
        bh_end = bh_first + 1;
    }
    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, r32 = lane & 31, g = lane >> 5;
    const int col0 = tile * TV;
    const bool a_act = 2 * lane < DK, b_act = 2 * lane < TV;
    const int ld_k = DENSE ? DK : (int)p.lay.sn_k, ld_v = DENSE ? DV : (int)p.lay.sn_v;   // token stride, elements
    const bool gate_bf16 = p.gate_bf16 != 0;
    const T* qsrc = static_cast<const T*>(p.q);
    const T* bsrc = static_cast<const T*>(p.bsrc);

    // raw rows of the chunk being prefetched; inactive lanes read column 0 and are ignored
    RawRows<RW> raw_f, raw_q, raw_b;
    const int col_a = a_act ? 2 * lane : 0, col_b = col0 + (b_act ? 2 * lane : 0);
    auto load_chunk = [&](const SeqView& s, int n) {
        const int row0 = chunk_rows(p.lay.sub, n, s.N).tok0 + RW * w;
        load_rows<RW>(raw_f, p.f, s.off_k, ld_k, col_a, row0, s.N, gate_bf16);
        if (MODE == kSweepGrad) load_rows<RW>(raw_q, qsrc, s.off_k, ld_k, col_a, row0, s.N, is_bf16_type<T>());
        load_rows<RW>(raw_b, bsrc, s.off_v, ld_v, col_b, row0, s.N, is_bf16_type<T>());
    };
    auto view = [&](int bh) { return seq_view<DENSE, DK, DV, true>(p.lay, p.N, p.NC, bh); };

    // A sequence without chunks ends in the slab it starts from (zero, and all gate products one,
    // for a walk from zero); these are dealt with first, the walk below steps over them.
    for (int b = bh_first; b < bh_end; b += bh_step) {
        if (view(b).NC > 0) continue;
        if (p.fin)
            for (int idx = tid; idx < DK * TV; idx += kThreads) {
                const size_t e = (size_t)b * DK * DV + (size_t)(idx / TV) * DV + col0 + idx % TV;
                p.fin[e] = (!ENDS && p.init) ? p.init[e] : 0.0f;
            }
        if (ENDS && tile == 0 && tid < DK && p.decay) p.decay[(size_t)b * DK + tid] = 1.0f;
    }

    // The walk: chunk `it` (in walking order) of sequence bh, then the next one, which may be the
    // first chunk of the group's next sequence with tokens.  The rows of the next chunk are always
    // requested (past the end: the current ones again), so that the number of loads in flight never
    // depends on where the walk is.
    int next_open = bh_first;                    // first sequence not opened yet
    auto open_sequence = [&](SeqView& v, int& bh_out) {
        while (next_open < bh_end) {
            const int b = next_open;
            next_open += bh_step;
            v = view(b);
            if (v.NC > 0) { bh_out = b; return true; }
        }
        return false;
    };
    SeqView sv, sv_next;
    int bh = 0, bh_next = 0, it = 0, it_next = 0;
    bool more = open_sequence(sv, bh);
    if (!more) return;                           // (uniform, before any barrier)
    load_chunk(sv, REVERSE ? sv.NC - 1 : 0);

    f32x16 acc[TPW];             // accumulator tiles of this wave: tile id = w + 4j -> (at, bt)
    float run_decay = 1.0f;      // ENDS: thread t < DK, gate product of channel t so far

    while (more) {
        const int N = sv.N, NC = sv.NC;
        const int n = REVERSE ? NC - 1 - it : it;
        // the chunk after this one (scalar work only)
        bool more_next = true;
        if (it + 1 < NC) { sv_next = sv; bh_next = bh; it_next = it + 1; }
        else { more_next = open_sequence(sv_next, bh_next); it_next = 0; }
        if (it == 0) {
            // a sequence starts: its initial slab, the product of its gates from one
            run_decay = 1.0f;
#pragma unroll
            for (int j = 0; j < TPW; ++j) {
                const int id = w + kWaves * j, at = id % NAT, bt = id / NAT;
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    float x = 0.0f;
                    if (!ENDS && p.init) {
                        const float* s0 = p.init + (size_t)bh * DK * DV;
                        x = TRANS ? s0[(size_t)(32 * at + r32) * DV + col0 + 32 * bt + acc_row(v, lane)]
                                  : s0[(size_t)(32 * at + acc_row(v, lane)) * DV + col0 + 32 * bt + r32];
                    }
                    acc[j][v] = x;
                }
            }
        }
        T* ws = static_cast<T*>(p.ws) + sv.chunk0 * DK * DV;
        f32x2 rf[RW], rq[RW], rb[RW];
        {
            const ChunkRows cr = chunk_rows(p.lay.sub, n, N);
            const int row0 = cr.tok0 + RW * w;
            convert_rows<RW>(rf, raw_f, row0, cr.end, a_act, gate_bf16, 1.0f, cr.first);
            if (p.beta) gate_rows<RW>(rf, p.beta + (size_t)(bh / p.lay.seg % p.H) * DK, col_a, a_act, row0, cr.end, cr.first);
            if (MODE == kSweepGrad) convert_rows<RW>(rq, raw_q, row0, cr.end, a_act, is_bf16_type<T>(), 0.0f, cr.first);
            convert_rows<RW>(rb, raw_b, row0, cr.end, b_act, is_bf16_type<T>(), 0.0f, cr.first);
        }

        // ---- gate products of this thread's RW tokens, channel pair (2*lane, 2*lane+1) ----
        float a0[RW], a1[RW], z0[RW], z1[RW];
        {
            float run0 = 1.0f, run1 = 1.0f;
#pragma unroll
            for (int i = 0; i < RW; ++i) { run0 *= rf[i].x; run1 *= rf[i].y; a0[i] = run0; a1[i] = run1; }
            run0 = 1.0f; run1 = 1.0f;
#pragma unroll
            for (int i = RW - 1; i >= 0; --i) { z0[i] = run0; z1[i] = run1; run0 *= rf[i].x; run1 *= rf[i].y; }
        }
        if (a_act) {
            tot[w * DK + 2 * lane] = a0[RW - 1];
            tot[w * DK + 2 * lane + 1] = a1[RW - 1];
        }
        __syncthreads();
        if (a_act) {
            const BlockDecay d0 = block_decay(tot, DK, w, 2 * lane);
            const BlockDecay d1 = block_decay(tot, DK, w, 2 * lane + 1);
            float x0[RW], x1[RW];
#pragma unroll
            for (int i = 0; i < RW; ++i) {
                if (MODE == kSweepGrad) {
                    x0[i] = rq[i].x * (d0.pre * a0[i]);
                    x1[i] = rq[i].y * (d1.pre * a1[i]);
                } else {
                    x0[i] = (1.0f - rf[i].x) * (z0[i] * d0.post);
                    x1[i] = (1.0f - rf[i].y) * (z1[i] * d1.post);
                }
            }
            store_run<T, RW>(AT + (2 * lane) * PC + RW * w, x0);
            store_run<T, RW>(AT + (2 * lane + 1) * PC + RW * w, x1);
            if (w == 0) {
                gam[2 * lane] = d0.all; gam[2 * lane + 1] = d1.all;
                // what the consumers multiply the state with anyway: the gate product of the first
                // half of the chunk for S_n (read-out side), of the second half for dS_{n+1}
                constexpr int h0 = REVERSE ? 2 : 0;
                hsc[2 * lane] = tot[h0 * DK + 2 * lane] * tot[(h0 + 1) * DK + 2 * lane];
                hsc[2 * lane + 1] = tot[h0 * DK + 2 * lane + 1] * tot[(h0 + 1) * DK + 2 * lane + 1];
            }
        }
        if (b_act) {
            float x0[RW], x1[RW];
#pragma unroll
            for (int i = 0; i < RW; ++i) { x0[i] = rb[i].x; x1[i] = rb[i].y; }
            store_run<T, RW>(BT + (2 * lane) * PC + RW * w, x0);
            store_run<T, RW>(BT + (2 * lane + 1) * PC + RW * w, x1);
        }
        // the next chunk's rows are in flight during the MFMAs (after the last chunk: this one's again)
        {
            SeqView pf = sv;
            int pn = n;
            if (more_next) { pf = sv_next; pn = REVERSE ? sv_next.NC - 1 - it_next : it_next; }
            load_chunk(pf, pn);
        }
        __syncthreads();

        // ---- hand the slab as it stands (state entering / gradient leaving chunk n) to the workspace
        T* wsn = ws + (size_t)n * DK * DV;
        if (ENDS && tid < DK) run_decay *= gam[tid];
#pragma unroll
        for (int j = 0; j < (ENDS ? 0 : TPW); ++j) {
            const int id = w + kWaves * j, at = id % NAT, bt = id / NAT;
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                float x[8];
                if (TRANS) {
                    const float sc = hsc[32 * at + r32];
#pragma unroll
                    for (int s = 0; s < 8; ++s) x[s] = acc[j][8 * half + s] * sc;
                } else {
                    const f32x4 sc0 = *reinterpret_cast<const f32x4*>(hsc + 32 * at + 16 * half + 4 * g);
                    const f32x4 sc1 = *reinterpret_cast<const f32x4*>(hsc + 32 * at + 16 * half + 8 + 4 * g);
#pragma unroll
                    for (int s = 0; s < 4; ++s) { x[s] = acc[j][8 * half + s] * sc0[s]; x[4 + s] = acc[j][8 * half + 4 + s] * sc1[s]; }
                }
                *reinterpret_cast<typename M::frag*>(
                    wsn + state_frag_offset(at, col0 / 32 + bt, DV / 32, half, lane)) = M::pack(x);
            }
        }

        // ---- slab = Diag(g) slab + A^T B over the chunk ----
#pragma unroll
        for (int j = 0; j < TPW; ++j) {
            const int id = w + kWaves * j, at = id % NAT;
            if (TRANS) {
                const float gm = gam[32 * at + r32];
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[j][v] *= gm;
            } else {
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const f32x4 gm = *reinterpret_cast<const f32x4*>(gam + 32 * at + 8 * c + 4 * g);
#pragma unroll
                    for (int jj = 0; jj < 4; ++jj) acc[j][4 * c + jj] *= gm[jj];
                }
            }
        }
#pragma unroll
        for (int ks = 0; ks < C / 16; ++ks) {
#pragma unroll
            for (int j = 0; j < TPW; ++j) {
                const int id = w + kWaves * j, at = id % NAT, bt = id / NAT;
                const typename M::frag fa = M::load(AT + (32 * at + r32) * PC + 16 * ks + 8 * g);
                const typename M::frag fb = M::load(BT + (32 * bt + r32) * PC + 16 * ks + 8 * g);
                if (TRANS) M::mma(acc[j], fb, fa);
                else       M::mma(acc[j], fa, fb);
            }
        }
        if (it == NC - 1) {
            // the sequence ends: the slab as it stands, and the product of the gates it passed
            if (ENDS && tile == 0 && tid < DK && p.decay) p.decay[(size_t)bh * DK + tid] = run_decay;
            if (p.fin) {
                float* s1 = p.fin + (size_t)bh * DK * DV;
#pragma unroll
                for (int j = 0; j < TPW; ++j) {
                    const int id = w + kWaves * j, at = id % NAT, bt = id / NAT;
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        if (TRANS) s1[(size_t)(32 * at + r32) * DV + col0 + 32 * bt + acc_row(v, lane)] = acc[j][v];
                        else       s1[(size_t)(32 * at + acc_row(v, lane)) * DV + col0 + 32 * bt + r32] = acc[j][v];
                    }
                }
            }
        }
        sv = sv_next; bh = bh_next; it = it_next; more = more_next;
    }
}

template <typename T, int DK, int DV, int TV, int MODE, bool ENDS>
__global__ __launch_bounds__(kThreads) void sweep_kernel(SweepParams p)
{
    if (p.dense) sweep_body<T, DK, DV, TV, MODE, true, ENDS>(p, blockIdx.x);
    else         sweep_body<T, DK, DV, TV, MODE, false, ENDS>(p, blockIdx.x);
}

// The two sweeps of the backward pass (forward states, reverse state gradients) are independent;
// one launch runs both, the first half of the grid walking forwards and the second backwards, so
// that two latency-bound sequential kernels share the chip instead of running one after the other.
template <typename T, int DK, int DV, int TV, bool ENDS>
__global__ __launch_bounds__(kThreads) void sweep_pair_kernel(SweepParams ps, SweepParams pg, int half)
{
    if (ps.dense) {
        if ((int)blockIdx.x < half) sweep_body<T, DK, DV, TV, kSweepStateBwd, true, ENDS>(ps, blockIdx.x);
        else                        sweep_body<T, DK, DV, TV, kSweepGrad, true, ENDS>(pg, blockIdx.x - half);
    } else {
        if ((int)blockIdx.x < half) sweep_body<T, DK, DV, TV, kSweepStateBwd, false, ENDS>(ps, blockIdx.x);
        else                        sweep_body<T, DK, DV, TV, kSweepGrad, false, ENDS>(pg, blockIdx.x - half);
    }
}

template <typename T, int DK, int DV, int TV, bool ENDS>
static hipError_t launch_pair_one(const SeqDims& d, const SweepParams& ps0, const SweepParams& pg0, hipStream_t stream)
{
    SweepParams ps = ps0, pg = pg0;
    ps.n_tile = pg.n_tile = DV / TV;
    constexpr int PC = kChunk + pad_elems<T>();
    const size_t lds = (size_t)(DK + TV) * PC * sizeof(T) + (size_t)(2 + kWaves) * DK * sizeof(float);
    auto kern = sweep_pair_kernel<T, DK, DV, TV, ENDS>;
    hipError_t e = allow_dynamic_lds(reinterpret_cast<const void*>(kern), (int)lds);
    if (e != hipSuccess) return e;
    const int half = (sweep_walkers<ENDS>(d) + 7) / 8 * 8 * ps.n_tile;
    hipLaunchKernelGGL(kern, dim3(2 * half), dim3(kThreads), lds, stream, ps, pg, half);
    return hipGetLastError();
}

template <typename T, int DK, int DV, bool ENDS>
static hipError_t launch_pair_tv(const SeqDims& d, const SweepParams& ps, const SweepParams& pg, hipStream_t stream)
{
    // The sweeps are bound by the element-wise work on the gates, which every column slab of a
    // sequence repeats, and two workgroups on one compute unit take twice as long: narrower slabs
    // only as long as all workgroups still find a compute unit of their own (two sweeps share the
    // grid: 2 x 32 sequences x 4 slabs, 2 x 64 x 2, 2 x 128 x 1 fill the 256 units).
    if constexpr (DV == 128 && DK == 128) {
        if (sweep_walkers<ENDS>(d) <= 32) return launch_pair_one<T, DK, DV, 32, ENDS>(d, ps, pg, stream);
    }
    if constexpr (DV == 128) {
        if (sweep_walkers<ENDS>(d) <= 64) return launch_pair_one<T, DK, DV, 64, ENDS>(d, ps, pg, stream);
    }
    return launch_pair_one<T, DK, DV, DV, ENDS>(d, ps, pg, stream);
}

template <typename T, int DK, int DV, int TV, int MODE, bool ENDS>
static hipError_t launch_one(const SeqDims& d, const SweepParams& p0, hipStream_t stream)
{
    SweepParams p = p0;
    p.n_tile = DV / TV;
    constexpr int PC = kChunk + pad_elems<T>();
    const size_t lds = (size_t)(DK + TV) * PC * sizeof(T) + (size_t)(2 + kWaves) * DK * sizeof(float);
    auto kern = sweep_kernel<T, DK, DV, TV, MODE, ENDS>;
    hipError_t e = allow_dynamic_lds(reinterpret_cast<const void*>(kern), (int)lds);
    if (e != hipSuccess) return e;
    const int seq_pad = (sweep_walkers<ENDS>(d) + 7) / 8 * 8;
    hipLaunchKernelGGL(kern, dim3(seq_pad * p.n_tile), dim3(kThreads), lds, stream, p);
    return hipGetLastError();
}

template <typename T, int DK, int DV, int MODE, bool ENDS>
static hipError_t launch_tv(const SeqDims& d, const SweepParams& p, hipStream_t stream)
{
    // Narrow slabs when there are few sequences, as long as every workgroup gets a compute unit of its own.
    if constexpr (DV == 128 && DK == 128) {
        if (sweep_walkers<ENDS>(d) <= 64) return launch_one<T, DK, DV, 32, MODE, ENDS>(d, p, stream);
    }
    if constexpr (DV == 128) {
        if (sweep_walkers<ENDS>(d) <= 128) return launch_one<T, DK, DV, 64, MODE, ENDS>(d, p, stream);
    }
    return launch_one<T, DK, DV, DV, MODE, ENDS>(d, p, stream);
}

template <typename T, int MODE, bool ENDS>
static hipError_t launch_dims_e(const SeqDims& d, const SweepParams& p, hipStream_t stream)
{
    if (d.dk == 128 && d.dv == 128) return launch_tv<T, 128, 128, MODE, ENDS>(d, p, stream);
    if (d.dk == 64 && d.dv == 64) return launch_tv<T, 64, 64, MODE, ENDS>(d, p, stream);
    if (d.dk == 128 && d.dv == 64) return launch_tv<T, 128, 64, MODE, ENDS>(d, p, stream);
    if (d.dk == 64 && d.dv == 128) return launch_tv<T, 64, 128, MODE, ENDS>(d, p, stream);
    return hipErrorInvalidValue;
}

// A caller that asks for the gate products wants a walk from zero: only the end state and the
// products, nothing per chunk.  (A null workspace alone does not say so: an empty sequence needs
// none, and its end state is the initial one.)
template <typename T, int MODE>
static hipError_t launch_dims(const SeqDims& d, const SweepParams& p, hipStream_t stream)
{
    return p.decay ? launch_dims_e<T, MODE, true>(d, p, stream) : launch_dims_e<T, MODE, false>(d, p, stream);
}

hipError_t launch_sweep(const SeqDims& d, SweepMode mode, const void* q, const void* f, const void* b_src,
                        const float* init_state, float* final_state, void* ws, float* decay, hipStream_t stream)
{
    if (d.BH == 0) return hipSuccess;
    SweepParams p;
    p.q = q; p.f = f; p.bsrc = b_src; p.init = init_state; p.fin = final_state; p.ws = ws; p.decay = decay;
    p.BH = d.BH; p.N = d.N; p.NC = d.NC; p.n_tile = 1; p.gate_bf16 = d.gate_bf16 ? 1 : 0;
    p.beta = d.beta; p.H = d.H; p.lay = d.lay; p.dense = d.dense() ? 1 : 0;
    if (d.io_bf16) {
        switch (mode) {
        case kSweepStateFwd: return launch_dims<__bf16, kSweepStateFwd>(d, p, stream);
        case kSweepStateBwd: return launch_dims<__bf16, kSweepStateBwd>(d, p, stream);
        case kSweepGrad:     return launch_dims<__bf16, kSweepGrad>(d, p, stream);
        }
    } else {
        switch (mode) {
        case kSweepStateFwd: return launch_dims<float, kSweepStateFwd>(d, p, stream);
        case kSweepStateBwd: return launch_dims<float, kSweepStateBwd>(d, p, stream);
        case kSweepGrad:     return launch_dims<float, kSweepGrad>(d, p, stream);
        }
    }
    return hipErrorInvalidValue;
}

hipError_t launch_sweep_pair(const SeqDims& d, const void* q, const void* f, const void* v, const void* grad_o,
                             const float* h0, const float* grad_hT, float* grad_h0, void* ws_state,
                             void* ws_dstate, hipStream_t stream)
{
    if (d.BH == 0) return hipSuccess;
    if (!d.io_bf16) return hipErrorInvalidValue;
    SweepParams ps, pg;
    ps.decay = pg.decay = nullptr;
    ps.q = nullptr; ps.f = f; ps.bsrc = v; ps.init = h0; ps.fin = nullptr; ps.ws = ws_state;
    pg.q = q; pg.f = f; pg.bsrc = grad_o; pg.init = grad_hT; pg.fin = grad_h0; pg.ws = ws_dstate;
    ps.BH = pg.BH = d.BH; ps.N = pg.N = d.N; ps.NC = pg.NC = d.NC; ps.n_tile = pg.n_tile = 1;
    ps.gate_bf16 = pg.gate_bf16 = d.gate_bf16 ? 1 : 0;
    ps.beta = pg.beta = d.beta; ps.H = pg.H = d.H; ps.lay = pg.lay = d.lay; ps.dense = pg.dense = d.dense() ? 1 : 0;
    if (d.dk == 128 && d.dv == 128) return launch_pair_tv<__bf16, 128, 128, false>(d, ps, pg, stream);
    if (d.dk == 64 && d.dv == 64) return launch_pair_tv<__bf16, 64, 64, false>(d, ps, pg, stream);
    if (d.dk == 128 && d.dv == 64) return launch_pair_tv<__bf16, 128, 64, false>(d, ps, pg, stream);
    if (d.dk == 64 && d.dv == 128) return launch_pair_tv<__bf16, 64, 128, false>(d, ps, pg, stream);
    return hipErrorInvalidValue;
}

hipError_t launch_sweep_pair_ends(const SeqDims& d, const void* q, const void* f, const void* v, const void* grad_o,
                                  float* run_state, float* run_dstate, float* run_decay, hipStream_t stream)
{
    if (d.BH == 0) return hipSuccess;
    if (!d.io_bf16) return hipErrorInvalidValue;
    SweepParams ps, pg;
    ps.decay = run_decay; pg.decay = nullptr;        // both walks pass the same gates: one copy of their product
    ps.q = nullptr; ps.f = f; ps.bsrc = v; ps.init = nullptr; ps.fin = run_state; ps.ws = nullptr;
    pg.q = q; pg.f = f; pg.bsrc = grad_o; pg.init = nullptr; pg.fin = run_dstate; pg.ws = nullptr;
    ps.BH = pg.BH = d.BH; ps.N = pg.N = d.N; ps.NC = pg.NC = d.NC; ps.n_tile = pg.n_tile = 1;
    ps.gate_bf16 = pg.gate_bf16 = d.gate_bf16 ? 1 : 0;
    ps.beta = pg.beta = d.beta; ps.H = pg.H = d.H; ps.lay = pg.lay = d.lay; ps.dense = pg.dense = d.dense() ? 1 : 0;
    if (d.dk == 128 && d.dv == 128) return launch_pair_tv<__bf16, 128, 128, true>(d, ps, pg, stream);
    if (d.dk == 64 && d.dv == 64) return launch_pair_tv<__bf16, 64, 64, true>(d, ps, pg, stream);
    if (d.dk == 128 && d.dv == 64) return launch_pair_tv<__bf16, 128, 64, true>(d, ps, pg, stream);
    if (d.dk == 64 && d.dv == 128) return launch_pair_tv<__bf16, 64, 128, true>(d, ps, pg, stream);
    return hipErrorInvalidValue;
}

// ---- segmented sweeps: the state entering every run ------------------------------------------
// run_state[s][r] holds what run r of sequence s adds (the slab a walk from zero leaves),
// run_decay[s][r][k] the product of the run's gates.  Walking the runs in order (backwards for
// the gradient) with  S <- Diag(decay_r) S + add_r  from the carried-in state gives the state
// entering each run, which replaces add_r in place, and the state leaving the sequence.
__global__ __launch_bounds__(256) void run_carry_kernel(const float* carried_in, float* run_state, const float* run_decay,
                                                        float* carried_out, int seg, const int* first_run, int H,
                                                        int dk, int dv, int reverse, const int* choice, int path)
{
    if (choice && table_read(choice, 0) != path) return;        // one of several alternatives, and not the one called for
    const size_t per = (size_t)dk * dv;
    const size_t e4 = ((size_t)blockIdx.x * blockDim.x + threadIdx.x) * 4;
    if (e4 >= per) return;
    const int s = blockIdx.y, k = (int)(e4 / dv);
    // runs of sequence s: `seg` consecutive slots, or (packed batch) those the table names, H slots apart
    size_t slot0 = (size_t)s * seg, step = 1;
    int n_runs = seg;
    if (first_run) {
        const int b = s / H, h = s - b * H;
        slot0 = (size_t)first_run[b] * H + h;
        step = H;
        n_runs = first_run[b + 1] - first_run[b];
    }
    f32x4 st = {0.0f, 0.0f, 0.0f, 0.0f};
    if (carried_in) st = *reinterpret_cast<const f32x4*>(carried_in + (size_t)s * per + e4);
    for (int j = 0; j < n_runs; ++j) {
        const size_t r = slot0 + step * (reverse ? n_runs - 1 - j : j);
        f32x4* slot = reinterpret_cast<f32x4*>(run_state + r * per + e4);
        const f32x4 add = *slot;
        const float g = run_decay[r * dk + k];
        *slot = st;
        st = st * g + add;
    }
    if (carried_out) *reinterpret_cast<f32x4*>(carried_out + (size_t)s * per + e4) = st;
}

hipError_t launch_run_carry(int n_seq, int seg, int dk, int dv, const float* carried_in, float* run_state,
                            const float* run_decay, float* carried_out, bool reverse, hipStream_t stream,
                            const int* choice, int path)
{
    if (n_seq == 0) return hipSuccess;
    const unsigned blocks = (unsigned)(((size_t)dk * dv / 4 + 255) / 256);
    hipLaunchKernelGGL(run_carry_kernel, dim3(blocks, n_seq), dim3(256), 0, stream, carried_in, run_state, run_decay,
                       carried_out, seg, static_cast<const int*>(nullptr), 1, dk, dv, reverse ? 1 : 0, choice, path);
    return hipGetLastError();
}

hipError_t launch_run_carry_packed(int B, int H, const int* first_run, int dk, int dv, const float* carried_in,
                                   float* run_state, const float* run_decay, float* carried_out, bool reverse,
                                   hipStream_t stream, const int* choice, int path)
{
    if (B * H == 0) return hipSuccess;
    const unsigned blocks = (unsigned)(((size_t)dk * dv / 4 + 255) / 256);
    hipLaunchKernelGGL(run_carry_kernel, dim3(blocks, B * H), dim3(256), 0, stream, carried_in, run_state, run_decay,
                       carried_out, 0, first_run, H, dk, dv, reverse ? 1 : 0, choice, path);
    return hipGetLastError();
}

size_t state_ws_bytes(const SeqDims& d)
{
    return d.total_chunks() * d.dk * d.dv * (d.io_bf16 ? 2 : 4);
}

}   // namespace hgrn2
