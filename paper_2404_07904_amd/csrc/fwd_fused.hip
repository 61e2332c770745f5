// Fused forward pass of the chunkwise HGRN2 algorithm (paper Section 3.2, Eq. 3): the
// chunk-to-chunk state recurrence and the per-chunk read-out in ONE pass over q, f, v,
//
//     O_n     = tril(Q~ K~^T) V + Q~ (G_m S_n)
//     S_{n+1} = h (G_m S_n + K~^T V)
//
// with Q~ = q G/G_m, K~ = k G_m/G (k = 1 - f, G the cumulative gate product inside the chunk, G_m
// its value after the first half of the chunk, h the product over the second half), so that the
// per-chunk states never travel through HBM (the two-kernel path writes and re-reads 2*dk*dv
// bytes per chunk, as much again as the chunk's own q, f, v, o).  One workgroup of eight wave64s
// owns a whole (batch, head) and walks its chunks in order, software-pipelined in two stages
// per chunk with one barrier after each:
//
//   stage A(n):  store O(n-1) from its LDS staging tile; copy V(n) into LDS; rescale the state
//                to G_m(n) S_n and publish it (bf16, MFMA-fragment order) to LDS; first half of
//                the element-wise work of chunk n+1 (gate products, per-wave block totals);
//                P(n) = tril(Q~ K~^T) on three waves
//   stage B(n):  all remaining contractions of chunk n (Q~ (G_m S_n), P V, K~^T V) while the
//                second half of the element-wise work of chunk n+1 (Q~, K~ tiles) fills the
//                other tile buffer; O(n) into its staging tile
//
//   * the dk x dv state lives in fp32 MFMA accumulators, two 32x32 tiles per wave;
//   * wave w owns rows 8w..8w+7 of the chunk for the element-wise work (gate products along time
//     serially in registers, channel pair per lane) and the 32x32 output tile (w/4, w%4);
//   * V is a raw row-major [token][channel] copy (no arithmetic on its way in) and is read with LDS
//     transpose loads; K~ is kept transposed ([channel][token], which the row-block layout writes
//     as 16-byte vectors), so that the state update reads it with plain 16-byte loads; Q~ keeps
//     its columns in the order the state fragments hold the contraction index (bits 2 and 3 of
//     the channel swapped), so that its operand of the read-out is one 16-byte load too;
//   * rows are fetched two chunks ahead into two alternating register sets.
//   * with fewer sequences than compute units, two workgroups share a sequence, each owning one
//     half of the dv columns (of V, O and the state): the element-wise work on q and f and the
//     P blocks are done twice, everything that scales with dv is halved, and the whole chip is busy.
//   * a packed batch with a group table gives a workgroup a group of consecutive sequences of one
//     head: the pipeline runs on across the sequence boundaries (the rows of the next sequence's
//     first chunks are fetched while the current one ends), the state is replaced by the next
//     sequence's initial state where it starts and written out where one ends.  Many short
//     sequences then cost the start-up of a workgroup once per group, not once per sequence.
// Used for bf16 storage with dk = dv = 128 when there are enough sequences to fill the chip;
// other cases take the sweep + read-out path.
#include "common.hpp"
#include "kernels.hpp"
#include <type_traits>

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
    void* save;          // null, or where every chunk's scaled incoming state G_m S_n goes for a later backward pass
    int N, NC, BH;
    const float* beta;   // [H][dk] lower bounds, or null: the gate tensor holds f itself
    int H;
    TokenLayout lay;     // used when dense == 0
    int dense;           // sequence tensors are [B][H][N][d]: token strides are the compile-time dk, dv
    int* flag;           // null, or set to 1 when a gate product falls below the floor of the reciprocals
};


template <int NSPLIT> struct FwdFusedLds {
    static constexpr int DK = 128, DV = 128, DVW = DV / NSPLIT, C = kChunk;   // DVW: dv columns of one workgroup
    // Row pitches in elements.  Tiles read row-major with 16-byte vectors want consecutive rows
    // 4 banks apart (+8 elements); tiles read with transpose loads (4 rows x 64 bytes per half
    // wave) want them 16 banks apart (+32 elements).
    static constexpr int PQ = DK + 8, PT = C + 8, PV = DVW + 32, PC = C + 8, PO = DVW + 8;
    static constexpr size_t qm = 0;                                     // Q~    [2][C][PQ], columns in fragment order
    static constexpr size_t km = qm + (size_t)2 * C * PQ * 2;           // K~^T  [2][DK][PT]
    static constexpr size_t vm = km + (size_t)2 * DK * PT * 2;          // V     [C][PV]
    static constexpr size_t pm = vm + (size_t)C * PV * 2;               // P   [C][PC]
    static constexpr size_t sb = pm + (size_t)C * PC * 2;               // G_m S_n, bf16, fragment order
    static constexpr int NSB = (NSPLIT == 2) ? 2 : 1;                  // copies of the published state (see LATE_QS)
    static constexpr size_t ost = sb + (size_t)NSB * DK * DVW * 2;      // O   [C][PO]
    static constexpr size_t tot = ost + (size_t)C * PO * 2;             // [8][DK] fp32 block totals + one row of ones
    static constexpr size_t ca = tot + (size_t)(kFusedWaves + 1) * DK * 4;   // [DK] fp32 state rescale
    static constexpr size_t ch = ca + (size_t)DK * 4;                   // [DK] fp32 h of the chunk before (grouped walks)
    static constexpr size_t total = ch + (size_t)DK * 4;
    static_assert(total <= 160 * 1024, "LDS budget of one workgroup");
};

// One chunk of the walk: tokens row0 .. row0 + C - 1 of a sequence of N tokens whose first token is
// token tok0 of the packed tensors (grouped walks; 0 otherwise).  N = 0: a pass past the end.
// `slot` is the chunk's place in an array with one entry per chunk of the batch (the kept states).
// Row r of the chunk stands for token row0 + r of the sequence where lo <= row0 + r < hi and for no
// token elsewhere (past the end of the sequence; in the small-gate modes, outside the chunk's middle
// rows: ChunkRows).
struct FusedChunk {
    int tok0, row0, N, bh, first, last, slot, lo, hi;
};

template <bool GATE_BF16, int NSPLIT, bool DENSE, bool GROUPED>
__device__ __forceinline__ void fwd_fused_body(const FwdFusedParams& p)
{
    static_assert(!(DENSE && GROUPED), "groups are a feature of packed batches");
    typedef __bf16 T;
    typedef Mma<T> M;
    typedef typename M::frag frag;
    typedef FwdFusedLds<NSPLIT> L;
    constexpr int DK = L::DK, DV = L::DV, DVW = L::DVW, C = L::C, NW = kFusedWaves, RW = C / NW;
    constexpr int PQ = L::PQ, PT = L::PT, PV = L::PV, PC = L::PC, PO = L::PO;
    constexpr int NBT = DVW / 32, NKS = DK / 16;
    constexpr int NST = (DK / 32) * NBT / NW;        // state tiles per wave: 2 (whole dv) or 1 (half)
    constexpr int NOT = (C / 32) * NBT;              // output tiles of the workgroup: waves 0 .. NOT-1 own one
    constexpr int PW0 = (NOT == NW) ? 0 : NOT;       // first of the three waves that compute the P blocks
    // With half the dv columns per workgroup only four waves own an output tile; their read-out of
    // the incoming state, Q~ (G_m S_n), is then issued one stage late, in stage A of the next pass,
    // next to the P blocks the other waves compute there (the published state is double-buffered
    // for that, and O(n) leaves in stage B of pass n+1).  This evens out the matrix work of the
    // two stages.
    constexpr bool LATE_QS = (NSPLIT == 2);
    // With the smaller register footprint of the split variant, every MFMA chain requests all its
    // operand fragments first and the instruction scheduler is told not to sink those loads back
    // between the MFMAs: one LDS latency per chain instead of one per k-step pair.
    constexpr bool BATCH_LOADS = (NSPLIT == 2);
    constexpr int KB8 = BATCH_LOADS ? DK / 16 : 2, KB4 = BATCH_LOADS ? kChunk / 16 : 1;   // k-steps per batch
    static_assert(RW == 8 && NST * NW == (DK / 32) * NBT && NOT <= NW && PW0 + 3 <= NW, "tile/wave mapping");

    extern __shared__ __align__(16) char smem[];
    T* Qm = reinterpret_cast<T*>(smem + L::qm);
    T* Km = reinterpret_cast<T*>(smem + L::km);
    T* Vm = reinterpret_cast<T*>(smem + L::vm);
    T* Pm = reinterpret_cast<T*>(smem + L::pm);
    T* Sb = reinterpret_cast<T*>(smem + L::sb);
    T* Ost = reinterpret_cast<T*>(smem + L::ost);
    float* tot = reinterpret_cast<float*>(smem + L::tot);
    float* cA = reinterpret_cast<float*>(smem + L::ca);
    float* cH = reinterpret_cast<float*>(smem + L::ch);

    if (not_chosen(p.lay)) return;       // one of several chunk lengths, and not the one called for
    // workgroup -> (sequence, dv half): ids 8 apart land on the same XCD (ids are dealt to the 8
    // XCDs round-robin), so the two halves of a sequence share an L2 for the q, f rows both read
    int bh, split;
    if (NSPLIT == 1) { bh = blockIdx.x; split = 0; }
    else { const int x = blockIdx.x & 7, r = blockIdx.x >> 3; split = r % NSPLIT; bh = (r / NSPLIT) * 8 + x; }
    // padding of the grid (uniform, before any barrier)
    if (bh >= (GROUPED ? p.lay.G * p.lay.H : p.BH)) return;
    // grouped: the sequences e0 .. e1 - 1 of head `head`, found through the table's arrays
    int e0 = 0, e1 = 0, head = 0;
    const int* t_start = p.lay.vl;
    const int* t_len = p.lay.vl + (p.lay.B + 1);
    if constexpr (GROUPED) {
        const int grp = bh / p.lay.H;
        head = bh - grp * p.lay.H;
        e0 = table_read(p.lay.groups, grp); e1 = table_read(p.lay.groups, grp + 1);
        bh = e0 * p.lay.H + head;            // (only for the view below, whose chunk count is replaced)
    } else {
        bh = sequence_of_workgroup<DENSE>(p.lay, bh);
    }
    const int dv0 = split * DVW;             // first dv column of this workgroup
    const int tid = threadIdx.x, lane = tid & 63, r32 = lane & 31, g = lane >> 5;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);      // wave index, in a scalar register
    SeqView sv;
    if constexpr (GROUPED) {
        // addresses are formed from token numbers: the view is the head's slice of the whole tensor
        sv.off_k = (size_t)head * p.lay.sh_k; sv.off_v = (size_t)head * p.lay.sh_v; sv.chunk0 = 0;
        sv.N = 0;
        sv.NC = table_read(p.lay.vl, 2 * (p.lay.B + 1) + e1) - table_read(p.lay.vl, 2 * (p.lay.B + 1) + e0);   // chunks of all the group's sequences
    } else {
        sv = seq_view<DENSE, DK, DV, true>(p.lay, p.N, p.NC, bh);
    }
    const size_t seq_k = sv.off_k, seq_v = sv.off_v;
    const int ld_k = DENSE ? DK : (int)p.lay.sn_k, ld_v = DENSE ? DV : (int)p.lay.sn_v;   // token stride, elements
    const T* qg = static_cast<const T*>(p.q);
    const T* vg = static_cast<const T*>(p.v);
    T* og = static_cast<T*>(p.o);
    const int NC = sv.NC;                    // passes over chunks with tokens

    const int rt = w / NBT, bt = w % NBT;    // output tile (rt, bt) of this wave, if w < NOT
    const int at0 = NST * (w / NBT);         // its state tiles: (at0 .. at0 + NST - 1, bt)
    const bool has_o = (NOT == NW) || w < NOT;
    const bool is_p = w >= PW0 && w < PW0 + 3;
    const bool after = w >= NW / 2;          // rows of this wave lie after the mid-chunk reference

    // a sequence without tokens ends in the state it starts from
    auto pass_state_on = [&](int seq) {
        if (p.hT)
            for (int idx = tid; idx < DK * DVW; idx += kFusedThreads) {
                const size_t e = (size_t)seq * DK * DV + (size_t)(idx / DVW) * DV + dv0 + idx % DVW;
                p.hT[e] = p.h0 ? p.h0[e] : 0.0f;
            }
    };
    if constexpr (GROUPED) {
        for (int e = e0; e < e1; ++e)
            if (table_read(t_len, e) == 0) pass_state_on(e * p.lay.H + head);
        if (NC == 0) return;                 // (uniform early exit, before any barrier)
    } else if (NC == 0) {
        pass_state_on(bh);
        return;
    }

    // ---- the chunks of the walk, in order.  Grouped walks step through the group's sequences with
    // a cursor that runs three chunks ahead of the pass (everything here is wave-uniform).
    int cur_e = e0 - 1, cur_n = 0, cur_nc = 0, cur_tok = 0, cur_N = 0, cur_slot = 0;
    auto next_chunk = [&]() {
        FusedChunk c;
        if (cur_n + 1 < cur_nc) ++cur_n;
        else {
            int e = cur_e + 1, len = 0;
            while (e < e1 && (len = table_read(t_len, e)) == 0) ++e;
            if (e < e1) {
                cur_e = e; cur_N = len; cur_nc = p.lay.chunks_of(len); cur_tok = table_read(t_start, e);
                // the chunks of (sequence, head) lie together, the heads of a sequence one after the other
                cur_slot = table_read(p.lay.vl, 2 * (p.lay.B + 1) + e) * p.lay.H + head * cur_nc;
            } else { cur_e = e1; cur_N = 0; cur_nc = 0; cur_tok = 0; cur_slot = 0; }          // past the end, for good
            cur_n = 0;
        }
        const ChunkRows cr = chunk_rows(p.lay.sub, cur_n, cur_N);
        c.tok0 = cur_tok; c.row0 = cr.tok0; c.lo = cr.first; c.hi = cr.end; c.N = cur_N; c.bh = cur_e * p.lay.H + head;
        c.first = cur_n == 0; c.last = cur_N > 0 && cur_n == cur_nc - 1; c.slot = cur_slot + cur_n;
        return c;
    };
    const int N_one = sv.N;
    auto chunk_at = [&](int c) {             // one sequence per workgroup: chunk c of it (any c >= -1)
        FusedChunk k;
        const ChunkRows cr = chunk_rows(p.lay.sub, c, N_one);
        k.tok0 = 0; k.row0 = cr.tok0; k.lo = cr.first; k.hi = cr.end;
        k.N = N_one; k.bh = bh; k.first = c == 0; k.last = c == NC - 1; k.slot = sv.chunk0 + c;
        return k;
    };
    // window of the pass: ck[j] = chunk n - 1 + j of pass n (grouped walks only)
    FusedChunk ck[5];
    if constexpr (GROUPED) {
        ck[0].tok0 = 0; ck[0].row0 = 0; ck[0].N = 0; ck[0].bh = bh; ck[0].first = 1; ck[0].last = 0; ck[0].slot = 0;
        ck[0].lo = 0; ck[0].hi = 0;
#pragma unroll
        for (int j = 1; j < 5; ++j) ck[j] = next_chunk();
    }
    auto chunk_rel = [&](int n, int rel) { return GROUPED ? ck[rel + 1] : chunk_at(n + rel); };

    // ---- state: fp32 accumulators.  Between chunks they hold S_n / h(n-1); see stage A. ----
    f32x16 accS[NST];
    // Element (tile j, register v) of this lane in a [dk][dv] fp32 state: a wave-uniform address
    // (sequence, tile, group of four registers) plus one per-lane 32-bit byte offset plus a small
    // constant, so that no access needs an address register of its own.
    const uint32_t st_lane = (uint32_t)(4 * g * DV + dv0 + 32 * bt + r32) * 4u;
    auto state_rows = [&](const float* base, int seq, int j, int c) {
        return reinterpret_cast<const char*>(base) + ((size_t)seq * DK * DV + (size_t)(32 * (at0 + j) + 8 * c) * DV) * 4;
    };
    auto initial_state = [&](int seq) {
#pragma unroll
        for (int j = 0; j < NST; ++j)
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const char* rows = state_rows(p.h0, seq, j, c);
#pragma unroll
                for (int jj = 0; jj < 4; ++jj)
                    accS[j][4 * c + jj] = p.h0 ? *reinterpret_cast<const float*>(rows + st_lane + jj * DV * 4) : 0.0f;
            }
    };
    // accumulators *= per-channel factors in LDS (channel = accumulator row)
    auto scale_state = [&](const float* factor) {
#pragma unroll
        for (int j = 0; j < NST; ++j)
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const f32x4 cm = *reinterpret_cast<const f32x4*>(factor + 32 * (at0 + j) + 8 * c + 4 * g);
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) accS[j][4 * c + jj] *= cm[jj];
            }
    };
    // the state after the chunk before: scale * accumulators, formed in place (what follows either
    // replaces the accumulators or is the end of the walk)
    auto final_state = [&](int seq, const float* scale) {
        scale_state(scale);
#pragma unroll
        for (int j = 0; j < NST; ++j)
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                char* rows = const_cast<char*>(state_rows(p.hT, seq, j, c));
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) *reinterpret_cast<float*>(rows + st_lane + jj * DV * 4) = accS[j][4 * c + jj];
            }
    };
    initial_state(GROUPED ? ck[1].bh : bh);
    float hprev0 = 1.0f, hprev1 = 1.0f;      // h of the previous chunk, channels 2*lane, 2*lane+1 (wave 0 only)

    // ---- row fetch, two chunks ahead, two register sets ----
    RawRows<RW> rawf[2], rawq[2];
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    constexpr int VPR = DVW / 8;             // 16-byte vectors per V / O row
    constexpr int NVV = VPR / 8;             // vectors per thread
    constexpr int VRS = 64 / VPR;            // rows one wave covers per vector
    // V: two chunks ahead too, in alternating sets, where the registers allow it (fp32 gates take
    // twice the prefetch registers of bf16 ones; V is then fetched one chunk ahead)
    constexpr int VD = GATE_BF16 ? 2 : 1;
    u32x4 rawv[VD][NVV];
    const int vrow = RW * w + lane / VPR, vcol = 8 * (lane % VPR);      // V copy: 16 bytes per lane, rows vrow (+ VRS)
    // Every load is issued unconditionally (a row past the end of the sequence re-reads the last
    // row), and the chunk loop always runs an even number of passes, so that its body is
    // straight-line code: the compiler can then count outstanding loads exactly and the two
    // register sets never have to be copied.  A pass over a chunk index >= NC sees gates equal
    // to one on every row and is an exact no-op on the state.  Row addresses are wave-uniform.
    const char* fbase = static_cast<const char*>(p.f) + seq_k * (GATE_BF16 ? 2 : 4);
    const char* qbase = reinterpret_cast<const char*>(qg + seq_k);
    const char* vbase = reinterpret_cast<const char*>(vg + seq_v + dv0);
    auto load_f = [&](RawRows<RW>& d, const FusedChunk& c) {
        load_rows_clamped<RW, GATE_BF16>(d, fbase + (size_t)c.tok0 * ((size_t)ld_k * (GATE_BF16 ? 2 : 4)), c.row0 + RW * w,
                                         max(c.N - 1, 0), ld_k, 2 * lane);
    };
    auto load_q = [&](RawRows<RW>& d, const FusedChunk& c) {
        load_rows_clamped<RW, true>(d, qbase + (size_t)c.tok0 * ((size_t)ld_k * 2), c.row0 + RW * w, max(c.N - 1, 0), ld_k, 2 * lane);
    };
    auto load_v = [&](u32x4 (&d)[NVV], const FusedChunk& c) {
        const int row0 = c.row0 + RW * w, last_row = max(c.N - 1, 0);
        const char* vb = vbase + (size_t)c.tok0 * ((size_t)ld_v * 2);
#pragma unroll
        for (int j = 0; j < NVV; ++j) {
            const int rc = min(max(row0 + lane / VPR + VRS * j, 0), last_row);
            d[j] = *reinterpret_cast<const u32x4*>(vb + (size_t)rc * ((size_t)ld_v * 2) + 2 * vcol);
        }
    };
    // Rows past the end of the sequence need no masking here: their K~ is zero (f = 1 there), so
    // whatever finite values stand in for them never reach a stored output or the state.
    auto store_v = [&](const u32x4 (&s)[NVV]) {
#pragma unroll
        for (int j = 0; j < NVV; ++j) *reinterpret_cast<u32x4*>(Vm + (vrow + VRS * j) * PV + vcol) = s[j];
    };

    // ---- element-wise work of one chunk, split around the exchange of the block totals ----
    // With a = inclusive gate product from the start of this wave's 8-row block, z = exclusive
    // product to its end, t = a z the block total, mid = product of the blocks between this block
    // and the mid-chunk reference row, and m = product of the gates between the reference row and
    // this row:
    //   rows after the reference:  Q~ = q m,   K~ = k / m,   m = mid a,  1/m = z / (mid t)
    //   rows before it:            Q~ = q / m, K~ = k m,     m = mid z,  1/m = a / (mid t)
    // so Q~ = (q a) s_a and K~ = (k z) s_z with per-channel block factors s_a, s_z in {mid,
    // 1/(mid t)}: one reciprocal per channel and block, floored so that it stays finite outside
    // the supported gate range.
    // First half (before the totals are exchanged): q a, k z, t.
    float qa0[RW], qa1[RW], kz0[RW], kz1[RW], bt0, bt1;
    float below_floor = 1.0f;            // smallest product a reciprocal was taken of (reported once, at the end)
    auto prep_gates = [&](const RawRows<RW>& rf_raw, const RawRows<RW>& rq_raw, const FusedChunk& c) {
        f32x2 rf[RW];
        convert_rows<RW>(rf, rf_raw, c.row0 + RW * w, c.hi, true, GATE_BF16, 1.0f, c.lo);
        if (p.beta)
            gate_rows<RW>(rf, p.beta + (size_t)(GROUPED ? head : bh / p.lay.seg % p.H) * DK, 2 * lane, true, c.row0 + RW * w, c.hi, c.lo);
        float run0 = 1.0f, run1 = 1.0f;
#pragma unroll
        for (int i = 0; i < RW; ++i) {
            const uint32_t u = __float_as_uint(rq_raw.r[i].x);
            run0 *= rf[i].x; run1 *= rf[i].y;
            qa0[i] = __uint_as_float(u << 16) * run0;
            qa1[i] = __uint_as_float(u & 0xffff0000u) * run1;
        }
        bt0 = run0; bt1 = run1;
        run0 = 1.0f; run1 = 1.0f;
#pragma unroll
        for (int i = RW - 1; i >= 0; --i) {      // k z = (1 - f) z = z_i - z_{i-1}
            const float n0 = run0 * rf[i].x, n1 = run1 * rf[i].y;
            kz0[i] = run0 - n0; kz1[i] = run1 - n1;
            run0 = n0; run1 = n1;
        }
        *reinterpret_cast<f32x2*>(tot + w * DK + 2 * lane) = f32x2{bt0, bt1};
    };
    // Second half: block factors from the exchanged totals, tiles to LDS.
    auto prep_tiles = [&](int c, bool starts_sequence) {      // c: only its parity matters (which tile buffer)
        // product of the (at most three) block totals between this block and the reference row;
        // the row addresses are wave-uniform, an absent factor reads the row of ones
        const float* ones = tot + NW * DK;
        const float* r1 = after ? (w > 4 ? tot + 4 * DK : ones) : (w < 3 ? tot + 3 * DK : ones);
        const float* r2 = after ? (w > 5 ? tot + 5 * DK : ones) : (w < 2 ? tot + 2 * DK : ones);
        const float* r3 = after ? (w > 6 ? tot + 6 * DK : ones) : (w < 1 ? tot + 1 * DK : ones);
        const f32x2 m1 = *reinterpret_cast<const f32x2*>(r1 + 2 * lane);
        const f32x2 m2 = *reinterpret_cast<const f32x2*>(r2 + 2 * lane);
        const f32x2 m3 = *reinterpret_cast<const f32x2*>(r3 + 2 * lane);
        const float mid0 = m1.x * m2.x * m3.x, mid1 = m1.y * m2.y * m3.y;
        const float R0 = fast_rcp(fmaxf(mid0 * bt0, kTinyProduct));
        const float R1 = fast_rcp(fmaxf(mid1 * bt1, kTinyProduct));
        below_floor = fminf(below_floor, fminf(mid0 * bt0, mid1 * bt1));
        const float sa0 = after ? mid0 : R0, sa1 = after ? mid1 : R1;       // multiplies q a
        const float sz0 = after ? R0 : mid0, sz1 = after ? R1 : mid1;       // multiplies k z
        // Q~: row-major, channel pair (2l, 2l+1) at column position sigma(2l) (bits 2 and 3 swapped);
        // K~^T: this thread's 8 tokens of each of its two channels as one 16-byte vector
        const int qcol = ((2 * lane) & ~12) | (((2 * lane) & 4) << 1) | (((2 * lane) & 8) >> 1);
        T* Qd = Qm + (size_t)(c & 1) * C * PQ + (size_t)(RW * w) * PQ + qcol;
        T* Kd = Km + (size_t)(c & 1) * DK * PT + (size_t)(2 * lane) * PT + RW * w;
        float k0[RW], k1[RW];
#pragma unroll
        for (int i = 0; i < RW; ++i) {
            store_pair_t<T>(Qd, (size_t)i * PQ, qa0[i] * sa0, qa1[i] * sa1);
            k0[i] = kz0[i] * sz0; k1[i] = kz1[i] * sz1;
        }
        *reinterpret_cast<frag*>(Kd) = M::pack(k0);
        *reinterpret_cast<frag*>(Kd + PT) = M::pack(k1);
        // state rescale of the chunk, by wave 0: h of the previous chunk times G_m of this one
        if (w == 0) {
            f32x2 t[NW];
#pragma unroll
            for (int i = 0; i < NW; ++i) t[i] = *reinterpret_cast<const f32x2*>(tot + i * DK + 2 * lane);
            const float gm0 = (t[0].x * t[1].x) * (t[2].x * t[3].x), gm1 = (t[0].y * t[1].y) * (t[2].y * t[3].y);
            if constexpr (GROUPED) {
                // the state of a sequence's first chunk is its initial state, not what the walk carries;
                // and h alone turns the carried accumulators into the state a sequence ends in
                *reinterpret_cast<f32x2*>(cH + 2 * lane) = f32x2{hprev0, hprev1};
                if (starts_sequence) { hprev0 = 1.0f; hprev1 = 1.0f; }
            }
            *reinterpret_cast<f32x2*>(cA + 2 * lane) = f32x2{hprev0 * gm0, hprev1 * gm1};
            hprev0 = (t[4].x * t[5].x) * (t[6].x * t[7].x); hprev1 = (t[4].y * t[5].y) * (t[6].y * t[7].y);
        }
    };

    // O leaves through registers that stay reserved for the whole pass (see the end of stage B):
    // a global store reads its data registers late, and overwriting them earlier would make the
    // wave wait for the store, and with it for every prefetch issued before it, to complete.
    u32x4 obuf[C * VPR / kFusedThreads];
    auto store_o = [&](const FusedChunk& c) {
#pragma unroll
        for (int k = 0; k < C * VPR / kFusedThreads; ++k) {
            const int idx = tid + k * kFusedThreads;
            const int row = idx / VPR, cv = idx % VPR;
            const int grow = c.row0 + row;
            obuf[k] = *reinterpret_cast<const u32x4*>(Ost + (size_t)row * PO + cv * 8);
            if (grow >= c.lo && grow < c.hi)       // also false for the chunk "-1" of the first pass
                *reinterpret_cast<u32x4*>(og + seq_v + ((size_t)c.tok0 + grow) * ld_v + dv0 + cv * 8) = obuf[k];
        }
    };


    // ---- prologue: rows of chunks 0 and 1 in flight, element-wise work of chunk 0 ----
    // the never-written block of P (rows 0..31 x columns 32..63) must read as zero
    for (int idx = tid; idx < 32 * 32; idx += kFusedThreads) Pm[(idx >> 5) * PC + 32 + (idx & 31)] = (T)0.0f;
    if (tid < DK) tot[NW * DK + tid] = 1.0f;
    load_f(rawf[0], chunk_rel(0, 0)); load_q(rawq[0], chunk_rel(0, 0)); load_v(rawv[0], chunk_rel(0, 0));
    load_f(rawf[1], chunk_rel(0, 1)); load_q(rawq[1], chunk_rel(0, 1));
    if (VD == 2) load_v(rawv[VD - 1], chunk_rel(0, 1));
    prep_gates(rawf[0], rawq[0], chunk_rel(0, 0));
    load_f(rawf[0], chunk_rel(0, 2)); load_q(rawq[0], chunk_rel(0, 2));
    __syncthreads();
    prep_tiles(0, true);
    __syncthreads();

    // output tile accumulator, transposed: accO[v] = O[token 32 rt + r32][channel 32 bt + 8 (v/4) + 4 g + v%4]
    f32x16 accO;
#pragma unroll
    for (int v = 0; v < 16; ++v) accO[v] = 0.0f;
    // (all operand fragments are requested before the first MFMA, so that one LDS latency is paid,
    // not one per k-step)
    auto read_out_state = [&](const T* Qx, const T* Sx) {        // accO += ((G_m S)^T Q~^T) tile (bt, rt)
#pragma unroll
        for (int k0 = 0; k0 < NKS; k0 += KB8) {
            frag sa[KB8], qa[KB8];
#pragma unroll
            for (int k = 0; k < KB8; ++k) {
                const int ks2 = k0 + k;
                sa[k] = *reinterpret_cast<const frag*>(Sx + state_frag_offset(ks2 >> 1, bt, NBT, ks2 & 1, lane));
                qa[k] = M::load(Qx + (32 * rt + r32) * PQ + 16 * ks2 + 8 * g);
            }
            if (BATCH_LOADS) __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int k = 0; k < KB8; ++k) M::mma(accO, sa[k], qa[k]);
        }
    };
    auto stage_o = [&]() {
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            bf16x4 pk;
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) pk[jj] = (T)accO[4 * c + jj];
            *reinterpret_cast<bf16x4*>(Ost + (size_t)(32 * rt + r32) * PO + 32 * bt + 8 * c + 4 * g) = pk;
        }
    };
    auto pin_obuf = [&]() {
#pragma unroll
        for (int k = 0; k < C * VPR / kFusedThreads; ++k) asm volatile("" :: "v"(obuf[k]));
    };

    // The published state holds, per lane, 8 channels of one dv column (the read-out contracts over
    // the channels).  A backward pass contracts over dv and wants 8 dv columns of one channel per
    // lane: the same bf16 values, regrouped by LDS transpose reads -- 16 lanes fetch 4 consecutive
    // channels of 4 dv columns each and get back 4 dv columns of one channel -- and written to
    // global memory as fragments (tile (channel tile, dv tile), half, lane) of 16 bytes per lane.
    constexpr int NSF = (DK / 32) * NBT * 2 / NW;        // fragments per wave and chunk
    auto save_state = [&](const T* Sx, int slot) {
        typedef __attribute__((address_space(3))) bf16x4 lds_bf16x4;
        T* dst = static_cast<T*>(p.save) + (size_t)slot * DK * DV;
        const int i16 = lane & 15;
        const int m = ((lane & 16) >> 2) + (i16 & 3);    // which 4 channels of the tile's 32 this lane fetches
        const int hs = m >> 2, q4 = (m >> 1) & 1, gs = m & 1;
#pragma unroll
        for (int j = 0; j < NSF; ++j) {
            const int id = w * NSF + j, half = id & 1, tb = (id >> 1) % NBT, ta = (id >> 1) / NBT;
            const int dl = 32 * tb + 16 * half + 4 * g + (i16 >> 2);        // local dv column this lane fetches (first read)
            const T* src = Sx + state_frag_offset(ta, tb, NBT, hs, 32 * gs + (dl & 31)) + 4 * q4;
            const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)(src));
            const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)(src + 8 * 8));   // dv column + 8: lane + 8
            const frag out = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            __builtin_nontemporal_store(__builtin_bit_cast(u32x4, out), reinterpret_cast<u32x4*>(dst + state_frag_offset(ta, dv0 / 32 + tb, DV / 32, half, lane)));
        }
    };

    auto chunk = [&](auto PAR, int n) {
        constexpr int par = decltype(PAR)::value;
        const T* Qc = Qm + (size_t)par * C * PQ;
        const T* Kc = Km + (size_t)par * DK * PT;
        T* Sp = Sb + (LATE_QS ? (size_t)par * DK * DVW : 0);      // where this pass publishes G_m(n) S_n
        // ======================= stage A =======================
        if (!LATE_QS) store_o(chunk_rel(n, -1));
        store_v(rawv[VD == 2 ? par : 0]);
        load_v(rawv[VD == 2 ? par : 0], chunk_rel(n, VD));
        if constexpr (GROUPED) {
            // sequence boundary: the walk's accumulators, times h of the chunk before, are the state
            // the sequence before ends in; this chunk starts from its own sequence's initial state
            if (ck[0].last && p.hT) final_state(ck[0].bh, cH);
            if (ck[1].first && n > 0 && ck[1].N > 0) initial_state(ck[1].bh);
        }
        // G_m(n) S_n = c(n) * accumulators, published as the bf16 operand of the read-out
        scale_state(cA);
#pragma unroll
        for (int j = 0; j < NST; ++j) {
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                float x[8];
#pragma unroll
                for (int s = 0; s < 8; ++s) x[s] = accS[j][8 * half + s];
                *reinterpret_cast<frag*>(Sp + state_frag_offset(at0 + j, bt, NBT, half, lane)) = M::pack(x);
            }
        }
        prep_gates(rawf[1 - par], rawq[1 - par], chunk_rel(n, 1));
        load_f(rawf[1 - par], chunk_rel(n, 3)); load_q(rawq[1 - par], chunk_rel(n, 3));
        if (LATE_QS) {
            // O(n-1) is completed here: its P V part was accumulated in stage B of the previous pass
            if (has_o) {
                read_out_state(Qm + (size_t)(1 - par) * C * PQ, Sb + (size_t)(1 - par) * DK * DVW);
                stage_o();
            }
            pin_obuf();
        }
        // P^T blocks (J <= I), one per wave
        if (is_p) {
            const int pb = w - PW0;
            const int I = (pb == 0) ? 0 : 1, J = (pb == 2) ? 1 : 0;   // 0:(0,0) 1:(0,1) 2:(1,1) as (J,I)
            f32x16 acc;
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[v] = 0.0f;
            // K~ operand: lane (token 32 J + r32, g) needs the channels of k-step ks in fragment order,
            // 16 ks + 4 g + {0..3} and 16 ks + 8 + 4 g + {0..3}: two transpose reads of K~^T rows
            typedef __attribute__((address_space(3))) bf16x4 lds_bf16x4;
            const int i16 = lane & 15;
            const T* kp = Kc + (size_t)(4 * g + (i16 >> 2)) * PT + 32 * J + (lane & 16) + 4 * (i16 & 3);
#pragma unroll
            for (int k0 = 0; k0 < NKS; k0 += KB8) {
                frag ka[KB8], qf[KB8];
#pragma unroll
                for (int k = 0; k < KB8; ++k) {
                    const int ks = k0 + k;
                    const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)(kp + (size_t)(16 * ks) * PT));
                    const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)(kp + (size_t)(16 * ks + 8) * PT));
                    ka[k] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                    qf[k] = M::load(Qc + (32 * I + r32) * PQ + 16 * ks + 8 * g);
                }
                if (BATCH_LOADS) __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int k = 0; k < KB8; ++k) M::mma(acc, ka[k], qf[k]);     // acc[row j][col i]
            }
            const int i_glob = 32 * I + r32;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const int j0 = 32 * J + 8 * c + 4 * g;
                float x[4];
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) x[jj] = (j0 + jj <= i_glob) ? acc[4 * c + jj] : 0.0f;
                bf16x4 pk;
                pk[0] = (T)x[0]; pk[1] = (T)x[1]; pk[2] = (T)x[2]; pk[3] = (T)x[3];
                *reinterpret_cast<bf16x4*>(Pm + (size_t)i_glob * PC + j0) = pk;
            }
        }
        __syncthreads();
        // ======================= stage B =======================
        // O^T tile (bt, rt) = V^T P^T + (G_m S)^T Q~^T   and   accumulators += K~^T V
        if (LATE_QS) store_o(chunk_rel(n, -1));
        if (p.save && n < NC) save_state(Sp, chunk_rel(n, 0).slot);
#pragma unroll
        for (int v = 0; v < 16; ++v) accO[v] = 0.0f;
#pragma unroll
        for (int k0 = 0; k0 < C / 16; k0 += KB4) {
            frag vf[KB4], kf[KB4][NST], pf[KB4];
#pragma unroll
            for (int k = 0; k < KB4; ++k) {
                const int ks = k0 + k;
                vf[k] = M::load_kmajor(Vm, PV, 16 * ks, 32 * bt, lane);
#pragma unroll
                for (int j = 0; j < NST; ++j) kf[k][j] = M::load(Kc + (32 * (at0 + j) + r32) * PT + 16 * ks + 8 * g);
                if (has_o) pf[k] = M::load(Pm + (32 * rt + r32) * PC + 16 * ks + 8 * g);   // zero block included
            }
            if (BATCH_LOADS) __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int k = 0; k < KB4; ++k) {
#pragma unroll
                for (int j = 0; j < NST; ++j) M::mma(accS[j], kf[k][j], vf[k]);
                if (has_o) M::mma(accO, vf[k], pf[k]);
            }
        }
        if (!LATE_QS) read_out_state(Qc, Sp);
        prep_tiles(n + 1, chunk_rel(n, 1).first != 0);
        if (!LATE_QS) {
            if (has_o) stage_o();
            pin_obuf();
        }
        if constexpr (GROUPED) {             // the window moves on by one chunk
#pragma unroll
            for (int j = 0; j < 4; ++j) ck[j] = ck[j + 1];
            ck[4] = next_chunk();
        }
        __syncthreads();
    };

    int n_end = 0;
    for (; n_end < NC; n_end += 2) {
        chunk(std::integral_constant<int, 0>(), n_end);
        chunk(std::integral_constant<int, 1>(), n_end + 1);
    }
    if (LATE_QS) {
        // an even number of chunks leaves the last one without its state read-out (an odd number
        // is followed by a pass over an empty chunk, which has done it)
        if (NC % 2 == 0) {
            if (has_o) {
                read_out_state(Qm + (size_t)((NC - 1) & 1) * C * PQ, Sb + (size_t)((NC - 1) & 1) * DK * DVW);
                stage_o();
            }
            __syncthreads();
            store_o(chunk_rel(NC, -1));
        }
    } else {
        store_o(chunk_rel(n_end, -1));
    }

    if (p.flag && below_floor < kTinyProduct) *p.flag = 1;
    if (p.hT) {
        // S_N = pending rescale * accumulators (the chunk after the last one has G_m = 1).  A
        // grouped walk has written the state of every sequence that a further pass followed; after
        // an even number of chunks the last sequence is still to do.
        if constexpr (GROUPED) {
            if (NC % 2 == 0) final_state(ck[0].bh, cH);
        } else {
            final_state(bh, cA);
        }
    }
}

template <bool GATE_BF16, int NSPLIT>
__global__ __launch_bounds__(kFusedThreads) void fwd_fused_kernel(FwdFusedParams p)
{
    if (p.dense) fwd_fused_body<GATE_BF16, NSPLIT, true, false>(p);
    else         fwd_fused_body<GATE_BF16, NSPLIT, false, false>(p);
}

// The walk over groups of a packed batch's sequences (a kernel of its own: its register needs are
// not those of the walk over one sequence).
template <bool GATE_BF16, int NSPLIT>
__global__ __launch_bounds__(kFusedThreads) void fwd_fused_grouped_kernel(FwdFusedParams p)
{
    fwd_fused_body<GATE_BF16, NSPLIT, false, true>(p);
}

// Groups of a packed batch's sequences are walked by one workgroup each from two sequences per
// group on (with fewer, a workgroup per sequence, longest first, balances uneven lengths better and
// needs less bookkeeping).
static bool fused_grouped(const SeqDims& d) { return d.lay.vl && d.lay.groups && d.lay.B >= 2 * d.lay.G; }
// workgroups' worth of independent walks
static int fused_walkers(const SeqDims& d) { return fused_grouped(d) ? d.lay.G * d.lay.H : d.BH; }

bool fwd_fused_supported(const SeqDims& d)
{
    return d.io_bf16 && d.dk == 128 && d.dv == 128 && fused_walkers(d) >= 64;
}

template <int NSPLIT>
static hipError_t launch_fused(const SeqDims& d, const FwdFusedParams& p, hipStream_t stream)
{
    typedef FwdFusedLds<NSPLIT> L;
    const bool grouped = fused_grouped(d);
    auto kern = grouped ? (d.gate_bf16 ? fwd_fused_grouped_kernel<true, NSPLIT> : fwd_fused_grouped_kernel<false, NSPLIT>)
                        : (d.gate_bf16 ? fwd_fused_kernel<true, NSPLIT> : fwd_fused_kernel<false, NSPLIT>);
    hipError_t e = allow_dynamic_lds(reinterpret_cast<const void*>(kern), (int)L::total);
    if (e != hipSuccess) return e;
    const int walkers = fused_walkers(d);
    const unsigned grid = (NSPLIT == 1) ? (unsigned)walkers : (unsigned)(NSPLIT * 8 * ((walkers + 7) / 8));
    hipLaunchKernelGGL(kern, dim3(grid), dim3(kFusedThreads), L::total, stream, p);
    return hipGetLastError();
}

hipError_t launch_fwd_fused(const SeqDims& d, const void* q, const void* f, const void* v, const float* h0,
                            void* o, float* hT, void* save_states, hipStream_t stream)
{
    if (d.BH == 0) return hipSuccess;
    FwdFusedParams p;
    p.q = q; p.f = f; p.v = v; p.h0 = h0; p.o = o; p.hT = hT; p.save = save_states;
    p.N = d.N; p.NC = d.NC; p.BH = d.BH; p.beta = d.beta; p.H = d.H; p.lay = d.lay; p.dense = d.dense() ? 1 : 0;
    p.flag = d.domain_flag;
    // Two workgroups per sequence (each half of the dv columns) keep twice as many compute units
    // busy, but a compute unit holds one workgroup: beyond 128 sequences the halves would no longer
    // all run at once (the rest waits for a free unit: 137 us instead of 84 us for 144 sequences of 2048 tokens), so
    // from there on a sequence gets one workgroup.
    return fused_walkers(d) > 128 ? launch_fused<1>(d, p, stream) : launch_fused<2>(d, p, stream);
}

}   // namespace hgrn2
