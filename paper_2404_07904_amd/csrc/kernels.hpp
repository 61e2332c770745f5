// Host-visible launch interface between the C-ABI translation unit and the kernel translation
// units.  Every launcher validates nothing (the C-ABI layer has done that), enqueues on the given
// stream and returns the hipError_t of the launch.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace hgrn2 {

// Compile-time chunk length of the chunkwise kernels.
constexpr int kChunk = 64;
constexpr int kFineChunk = 16;     // closest spacing of the reference rows in the small-gate modes; 32 is the other

// Where token (b, h, n) of q / f (channel count dk) and of v / o (dv) starts, in elements:
// b * sb + h * sh + n * sn.  [B][H][N][d] has sb = H N d, sh = N d, sn = d; [B][N][H][d] (what a
// projection writes) has sb = N H d, sh = d, sn = H d.  The d channels of a token are contiguous.
struct TokenLayout {
    long long sb_k, sh_k, sn_k, sb_v, sh_v, sn_v;
    int H;
    // Variable-length batches: B sequences packed back to back along the token axis of [T][H][d]
    // tensors.  `vl` is then the device table launch_varlen_table() builds, four arrays of B + 1
    // ints: first token of sequence b, its length, the number of chunks of the sequences before it
    // (entry B: of all sequences), and the sequences ordered by falling length.  Null for
    // equal-length batches.
    const int* vl = nullptr;
    int B = 0;
    // Packed batches of many short sequences: the kernels that walk sequences chunk by chunk give
    // a workgroup a GROUP of consecutive sequences of one head, sequences [groups[g], groups[g+1])
    // for group g of G (device array of G + 1 ints, launch_varlen_groups()), and walk them back to
    // back.  Null: one workgroup per sequence.
    const int* groups = nullptr;
    int G = 0;
    // The table kernel's choice between the two backward passes of such a batch (*choice = 1: the
    // fused reverse walk over groups; 0: the two sweeps, a workgroup per sequence, and the per-chunk
    // gradient kernel), made from the sizes of the groups; it is the int behind the group array.  The
    // kernels of both passes are enqueued, each with `path` set to the choice it belongs to, and
    // those of the other one return at once.  Null: no choice to make.
    // Equal-length batches use the same pair for the chunk length chosen on the device
    // (hgrn2_shape::chunk = HGRN2_CHUNK_AUTO): the passes for 64, 32 and 16 tokens per chunk are
    // enqueued one after the other and those not called for return at once.
    const int* choice = nullptr;
    int path = -1;
    // A second such pair, for packed batches (whose first one is taken by the choice of backward pass).
    const int* alt = nullptr;
    int alt_path = 0;
    // The fused reverse walk of a packed batch cuts the chunks of a head -- sequence after sequence,
    // `total` of them -- into `spans` equal pieces, span s = chunks [s total / spans, (s + 1) total /
    // spans), a workgroup each; a span may start and end inside a sequence.  0: no such walk.
    // `span_seq` names, span by span, the sequence the span ends in (device array of `spans` ints,
    // launch_varlen_groups() writes it behind the choice).
    int spans = 0;
    const int* span_seq = nullptr;
    // Segmented sweeps: each of the sequences the strides describe is cut into `seg` runs of whole
    // chunks that the sequential kernels treat as sequences of their own, `seg` per original one,
    // numbered run-fastest.  The kernels' N and NC are then those of a full run; `n_tokens` keeps
    // the length of the uncut sequence, whose last run may be shorter.
    int seg = 1;
    int n_tokens = 0;
    // Tokens per chunk: kChunk, or fewer in the small-gate modes, where a chunk's other rows stand for
    // no token (ChunkRows in common.hpp).  NC and the chunk counts of the tables count chunks of `sub` tokens.
    int sub = kChunk;
    // (a power of two: the chunks of `len` tokens are counted with a shift, not a division)
    __host__ __device__ int chunks_of(int len) const { return (len + sub - 1) >> (31 - __builtin_clz((unsigned)sub)); }
    __host__ __device__ size_t off_k(int bh) const { return (size_t)(bh / H) * sb_k + (size_t)(bh % H) * sh_k; }
    __host__ __device__ size_t off_v(int bh) const { return (size_t)(bh / H) * sb_v + (size_t)(bh % H) * sh_v; }
};

struct SeqDims {
    int BH;          // B * H independent sequences
    int N;           // tokens per sequence (variable-length batches: tokens of all sequences)
    int NC;          // chunks per sequence = ceil(N / kChunk) (variable-length: upper bound N / kChunk + B of all sequences' chunks)
    int dk, dv;
    bool io_bf16;    // q, v, o, grad_* storage: bf16 (else fp32)
    bool gate_bf16;  // f storage
    // Gate formed on the fly (paper Eq. 2): when `beta` is set, the gate tensor holds the
    // pre-activation z and f = beta + (1 - beta) sigmoid(z); beta is [H][dk] fp32 on the device.
    int H = 1;
    const float* beta = nullptr;
    // Set to 1 (device int, may be null) by a kernel that meets a gate product below the floor of
    // its reciprocals: its results are then not exact.  Never cleared by the library.
    int* domain_flag = nullptr;
    TokenLayout lay;
    // [B][H][N][d]: the kernels then use compile-time token strides
    // variable-length batch: N and NC then describe the packed token axis (lay.vl is set once the
    // workspace that holds the sequence table is known)
    bool packed = false;
    // the tensors are a window of larger ones (the tokens after a sequence's first run): strides
    // come from `lay` even when a token's row is as wide as the head
    bool window = false;
    bool dense() const { return lay.sn_k == dk && lay.sn_v == dv && !packed && !window; }
    // chunk slots of the per-chunk workspaces and of the per-chunk grids
    size_t total_chunks() const { return packed ? (size_t)H * NC : (size_t)BH * NC; }
};

// A kernel that uses more dynamic LDS than the default limit must have the limit raised once per
// device; the setting is remembered here so that a launch does not repeat the runtime call.
inline hipError_t allow_dynamic_lds(const void* kernel, int bytes)
{
    struct Slot { const void* kernel; unsigned long long devices; };
    static Slot slots[256];                 // racing first launches at worst repeat the runtime call
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const unsigned long long bit = 1ull << (dev & 63);
    size_t i = (reinterpret_cast<size_t>(kernel) >> 4) & 255;
    for (int probe = 0; probe < 256; ++probe, i = (i + 1) & 255) {
        if (slots[i].kernel == kernel) {
            if (slots[i].devices & bit) return hipSuccess;
            break;
        }
        if (slots[i].kernel == nullptr) break;
    }
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e != hipSuccess) return e;
    if (slots[i].kernel == nullptr || slots[i].kernel == kernel) {
        slots[i].kernel = kernel;
        slots[i].devices |= bit;
    }
    return hipSuccess;
}

// What a state sweep accumulates.
enum SweepMode {
    kSweepStateFwd = 0,   // S_n for the forward read-out   (fragments contract over dk)
    kSweepStateBwd = 1,   // S_n for the backward pass      (fragments contract over dv)
    kSweepGrad = 2        // dS_{n+1}, reverse order        (fragments contract over dv)
};

// Chunk-to-chunk recurrence.  Writes, for every chunk n, the state entering it (modes 0/1) or
// the state gradient leaving it (mode 2) into `ws` as MFMA fragments, and the final state
// (`final_state`, may be null) in plain fp32 [dk][dv].  `a_src` is f (modes 0/1) or q (mode 2);
// `b_src` is v (modes 0/1) or grad_o (mode 2).
hipError_t launch_sweep(const SeqDims& d, SweepMode mode, const void* q, const void* f, const void* b_src,
                        const float* init_state, float* final_state, void* ws, float* decay, hipStream_t stream);

// Both sweeps of the backward pass (kSweepStateBwd into ws_state, kSweepGrad into ws_dstate) in
// one launch.
hipError_t launch_sweep_pair(const SeqDims& d, const void* q, const void* f, const void* v, const void* grad_o,
                             const float* h0, const float* grad_hT, float* grad_h0, void* ws_state,
                             void* ws_dstate, hipStream_t stream);

// Segmented sweeps.  A sweep given a `decay` array walks every sequence from a zero state, writes
// nothing per chunk (`ws` is ignored) and leaves the state after its last chunk in `final_state` and the per-channel product of all its
// gates in `decay` ([BH][dk]); launch_sweep_pair_ends does so for both backward sweeps (one copy of
// the gate products).  Called on the runs of segmented sequences (TokenLayout::seg), these give
// launch_run_carry what it needs to turn run_state ([n_seq * seg][dk][dv], overwritten) into the
// state entering each run, from which the ordinary sweeps then start run by run.
hipError_t launch_sweep_pair_ends(const SeqDims& d, const void* q, const void* f, const void* v, const void* grad_o,
                                  float* run_state, float* run_dstate, float* run_decay, hipStream_t stream);
// (choice, path: as TokenLayout's; the kernel returns at once when *choice != path)
hipError_t launch_run_carry(int n_seq, int seg, int dk, int dv, const float* carried_in, float* run_state,
                            const float* run_decay, float* carried_out, bool reverse, hipStream_t stream,
                            const int* choice = nullptr, int path = 0);
// The same for a packed batch cut by launch_varlen_run_table: sequence b of head h owns the runs
// first_run[b] .. first_run[b + 1] - 1, whose states sit at [run * H + h].
hipError_t launch_run_carry_packed(int B, int H, const int* first_run, int dk, int dv, const float* carried_in,
                                   float* run_state, const float* run_decay, float* carried_out, bool reverse,
                                   hipStream_t stream, const int* choice = nullptr, int path = 0);

// Per-chunk forward read-out  O = tril(Q~ K~^T) V + (Q G) S_n.
hipError_t launch_fwd_out(const SeqDims& d, const void* q, const void* f, const void* v, const void* ws_state,
                          void* o, hipStream_t stream);

// Fused forward (state recurrence + read-out in one pass, states never leave the chip); only for
// the shapes fwd_fused_supported() accepts.
bool fwd_fused_supported(const SeqDims& d);
// `save_states` (may be null): receives G_m S_n of every chunk in the fragment order of a
// kSweepStateBwd sweep, state_ws_bytes() in all, for a backward pass that then needs no such sweep.
hipError_t launch_fwd_fused(const SeqDims& d, const void* q, const void* f, const void* v, const float* h0,
                            void* o, float* hT, void* save_states, hipStream_t stream);

// Per-chunk gradients dq, df, dv from the two state sweeps.
// With d.beta set, grad_f receives the gradient w.r.t. the pre-activation z, and every wave of
// every chunk (launch_bwd_fused: of every run) leaves its partial sum of the gradient w.r.t. beta in `beta_partials`
// ([B*H*NC][8][dk] fp32, followed by room for the sums of the reduction's first pass:
// beta_partials_bytes() in all), which reduce_beta_partials() adds up in a fixed order.
hipError_t launch_bwd_grad(const SeqDims& d, const void* q, const void* f, const void* v, const void* grad_o,
                           const void* ws_state, const void* ws_dstate, void* grad_q, void* grad_f,
                           void* grad_v, float* beta_partials, hipStream_t stream);
// The same gradients from the forward states alone: one workgroup per run of a sequence walks the
// run's chunks from the last to the first with the state gradient in registers (bwd_grad.hip).
// plan_bwd_fused() cuts the sequences into R runs of rc chunks; for R > 1 the caller provides the
// state gradient at the run boundaries: a zero-start gradient sweep over the tokens after run 0, cut
// into seg_tail sub-runs of sub_chunks chunks, and its reverse carry from grad_hT leave it in
// run_state ([BH][seg_tail][dk][dv], entry t = at the end of sub-run t) and bound0 ([BH][dk][dv], at
// the end of run 0).  grad_h0 may be null.  Equal-length batches only.
// With few runs (light != 0) nothing of that is needed: every workgroup first walks the chunks after
// its own run from grad_hT, carrying only the state gradient, and the runs are cut at bnd[0..R].
struct BwdFusedPlan { int R, rc, s_sub, sub_chunks, seg_tail, light, bnd[5]; };
BwdFusedPlan plan_bwd_fused(const SeqDims& d);
hipError_t launch_bwd_fused(const SeqDims& d, const BwdFusedPlan& pl, const void* q, const void* f, const void* v,
                            const void* grad_o, const void* ws_state, const float* grad_hT, float* grad_h0,
                            const float* bound0, const float* run_state, void* grad_q, void* grad_f, void* grad_v,
                            float* beta_partials, hipStream_t stream);
// The fused reverse walk for a packed batch with a group table (TokenLayout::groups): one workgroup
// per (group, head) walks the group's sequences from the last to the first, each from its own
// grad_hT[b] (may be null: zero) to its own grad_h0[b] (may be null).  ws_state: the forward states
// of a kSweepStateBwd sweep over the same table.
hipError_t launch_bwd_fused_grouped(const SeqDims& d, const void* q, const void* f, const void* v, const void* grad_o,
                                    const void* ws_state, const float* grad_hT, float* grad_h0, void* grad_q,
                                    void* grad_f, void* grad_v, float* beta_partials, hipStream_t stream);
size_t beta_partials_bytes(const SeqDims& d);
// runs > 0: the partial sums come from launch_bwd_fused with a plan of that many runs, which leaves one
// row per wave and RUN (in the first `runs` chunk slots of every sequence) instead of one per chunk.
hipError_t reduce_beta_partials(const SeqDims& d, float* beta_partials, float* grad_beta, hipStream_t stream, int runs = 0);

// Lower bounds of all layers from Gamma [L][d] (paper Section 2): cumulative softmax over the
// layer axis minus its first row.
hipError_t launch_cumax(int L, int d, const float* gamma, float* beta, hipStream_t stream);

// Decode step.  With `beta` ([H][dk] fp32) set, the gate tensor holds the pre-activation of Eq. 2.
hipError_t launch_step(int BH, int dk, int dv, bool io_bf16, bool gate_bf16, const void* q, const void* f,
                       const void* v, float* state, void* o, const float* beta, int H, hipStream_t stream);

// HGRN1, the element-wise recurrence h_t = f_t h_{t-1} + (1 - f_t) i_t, y_t = h_t o_t (paper Eq. 1),
// on [B][N][d] bf16 tensors (d a multiple of 64), states [B][d] fp32; `ws` holds hgrn1_ws_bytes().
// With `beta` ([d] fp32) set, f, i, o are the pre-activations of Eq. 1 and the gate gets the lower
// bound of Eq. 2; the backward then returns the gradients of the pre-activations and of beta.
size_t hgrn1_ws_bytes(int B, int N, int d);
hipError_t launch_hgrn1_fwd(int B, int N, int d, bool gate_bf16, const void* f, const void* i, const void* o,
                            const float* beta, const float* h0, void* y, float* hN, void* ws, hipStream_t stream);
// states_saved: `ws` still holds what launch_hgrn1_fwd on the same inputs left there (the state entering
// every 16-token segment); the backward pass then does not walk f and i forwards first.
hipError_t launch_hgrn1_bwd(int B, int N, int d, bool gate_bf16, const void* f, const void* i, const void* o,
                            const float* beta, const float* h0, const void* dy, const float* dhN, void* df, void* di,
                            void* dout, float* dbeta, float* dh0, void* ws, bool states_saved, hipStream_t stream);

// Smallest product of the gates of one channel over `window` consecutive tokens (windows aligned at
// multiples of `window` in every sequence), over the whole call: what the exactness of the chunkwise
// kernels depends on, with window = half a chunk (32; 8 in the small-gate mode).  `out`: one float
// on the device.
hipError_t launch_min_gate_product(const SeqDims& d, int window, const void* f, float* out, hipStream_t stream);

// Bytes of one per-chunk state set in the workspace.
size_t state_ws_bytes(const SeqDims& d);

// Variable-length batches: builds the table TokenLayout::vl points to from cu_seqlens (device,
// B + 1 ints, cu_seqlens[b] = first token of sequence b, cu_seqlens[B] = T).  Offsets are clamped
// to [0, T] and made non-decreasing, so that whatever the array holds, the sequences the kernels
// see are disjoint pieces of the T tokens.
size_t varlen_table_bytes(int B);
// Run table of a packed batch (see varlen.hip): R entries and, behind them, first_run[B + 1].
size_t varlen_run_table_bytes(int B, int R);
// (sub: tokens per chunk, TokenLayout::sub)
// (choice, path: the kernel returns at once when *choice != path)
hipError_t launch_varlen_run_table(const int* seq_table, int B, int T, int run_chunks, int R, int* run_table,
                                   int* first_run, hipStream_t stream, int sub = kChunk, const int* choice = nullptr, int path = 0);
// Groups of a table's sequences (sequence or run table with n_entries entries): G + 1 ints, group g
// = entries [groups[g], groups[g + 1]), cut where the chunk count reaches g / G of the total, so that
// groups hold about equally many chunks (a group is never finer than one entry); and one more int,
// the choice of backward pass (TokenLayout::path): the reverse walk over groups takes as long as its
// largest group, the per-chunk pass as long as all chunks shared among the compute units.
size_t varlen_groups_bytes(int G);
hipError_t launch_varlen_groups(const int* table, int n_entries, int G, int* groups, hipStream_t stream,
                                const int* choice = nullptr, int path = 0);
// dst[0 .. n) = 0, as a kernel (safe under graph capture)
hipError_t launch_zero_floats(float* dst, size_t n, hipStream_t stream);
// *out = src[0] + ... + src[n - 1], on the device
hipError_t launch_sum_ints(const int* src, int n, int* out, hipStream_t stream);
// (groups != null: the group array over the table's G groups, launch_varlen_groups(), in the same launch)
hipError_t launch_varlen_table(const int* cu_seqlens, int B, int T, int* table, hipStream_t stream, int G = 0,
                               int* groups = nullptr, int sub = kChunk, const int* choice = nullptr, int path = 0);

}   // namespace hgrn2
