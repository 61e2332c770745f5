// C-ABI layer of the HGRN2 library: argument validation on the host, workspace carving and the
// sequence of kernel launches.  See include/hgrn2.h for the contract of every entry point.
#include "../../include/hgrn2.h"
#include "kernels.hpp"

#include <limits.h>

using namespace hgrn2;

namespace {

bool dtype_ok(int32_t t) { return t == HGRN2_F32 || t == HGRN2_BF16; }
bool dim_ok(int32_t d) { return d == 64 || d == 128; }

// Validates a shape; on success fills `d`.  `fine_ok`: the entry point also takes chunk = 16 or 32,
// the small-gate modes: the batch is then walked in chunks that hold only that many tokens
// (TokenLayout::sub).
int check_shape(const hgrn2_shape* s, bool backward, SeqDims* d, bool packed = false, bool fine_ok = false)
{
    if (!s) return HGRN2_ERR_NULL;
    if (s->B < 0 || s->H < 0 || s->N < 0 || s->dk <= 0 || s->dv <= 0 || s->chunk < 0) return HGRN2_ERR_SHAPE;
    if (!dtype_ok(s->io_dtype) || !dtype_ok(s->gate_dtype)) return HGRN2_ERR_SHAPE;
    if (s->layout != HGRN2_LAYOUT_BHND && s->layout != HGRN2_LAYOUT_BNHD) return HGRN2_ERR_SHAPE;
    const long long bh = (long long)s->B * s->H;
    if (bh > INT_MAX / 16) return HGRN2_ERR_SHAPE;
    const bool fine = s->chunk == kFineChunk || s->chunk == 2 * kFineChunk || s->chunk == kFineChunk / 2;
    const int sub = fine ? s->chunk : kChunk;                               // tokens per chunk
    const long long nc = ((long long)s->N + sub - 1) / sub;
    if (!packed && bh * nc > INT_MAX / 2) return HGRN2_ERR_SHAPE;          // one workgroup per chunk (packed sequences: checked by the caller)
    if (!dim_ok(s->dk) || !dim_ok(s->dv)) return HGRN2_ERR_UNSUPPORTED;
    if (fine ? !fine_ok : (s->chunk != 0 && s->chunk != kChunk)) return HGRN2_ERR_UNSUPPORTED;
    if (s->N > INT_MAX / 8) return HGRN2_ERR_SHAPE;                         // row numbers around the sequence stay ints
    // fp32 storage in the backward pass: heads of 64 x 64 only (the fp32 tiles of wider heads exceed
    // the LDS), equal-length batches only
    if (backward && s->io_dtype != HGRN2_BF16 && (packed || s->dk != 64 || s->dv != 64)) return HGRN2_ERR_UNSUPPORTED;
    d->BH = (int)bh;
    d->N = s->N;
    d->NC = (int)nc;
    d->dk = s->dk;
    d->dv = s->dv;
    d->io_bf16 = s->io_dtype == HGRN2_BF16;
    d->gate_bf16 = s->gate_dtype == HGRN2_BF16;
    d->H = s->H > 0 ? s->H : 1;
    d->beta = nullptr;
    d->domain_flag = s->gate_domain_flag;
    const long long H = s->H, N = s->N, dk = s->dk, dv = s->dv;
    d->lay.H = d->H;
    d->lay.sub = sub;
    if (s->layout == HGRN2_LAYOUT_BNHD) {
        if (H * dk > INT_MAX / 8 || H * dv > INT_MAX / 8) return HGRN2_ERR_SHAPE;      // token stride is kept in an int
        d->lay.sb_k = N * H * dk; d->lay.sh_k = dk; d->lay.sn_k = H * dk;
        d->lay.sb_v = N * H * dv; d->lay.sh_v = dv; d->lay.sn_v = H * dv;
    } else {
        d->lay.sb_k = H * N * dk; d->lay.sh_k = N * dk; d->lay.sn_k = dk;
        d->lay.sb_v = H * N * dv; d->lay.sh_v = N * dv; d->lay.sn_v = dv;
    }
    return HGRN2_OK;
}

// Variable-length batches: shape->B sequences packed into shape->N tokens of [T][H][d] tensors.
// Fills `d` with NC = the host's bound on the chunks of all sequences (N / chunk + B); the table
// pointer is set by the caller once the workspace is known.
int check_shape_varlen(const hgrn2_shape* s, bool backward, SeqDims* d, bool fine_ok = false)
{
    const int rc = check_shape(s, backward, d, true, fine_ok);
    if (rc != HGRN2_OK) return rc;
    if (s->layout != HGRN2_LAYOUT_BNHD) return HGRN2_ERR_SHAPE;          // packed tokens are token-major
    const long long bound = (long long)s->N / d->lay.sub + s->B;
    if (bound * (s->H > 0 ? s->H : 1) > INT_MAX / 2 || s->B > INT_MAX / 8) return HGRN2_ERR_SHAPE;
    d->NC = (int)bound;
    d->packed = true;
    d->lay.sb_k = d->lay.sb_v = 0;
    d->lay.B = s->B;
    return HGRN2_OK;
}

size_t round256(size_t x) { return (x + 255) & ~(size_t)255; }

// Long sequences in a small batch leave most of the chip idle in the kernels that walk a sequence
// chunk by chunk.  Those then see every sequence cut into runs of whole chunks: a first walk per
// run from a zero state yields what the run adds and how it decays what enters it, a carry over
// the runs turns that into the state entering each run, and the usual walk starts run by run.
// Returns the number of runs (1: not cut) and the chunks of a full run.
int plan_runs(const SeqDims& d, bool backward, int* run_chunks)
{
    *run_chunks = d.NC;
    // Measured with 64- and 128-wide heads: the forward gains from 16 chunks on, up to 64 sequences
    // and with about 256 runs in all, down to runs of 4 chunks; the backward pass of a packed batch
    // (the only one planned here: equal lengths have a plan of their own) cuts the same way, but
    // only from 32 chunks on and up to 32 sequences.
    if (d.packed || d.NC < (backward ? 32 : 16) || d.BH == 0 || d.BH > (backward ? 32 : 64)) return 1;
    const int fill = 256 / d.BH;                         // rounded down: a walk more than there are units has to wait for a free one
    const int by_length = d.NC / 4;
    const int seg = fill < by_length ? fill : by_length;
    if (seg < 2) return 1;
    const int rc = (d.NC + seg - 1) / seg;
    *run_chunks = rc;
    return (d.NC + rc - 1) / rc;                         // every run holds at least one chunk
}

SeqDims as_runs(const SeqDims& d, int seg, int run_chunks)
{
    if (seg <= 1) return d;               // one run: the sequence itself, with its own length
    SeqDims r = d;
    r.BH = d.BH * seg; r.NC = run_chunks; r.N = run_chunks * d.lay.sub;
    r.lay.seg = seg; r.lay.n_tokens = d.N;
    return r;
}

// per sweep: what every run adds to the state, fp32 [BH * seg][dk][dv]
size_t run_state_bytes(const SeqDims& d, bool backward)
{
    int rc;
    const int seg = plan_runs(d, backward, &rc);
    return seg > 1 ? round256((size_t)d.BH * seg * d.dk * d.dv * sizeof(float)) : 0;
}

// the gate products of the runs, fp32 [BH * seg][dk]
size_t run_decay_bytes(const SeqDims& d, bool backward)
{
    int rc;
    const int seg = plan_runs(d, backward, &rc);
    return seg > 1 ? round256((size_t)d.BH * seg * d.dk * sizeof(float)) : 0;
}

// Workspace of the backward pass of an equal-length batch: the forward states of every chunk (with
// the run states of their sweep when few long sequences are walked in runs), what the reverse walk
// needs at its run boundaries, and the partial sums of the gradient of beta.
struct BwdLayout {
    BwdFusedPlan plan;
    size_t states = 0;                    // at offset 0
    size_t fwd_run_state = 0, fwd_run_decay = 0;
    size_t tail_state = 0, tail_decay = 0, bound0 = 0;
    size_t partials = 0;
    size_t total() const { return states + fwd_run_state + fwd_run_decay + tail_state + tail_decay + bound0 + partials; }
};

BwdLayout bwd_layout(const SeqDims& d, bool gated, bool states_given = false)
{
    BwdLayout l;
    l.plan = plan_bwd_fused(d);
    if (!states_given) {
        l.states = round256(state_ws_bytes(d));
        l.fwd_run_state = run_state_bytes(d, false);
        l.fwd_run_decay = run_decay_bytes(d, false);
    }
    if (l.plan.R > 1 && !l.plan.light) {
        const size_t slots = (size_t)d.BH * l.plan.seg_tail;
        l.tail_state = round256(slots * d.dk * d.dv * sizeof(float));
        l.tail_decay = round256(slots * d.dk * sizeof(float));
        l.bound0 = round256((size_t)d.BH * d.dk * d.dv * sizeof(float));
    }
    l.partials = gated ? round256(beta_partials_bytes(d)) : 0;
    return l;
}

// A packed batch is cut the way an equal-length batch of its mean sequence length would be (the
// host does not know the lengths): runs of `run_chunks` chunks (0: not cut), at most `R` of them.
struct PackedRuns {
    int run_chunks = 0, R = 0;
    int G = 0;                   // groups of table entries per head (walked back to back by one workgroup); also the spans of the reverse walk
    bool by_groups = false;      // enough sequences for the forward walks and sweeps to take a group each
    size_t groups_at = 0;        // where the group array starts
    size_t table_bytes = 0;      // sequence table, then run table and first_run, then the groups
    size_t state_bytes = 0;      // per sweep: fp32 [R * H][dk][dv]
    size_t decay_bytes = 0;      // fp32 [R * H][dk]
};

PackedRuns plan_packed_runs(const hgrn2_shape* s, const SeqDims& d, bool backward)
{
    PackedRuns p;
    p.R = s->B;
    p.table_bytes = round256(varlen_table_bytes(s->B));
    if (s->B == 0) return p;
    // A batch that is not cut into runs gets a group array of about one group per compute unit:
    // the reverse walk takes equal spans of a head's chunks (the array's last int holds the table
    // kernel's choice between the two backward passes), and with at least as many entries per head
    // as groups the forward walks and sweeps take a group of entries each (fewer, longer ones keep a
    // workgroup each).
    auto with_groups = [&](PackedRuns& r) {
        const int per_head = 256 / (s->H > 0 ? s->H : 1) > 0 ? 256 / (s->H > 0 ? s->H : 1) : 1;
        r.by_groups = r.R >= per_head;
        r.G = per_head;
        r.groups_at = r.table_bytes;
        r.table_bytes += round256(varlen_groups_bytes(r.G));
    };
    SeqDims mean = d;
    mean.packed = false;
    mean.NC = (int)(((long long)d.N / d.lay.sub + s->B - 1) / s->B);
    int rc;
    const long long bound = plan_runs(mean, backward, &rc) <= 1 ? 0
                          : s->B + ((long long)d.N / d.lay.sub + s->B) / rc + 1;    // >= sum_b ceil(NC_b / rc)
    if (bound == 0 || bound * (s->H > 0 ? s->H : 1) > INT_MAX / 2) {
        with_groups(p);
        return p;
    }
    p.run_chunks = rc;
    p.R = (int)bound;
    p.table_bytes += round256(varlen_run_table_bytes(s->B, p.R));
    if (backward) {          // the reverse walk takes spans of the runs' chunks
        p.G = 256 / (s->H > 0 ? s->H : 1) > 0 ? 256 / (s->H > 0 ? s->H : 1) : 1;
        p.groups_at = p.table_bytes;
        p.table_bytes += round256(varlen_groups_bytes(p.G));
    }
    p.state_bytes = round256((size_t)p.R * s->H * d.dk * d.dv * sizeof(float));
    p.decay_bytes = round256((size_t)p.R * s->H * d.dk * sizeof(float));
    return p;             // (runs are many and equally long: a workgroup each)
}

// Builds the table(s) at `workspace` (p.table_bytes bytes) and points `d` at the one the kernels
// use; returns first_run (null when the batch is not cut).  launch = false: the tables are there
// already (the forward pass of a training pair has left them), only `d` is set up.
hipError_t build_packed_tables(const hgrn2_shape* s, const PackedRuns& p, const int32_t* cu_seqlens, void* workspace,
                               SeqDims* d, const int** first_run, hipStream_t stream, bool launch = true)
{
    int* seq_table = static_cast<int*>(workspace);
    *first_run = nullptr;
    d->lay.vl = seq_table;
    // (a batch that is not cut gets its group array, over the sequence table, in the same launch)
    int* groups_here = (p.G > 0 && p.run_chunks == 0) ? reinterpret_cast<int*>(static_cast<char*>(workspace) + p.groups_at) : nullptr;
    hipError_t e = launch ? launch_varlen_table(cu_seqlens, s->B, d->N, seq_table, stream, p.G, groups_here, d->lay.sub,
                                                d->lay.alt, d->lay.alt_path) : hipSuccess;
    if (e != hipSuccess) return e;
    if (p.run_chunks != 0) {
        int* run_table = reinterpret_cast<int*>(static_cast<char*>(workspace) + round256(varlen_table_bytes(s->B)));
        int* fr = run_table + 4 * ((size_t)p.R + 1);
        e = launch ? launch_varlen_run_table(seq_table, s->B, d->N, p.run_chunks, p.R, run_table, fr, stream, d->lay.sub,
                                             d->lay.alt, d->lay.alt_path) : hipSuccess;
        if (e != hipSuccess) return e;
        d->lay.vl = run_table;
        d->lay.B = p.R;
        d->BH = p.R * s->H;
        *first_run = fr;
    }
    if (p.G > 0) {
        int* groups = reinterpret_cast<int*>(static_cast<char*>(workspace) + p.groups_at);
        if (launch && !groups_here) e = launch_varlen_groups(d->lay.vl, d->lay.B, p.G, groups, stream, d->lay.alt, d->lay.alt_path);
        if (p.by_groups) {
            d->lay.groups = groups;
            d->lay.G = p.G;
        }
        d->lay.spans = p.G;
        d->lay.span_seq = groups + p.G + 2;
    }
    return e;
}

// ---- small-gate modes -----------------------------------------------------------------------------
bool fine_mode(const hgrn2_shape* s) { return s && (s->chunk == kFineChunk || s->chunk == 2 * kFineChunk || s->chunk == kFineChunk / 2); }

// chunk = HGRN2_CHUNK_AUTO (equal-length batches): the pass is enqueued for 64, then 32, then 16
// tokens per chunk.  The kernels of the first raise a flag when a gate product falls below the floor
// of their reciprocals; those of the second run only if it is set (the others return at once) and
// raise a second flag, on which the third depends: the results are those of the longest chunk the
// gates allow, at the cost of two launches that do nothing when the gates are ordinary.
bool auto_mode(const hgrn2_shape* s) { return s && s->chunk == HGRN2_CHUNK_AUTO; }
constexpr size_t kAutoHead = 256;         // the flags, at the head of the workspace (ints: flag of 64, flag of 32)
constexpr int kAlternatives = 3;

// the shapes the pass is run on: the caller's, or its three alternatives
int alternatives(const hgrn2_shape* shape, hgrn2_shape (&alt)[kAlternatives])
{
    alt[0] = *shape;
    if (!auto_mode(shape)) return 1;
    static const int32_t chunks[kAlternatives] = {0, 2 * kFineChunk, kFineChunk};
    for (int i = 0; i < kAlternatives; ++i) { alt[i] = *shape; alt[i].chunk = chunks[i]; }
    return kAlternatives;
}

// largest value of a size over the alternatives (plus, with `head`, the flags' place when there are several)
// (`sum`: the total instead -- every alternative keeps a place of its own)
template <typename F> size_t max_over_alternatives(const hgrn2_shape* shape, F bytes_of, bool head, bool backward,
                                                   bool packed = false, bool sum = false)
{
    if (!shape) return 0;
    hgrn2_shape alt[kAlternatives];
    const int n = alternatives(shape, alt);
    SeqDims d;
    if (check_shape(&alt[0], backward, &d, packed, true) != HGRN2_OK) return 0;      // an invalid shape needs nothing
    size_t m = 0;
    for (int i = 0; i < n; ++i) { const size_t b = bytes_of(&alt[i]); m = sum ? m + b : (b > m ? b : m); }
    return m + ((n > 1 && head) ? kAutoHead : 0);
}

// How one alternative is enqueued: which device int its kernels compare with `path` before doing
// anything (null: they always run), and which device int they raise when a gate product falls below
// the floor (instead of the shape's own).
struct Alternative {
    const int* choice = nullptr;
    int path = 0;
    const int* choice2 = nullptr;         // a second condition of the same kind (equal-length batches)
    int path2 = 0;
    int* flag = nullptr;
    bool validate_only = false;           // stop after the argument checks
};

}   // namespace

extern "C" {

size_t hgrn2_fwd_workspace_bytes(const hgrn2_shape* shape)
{
    return max_over_alternatives(shape, [](const hgrn2_shape* s) -> size_t {
        SeqDims d;
        if (check_shape(s, false, &d, false, true) != HGRN2_OK) return 0;
        return round256(state_ws_bytes(d)) + run_state_bytes(d, false) + run_decay_bytes(d, false);
    }, true, false);
}

size_t hgrn2_bwd_workspace_bytes(const hgrn2_shape* shape)
{
    return max_over_alternatives(shape, [](const hgrn2_shape* s) -> size_t {
        SeqDims d;
        if (check_shape(s, true, &d, false, true) != HGRN2_OK) return 0;
        return bwd_layout(d, false).total();
    }, true, true);
}

static int fwd_impl(const hgrn2_shape* shape, const void* q, const void* f, const float* beta, bool gated,
                    const void* v, const float* h0, void* o, float* hT, void* workspace, size_t workspace_bytes,
                    void* hip_stream, void* save_states = nullptr);
static int fwd_one(const hgrn2_shape* shape, const void* q, const void* f, const float* beta, bool gated,
                   const void* v, const float* h0, void* o, float* hT, void* workspace, size_t workspace_bytes,
                   void* hip_stream, void* save_states, const Alternative* alt);
static int bwd_one(const hgrn2_shape* shape, const void* q, const void* f, const float* beta, bool gated,
                   const void* v, const float* h0, const void* grad_o, const float* grad_hT, void* grad_q,
                   void* grad_f, float* grad_beta, void* grad_v, float* grad_h0, void* workspace,
                   size_t workspace_bytes, void* hip_stream, const void* saved_states, const Alternative* alt);
static int bwd_impl(const hgrn2_shape* shape, const void* q, const void* f, const float* beta, bool gated,
                    const void* v, const float* h0, const void* grad_o, const float* grad_hT, void* grad_q,
                    void* grad_f, float* grad_beta, void* grad_v, float* grad_h0, void* workspace,
                    size_t workspace_bytes, void* hip_stream, const void* saved_states = nullptr);

// Forward pass; `beta` null: `f` holds the gates; else `f` holds their pre-activations (Eq. 2).
// With chunk = HGRN2_CHUNK_AUTO: its three alternatives.  `save_states` then ends in kAutoHead bytes
// that hold the two flags, for the backward pass of the pair.
static int fwd_impl(const hgrn2_shape* shape, const void* q, const void* f, const float* beta, bool gated,
                    const void* v, const float* h0, void* o, float* hT, void* workspace, size_t workspace_bytes,
                    void* hip_stream, void* save_states)
{
    if (!auto_mode(shape)) return fwd_one(shape, q, f, beta, gated, v, h0, o, hT, workspace, workspace_bytes, hip_stream, save_states, nullptr);
    hgrn2_shape alt[kAlternatives];
    alternatives(shape, alt);
    const size_t need = hgrn2_fwd_workspace_bytes(shape);
    if (need == 0) {                      // an invalid shape: the first alternative names the error
        SeqDims d;
        const int rc = check_shape(&alt[0], false, &d, false, true);
        return rc != HGRN2_OK ? rc : HGRN2_ERR_SHAPE;
    }
    if (!workspace || workspace_bytes < need || ((uintptr_t)workspace & 255)) return HGRN2_ERR_WORKSPACE;
    char* rest = static_cast<char*>(workspace) + kAutoHead;
    Alternative a;
    a.validate_only = true;
    for (int i = 0; i < kAlternatives; ++i) {
        const int rc = fwd_one(&alt[i], q, f, beta, gated, v, h0, o, hT, rest, workspace_bytes - kAutoHead, hip_stream, save_states, &a);
        if (rc != HGRN2_OK) return rc;
    }
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    // (a training pair keeps the two flags behind the states: the backward pass reads them there)
    int* flags = save_states ? reinterpret_cast<int*>(static_cast<char*>(save_states) + hgrn2_saved_states_bytes(shape) - kAutoHead)
                             : static_cast<int*>(workspace);
    if (launch_zero_floats(reinterpret_cast<float*>(flags), 4, stream) != hipSuccess) return HGRN2_ERR_HIP;
    a.validate_only = false;
    for (int i = 0; i < kAlternatives; ++i) {
        a.choice = i == 0 ? nullptr : flags + (i - 1);
        a.path = 1;
        a.flag = i + 1 < kAlternatives ? flags + i : shape->gate_domain_flag;
        const int rc = fwd_one(&alt[i], q, f, beta, gated, v, h0, o, hT, rest, workspace_bytes - kAutoHead, hip_stream, save_states, &a);
        if (rc != HGRN2_OK) return rc;
    }
    return HGRN2_OK;
}

static int fwd_one(const hgrn2_shape* shape, const void* q, const void* f, const float* beta, bool gated,
                   const void* v, const float* h0, void* o, float* hT, void* workspace, size_t workspace_bytes,
                   void* hip_stream, void* save_states, const Alternative* alt)
{
    SeqDims d;
    const int rc = check_shape(shape, false, &d, false, true);
    if (rc != HGRN2_OK) return rc;
    const bool has_tokens = (size_t)d.BH * d.N > 0;
    if (has_tokens && (!q || !f || !v || !o)) return HGRN2_ERR_NULL;
    if (gated && has_tokens && !beta) return HGRN2_ERR_NULL;
    d.beta = gated ? beta : nullptr;
    if (alt) { d.lay.choice = alt->choice; d.lay.path = alt->path; d.lay.alt = alt->choice2; d.lay.alt_path = alt->path2; d.domain_flag = alt->flag; }
    const size_t one = round256(state_ws_bytes(d));
    const size_t need = one + run_state_bytes(d, false) + run_decay_bytes(d, false);
    if (need > 0 && (!workspace || workspace_bytes < need || ((uintptr_t)workspace & 255))) return HGRN2_ERR_WORKSPACE;
    if (alt && alt->validate_only) return HGRN2_OK;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if (d.BH == 0) return HGRN2_OK;
    if (!has_tokens && !hT) return HGRN2_OK;
    // States for a later backward pass: the single-pass kernel hands them over as it goes; the
    // other paths (whose sweep keeps the states in the read-out's orientation) run a sweep for them.
    auto save_by_sweep = [&]() {
        return !save_states || !has_tokens ||
               launch_sweep(d, kSweepStateBwd, nullptr, f, v, h0, nullptr, save_states, nullptr, stream) == hipSuccess;
    };
    int run_chunks;
    const int seg = plan_runs(d, false, &run_chunks);
    if (seg > 1) {
        const SeqDims r = as_runs(d, seg, run_chunks);
        float* run_state = reinterpret_cast<float*>(static_cast<char*>(workspace) + one);
        float* run_decay = reinterpret_cast<float*>(reinterpret_cast<char*>(run_state) + run_state_bytes(d, false));
        if (launch_sweep(r, kSweepStateFwd, q, f, v, nullptr, run_state, nullptr, run_decay, stream) != hipSuccess ||
            launch_run_carry(d.BH, seg, d.dk, d.dv, h0, run_state, run_decay, hT, false, stream, d.lay.choice, d.lay.path) != hipSuccess)
            return HGRN2_ERR_HIP;
        if (fwd_fused_supported(r))
            return launch_fwd_fused(r, q, f, v, run_state, o, nullptr, save_states, stream) == hipSuccess ? HGRN2_OK : HGRN2_ERR_HIP;
        if (launch_sweep(r, kSweepStateFwd, q, f, v, run_state, nullptr, workspace, nullptr, stream) != hipSuccess ||
            launch_fwd_out(d, q, f, v, workspace, o, stream) != hipSuccess || !save_by_sweep())
            return HGRN2_ERR_HIP;
        return HGRN2_OK;
    }
    if (fwd_fused_supported(d))
        return launch_fwd_fused(d, q, f, v, h0, o, hT, save_states, stream) == hipSuccess ? HGRN2_OK : HGRN2_ERR_HIP;
    if (launch_sweep(d, kSweepStateFwd, q, f, v, h0, hT, workspace, nullptr, stream) != hipSuccess) return HGRN2_ERR_HIP;
    if (launch_fwd_out(d, q, f, v, workspace, o, stream) != hipSuccess || !save_by_sweep()) return HGRN2_ERR_HIP;
    return HGRN2_OK;
}

int hgrn2_fwd(const hgrn2_shape* shape, const void* q, const void* f, const void* v, const float* h0,
              void* o, float* hT, void* workspace, size_t workspace_bytes, void* hip_stream)
{
    return fwd_impl(shape, q, f, nullptr, false, v, h0, o, hT, workspace, workspace_bytes, hip_stream);
}

int hgrn2_fwd_gated(const hgrn2_shape* shape, const void* q, const void* z, const float* beta, const void* v,
                    const float* h0, void* o, float* hT, void* workspace, size_t workspace_bytes,
                    void* hip_stream)
{
    return fwd_impl(shape, q, z, beta, true, v, h0, o, hT, workspace, workspace_bytes, hip_stream);
}

size_t hgrn2_bwd_gated_workspace_bytes(const hgrn2_shape* shape)
{
    return max_over_alternatives(shape, [](const hgrn2_shape* s) -> size_t {
        SeqDims d;
        if (check_shape(s, true, &d, false, true) != HGRN2_OK) return 0;
        return bwd_layout(d, true).total();
    }, true, true);
}

// Backward pass; `gated`: `f` holds pre-activations, grad_f receives dL/dz and grad_beta dL/dbeta.
// With chunk = HGRN2_CHUNK_AUTO: its three alternatives, chosen as in the forward pass, or (with the
// states a forward pass kept) by the int that pass left behind them.
static int bwd_impl(const hgrn2_shape* shape, const void* q, const void* f, const float* beta, bool gated,
                    const void* v, const float* h0, const void* grad_o, const float* grad_hT, void* grad_q,
                    void* grad_f, float* grad_beta, void* grad_v, float* grad_h0, void* workspace,
                    size_t workspace_bytes, void* hip_stream, const void* saved_states)
{
    if (!auto_mode(shape))
        return bwd_one(shape, q, f, beta, gated, v, h0, grad_o, grad_hT, grad_q, grad_f, grad_beta, grad_v, grad_h0, workspace,
                       workspace_bytes, hip_stream, saved_states, nullptr);
    hgrn2_shape alt[kAlternatives];
    alternatives(shape, alt);
    const size_t head = saved_states ? 0 : kAutoHead;
    const size_t need = saved_states ? hgrn2_bwd_saved_workspace_bytes(shape, gated ? 1 : 0)
                                     : (gated ? hgrn2_bwd_gated_workspace_bytes(shape) : hgrn2_bwd_workspace_bytes(shape));
    {
        SeqDims d;
        const int rc = check_shape(&alt[0], true, &d, false, true);
        if (rc != HGRN2_OK) return rc;
    }
    if (need > 0 && (!workspace || workspace_bytes < need || ((uintptr_t)workspace & 255))) return HGRN2_ERR_WORKSPACE;
    char* rest = static_cast<char*>(workspace) + head;
    const size_t rest_bytes = workspace_bytes - (workspace ? head : 0);
    Alternative a;
    a.validate_only = true;
    for (int i = 0; i < kAlternatives; ++i) {
        const int rc = bwd_one(&alt[i], q, f, beta, gated, v, h0, grad_o, grad_hT, grad_q, grad_f, grad_beta, grad_v, grad_h0,
                               rest, rest_bytes, hip_stream, saved_states, &a);
        if (rc != HGRN2_OK) return rc;
    }
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    int* flags = static_cast<int*>(workspace);
    // the flags the forward pass of the pair left behind the states: 64 tokens per chunk ran alone if the
    // first is clear, 16 if the second is set, 32 otherwise
    const int* kept = saved_states ? reinterpret_cast<const int*>(static_cast<const char*>(saved_states) +
                                                                  hgrn2_saved_states_bytes(shape) - kAutoHead)
                                   : nullptr;
    if (!saved_states && launch_zero_floats(reinterpret_cast<float*>(flags), 4, stream) != hipSuccess) return HGRN2_ERR_HIP;
    a.validate_only = false;
    for (int i = 0; i < kAlternatives; ++i) {
        a.choice2 = nullptr; a.path2 = 0;
        if (saved_states) {
            a.choice = i == 2 ? kept + 1 : kept; a.path = i == 0 ? 0 : 1;
            if (i == 1) a.choice2 = kept + 1;
            a.flag = i + 1 < kAlternatives ? nullptr : shape->gate_domain_flag;
        } else {
            a.choice = i == 0 ? nullptr : flags + (i - 1); a.path = 1;
            a.flag = i + 1 < kAlternatives ? flags + i : shape->gate_domain_flag;
        }
        const int rc = bwd_one(&alt[i], q, f, beta, gated, v, h0, grad_o, grad_hT, grad_q, grad_f, grad_beta, grad_v, grad_h0,
                               rest, rest_bytes, hip_stream, saved_states, &a);
        if (rc != HGRN2_OK) return rc;
    }
    return HGRN2_OK;
}

static int bwd_one(const hgrn2_shape* shape, const void* q, const void* f, const float* beta, bool gated,
                   const void* v, const float* h0, const void* grad_o, const float* grad_hT, void* grad_q,
                   void* grad_f, float* grad_beta, void* grad_v, float* grad_h0, void* workspace,
                   size_t workspace_bytes, void* hip_stream, const void* saved_states, const Alternative* alt)
{
    SeqDims d;
    const int rc = check_shape(shape, true, &d, false, true);
    if (rc != HGRN2_OK) return rc;
    const bool has_tokens = (size_t)d.BH * d.N > 0;
    if (has_tokens && (!q || !f || !v || !grad_o || !grad_q || !grad_f || !grad_v)) return HGRN2_ERR_NULL;
    if (gated && (size_t)shape->H * d.dk > 0 && (!grad_beta || (has_tokens && !beta))) return HGRN2_ERR_NULL;
    d.beta = gated ? beta : nullptr;
    if (alt) { d.lay.choice = alt->choice; d.lay.path = alt->path; d.lay.alt = alt->choice2; d.lay.alt_path = alt->path2; d.domain_flag = alt->flag; }
    const BwdLayout l = bwd_layout(d, gated, saved_states != nullptr);
    const size_t need = l.total();
    if (need > 0 && (!workspace || workspace_bytes < need || ((uintptr_t)workspace & 255))) return HGRN2_ERR_WORKSPACE;
    if (alt && alt->validate_only) return HGRN2_OK;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    char* at = static_cast<char*>(workspace);
    auto take = [&](size_t bytes) { char* r = at; at += bytes; return r; };
    const void* ws_s = saved_states ? saved_states : take(l.states);
    float* fwd_run_state = reinterpret_cast<float*>(take(l.fwd_run_state));
    float* fwd_run_decay = reinterpret_cast<float*>(take(l.fwd_run_decay));
    float* tail_state = reinterpret_cast<float*>(take(l.tail_state));
    float* tail_decay = reinterpret_cast<float*>(take(l.tail_decay));
    float* bound0 = reinterpret_cast<float*>(take(l.bound0));
    float* ws_part = gated ? reinterpret_cast<float*>(take(l.partials)) : nullptr;
    if (d.BH > 0 && !has_tokens) {
        // no tokens: the state gradient passes through unchanged (the sweep of an empty sequence does that)
        if (grad_h0 && launch_sweep(d, kSweepGrad, q, f, grad_o, grad_hT, grad_h0, nullptr, nullptr, stream) != hipSuccess)
            return HGRN2_ERR_HIP;
    } else if (d.BH > 0) {
        // 1. forward states of every chunk (few long sequences: in runs, as the forward pass walks them)
        int run_chunks;
        const int seg = saved_states ? 1 : plan_runs(d, false, &run_chunks);
        void* ws_out = saved_states ? nullptr : const_cast<void*>(ws_s);
        if (saved_states) {
            // a forward pass has left them
        } else if (seg > 1) {
            const SeqDims r = as_runs(d, seg, run_chunks);
            if (launch_sweep(r, kSweepStateBwd, nullptr, f, v, nullptr, fwd_run_state, nullptr, fwd_run_decay, stream) != hipSuccess ||
                launch_run_carry(d.BH, seg, d.dk, d.dv, h0, fwd_run_state, fwd_run_decay, nullptr, false, stream, d.lay.choice, d.lay.path) != hipSuccess ||
                launch_sweep(r, kSweepStateBwd, nullptr, f, v, fwd_run_state, nullptr, ws_out, nullptr, stream) != hipSuccess)
                return HGRN2_ERR_HIP;
        } else if (launch_sweep(d, kSweepStateBwd, nullptr, f, v, h0, nullptr, ws_out, nullptr, stream) != hipSuccess) {
            return HGRN2_ERR_HIP;
        }
        // 2. the state gradient at the run boundaries of the reverse walk: a zero-start gradient sweep
        //    over the tokens after run 0, in short sub-runs, and its carry from grad_hT
        const BwdFusedPlan& pl = l.plan;
        if (pl.R > 1 && !pl.light) {
            SeqDims t = d;
            t.window = true;
            const long long skip = (long long)pl.rc * d.lay.sub;          // tokens of run 0
            t.N = d.N - (int)skip;
            t.NC = d.NC - pl.rc;
            const SeqDims r = as_runs(t, pl.seg_tail, pl.sub_chunks);
            const size_t io = d.io_bf16 ? 2 : 4, ge = d.gate_bf16 ? 2 : 4;   // bytes per element
            const char* q_t = static_cast<const char*>(q) + (size_t)skip * d.lay.sn_k * io;
            const char* f_t = static_cast<const char*>(f) + (size_t)skip * d.lay.sn_k * ge;
            const char* g_t = static_cast<const char*>(grad_o) + (size_t)skip * d.lay.sn_v * io;
            if (launch_sweep(r, kSweepGrad, q_t, f_t, g_t, nullptr, tail_state, nullptr, tail_decay, stream) != hipSuccess ||
                launch_run_carry(d.BH, pl.seg_tail, d.dk, d.dv, grad_hT, tail_state, tail_decay, bound0, true, stream, d.lay.choice, d.lay.path) != hipSuccess)
                return HGRN2_ERR_HIP;
        }
        // 3. the reverse walk: dq, df, dv of every chunk, grad_h0
        if (launch_bwd_fused(d, pl, q, f, v, grad_o, ws_s, grad_hT, grad_h0, bound0, tail_state, grad_q, grad_f, grad_v,
                             ws_part, stream) != hipSuccess)
            return HGRN2_ERR_HIP;
    }
    // an empty batch or sequence has NC = 0 or B = 0: the reduction then writes zeros
    if (gated && reduce_beta_partials(d, ws_part, grad_beta, stream, has_tokens ? l.plan.R : 0) != hipSuccess) return HGRN2_ERR_HIP;
    return HGRN2_OK;
}

int hgrn2_bwd(const hgrn2_shape* shape, const void* q, const void* f, const void* v, const float* h0,
              const void* grad_o, const float* grad_hT, void* grad_q, void* grad_f, void* grad_v,
              float* grad_h0, void* workspace, size_t workspace_bytes, void* hip_stream)
{
    return bwd_impl(shape, q, f, nullptr, false, v, h0, grad_o, grad_hT, grad_q, grad_f, nullptr, grad_v, grad_h0,
                    workspace, workspace_bytes, hip_stream);
}

// ---- hgrn2_bwd for callers that may not allocate ------------------------------------------------
// The workspace is a fixed array in device memory that belongs to the library's code object: every
// GPU the library runs on holds its own copy, at its own address, until the process ends.
namespace {
constexpr size_t kScratchBytes = (size_t)32 << 20;
constexpr int kMaxDevices = 64;
}
static __device__ __align__(256) unsigned char scratch[kScratchBytes];
namespace {
void* scratch_ptr[kMaxDevices];          // address of `scratch` on each device, once asked for

// The array's name is only a handle on the host; its device address has to be looked up, once per
// device, with that device current.
int scratch_of_current_device(void** out)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return HGRN2_ERR_HIP;
    if (!scratch_ptr[dev]) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return HGRN2_ERR_HIP;
        scratch_ptr[dev] = ptr;
    }
    *out = scratch_ptr[dev];
    return HGRN2_OK;
}
}   // namespace

size_t hgrn2_noalloc_workspace_limit(void) { return kScratchBytes; }

int hgrn2_noalloc_init(void)
{
    void* ptr;
    return scratch_of_current_device(&ptr);
}

int hgrn2_bwd_noalloc(const hgrn2_shape* shape, const void* q, const void* f, const void* v, const float* h0,
                      const void* grad_o, const float* grad_hT, void* grad_q, void* grad_f, void* grad_v,
                      float* grad_h0, void* hip_stream)
{
    SeqDims d;
    hgrn2_shape alt[kAlternatives];
    if (!shape) return HGRN2_ERR_NULL;
    alternatives(shape, alt);
    const int rc = check_shape(&alt[0], true, &d, false, true);
    if (rc != HGRN2_OK) return rc;
    if (hgrn2_bwd_workspace_bytes(shape) > kScratchBytes) return HGRN2_ERR_WORKSPACE;
    void* ws = nullptr;
    const int rs = scratch_of_current_device(&ws);
    if (rs != HGRN2_OK) return rs;
    return bwd_impl(shape, q, f, nullptr, false, v, h0, grad_o, grad_hT, grad_q, grad_f, nullptr, grad_v, grad_h0, ws,
                    kScratchBytes, hip_stream);
}

int hgrn2_bwd_gated(const hgrn2_shape* shape, const void* q, const void* z, const float* beta, const void* v,
                    const float* h0, const void* grad_o, const float* grad_hT, void* grad_q, void* grad_z,
                    float* grad_beta, void* grad_v, float* grad_h0, void* workspace, size_t workspace_bytes,
                    void* hip_stream)
{
    return bwd_impl(shape, q, z, beta, true, v, h0, grad_o, grad_hT, grad_q, grad_z, grad_beta, grad_v, grad_h0,
                    workspace, workspace_bytes, hip_stream);
}

size_t hgrn2_saved_states_bytes(const hgrn2_shape* shape)
{
    // (chunk = HGRN2_CHUNK_AUTO: room for the alternative with most chunks, then the int that names the one that ran)
    return max_over_alternatives(shape, [](const hgrn2_shape* s) -> size_t {
        SeqDims d;
        if (check_shape(s, true, &d, false, true) != HGRN2_OK) return 0;
        return round256(state_ws_bytes(d));
    }, true, true);
}

size_t hgrn2_bwd_saved_workspace_bytes(const hgrn2_shape* shape, int32_t gated)
{
    const bool g = gated != 0;
    return max_over_alternatives(shape, [g](const hgrn2_shape* s) -> size_t {
        SeqDims d;
        if (check_shape(s, true, &d, false, true) != HGRN2_OK) return 0;
        return bwd_layout(d, g, true).total();
    }, false, true);
}

int hgrn2_fwd_saving(const hgrn2_shape* shape, const void* q, const void* f, const float* beta, const void* v,
                     const float* h0, void* o, float* hT, void* saved_states, size_t saved_states_bytes,
                     void* workspace, size_t workspace_bytes, void* hip_stream)
{
    SeqDims d;
    hgrn2_shape alt[kAlternatives];
    if (!shape) return HGRN2_ERR_NULL;
    alternatives(shape, alt);
    const int rc = check_shape(&alt[0], true, &d, false, true);      // the shapes the backward pass takes
    if (rc != HGRN2_OK) return rc;
    const size_t need = state_ws_bytes(d) > 0 ? hgrn2_saved_states_bytes(shape) : 0;
    if (need > 0 && (!saved_states || saved_states_bytes < need || ((uintptr_t)saved_states & 255))) return HGRN2_ERR_WORKSPACE;
    return fwd_impl(shape, q, f, beta, beta != nullptr, v, h0, o, hT, workspace, workspace_bytes, hip_stream,
                    need > 0 ? saved_states : nullptr);
}

int hgrn2_bwd_saved(const hgrn2_shape* shape, const void* q, const void* f, const float* beta, const void* v,
                    const void* saved_states, size_t saved_states_bytes, const void* grad_o, const float* grad_hT,
                    void* grad_q, void* grad_f, float* grad_beta, void* grad_v, float* grad_h0, void* workspace,
                    size_t workspace_bytes, void* hip_stream)
{
    SeqDims d;
    hgrn2_shape alt[kAlternatives];
    if (!shape) return HGRN2_ERR_NULL;
    alternatives(shape, alt);
    const int rc = check_shape(&alt[0], true, &d, false, true);
    if (rc != HGRN2_OK) return rc;
    const size_t need = state_ws_bytes(d) > 0 ? hgrn2_saved_states_bytes(shape) : 0;
    if (need == 0)      // no chunks: nothing was saved, the ordinary pass handles what is left (grad_h0, grad_beta)
        return bwd_impl(&alt[0], q, f, beta, beta != nullptr, v, nullptr, grad_o, grad_hT, grad_q, grad_f, grad_beta, grad_v,
                        grad_h0, workspace, workspace_bytes, hip_stream);
    if (!saved_states || saved_states_bytes < need || ((uintptr_t)saved_states & 255)) return HGRN2_ERR_WORKSPACE;
    return bwd_impl(shape, q, f, beta, beta != nullptr, v, nullptr, grad_o, grad_hT, grad_q, grad_f, grad_beta, grad_v,
                    grad_h0, workspace, workspace_bytes, hip_stream, saved_states);
}

static size_t fwd_varlen_ws_one(const hgrn2_shape* shape)
{
    SeqDims d;
    if (check_shape_varlen(shape, false, &d, true) != HGRN2_OK) return 0;
    const PackedRuns p = plan_packed_runs(shape, d, false);
    return p.table_bytes + round256(state_ws_bytes(d)) + p.state_bytes + p.decay_bytes;
}

static size_t bwd_varlen_ws_one(const hgrn2_shape* shape)
{
    SeqDims d;
    if (check_shape_varlen(shape, true, &d, true) != HGRN2_OK) return 0;
    const PackedRuns p = plan_packed_runs(shape, d, true);
    return p.table_bytes + 2 * (round256(state_ws_bytes(d)) + p.state_bytes) + p.decay_bytes +
           round256(beta_partials_bytes(d));
}

size_t hgrn2_fwd_varlen_workspace_bytes(const hgrn2_shape* shape)
{
    return max_over_alternatives(shape, fwd_varlen_ws_one, true, false, true);
}

size_t hgrn2_bwd_varlen_workspace_bytes(const hgrn2_shape* shape)
{
    return max_over_alternatives(shape, bwd_varlen_ws_one, true, true, true);
}

// A packed batch's forward pass can hand its per-chunk states to the backward pass only when both
// see the batch the same way: not cut into runs, or cut into the same runs (the chunk slots follow
// the runs; the forward pass starts cutting at shorter and more sequences than the backward pass).
// Known from the shape alone, so both entry points of the pair decide alike.
static bool packed_states_kept(const hgrn2_shape* shape, const SeqDims& d)
{
    return plan_packed_runs(shape, d, false).run_chunks == plan_packed_runs(shape, d, true).run_chunks;
}

static int fwd_varlen_one(const hgrn2_shape* shape, const int32_t* cu_seqlens, const void* q, const void* f,
                          const float* beta, const void* v, const float* h0, void* o, float* hT, void* workspace,
                          size_t workspace_bytes, void* hip_stream, void* save_states, const Alternative* alt)
{
    SeqDims d;
    const int rc = check_shape_varlen(shape, false, &d, true);
    if (rc != HGRN2_OK) return rc;
    d.beta = beta;
    if (alt) { d.lay.alt = alt->choice; d.lay.alt_path = alt->path; d.domain_flag = alt->flag; }
    if (d.BH == 0) return HGRN2_OK;
    const bool has_tokens = d.N > 0;
    if (!cu_seqlens || (has_tokens && (!q || !f || !v || !o))) return HGRN2_ERR_NULL;
    const size_t need = fwd_varlen_ws_one(shape);
    if (!workspace || workspace_bytes < need || ((uintptr_t)workspace & 255)) return HGRN2_ERR_WORKSPACE;
    if (alt && alt->validate_only) return HGRN2_OK;
    if (!has_tokens && !hT) return HGRN2_OK;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const PackedRuns pr = plan_packed_runs(shape, d, false);
    const size_t one = round256(state_ws_bytes(d));
    void* ws_s = static_cast<char*>(workspace) + pr.table_bytes;
    const int* first_run;
    // A forward pass that keeps the states also leaves the tables, as the backward pass lays them
    // out (the same entries, plus the spans of its walk), behind the states: that pass builds none.
    const bool leave_tables = save_states != nullptr;
    if (build_packed_tables(shape, leave_tables ? plan_packed_runs(shape, d, true) : pr, cu_seqlens,
                            leave_tables ? static_cast<char*>(save_states) + one : workspace, &d, &first_run,
                            stream) != hipSuccess)
        return HGRN2_ERR_HIP;
    if (first_run) {
        // d now describes the runs: walk each from zero, carry the states over the runs of a sequence, walk again
        float* run_state = reinterpret_cast<float*>(static_cast<char*>(ws_s) + one);
        float* run_decay = reinterpret_cast<float*>(static_cast<char*>(ws_s) + one + pr.state_bytes);
        if (launch_sweep(d, kSweepStateFwd, q, f, v, nullptr, run_state, nullptr, run_decay, stream) != hipSuccess ||
            launch_run_carry_packed(shape->B, shape->H, first_run, d.dk, d.dv, h0, run_state, run_decay, hT, false,
                                    stream, d.lay.alt, d.lay.alt_path) != hipSuccess)
            return HGRN2_ERR_HIP;
        if (fwd_fused_supported(d))
            return launch_fwd_fused(d, q, f, v, run_state, o, nullptr, save_states, stream) == hipSuccess ? HGRN2_OK : HGRN2_ERR_HIP;
        if (launch_sweep(d, kSweepStateFwd, q, f, v, run_state, nullptr, ws_s, nullptr, stream) != hipSuccess ||
            launch_fwd_out(d, q, f, v, ws_s, o, stream) != hipSuccess)
            return HGRN2_ERR_HIP;
        if (save_states && has_tokens &&
            launch_sweep(d, kSweepStateBwd, nullptr, f, v, run_state, nullptr, save_states, nullptr, stream) != hipSuccess)
            return HGRN2_ERR_HIP;
        return HGRN2_OK;
    }
    if (fwd_fused_supported(d))
        return launch_fwd_fused(d, q, f, v, h0, o, hT, save_states, stream) == hipSuccess ? HGRN2_OK : HGRN2_ERR_HIP;
    if (launch_sweep(d, kSweepStateFwd, q, f, v, h0, hT, ws_s, nullptr, stream) != hipSuccess) return HGRN2_ERR_HIP;
    if (launch_fwd_out(d, q, f, v, ws_s, o, stream) != hipSuccess) return HGRN2_ERR_HIP;
    // (this sweep keeps the states in the read-out's orientation: the backward pass's come from one of their own)
    if (save_states && has_tokens &&
        launch_sweep(d, kSweepStateBwd, nullptr, f, v, h0, nullptr, save_states, nullptr, stream) != hipSuccess)
        return HGRN2_ERR_HIP;
    return HGRN2_OK;
}

// what the forward pass of a packed training pair leaves: the chunk states, then the tables
static size_t packed_saved_bytes(const hgrn2_shape* shape, const SeqDims& d)
{
    return round256(state_ws_bytes(d)) + plan_packed_runs(shape, d, true).table_bytes;
}

static size_t packed_saved_one(const hgrn2_shape* shape)
{
    SeqDims d;
    if (check_shape_varlen(shape, true, &d, true) != HGRN2_OK) return 0;
    return packed_saved_bytes(shape, d);
}

// (chunk = HGRN2_CHUNK_AUTO: every alternative keeps its states and tables in a place of its own, one
// after the other, and the int that names the alternative that ran follows them)
size_t hgrn2_saved_states_varlen_bytes(const hgrn2_shape* shape)
{
    return max_over_alternatives(shape, packed_saved_one, true, true, true, true);
}

// where alternative i of `shape` keeps its states inside `saved` (null stays null), or null when that
// alternative's pair keeps none (see packed_states_kept)
static void* packed_saved_place(const hgrn2_shape* shape, int i, const void* saved)
{
    if (!saved) return nullptr;
    hgrn2_shape alt[kAlternatives];
    alternatives(shape, alt);
    size_t off = 0;
    for (int j = 0; j < i; ++j) off += packed_saved_one(&alt[j]);
    SeqDims d;
    if (check_shape_varlen(&alt[i], true, &d, true) != HGRN2_OK) return nullptr;
    if (state_ws_bytes(d) == 0 || !packed_states_kept(&alt[i], d)) return nullptr;
    return const_cast<char*>(static_cast<const char*>(saved)) + off;
}

// Forward pass of a packed batch, or (chunk = HGRN2_CHUNK_AUTO) its three alternatives, as fwd_impl.
static int fwd_varlen_impl(const hgrn2_shape* shape, const int32_t* cu_seqlens, const void* q, const void* f,
                           const float* beta, const void* v, const float* h0, void* o, float* hT, void* workspace,
                           size_t workspace_bytes, void* hip_stream, void* save_states)
{
    if (!shape) return HGRN2_ERR_NULL;
    if (!auto_mode(shape))
        return fwd_varlen_one(shape, cu_seqlens, q, f, beta, v, h0, o, hT, workspace, workspace_bytes, hip_stream,
                              packed_saved_place(shape, 0, save_states), nullptr);
    hgrn2_shape alt[kAlternatives];
    alternatives(shape, alt);
    {
        SeqDims d;
        const int rc = check_shape_varlen(&alt[0], false, &d, true);
        if (rc != HGRN2_OK) return rc;
        if (d.BH == 0) return HGRN2_OK;
    }
    const size_t need = hgrn2_fwd_varlen_workspace_bytes(shape);
    if (!workspace || workspace_bytes < need || ((uintptr_t)workspace & 255)) return HGRN2_ERR_WORKSPACE;
    char* rest = static_cast<char*>(workspace) + kAutoHead;
    Alternative a;
    a.validate_only = true;
    for (int i = 0; i < kAlternatives; ++i) {
        const int rc = fwd_varlen_one(&alt[i], cu_seqlens, q, f, beta, v, h0, o, hT, rest, workspace_bytes - kAutoHead, hip_stream,
                                      nullptr, &a);
        if (rc != HGRN2_OK) return rc;
    }
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    int* flags = static_cast<int*>(workspace);
    if (launch_zero_floats(reinterpret_cast<float*>(flags), 4, stream) != hipSuccess) return HGRN2_ERR_HIP;
    a.validate_only = false;
    for (int i = 0; i < kAlternatives; ++i) {
        a.choice = i == 0 ? nullptr : flags + (i - 1);
        a.path = 1;
        a.flag = i + 1 < kAlternatives ? flags + i : shape->gate_domain_flag;
        const int rc = fwd_varlen_one(&alt[i], cu_seqlens, q, f, beta, v, h0, o, hT, rest, workspace_bytes - kAutoHead, hip_stream,
                                      packed_saved_place(shape, i, save_states), &a);
        if (rc != HGRN2_OK) return rc;
    }
    if (save_states) {
        int* which = reinterpret_cast<int*>(static_cast<char*>(save_states) + hgrn2_saved_states_varlen_bytes(shape) - kAutoHead);
        if (launch_sum_ints(flags, 2, which, stream) != hipSuccess) return HGRN2_ERR_HIP;
    }
    return HGRN2_OK;
}

int hgrn2_fwd_varlen(const hgrn2_shape* shape, const int32_t* cu_seqlens, const void* q, const void* f,
                     const float* beta, const void* v, const float* h0, void* o, float* hT, void* workspace,
                     size_t workspace_bytes, void* hip_stream)
{
    return fwd_varlen_impl(shape, cu_seqlens, q, f, beta, v, h0, o, hT, workspace, workspace_bytes, hip_stream, nullptr);
}

int hgrn2_fwd_varlen_saving(const hgrn2_shape* shape, const int32_t* cu_seqlens, const void* q, const void* f,
                            const float* beta, const void* v, const float* h0, void* o, float* hT, void* saved_states,
                            size_t saved_states_bytes, void* workspace, size_t workspace_bytes, void* hip_stream)
{
    if (!shape) return HGRN2_ERR_NULL;
    SeqDims d;
    hgrn2_shape alt[kAlternatives];
    alternatives(shape, alt);
    const int rc = check_shape_varlen(&alt[0], true, &d, true);      // the shapes the backward pass takes
    if (rc != HGRN2_OK) return rc;
    const size_t need = hgrn2_saved_states_varlen_bytes(shape);
    if (need > 0 && (!saved_states || saved_states_bytes < need || ((uintptr_t)saved_states & 255))) return HGRN2_ERR_WORKSPACE;
    return fwd_varlen_impl(shape, cu_seqlens, q, f, beta, v, h0, o, hT, workspace, workspace_bytes, hip_stream, saved_states);
}

static int bwd_varlen_one(const hgrn2_shape* shape, const int32_t* cu_seqlens, const void* q, const void* f,
                          const float* beta, const void* v, const float* h0, const void* grad_o, const float* grad_hT,
                          void* grad_q, void* grad_f, float* grad_beta, void* grad_v, float* grad_h0, void* workspace,
                          size_t workspace_bytes, void* hip_stream, const void* saved_states, const Alternative* alt)
{
    SeqDims d;
    const int rc = check_shape_varlen(shape, true, &d, true);
    if (rc != HGRN2_OK) return rc;
    d.beta = beta;
    if (alt) { d.lay.alt = alt->choice; d.lay.alt_path = alt->path; d.domain_flag = alt->flag; }
    if (beta && !grad_beta && (size_t)shape->H * d.dk > 0) return HGRN2_ERR_NULL;
    if (d.BH == 0) {
        if (alt && alt->validate_only) return HGRN2_OK;
        // no sequences: nothing contributes to the gradient of beta
        if (beta && (size_t)shape->H * d.dk > 0 &&
            launch_zero_floats(grad_beta, (size_t)shape->H * d.dk, static_cast<hipStream_t>(hip_stream)) != hipSuccess)
            return HGRN2_ERR_HIP;
        return HGRN2_OK;
    }
    const bool has_tokens = d.N > 0;
    if (!cu_seqlens || (has_tokens && (!q || !f || !v || !grad_o || !grad_q || !grad_f || !grad_v)))
        return HGRN2_ERR_NULL;
    const size_t need = bwd_varlen_ws_one(shape);
    if (!workspace || workspace_bytes < need || ((uintptr_t)workspace & 255)) return HGRN2_ERR_WORKSPACE;
    if (alt && alt->validate_only) return HGRN2_OK;
    if (!has_tokens && !grad_h0 && !beta) return HGRN2_OK;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const PackedRuns pr = plan_packed_runs(shape, d, true);
    const size_t one = round256(state_ws_bytes(d));
    char* base = static_cast<char*>(workspace) + pr.table_bytes;
    if (!has_tokens) saved_states = nullptr;          // none were kept
    // with states left by the forward pass, only the sweep of the state gradient remains to be run
    void* ws_s = saved_states ? const_cast<void*>(saved_states) : base;
    void* ws_ds = base + one;
    float* ws_part = beta ? reinterpret_cast<float*>(base + 2 * (one + pr.state_bytes) + pr.decay_bytes) : nullptr;
    const int* first_run;
    // (states kept: the forward pass has left the tables behind them)
    void* tables = saved_states ? const_cast<char*>(static_cast<const char*>(saved_states)) + one : workspace;
    if (build_packed_tables(shape, pr, cu_seqlens, tables, &d, &first_run, stream, saved_states == nullptr) != hipSuccess)
        return HGRN2_ERR_HIP;
    if (first_run) {
        float* run_s = reinterpret_cast<float*>(base + 2 * one);
        float* run_ds = reinterpret_cast<float*>(base + 2 * one + pr.state_bytes);
        float* run_decay = reinterpret_cast<float*>(base + 2 * (one + pr.state_bytes));
        // d now describes the runs.  What every run adds to the state gradient (and, unless the
        // forward pass has left the states, to the state) from zero, the carries over the runs of a
        // sequence, the forward states run by run, and the reverse walk over spans of the runs'
        // chunks, for which a run is a sequence whose grad_hT is the state gradient the carry left
        // at its end (the carry has written the sequences' grad_h0).
        if (saved_states) {
            if (launch_sweep(d, kSweepGrad, q, f, grad_o, nullptr, run_ds, nullptr, run_decay, stream) != hipSuccess)
                return HGRN2_ERR_HIP;
        } else if (launch_sweep_pair_ends(d, q, f, v, grad_o, run_s, run_ds, run_decay, stream) != hipSuccess ||
                   launch_run_carry_packed(shape->B, shape->H, first_run, d.dk, d.dv, h0, run_s, run_decay, nullptr, false,
                                           stream, d.lay.alt, d.lay.alt_path) != hipSuccess ||
                   launch_sweep(d, kSweepStateBwd, nullptr, f, v, run_s, nullptr, ws_s, nullptr, stream) != hipSuccess) {
            return HGRN2_ERR_HIP;
        }
        if (launch_run_carry_packed(shape->B, shape->H, first_run, d.dk, d.dv, grad_hT, run_ds, run_decay, grad_h0, true,
                                    stream, d.lay.alt, d.lay.alt_path) != hipSuccess ||
            launch_bwd_fused_grouped(d, q, f, v, grad_o, ws_s, run_ds, nullptr, grad_q, grad_f, grad_v, ws_part,
                                     stream) != hipSuccess)
            return HGRN2_ERR_HIP;
    } else {
        // Two ways, and only the lengths (device data) tell which is faster: (1) one forward-state
        // sweep, then the reverse walk over equal spans of chunks that carries the state gradient in
        // registers and produces the gradients chunk by chunk; (0) both sweeps and the per-chunk
        // gradient kernel (one sequence far longer than a span).  The table kernel has chosen; the
        // kernels of both are enqueued and those of the other way return at once.  With the states
        // left by the forward pass the walk is the faster one for any lengths (measured also with one
        // document of half or all of the tokens): it alone is enqueued then.
        if (saved_states) {
            if (launch_bwd_fused_grouped(d, q, f, v, grad_o, ws_s, grad_hT, grad_h0, grad_q, grad_f, grad_v, ws_part,
                                         stream) != hipSuccess)
                return HGRN2_ERR_HIP;
            if (beta && reduce_beta_partials(d, ws_part, grad_beta, stream) != hipSuccess) return HGRN2_ERR_HIP;
            return HGRN2_OK;
        }
        SeqDims walk = d, split = d;
        walk.lay.choice = split.lay.choice = reinterpret_cast<const int*>(static_cast<char*>(tables) + pr.groups_at) + pr.G + 1;
        walk.lay.path = 1;
        split.lay.path = 0;
        if (shape->B < 4 * d.lay.spans) {    // few sequences: longest first, a workgroup each, suits uneven lengths
            split.lay.groups = nullptr;      // (with many, the walk is chosen nearly always, and a grid of
            split.lay.G = 0;                 // groups that only has to return is the cheaper one)
        }
        if (launch_sweep(walk, kSweepStateBwd, nullptr, f, v, h0, nullptr, ws_s, nullptr, stream) != hipSuccess ||
            launch_bwd_fused_grouped(walk, q, f, v, grad_o, ws_s, grad_hT, grad_h0, grad_q, grad_f, grad_v, ws_part,
                                     stream) != hipSuccess ||
            launch_sweep_pair(split, q, f, v, grad_o, h0, grad_hT, grad_h0, ws_s, ws_ds, stream) != hipSuccess ||
            (has_tokens &&
             launch_bwd_grad(split, q, f, v, grad_o, ws_s, ws_ds, grad_q, grad_f, grad_v, ws_part, stream) != hipSuccess))
            return HGRN2_ERR_HIP;
    }
    if (beta && reduce_beta_partials(d, ws_part, grad_beta, stream) != hipSuccess) return HGRN2_ERR_HIP;
    return HGRN2_OK;
}

// Backward pass of a packed batch, or (chunk = HGRN2_CHUNK_AUTO) its three alternatives, as bwd_impl.
static int bwd_varlen_impl(const hgrn2_shape* shape, const int32_t* cu_seqlens, const void* q, const void* f,
                           const float* beta, const void* v, const float* h0, const void* grad_o, const float* grad_hT,
                           void* grad_q, void* grad_f, float* grad_beta, void* grad_v, float* grad_h0, void* workspace,
                           size_t workspace_bytes, void* hip_stream, const void* saved_states)
{
    if (!shape) return HGRN2_ERR_NULL;
    if (!auto_mode(shape))
        return bwd_varlen_one(shape, cu_seqlens, q, f, beta, v, h0, grad_o, grad_hT, grad_q, grad_f, grad_beta, grad_v, grad_h0,
                              workspace, workspace_bytes, hip_stream, packed_saved_place(shape, 0, saved_states), nullptr);
    hgrn2_shape alt[kAlternatives];
    alternatives(shape, alt);
    bool no_sequences = false;
    {
        SeqDims d;
        const int rc = check_shape_varlen(&alt[0], true, &d, true);
        if (rc != HGRN2_OK) return rc;
        no_sequences = d.BH == 0;
    }
    if (no_sequences)       // (grad_beta = 0: any alternative does that, and none needs a workspace)
        return bwd_varlen_one(&alt[0], cu_seqlens, q, f, beta, v, h0, grad_o, grad_hT, grad_q, grad_f, grad_beta, grad_v, grad_h0,
                              workspace, workspace_bytes, hip_stream, nullptr, nullptr);
    const size_t need = hgrn2_bwd_varlen_workspace_bytes(shape);
    if (!workspace || workspace_bytes < need || ((uintptr_t)workspace & 255)) return HGRN2_ERR_WORKSPACE;
    char* rest = static_cast<char*>(workspace) + kAutoHead;
    Alternative a;
    a.validate_only = true;
    for (int i = 0; i < kAlternatives; ++i) {
        const int rc = bwd_varlen_one(&alt[i], cu_seqlens, q, f, beta, v, h0, grad_o, grad_hT, grad_q, grad_f, grad_beta, grad_v,
                                      grad_h0, rest, workspace_bytes - kAutoHead, hip_stream, nullptr, &a);
        if (rc != HGRN2_OK) return rc;
    }
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    int* flags = static_cast<int*>(workspace);
    const int* which = saved_states ? reinterpret_cast<const int*>(static_cast<const char*>(saved_states) +
                                                                   hgrn2_saved_states_varlen_bytes(shape) - kAutoHead)
                                    : nullptr;
    if (!saved_states && launch_zero_floats(reinterpret_cast<float*>(flags), 4, stream) != hipSuccess) return HGRN2_ERR_HIP;
    a.validate_only = false;
    for (int i = 0; i < kAlternatives; ++i) {
        if (saved_states) {
            a.choice = which; a.path = i;
            a.flag = i + 1 < kAlternatives ? nullptr : shape->gate_domain_flag;
        } else {
            a.choice = i == 0 ? nullptr : flags + (i - 1); a.path = 1;
            a.flag = i + 1 < kAlternatives ? flags + i : shape->gate_domain_flag;
        }
        const int rc = bwd_varlen_one(&alt[i], cu_seqlens, q, f, beta, v, h0, grad_o, grad_hT, grad_q, grad_f, grad_beta, grad_v,
                                      grad_h0, rest, workspace_bytes - kAutoHead, hip_stream,
                                      packed_saved_place(shape, i, saved_states), &a);
        if (rc != HGRN2_OK) return rc;
    }
    return HGRN2_OK;
}

int hgrn2_bwd_varlen(const hgrn2_shape* shape, const int32_t* cu_seqlens, const void* q, const void* f,
                     const float* beta, const void* v, const float* h0, const void* grad_o, const float* grad_hT,
                     void* grad_q, void* grad_f, float* grad_beta, void* grad_v, float* grad_h0, void* workspace,
                     size_t workspace_bytes, void* hip_stream)
{
    return bwd_varlen_impl(shape, cu_seqlens, q, f, beta, v, h0, grad_o, grad_hT, grad_q, grad_f, grad_beta, grad_v, grad_h0,
                           workspace, workspace_bytes, hip_stream, nullptr);
}

int hgrn2_bwd_varlen_saved(const hgrn2_shape* shape, const int32_t* cu_seqlens, const void* q, const void* f,
                           const float* beta, const void* v, const float* h0, const void* saved_states,
                           size_t saved_states_bytes, const void* grad_o, const float* grad_hT, void* grad_q, void* grad_f,
                           float* grad_beta, void* grad_v, float* grad_h0, void* workspace, size_t workspace_bytes,
                           void* hip_stream)
{
    if (!shape) return HGRN2_ERR_NULL;
    SeqDims d;
    hgrn2_shape alt[kAlternatives];
    alternatives(shape, alt);
    const int rc = check_shape_varlen(&alt[0], true, &d, true);
    if (rc != HGRN2_OK) return rc;
    const size_t need = hgrn2_saved_states_varlen_bytes(shape);
    if (need > 0 && (!saved_states || saved_states_bytes < need || ((uintptr_t)saved_states & 255))) return HGRN2_ERR_WORKSPACE;
    return bwd_varlen_impl(shape, cu_seqlens, q, f, beta, v, h0, grad_o, grad_hT, grad_q, grad_f, grad_beta, grad_v, grad_h0,
                           workspace, workspace_bytes, hip_stream, saved_states);
}

int hgrn2_min_gate_product(const hgrn2_shape* shape, const void* f, const float* beta, float* min_product,
                           void* hip_stream)
{
    SeqDims d;
    const int rc = check_shape(shape, false, &d, false, true);
    if (rc != HGRN2_OK) return rc;
    if (!min_product) return HGRN2_ERR_NULL;
    if ((size_t)d.BH * d.N > 0 && !f) return HGRN2_ERR_NULL;
    d.beta = beta;
    if (launch_min_gate_product(d, (fine_mode(shape) ? shape->chunk : kChunk) / 2, f, min_product,
                                static_cast<hipStream_t>(hip_stream)) != hipSuccess)
        return HGRN2_ERR_HIP;
    return HGRN2_OK;
}

size_t hgrn2_min_gate_product_varlen_workspace_bytes(const hgrn2_shape* shape)
{
    SeqDims d;
    if (check_shape_varlen(shape, false, &d, true) != HGRN2_OK) return 0;
    return round256(varlen_table_bytes(shape->B));
}

int hgrn2_min_gate_product_varlen(const hgrn2_shape* shape, const int32_t* cu_seqlens, const void* f, const float* beta,
                                  float* min_product, void* workspace, size_t workspace_bytes, void* hip_stream)
{
    SeqDims d;
    const int rc = check_shape_varlen(shape, false, &d, true);
    if (rc != HGRN2_OK) return rc;
    if (!min_product) return HGRN2_ERR_NULL;
    if (d.BH > 0 && (!cu_seqlens || (d.N > 0 && !f))) return HGRN2_ERR_NULL;
    const size_t need = hgrn2_min_gate_product_varlen_workspace_bytes(shape);
    if (!workspace || workspace_bytes < need || ((uintptr_t)workspace & 255)) return HGRN2_ERR_WORKSPACE;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    d.beta = beta;
    // the probe's windows lie in a table of 64-token chunks whatever chunk length it is asked about
    d.lay.sub = kChunk;
    d.NC = (int)((long long)d.N / kChunk + shape->B);
    if (d.BH == 0) d.NC = 0;                  // no sequences: the probe writes 1
    else {
        int* table = static_cast<int*>(workspace);
        d.lay.vl = table;
        if (launch_varlen_table(cu_seqlens, shape->B, d.N, table, stream) != hipSuccess) return HGRN2_ERR_HIP;
    }
    if (launch_min_gate_product(d, (fine_mode(shape) ? shape->chunk : kChunk) / 2, f, min_product, stream) != hipSuccess)
        return HGRN2_ERR_HIP;
    return HGRN2_OK;
}

int hgrn2_cumax(int32_t L, int32_t d, const float* gamma, float* beta, void* hip_stream)
{
    if (L < 0 || d < 0) return HGRN2_ERR_SHAPE;
    if ((size_t)L * d == 0) return HGRN2_OK;
    if (!gamma || !beta) return HGRN2_ERR_NULL;
    if (launch_cumax(L, d, gamma, beta, static_cast<hipStream_t>(hip_stream)) != hipSuccess) return HGRN2_ERR_HIP;
    return HGRN2_OK;
}

static int step_impl(int32_t B, int32_t H, int32_t dk, int32_t dv, int32_t io_dtype, int32_t gate_dtype,
                     const void* q_t, const void* f_t, const float* beta, bool gated, const void* v_t, float* state,
                     void* o_t, void* hip_stream)
{
    if (B < 0 || H < 0 || dk <= 0 || dv <= 0) return HGRN2_ERR_SHAPE;
    if (!dtype_ok(io_dtype) || !dtype_ok(gate_dtype)) return HGRN2_ERR_SHAPE;
    const long long bh = (long long)B * H;
    if (bh > INT_MAX / 2) return HGRN2_ERR_SHAPE;
    if (!dim_ok(dk) || !dim_ok(dv)) return HGRN2_ERR_UNSUPPORTED;
    if (bh > 0 && (!q_t || !f_t || !v_t || !state || !o_t || (gated && !beta))) return HGRN2_ERR_NULL;
    if (launch_step((int)bh, dk, dv, io_dtype == HGRN2_BF16, gate_dtype == HGRN2_BF16, q_t, f_t, v_t, state, o_t,
                    gated ? beta : nullptr, H > 0 ? H : 1, static_cast<hipStream_t>(hip_stream)) != hipSuccess)
        return HGRN2_ERR_HIP;
    return HGRN2_OK;
}

int hgrn2_step(int32_t B, int32_t H, int32_t dk, int32_t dv, int32_t io_dtype, int32_t gate_dtype,
               const void* q_t, const void* f_t, const void* v_t, float* state, void* o_t, void* hip_stream)
{
    return step_impl(B, H, dk, dv, io_dtype, gate_dtype, q_t, f_t, nullptr, false, v_t, state, o_t, hip_stream);
}

int hgrn2_step_gated(int32_t B, int32_t H, int32_t dk, int32_t dv, int32_t io_dtype, int32_t gate_dtype,
                     const void* q_t, const void* z_t, const float* beta, const void* v_t, float* state, void* o_t,
                     void* hip_stream)
{
    return step_impl(B, H, dk, dv, io_dtype, gate_dtype, q_t, z_t, beta, true, v_t, state, o_t, hip_stream);
}

int hgrn2_state_sweep(const hgrn2_shape* shape, int32_t mode, const void* q, const void* f, const void* b_src,
                      const float* init_state, float* final_state, void* chunk_states,
                      size_t chunk_states_bytes, void* hip_stream)
{
    if (mode < 0 || mode > 2) return HGRN2_ERR_SHAPE;
    SeqDims d;
    const int rc = check_shape(shape, mode != HGRN2_SWEEP_STATE_FWD, &d);
    if (rc != HGRN2_OK) return rc;
    const bool has_tokens = (size_t)d.BH * d.N > 0;
    if (has_tokens && (!f || !b_src || (mode == HGRN2_SWEEP_STATE_GRAD && !q))) return HGRN2_ERR_NULL;
    const size_t need = round256(state_ws_bytes(d));
    if (need > 0 && (!chunk_states || chunk_states_bytes < need || ((uintptr_t)chunk_states & 255)))
        return HGRN2_ERR_WORKSPACE;
    if (d.BH == 0) return HGRN2_OK;
    if (launch_sweep(d, static_cast<SweepMode>(mode), q, f, b_src, init_state, final_state, chunk_states, nullptr,
                     static_cast<hipStream_t>(hip_stream)) != hipSuccess)
        return HGRN2_ERR_HIP;
    return HGRN2_OK;
}

int hgrn2_fwd_readout(const hgrn2_shape* shape, const void* q, const void* f, const void* v,
                      const void* chunk_states, void* o, void* hip_stream)
{
    SeqDims d;
    const int rc = check_shape(shape, false, &d);
    if (rc != HGRN2_OK) return rc;
    if ((size_t)d.BH * d.N == 0) return HGRN2_OK;
    if (!q || !f || !v || !chunk_states || !o) return HGRN2_ERR_NULL;
    if ((uintptr_t)chunk_states & 255) return HGRN2_ERR_WORKSPACE;
    if (launch_fwd_out(d, q, f, v, chunk_states, o, static_cast<hipStream_t>(hip_stream)) != hipSuccess)
        return HGRN2_ERR_HIP;
    return HGRN2_OK;
}

int hgrn2_bwd_chunk_grads(const hgrn2_shape* shape, const void* q, const void* f, const void* v,
                          const void* grad_o, const void* chunk_states, const void* chunk_state_grads,
                          void* grad_q, void* grad_f, void* grad_v, void* hip_stream)
{
    SeqDims d;
    const int rc = check_shape(shape, true, &d);
    if (rc != HGRN2_OK) return rc;
    if (!d.io_bf16) return HGRN2_ERR_UNSUPPORTED;          // this stage exists for bf16 storage only
    if ((size_t)d.BH * d.N == 0) return HGRN2_OK;
    if (!q || !f || !v || !grad_o || !chunk_states || !chunk_state_grads || !grad_q || !grad_f || !grad_v)
        return HGRN2_ERR_NULL;
    if (((uintptr_t)chunk_states & 255) || ((uintptr_t)chunk_state_grads & 255)) return HGRN2_ERR_WORKSPACE;
    if (launch_bwd_grad(d, q, f, v, grad_o, chunk_states, chunk_state_grads, grad_q, grad_f, grad_v, nullptr,
                        static_cast<hipStream_t>(hip_stream)) != hipSuccess)
        return HGRN2_ERR_HIP;
    return HGRN2_OK;
}

static int h1_check(int32_t B, int32_t N, int32_t d, int32_t io_dtype, int32_t gate_dtype)
{
    if (B < 0 || N < 0 || d < 0) return HGRN2_ERR_SHAPE;
    if (!dtype_ok(io_dtype) || !dtype_ok(gate_dtype)) return HGRN2_ERR_SHAPE;
    if ((long long)B * (d / 128 + 1) > INT_MAX / 2 || d > (1 << 20)) return HGRN2_ERR_SHAPE;   // grid size; 32-bit byte offsets inside a block of rows
    if (d % 64 != 0 || io_dtype != HGRN2_BF16) return HGRN2_ERR_UNSUPPORTED;          // a workgroup owns 64 channels
    return HGRN2_OK;
}

size_t hgrn1_workspace_bytes(int32_t B, int32_t N, int32_t d)
{
    if (h1_check(B, N, d, HGRN2_BF16, HGRN2_BF16) != HGRN2_OK) return 0;
    return round256(hgrn1_ws_bytes(B, N, d));
}

static int h1_fwd_impl(int32_t B, int32_t N, int32_t d, int32_t io_dtype, int32_t gate_dtype, const void* f,
                       const void* i, const void* o, const float* beta, bool act, const float* h0, void* y, float* hN,
                       void* workspace, size_t workspace_bytes, void* hip_stream)
{
    const int rc = h1_check(B, N, d, io_dtype, gate_dtype);
    if (rc != HGRN2_OK) return rc;
    const bool has_tokens = (size_t)B * N * d > 0;
    if (has_tokens && (!f || !i || !o || !y || (act && !beta))) return HGRN2_ERR_NULL;
    const size_t need = round256(hgrn1_ws_bytes(B, N, d));
    if (need > 0 && (!workspace || workspace_bytes < need || ((uintptr_t)workspace & 255))) return HGRN2_ERR_WORKSPACE;
    if (launch_hgrn1_fwd(B, N, d, gate_dtype == HGRN2_BF16, f, i, o, act ? beta : nullptr, h0, y, hN, workspace,
                         static_cast<hipStream_t>(hip_stream)) != hipSuccess)
        return HGRN2_ERR_HIP;
    return HGRN2_OK;
}

static int h1_bwd_impl(int32_t B, int32_t N, int32_t d, int32_t io_dtype, int32_t gate_dtype, const void* f,
                       const void* i, const void* o, const float* beta, bool act, const float* h0, const void* grad_y,
                       const float* grad_hN, void* grad_f, void* grad_i, void* grad_o, float* grad_beta,
                       float* grad_h0, void* workspace, size_t workspace_bytes, void* hip_stream, bool states_saved = false)
{
    const int rc = h1_check(B, N, d, io_dtype, gate_dtype);
    if (rc != HGRN2_OK) return rc;
    const bool has_tokens = (size_t)B * N * d > 0;
    if (has_tokens && (!f || !i || !o || !grad_y || !grad_f || !grad_i || !grad_o || (act && !beta)))
        return HGRN2_ERR_NULL;
    if (act && d > 0 && !grad_beta) return HGRN2_ERR_NULL;
    const size_t need = round256(hgrn1_ws_bytes(B, N, d));
    if (need > 0 && (!workspace || workspace_bytes < need || ((uintptr_t)workspace & 255))) return HGRN2_ERR_WORKSPACE;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if (act && !has_tokens && d > 0) {        // nothing contributes: the gradient of beta is zero
        if (launch_zero_floats(grad_beta, (size_t)d, stream) != hipSuccess) return HGRN2_ERR_HIP;
    }
    if (launch_hgrn1_bwd(B, N, d, gate_dtype == HGRN2_BF16, f, i, o, act ? beta : nullptr, h0, grad_y, grad_hN, grad_f,
                         grad_i, grad_o, act && has_tokens ? grad_beta : nullptr, grad_h0, workspace, states_saved, stream) != hipSuccess)
        return HGRN2_ERR_HIP;
    return HGRN2_OK;
}

int hgrn1_fwd(int32_t B, int32_t N, int32_t d, int32_t io_dtype, int32_t gate_dtype, const void* f,
              const void* i, const void* o, const float* h0, void* y, float* hN, void* workspace,
              size_t workspace_bytes, void* hip_stream)
{
    return h1_fwd_impl(B, N, d, io_dtype, gate_dtype, f, i, o, nullptr, false, h0, y, hN, workspace, workspace_bytes,
                       hip_stream);
}

int hgrn1_bwd(int32_t B, int32_t N, int32_t d, int32_t io_dtype, int32_t gate_dtype, const void* f,
              const void* i, const void* o, const float* h0, const void* grad_y, const float* grad_hN,
              void* grad_f, void* grad_i, void* grad_o, float* grad_h0, void* workspace, size_t workspace_bytes,
              void* hip_stream)
{
    return h1_bwd_impl(B, N, d, io_dtype, gate_dtype, f, i, o, nullptr, false, h0, grad_y, grad_hN, grad_f, grad_i,
                       grad_o, nullptr, grad_h0, workspace, workspace_bytes, hip_stream);
}

int hgrn1_fwd_act(int32_t B, int32_t N, int32_t d, int32_t io_dtype, int32_t gate_dtype, const void* zf,
                  const void* zi, const void* zo, const float* beta, const float* h0, void* y, float* hN,
                  void* workspace, size_t workspace_bytes, void* hip_stream)
{
    return h1_fwd_impl(B, N, d, io_dtype, gate_dtype, zf, zi, zo, beta, true, h0, y, hN, workspace, workspace_bytes,
                       hip_stream);
}

int hgrn1_bwd_act(int32_t B, int32_t N, int32_t d, int32_t io_dtype, int32_t gate_dtype, const void* zf,
                  const void* zi, const void* zo, const float* beta, const float* h0, const void* grad_y,
                  const float* grad_hN, void* grad_zf, void* grad_zi, void* grad_zo, float* grad_beta,
                  float* grad_h0, void* workspace, size_t workspace_bytes, void* hip_stream)
{
    return h1_bwd_impl(B, N, d, io_dtype, gate_dtype, zf, zi, zo, beta, true, h0, grad_y, grad_hN, grad_zf, grad_zi,
                       grad_zo, grad_beta, grad_h0, workspace, workspace_bytes, hip_stream);
}

int hgrn1_bwd_saved(int32_t B, int32_t N, int32_t d, int32_t io_dtype, int32_t gate_dtype, const void* f,
                    const void* i, const void* o, const float* h0, const void* grad_y, const float* grad_hN,
                    void* grad_f, void* grad_i, void* grad_o, float* grad_h0, void* workspace, size_t workspace_bytes,
                    void* hip_stream)
{
    return h1_bwd_impl(B, N, d, io_dtype, gate_dtype, f, i, o, nullptr, false, h0, grad_y, grad_hN, grad_f, grad_i,
                       grad_o, nullptr, grad_h0, workspace, workspace_bytes, hip_stream, true);
}

int hgrn1_bwd_act_saved(int32_t B, int32_t N, int32_t d, int32_t io_dtype, int32_t gate_dtype, const void* zf,
                        const void* zi, const void* zo, const float* beta, const float* h0, const void* grad_y,
                        const float* grad_hN, void* grad_zf, void* grad_zi, void* grad_zo, float* grad_beta,
                        float* grad_h0, void* workspace, size_t workspace_bytes, void* hip_stream)
{
    return h1_bwd_impl(B, N, d, io_dtype, gate_dtype, zf, zi, zo, beta, true, h0, grad_y, grad_hN, grad_zf, grad_zi,
                       grad_zo, grad_beta, grad_h0, workspace, workspace_bytes, hip_stream, true);
}

const char* hgrn2_status_string(int status)
{
    switch (status) {
    case HGRN2_OK: return "ok";
    case HGRN2_ERR_NULL: return "a required pointer is NULL";
    case HGRN2_ERR_SHAPE: return "invalid shape or dtype";
    case HGRN2_ERR_UNSUPPORTED: return "shape, chunk or dtype outside the supported set";
    case HGRN2_ERR_WORKSPACE: return "workspace missing, too small or misaligned (or the shape needs more than the built-in scratch array holds)";
    case HGRN2_ERR_HIP: return "HIP launch error";
    default: return "unknown status";
    }
}

}   // extern "C"
