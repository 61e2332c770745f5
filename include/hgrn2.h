/*
 * hgrn2.h -- C ABI of the MI355X (gfx950) HGRN2 recurrence library.
 *
 * The operation is the multi-head HGRN2 recurrence of the paper (Section 3.2, Eq. 3, and the
 * "Multihead Variant" paragraph), in the query/key/value naming of its Table 4:
 *
 *     S_t = Diag(f_t) S_{t-1} + k_t^T v_t ,   k_t = 1 - f_t ,        S_t in R^{dk x dv}
 *     o_t = q_t S_t                                                   (reads the UPDATED state)
 *
 * where q is the paper's output gate, f the (lower-bounded) forget gate, v the input vector and
 * the input gate (key) is tied to the forget gate.  S is the transpose of the paper's h.  No
 * scaling of q, no output gate and no normalisation are applied (Table 4 omits GLA's output gate).
 * Every (batch, head) pair is an independent recurrence.
 *
 * Conventions common to all entry points
 *   - All tensor pointers are DEVICE pointers to dense row-major arrays, last index fastest:
 *         q, f, grad_q, grad_f : [B][H][N][dk]
 *         v, o, grad_o, grad_v : [B][H][N][dv]
 *         h0, hT, grad_h0, grad_hT, state : [B][H][dk][dv], always fp32
 *     q, v, o and all grad_* sequence tensors have element type `io_dtype`; f has `gate_dtype`.
 *   - The caller owns every buffer, including the workspace.  The library never allocates,
 *     frees or retains device memory and keeps no state between calls.
 *   - Work is enqueued on the caller's HIP stream (`hip_stream` is a hipStream_t, NULL = the
 *     default stream).  No entry point synchronises with the host.
 *   - Return value: an hgrn2_status.  Argument errors (every status but HGRN2_ERR_HIP) are
 *     detected on the host before anything is launched: nothing has been enqueued then.
 *     HGRN2_ERR_HIP reports a failed launch; earlier kernels of the same call may have been
 *     enqueued.  Nothing throws or aborts across the ABI.
 *   - Gate domain: f in [0, 1].  The chunkwise kernels factor the decay between two tokens of a
 *     chunk around the chunk's middle row, which needs the reciprocal of a product of up to 32
 *     consecutive gates of one channel.  Results are exact (up to rounding) while every such
 *     product stays above 2^-100 -- guaranteed for f >= 0.12 and true by a wide margin for
 *     sigmoid-type gates.  Below that the reciprocal is taken of 2^-100 instead: everything stays
 *     finite, but the affected chunks' outputs and gradients are WRONG (by up to 100%), and the
 *     call still returns HGRN2_OK -- the host cannot know the gates.  Two ways to know:
 *     shape->gate_domain_flag (a device int the kernels set when it happens, at no cost), and
 *     hgrn2_min_gate_product (a probe that reads the gates once, before the call).  grad_f also
 *     divides by f itself (floored at 1e-30): at f = 0 exactly it is not meaningful.
 *     Small-gate modes: with chunk = 32 or 16, hgrn2_fwd, hgrn2_bwd and their _gated and
 *     _varlen forms place their reference rows every 32 or 16 tokens instead of every 64, and
 *     the bound applies to the product of 16 or 8 consecutive gates (guaranteed for
 *     f >= 0.014, f >= 1.8e-4).  A chunk of the kernels then holds 32 or 16 tokens in its middle
 *     rows and nothing in the others: twice or four times the chunks (1.8 or 3.6 times the time
 *     of the training pair, and workspaces and saved states for as many chunks; the training
 *     pair hgrn2_fwd_saving / hgrn2_bwd_saved takes the modes as well).  chunk = 8 goes one
 *     step further (products of 4 gates: f >= 3e-8, eight times the chunks).  Packed batches
 *     (_varlen, with their training pair) take the three modes the same way.
 *     hgrn2_min_gate_product tells which mode a set of gates needs.
 *     chunk = HGRN2_CHUNK_AUTO (hgrn2_fwd, hgrn2_bwd, their _gated, _saving / _saved, _noalloc and
 *     _varlen forms) needs no probe: the pass is enqueued for 64, then 32, then 16 tokens
 *     per chunk; the kernels of the first raise a flag inside the workspace when a product falls
 *     below the floor, those of the next run only if it is set (they return at once otherwise) and
 *     overwrite every result, and so on.  The results are those of the longest chunk the gates
 *     allow; shape->gate_domain_flag is raised only when even 16 tokens per chunk are too many.
 *     Ordinary gates pay the launches that do nothing (about ten microseconds per pass); the
 *     workspaces and saved states are sized for 16 tokens per chunk (the saved states of a packed
 *     batch: for all three chunk lengths, one after the other).
 *   - Supported shapes: dk, dv in {64, 128}; chunk in {0 (= 64), 64}, and 32, 16, 8, HGRN2_CHUNK_AUTO where stated;
 *     any B, H, N >= 0.
 *     A sequence length that is not a multiple of the chunk is handled inside the kernels.
 *     io_dtype F32 is supported by hgrn2_fwd, hgrn2_step and, for heads of dk = dv = 64, by hgrn2_bwd
 *     and its gated / saving forms (the same kernels with fp32 tiles and fp32 matrix instructions:
 *     the fp32 tiles of wider heads exceed the LDS); packed batches and the chunk-gradient stage
 *     call are BF16-only in the backward direction.
 */
#ifndef HGRN2_H
#define HGRN2_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    HGRN2_OK = 0,
    HGRN2_ERR_NULL = 1,        /* a required pointer is NULL */
    HGRN2_ERR_SHAPE = 2,       /* negative or zero size, or a size product that overflows */
    HGRN2_ERR_UNSUPPORTED = 3, /* well-formed but outside the supported set listed above */
    HGRN2_ERR_WORKSPACE = 4,   /* workspace missing, too small or not 256-byte aligned */
    HGRN2_ERR_HIP = 5          /* a HIP call or kernel launch reported an error */
} hgrn2_status;

typedef enum { HGRN2_F32 = 0, HGRN2_BF16 = 1 } hgrn2_dtype;
/* hgrn2_shape::chunk value that lets the device choose the chunk length (see "Gate domain" above) */
#define HGRN2_CHUNK_AUTO (-1)

/* Memory order of the sequence tensors.  The d channels of one token of one head are always
 * contiguous; HGRN2_LAYOUT_BNHD is what a projection of a [B][N][model width] activation writes
 * (heads side by side inside a token), so no transposition is needed before or after the call.
 * States (h0, hT, their gradients, the decode state) are [B][H][dk][dv] in either case. */
typedef enum { HGRN2_LAYOUT_BHND = 0, HGRN2_LAYOUT_BNHD = 1 } hgrn2_layout;

typedef struct {
    int32_t B, H, N, dk, dv;
    int32_t chunk;      /* tokens per chunk of the chunkwise algorithm: 0 selects the default (64); 32, 16, 8 and
                           HGRN2_CHUNK_AUTO where stated (see "Gate domain" above) */
    int32_t io_dtype;   /* hgrn2_dtype of q, v, o and of every grad_* sequence tensor */
    int32_t gate_dtype; /* hgrn2_dtype of f (grad_f follows io_dtype) */
    int32_t layout;     /* hgrn2_layout of every sequence tensor (q, f, v, o, grad_*); 0 = [B][H][N][d] */
    int32_t* gate_domain_flag; /* NULL, or a DEVICE int32 that the forward / backward kernels set to 1 when
                           the gates of the call leave the gate domain described above (they never
                           clear it: the caller zeroes it, and reads it after the stream has finished) */
} hgrn2_shape;

/* Bytes of device workspace hgrn2_fwd / hgrn2_bwd need for this shape (0 if the shape is
 * invalid or unsupported; the corresponding call then reports the precise error). */
size_t hgrn2_fwd_workspace_bytes(const hgrn2_shape* shape);
size_t hgrn2_bwd_workspace_bytes(const hgrn2_shape* shape);

/*
 * Chunkwise-parallel forward pass of Eq. 3 over whole sequences (the "hardware-efficient
 * training" form the paper refers to in Section 3.2: an exact regrouping of the recurrence
 * into per-chunk matrix products plus a chunk-to-chunk state recurrence).
 *   q, f, v   in   device, read-only
 *   h0        in   device fp32 [B][H][dk][dv], or NULL for a zero initial state
 *   o         out  device [B][H][N][dv], io_dtype
 *   hT        out  device fp32 [B][H][dk][dv] final state S_N, or NULL if not wanted
 *   workspace      device scratch of at least hgrn2_fwd_workspace_bytes(shape) bytes, 256-byte
 *                  aligned; contents on entry are ignored, contents on return are unspecified
 */
int hgrn2_fwd(const hgrn2_shape* shape, const void* q, const void* f, const void* v,
              const float* h0, void* o, float* hT, void* workspace, size_t workspace_bytes,
              void* hip_stream);

/*
 * Backward pass of hgrn2_fwd: gradients of L = sum(o * grad_o) + sum(hT * grad_hT).
 * Stateless: everything needed is recomputed from q, f, v, h0.  The paper gives no backward
 * algorithm; this is reverse-mode differentiation of Eq. 3 in chunkwise form.
 *   grad_o    in   device [B][H][N][dv], io_dtype
 *   grad_hT   in   device fp32 [B][H][dk][dv], or NULL for zero
 *   grad_q, grad_f, grad_v   out  device, io_dtype.  grad_f is the gradient w.r.t. the gate f
 *             INCLUDING the tied path k = 1 - f, so callers never see k or its gradient.
 *   grad_h0   out  device fp32 [B][H][dk][dv], or NULL if not wanted
 *   workspace as for hgrn2_fwd, sized by hgrn2_bwd_workspace_bytes(shape)
 */
int hgrn2_bwd(const hgrn2_shape* shape, const void* q, const void* f, const void* v,
              const float* h0, const void* grad_o, const float* grad_hT, void* grad_q,
              void* grad_f, void* grad_v, float* grad_h0, void* workspace, size_t workspace_bytes,
              void* hip_stream);

/*
 * Single-token recurrent (decode) step: one application of Eq. 3 per (batch, head).
 *   q_t, f_t  in   device [B][H][dk]        v_t  in   device [B][H][dv]
 *   state     in/out device fp32 [B][H][dk][dv], updated IN PLACE to S_t
 *   o_t       out  device [B][H][dv], io_dtype; computed from the updated state
 * Needs no workspace.
 */
int hgrn2_step(int32_t B, int32_t H, int32_t dk, int32_t dv, int32_t io_dtype, int32_t gate_dtype,
               const void* q_t, const void* f_t, const void* v_t, float* state, void* o_t,
               void* hip_stream);

/*
 * The same passes with the lower-bounded forget gate of the paper's Section 2, Eq. 2, formed
 * inside the kernels, so that the gate tensor itself is never written to memory:
 *     f = beta + (1 - beta) * sigmoid(z)
 *   z         in   device [B][H][N][dk], gate_dtype: pre-activation of the gate (takes the place of f)
 *   beta      in   device fp32 [H][dk]: lower bound of every channel of this layer, 0 <= beta < 1,
 *                  shared by batch and time
 *   grad_z    out  device [B][H][N][dk], io_dtype: gradient w.r.t. z, tied path k = 1 - f included
 *   grad_beta out  device fp32 [H][dk]: gradient w.r.t. beta, summed over batch and time in a fixed
 *                  order (bit-reproducible)
 * Everything else as for hgrn2_fwd / hgrn2_bwd; the backward workspace is sized by
 * hgrn2_bwd_gated_workspace_bytes(shape), the forward one by hgrn2_fwd_workspace_bytes(shape).
 */
size_t hgrn2_bwd_gated_workspace_bytes(const hgrn2_shape* shape);
int hgrn2_fwd_gated(const hgrn2_shape* shape, const void* q, const void* z, const float* beta,
                    const void* v, const float* h0, void* o, float* hT, void* workspace,
                    size_t workspace_bytes, void* hip_stream);
int hgrn2_bwd_gated(const hgrn2_shape* shape, const void* q, const void* z, const float* beta,
                    const void* v, const float* h0, const void* grad_o, const float* grad_hT,
                    void* grad_q, void* grad_z, float* grad_beta, void* grad_v, float* grad_h0,
                    void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Training pair.  The backward pass needs the state S_n entering every chunk of 64 tokens (the
 * chunkwise regrouping of Eq. 3, Section 3.2).  hgrn2_bwd recomputes them with a sweep over f and v;
 * a caller that runs the forward pass of the same step anyway can have it keep them instead:
 * hgrn2_fwd_saving is hgrn2_fwd (beta == NULL) or hgrn2_fwd_gated (beta given: `f` holds the
 * pre-activations z of Eq. 2) that also fills `saved_states`, and hgrn2_bwd_saved is hgrn2_bwd /
 * hgrn2_bwd_gated that reads them and runs no sweep of its own.
 *   saved_states   device, hgrn2_saved_states_bytes(shape) bytes (2 dk dv bytes per chunk and
 *                  (batch, head): bf16, in a private order), 256-byte aligned.  Valid for the very
 *                  q, f (or z, beta), v, h0 and shape of the forward call that wrote it.
 *   workspace      hgrn2_fwd_workspace_bytes(shape) for the forward call,
 *                  hgrn2_bwd_saved_workspace_bytes(shape, gated) for the backward call
 *   grad_beta      required when beta is given, ignored otherwise
 * BF16 storage (fp32 for heads of 64 x 64), equal-length batches in either layout; other arguments, results
 * (those of the stateless calls up to the rounding of the states), status codes and stream
 * semantics as above.
 */
size_t hgrn2_saved_states_bytes(const hgrn2_shape* shape);
size_t hgrn2_bwd_saved_workspace_bytes(const hgrn2_shape* shape, int32_t gated);
int hgrn2_fwd_saving(const hgrn2_shape* shape, const void* q, const void* f, const float* beta, const void* v,
                     const float* h0, void* o, float* hT, void* saved_states, size_t saved_states_bytes,
                     void* workspace, size_t workspace_bytes, void* hip_stream);
int hgrn2_bwd_saved(const hgrn2_shape* shape, const void* q, const void* f, const float* beta, const void* v,
                    const void* saved_states, size_t saved_states_bytes, const void* grad_o,
                    const float* grad_hT, void* grad_q, void* grad_f, float* grad_beta, void* grad_v,
                    float* grad_h0, void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Lower bounds of all L layers from the learnable matrix Gamma (Section 2): softmax over the layer
 * axis, cumulative sum over the layer axis, minus the first layer's row, so that the bounds rise
 * monotonically from zero in the first layer and stay below one in the last.
 *   gamma     in   device fp32 [L][d]        beta  out  device fp32 [L][d]
 * (row l of beta, viewed as [H][dk], is the `beta` argument of layer l above).  Needs no workspace.
 */
int hgrn2_cumax(int32_t L, int32_t d, const float* gamma, float* beta, void* hip_stream);

/*
 * Decode step with the gate of Eq. 2 formed inside the kernel: z_t [B][H][dk] (gate_dtype) holds
 * the pre-activations of this token's forget gate, beta [H][dk] fp32 the layer's lower bounds.
 * Everything else as for hgrn2_step.
 */
int hgrn2_step_gated(int32_t B, int32_t H, int32_t dk, int32_t dv, int32_t io_dtype, int32_t gate_dtype,
                     const void* q_t, const void* z_t, const float* beta, const void* v_t, float* state, void* o_t,
                     void* hip_stream);

/*
 * Gate-domain probe for the contract stated at the top ("Gate domain"): writes to *min_product
 * (device, one float) the smallest product of the gates of one channel over a half chunk -- tokens
 * [64 n, 64 n + 32) and [64 n + 32, 64 n + 64) of every sequence, n = 0, 1, ... -- of the whole
 * call.  hgrn2_fwd / hgrn2_bwd are exact up to rounding while it is above 2^-100 (7.9e-31).
 * With shape->chunk = 32 or 16 the products are those that small-gate mode depends on: over
 * tokens [16 m, 16 m + 16) or [8 m, 8 m + 8) of every sequence.
 * Reads f once; equal-length batches in either layout; with beta (device fp32 [H][dk]) `f` holds
 * pre-activations and the gate of Eq. 2 is formed first.  An empty call writes 1.
 */
int hgrn2_min_gate_product(const hgrn2_shape* shape, const void* f, const float* beta, float* min_product,
                           void* hip_stream);

/*
 * Variable-length batches: shape->B sequences of different lengths packed back to back along the
 * token axis, as training on packed documents and serving ragged prefill batches produce them.
 * The recurrence of Eq. 3 (Section 3.2) restarts at every sequence boundary: sequence b starts
 * from its own h0[b] (zero if NULL) and ends in its own hT[b].
 *   shape           B = number of sequences, N = T = total number of tokens of all sequences,
 *                   layout = HGRN2_LAYOUT_BNHD (else HGRN2_ERR_SHAPE); other fields as above
 *   cu_seqlens  in  device int32 [B + 1]: sequence b owns tokens cu_seqlens[b] ..
 *                   cu_seqlens[b + 1] - 1 (cu_seqlens[0] = 0, cu_seqlens[B] = T; empty sequences
 *                   are fine).  The array is read on the device only; it is not validated, but
 *                   offsets are clamped to [0, T] and made non-decreasing first, so a wrong array
 *                   gives wrong results and never an access outside the tensors.
 *   q, f, v, o, grad_*   device [T][H][d]    h0, hT, grad_hT, grad_h0   device fp32 [B][H][dk][dv]
 *   workspace       hgrn2_fwd_varlen_workspace_bytes / hgrn2_bwd_varlen_workspace_bytes bytes
 *                   (sized for the worst split of the T tokens into B sequences), 256-byte aligned
 *   beta            NULL: `f` holds the gates.  Else device fp32 [H][dk], the layer's lower bounds:
 *                   `f` then holds the gates' pre-activations z and the gate of Eq. 2 is formed in the
 *                   kernels, grad_f receives dL/dz and grad_beta (device fp32 [H][dk], required then)
 *                   dL/dbeta, as for hgrn2_fwd_gated / hgrn2_bwd_gated.
 * Same status codes, stream semantics and numerical contract as hgrn2_fwd / hgrn2_bwd.
 */
size_t hgrn2_fwd_varlen_workspace_bytes(const hgrn2_shape* shape);
size_t hgrn2_bwd_varlen_workspace_bytes(const hgrn2_shape* shape);
int hgrn2_fwd_varlen(const hgrn2_shape* shape, const int32_t* cu_seqlens, const void* q, const void* f,
                     const float* beta, const void* v, const float* h0, void* o, float* hT, void* workspace,
                     size_t workspace_bytes, void* hip_stream);
int hgrn2_bwd_varlen(const hgrn2_shape* shape, const int32_t* cu_seqlens, const void* q, const void* f,
                     const float* beta, const void* v, const float* h0, const void* grad_o, const float* grad_hT,
                     void* grad_q, void* grad_f, float* grad_beta, void* grad_v, float* grad_h0, void* workspace,
                     size_t workspace_bytes, void* hip_stream);

/*
 * Training pair for packed batches (the chunk states of Eq. 3's chunkwise regrouping, Section 3.2,
 * kept by the forward pass of a step for its backward pass; see hgrn2_fwd_saving above):
 * hgrn2_fwd_varlen_saving is hgrn2_fwd_varlen that also fills `saved_states`, and
 * hgrn2_bwd_varlen_saved is hgrn2_bwd_varlen that reads them instead of running a sweep over f and
 * v of its own.
 *   saved_states   device, hgrn2_saved_states_varlen_bytes(shape) bytes (the chunk states, sized
 *                  like the workspaces for the worst split of the T tokens, and the tables made
 *                  from cu_seqlens, which the backward call then does not build again), 256-byte
 *                  aligned.  Valid for the very cu_seqlens, q, f (or z, beta), v, h0 and shape of
 *                  the forward call.
 *   h0             both calls take the one initial state array.  A batch of few long sequences is
 *                  cut into runs, and for some shapes only by the forward pass: nothing is kept
 *                  then (the shape alone decides, so both calls agree) and the backward call
 *                  recomputes the states, from h0, as hgrn2_bwd_varlen does.
 *   workspace      hgrn2_fwd_varlen_workspace_bytes(shape) / hgrn2_bwd_varlen_workspace_bytes(shape)
 * BF16 storage, chunk = 0 or 64 (HGRN2_ERR_UNSUPPORTED otherwise); other arguments, results (those
 * of the stateless calls up to the rounding of the states), status codes and stream semantics as
 * for hgrn2_fwd_varlen / hgrn2_bwd_varlen.
 */
size_t hgrn2_saved_states_varlen_bytes(const hgrn2_shape* shape);
int hgrn2_fwd_varlen_saving(const hgrn2_shape* shape, const int32_t* cu_seqlens, const void* q, const void* f,
                            const float* beta, const void* v, const float* h0, void* o, float* hT, void* saved_states,
                            size_t saved_states_bytes, void* workspace, size_t workspace_bytes, void* hip_stream);
int hgrn2_bwd_varlen_saved(const hgrn2_shape* shape, const int32_t* cu_seqlens, const void* q, const void* f,
                           const float* beta, const void* v, const float* h0, const void* saved_states,
                           size_t saved_states_bytes, const void* grad_o, const float* grad_hT, void* grad_q, void* grad_f,
                           float* grad_beta, void* grad_v, float* grad_h0, void* workspace, size_t workspace_bytes,
                           void* hip_stream);

/*
 * hgrn2_min_gate_product for a packed batch: the windows (half chunks: 32 tokens; 16 or 8 with
 * shape->chunk = 32 or 16) start anew with every sequence, as they do inside hgrn2_fwd_varlen /
 * hgrn2_bwd_varlen.  f (or the pre-activations, with beta) is [T][H][dk]; the workspace of
 * hgrn2_min_gate_product_varlen_workspace_bytes(shape) bytes holds the sequence table.
 */
size_t hgrn2_min_gate_product_varlen_workspace_bytes(const hgrn2_shape* shape);
int hgrn2_min_gate_product_varlen(const hgrn2_shape* shape, const int32_t* cu_seqlens, const void* f, const float* beta,
                                  float* min_product, void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * HGRN1, the element-wise gated linear recurrence the paper starts from (Section 2, Eq. 1, with the
 * forget gate f of Eq. 2 given), per channel:
 *     h_t = f_t * h_{t-1} + (1 - f_t) * i_t,      y_t = h_t * o_t
 * and its reverse mode for L = sum(y * grad_y) + sum(h_N * grad_hN).  A second, bandwidth-bound
 * workload beside the state-expanded recurrence above (which reduces to it for a 1 x 1 state).
 *   f, i, o, y, grad_*   device [B][N][d], io_dtype (bf16 only; f may be fp32 via gate_dtype);
 *                        d a multiple of 64
 *   h0, grad_hN     in   device fp32 [B][d], or NULL for zero
 *   hN, grad_h0     out  device fp32 [B][d], or NULL if not wanted
 *   grad_f          out  includes the tied input gate 1 - f
 *   workspace            device scratch of hgrn1_workspace_bytes(B, N, d) bytes, 256-byte aligned
 * Status codes as above; hgrn2_status_string() describes them.
 */
size_t hgrn1_workspace_bytes(int32_t B, int32_t N, int32_t d);
int hgrn1_fwd(int32_t B, int32_t N, int32_t d, int32_t io_dtype, int32_t gate_dtype, const void* f,
              const void* i, const void* o, const float* h0, void* y, float* hN, void* workspace,
              size_t workspace_bytes, void* hip_stream);
int hgrn1_bwd(int32_t B, int32_t N, int32_t d, int32_t io_dtype, int32_t gate_dtype, const void* f,
              const void* i, const void* o, const float* h0, const void* grad_y, const float* grad_hN,
              void* grad_f, void* grad_i, void* grad_o, float* grad_h0, void* workspace,
              size_t workspace_bytes, void* hip_stream);

/*
 * The same recurrence taken from the pre-activations of Eq. 1 (Section 2), i.e. from what the
 * layer's three projections (biases included) write, with the forget gate's lower bound of Eq. 2:
 *     f = beta + (1 - beta) * sigmoid(zf),   i = SiLU(zi),   o = sigmoid(zo)
 * formed inside the kernels, so that f, i and o never reach memory.
 *   zf, zi, zo      in   device [B][N][d] (zf in gate_dtype, the others bf16)
 *   beta            in   device fp32 [d]: the layer's lower bounds, each in [0, 1) (hgrn2_cumax)
 *   grad_zf, grad_zi, grad_zo   out  device [B][N][d] bf16
 *   grad_beta       out  device fp32 [d], summed over batch and time in a fixed order
 * Everything else (states, workspace, status codes) as for hgrn1_fwd / hgrn1_bwd.
 */
int hgrn1_fwd_act(int32_t B, int32_t N, int32_t d, int32_t io_dtype, int32_t gate_dtype, const void* zf,
                  const void* zi, const void* zo, const float* beta, const float* h0, void* y, float* hN,
                  void* workspace, size_t workspace_bytes, void* hip_stream);
int hgrn1_bwd_act(int32_t B, int32_t N, int32_t d, int32_t io_dtype, int32_t gate_dtype, const void* zf,
                  const void* zi, const void* zo, const float* beta, const float* h0, const void* grad_y,
                  const float* grad_hN, void* grad_zf, void* grad_zi, void* grad_zo, float* grad_beta,
                  float* grad_h0, void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * The backward passes of a training step whose forward pass has just run: hgrn1_fwd / hgrn1_fwd_act
 * leave the state entering every 16-token segment of every sequence in their workspace (a few MB;
 * the reverse mode of Eq. 1 needs h_{t-1} at every token), and hgrn1_bwd_saved / hgrn1_bwd_act_saved
 * are hgrn1_bwd / hgrn1_bwd_act that read them there instead of walking f and i forwards once more.
 * The workspace must be the one the forward call of the same B, N, d, inputs and h0 was given, untouched
 * since (hgrn1_bwd / hgrn1_bwd_act overwrite it); everything else as for the calls above.
 */
int hgrn1_bwd_saved(int32_t B, int32_t N, int32_t d, int32_t io_dtype, int32_t gate_dtype, const void* f,
                    const void* i, const void* o, const float* h0, const void* grad_y, const float* grad_hN,
                    void* grad_f, void* grad_i, void* grad_o, float* grad_h0, void* workspace, size_t workspace_bytes,
                    void* hip_stream);
int hgrn1_bwd_act_saved(int32_t B, int32_t N, int32_t d, int32_t io_dtype, int32_t gate_dtype, const void* zf,
                        const void* zi, const void* zo, const float* beta, const float* h0, const void* grad_y,
                        const float* grad_hN, void* grad_zf, void* grad_zi, void* grad_zo, float* grad_beta,
                        float* grad_h0, void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Stage entry points.  hgrn2_fwd is hgrn2_state_sweep(HGRN2_SWEEP_STATE_FWD) followed by
 * hgrn2_fwd_readout; hgrn2_bwd is hgrn2_state_sweep(HGRN2_SWEEP_STATE_BWD), then
 * hgrn2_state_sweep(HGRN2_SWEEP_STATE_GRAD), then hgrn2_bwd_chunk_grads.  They exist for callers
 * that time or schedule the stages themselves (e.g. overlap the two backward sweeps on two
 * streams).  All follow from regrouping Eq. 3 (Section 3.2) into chunks of 64 tokens:
 *   state sweep      S_{n+1} = Diag(g_n) S_n + K^_n^T V_n   (or its transpose-gradient
 *                    dS_n = Diag(g_n) dS_{n+1} + Q^_n^T dO_n, walking the chunks backwards);
 *   forward read-out o = tril(Q~ K~^T) V + (q G) S_n per chunk;
 *   chunk gradients  grad_q, grad_f, grad_v per chunk from S_n and dS_{n+1}.
 * `chunk_states` buffers are device memory of hgrn2_fwd_workspace_bytes(shape) bytes, 256-byte
 * aligned, in a private MFMA-fragment order that depends on the sweep mode: a buffer written
 * in one mode may only be consumed by the stage that expects that mode.
 *   hgrn2_state_sweep: b_src is v (STATE_FWD, STATE_BWD) or grad_o (STATE_GRAD); q is read only
 *     in STATE_GRAD; init_state is h0 (or grad_hT), may be NULL = 0; final_state receives hT
 *     (or grad_h0), may be NULL.
 * A stage call walks every sequence in one piece; hgrn2_fwd / hgrn2_bwd cut few, long sequences
 * into runs that are walked at the same time (same results up to fp32 summation order), which is
 * why their workspaces can be larger than the chunk_states buffers here.
 */
typedef enum { HGRN2_SWEEP_STATE_FWD = 0, HGRN2_SWEEP_STATE_BWD = 1, HGRN2_SWEEP_STATE_GRAD = 2 } hgrn2_sweep_mode;

int hgrn2_state_sweep(const hgrn2_shape* shape, int32_t mode, const void* q, const void* f, const void* b_src,
                      const float* init_state, float* final_state, void* chunk_states,
                      size_t chunk_states_bytes, void* hip_stream);
int hgrn2_fwd_readout(const hgrn2_shape* shape, const void* q, const void* f, const void* v,
                      const void* chunk_states /* STATE_FWD */, void* o, void* hip_stream);
int hgrn2_bwd_chunk_grads(const hgrn2_shape* shape, const void* q, const void* f, const void* v,
                          const void* grad_o, const void* chunk_states /* STATE_BWD */,
                          const void* chunk_state_grads /* STATE_GRAD */, void* grad_q, void* grad_f,
                          void* grad_v, void* hip_stream);

/*
 * hgrn2_bwd for callers that cannot allocate device memory or pass a workspace: code that runs
 * under HIP graph capture, tight serving or training loops, harnesses that forbid hipMalloc.  The
 * call allocates nothing; its workspace is a fixed array of hgrn2_noalloc_workspace_limit() bytes
 * (32 MiB) of device memory that is part of the library itself (every GPU the library is used on
 * holds its own copy until the process ends).  Arguments, results and status codes are those of
 * hgrn2_bwd; a shape whose hgrn2_bwd_workspace_bytes exceeds the limit returns
 * HGRN2_ERR_WORKSPACE before anything is launched.  The array is shared by all calls on a GPU
 * and keeps the last call's contents (the kernels write every part of it before they read it):
 * two such calls that overlap in time on one GPU, e.g. on two streams, race.
 * hgrn2_noalloc_init() looks up the array's address on the current device (the entry point does
 * so itself on its first call on a device; a caller that captures graphs calls it, or the entry
 * point, once beforehand).
 */
size_t hgrn2_noalloc_workspace_limit(void);
int hgrn2_noalloc_init(void);
int hgrn2_bwd_noalloc(const hgrn2_shape* shape, const void* q, const void* f, const void* v,
                      const float* h0, const void* grad_o, const float* grad_hT, void* grad_q,
                      void* grad_f, void* grad_v, float* grad_h0, void* hip_stream);

/*
 * Input side of the HGRU2 token mixer (Section 2, Eq. 1, feeding Eq. 2 and Eq. 3): the three
 * projections of the layer input x_t and their activations, as one bf16 matrix product with bias
 * and activation applied to the fp32 accumulators,
 *     z = U x + b_u              pre-activation of the forget gate (Eq. 2 is formed inside
 *                                hgrn2_fwd_gated and its relatives, which take z and beta),
 *     v = SiLU(V x + b_v)        the paper's input vector i,
 *     q = sigmoid(W x + b_w)     the paper's output gate o.
 * The outputs are token-major [M][d] = [B][N][H][d/H], the layout HGRN2_LAYOUT_BNHD names, so
 * projection -> recurrence needs no transposition and neither the gate nor the pre-activation of q
 * reaches memory.  (What follows the recurrence in the block -- normalisation, output projection,
 * the GLU channel mixer -- is defined by the paper only through a figure and is not part of this
 * library.)
 *   M = B * N tokens; d the model width, a multiple of 256 (else HGRN2_ERR_UNSUPPORTED)
 *   x        in   device bf16 [M][d]
 *   w3       in   device bf16 [3 d][d]: the rows of U, then of V, then of W (row = output channel)
 *   b3       in   device fp32 [3 d]: b_u, b_v, b_w
 *   z, v, q  out  device bf16 [M][d]
 *   av       out  device bf16 [M][d] or NULL: V x + b_v, which the reverse mode needs (SiLU is not
 *                 invertible)
 * hgru2_proj_bwd: reverse mode for L = sum(z grad_z) + sum(v grad_v) + sum(q grad_q):
 *   grad_x   out  device bf16 [M][d]
 *   grad_w3  out  device fp32 [3 d][d];   grad_b3  out  device fp32 [3 d] (summed in a fixed order)
 *   workspace     hgru2_proj_bwd_workspace_bytes(M, d) bytes, 256-byte aligned
 * Status codes and stream semantics as everywhere in this header.
 */
size_t hgru2_proj_bwd_workspace_bytes(int32_t M, int32_t d);
int hgru2_proj_fwd(int32_t M, int32_t d, const void* x, const void* w3, const float* b3, void* z, void* v,
                   void* q, void* av, void* hip_stream);
int hgru2_proj_bwd(int32_t M, int32_t d, const void* x, const void* w3, const void* q, const void* av,
                   const void* grad_z, const void* grad_v, const void* grad_q, void* grad_x, float* grad_w3,
                   float* grad_b3, void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Measurement probes (no part of the method): what this GPU sustains for a plain copy and for a
 * loop of bf16 matrix instructions, the practical ceilings next to the published peaks of
 * mi355x_peaks.h that roofline fractions are quoted against.
 *   hgrn2_probe_copy   copies `bytes` (a multiple of 16; both pointers 16-byte aligned) from src to
 *                      dst on the device: 2 * bytes of traffic.
 *   hgrn2_probe_mfma   every wave of a grid that fills the chip issues `iters` rounds of four
 *                      independent 32x32x16 bf16 matrix instructions; *flops (host, may be NULL)
 *                      receives the number of floating-point operations of the launch; `out`
 *                      (device, hgrn2_probe_mfma_out_floats() floats) receives one sum per thread.
 */
int hgrn2_probe_copy(void* dst, const void* src, size_t bytes, void* hip_stream);
size_t hgrn2_probe_mfma_out_floats(void);
int hgrn2_probe_mfma(int32_t iters, float* out, double* flops, void* hip_stream);

/* Static, NUL-terminated description of a status code (never NULL). */
const char* hgrn2_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* HGRN2_H */
