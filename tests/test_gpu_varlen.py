"""GPU parity of the variable-length entry points (hgrn2_fwd_varlen, hgrn2_bwd_varlen, and the
training pair hgrn2_fwd_varlen_saving / hgrn2_bwd_varlen_saved on the same inputs): sequences
of different lengths packed along the token axis of [T][H][d] tensors, against the fp64 oracle run
on every sequence by itself.  The recurrence restarts at every boundary, so a token of one
sequence must not influence another: the oracle side never sees the packing.
Inputs: one seeded [1][H][T][d] draw of the usual recipe, cut at the boundaries.
Tolerance: max|x-y|/max|y| <= 2e-2 per tensor (bf16 storage), over the whole packed tensor."""
import numpy as np
import pytest
import torch

import oracle
from paper_2404_07904_amd import binding, synth
from gpu_util import TOL, check, dev, host

pytestmark = pytest.mark.gpu


def packed(x, dtype):
    """[1][H][T][d] host array -> [T][H][d] device tensor"""
    return dev(x, dtype)[0].permute(1, 0, 2).contiguous()


def unpacked(t):
    """[T][H][d] device tensor -> [H][T][d] host array"""
    return host(t.permute(1, 0, 2))


def states_buffer(q, v, f, n_seq):
    """Room for the states a forward pass keeps, filled with bytes that read as NaN: a state the
    backward pass reads without the forward pass having written it cannot go unnoticed."""
    shape = binding.make_shape_varlen(q, v, f, n_seq)
    return torch.full((binding.hgrn2_saved_states_varlen_bytes(shape),), 0xFF, dtype=torch.uint8, device=q.device)


def run(seed, lens, H, dk, dv, gate_dtype="bf16", lb=0.3, with_states=True, cu_override=None):
    lens = list(lens)
    B, T = len(lens), int(sum(lens))
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    w = synth.make_sequence(seed, 1, H, max(T, 1), dk, dv, io_dtype="bf16", gate_dtype=gate_dtype, lb=lb,
                            with_dO=True)
    rng = np.random.default_rng(seed + 1)
    h0 = rng.standard_normal((B, H, dk, dv)).astype(np.float32) if with_states else None
    dhT = (0.1 * rng.standard_normal((B, H, dk, dv))).astype(np.float32) if with_states else None
    wq, wf, wv, wd = (x[:, :, :T] for x in (w.q, w.f, w.v, w.dO))
    q, f, v, dO = packed(wq, "bf16"), packed(wf, gate_dtype), packed(wv, "bf16"), packed(wd, "bf16")
    cud = torch.from_numpy(cu if cu_override is None else np.asarray(cu_override, dtype=np.int32)).cuda()
    o, hT = binding.hgrn2_fwd_varlen(q, f, v, cud, dev(h0))
    gq, gf, gv, gh0 = binding.hgrn2_bwd_varlen(q, f, v, dO, cud, dev(h0), dev(dhT), want_grad_h0=True)
    # the same step as a training pair: the forward pass keeps the chunk states for the backward pass
    saved = states_buffer(q, v, f, B)
    o_s, hT_s = binding.hgrn2_fwd_varlen(q, f, v, cud, dev(h0), saved_states=saved)
    gq_s, gf_s, gv_s, gh0_s = binding.hgrn2_bwd_varlen(q, f, v, dO, cud, dev(h0), dev(dhT), want_grad_h0=True,
                                                       saved_states=saved)
    torch.cuda.synchronize()
    # oracle: every sequence on its own
    ro, rq, rf, rv = (np.zeros((H, T, d)) for d in (dv, dk, dk, dv))
    rhT, rh0 = np.zeros((B, H, dk, dv)), np.zeros((B, H, dk, dv))
    for b in range(B):
        s, e = int(cu[b]), int(cu[b + 1])
        sl = (slice(None), slice(None), slice(s, e))
        hb = None if h0 is None else h0[b:b + 1]
        db = None if dhT is None else dhT[b:b + 1]
        ob, hTb = oracle.fwd(wq[sl], wf[sl], wv[sl], hb)
        gqb, gfb, gvb, gh0b = oracle.bwd(wq[sl], wf[sl], wv[sl], wd[sl], hb, db)
        ro[:, s:e], rq[:, s:e], rf[:, s:e], rv[:, s:e] = ob[0], gqb[0], gfb[0], gvb[0]
        rhT[b], rh0[b] = hTb[0], gh0b[0]
    tol = TOL["bf16"]
    check("o", unpacked(o), ro, tol)
    check("hT", host(hT), rhT, tol)
    check("dq", unpacked(gq), rq, tol)
    check("dv", unpacked(gv), rv, tol)
    check("df", unpacked(gf), rf, tol)
    check("dh0", host(gh0), rh0, tol)
    check("o (pair)", unpacked(o_s), ro, tol)
    check("hT (pair)", host(hT_s), rhT, tol)
    check("dq (pair)", unpacked(gq_s), rq, tol)
    check("dv (pair)", unpacked(gv_s), rv, tol)
    check("df (pair)", unpacked(gf_s), rf, tol)
    check("dh0 (pair)", host(gh0_s), rh0, tol)


@pytest.mark.parametrize("dk,dv", [(64, 64), (128, 128), (64, 128), (128, 64)])
def test_varlen_mixed_lengths(dk, dv):
    lens = [70, 1, 64, 129, 5, 200]
    print("\n[varlen] dk=%d dv=%d H=3 lens=%s" % (dk, dv, lens), flush=True)
    run(6000 + dk + 2 * dv, lens, 3, dk, dv)


def test_varlen_empty_sequences_and_no_states():
    lens = [0, 37, 0, 0, 64, 1, 0]
    print("\n[varlen] empty sequences, lens=%s" % lens, flush=True)
    run(6100, lens, 2, 64, 64)
    run(6101, lens, 2, 128, 128, with_states=False)


def test_varlen_single_sequence_equals_fixed_length():
    print("\n[varlen] one sequence of 300 tokens", flush=True)
    run(6200, [300], 4, 128, 128)


@pytest.mark.parametrize("gate_dtype", ["bf16", "f32"])
def test_varlen_fused_forward_path(gate_dtype):
    """Enough sequences (B*H >= 64) for the single-pass forward; both of its grid shapes."""
    rng = np.random.default_rng(6300)
    lens = [int(x) for x in rng.integers(1, 200, size=12)]
    print("\n[varlen] fused forward, H=8, 12 sequences, lens=%s gate=%s" % (lens, gate_dtype), flush=True)
    run(6301, lens, 8, 128, 128, gate_dtype=gate_dtype)
    lens = [int(x) for x in rng.integers(1, 150, size=26)]
    print("[varlen] fused forward, H=8, 26 sequences", flush=True)
    run(6302, lens, 8, 128, 128, gate_dtype=gate_dtype)


def test_varlen_all_empty():
    print("\n[varlen] T = 0", flush=True)
    run(6400, [0, 0, 0], 2, 64, 64)
    print("[varlen] T = 0, enough sequences for groups", flush=True)
    run(6401, [0] * 20, 16, 128, 128)


def test_varlen_document_mix_layer_width():
    """H=16, d=128, 8192 tokens cut into documents with a long-tailed length mix."""
    rng = np.random.default_rng(6500)
    lens = []
    while sum(lens) < 8192:
        lens.append(int(min(8192 - sum(lens), max(1, rng.lognormal(5.5, 1.0)))))
    print("\n[varlen] H=16 d=128 T=8192, %d documents, longest %d" % (len(lens), max(lens)), flush=True)
    run(6501, lens, 16, 128, 128, lb=0.5)


@pytest.mark.parametrize("H,dk,dv,gate_dtype", [(16, 128, 128, "bf16"), (8, 128, 128, "f32"), (4, 64, 64, "bf16"), (2, 128, 64, "bf16")])
def test_varlen_many_short_documents(H, dk, dv, gate_dtype):
    """More sequences than workgroups: the walks take a group of consecutive sequences each, one
    after the other.  Lengths of one token to a few chunks, empty sequences at the start, in the
    middle (several in a row) and at the end, with every sequence's own initial and final state."""
    rng = np.random.default_rng(6800 + H)
    # (the walks go by groups from 256 / H sequences on)
    lens = [0, 0] + [int(x) for x in rng.integers(1, 150 if H > 2 else 40, size=max(70, 256 // H + 12))]
    for i in (5, 6, 7, 30, 51):
        lens[i] = 0
    lens += [64, 128, 1, 0, 0]
    print("\n[varlen] H=%d dk=%d dv=%d, %d short documents (%d tokens) gate=%s"
          % (H, dk, dv, len(lens), sum(lens), gate_dtype), flush=True)
    run(6801 + H, lens, H, dk, dv, gate_dtype=gate_dtype)
    run(6851 + H, lens, H, dk, dv, gate_dtype=gate_dtype, with_states=False)


def test_varlen_one_long_document_among_short_ones():
    """One document many times longer than a span of the reverse walk (16384 tokens among 1200 at 16
    spans per head: a tail of up to 240 chunks after a span of 18): the table kernel then sends the
    backward pass through the two sweeps and the per-chunk kernel instead (both are enqueued; the
    choice is made on the device).  And one that is long, but not that long: the walk."""
    run(6951, [40, 16384] + [50, 7, 64, 90] * 5, 16, 128, 128)
    lens = [40, 3000] + [50, 7, 64, 90] * 5
    print("\n[varlen] H=16, one document of 3000 tokens among %d short ones" % (len(lens) - 1), flush=True)
    run(6950, lens, 16, 128, 128)


@pytest.mark.parametrize("H,dk,dv,lens", [
    (16, 128, 128, [700, 130, 0, 1500, 64, 1]),           # 16 spans per head over 6 documents: most spans end inside one
    (4, 64, 128, [2000, 0, 0, 333]),                      # 64 spans per head, more than there are chunks: empty spans
    (16, 128, 128, [40]),                                 # one chunk in all: every span but one is empty
    (2, 128, 64, [1000, 3000, 500]),                      # 128 spans per head, one or no chunk each
])
def test_varlen_reverse_walk_over_spans(H, dk, dv, lens):
    """The reverse walk cuts a head's chunks into equal spans whatever the documents: spans that
    start and end inside a document (the state gradient at their end comes from a light walk over
    the rest of the document), documents inside a span, spans without chunks, with every sequence's
    own grad_hT / grad_h0, and without."""
    print("\n[varlen] H=%d dk=%d dv=%d lens=%s" % (H, dk, dv, lens), flush=True)
    run(7000 + H, lens, H, dk, dv)
    run(7050 + H, lens, H, dk, dv, with_states=False)


def test_varlen_one_chunk_documents_even_and_odd_counts():
    """Groups whose chunk count is even and odd (the single-pass forward runs an even number of
    passes and finishes the last sequence differently in the two cases)."""
    for n_docs in (16, 17, 33):
        lens = [64] * n_docs
        print("\n[varlen] %d documents of 64 tokens, H=16" % n_docs, flush=True)
        run(6900 + n_docs, lens, 16, 128, 128)


def test_varlen_offsets_out_of_order_stay_in_bounds():
    """A non-monotone cu_seqlens is not an error the library can report (it is device data), but it
    must not reach outside the tensors: the call completes and the outputs of the well-formed
    part are finite."""
    H, dk, dv, T = 2, 64, 64, 150
    w = synth.make_sequence(6600, 1, H, T, dk, dv, io_dtype="bf16", lb=0.3, with_dO=True)
    q, f, v = packed(w.q, "bf16"), packed(w.f, "bf16"), packed(w.v, "bf16")
    cud = torch.tensor([0, 100, 40, 9999, 150], dtype=torch.int32).cuda()
    o, hT = binding.hgrn2_fwd_varlen(q, f, v, cud, None)
    torch.cuda.synchronize()
    assert torch.isfinite(hT).all()
    # the table turns the offsets into 0, 100, 100, 150, 150: the first sequence is well formed
    ro, _ = oracle.fwd(w.q[:, :, :100], w.f[:, :, :100], w.v[:, :, :100], None)
    check("o[:100]", unpacked(o)[:, :100], ro[0], TOL["bf16"])


@pytest.mark.parametrize("H,dk,dv,nseq", [(3, 64, 64, 5), (8, 128, 128, 10), (16, 128, 128, 40), (8, 64, 128, 45)])
def test_varlen_with_gate_formed_in_the_kernels(H, dk, dv, nseq):
    """Packed sequences with the pre-activations of the gate and the layer's lower bounds (Eq. 2):
    dz per token and dbeta summed over all sequences, against the oracle run per sequence."""
    rng = np.random.default_rng(6700 + H)
    lens = [int(x) for x in rng.integers(0, 180, size=nseq)]
    B, T = len(lens), int(sum(lens))
    print("\n[varlen gated] H=%d dk=%d dv=%d lens=%s" % (H, dk, dv, lens), flush=True)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    w = synth.make_sequence(6701 + H, 1, H, T, dk, dv, io_dtype="bf16", with_dO=True)
    z = synth.bf16_round((1.5 * rng.standard_normal((1, H, T, dk), dtype=np.float32)).astype(np.float32))
    beta = rng.uniform(0.0, 0.9, size=(H, dk)).astype(np.float32)
    h0 = rng.standard_normal((B, H, dk, dv)).astype(np.float32)
    dhT = (0.1 * rng.standard_normal((B, H, dk, dv))).astype(np.float32)
    q, zd, v, dO = packed(w.q, "bf16"), packed(z, "bf16"), packed(w.v, "bf16"), packed(w.dO, "bf16")
    cud, bd = torch.from_numpy(cu).cuda(), torch.from_numpy(beta).cuda()
    o, hT = binding.hgrn2_fwd_varlen(q, zd, v, cud, dev(h0), beta=bd)
    gq, gz, gv, gh0, gb = binding.hgrn2_bwd_varlen(q, zd, v, dO, cud, dev(h0), dev(dhT), beta=bd, want_grad_h0=True)
    saved = states_buffer(q, v, zd, B)
    o_s, hT_s = binding.hgrn2_fwd_varlen(q, zd, v, cud, dev(h0), beta=bd, saved_states=saved)
    gq_s, gz_s, gv_s, gh0_s, gb_s = binding.hgrn2_bwd_varlen(q, zd, v, dO, cud, dev(h0), dev(dhT), beta=bd,
                                                             want_grad_h0=True, saved_states=saved)
    torch.cuda.synchronize()
    ro, rq, rz, rv = (np.zeros((H, T, d)) for d in (dv, dk, dk, dv))
    rhT, rh0, rb = np.zeros((B, H, dk, dv)), np.zeros((B, H, dk, dv)), np.zeros((H, dk))
    for b in range(B):
        s, e = int(cu[b]), int(cu[b + 1])
        sl = (slice(None), slice(None), slice(s, e))
        ob, hTb = oracle.fwd_gated(w.q[sl], z[sl], beta, w.v[sl], h0[b:b + 1])
        gqb, gzb, gbb, gvb, gh0b = oracle.bwd_gated(w.q[sl], z[sl], beta, w.v[sl], w.dO[sl], h0[b:b + 1], dhT[b:b + 1])
        ro[:, s:e], rq[:, s:e], rz[:, s:e], rv[:, s:e] = ob[0], gqb[0], gzb[0], gvb[0]
        rhT[b], rh0[b] = hTb[0], gh0b[0]
        rb += gbb
    tol = TOL["bf16"]
    check("o", unpacked(o), ro, tol)
    check("hT", host(hT), rhT, tol)
    check("dq", unpacked(gq), rq, tol)
    check("dv", unpacked(gv), rv, tol)
    check("dz", unpacked(gz), rz, tol)
    check("dbeta", host(gb), rb, tol)
    check("dh0", host(gh0), rh0, tol)
    check("o (pair)", unpacked(o_s), ro, tol)
    check("hT (pair)", host(hT_s), rhT, tol)
    check("dq (pair)", unpacked(gq_s), rq, tol)
    check("dv (pair)", unpacked(gv_s), rv, tol)
    check("dz (pair)", unpacked(gz_s), rz, tol)
    check("dbeta (pair)", host(gb_s), rb, tol)
    check("dh0 (pair)", host(gh0_s), rh0, tol)
