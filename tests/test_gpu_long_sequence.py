"""Long sequences in a small batch: the kernels that walk a sequence chunk by chunk then see it cut
into runs (a walk per run from a zero state, a carry over the runs, the walk proper run by run),
so these shapes get parity cases of their own against the fp64 oracle: ragged and whole last
chunks and runs, all four head-dimension pairs, both layouts, both gate storages, gates given and
formed from pre-activations, with and without carried states, and the fp32 forward.
Tolerance: max|x-y|/max|y| <= 2e-2 per tensor for bf16 tensors, 1e-4 for fp32 ones."""
import numpy as np
import pytest
import torch

import oracle
from paper_2404_07904_amd import binding, synth
from gpu_util import TOL, check, dev, host

pytestmark = pytest.mark.gpu
BNHD = binding.HGRN2_LAYOUT_BNHD

CASES = [
    # B, H, N, dk, dv, layout, gate, states, lower bound
    (1, 2, 4133, 128, 128, 0, "bf16", True, 0.9),
    (2, 1, 4096, 64, 128, 1, "f32", False, 0.8),
    (1, 3, 4100, 128, 64, 0, "f32", True, 0.95),
    (2, 2, 4225, 64, 64, 1, "bf16", True, 0.5),
]


@pytest.mark.parametrize("case", CASES, ids=lambda c: "B%dH%dN%d_%dx%d_l%d_%s" % c[:7])
def test_long_sequence_fwd_bwd(case):
    B, H, N, dk, dv, layout, gate_dtype, with_state, lb = case
    print("\n[long] B=%d H=%d N=%d dk=%d dv=%d layout=%d gate=%s states=%s lb=%.2f" % case, flush=True)
    w = synth.make_sequence(7100 + N, B, H, N, dk, dv, io_dtype="bf16", gate_dtype=gate_dtype, lb=lb,
                            with_h0=with_state, with_dO=True, with_dhT=with_state)
    put = (lambda t: t.permute(0, 2, 1, 3).contiguous()) if layout == BNHD else (lambda t: t)
    get = (lambda t: host(t.permute(0, 2, 1, 3))) if layout == BNHD else host
    q, f, v, dO = put(dev(w.q, "bf16")), put(dev(w.f, gate_dtype)), put(dev(w.v, "bf16")), put(dev(w.dO, "bf16"))
    h0, dhT = dev(w.h0), dev(w.dhT)
    o, hT = binding.hgrn2_fwd(q, f, v, h0, layout=layout)
    gq, gf, gv, gh0 = binding.hgrn2_bwd(q, f, v, dO, h0, dhT, want_grad_h0=True, layout=layout)
    torch.cuda.synchronize()
    tol = TOL["bf16"]
    ro, rhT = oracle.fwd(w.q, w.f, w.v, w.h0)
    rq, rf, rv, rh = oracle.bwd(w.q, w.f, w.v, w.dO, w.h0, w.dhT)
    check("o", get(o), ro, tol); check("hT", host(hT), rhT, tol)
    check("dq", get(gq), rq, tol); check("df", get(gf), rf, tol); check("dv", get(gv), rv, tol)
    check("dh0", host(gh0), rh, tol)


def test_long_sequence_gated():
    B, H, N, dk, dv = 1, 2, 4170, 128, 128
    print("\n[long gated] B=%d H=%d N=%d dk=%d dv=%d" % (B, H, N, dk, dv), flush=True)
    rng = np.random.default_rng(7301)
    w = synth.make_sequence(7300, B, H, N, dk, dv, io_dtype="bf16", with_h0=True, with_dO=True, with_dhT=True)
    z = synth.bf16_round((1.5 * rng.standard_normal((B, H, N, dk))).astype(np.float32))
    beta = rng.uniform(0.6, 0.98, size=(H, dk)).astype(np.float32)
    q, zd, v, dO = dev(w.q, "bf16"), dev(z, "bf16"), dev(w.v, "bf16"), dev(w.dO, "bf16")
    bd = torch.from_numpy(beta).cuda()
    o, hT = binding.hgrn2_fwd_gated(q, zd, bd, v, dev(w.h0))
    gq, gz, gb, gv, gh0 = binding.hgrn2_bwd_gated(q, zd, bd, v, dO, dev(w.h0), dev(w.dhT), want_grad_h0=True)
    torch.cuda.synchronize()
    ro, rhT = oracle.fwd_gated(w.q, z, beta, w.v, w.h0)
    rq, rz, rb, rv, rh = oracle.bwd_gated(w.q, z, beta, w.v, w.dO, w.h0, w.dhT)
    tol = TOL["bf16"]
    check("o", host(o), ro, tol); check("hT", host(hT), rhT, tol)
    check("dq", host(gq), rq, tol); check("dz", host(gz), rz, tol); check("dbeta", host(gb), rb, tol)
    check("dv", host(gv), rv, tol); check("dh0", host(gh0), rh, tol)


def test_long_sequence_fp32_forward():
    B, H, N, dk, dv = 1, 2, 4160, 64, 64
    print("\n[long fp32] B=%d H=%d N=%d dk=%d dv=%d" % (B, H, N, dk, dv), flush=True)
    w = synth.make_sequence(7400, B, H, N, dk, dv, io_dtype="f32", lb=0.9, with_h0=True)
    o, hT = binding.hgrn2_fwd(dev(w.q), dev(w.f), dev(w.v), dev(w.h0))
    torch.cuda.synchronize()
    ro, rhT = oracle.fwd(w.q, w.f, w.v, w.h0)
    check("o", host(o), ro, TOL["f32"]); check("hT", host(hT), rhT, TOL["f32"])


@pytest.mark.parametrize("n", [16, 32])
def test_cut_and_uncut_walks_agree(n):
    """The forward cuts sequences from 16 chunks on, the backward from 32: n - 1 chunks are walked in
    one piece, n in runs.  The first n - 1 chunks of outputs of the longer sequence see the same
    tokens, so the two must agree to the rounding of the stored states."""
    B, H, dk, dv = 1, 4, 128, 128
    print("\n[long boundary] %d against %d chunks" % (n - 1, n), flush=True)
    w = synth.make_sequence(7500 + n, B, H, n * 64, dk, dv, io_dtype="bf16", lb=0.9, with_dO=True)
    q, f, v, dO = dev(w.q, "bf16"), dev(w.f, "bf16"), dev(w.v, "bf16"), dev(w.dO, "bf16")
    m = (n - 1) * 64
    cut = lambda t: t[:, :, :m].contiguous()
    o_n, _ = binding.hgrn2_fwd(q, f, v, None)
    o_m, _ = binding.hgrn2_fwd(cut(q), cut(f), cut(v), None)
    torch.cuda.synchronize()
    check("o", host(o_n[:, :, :m]), host(o_m), 1e-2)
    # the backward of the longer sequence with no gradient arriving at its last chunk
    dO0 = dO.clone()
    dO0[:, :, m:] = 0
    g_n = binding.hgrn2_bwd(q, f, v, dO0, None, None)
    g_m = binding.hgrn2_bwd(cut(q), cut(f), cut(v), cut(dO), None, None)
    torch.cuda.synchronize()
    for name, a, b in zip(("dq", "df", "dv"), g_n, g_m):
        check(name, host(a[:, :, :m]), host(b), 1e-2)


@pytest.mark.parametrize("lens,H,dk,dv,gated", [
    ([3000, 700, 0, 4600], 2, 128, 128, False),
    ([2112, 6100], 1, 64, 128, True),
    ([5000, 1, 3333], 3, 64, 64, False),
], ids=["4docs_128", "2docs_gated_64x128", "3docs_64"])
def test_long_documents_in_a_packed_batch(lens, H, dk, dv, gated):
    """Packed batches are cut as an equal-length batch of their mean length would be, so the long
    documents here span several runs, the short ones one, the empty one none."""
    B, T = len(lens), int(sum(lens))
    print("\n[long packed] H=%d dk=%d dv=%d gated=%s lens=%s" % (H, dk, dv, gated, lens), flush=True)
    rng = np.random.default_rng(7600 + T)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    w = synth.make_sequence(7600 + B, 1, H, T, dk, dv, io_dtype="bf16", lb=0.9, with_dO=True)
    z = synth.bf16_round((1.5 * rng.standard_normal((1, H, T, dk))).astype(np.float32))
    beta = rng.uniform(0.7, 0.98, size=(H, dk)).astype(np.float32)
    gate_in = z if gated else w.f
    pk = lambda x: dev(x, "bf16")[0].permute(1, 0, 2).contiguous()
    un = lambda t: host(t.permute(1, 0, 2))
    h0 = (0.1 * rng.standard_normal((B, H, dk, dv))).astype(np.float32)
    dhT = (0.1 * rng.standard_normal((B, H, dk, dv))).astype(np.float32)
    q, g, v, dO = pk(w.q), pk(gate_in), pk(w.v), pk(w.dO)
    cud = torch.from_numpy(cu).cuda()
    bd = torch.from_numpy(beta).cuda() if gated else None
    o, hT = binding.hgrn2_fwd_varlen(q, g, v, cud, dev(h0), beta=bd)
    res = binding.hgrn2_bwd_varlen(q, g, v, dO, cud, dev(h0), dev(dhT), beta=bd, want_grad_h0=True)
    # the same step as a training pair (states kept by the forward pass, run by run; the buffer starts as NaN patterns)
    kept = torch.full((binding.hgrn2_saved_states_varlen_bytes(binding.make_shape_varlen(q, v, g, B)),), 0xFF,
                      dtype=torch.uint8, device=q.device)
    o_s, hT_s = binding.hgrn2_fwd_varlen(q, g, v, cud, dev(h0), beta=bd, saved_states=kept)
    res_s = binding.hgrn2_bwd_varlen(q, g, v, dO, cud, dev(h0), dev(dhT), beta=bd, want_grad_h0=True, saved_states=kept)
    torch.cuda.synchronize()
    ro, rq, rg, rv = (np.zeros((H, T, d)) for d in (dv, dk, dk, dv))
    rhT, rh0, rb = np.zeros((B, H, dk, dv)), np.zeros((B, H, dk, dv)), np.zeros((H, dk))
    for b in range(B):
        s, e = int(cu[b]), int(cu[b + 1])
        sl = (slice(None), slice(None), slice(s, e))
        if gated:
            ob, hTb = oracle.fwd_gated(w.q[sl], z[sl], beta, w.v[sl], h0[b:b + 1])
            gqb, ggb, gbb, gvb, gh0b = oracle.bwd_gated(w.q[sl], z[sl], beta, w.v[sl], w.dO[sl], h0[b:b + 1], dhT[b:b + 1])
            rb += gbb
        else:
            ob, hTb = oracle.fwd(w.q[sl], w.f[sl], w.v[sl], h0[b:b + 1])
            gqb, ggb, gvb, gh0b = oracle.bwd(w.q[sl], w.f[sl], w.v[sl], w.dO[sl], h0[b:b + 1], dhT[b:b + 1])
        ro[:, s:e], rq[:, s:e], rg[:, s:e], rv[:, s:e] = ob[0], gqb[0], ggb[0], gvb[0]
        rhT[b], rh0[b] = hTb[0], gh0b[0]
    tol = TOL["bf16"]
    check("o", un(o), ro, tol); check("hT", host(hT), rhT, tol)
    check("dq", un(res[0]), rq, tol); check("dgate", un(res[1]), rg, tol); check("dv", un(res[2]), rv, tol)
    check("dh0", host(res[3]), rh0, tol)
    if gated:
        check("dbeta", host(res[4]), rb, tol)
    check("o (pair)", un(o_s), ro, tol); check("hT (pair)", host(hT_s), rhT, tol)
    check("dq (pair)", un(res_s[0]), rq, tol); check("dgate (pair)", un(res_s[1]), rg, tol); check("dv (pair)", un(res_s[2]), rv, tol)
    check("dh0 (pair)", host(res_s[3]), rh0, tol)
    if gated:
        check("dbeta (pair)", host(res_s[4]), rb, tol)
