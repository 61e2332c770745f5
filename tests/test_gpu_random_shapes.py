"""Seeded random shapes through every entry-point family against the fp64 oracle: batch, head and
token counts, head dimensions, layouts, gate storage, optional states and sequence packings are
drawn from a fixed seed per case, so the index arithmetic of the kernels (ragged chunks, grid
padding, the two grid shapes of the single-pass forward, per-sequence tables) is exercised at
combinations no hand-written case lists.  Tolerance: max|x-y|/max|y| <= 2e-2 per tensor (bf16)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2404_07904_amd import binding, synth
from gpu_util import TOL, check, dev, host

pytestmark = pytest.mark.gpu
BNHD = binding.HGRN2_LAYOUT_BNHD


def draw(seed):
    rng = np.random.default_rng(seed)
    dk, dv = (int(rng.choice([64, 128])) for _ in range(2))
    many = bool(rng.integers(0, 2))                       # enough sequences for the single-pass forward?
    B = int(rng.integers(5, 12)) if many else int(rng.integers(1, 4))
    H = int(rng.integers(8, 30)) if many else int(rng.integers(1, 6))
    N = int(rng.integers(1, 330)) if not many else int(rng.integers(1, 200))
    return rng, B, H, N, dk, dv


@pytest.mark.parametrize("seed", range(9000, 9012))
def test_random_equal_length(seed):
    rng, B, H, N, dk, dv = draw(seed)
    layout = int(rng.integers(0, 2))
    gate_dtype = str(rng.choice(["bf16", "f32"]))
    with_state = bool(rng.integers(0, 2))
    lb = float(rng.choice([0.15, 0.5, 0.9]))
    print("\n[random] seed=%d B=%d H=%d N=%d dk=%d dv=%d layout=%d gate=%s states=%s lb=%.2f"
          % (seed, B, H, N, dk, dv, layout, gate_dtype, with_state, lb), flush=True)
    w = synth.make_sequence(seed, B, H, N, dk, dv, io_dtype="bf16", gate_dtype=gate_dtype, lb=lb,
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


@pytest.mark.parametrize("seed", range(9050, 9062))
def test_random_equal_length_shorter_chunks(seed):
    """The same with 32, 16 or 8 tokens per chunk, or the chunk length chosen on the device, as the stateless
    calls or as the training pair: on gates every mode can take, all of them must agree with the oracle."""
    rng, B, H, N, dk, dv = draw(seed)
    N = int(N * rng.choice([1, 1, 4]))                     # some long enough for runs of the shorter chunks
    layout = int(rng.integers(0, 2))
    chunk = int(rng.choice([32, 16, 8, -1]))
    pair = bool(rng.integers(0, 2))
    with_state = bool(rng.integers(0, 2))
    print("\n[random] seed=%d B=%d H=%d N=%d dk=%d dv=%d layout=%d chunk=%d pair=%s states=%s"
          % (seed, B, H, N, dk, dv, layout, chunk, pair, with_state), flush=True)
    w = synth.make_sequence(seed, B, H, N, dk, dv, io_dtype="bf16", lb=0.3, with_h0=with_state, with_dO=True, with_dhT=with_state)
    put = (lambda t: t.permute(0, 2, 1, 3).contiguous()) if layout == BNHD else (lambda t: t)
    get = (lambda t: host(t.permute(0, 2, 1, 3))) if layout == BNHD else host
    q, f, v, dO = put(dev(w.q, "bf16")), put(dev(w.f, "bf16")), put(dev(w.v, "bf16")), put(dev(w.dO, "bf16"))
    h0, dhT = dev(w.h0), dev(w.dhT)
    if pair:
        o, hT, saved = binding.hgrn2_fwd_saving(q, f, v, h0, layout=layout, chunk=chunk)
        gq, gf, gv, gh0 = binding.hgrn2_bwd_saved(q, f, v, saved, dO, dhT, want_grad_h0=True, layout=layout, chunk=chunk)
    else:
        o, hT = binding.hgrn2_fwd(q, f, v, h0, layout=layout, chunk=chunk)
        gq, gf, gv, gh0 = binding.hgrn2_bwd(q, f, v, dO, h0, dhT, want_grad_h0=True, layout=layout, chunk=chunk)
    torch.cuda.synchronize()
    tol = TOL["bf16"]
    ro, rhT = oracle.fwd(w.q, w.f, w.v, w.h0)
    rq, rf, rv, rh = oracle.bwd(w.q, w.f, w.v, w.dO, w.h0, w.dhT)
    check("o", get(o), ro, tol); check("hT", host(hT), rhT, tol)
    check("dq", get(gq), rq, tol); check("df", get(gf), rf, tol); check("dv", get(gv), rv, tol)
    check("dh0", host(gh0), rh, tol)


@pytest.mark.parametrize("seed", range(9100, 9108))
def test_random_packed_sequences(seed):
    rng, B, H, _, dk, dv = draw(seed)
    lens = [int(x) for x in rng.integers(0, 150, size=B)]
    T = int(sum(lens))
    gated = bool(rng.integers(0, 2))
    chunk = (0, 32, 16, 8)[seed % 4]                      # tokens per chunk (0: 64); these gates allow any
    print("\n[random packed] seed=%d H=%d dk=%d dv=%d gated=%s chunk=%d lens=%s" % (seed, H, dk, dv, gated, chunk, lens), flush=True)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    w = synth.make_sequence(seed, 1, H, max(T, 1), dk, dv, io_dtype="bf16", lb=0.3, with_dO=True)
    z = synth.bf16_round((1.5 * rng.standard_normal((1, H, max(T, 1), dk), dtype=np.float32)).astype(np.float32))
    beta = rng.uniform(0.0, 0.9, size=(H, dk)).astype(np.float32)
    gate_in = z if gated else w.f
    cut = lambda x: x[:, :, :T]
    pk = lambda x: dev(cut(x), "bf16")[0].permute(1, 0, 2).contiguous()
    un = lambda t: host(t.permute(1, 0, 2))
    h0 = rng.standard_normal((B, H, dk, dv)).astype(np.float32)
    dhT = (0.1 * rng.standard_normal((B, H, dk, dv))).astype(np.float32)
    q, g, v, dO = pk(w.q), pk(gate_in), pk(w.v), pk(w.dO)
    cud = torch.from_numpy(cu).cuda()
    bd = torch.from_numpy(beta).cuda() if gated else None
    o, hT = binding.hgrn2_fwd_varlen(q, g, v, cud, dev(h0), beta=bd, chunk=chunk)
    res = binding.hgrn2_bwd_varlen(q, g, v, dO, cud, dev(h0), dev(dhT), beta=bd, want_grad_h0=True, chunk=chunk)
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


@pytest.mark.parametrize("seed", range(9200, 9208))
def test_random_elementwise_recurrence(seed):
    """The element-wise recurrence, with f, i, o given or formed from pre-activations (alternating)."""
    rng = np.random.default_rng(seed)
    B, N, d = int(rng.integers(1, 5)), int(rng.integers(0, 700)), 64 * int(rng.integers(1, 7))
    act = seed % 2 == 1
    gate_dtype = str(rng.choice(["bf16", "f32"]))
    print("\n[random hgrn1] seed=%d B=%d N=%d d=%d act=%s gate=%s" % (seed, B, N, d, act, gate_dtype), flush=True)
    sig = lambda z: 1.0 / (1.0 + np.exp(-z))
    zf = (1.5 * rng.standard_normal((B, N, d))).astype(np.float32)
    zi = synth.bf16_round((1.5 * rng.standard_normal((B, N, d))).astype(np.float32))
    zo = synth.bf16_round((1.5 * rng.standard_normal((B, N, d))).astype(np.float32))
    dy = synth.bf16_round(rng.standard_normal((B, N, d)).astype(np.float32))
    beta = rng.uniform(0.0, 0.9, size=d).astype(np.float32)
    h0 = rng.standard_normal((B, d)).astype(np.float32)
    dhN = rng.standard_normal((B, d)).astype(np.float32)
    rnd = (lambda x: x) if gate_dtype == "f32" else synth.bf16_round
    tol = TOL["bf16"]
    if act:
        zf = rnd(zf)
        args = (dev(zf, gate_dtype), dev(zi, "bf16"), dev(zo, "bf16"), torch.from_numpy(beta).cuda())
        y, hN = binding.hgrn1_fwd_act(*args, dev(h0))
        gf, gi, go, gb, gh0 = binding.hgrn1_bwd_act(*args, dev(dy, "bf16"), dev(h0), dev(dhN), want_grad_h0=True)
        torch.cuda.synchronize()
        ry, rh = oracle.hgrn1_fwd_act(zf, zi, zo, beta, h0)
        rf, ri, ro, rb, rh0 = oracle.hgrn1_bwd_act(zf, zi, zo, beta, dy, h0, dhN)
        check("dbeta", host(gb), rb, tol)
    else:
        f = np.minimum(rnd((0.2 + 0.8 * sig(zf)).astype(np.float32)), np.float32(1.0))
        o = synth.bf16_round(sig(zo).astype(np.float32))
        y, hN = binding.hgrn1_fwd(dev(f, gate_dtype), dev(zi, "bf16"), dev(o, "bf16"), dev(h0))
        gf, gi, go, gh0 = binding.hgrn1_bwd(dev(f, gate_dtype), dev(zi, "bf16"), dev(o, "bf16"), dev(dy, "bf16"), dev(h0),
                                            dev(dhN), want_grad_h0=True)
        torch.cuda.synchronize()
        ry, rh = oracle.hgrn1_fwd(f, zi, o, h0)
        rf, ri, ro, rh0 = oracle.hgrn1_bwd(f, zi, o, dy, h0, dhN)
    check("y", host(y), ry, tol); check("hN", host(hN), rh, tol)
    check("df", host(gf), rf, tol); check("di", host(gi), ri, tol); check("do", host(go), ro, tol)
    check("dh0", host(gh0), rh0, tol)


@pytest.mark.parametrize("seed", range(9300, 9306))
def test_random_long_sequences(seed):
    """Few sequences of 32 chunks or more: the sweeps and the single-pass forward walk them in runs
    (uneven run counts, a shorter last run, a ragged last chunk)."""
    rng = np.random.default_rng(seed)
    dk, dv = (int(rng.choice([64, 128])) for _ in range(2))
    B, H = int(rng.integers(1, 3)), int(rng.integers(1, 4))
    N = int(rng.integers(2048, 5200))
    layout = int(rng.integers(0, 2))
    gate_dtype = str(rng.choice(["bf16", "f32"]))
    with_state = bool(rng.integers(0, 2))
    lb = float(rng.choice([0.5, 0.9, 0.97]))
    print("\n[random long] seed=%d B=%d H=%d N=%d dk=%d dv=%d layout=%d gate=%s states=%s lb=%.2f"
          % (seed, B, H, N, dk, dv, layout, gate_dtype, with_state, lb), flush=True)
    w = synth.make_sequence(seed, B, H, N, dk, dv, io_dtype="bf16", gate_dtype=gate_dtype, lb=lb,
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


@pytest.mark.parametrize("seed", range(9400, 9405))
def test_random_packed_long_documents(seed):
    """Packed batches long enough on average to be cut into runs: documents of many runs, of one,
    of none, in random order; gates given or formed in the kernels."""
    rng = np.random.default_rng(seed)
    dk, dv = (int(rng.choice([64, 128])) for _ in range(2))
    B, H = int(rng.integers(2, 5)), int(rng.integers(1, 3))
    lens = [int(rng.choice([0, int(rng.integers(1, 200)), int(rng.integers(2000, 4500))], p=[0.15, 0.25, 0.6]))
            for _ in range(B)]
    lens[int(rng.integers(0, B))] = int(rng.integers(B * 2100, B * 2100 + 1500))      # the mean length is past the cut
    T = int(sum(lens))
    gated = bool(rng.integers(0, 2))
    chunk = (0, 0, 32, 16, 0)[seed % 5]                   # tokens per chunk (0: 64); these gates allow any
    print("\n[random packed long] seed=%d H=%d dk=%d dv=%d gated=%s chunk=%d lens=%s" % (seed, H, dk, dv, gated, chunk, lens), flush=True)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    w = synth.make_sequence(seed, 1, H, T, dk, dv, io_dtype="bf16", lb=0.8, with_dO=True)
    z = synth.bf16_round((1.0 + 1.5 * rng.standard_normal((1, H, T, dk), dtype=np.float32)).astype(np.float32))
    beta = rng.uniform(0.5, 0.95, size=(H, dk)).astype(np.float32)
    gate_in = z if gated else w.f
    pk = lambda x: dev(x, "bf16")[0].permute(1, 0, 2).contiguous()
    un = lambda t: host(t.permute(1, 0, 2))
    h0 = (0.1 * rng.standard_normal((B, H, dk, dv))).astype(np.float32)
    dhT = (0.1 * rng.standard_normal((B, H, dk, dv))).astype(np.float32)
    q, g, v, dO = pk(w.q), pk(gate_in), pk(w.v), pk(w.dO)
    cud = torch.from_numpy(cu).cuda()
    bd = torch.from_numpy(beta).cuda() if gated else None
    o, hT = binding.hgrn2_fwd_varlen(q, g, v, cud, dev(h0), beta=bd, chunk=chunk)
    res = binding.hgrn2_bwd_varlen(q, g, v, dO, cud, dev(h0), dev(dhT), beta=bd, want_grad_h0=True, chunk=chunk)
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
