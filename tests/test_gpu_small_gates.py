"""Small gates.  With a reference row every 64 tokens the chunkwise kernels are exact while the gate
product of every half chunk stays above 2^-100; chunk = 16 (32) in the shape asks for reference rows
every 16 (32) tokens (a chunk of the kernels then holds only that many tokens, in its middle rows),
which moves that bound to products of 8 (16) gates.  The cases here lie outside the first domain and inside the
second and are compared with the fp64 oracle, which has no such limit; the probe must say so for
both spacings.  Tolerance: max|x-y|/max|y| <= 2e-2 per tensor (bf16), 1e-4 (fp32 forward)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2404_07904_amd import binding, synth
from gpu_util import TOL, check, dev, host, rel_err

pytestmark = pytest.mark.gpu
BNHD = binding.HGRN2_LAYOUT_BNHD
LIMIT = 2.0 ** -100


def small_gate_workload(seed, B, H, N, dk, dv, kind, io_dtype="bf16"):
    """q, v, dO, states as everywhere; gates log-uniform in [1e-3, 1] ("loguniform"), or mostly
    near one with one token in twelve at 1e-4, a reset of the state ("resets")."""
    w = synth.make_sequence(seed, B, H, N, dk, dv, io_dtype=io_dtype, lb=0.9, with_h0=True, with_dO=True, with_dhT=True)
    rng = np.random.default_rng(seed + 1)
    if kind == "loguniform":
        f = 10.0 ** rng.uniform(-3.0, 0.0, size=w.f.shape)
    elif kind == "loguniform8":           # for reference rows every 8 tokens: 4 gates multiply to 1e-20 at worst, 8 gates to 1e-40
        f = 10.0 ** rng.uniform(-5.0, 0.0, size=w.f.shape)
    elif kind == "loguniform32":          # for reference rows every 32 tokens: 16 gates multiply to 6e-28 at worst
        f = 10.0 ** rng.uniform(np.log10(0.02), 0.0, size=w.f.shape)
    else:
        f = np.where(rng.random(w.f.shape) < 1.0 / 12.0, 1e-4, 0.9 + 0.1 * rng.random(w.f.shape))
    w.f = synth.bf16_round(f.astype(np.float32)) if io_dtype == "bf16" else f.astype(np.float32)
    return w


@pytest.mark.parametrize("kind,B,H,N,dk,dv,layout,chunk", [
    ("loguniform", 2, 3, 200, 64, 64, 0, 16),
    ("resets", 1, 2, 333, 128, 128, 1, 16),
    ("loguniform", 9, 8, 130, 128, 128, 0, 16),      # enough sequences for the single-pass forward
    ("resets", 1, 2, 1100, 64, 128, 0, 16),          # 69 chunks of 16 tokens: walked in runs
    ("loguniform32", 2, 2, 300, 128, 64, 1, 32),
    ("loguniform32", 1, 3, 700, 64, 64, 0, 32),
    ("loguniform8", 2, 2, 150, 128, 128, 0, 8),      # a chunk holds 8 tokens, in rows 28 .. 35: half a row block of two waves each
    ("loguniform8", 1, 3, 100, 64, 128, 1, 8),
])
def test_small_gates_fwd_bwd(kind, B, H, N, dk, dv, layout, chunk):
    print("\n[small gates] %s B=%d H=%d N=%d dk=%d dv=%d layout=%d chunk=%d" % (kind, B, H, N, dk, dv, layout, chunk), flush=True)
    w = small_gate_workload(7700 + N, B, H, N, dk, dv, kind)
    put = (lambda t: t.permute(0, 2, 1, 3).contiguous()) if layout == BNHD else (lambda t: t)
    get = (lambda t: host(t.permute(0, 2, 1, 3))) if layout == BNHD else host
    q, f, v, dO = put(dev(w.q, "bf16")), put(dev(w.f, "bf16")), put(dev(w.v, "bf16")), put(dev(w.dO, "bf16"))
    h0, dhT = dev(w.h0), dev(w.dhT)
    coarse = float(binding.hgrn2_min_gate_product(f, layout=layout).item())
    fine = float(binding.hgrn2_min_gate_product(f, layout=layout, chunk=chunk).item())
    print("    smallest gate product: %.3e over 32 tokens, %.3e over %d tokens (limit %.3e)"
          % (coarse, fine, chunk // 2, LIMIT), flush=True)
    assert coarse < LIMIT < fine
    assert abs(fine - oracle.min_gate_product(w.f, chunk=chunk)) <= 1e-4 * fine
    o, hT = binding.hgrn2_fwd(q, f, v, h0, layout=layout, chunk=chunk)
    gq, gf, gv, gh0 = binding.hgrn2_bwd(q, f, v, dO, h0, dhT, want_grad_h0=True, layout=layout, chunk=chunk)
    o64, _ = binding.hgrn2_fwd(q, f, v, h0, layout=layout)
    torch.cuda.synchronize()
    tol = TOL["bf16"]
    ro, rhT = oracle.fwd(w.q, w.f, w.v, w.h0)
    rq, rf, rv, rh = oracle.bwd(w.q, w.f, w.v, w.dO, w.h0, w.dhT)
    check("o", get(o), ro, tol); check("hT", host(hT), rhT, tol)
    check("dq", get(gq), rq, tol); check("df", get(gf), rf, tol); check("dv", get(gv), rv, tol)
    check("dh0", host(gh0), rh, tol)
    print("    for comparison, o with reference rows every 64 tokens: error %.3e" % rel_err(get(o64), ro), flush=True)


@pytest.mark.parametrize("kind,B,H,N,dk,dv,layout,chunk,io", [
    ("loguniform", 8, 16, 200, 128, 128, 0, 16, "bf16"),      # single-pass forward hands its states over; two light runs backward
    ("loguniform32", 2, 2, 1500, 128, 128, 1, 32, "bf16"),    # 47 chunks of 32 tokens: runs forward, boundary sweeps backward
    ("resets", 1, 3, 130, 64, 128, 0, 16, "bf16"),
    ("loguniform32", 2, 2, 150, 64, 64, 0, 16, "f32"),        # fp32 storage: the chunkwise algebra of the mode at 1e-4 (gates
                                                               # >= 0.02: grad_f divides by f, which multiplies fp32 rounding by 1/f)
])
def test_small_gates_training_pair(kind, B, H, N, dk, dv, layout, chunk, io):
    """hgrn2_fwd_saving / hgrn2_bwd_saved with reference rows every 16 / 32 tokens: the kept states are those
    of the shorter chunks."""
    print("\n[small gates, training pair] %s B=%d H=%d N=%d dk=%d dv=%d layout=%d chunk=%d %s"
          % (kind, B, H, N, dk, dv, layout, chunk, io), flush=True)
    w = small_gate_workload(7750 + N, B, H, N, dk, dv, kind, io_dtype=io)
    put = (lambda t: t.permute(0, 2, 1, 3).contiguous()) if layout == BNHD else (lambda t: t)
    get = (lambda t: host(t.permute(0, 2, 1, 3))) if layout == BNHD else host
    q, f, v, dO = put(dev(w.q, io)), put(dev(w.f, io)), put(dev(w.v, io)), put(dev(w.dO, io))
    h0, dhT = dev(w.h0), dev(w.dhT)
    fine = float(binding.hgrn2_min_gate_product(f, layout=layout, chunk=chunk).item())
    assert LIMIT < fine
    flag = torch.zeros(1, dtype=torch.int32, device="cuda")
    o, hT, saved = binding.hgrn2_fwd_saving(q, f, v, h0, layout=layout, chunk=chunk, domain_flag=flag)
    gq, gf, gv, gh0 = binding.hgrn2_bwd_saved(q, f, v, saved, dO, dhT, want_grad_h0=True, layout=layout, chunk=chunk,
                                             domain_flag=flag)
    torch.cuda.synchronize()
    assert int(flag.item()) == 0
    tol = TOL[io]
    ro, rhT = oracle.fwd(w.q, w.f, w.v, w.h0)
    rq, rf, rv, rh = oracle.bwd(w.q, w.f, w.v, w.dO, w.h0, w.dhT)
    check("o", get(o), ro, tol); check("hT", host(hT), rhT, tol)
    check("dq", get(gq), rq, tol); check("df", get(gf), rf, tol); check("dv", get(gv), rv, tol)
    check("dh0", host(gh0), rh, tol)


@pytest.mark.parametrize("kind,expect,B,H,N,dk,dv,layout", [
    ("ordinary", 0, 2, 3, 300, 128, 128, 0),
    ("loguniform32", 32, 8, 16, 200, 128, 128, 0),     # single-pass forward, light runs backward
    ("loguniform32", 32, 2, 2, 1500, 64, 128, 1),      # runs forward and backward
    ("loguniform", 16, 2, 3, 333, 128, 64, 1),
    ("resets", None, 1, 2, 200, 64, 64, 0),           # (whichever spacing these gates turn out to need)
])
def test_chunk_length_chosen_on_the_device(kind, expect, B, H, N, dk, dv, layout):
    """chunk = HGRN2_CHUNK_AUTO: the passes for 64, 32 and 16 tokens per chunk are enqueued and the flags
    the kernels raise decide which of them run.  The results must be those of the chunk length the
    gates need, bit for bit, for the stateless calls and for the training pair, and agree with the oracle."""
    AUTO = -1
    print("\n[chunk chosen on the device] %s (expect %s) B=%d H=%d N=%d dk=%d dv=%d layout=%d" % (kind, expect, B, H, N, dk, dv, layout), flush=True)
    if kind == "ordinary":
        w = synth.make_sequence(7600 + N, B, H, N, dk, dv, io_dtype="bf16", lb=0.0, with_h0=True, with_dO=True, with_dhT=True)
    else:
        w = small_gate_workload(7600 + N, B, H, N, dk, dv, kind)
    put = (lambda t: t.permute(0, 2, 1, 3).contiguous()) if layout == BNHD else (lambda t: t)
    get = (lambda t: host(t.permute(0, 2, 1, 3))) if layout == BNHD else host
    q, f, v, dO = put(dev(w.q, "bf16")), put(dev(w.f, "bf16")), put(dev(w.v, "bf16")), put(dev(w.dO, "bf16"))
    h0, dhT = dev(w.h0), dev(w.dhT)
    # which spacing the gates need, by the probe
    need = 0
    for ck in (0, 32, 16):
        if float(binding.hgrn2_min_gate_product(f, layout=layout, chunk=ck).item()) > LIMIT:
            need = ck
            break
    else:
        raise AssertionError("gates outside every domain")
    print("    the probe says: chunk = %d" % need, flush=True)
    assert expect is None or need == expect
    flag = torch.zeros(1, dtype=torch.int32, device="cuda")
    o_a, hT_a = binding.hgrn2_fwd(q, f, v, h0, layout=layout, chunk=AUTO, domain_flag=flag)
    g_a = binding.hgrn2_bwd(q, f, v, dO, h0, dhT, want_grad_h0=True, layout=layout, chunk=AUTO, domain_flag=flag)
    o_r, hT_r = binding.hgrn2_fwd(q, f, v, h0, layout=layout, chunk=need)
    g_r = binding.hgrn2_bwd(q, f, v, dO, h0, dhT, want_grad_h0=True, layout=layout, chunk=need)
    torch.cuda.synchronize()
    assert int(flag.item()) == 0
    assert torch.equal(o_a, o_r) and torch.equal(hT_a, hT_r)
    for x, y in zip(g_a, g_r):
        assert torch.equal(x, y)
    # the training pair
    o_p, hT_p, saved = binding.hgrn2_fwd_saving(q, f, v, h0, layout=layout, chunk=AUTO, domain_flag=flag)
    g_p = binding.hgrn2_bwd_saved(q, f, v, saved, dO, dhT, want_grad_h0=True, layout=layout, chunk=AUTO, domain_flag=flag)
    o_s, hT_s, saved_r = binding.hgrn2_fwd_saving(q, f, v, h0, layout=layout, chunk=need)
    g_s = binding.hgrn2_bwd_saved(q, f, v, saved_r, dO, dhT, want_grad_h0=True, layout=layout, chunk=need)
    torch.cuda.synchronize()
    assert int(flag.item()) == 0
    assert torch.equal(o_p, o_s) and torch.equal(hT_p, hT_s)
    for x, y in zip(g_p, g_s):
        assert torch.equal(x, y)
    tol = TOL["bf16"]
    ro, rhT = oracle.fwd(w.q, w.f, w.v, w.h0)
    rq, rf, rv, rh = oracle.bwd(w.q, w.f, w.v, w.dO, w.h0, w.dhT)
    check("o", get(o_a), ro, tol); check("hT", host(hT_a), rhT, tol)
    check("dq", get(g_p[0]), rq, tol); check("df", get(g_p[1]), rf, tol); check("dv", get(g_p[2]), rv, tol)
    check("dh0", host(g_p[3]), rh, tol)


def test_chunk_length_chosen_on_the_device_gated_and_out_of_every_domain():
    """The same with the gate formed in the kernels (grad_beta is reduced by the alternative that ran), and
    gates that even 16 tokens per chunk cannot take: only then is the caller's flag raised."""
    AUTO = -1
    B, H, N, dk, dv = 2, 2, 170, 128, 64
    rng = np.random.default_rng(8051)
    w = synth.make_sequence(8050, B, H, N, dk, dv, io_dtype="bf16", with_h0=True, with_dO=True, with_dhT=True)
    z = synth.bf16_round((-5.0 + 1.5 * rng.standard_normal((B, H, N, dk))).astype(np.float32))
    beta = rng.uniform(0.0, 1e-3, size=(H, dk)).astype(np.float32)
    q, zd, v, dO = dev(w.q, "bf16"), dev(z, "bf16"), dev(w.v, "bf16"), dev(w.dO, "bf16")
    bd = torch.from_numpy(beta).cuda()
    h0, dhT = dev(w.h0), dev(w.dhT)
    flag = torch.zeros(1, dtype=torch.int32, device="cuda")
    o, hT = binding.hgrn2_fwd_gated(q, zd, bd, v, h0, chunk=AUTO, domain_flag=flag)
    got = binding.hgrn2_bwd_gated(q, zd, bd, v, dO, h0, dhT, want_grad_h0=True, chunk=AUTO, domain_flag=flag)
    want = binding.hgrn2_bwd_gated(q, zd, bd, v, dO, h0, dhT, want_grad_h0=True, chunk=16)
    torch.cuda.synchronize()
    assert int(flag.item()) == 0
    for x, y in zip(got, want):
        assert torch.equal(x, y)
    ro, rhT = oracle.fwd_gated(w.q, z, beta, w.v, w.h0)
    check("o", host(o), ro, TOL["bf16"]); check("hT", host(hT), rhT, TOL["bf16"])
    rb = oracle.bwd_gated(w.q, z, beta, w.v, w.dO, w.h0, w.dhT)[2]
    check("dbeta", host(got[2]), rb, TOL["bf16"])
    # gates of 1e-6 throughout: 8 of them multiply to 1e-48 < 2^-100
    tiny = torch.full((B, H, N, dk), 1e-6, device="cuda").to(torch.bfloat16)
    binding.hgrn2_fwd(q, tiny, v, h0, chunk=AUTO, domain_flag=flag)
    torch.cuda.synchronize()
    assert int(flag.item()) == 1


def test_chunk_length_chosen_on_the_device_without_tokens():
    """N = 0 in every form of the call: the final state is the initial one, the state gradient passes through."""
    AUTO = -1
    B, H, d = 2, 3, 64
    e = torch.empty((B, H, 0, d), dtype=torch.bfloat16, device="cuda")
    g = torch.Generator(device="cuda").manual_seed(3)
    h0 = torch.randn((B, H, d, d), generator=g, device="cuda")
    dhT = torch.randn((B, H, d, d), generator=g, device="cuda")
    o, hT = binding.hgrn2_fwd(e, e, e, h0, chunk=AUTO)
    res = binding.hgrn2_bwd(e, e, e, e, h0, dhT, want_grad_h0=True, chunk=AUTO)
    o2, hT2, saved = binding.hgrn2_fwd_saving(e, e, e, h0, chunk=AUTO)
    res2 = binding.hgrn2_bwd_saved(e, e, e, saved, e, dhT, want_grad_h0=True, chunk=AUTO)
    torch.cuda.synchronize()
    assert torch.equal(hT, h0) and torch.equal(hT2, h0)
    assert torch.equal(res[3], dhT) and torch.equal(res2[3], dhT)


def test_small_gates_fp32_forward():
    B, H, N, dk, dv = 1, 2, 150, 64, 64
    print("\n[small gates fp32] B=%d H=%d N=%d" % (B, H, N), flush=True)
    w = small_gate_workload(7800, B, H, N, dk, dv, "loguniform", io_dtype="f32")
    o, hT = binding.hgrn2_fwd(dev(w.q), dev(w.f), dev(w.v), dev(w.h0), chunk=16)
    torch.cuda.synchronize()
    ro, rhT = oracle.fwd(w.q, w.f, w.v, w.h0)
    check("o", host(o), ro, TOL["f32"]); check("hT", host(hT), rhT, TOL["f32"])


def test_fine_and_coarse_reference_rows_agree_on_ordinary_gates():
    B, H, N, d = 2, 2, 211, 128
    print("\n[small gates] ordinary gates, both spacings", flush=True)
    w = synth.make_sequence(7900, B, H, N, d, d, io_dtype="bf16", lb=0.3, with_h0=True, with_dO=True, with_dhT=True)
    q, f, v, dO = (dev(x, "bf16") for x in (w.q, w.f, w.v, w.dO))
    a = binding.hgrn2_bwd(q, f, v, dO, dev(w.h0), dev(w.dhT), want_grad_h0=True)
    b = binding.hgrn2_bwd(q, f, v, dO, dev(w.h0), dev(w.dhT), want_grad_h0=True, chunk=16)
    torch.cuda.synchronize()
    for name, x, y in zip(("dq", "df", "dv", "dh0"), a, b):
        check(name, host(y), host(x), 1e-2)
    # empty sequences pass in this mode as well
    e = torch.empty((B, H, 0, d), dtype=torch.bfloat16, device="cuda")
    o, hT = binding.hgrn2_fwd(e, e, e, dev(w.h0), chunk=16)
    torch.cuda.synchronize()
    assert o.shape[2] == 0 and torch.equal(hT, dev(w.h0))


def test_small_gates_with_the_gate_formed_in_the_kernels():
    """Pre-activations around -5 and next to no lower bound: gates of 7e-3, far outside the ordinary domain."""
    B, H, N, dk, dv = 2, 2, 170, 128, 64
    print("\n[small gates gated] B=%d H=%d N=%d dk=%d dv=%d" % (B, H, N, dk, dv), flush=True)
    rng = np.random.default_rng(8001)
    w = synth.make_sequence(8000, B, H, N, dk, dv, io_dtype="bf16", with_h0=True, with_dO=True, with_dhT=True)
    z = synth.bf16_round((-5.0 + 1.5 * rng.standard_normal((B, H, N, dk))).astype(np.float32))
    beta = rng.uniform(0.0, 1e-3, size=(H, dk)).astype(np.float32)
    q, zd, v, dO = dev(w.q, "bf16"), dev(z, "bf16"), dev(w.v, "bf16"), dev(w.dO, "bf16")
    bd = torch.from_numpy(beta).cuda()
    coarse = float(binding.hgrn2_min_gate_product(zd, bd).item())
    fine = float(binding.hgrn2_min_gate_product(zd, bd, chunk=16).item())
    print("    smallest gate product: %.3e over 32 tokens, %.3e over 8 tokens (limit %.3e)" % (coarse, fine, LIMIT), flush=True)
    assert coarse < LIMIT < fine
    h0, dhT = dev(w.h0), dev(w.dhT)
    o, hT = binding.hgrn2_fwd_gated(q, zd, bd, v, h0, chunk=16)
    gq, gz, gb, gv, gh0 = binding.hgrn2_bwd_gated(q, zd, bd, v, dO, h0, dhT, want_grad_h0=True, chunk=16)
    torch.cuda.synchronize()
    ro, rhT = oracle.fwd_gated(w.q, z, beta, w.v, w.h0)
    rq, rz, rb, rv, rh = oracle.bwd_gated(w.q, z, beta, w.v, w.dO, w.h0, w.dhT)
    tol = TOL["bf16"]
    check("o", host(o), ro, tol); check("hT", host(hT), rhT, tol)
    check("dq", host(gq), rq, tol); check("dz", host(gz), rz, tol); check("dbeta", host(gb), rb, tol)
    check("dv", host(gv), rv, tol); check("dh0", host(gh0), rh, tol)


@pytest.mark.parametrize("lens,H,dk,dv,gated,chunk,pair", [
    ([150, 0, 37, 260], 2, 64, 64, False, 16, False),
    ([90, 300], 3, 128, 64, True, 16, False),
    ([200, 1, 333], 2, 128, 128, False, 32, False),
    ([150, 0, 37, 260], 2, 64, 64, False, 16, True),
    ([70, 45, 0, 33, 90, 17, 64, 1, 80, 5, 120, 31, 66, 48, 12, 100] * 3, 16, 128, 128, False, 32, True),  # groups of sequences per workgroup
    ([1300, 900], 2, 128, 128, False, 16, True),       # documents walked in runs of the shorter chunks
    ([60, 9, 100], 3, 64, 128, False, 8, False),
])
def test_small_gates_in_a_packed_batch(lens, H, dk, dv, gated, chunk, pair):
    """Packed batches take the shorter chunks like equal-length ones (the tables count chunks of 32, 16 or 8
    tokens): ragged last chunks, empty and one-token sequences, groups of sequences per workgroup,
    documents cut into runs, the gates given or formed in the kernels, stateless or as the training pair."""
    B, T = len(lens), int(sum(lens))
    print("\n[small gates packed] H=%d dk=%d dv=%d gated=%s chunk=%d pair=%s lens=%s" % (H, dk, dv, gated, chunk, pair, lens), flush=True)
    rng = np.random.default_rng(8100 + T)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    w = small_gate_workload(8100 + B, 1, H, T, dk, dv, "loguniform" if chunk == 16 else "loguniform32")
    z = synth.bf16_round((-4.5 + 1.5 * rng.standard_normal((1, H, T, dk))).astype(np.float32))
    beta = rng.uniform(0.0, 1e-3, size=(H, dk)).astype(np.float32)
    gate_in = z if gated else w.f
    pk = lambda x: dev(x, "bf16")[0].permute(1, 0, 2).contiguous()
    un = lambda t: host(t.permute(1, 0, 2))
    h0 = (0.1 * rng.standard_normal((B, H, dk, dv))).astype(np.float32)
    dhT = (0.1 * rng.standard_normal((B, H, dk, dv))).astype(np.float32)
    q, g, v, dO = pk(w.q), pk(gate_in), pk(w.v), pk(w.dO)
    cud = torch.from_numpy(cu).cuda()
    bd = torch.from_numpy(beta).cuda() if gated else None
    saved = None
    if pair:
        saved = torch.empty(max(binding.hgrn2_saved_states_varlen_bytes(binding.make_shape_varlen(q, v, g, B, chunk)), 256),
                            dtype=torch.uint8, device="cuda")
    o, hT = binding.hgrn2_fwd_varlen(q, g, v, cud, dev(h0), beta=bd, chunk=chunk, saved_states=saved)
    res = binding.hgrn2_bwd_varlen(q, g, v, dO, cud, dev(h0), dev(dhT), beta=bd, want_grad_h0=True, chunk=chunk,
                                   saved_states=saved)
    # the probe on the packed batch: windows restart with every sequence
    gates = oracle.gate(z, beta) if gated else w.f
    for ck in (0, chunk):
        got = float(binding.hgrn2_min_gate_product_varlen(g, cud, beta=bd, chunk=ck).item())
        ref = min([oracle.min_gate_product(gates[:, :, int(cu[b]):int(cu[b + 1])], chunk=ck or 64) for b in range(B)] + [1.0])
        print("    smallest gate product, chunk=%d: %.3e (oracle %.3e)" % (ck, got, ref), flush=True)
        assert abs(got - ref) <= 1e-3 * ref + 1e-44
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


@pytest.mark.parametrize("kind,lens,H,dk,dv,pair", [
    ("ordinary", [150, 0, 37, 260], 2, 64, 64, False),
    ("loguniform32", [200, 1, 333], 2, 128, 128, True),
    ("loguniform", [90, 300, 45], 3, 128, 64, True),
    ("loguniform32", [70, 45, 0, 33, 90, 17, 64, 1, 80, 5, 120, 31, 66, 48, 12, 100] * 3, 16, 128, 128, True),   # groups of sequences
    ("loguniform", [1300, 900], 2, 128, 128, False),      # documents walked in runs
])
def test_chunk_length_chosen_on_the_device_in_a_packed_batch(kind, lens, H, dk, dv, pair):
    """chunk = HGRN2_CHUNK_AUTO for packed batches: the three passes build their own tables and those not called
    for return at once, table kernels included.  The results must be those of the chunk length the probe
    names, bit for bit, stateless or as the training pair (whose kept states lie in a place per alternative)."""
    AUTO = -1
    B, T = len(lens), int(sum(lens))
    print("\n[chunk chosen on the device, packed] %s H=%d dk=%d dv=%d pair=%s lens=%s" % (kind, H, dk, dv, pair, lens), flush=True)
    rng = np.random.default_rng(8300 + T)
    cu = torch.from_numpy(np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)).cuda()
    if kind == "ordinary":
        w = synth.make_sequence(8300 + B, 1, H, T, dk, dv, io_dtype="bf16", lb=0.0, with_dO=True)
    else:
        w = small_gate_workload(8300 + B, 1, H, T, dk, dv, kind)
    pk = lambda x: dev(x, "bf16")[0].permute(1, 0, 2).contiguous()
    q, f, v, dO = pk(w.q), pk(w.f), pk(w.v), pk(w.dO)
    h0 = dev((0.1 * rng.standard_normal((B, H, dk, dv))).astype(np.float32))
    dhT = dev((0.1 * rng.standard_normal((B, H, dk, dv))).astype(np.float32))
    need = [c for c in (0, 32, 16) if float(binding.hgrn2_min_gate_product_varlen(f, cu, chunk=c).item()) > LIMIT][0]
    print("    the probe says: chunk = %d" % need, flush=True)
    assert need == {"ordinary": 0, "loguniform32": 32, "loguniform": 16}[kind]

    def run(chunk, flag):
        saved = None
        if pair:
            saved = torch.empty(max(binding.hgrn2_saved_states_varlen_bytes(binding.make_shape_varlen(q, v, f, B, chunk)), 256),
                                dtype=torch.uint8, device="cuda")
        o, hT = binding.hgrn2_fwd_varlen(q, f, v, cu, h0, chunk=chunk, saved_states=saved, domain_flag=flag)
        return (o, hT) + tuple(binding.hgrn2_bwd_varlen(q, f, v, dO, cu, h0, dhT, want_grad_h0=True, chunk=chunk,
                                                        saved_states=saved, domain_flag=flag))

    flag = torch.zeros(1, dtype=torch.int32, device="cuda")
    got = run(AUTO, flag)
    want = run(need, None)
    torch.cuda.synchronize()
    assert int(flag.item()) == 0
    for name, x, y in zip(("o", "hT", "dq", "df", "dv", "dh0"), got, want):
        assert torch.equal(x, y), "%s differs from the call with chunk = %d" % (name, need)


@pytest.mark.parametrize("dk,dv,B,H", [(64, 64, 2, 3), (128, 128, 8, 8), (128, 64, 1, 2)])
def test_gate_domain_flag(dk, dv, B, H):
    """shape->gate_domain_flag: set by the forward and by the backward kernels exactly when a product of
    up to 32 gates falls below the floor of their reciprocals (the probe says the same), left alone by
    ordinary gates and by the small-gate mode on gates inside ITS domain; never cleared by the library.
    Covers the read-out kernel (64 x 64), the single-pass forward (64 sequences of 128 x 128) and the
    reverse walk of the backward pass."""
    N = 200
    print("\n[domain flag] dk=%d dv=%d B=%d H=%d" % (dk, dv, B, H), flush=True)
    w = small_gate_workload(9100 + dk, B, H, N, dk, dv, "loguniform")
    q, f, v, dO = (dev(x, "bf16") for x in (w.q, w.f, w.v, w.dO))
    ok = synth.make_sequence(9101, B, H, N, dk, dv, io_dtype="bf16", lb=0.0, with_dO=True)
    fo = dev(ok.f, "bf16")
    assert float(binding.hgrn2_min_gate_product(f).item()) < LIMIT < float(binding.hgrn2_min_gate_product(fo).item())
    flag = lambda: torch.zeros(1, dtype=torch.int32, device="cuda")
    a, b, c, d_, e, g = flag(), flag(), flag(), flag(), flag(), flag()
    binding.hgrn2_fwd(q, f, v, domain_flag=a)                     # small gates, ordinary mode: outside the domain
    binding.hgrn2_bwd(q, f, v, dO, domain_flag=b)
    binding.hgrn2_fwd(q, fo, v, domain_flag=c)                    # sigmoid gates: inside
    binding.hgrn2_bwd(q, fo, v, dO, domain_flag=d_)
    binding.hgrn2_fwd(q, f, v, chunk=16, domain_flag=e)           # small gates, reference rows every 16 tokens: inside
    binding.hgrn2_bwd(q, f, v, dO, chunk=16, domain_flag=g)
    torch.cuda.synchronize()
    got = [int(t.item()) for t in (a, b, c, d_, e, g)]
    print("    flags: small gates fwd/bwd %s, ordinary gates %s, small-gate mode %s" % (got[:2], got[2:4], got[4:]), flush=True)
    assert got == [1, 1, 0, 0, 0, 0]
    binding.hgrn2_fwd(q, fo, v, domain_flag=a)                    # the library never clears a flag
    torch.cuda.synchronize()
    assert int(a.item()) == 1
