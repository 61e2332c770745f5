"""Small gates.  With a reference row every 64 tokens the chunkwise kernels are exact while the gate
product of every half chunk stays above 2^-100; chunk = 16 (32) in the shape asks for reference rows
every 16 (32) tokens (the passes then run on sequences spread to four times (twice) their length),
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
    ("resets", 1, 2, 1100, 64, 128, 0, 16),          # spread to 69 chunks: walked in runs
    ("loguniform32", 2, 2, 300, 128, 64, 1, 32),
    ("loguniform32", 1, 3, 700, 64, 64, 0, 32),
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
    # empty sequences pass through the spreading as well
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
