"""The torch.autograd wrappers are plumbing over the binding: their outputs and gradients must be
the very tensors the C-ABI calls produce (bitwise), gradients must reach every differentiable
argument (initial state and lower bounds included), and a loss that uses only one of the two
outputs must still work (the other output's gradient arrives as None).  Parity of the kernels
with the oracle is covered by the other GPU tests; one case here goes through autograd to the
oracle as an end-to-end check."""
import numpy as np
import pytest
import torch

import oracle
from paper_2404_07904_amd import autograd, binding, synth
from gpu_util import TOL, check, dev, host

pytestmark = pytest.mark.gpu


def leaf(x, dtype="bf16", grad=True):
    t = dev(x, dtype)
    t.requires_grad_(grad)
    return t


def same(a, b):
    assert a.dtype == b.dtype and torch.equal(a, b)


def test_hgrn2_autograd_matches_binding_and_oracle():
    print("\n[autograd] hgrn2 B=2 H=3 N=150 d=64", flush=True)
    w = synth.make_sequence(8100, 2, 3, 150, 64, 64, io_dtype="bf16", lb=0.3, with_h0=True, with_dO=True, with_dhT=True)
    q, f, v = leaf(w.q), leaf(w.f), leaf(w.v)
    h0 = leaf(w.h0, "f32")
    dO, dhT = dev(w.dO, "bf16"), dev(w.dhT)
    o, hT = autograd.hgrn2_recurrence(q, f, v, h0)
    ((o.float() * dO.float()).sum() + (hT * dhT).sum()).backward()
    ro, rhT = binding.hgrn2_fwd(q.detach(), f.detach(), v.detach(), h0.detach())
    rq, rf, rv, rh0 = binding.hgrn2_bwd(q.detach(), f.detach(), v.detach(), dO, h0.detach(), dhT, want_grad_h0=True)
    torch.cuda.synchronize()
    same(o.detach(), ro); same(hT.detach(), rhT)
    same(q.grad, rq); same(f.grad, rf); same(v.grad, rv); same(h0.grad, rh0)
    oq, of, ov, oh = oracle.bwd(w.q, w.f, w.v, w.dO, w.h0, w.dhT)
    for name, g, r in (("dq", q.grad, oq), ("df", f.grad, of), ("dv", v.grad, ov), ("dh0", h0.grad, oh)):
        check(name, host(g), r, TOL["bf16"])


def test_hgrn2_autograd_partial_losses_and_fp32_gates():
    w = synth.make_sequence(8200, 1, 2, 70, 64, 64, io_dtype="bf16", gate_dtype="f32", lb=0.5, with_dO=True, with_dhT=True)
    dO, dhT = dev(w.dO, "bf16"), dev(w.dhT)
    # only o in the loss, no initial state
    q, f, v = leaf(w.q), leaf(w.f, "f32"), leaf(w.v)
    o, hT = autograd.hgrn2_recurrence(q, f, v)
    (o.float() * dO.float()).sum().backward()
    rq, rf, rv, _ = binding.hgrn2_bwd(q.detach(), f.detach(), v.detach(), dO, None, None)
    torch.cuda.synchronize()
    same(q.grad, rq); same(v.grad, rv)
    assert f.grad.dtype == torch.float32 and torch.equal(f.grad, rf.float())
    # only hT in the loss
    q2, f2, v2 = leaf(w.q), leaf(w.f, "f32"), leaf(w.v)
    _, hT2 = autograd.hgrn2_recurrence(q2, f2, v2)
    (hT2 * dhT).sum().backward()
    zq, zf, zv, _ = binding.hgrn2_bwd(q2.detach(), f2.detach(), v2.detach(), torch.zeros_like(dO), None, dhT)
    torch.cuda.synchronize()
    same(v2.grad, zv); assert torch.equal(f2.grad, zf.float())
    assert torch.count_nonzero(q2.grad) == 0          # q does not reach the final state


def test_gated_and_token_major_autograd():
    B, H, N, d = 2, 4, 100, 64
    w = synth.make_sequence(8300, B, H, N, d, d, io_dtype="bf16", with_dO=True)
    rng = np.random.default_rng(8301)
    z = synth.bf16_round((1.5 * rng.standard_normal((B, H, N, d), dtype=np.float32)).astype(np.float32))
    beta = torch.from_numpy(rng.uniform(0, 0.9, (H, d)).astype(np.float32)).cuda().requires_grad_(True)
    perm = lambda x: dev(x, "bf16").permute(0, 2, 1, 3).contiguous()
    q, zz, v = perm(w.q).requires_grad_(True), perm(z).requires_grad_(True), perm(w.v).requires_grad_(True)
    dO = perm(w.dO)
    o, _ = autograd.hgrn2_recurrence_gated(q, zz, beta, v, None, layout=binding.HGRN2_LAYOUT_BNHD)
    (o.float() * dO.float()).sum().backward()
    rq, rz, rb, rv, _ = binding.hgrn2_bwd_gated(q.detach(), zz.detach(), beta.detach(), v.detach(), dO, None, None,
                                                layout=binding.HGRN2_LAYOUT_BNHD)
    torch.cuda.synchronize()
    same(q.grad, rq); same(zz.grad, rz); same(v.grad, rv); same(beta.grad, rb)


def test_varlen_autograd():
    H, d, lens = 3, 64, [40, 0, 90, 7]
    T = sum(lens)
    w = synth.make_sequence(8400, 1, H, T, d, d, io_dtype="bf16", lb=0.3, with_dO=True)
    pk = lambda x: dev(x, "bf16")[0].permute(1, 0, 2).contiguous()
    q, f, v = pk(w.q).requires_grad_(True), pk(w.f).requires_grad_(True), pk(w.v).requires_grad_(True)
    dO = pk(w.dO)
    cu = torch.tensor(np.concatenate([[0], np.cumsum(lens)]), dtype=torch.int32).cuda()
    h0 = torch.randn(len(lens), H, d, d, device="cuda").requires_grad_(True)
    o, hT = autograd.hgrn2_recurrence_varlen(q, f, v, cu, h0)
    ((o.float() * dO.float()).sum() + hT.sum()).backward()
    rq, rf, rv, rh0 = binding.hgrn2_bwd_varlen(q.detach(), f.detach(), v.detach(), dO, cu, h0.detach(),
                                               torch.ones_like(hT), want_grad_h0=True)
    torch.cuda.synchronize()
    same(q.grad, rq); same(f.grad, rf); same(v.grad, rv); same(h0.grad, rh0)


def test_hgrn1_autograd_both_forms():
    B, N, d = 2, 90, 128
    rng = np.random.default_rng(8500)
    mk = lambda: synth.bf16_round((1.5 * rng.standard_normal((B, N, d), dtype=np.float32)).astype(np.float32))
    zf, zi, zo, dy = mk(), mk(), mk(), mk()
    beta = torch.from_numpy(rng.uniform(0, 0.9, d).astype(np.float32)).cuda().requires_grad_(True)
    a, b_, c = leaf(zf), leaf(zi), leaf(zo)
    h0 = torch.randn(B, d, device="cuda").requires_grad_(True)
    dyd = dev(dy, "bf16")
    y, hN = autograd.hgrn1_layer(a, b_, c, beta, h0)
    ((y.float() * dyd.float()).sum() + hN.sum()).backward()
    rf, ri, ro, rb, rh0 = binding.hgrn1_bwd_act(a.detach(), b_.detach(), c.detach(), beta.detach(), dyd, h0.detach(),
                                                torch.ones_like(hN), want_grad_h0=True)
    torch.cuda.synchronize()
    same(a.grad, rf); same(b_.grad, ri); same(c.grad, ro); same(beta.grad, rb); same(h0.grad, rh0)
    # plain form, gates in (0, 1)
    f = torch.sigmoid(dev(zf, "bf16").float()).bfloat16().requires_grad_(True)
    i, o = leaf(zi), torch.sigmoid(dev(zo, "bf16").float()).bfloat16().requires_grad_(True)
    y2, _ = autograd.hgrn1_recurrence(f, i, o)
    (y2.float() * dyd.float()).sum().backward()
    pf, pi, po, _ = binding.hgrn1_bwd(f.detach(), i.detach(), o.detach(), dyd, None, None)
    torch.cuda.synchronize()
    same(f.grad, pf); same(i.grad, pi); same(o.grad, po)


def test_autograd_passes_the_small_gate_mode_on():
    """chunk=16 reaches both library calls of a wrapper: same tensors as the binding with chunk=16."""
    w = synth.make_sequence(8300, 1, 2, 90, 64, 64, io_dtype="bf16", lb=0.3, with_dO=True)
    dO = dev(w.dO, "bf16")
    q, f, v = leaf(w.q), leaf(w.f), leaf(w.v)
    o, _ = autograd.hgrn2_recurrence(q, f, v, chunk=16)
    (o.float() * dO.float()).sum().backward()
    ro, _ = binding.hgrn2_fwd(q.detach(), f.detach(), v.detach(), None, chunk=16)
    rq, rf, rv, _ = binding.hgrn2_bwd(q.detach(), f.detach(), v.detach(), dO, None, None, chunk=16)
    torch.cuda.synchronize()
    same(o.detach(), ro); same(q.grad, rq); same(f.grad, rf); same(v.grad, rv)
    beta = torch.full((2, 64), 0.2, device="cuda", requires_grad=True)
    q2, z2, v2 = leaf(w.q), leaf(w.f), leaf(w.v)
    o2, _ = autograd.hgrn2_recurrence_gated(q2, z2, beta, v2, chunk=16)
    (o2.float() * dO.float()).sum().backward()
    g = binding.hgrn2_bwd_gated(q2.detach(), z2.detach(), beta.detach(), v2.detach(), dO, None, None, chunk=16)
    torch.cuda.synchronize()
    same(q2.grad, g[0]); same(z2.grad, g[1]); same(beta.grad, g[2]); same(v2.grad, g[3])
