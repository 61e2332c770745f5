"""The training pair hgrn2_fwd_saving / hgrn2_bwd_saved: the forward pass keeps the state entering
every chunk, the backward pass reads it instead of recomputing it.  Checked against the fp64 oracle
(max|x-y|/max|y| <= 2e-2, bf16 storage) on shapes that take the single-pass forward (both of its grid
shapes), the sweep + read-out forward, runs, ragged lengths, both layouts and the gate of Eq. 2 formed
in the kernels.  The forward outputs must equal those of hgrn2_fwd bit for bit; the gradients need not
equal those of the stateless hgrn2_bwd (the single-pass forward carries its fp32 state in another
scaling than the sweep, so the bf16 states can differ in the last bit), which is printed."""
import numpy as np
import pytest
import torch

import oracle
from paper_2404_07904_amd import binding, synth
from gpu_util import TOL, check, dev, host

pytestmark = pytest.mark.gpu
BNHD = binding.HGRN2_LAYOUT_BNHD


@pytest.mark.parametrize("B,H,N,dk,dv,layout", [
    (8, 8, 300, 128, 128, 0),       # 64 sequences: single-pass forward, two workgroups per sequence
    (9, 16, 200, 128, 128, 1),      # 144 sequences: one workgroup per sequence, token-major
    (2, 3, 203, 64, 64, 0),         # sweep + read-out forward
    (1, 2, 1100, 128, 64, 1),       # reverse walk in runs
    (2, 16, 1088, 128, 128, 0),     # 32 sequences of 17 chunks: single-pass forward on runs
])
def test_training_pair(B, H, N, dk, dv, layout):
    print("\n[saved states] B=%d H=%d N=%d dk=%d dv=%d layout=%d" % (B, H, N, dk, dv, layout), flush=True)
    w = synth.make_sequence(6100 + N + dk, B, H, N, dk, dv, io_dtype="bf16", lb=0.3, with_h0=True, with_dO=True,
                            with_dhT=True)
    put = (lambda t: t.permute(0, 2, 1, 3).contiguous()) if layout == BNHD else (lambda t: t)
    get = (lambda t: host(t.permute(0, 2, 1, 3))) if layout == BNHD else host
    q, f, v, dO = (put(dev(x, "bf16")) for x in (w.q, w.f, w.v, w.dO))
    h0, dhT = dev(w.h0), dev(w.dhT)
    o, hT, saved = binding.hgrn2_fwd_saving(q, f, v, h0, layout=layout)
    dq, df, dv_, dh0 = binding.hgrn2_bwd_saved(q, f, v, saved, dO, dhT, want_grad_h0=True, layout=layout)
    o2, hT2 = binding.hgrn2_fwd(q, f, v, h0, layout=layout)
    ref = binding.hgrn2_bwd(q, f, v, dO, h0, dhT, want_grad_h0=True, layout=layout)
    torch.cuda.synchronize()
    ro, rhT = oracle.fwd(w.q, w.f, w.v, w.h0)
    rq, rf, rv, rh = oracle.bwd(w.q, w.f, w.v, w.dO, w.h0, w.dhT)
    tol = TOL["bf16"]
    check("o", get(o), ro, tol); check("hT", host(hT), rhT, tol)
    check("dq", get(dq), rq, tol); check("df", get(df), rf, tol); check("dv", get(dv_), rv, tol)
    check("dh0", host(dh0), rh, tol)
    assert torch.equal(o, o2) and torch.equal(hT, hT2)
    same = [torch.equal(a, b) for a, b in zip((dq, df, dv_, dh0), ref)]
    print("    bitwise equal to the stateless backward:", same, flush=True)


def test_training_pair_gate_formed_in_the_kernels():
    B, H, N, d = 4, 16, 260, 128
    print("\n[saved states, gated] B=%d H=%d N=%d" % (B, H, N), flush=True)
    rng = np.random.default_rng(6200)
    w = synth.make_sequence(6201, B, H, N, d, d, io_dtype="bf16", with_h0=True, with_dO=True, with_dhT=True)
    z = synth.bf16_round(rng.standard_normal((B, H, N, d)).astype(np.float32))
    beta = rng.uniform(0.0, 0.9, size=(H, d)).astype(np.float32)
    q, zd, v, dO = dev(w.q, "bf16"), dev(z, "bf16"), dev(w.v, "bf16"), dev(w.dO, "bf16")
    bd = torch.from_numpy(beta).cuda()
    o, hT, saved = binding.hgrn2_fwd_saving(q, zd, v, dev(w.h0), beta=bd)
    gq, gz, gv, gh0, gb = binding.hgrn2_bwd_saved(q, zd, v, saved, dO, dev(w.dhT), beta=bd, want_grad_h0=True)
    torch.cuda.synchronize()
    ro, rhT = oracle.fwd_gated(w.q, z, beta, w.v, w.h0)
    rq, rz, rb, rv, rh = oracle.bwd_gated(w.q, z, beta, w.v, w.dO, w.h0, w.dhT)
    tol = TOL["bf16"]
    check("o", host(o), ro, tol); check("hT", host(hT), rhT, tol)
    check("dq", host(gq), rq, tol); check("dz", host(gz), rz, tol); check("dbeta", host(gb), rb, tol)
    check("dv", host(gv), rv, tol); check("dh0", host(gh0), rh, tol)


def test_training_pair_empty_and_errors():
    e = torch.empty((2, 3, 0, 64), dtype=torch.bfloat16, device="cuda")
    h0 = torch.randn((2, 3, 64, 64), dtype=torch.float32, device="cuda")
    o, hT, saved = binding.hgrn2_fwd_saving(e, e, e, h0)
    dq, df, dv_, dh0 = binding.hgrn2_bwd_saved(e, e, e, saved, e, h0, want_grad_h0=True)
    torch.cuda.synchronize()
    assert torch.equal(hT, h0) and torch.equal(dh0, h0)
    q = torch.zeros((1, 1, 64, 64), dtype=torch.bfloat16, device="cuda")
    small = torch.empty(256, dtype=torch.uint8, device="cuda")
    with pytest.raises(binding.Hgrn2Error) as err:
        binding.hgrn2_fwd_saving(q, q, q, saved_states=small)
    assert err.value.status == 4
    q32 = torch.zeros((1, 1, 64, 128), dtype=torch.float32, device="cuda")      # fp32 storage: heads of 64 x 64 only
    with pytest.raises(binding.Hgrn2Error) as err:
        binding.hgrn2_fwd_saving(q32, q32, q32)
    assert err.value.status == 3
