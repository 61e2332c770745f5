"""GPU parity with the sequence tensors in [B][N][H][d] order (heads side by side inside a token,
what a projection writes): the same seeded inputs as the other parity tests, permuted on the way
in and out, against the fp64 oracle, through the C ABI with layout = HGRN2_LAYOUT_BNHD."""
import numpy as np
import pytest
import torch

import oracle
from paper_2404_07904_amd import binding, synth
from gpu_util import TOL, check, dev, host

pytestmark = pytest.mark.gpu
BNHD = binding.HGRN2_LAYOUT_BNHD


def to_bnhd(t):
    return t.permute(0, 2, 1, 3).contiguous()


def from_bnhd(t):
    return host(t.permute(0, 2, 1, 3))


def run(w, gate_dtype="bf16", with_dh0=True):
    q, f, v, dO = (to_bnhd(dev(x, dt)) for x, dt in ((w.q, "bf16"), (w.f, gate_dtype), (w.v, "bf16"), (w.dO, "bf16")))
    h0, dhT = dev(w.h0), dev(w.dhT)
    o, hT = binding.hgrn2_fwd(q, f, v, h0, layout=BNHD)
    gq, gf, gv, gh0 = binding.hgrn2_bwd(q, f, v, dO, h0, dhT, want_grad_h0=with_dh0, layout=BNHD)
    torch.cuda.synchronize()
    assert o.shape == v.shape and gq.shape == q.shape
    tol = TOL["bf16"]
    ro, rhT = oracle.fwd(w.q, w.f, w.v, w.h0)
    check("o", from_bnhd(o), ro, tol)
    check("hT", host(hT), rhT, tol)
    rq, rf, rv, rh = oracle.bwd(w.q, w.f, w.v, w.dO, w.h0, w.dhT)
    check("dq", from_bnhd(gq), rq, tol)
    check("dv", from_bnhd(gv), rv, tol)
    check("df", from_bnhd(gf), rf, tol)
    if with_dh0:
        check("dh0", host(gh0), rh, tol)


@pytest.mark.parametrize("dk,dv", [(64, 64), (128, 128), (64, 128), (128, 64)])
def test_bnhd_small_shapes(dk, dv):
    print("\n[BNHD] dk=%d dv=%d B=2 H=3 N=203" % (dk, dv), flush=True)
    w = synth.make_sequence(4000 + dk + 2 * dv, 2, 3, 203, dk, dv, io_dtype="bf16", lb=0.2, with_h0=True,
                            with_dO=True, with_dhT=True)
    run(w)


@pytest.mark.parametrize("BH", [(8, 9), (29, 7)])
@pytest.mark.parametrize("gate_dtype", ["bf16", "f32"])
def test_bnhd_fused_forward_paths(BH, gate_dtype):
    B, H = BH
    print("\n[BNHD] fused forward B*H=%d N=130 gate=%s" % (B * H, gate_dtype), flush=True)
    w = synth.make_sequence(4100 + B, B, H, 130, 128, 128, io_dtype="bf16", gate_dtype=gate_dtype, lb=0.3,
                            with_h0=True, with_dO=True, with_dhT=True)
    run(w, gate_dtype=gate_dtype, with_dh0=False)


@pytest.mark.parametrize("N", [1, 63, 64, 65])
def test_bnhd_edge_lengths(N):
    print("\n[BNHD] edge N=%d" % N, flush=True)
    w = synth.make_sequence(4200 + N, 2, 2, N, 64, 64, io_dtype="bf16", lb=0.3, with_h0=True, with_dO=True,
                            with_dhT=True)
    run(w)


def test_bnhd_layer_shape_reduced_batch_gated():
    """Layer shape with a reduced batch (B=2, H=16, N=2048, d=128), gate formed inside the kernels."""
    print("\n[BNHD] gated, B=2 H=16 N=2048 d=128", flush=True)
    B, H, N, d = 2, 16, 2048, 128
    w = synth.make_sequence(4300, B, H, N, d, d, io_dtype="bf16", with_dO=True)
    rng = np.random.default_rng(4301)
    z = synth.bf16_round((1.5 * rng.standard_normal((B, H, N, d), dtype=np.float32)).astype(np.float32))
    beta = rng.uniform(0.0, 0.9, size=(H, d)).astype(np.float32)
    q, zd, v, dO = (to_bnhd(dev(x, "bf16")) for x in (w.q, z, w.v, w.dO))
    bd = torch.from_numpy(beta).cuda()
    o, hT = binding.hgrn2_fwd_gated(q, zd, bd, v, None, layout=BNHD)
    gq, gz, gb, gv, _ = binding.hgrn2_bwd_gated(q, zd, bd, v, dO, None, None, layout=BNHD)
    torch.cuda.synchronize()
    tol = TOL["bf16"]
    ro, rhT = oracle.fwd_gated(w.q, z, beta, w.v, None)
    check("o", from_bnhd(o), ro, tol)
    check("hT", host(hT), rhT, tol)
    rq, rz, rb, rv, _ = oracle.bwd_gated(w.q, z, beta, w.v, w.dO, None, None, want_dh0=False)
    check("dq", from_bnhd(gq), rq, tol)
    check("dv", from_bnhd(gv), rv, tol)
    check("dz", from_bnhd(gz), rz, tol)
    check("dbeta", host(gb), rb, tol)
