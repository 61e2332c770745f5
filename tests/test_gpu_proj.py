"""Input side of the HGRU2 token mixer (Eq. 1) on the GPU -- hgru2_proj_fwd / hgru2_proj_bwd, the bf16
matrix product with bias and activation in its epilogue -- against the fp64 oracle, alone and as
the layer Eq. 1 -> Eq. 2 -> Eq. 3 (projection, hgrn2_fwd_gated on its token-major outputs, and the
whole reverse mode).  Inputs are rounded to bf16 once and the oracle sees the rounded values.
Tolerance: max|x-y|/max|y| <= 2e-2 per tensor (bf16 storage, fp32 accumulation)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2404_07904_amd import binding, synth
from gpu_util import TOL, check, dev, host

pytestmark = pytest.mark.gpu
BNHD = binding.HGRN2_LAYOUT_BNHD


def weights(seed, d):
    rng = np.random.default_rng(seed)
    w3 = synth.bf16_round((rng.standard_normal((3 * d, d)) / np.sqrt(d)).astype(np.float32))
    b3 = (0.5 * rng.standard_normal(3 * d)).astype(np.float32)
    return w3, b3


def split(w3, b3, d):
    return w3[:d], w3[d:2 * d], w3[2 * d:], b3[:d], b3[d:2 * d], b3[2 * d:]


@pytest.mark.parametrize("B,N,d", [(1, 256, 256), (3, 77, 256), (2, 300, 512), (1, 1, 256), (4, 129, 1024),
                                   (2, 160, 512), (1, 96, 1024), (1, 64, 3072)])   # whole 64-token steps of the dW3 product; a width whose dW3 takes 256-row tiles
def test_proj_fwd_bwd(B, N, d):
    print("\n[proj] B=%d N=%d d=%d" % (B, N, d), flush=True)
    rng = np.random.default_rng(9200 + N + d)
    x = synth.bf16_round(rng.standard_normal((B, N, d)).astype(np.float32))
    w3, b3 = weights(9201 + d, d)
    gz, gv, gq = (synth.bf16_round(rng.standard_normal((B, N, d)).astype(np.float32)) for _ in range(3))
    xd, wd, bd = dev(x, "bf16"), dev(w3, "bf16"), dev(b3)
    z, v, q, av = binding.hgru2_proj_fwd(xd, wd, bd)
    dx, dw, db = binding.hgru2_proj_bwd(xd, wd, q, av, dev(gz, "bf16"), dev(gv, "bf16"), dev(gq, "bf16"))
    torch.cuda.synchronize()
    U, V, W, bu, bv, bw = split(w3, b3, d)
    rz, ri, ro = oracle.hgru2_proj(x, U, V, W, bu, bv, bw)
    tol = TOL["bf16"]
    check("z", host(z), rz, tol); check("v", host(v), ri, tol); check("q", host(q), ro, tol)
    check("av", host(av), x.astype(np.float64) @ V.astype(np.float64).T + bv, tol)
    rdx, rdU, rdV, rdW, rbu, rbv, rbw = oracle.hgru2_proj_bwd(x, U, V, W, bu, bv, bw, gz, gv, gq)
    check("dx", host(dx), rdx, tol)
    check("dw3", host(dw), np.concatenate([rdU, rdV, rdW], axis=0), tol)
    check("db3", host(db), np.concatenate([rbu, rbv, rbw]), tol)


def test_proj_without_av_and_empty():
    d = 256
    w3, b3 = weights(9300, d)
    x = synth.bf16_round(np.random.default_rng(9301).standard_normal((2, 40, d)).astype(np.float32))
    z, v, q, av = binding.hgru2_proj_fwd(dev(x, "bf16"), dev(w3, "bf16"), dev(b3), keep_av=False)
    z2, v2, q2, _ = binding.hgru2_proj_fwd(dev(x, "bf16"), dev(w3, "bf16"), dev(b3))
    torch.cuda.synchronize()
    assert av is None and torch.equal(z, z2) and torch.equal(v, v2) and torch.equal(q, q2)
    e = torch.empty((0, d), dtype=torch.bfloat16, device="cuda")
    binding.hgru2_proj_fwd(e, dev(w3, "bf16"), dev(b3))
    dx, dw, db = binding.hgru2_proj_bwd(e, dev(w3, "bf16"), e, e, e, e, e)
    torch.cuda.synchronize()
    assert float(dw.abs().max()) == 0.0 and float(db.abs().max()) == 0.0
    with pytest.raises(binding.Hgrn2Error) as err:
        binding.hgru2_proj_fwd(torch.zeros((4, 192), dtype=torch.bfloat16, device="cuda"),
                               torch.zeros((576, 192), dtype=torch.bfloat16, device="cuda"), torch.zeros(576, device="cuda"))
    assert err.value.status == 3


@pytest.mark.parametrize("B,N,d,H", [(2, 200, 256, 2), (1, 333, 512, 4)])
def test_layer_projection_recurrence_and_reverse_mode(B, N, d, H):
    """Eq. 1 -> Eq. 2 -> Eq. 3: projection, then hgrn2_fwd_gated on its token-major outputs (no copy in
    between), then the reverse mode back to x, the weights, the biases and beta."""
    print("\n[layer] B=%d N=%d d=%d H=%d" % (B, N, d, H), flush=True)
    dh = d // H
    rng = np.random.default_rng(9400 + d)
    x = synth.bf16_round(rng.standard_normal((B, N, d)).astype(np.float32))
    w3, b3 = weights(9401 + d, d)
    beta = rng.uniform(0.0, 0.8, size=d).astype(np.float32)
    dy = synth.bf16_round(rng.standard_normal((B, N, d)).astype(np.float32))
    h0 = (0.1 * rng.standard_normal((B, H, dh, dh))).astype(np.float32)
    dhT = (0.1 * rng.standard_normal((B, H, dh, dh))).astype(np.float32)
    xd, wd, bd = dev(x, "bf16"), dev(w3, "bf16"), dev(b3)
    betad = torch.from_numpy(beta.reshape(H, dh)).cuda()
    z, v, q, av = binding.hgru2_proj_fwd(xd, wd, bd)
    as4 = lambda t: t.view(B, N, H, dh)
    y, hT = binding.hgrn2_fwd_gated(as4(q), as4(z), betad, as4(v), dev(h0), layout=BNHD)
    gq, gz, gb, gv, gh0 = binding.hgrn2_bwd_gated(as4(q), as4(z), betad, as4(v), as4(dev(dy, "bf16")), dev(h0), dev(dhT),
                                                  want_grad_h0=True, layout=BNHD)
    dx, dw, db = binding.hgru2_proj_bwd(xd, wd, q, av, gz.view(B, N, d), gv.view(B, N, d), gq.view(B, N, d))
    torch.cuda.synchronize()
    U, V, W, bu, bv, bw = split(w3, b3, d)
    ry, rhT = oracle.hgru2_layer_fwd(x, U, V, W, bu, bv, bw, beta, H, h0)
    g = oracle.hgru2_layer_bwd(x, U, V, W, bu, bv, bw, beta, H, dy, h0, dhT)
    tol = TOL["bf16"]
    check("y", host(y).reshape(B, N, d), ry, tol); check("hT", host(hT), rhT, tol)
    check("dx", host(dx), g[0], tol)
    check("dw3", host(dw), np.concatenate([g[1], g[2], g[3]], axis=0), tol)
    check("db3", host(db), np.concatenate([g[4], g[5], g[6]]), tol)
    check("dbeta", host(gb).reshape(-1), g[7], tol); check("dh0", host(gh0), g[8], tol)


def test_proj_full_width_sampled_rows():
    """The benchmark's projection (16384 tokens, width 2048): 512 seeded rows of z, v, q against the
    oracle (each row of the product is independent of the others)."""
    M, d = 16384, 2048
    print("\n[proj] full width: M=%d d=%d" % (M, d), flush=True)
    gen = torch.Generator(device="cuda").manual_seed(9500)
    xd = torch.randn((M, d), generator=gen, device="cuda").to(torch.bfloat16)
    w3, b3 = weights(9501, d)
    z, v, q, av = binding.hgru2_proj_fwd(xd, dev(w3, "bf16"), dev(b3))
    torch.cuda.synchronize()
    rows = np.sort(np.random.default_rng(9502).choice(M, 512, replace=False))
    rows[0], rows[-1] = 0, M - 1
    rt = torch.from_numpy(rows).cuda()
    xs = host(xd[rt])
    U, V, W, bu, bv, bw = split(w3, b3, d)
    rz, ri, ro = oracle.hgru2_proj(xs[None], U, V, W, bu, bv, bw)
    tol = TOL["bf16"]
    check("z", host(z[rt]), rz[0], tol); check("v", host(v[rt]), ri[0], tol); check("q", host(q[rt]), ro[0], tol)
