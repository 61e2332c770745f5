"""GPU parity of the passes that form the lower-bounded gate of Eq. 2 inside the kernels
(hgrn2_fwd_gated, hgrn2_bwd_gated, hgrn2_cumax) against the fp64 oracle, through the C ABI.
The pre-activations z and the bounds beta are drawn here (seeded), z is rounded once to its
storage type, and the same rounded values go to both sides.  Tolerance as for the plain passes:
max|x-y|/max|y| <= 2e-2 per tensor (bf16 storage); the bounds and their gradient are fp32."""
import numpy as np
import pytest
import torch

import oracle
from paper_2404_07904_amd import binding, synth
from gpu_util import TOL, check, dev, host

pytestmark = pytest.mark.gpu


def make(seed, B, H, N, dk, dv, gate_dtype="bf16", beta_hi=0.9, layer_beta=None, with_state=True):
    w = synth.make_sequence(seed, B, H, N, dk, dv, io_dtype="bf16", with_h0=with_state, with_dO=True,
                            with_dhT=with_state)
    rng = np.random.default_rng(seed + 1)
    z = (1.5 * rng.standard_normal((B, H, N, dk), dtype=np.float32)).astype(np.float32)
    z = synth.bf16_round(z) if gate_dtype == "bf16" else z
    if layer_beta is None:
        beta = rng.uniform(0.0, beta_hi, size=(H, dk)).astype(np.float32)
    else:
        beta = np.full((H, dk), layer_beta, dtype=np.float32)
    return w, z, beta


def run(w, z, beta, gate_dtype="bf16", with_dh0=True):
    q, v, dO = dev(w.q, "bf16"), dev(w.v, "bf16"), dev(w.dO, "bf16")
    zd = dev(z, gate_dtype)
    bd = torch.from_numpy(beta).cuda()
    h0, dhT = dev(w.h0), dev(w.dhT)
    o, hT = binding.hgrn2_fwd_gated(q, zd, bd, v, h0)
    gq, gz, gb, gv, gh0 = binding.hgrn2_bwd_gated(q, zd, bd, v, dO, h0, dhT, want_grad_h0=with_dh0)
    torch.cuda.synchronize()
    tol = TOL["bf16"]
    ro, rhT = oracle.fwd_gated(w.q, z, beta, w.v, w.h0)
    check("o", host(o), ro, tol)
    check("hT", host(hT), rhT, tol)
    rq, rz, rb, rv, rh = oracle.bwd_gated(w.q, z, beta, w.v, w.dO, w.h0, w.dhT)
    check("dq", host(gq), rq, tol)
    check("dv", host(gv), rv, tol)
    check("dz", host(gz), rz, tol)
    check("dbeta", host(gb), rb, tol)
    if with_dh0:
        check("dh0", host(gh0), rh, tol)
    return gb


@pytest.mark.parametrize("dk,dv", [(64, 64), (128, 128), (64, 128), (128, 64)])
def test_gated_small_shapes_two_kernel_forward(dk, dv):
    print("\n[gated] dk=%d dv=%d B*H=6 N=203" % (dk, dv), flush=True)
    w, z, beta = make(3000 + dk + 2 * dv, 2, 3, 203, dk, dv)
    run(w, z, beta)


@pytest.mark.parametrize("gate_dtype", ["bf16", "f32"])
@pytest.mark.parametrize("BH", [(8, 9), (29, 7)])
def test_gated_fused_forward_paths(BH, gate_dtype):
    """B*H = 72 (two workgroups per sequence) and 203 (one) at d = 128: the single-pass forward."""
    B, H = BH
    print("\n[gated] fused forward B*H=%d N=130 gate=%s" % (B * H, gate_dtype), flush=True)
    w, z, beta = make(3100 + B, B, H, 130, 128, 128, gate_dtype=gate_dtype)
    run(w, z, beta, gate_dtype=gate_dtype, with_dh0=False)


@pytest.mark.parametrize("N", [0, 1, 63, 64, 65])
def test_gated_edge_lengths(N):
    print("\n[gated] edge N=%d" % N, flush=True)
    w, z, beta = make(3200 + N, 2, 2, N, 64, 64)
    run(w, z, beta)


def test_gated_zero_bound_equals_plain_sigmoid_gate():
    """beta = 0: the gate is the plain logistic gate; the result must match the plain entry points
    fed with that gate up to the rounding of f to its storage type."""
    print("\n[gated] beta = 0 against hgrn2_fwd with f = sigmoid(z)", flush=True)
    w, z, beta = make(3300, 2, 4, 192, 128, 128, layer_beta=0.0)
    run(w, z, beta)
    f = (1.0 / (1.0 + np.exp(-z.astype(np.float64)))).astype(np.float32)
    o1, _ = binding.hgrn2_fwd_gated(dev(w.q, "bf16"), dev(z, "bf16"), torch.zeros(4, 128, device="cuda"),
                                    dev(w.v, "bf16"), dev(w.h0))
    o2, _ = binding.hgrn2_fwd(dev(w.q, "bf16"), dev(f, "f32"), dev(w.v, "bf16"), dev(w.h0))
    check("o vs plain", host(o1), host(o2), 5e-3)


def test_gated_layer_shape_reduced_batch_and_determinism():
    """Bounds of layer 12 of 24 (0.5 on every channel) at the layer shape with a reduced batch; two
    runs must agree bit for bit, the reduction over batch and time included."""
    print("\n[gated] layer 12 bounds, B=2 H=16 N=2048 d=128", flush=True)
    w, z, beta = make(3400, 2, 16, 2048, 128, 128, layer_beta=synth.layer_lower_bound(12), with_state=False)
    g1 = run(w, z, beta, with_dh0=False)
    g2 = run(w, z, beta, with_dh0=False)
    assert torch.equal(g1, g2)


def test_cumax_parity():
    rng = np.random.default_rng(9)
    gamma = rng.standard_normal((24, 2048)).astype(np.float32)
    beta = binding.hgrn2_cumax(torch.from_numpy(gamma).cuda())
    torch.cuda.synchronize()
    ref = oracle.cumax(gamma)
    check("beta", host(beta), ref, 1e-5)
    assert float(beta[0].abs().max()) == 0.0
    uni = binding.hgrn2_cumax(torch.full((24, 64), 0.25, device="cuda"))
    check("uniform", host(uni), np.broadcast_to((np.arange(24) / 24.0)[:, None], (24, 64)), 1e-6)


@pytest.mark.parametrize("dk,dv", [(64, 64), (128, 128), (64, 128), (128, 64)])
@pytest.mark.parametrize("gate_dtype", ["bf16", "f32"])
def test_gated_decode_steps(dk, dv, gate_dtype):
    """Twelve consecutive decode steps from the gate's pre-activations, in place, against the oracle's
    step fed with the gate of Eq. 2; the fp32 state after the last step is compared too, at the fp32
    tolerance of 1e-4 (the gate's exp / rcp approximations leave about 2e-7)."""
    B, H, T = 3, 5, 12
    print("\n[gated step] dk=%d dv=%d gate=%s" % (dk, dv, gate_dtype), flush=True)
    rng = np.random.default_rng(7700 + dk + 2 * dv)
    q = synth.bf16_round(rng.standard_normal((T, B, H, dk), dtype=np.float32))
    v = synth.bf16_round(rng.standard_normal((T, B, H, dv), dtype=np.float32))
    z = (1.5 * rng.standard_normal((T, B, H, dk), dtype=np.float32)).astype(np.float32)
    z = synth.bf16_round(z) if gate_dtype == "bf16" else z
    beta = rng.uniform(0.0, 0.9, size=(H, dk)).astype(np.float32)
    s0 = (0.1 * rng.standard_normal((B, H, dk, dv))).astype(np.float32)
    qd, vd, zd = dev(q, "bf16"), dev(v, "bf16"), dev(z, gate_dtype)
    bd = torch.from_numpy(beta).cuda()
    st = dev(s0)
    ref_state = s0.astype(np.float64).copy()
    for t in range(T):
        o = binding.hgrn2_step_gated(qd[t], zd[t], bd, vd[t], st)
        f_t = oracle.gate(z[t][:, :, None, :], beta)[:, :, 0, :]
        ro = oracle.step(q[t], f_t, v[t], ref_state)
        torch.cuda.synchronize()
        check("o[%d]" % t, host(o), ro, TOL["bf16"])
    check("state", host(st), ref_state, TOL["f32"])


@pytest.mark.parametrize("case", ["bf16", "f32", "bnhd", "gated", "ragged"])
def test_min_gate_product_probe(case):
    """hgrn2_min_gate_product against the oracle's half-chunk minimum (products of 32 fp32 factors:
    1e-4 relative), and what it is for: an input that leaves the stated domain is reported as such."""
    rng = np.random.default_rng(7800)
    B, H, N, dk = 2, 3, 203 if case == "ragged" else 256, 64
    lo = 2.0 ** -100
    if case == "gated":
        z = synth.bf16_round((2.0 * rng.standard_normal((B, H, N, dk), dtype=np.float32)).astype(np.float32))
        beta = rng.uniform(0.0, 0.5, size=(H, dk)).astype(np.float32)
        got = binding.hgrn2_min_gate_product(dev(z, "bf16"), torch.from_numpy(beta).cuda())
        ref = oracle.min_gate_product(oracle.gate(z, beta))
    else:
        f = rng.uniform(0.2, 1.0, (B, H, N, dk)).astype(np.float32)
        dt = "f32" if case == "f32" else "bf16"
        f = f if dt == "f32" else synth.bf16_round(f)
        fd = dev(f, dt)
        if case == "bnhd":
            got = binding.hgrn2_min_gate_product(fd.permute(0, 2, 1, 3).contiguous(), layout=binding.HGRN2_LAYOUT_BNHD)
        else:
            got = binding.hgrn2_min_gate_product(fd)
        ref = oracle.min_gate_product(f)
    torch.cuda.synchronize()
    print("\n[domain probe] %s: %.6e (oracle %.6e)" % (case, float(got), ref), flush=True)
    assert abs(float(got) - ref) <= 1e-4 * ref
    assert float(got) > lo
    # a run of small gates in one channel takes the call out of the domain, and the probe says so
    bad = np.ones((1, 1, 128, 64), dtype=np.float32)
    bad[0, 0, 64:96, 5] = 0.05
    got = float(binding.hgrn2_min_gate_product(dev(bad, "bf16")))
    torch.cuda.synchronize()
    assert got < lo and abs(got - oracle.min_gate_product(synth.bf16_round(bad))) <= 1e-3 * got
