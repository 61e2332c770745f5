"""GPU parity of the element-wise HGRN1 recurrence (hgrn1_fwd, hgrn1_bwd) against the fp64 oracle,
through the C ABI.  Inputs: i, dy ~ N(0,1), o = sigmoid(N(0,1)), f = lb + (1 - lb) sigmoid(N(0,1))
(the gate shape of Eq. 2), rounded once to the storage type; the same rounded values go to both
sides.  Tolerance: max|x-y|/max|y| <= 2e-2 per tensor (bf16 storage)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2404_07904_amd import binding, synth
from gpu_util import TOL, check, dev, host

pytestmark = pytest.mark.gpu


def make(seed, B, N, d, lb=0.3, gate_dtype="bf16"):
    rng = np.random.default_rng(seed)
    sig = lambda z: 1.0 / (1.0 + np.exp(-z))
    i = synth.bf16_round(rng.standard_normal((B, N, d), dtype=np.float32))
    o = synth.bf16_round(sig(rng.standard_normal((B, N, d))).astype(np.float32))
    f = (lb + (1.0 - lb) * sig(rng.standard_normal((B, N, d)))).astype(np.float32)
    f = np.minimum(synth.bf16_round(f) if gate_dtype == "bf16" else f, np.float32(1.0))
    dy = synth.bf16_round(rng.standard_normal((B, N, d), dtype=np.float32))
    h0 = rng.standard_normal((B, d)).astype(np.float32)
    dhN = rng.standard_normal((B, d)).astype(np.float32)
    return f, i, o, dy, h0, dhN


def run(f, i, o, dy, h0, dhN, gate_dtype="bf16"):
    fd, idv, od, dyd = dev(f, gate_dtype), dev(i, "bf16"), dev(o, "bf16"), dev(dy, "bf16")
    h0d = None if h0 is None else dev(h0)
    dhNd = None if dhN is None else dev(dhN)
    y, hN = binding.hgrn1_fwd(fd, idv, od, h0d)
    gf, gi, go, gh0 = binding.hgrn1_bwd(fd, idv, od, dyd, h0d, dhNd, want_grad_h0=True)
    torch.cuda.synchronize()
    tol = TOL["bf16"]
    ry, rh = oracle.hgrn1_fwd(f, i, o, h0)
    check("y", host(y), ry, tol)
    check("hN", host(hN), rh, 3e-5)
    rf, ri, ro, rh0 = oracle.hgrn1_bwd(f, i, o, dy, h0, dhN)
    check("df", host(gf), rf, tol)
    check("di", host(gi), ri, tol)
    check("do", host(go), ro, tol)
    check("dh0", host(gh0), rh0, 3e-5)
    # the same as a training pair: the forward pass leaves the segment states in the workspace,
    # hgrn1_bwd_saved reads them instead of walking f and i forwards again
    B, N, d = i.shape
    ws = torch.empty(max(binding.hgrn1_workspace_bytes(B, N, d), 256), dtype=torch.uint8, device="cuda")
    y2, hN2 = binding.hgrn1_fwd(fd, idv, od, h0d, workspace=ws)
    gf2, gi2, go2, gh02 = binding.hgrn1_bwd(fd, idv, od, dyd, h0d, dhNd, want_grad_h0=True, workspace=ws, saved=True)
    torch.cuda.synchronize()
    check("y (pair)", host(y2), ry, tol)
    check("df (saved)", host(gf2), rf, tol)
    check("di (saved)", host(gi2), ri, tol)
    check("do (saved)", host(go2), ro, tol)
    check("dh0 (saved)", host(gh02), rh0, 3e-5)


@pytest.mark.parametrize("d", [64, 128, 384])
@pytest.mark.parametrize("gate_dtype", ["bf16", "f32"])
def test_hgrn1_ragged(d, gate_dtype):
    print("\n[hgrn1] B=3 N=203 d=%d gate=%s" % (d, gate_dtype), flush=True)
    run(*make(5000 + d, 3, 203, d, gate_dtype=gate_dtype), gate_dtype=gate_dtype)


@pytest.mark.parametrize("N", [0, 1, 31, 32, 33, 64, 65, 97, 255, 256, 257, 511, 512, 513, 545, 1100])
def test_hgrn1_edge_lengths(N):
    print("\n[hgrn1] edge N=%d" % N, flush=True)
    run(*make(5100 + N, 2, N, 128))


def test_hgrn1_no_states():
    f, i, o, dy, _, _ = make(5200, 2, 100, 256)
    print("\n[hgrn1] no h0 / grad_hN", flush=True)
    run(f, i, o, dy, None, None)


def test_hgrn1_gate_extremes():
    """f = 1 freezes the state at h0, f = 0 copies the input."""
    f, i, o, dy, h0, dhN = make(5300, 1, 70, 128)
    f[:, :, :64] = 1.0
    f[:, :, 64:] = 0.0
    print("\n[hgrn1] gates 1 and 0", flush=True)
    run(f, i, o, dy, h0, dhN)


@pytest.mark.parametrize("lb", [0.0, 0.5, 23.0 / 24.0])
def test_hgrn1_layer_shape(lb):
    """Model width 2048 at sequence length 2048, B = 8 (the layer the HGRN2 benchmark shape comes from)."""
    print("\n[hgrn1] B=8 N=2048 d=2048 lb=%.3f" % lb, flush=True)
    run(*make(5400, 8, 2048, 2048, lb=lb))


def test_hgrn1_long_sequence_gates_near_one():
    print("\n[hgrn1] B=2 N=16384 d=2048, f in [0.99, 1], fp32 gates", flush=True)
    run(*make(5500, 2, 16384, 2048, lb=0.99, gate_dtype="f32"), gate_dtype="f32")


# ------------------------------------------------------------------ activations formed inside the kernels
def make_act(seed, B, N, d, gate_dtype="bf16", beta_max=0.9):
    """Pre-activations zf, zi, zo ~ 1.5 N(0,1), rounded once to their storage type; beta ~ U(0, beta_max)."""
    rng = np.random.default_rng(seed)
    mk = lambda: synth.bf16_round((1.5 * rng.standard_normal((B, N, d), dtype=np.float32)).astype(np.float32))
    zf = (1.5 * rng.standard_normal((B, N, d), dtype=np.float32)).astype(np.float32)
    zf = synth.bf16_round(zf) if gate_dtype == "bf16" else zf
    zi, zo = mk(), mk()
    beta = rng.uniform(0.0, beta_max, size=d).astype(np.float32)
    dy = synth.bf16_round(rng.standard_normal((B, N, d), dtype=np.float32))
    h0 = rng.standard_normal((B, d)).astype(np.float32)
    dhN = rng.standard_normal((B, d)).astype(np.float32)
    return zf, zi, zo, beta, dy, h0, dhN


def run_act(zf, zi, zo, beta, dy, h0, dhN, gate_dtype="bf16"):
    zfd, zid, zod, dyd = dev(zf, gate_dtype), dev(zi, "bf16"), dev(zo, "bf16"), dev(dy, "bf16")
    bd = torch.from_numpy(beta).cuda()
    h0d = None if h0 is None else dev(h0)
    dhNd = None if dhN is None else dev(dhN)
    y, hN = binding.hgrn1_fwd_act(zfd, zid, zod, bd, h0d)
    gf, gi, go, gb, gh0 = binding.hgrn1_bwd_act(zfd, zid, zod, bd, dyd, h0d, dhNd, want_grad_h0=True)
    torch.cuda.synchronize()
    tol = TOL["bf16"]
    ry, rh = oracle.hgrn1_fwd_act(zf, zi, zo, beta, h0)
    check("y", host(y), ry, tol)
    check("hN", host(hN), rh, tol)           # i is rounded to bf16 once it is formed
    rf, ri, ro, rb, rh0 = oracle.hgrn1_bwd_act(zf, zi, zo, beta, dy, h0, dhN)
    check("dzf", host(gf), rf, tol)
    check("dzi", host(gi), ri, tol)
    check("dzo", host(go), ro, tol)
    check("dbeta", host(gb), rb, tol)
    check("dh0", host(gh0), rh0, tol)
    B, N, d = zi.shape
    ws = torch.empty(max(binding.hgrn1_workspace_bytes(B, N, d), 256), dtype=torch.uint8, device="cuda")
    binding.hgrn1_fwd_act(zfd, zid, zod, bd, h0d, workspace=ws)
    gf2, gi2, go2, gb2, gh02 = binding.hgrn1_bwd_act(zfd, zid, zod, bd, dyd, h0d, dhNd, want_grad_h0=True, workspace=ws,
                                                     saved=True)
    torch.cuda.synchronize()
    check("dzf (saved)", host(gf2), rf, tol)
    check("dzi (saved)", host(gi2), ri, tol)
    check("dzo (saved)", host(go2), ro, tol)
    check("dbeta (saved)", host(gb2), rb, tol)
    check("dh0 (saved)", host(gh02), rh0, tol)


@pytest.mark.parametrize("d", [192, 384])
@pytest.mark.parametrize("gate_dtype", ["bf16", "f32"])
def test_hgrn1_act_ragged(d, gate_dtype):
    print("\n[hgrn1 act] B=3 N=203 d=%d gate=%s" % (d, gate_dtype), flush=True)
    run_act(*make_act(5600 + d, 3, 203, d, gate_dtype=gate_dtype), gate_dtype=gate_dtype)


@pytest.mark.parametrize("N", [0, 1, 15, 16, 17, 255, 256, 257, 511, 512, 513, 800])
def test_hgrn1_act_edge_lengths(N):
    print("\n[hgrn1 act] edge N=%d" % N, flush=True)
    run_act(*make_act(5700 + N, 2, N, 128))


def test_hgrn1_act_no_states_and_zero_bound():
    zf, zi, zo, beta, dy, _, _ = make_act(5800, 2, 100, 256)
    beta[:] = 0.0                                     # the first layer: plain sigmoid gate
    print("\n[hgrn1 act] no h0 / grad_hN, beta = 0", flush=True)
    run_act(zf, zi, zo, beta, dy, None, None)


def test_hgrn1_act_layer_shape():
    print("\n[hgrn1 act] B=8 N=2048 d=2048", flush=True)
    run_act(*make_act(5900, 8, 2048, 2048))
