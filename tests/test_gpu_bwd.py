"""GPU parity of hgrn2_bwd against the fp64 CPU oracle (itself pinned by finite differences and
torch autograd), through the C ABI.  Error measure and tolerance: max|x-y|/max|y| <= 2e-2 per
gradient tensor for bf16 storage."""
import numpy as np
import pytest
import torch

import oracle
from paper_2404_07904_amd import binding, synth
from gpu_util import TOL, check, dev, host

pytestmark = pytest.mark.gpu


def run_bwd(w, with_dh0=True):
    io = w.io_dtype
    q, f, v, dO = dev(w.q, io), dev(w.f, w.gate_dtype), dev(w.v, io), dev(w.dO, io)
    h0, dhT = dev(w.h0), dev(w.dhT)
    dq, df, dv, dh0 = binding.hgrn2_bwd(q, f, v, dO, h0, dhT, want_grad_h0=with_dh0)
    torch.cuda.synchronize()
    rq, rf, rv, rh = oracle.bwd(w.q, w.f, w.v, w.dO, w.h0, w.dhT)
    tol = TOL[io]
    check("dq", host(dq), rq, tol)
    check("dv", host(dv), rv, tol)
    check("df", host(df), rf, tol)
    if with_dh0:
        check("dh0", host(dh0), rh, tol)


@pytest.mark.parametrize("dk,dv", [(64, 64), (128, 128), (64, 128), (128, 64)])
def test_bwd_shapes_ragged(dk, dv):
    print("\n[bwd] ragged dk=%d dv=%d N=203 with h0, dhT" % (dk, dv), flush=True)
    w = synth.make_sequence(2000 + dk + 2 * dv, 3, 3, 203, dk, dv, io_dtype="bf16", lb=0.2,
                            with_h0=True, with_dO=True, with_dhT=True)
    run_bwd(w)


@pytest.mark.parametrize("N", [0, 1, 63, 64, 65, 128])
def test_bwd_edge_lengths(N):
    print("\n[bwd] edge N=%d" % N, flush=True)
    w = synth.make_sequence(300 + N, 2, 2, N, 64, 64, io_dtype="bf16", lb=0.3, with_h0=True,
                            with_dO=True, with_dhT=True)
    run_bwd(w)


def test_bwd_no_optional_tensors():
    print("\n[bwd] no h0 / dhT / dh0", flush=True)
    w = synth.make_sequence(41, 2, 3, 256, 128, 128, io_dtype="bf16", lb=0.5, with_dO=True)
    run_bwd(w, with_dh0=False)


@pytest.mark.parametrize("layer", [0, 12, 23])
def test_bwd_layer_gates_reduced_batch(layer):
    """Gate statistics of layers 0, 12 and 23 of the 24-layer stack at the layer shape
    (H=16 -> here B=1, H=4), d=128, N=2048."""
    print("\n[bwd] layer %d gates, B=1 H=4 N=2048 d=128" % layer, flush=True)
    w = synth.config2(layer, B=1, H=4)
    run_bwd(w, with_dh0=False)


def test_bwd_gate_f32_near_one():
    print("\n[bwd] fp32 gate in [0.99, 1], N=1024", flush=True)
    w = synth.config3(gate_dtype="f32", B=1, H=2, N=1024)
    run_bwd(w, with_dh0=False)


def test_bwd_gate_bf16_near_one():
    print("\n[bwd] bf16 gate in [0.99, 1] (three distinct values), N=1024", flush=True)
    w = synth.config3(gate_dtype="bf16", B=1, H=2, N=1024)
    run_bwd(w, with_dh0=False)


def test_bwd_f_equal_one():
    """f == 1: k = 0, the state is frozen at h0; dq = dO h0^T, dv = 0."""
    print("\n[bwd] f == 1", flush=True)
    w = synth.make_sequence(43, 1, 2, 100, 64, 64, io_dtype="bf16", lb=0.5, with_h0=True, with_dO=True)
    w.f = np.ones_like(w.f)
    run_bwd(w)


def test_bwd_deterministic():
    w = synth.make_sequence(44, 2, 3, 300, 128, 128, io_dtype="bf16", lb=0.1, with_h0=True,
                            with_dO=True, with_dhT=True)
    a = [dev(x, "bf16") for x in (w.q, w.f, w.v, w.dO)]
    h0, dhT = dev(w.h0), dev(w.dhT)
    r1 = binding.hgrn2_bwd(*a, h0, dhT, want_grad_h0=True)
    r2 = binding.hgrn2_bwd(*a, h0, dhT, want_grad_h0=True)
    torch.cuda.synchronize()
    for x, y in zip(r1, r2):
        assert torch.equal(x, y)


# ---- fp32 storage (heads of 64 x 64): the same kernels with fp32 tiles and fp32 matrix
# instructions, which holds the chunkwise backward algebra to 1e-4 instead of the 2e-2 that bf16
# operands allow.  Wider heads are bf16-only: their fp32 tiles do not fit the LDS.
@pytest.mark.parametrize("B,H,N,gate_dtype,note", [
    (2, 3, 203, "f32", "one run, ragged last chunk"),
    (1, 2, 1, "f32", "a single token"),
    (3, 2, 64, "f32", "exactly one chunk"),
    (1, 2, 640, "f32", "two runs, light walk over the second"),
    (1, 3, 1100, "bf16", "four runs"),
    (1, 1, 2500, "f32", "nine runs: boundary states from the zero-start sweep"),
    (4, 16, 520, "f32", "64 sequences of 9 chunks"),
])
def test_bwd_fp32_storage(B, H, N, gate_dtype, note):
    print("\n[bwd fp32] B=%d H=%d N=%d gate=%s (%s)" % (B, H, N, gate_dtype, note), flush=True)
    w = synth.make_sequence(2600 + N, B, H, N, 64, 64, io_dtype="f32", gate_dtype=gate_dtype, lb=0.1,
                            with_h0=True, with_dO=True, with_dhT=True)
    run_bwd(w)


def test_bwd_fp32_storage_token_major_and_gated():
    B, H, N, d = 2, 3, 333, 64
    print("\n[bwd fp32] token-major, gate formed in the kernels", flush=True)
    rng = np.random.default_rng(2700)
    w = synth.make_sequence(2701, B, H, N, d, d, io_dtype="f32", with_h0=True, with_dO=True, with_dhT=True)
    z = rng.standard_normal((B, H, N, d)).astype(np.float32)
    beta = rng.uniform(0.0, 0.9, size=(H, d)).astype(np.float32)
    tm = lambda x: dev(x).permute(0, 2, 1, 3).contiguous()
    back = lambda t: host(t.permute(0, 2, 1, 3))
    BNHD = binding.HGRN2_LAYOUT_BNHD
    bd = torch.from_numpy(beta).cuda()
    gq, gz, gb, gv, gh0 = binding.hgrn2_bwd_gated(tm(w.q), tm(z), bd, tm(w.v), tm(w.dO), dev(w.h0), dev(w.dhT),
                                                  want_grad_h0=True, layout=BNHD)
    torch.cuda.synchronize()
    rq, rz, rb, rv, rh = oracle.bwd_gated(w.q, z, beta, w.v, w.dO, w.h0, w.dhT)
    tol = TOL["f32"]
    check("dq", back(gq), rq, tol); check("dz", back(gz), rz, tol); check("dbeta", host(gb), rb, tol)
    check("dv", back(gv), rv, tol); check("dh0", host(gh0), rh, tol)


def test_bwd_fp32_storage_small_gates():
    """The chunk-local gate gradient at small gates, where the cancelling pair terms matter most:
    gates down to 0.05 (inside the ordinary domain), fp32, 1e-4."""
    B, H, N = 2, 2, 300
    print("\n[bwd fp32] gates in [0.05, 1]", flush=True)
    w = synth.make_sequence(2800, B, H, N, 64, 64, io_dtype="f32", lb=0.05, with_h0=True, with_dO=True, with_dhT=True)
    rng = np.random.default_rng(2801)
    w.f = (0.05 + 0.95 * rng.random(w.f.shape)).astype(np.float32)
    run_bwd(w)
