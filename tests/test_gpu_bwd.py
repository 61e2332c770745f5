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
