"""GPU parity of hgrn2_fwd and hgrn2_step against the fp64 CPU oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
from paper_2404_07904_amd import binding, synth
from gpu_util import TOL, check, dev, host

pytestmark = pytest.mark.gpu


def run_fwd(w, want_hT=True):
    q, f, v = dev(w.q, w.io_dtype), dev(w.f, w.gate_dtype), dev(w.v, w.io_dtype)
    h0 = dev(w.h0)
    o, hT = binding.hgrn2_fwd(q, f, v, h0, want_hT=want_hT)
    torch.cuda.synchronize()
    o_ref, hT_ref = oracle.fwd(w.q, w.f, w.v, w.h0)
    tol = TOL[w.io_dtype]
    check("o", host(o), o_ref, tol)
    if want_hT:
        check("hT", host(hT), hT_ref, tol)


def test_fwd_config0_tiny_f32():
    print("\n[fwd] config0 tiny fp32", flush=True)
    run_fwd(synth.config0())


def test_fwd_config1_bf16():
    print("\n[fwd] config1 bf16 B=4 H=8 N=1024 d=64 with h0", flush=True)
    run_fwd(synth.config1())


@pytest.mark.parametrize("dk,dv", [(64, 64), (128, 128), (64, 128), (128, 64)])
@pytest.mark.parametrize("io", ["bf16", "f32"])
def test_fwd_shapes_ragged(dk, dv, io):
    # several chunks plus a ragged tail; B*H not a multiple of 8
    print("\n[fwd] ragged dk=%d dv=%d io=%s N=203" % (dk, dv, io), flush=True)
    w = synth.make_sequence(1000 + dk + 2 * dv, 3, 3, 203, dk, dv, io_dtype=io, lb=0.2, with_h0=True)
    run_fwd(w)


@pytest.mark.parametrize("N", [0, 1, 63, 64, 65])
def test_fwd_edge_lengths(N):
    print("\n[fwd] edge N=%d" % N, flush=True)
    w = synth.make_sequence(77 + N, 2, 2, N, 64, 64, io_dtype="bf16", lb=0.3, with_h0=True)
    run_fwd(w)


def test_fwd_gate_f32_with_bf16_io():
    print("\n[fwd] bf16 io, fp32 gate near one", flush=True)
    w = synth.make_sequence(5, 2, 4, 512, 128, 128, io_dtype="bf16", gate_dtype="f32", lb=0.99)
    run_fwd(w)


def test_fwd_small_gates_lb0():
    print("\n[fwd] lb=0 (sigmoid gates) d=128", flush=True)
    w = synth.make_sequence(6, 2, 4, 384, 128, 128, io_dtype="bf16", lb=0.0)
    run_fwd(w)


def test_fwd_gate_extremes():
    """f == 1 everywhere (state frozen) and a constant small gate (closed form 1 - c^t)."""
    print("\n[fwd] f == 1 and constant gate", flush=True)
    w = synth.make_sequence(8, 1, 2, 130, 64, 64, io_dtype="f32", lb=0.5, with_h0=True)
    w.f = np.ones_like(w.f)
    run_fwd(w)
    w2 = synth.make_sequence(9, 1, 2, 130, 64, 64, io_dtype="f32", lb=0.5)
    w2.f = np.full_like(w2.f, 0.25)
    w2.q = np.ones_like(w2.q)
    w2.v = np.ones_like(w2.v)
    o, _ = binding.hgrn2_fwd(dev(w2.q), dev(w2.f), dev(w2.v))
    t = np.arange(1, 131, dtype=np.float64)
    want = np.broadcast_to((64 * (1 - 0.25 ** t))[None, None, :, None], o.shape)
    check("closed", host(o), want, 1e-4)


def test_fwd_deterministic():
    w = synth.make_sequence(11, 2, 3, 300, 128, 128, io_dtype="bf16", lb=0.1, with_h0=True)
    q, f, v, h0 = dev(w.q, "bf16"), dev(w.f, "bf16"), dev(w.v, "bf16"), dev(w.h0)
    o1, h1 = binding.hgrn2_fwd(q, f, v, h0)
    o2, h2 = binding.hgrn2_fwd(q, f, v, h0)
    torch.cuda.synchronize()
    assert torch.equal(o1, o2) and torch.equal(h1, h2)


def test_fwd_split_handoff():
    """fwd(x[:m], h0) then fwd(x[m:], hT) equals fwd(x) up to the bf16 tolerance."""
    w = synth.make_sequence(12, 1, 2, 256, 64, 64, io_dtype="bf16", lb=0.4, with_h0=True)
    q, f, v, h0 = dev(w.q, "bf16"), dev(w.f, "bf16"), dev(w.v, "bf16"), dev(w.h0)
    o, hT = binding.hgrn2_fwd(q, f, v, h0)
    m = 128
    o1, h1 = binding.hgrn2_fwd(q[:, :, :m].contiguous(), f[:, :, :m].contiguous(), v[:, :, :m].contiguous(), h0)
    o2, h2 = binding.hgrn2_fwd(q[:, :, m:].contiguous(), f[:, :, m:].contiguous(), v[:, :, m:].contiguous(), h1)
    check("o", host(torch.cat([o1, o2], 2)), host(o), 2e-2)
    check("hT", host(h2), host(hT), 1e-5)


@pytest.mark.parametrize("N", [1, 64, 203, 448])
@pytest.mark.parametrize("gate", ["bf16", "f32"])
def test_fwd_fused_path(N, gate):
    """B*H >= 64 at d = 128 takes the single-pass kernel (state kept on chip)."""
    print("\n[fwd fused] B*H=72 N=%d gate=%s" % (N, gate), flush=True)
    w = synth.make_sequence(500 + N, 8, 9, N, 128, 128, io_dtype="bf16", gate_dtype=gate, lb=0.1, with_h0=True)
    run_fwd(w)


@pytest.mark.parametrize("N", [65, 200])
@pytest.mark.parametrize("gate", ["bf16", "f32"])
def test_fwd_fused_path_many_sequences(N, gate):
    """More than 128 sequences: one workgroup per sequence owning all dv columns (up to 128, two
    workgroups share a sequence, which is what the other fused-path cases run)."""
    print("\n[fwd fused] B*H=203 N=%d gate=%s" % (N, gate), flush=True)
    w = synth.make_sequence(700 + N, 29, 7, N, 128, 128, io_dtype="bf16", gate_dtype=gate, lb=0.2, with_h0=True)
    run_fwd(w)


def test_fwd_fused_path_no_h0_no_hT():
    print("\n[fwd fused] B*H=66, no h0, no hT", flush=True)
    w = synth.make_sequence(91, 6, 11, 130, 128, 128, io_dtype="bf16", lb=0.3)
    q, f, v = dev(w.q, "bf16"), dev(w.f, "bf16"), dev(w.v, "bf16")
    o, hT = binding.hgrn2_fwd(q, f, v, None, want_hT=False)
    torch.cuda.synchronize()
    assert hT is None
    ro, _ = oracle.fwd(w.q, w.f, w.v, None)
    check("o", host(o), ro, TOL["bf16"])


def test_fwd_fused_matches_two_kernel_path():
    """The single-pass kernel and sweep + read-out agree to bf16 rounding on the same inputs."""
    w = synth.make_sequence(77, 8, 8, 300, 128, 128, io_dtype="bf16", lb=0.3, with_h0=True)
    q, f, v, h0 = dev(w.q, "bf16"), dev(w.f, "bf16"), dev(w.v, "bf16"), dev(w.h0)
    o1, hT1 = binding.hgrn2_fwd(q, f, v, h0)
    shape = binding.make_shape(q, v, f)
    ws = torch.empty(binding.hgrn2_fwd_workspace_bytes(shape), dtype=torch.uint8, device="cuda")
    o2, hT2 = torch.empty_like(o1), torch.empty_like(hT1)
    binding.hgrn2_state_sweep(shape, binding.SWEEP_STATE_FWD, None, f, v, ws, h0, hT2)
    binding.hgrn2_fwd_readout(shape, q, f, v, ws, o2)
    torch.cuda.synchronize()
    check("o", host(o1), host(o2), 8e-3)
    check("hT", host(hT1), host(hT2), 8e-3)      # the two paths round differently scaled keys to bf16


# ------------------------------------------------------------------------------------ step
@pytest.mark.parametrize("dk,dv", [(64, 64), (128, 128), (64, 128), (128, 64)])
@pytest.mark.parametrize("io", ["bf16", "f32"])
def test_step_parity(dk, dv, io):
    print("\n[step] dk=%d dv=%d io=%s" % (dk, dv, io), flush=True)
    rng = np.random.default_rng(dk * 7 + dv)
    B, H, T = 3, 5, 6
    rnd = synth.bf16_round if io == "bf16" else (lambda x: x.astype(np.float32))
    q = rnd(rng.standard_normal((T, B, H, dk), dtype=np.float32))
    v = rnd(rng.standard_normal((T, B, H, dv), dtype=np.float32))
    f = rnd((0.2 + 0.8 * rng.uniform(size=(T, B, H, dk))).astype(np.float32))
    st0 = (0.1 * rng.standard_normal((B, H, dk, dv))).astype(np.float32)
    st_ref = st0.astype(np.float64)
    o_ref = oracle.steps(q, f, v, st_ref)
    st = dev(st0)
    tol = TOL[io]
    for t in range(T):
        o = binding.hgrn2_step(dev(q[t], io), dev(f[t], io), dev(v[t], io), st)
        check("o[%d]" % t, host(o), o_ref[t], tol)
    check("state", host(st), st_ref, 1e-5)


def test_step_config4_shape_reduced_steps():
    """Decode workload at its real shape (B=256, H=16, d=128), 8 of the 512 steps."""
    print("\n[step] config4 shape, 8 steps", flush=True)
    w = synth.config4(T=8)
    st_ref = w.state.astype(np.float64)
    o_ref = oracle.steps(w.q, w.f, w.v, st_ref)
    st = dev(w.state)
    q, f, v = dev(w.q, "bf16"), dev(w.f, "bf16"), dev(w.v, "bf16")
    for t in range(8):
        o = binding.hgrn2_step(q[t], f[t], v[t], st)
        if t in (0, 7):
            check("o[%d]" % t, host(o), o_ref[t], 2e-2)
    check("state", host(st), st_ref, 1e-5)


def test_steps_equal_fwd():
    """N single-token steps reproduce the chunked forward (hand-off invariant on the GPU)."""
    w = synth.make_sequence(21, 1, 2, 70, 64, 64, io_dtype="bf16", lb=0.3, with_h0=True)
    q, f, v, h0 = dev(w.q, "bf16"), dev(w.f, "bf16"), dev(w.v, "bf16"), dev(w.h0)
    o, hT = binding.hgrn2_fwd(q, f, v, h0)
    st = h0.clone()
    outs = [binding.hgrn2_step(q[:, :, t].contiguous(), f[:, :, t].contiguous(), v[:, :, t].contiguous(), st)
            for t in range(70)]
    check("o", host(torch.stack(outs, 2)), host(o), 2e-2)
    check("hT", host(st), host(hT), 1e-2)


@pytest.mark.parametrize("B,H,dk,dv,io", [(2, 3, 64, 64, 0), (2, 3, 128, 64, 1), (9, 8, 128, 128, 1)])
def test_empty_sequences_with_no_workspace_at_all(B, H, dk, dv, io):
    """N = 0 needs no workspace, so NULL is a legal one: the final state is the initial one and the gradient
    of the final state passes through, on the paths with separate sweeps and on the single-pass one."""
    import ctypes
    print("\n[fwd/bwd] N=0, workspace NULL, B=%d H=%d dk=%d dv=%d io=%d" % (B, H, dk, dv, io), flush=True)
    L = binding.lib()
    shape = binding.hgrn2_shape(B, H, 0, dk, dv, 0, io, io, 0)
    assert binding.hgrn2_fwd_workspace_bytes(shape) == 0 and binding.hgrn2_bwd_workspace_bytes(shape) == 0
    g = torch.Generator(device="cuda").manual_seed(5)
    h0 = torch.randn((B, H, dk, dv), generator=g, device="cuda")
    dhT = torch.randn((B, H, dk, dv), generator=g, device="cuda")
    hT, dh0 = torch.full_like(h0, 7.0), torch.full_like(h0, 7.0)
    P = lambda t: ctypes.c_void_p(t.data_ptr())
    s = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    assert L.hgrn2_fwd(ctypes.byref(shape), None, None, None, P(h0), None, P(hT), None, ctypes.c_size_t(0), s) == 0
    assert L.hgrn2_bwd(ctypes.byref(shape), None, None, None, P(h0), None, P(dhT), None, None, None, P(dh0), None,
                       ctypes.c_size_t(0), s) == 0
    torch.cuda.synchronize()
    assert torch.equal(hT, h0) and torch.equal(dh0, dhT)
    # no initial state: the final state of an empty sequence is zero
    assert L.hgrn2_fwd(ctypes.byref(shape), None, None, None, None, None, P(hT), None, ctypes.c_size_t(0), s) == 0
    torch.cuda.synchronize()
    assert float(hT.abs().max()) == 0.0
