"""The entry points enqueue kernels only (no allocation, no memset node, no host synchronisation), so
a caller can capture them into a HIP graph.  A captured forward + backward (and a captured run of
decode steps) is replayed several times on fresh inputs, with eager work and synchronisations
between the replays, and every replay must give exactly what the eager calls give."""
import numpy as np
import pytest
import torch

from paper_2404_07904_amd import binding, synth
from gpu_util import dev

pytestmark = pytest.mark.gpu


def fresh(seed, B, H, N, d):
    w = synth.make_sequence(seed, B, H, N, d, d, io_dtype="bf16", lb=0.3, with_h0=True, with_dO=True, with_dhT=True)
    return [dev(x, "bf16") for x in (w.q, w.f, w.v, w.dO)] + [dev(w.h0), dev(w.dhT)]


@pytest.mark.parametrize("B,H,N,d", [(2, 3, 200, 64), (8, 9, 130, 128), (1, 2, 2400, 128)])      # the last: sequences walked in runs
def test_captured_forward_backward_replays(B, H, N, d):
    print("\n[graph] B=%d H=%d N=%d d=%d" % (B, H, N, d), flush=True)
    static = fresh(8600, B, H, N, d)
    q, f, v, dO, h0, dhT = static
    shape = binding.make_shape(q, v, f)
    ws = torch.empty(binding.hgrn2_bwd_workspace_bytes(shape), dtype=torch.uint8, device="cuda")
    o, hT = torch.empty_like(v), torch.empty((B, H, d, d), device="cuda")
    gq, gf, gv, gh0 = torch.empty_like(q), torch.empty_like(q), torch.empty_like(v), torch.empty_like(hT)

    def step():
        binding.hgrn2_fwd(q, f, v, h0, o=o, hT=hT, workspace=ws)
        binding.hgrn2_bwd(q, f, v, dO, h0, dhT, workspace=ws, grad_q=gq, grad_f=gf, grad_v=gv, grad_h0=gh0)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                                   # warm-up outside the capture (first-launch set-up)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for k in range(4):
        new = fresh(8601 + k, B, H, N, d)
        for dst, src in zip(static, new):
            dst.copy_(src)
        graph.replay()
        torch.cuda.synchronize()
        got = [t.clone() for t in (o, hT, gq, gf, gv, gh0)]
        for t in (o, hT, gq, gf, gv, gh0):
            t.zero_()                           # eager work between the replays
        step()
        torch.cuda.synchronize()
        for name, a, b in zip(("o", "hT", "dq", "df", "dv", "dh0"), got, (o, hT, gq, gf, gv, gh0)):
            assert torch.equal(a, b), "replay %d: %s differs from the eager result" % (k, name)


def test_captured_training_pair_chooses_the_chunk_length_at_every_replay():
    """chunk = HGRN2_CHUNK_AUTO in a captured training pair: the graph holds the passes for all three chunk
    lengths, and the gates of each replay decide on the device which of them run -- ordinary gates, gates
    that need 32 tokens per chunk, gates that need 16, ordinary ones again -- with no new capture.  Every
    replay must give exactly what the eager call with that chunk length gives."""
    B, H, N, d = 2, 3, 300, 128
    AUTO = -1
    print("\n[graph] chunk length chosen on the device, B=%d H=%d N=%d d=%d" % (B, H, N, d), flush=True)
    static = fresh(8700, B, H, N, d)
    q, f, v, dO, h0, dhT = static
    shape = binding.make_shape(q, v, f, AUTO)
    ws = torch.empty(binding.hgrn2_bwd_workspace_bytes(shape), dtype=torch.uint8, device="cuda")
    saved = torch.empty(binding.hgrn2_saved_states_bytes(shape), dtype=torch.uint8, device="cuda")
    o, hT = torch.empty_like(v), torch.empty((B, H, d, d), device="cuda")
    gq, gf, gv, gh0 = torch.empty_like(q), torch.empty_like(q), torch.empty_like(v), torch.empty_like(hT)
    outs = (o, hT, gq, gf, gv, gh0)

    def step(chunk):
        binding.hgrn2_fwd_saving(q, f, v, h0, o=o, hT=hT, saved_states=saved, workspace=ws, chunk=chunk)
        binding.hgrn2_bwd_saved(q, f, v, saved, dO, dhT, workspace=ws, grad_q=gq, grad_f=gf, grad_v=gv, grad_h0=gh0, chunk=chunk)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        for c in (AUTO, 0, 32, 16):
            step(c)                              # warm-up outside the capture (first-launch set-up)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step(AUTO)
    rng = np.random.default_rng(8701)
    for k, (lo, need) in enumerate(((None, 0), (0.02, 32), (1e-3, 16), (None, 0), (0.02, 32))):
        new = fresh(8702 + k, B, H, N, d)
        if lo is not None:       # gates log-uniform in [lo, 1]
            g = 10.0 ** rng.uniform(np.log10(lo), 0.0, size=(B, H, N, d))
            new[1] = dev(synth.bf16_round(g.astype(np.float32)), "bf16")
        for dst, src in zip(static, new):
            dst.copy_(src)
        graph.replay()
        torch.cuda.synchronize()
        got = [t.clone() for t in outs]
        for t in outs:
            t.zero_()                            # eager work between the replays
        limit = 2.0 ** -100
        ok = [float(binding.hgrn2_min_gate_product(f, chunk=c).item()) > limit for c in (0, 32, 16)]
        assert (0, 32, 16)[ok.index(True)] == need
        step(need)
        torch.cuda.synchronize()
        for name, a, b in zip(("o", "hT", "dq", "df", "dv", "dh0"), got, outs):
            assert torch.equal(a, b), "replay %d (chunk %d): %s differs from the eager result" % (k, need, name)


def test_captured_decode_steps_replay():
    B, H, d, T = 4, 3, 64, 6
    print("\n[graph] decode B=%d H=%d d=%d, %d steps per replay" % (B, H, d, T), flush=True)
    w = synth.config4(T=T, B=B, H=H, d=d)
    qs, fs, vs = (dev(x, "bf16") for x in (w.q, w.f, w.v))
    state = dev(w.state)
    outs = torch.empty((T, B, H, d), dtype=torch.bfloat16, device="cuda")

    def run():
        for t in range(T):
            binding.hgrn2_step(qs[t], fs[t], vs[t], state, outs[t])

    s0 = state.clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    state.copy_(s0)
    with torch.cuda.graph(graph):
        run()
    for k in range(3):
        state.copy_(s0 * (1.0 + 0.25 * k))
        graph.replay()
        torch.cuda.synchronize()
        got_o, got_s = outs.clone(), state.clone()
        state.copy_(s0 * (1.0 + 0.25 * k))
        outs.zero_()
        run()
        torch.cuda.synchronize()
        assert torch.equal(got_o, outs) and torch.equal(got_s, state), "replay %d differs from eager" % k


def test_two_streams_with_their_own_workspaces():
    """The library keeps no state between calls: two calls on two streams, each with its own
    workspace and outputs, give what the same calls give one after the other."""
    B, H, N, d = 2, 3, 300, 64
    a, b = fresh(8700, B, H, N, d), fresh(8701, B, H, N, d)
    torch.cuda.synchronize()
    ref = []
    for q, f, v, dO, h0, dhT in (a, b):
        o, hT = binding.hgrn2_fwd(q, f, v, h0)
        g = binding.hgrn2_bwd(q, f, v, dO, h0, dhT, want_grad_h0=True)
        ref.append((o, hT) + tuple(g))
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    got = [None, None]
    for rep in range(3):
        for k, (q, f, v, dO, h0, dhT) in enumerate((a, b)):
            with torch.cuda.stream(streams[k]):
                o, hT = binding.hgrn2_fwd(q, f, v, h0)
                g = binding.hgrn2_bwd(q, f, v, dO, h0, dhT, want_grad_h0=True)
                got[k] = (o, hT) + tuple(g)
        torch.cuda.synchronize()
        for k in range(2):
            for x, y in zip(got[k], ref[k]):
                assert torch.equal(x, y)


@pytest.mark.parametrize("H,d,n_docs,chunk", [(16, 128, 24, 0), (4, 64, 5, 0), (4, 128, 7, -1)])
def test_captured_packed_training_pair_replays(H, d, n_docs, chunk):
    """The packed entry points read cu_seqlens on the device only (their tables are built by a
    kernel of the call), so a captured step serves batches cut differently: every replay gets new
    tokens AND new document boundaries (same token count, same number of documents).  With the chunk length
    chosen on the device (chunk = -1) every other replay also gets gates outside the domain of 64-token
    chunks, so that the replays take different chunk lengths."""
    T = 3000
    print("\n[graph] packed pair T=%d H=%d d=%d, %d documents, chunk=%d" % (T, H, d, n_docs, chunk), flush=True)
    rng = np.random.default_rng(8700 + H)

    def fresh_packed(seed):
        w = synth.make_sequence(seed, 1, H, T, d, d, io_dtype="bf16", lb=0.3, with_dO=True)
        if chunk == -1 and seed % 2 == 1:          # log-uniform gates in [0.02, 1]: 32 tokens per chunk
            w.f = synth.bf16_round((10.0 ** rng.uniform(np.log10(0.02), 0.0, size=w.f.shape)).astype(np.float32))
        pk = lambda x: dev(x, "bf16")[0].permute(1, 0, 2).contiguous()
        cuts = np.sort(rng.integers(0, T + 1, size=n_docs - 1))
        cu = torch.from_numpy(np.concatenate([[0], cuts, [T]]).astype(np.int32)).cuda()
        return [pk(w.q), pk(w.f), pk(w.v), pk(w.dO), cu]

    static = fresh_packed(8700)
    q, f, v, dO, cu = static
    shape = binding.make_shape_varlen(q, v, f, n_docs, chunk)
    ws = torch.empty(binding.hgrn2_bwd_varlen_workspace_bytes(shape), dtype=torch.uint8, device="cuda")
    kept = torch.empty(binding.hgrn2_saved_states_varlen_bytes(shape), dtype=torch.uint8, device="cuda")
    o, hT = torch.empty_like(v), torch.empty((n_docs, H, d, d), device="cuda")
    gq, gf, gv = torch.empty_like(q), torch.empty_like(q), torch.empty_like(v)

    def step():
        binding.hgrn2_fwd_varlen(q, f, v, cu, None, o=o, hT=hT, workspace=ws, saved_states=kept, chunk=chunk)
        binding.hgrn2_bwd_varlen(q, f, v, dO, cu, None, None, workspace=ws, grad_q=gq, grad_f=gf, grad_v=gv,
                                 saved_states=kept, chunk=chunk)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for k in range(4):
        new = fresh_packed(8701 + k)
        for dst, src in zip(static, new):
            dst.copy_(src)
        graph.replay()
        torch.cuda.synchronize()
        got = [t.clone() for t in (o, hT, gq, gf, gv)]
        for t in (o, hT, gq, gf, gv):
            t.zero_()
        kept.fill_(0xFF)
        step()
        torch.cuda.synchronize()
        for name, a, b in zip(("o", "hT", "dq", "df", "dv"), got, (o, hT, gq, gf, gv)):
            assert torch.equal(a, b), "replay %d: %s differs from the eager result" % (k, name)
