#!/usr/bin/env python3
"""Benchmark of the HGRN2 hot path on one MI355X.

One "step" is one pass of the whole training path over one batch of seeded synthetic input at
the layer shape B=8, H=16, N=2048, dk=dv=128 (bf16 storage, fp32 accumulation): the training
pair hgrn2_fwd_saving (the forward pass, which keeps the state entering every chunk) followed by
hgrn2_bwd_saved (the backward pass, which reads those states); the stateless pair hgrn2_fwd +
hgrn2_bwd, which recomputes the states, is timed next to it ("calls").
value = B*N / (time per step) in tokens/s.  The decode path
(hgrn2_step at B=256, H=16, d=128, 512 consecutive in-place steps) is timed in the same run and
reported under "decode" in GB/s of algorithmic bytes.

Also reported on the same JSON line:
  roofline      the dominant kernel of the step against the HBM roofline (8 TB/s), from HIP-event
                timings of the individual stages taken in this run
  mfma          algorithmic flops of fwd+bwd against the dense bf16 MFMA peak (2.5 PFLOP/s)
  cpu_baseline  the fp64 CPU oracle on the same inputs, all host cores, same run
  hgrn1         the element-wise recurrence of Eq. 1 at the same layer width (hgrn1_fwd, hgrn1_bwd)
  gated         the same step through hgrn2_fwd_gated / hgrn2_bwd_gated (gate of Eq. 2 formed from
                its pre-activation inside the kernels)
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

CHUNK = 64


def published_peaks():
    """The published MI355X peaks, kept in one header (include/mi355x_peaks.h)."""
    import re
    text = open(os.path.join(ROOT, "include", "mi355x_peaks.h")).read()
    return {m.group(1): float(m.group(2)) for m in re.finditer(r"#define\s+MI355X_(\w+)\s+([0-9.]+)", text)}


PEAKS = published_peaks()
HBM_PEAK_GBS = PEAKS["HBM_GBPS"]
MFMA_BF16_PEAK_TFLOPS = PEAKS["MFMA_BF16_TFLOPS"]


def measured_traffic():
    """HBM bytes per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this benchmark, as
    paper_2404_07904_amd/pmc_summary.py wrote them (scaled by the copy probe); {} if never taken."""
    path = os.path.join(ROOT, "profiles", "measured_traffic.json")
    if not os.path.exists(path):
        return {}
    with open(path) as fh:
        data = json.load(fh)
    return {k: v["bytes"] for k, v in data.get("kernels", {}).items()}


MEASURED_TRAFFIC_BYTES = measured_traffic()


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--layer", type=int, default=12, help="gate statistics: layer of the 24-layer stack (0, 12, 23)")
    ap.add_argument("--decode-steps", type=int, default=512)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-decode", action="store_true")
    ap.add_argument("--no-hgrn1", action="store_true", help="skip the element-wise HGRN1 workload")
    ap.add_argument("--no-varlen", action="store_true", help="skip the packed variable-length run")
    ap.add_argument("--no-handoff", action="store_true", help="skip the prefill -> decode hand-off run")
    ap.add_argument("--no-gated", action="store_true", help="skip the run with the gate formed inside the kernels")
    ap.add_argument("--no-long", action="store_true", help="skip the long-sequence shape (B=2, N=16384)")
    ap.add_argument("--no-layer", action="store_true", help="skip the layer run (projections + recurrence)")
    ap.add_argument("--no-layers", action="store_true", help="skip the runs on the gates of the other layers (0, 23)")
    ap.add_argument("--no-small-gates", action="store_true", help="skip the small-gate modes (chunk = 32, 16)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 1 GiB device copy, the known-size kernel that rocprofv3 --pmc "
                         "FETCH_SIZE / WRITE_SIZE readings are scaled by")
    return ap.parse_args()


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU; every (batch, head) pair is an independent "
              "recurrence, so more GPUs would only split the batch. Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2404_07904_amd import binding, synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    binding.lib()          # fail loudly if the native library is missing
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    B, H, N, D = 8, 16, 2048, 128
    tokens = B * N
    token_heads = B * H * N

    def to_dev(x, dt=torch.bfloat16):
        return torch.from_numpy(np.ascontiguousarray(x)).to(dev).to(dt).contiguous()

    # two seeded input sets, used alternately so that no step finds its inputs in cache
    sets = []
    hosts = []
    for i in range(2):
        w = synth.config2(args.layer if i == 0 else (args.layer + 1) % 24)
        hosts.append(w)
        sets.append(tuple(to_dev(x) for x in (w.q, w.f, w.v, w.dO)))
    shape = binding.make_shape(sets[0][0], sets[0][2], sets[0][1])
    ws = torch.empty(max(binding.hgrn2_bwd_workspace_bytes(shape), binding.hgrn2_fwd_workspace_bytes(shape)),
                     dtype=torch.uint8, device=dev)
    saved = [torch.empty(binding.hgrn2_saved_states_bytes(shape), dtype=torch.uint8, device=dev) for _ in range(2)]
    o = torch.empty_like(sets[0][2])
    hT = torch.empty((B, H, D, D), dtype=torch.float32, device=dev)
    gq, gf, gv = (torch.empty_like(sets[0][0]) for _ in range(3))

    # the kernels raise this device int when a gate product leaves the domain of the 64-token chunks
    # (it costs nothing in the timed region; read once, at the end)
    domain_flag = torch.zeros(1, dtype=torch.int32, device=dev)

    def train_fwd(i):
        q, f, v, _ = sets[i % 2]
        binding.hgrn2_fwd_saving(q, f, v, None, o=o, hT=hT, saved_states=saved[i % 2], workspace=ws, domain_flag=domain_flag)

    def train_bwd(i):
        q, f, v, dO = sets[i % 2]
        binding.hgrn2_bwd_saved(q, f, v, saved[i % 2], dO, None, workspace=ws, grad_q=gq, grad_f=gf, grad_v=gv,
                                domain_flag=domain_flag)

    def step(i):
        train_fwd(i)
        train_bwd(i)

    # wake the GPU up before anything is timed (its clocks take tens of milliseconds of work to come
    # up; a few launches of the matrix probe and of the step itself)
    _, warm_out = binding.hgrn2_probe_mfma(2000)
    for i in range(20):
        binding.hgrn2_probe_mfma(2000, warm_out)
        step(i)
    torch.cuda.synchronize()
    del warm_out

    if args.calibrate_copy:          # the known-size kernel the --pmc byte counters are scaled by
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(3):
            binding.hgrn2_probe_copy(dst, src)
        torch.cuda.synchronize()
        del src, dst

    # ---- per-stage durations with HIP events on the stream the kernels run on ----
    one_set = binding.hgrn2_fwd_workspace_bytes(shape)       # one set of per-chunk states, for the stage calls
    ws_a = torch.empty(one_set, dtype=torch.uint8, device=dev)
    ws_b = torch.empty(one_set, dtype=torch.uint8, device=dev)

    def timed_all(fn, reps=30):
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
        for i, (a, b) in enumerate(ev):
            a.record()
            fn(i)
            b.record()
        torch.cuda.synchronize()
        return [a.elapsed_time(b) * 1e-3 for a, b in ev]             # seconds, per call

    def timed(fn, reps=30):
        return sum(timed_all(fn, reps)) / reps                       # seconds

    def timed_run(fn, reps=30):
        # `reps` calls back to back between ONE pair of events, as the headline's timed region runs them
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for i in range(reps):
            fn(i)
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) * 1e-3 / reps                        # seconds per call

    def s_fwd(i):
        q, f, v, _ = sets[i % 2]
        binding.hgrn2_state_sweep(shape, binding.SWEEP_STATE_FWD, None, f, v, ws_a, None, hT)

    def s_out(i):
        q, f, v, _ = sets[i % 2]
        binding.hgrn2_fwd_readout(shape, q, f, v, ws_a, o)

    def s_bst(i):
        q, f, v, _ = sets[i % 2]
        binding.hgrn2_state_sweep(shape, binding.SWEEP_STATE_BWD, None, f, v, ws_a)

    def s_grad(i):
        q, f, v, dO = sets[i % 2]
        binding.hgrn2_state_sweep(shape, binding.SWEEP_STATE_GRAD, q, f, dO, ws_b)

    def s_chunk(i):
        q, f, v, dO = sets[i % 2]
        binding.hgrn2_bwd_chunk_grads(shape, q, f, v, dO, ws_a, ws_b, gq, gf, gv)

    def s_whole_fwd(i):
        q, f, v, _ = sets[i % 2]
        binding.hgrn2_fwd(q, f, v, None, o=o, hT=hT, workspace=ws)

    def s_whole_bwd(i):
        q, f, v, dO = sets[i % 2]
        binding.hgrn2_bwd(q, f, v, dO, None, None, workspace=ws, grad_q=gq, grad_f=gf, grad_v=gv)

    # the backward call of the training pair is ONE kernel launch at this shape (bwd_fused_kernel: the
    # reverse walk with the state gradient in registers), so its event time is that kernel's duration
    s_train_fwd, s_train_bwd = train_fwd, train_bwd

    el = 2  # bytes per bf16 element
    state_bytes = B * H * (N // CHUNK) * D * D * el
    seq_k = token_heads * D * el
    # algorithmic bytes: the operation's own inputs/outputs each stage has to touch (workspace
    # traffic is overhead of the implementation and is not counted)
    stages = [
        ("state_sweep_fwd", s_fwd, 2 * seq_k),            # f, v
        ("fwd_readout", s_out, 4 * seq_k),                 # q, f, v -> o           (1024 B / token-head)
        ("state_sweep_bwd", s_bst, 2 * seq_k),             # f, v
        ("state_sweep_grad", s_grad, 3 * seq_k),           # q, f, dO
        ("bwd_chunk_grads", s_chunk, 7 * seq_k),           # q, f, v, dO -> dq, df, dv (1792 B / token-head)
    ]
    calls = [("hgrn2_fwd_saving", s_train_fwd, 4 * seq_k), ("hgrn2_bwd_saved", s_train_bwd, 7 * seq_k),
             ("hgrn2_fwd", s_whole_fwd, 4 * seq_k), ("hgrn2_bwd", s_whole_bwd, 7 * seq_k)]
    stage_out = {}
    call_out = {}
    for name, fn, abytes in calls:
        for i in range(2):
            fn(i)
        dt = timed(fn)
        call_out[name] = {"us": round(dt * 1e6, 2), "algorithmic_GB": round(abytes / 1e9, 4),
                          "GBps": round(abytes / dt / 1e9, 1)}
    for name, fn, abytes in stages:
        for i in range(2):
            fn(i)
        dt = timed(fn)
        stage_out[name] = {"us": round(dt * 1e6, 2), "algorithmic_GB": round(abytes / 1e9, 4),
                           "GBps": round(abytes / dt / 1e9, 1)}
    # ---- the headline: W untimed steps, then exactly K timed ones between two synchronisations.
    # It comes after the per-call timings above, so that the timed region does not start on a GPU
    # that has just woken up (its clocks take tens of milliseconds of work to come up).
    # The per-call timings leave gaps between launches, during which the clocks fall back: a burst of
    # back-to-back work (the matrix probe and the step, about 0.1 s) brings them up again first.
    _, warm_out = binding.hgrn2_probe_mfma(2000)
    for i in range(150):
        binding.hgrn2_probe_mfma(2000, warm_out)
        step(i)
    torch.cuda.synchronize()
    del warm_out
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    value = tokens / (ms_per_step * 1e-3)

    # dominant kernel of the step: the reverse walk of the backward pass, timed once more with HIP
    # events right after the headline, on the stream it is launched on
    for i in range(4):
        s_train_bwd(i)
    # (the median of the per-launch times: one launch delayed by something else on the machine would
    # otherwise move the figure; mean, minimum and maximum are reported next to it)
    dom_all = sorted(timed_all(s_train_bwd, reps=max(20, args.steps)))
    dom_s = dom_all[len(dom_all) // 2]
    dom_bytes = 7 * seq_k
    achieved = dom_bytes / dom_s / 1e9
    roofline = {"kernel": "bwd_fused_kernel (hgrn2_bwd_saved)", "bound": "hbm", "achieved": round(achieved, 1),
                "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                "us": round(dom_s * 1e6, 2), "us_mean_min_max": [round(x * 1e6, 1) for x in (sum(dom_all) / len(dom_all), dom_all[0], dom_all[-1])],
                "algorithmic_bytes": dom_bytes,
                "traffic": MEASURED_TRAFFIC_BYTES.get("bwd_fused_kernel")}

    flops = token_heads * ((4 * D * D + CHUNK * 2 * D) + (8 * D * D + CHUNK * 5 * D))   # fwd + bwd, algorithmic
    mfma_tflops = flops / (ms_per_step * 1e-3) / 1e12
    io_bytes = token_heads * (1024 + 1792)
    result = {
        "metric": "tokens/s fwd+bwd (H=16,dk=dv=128,N=2048) + % MFMA peak; step GB/s",
        "value": round(value, 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "configs[2]: layer-shaped fwd+bwd, B=8 H=16 N=2048 dk=dv=128 bf16, gates of layer %d of 24"
                               % args.layer, "global_batch": B, "seq_len": N, "heads": H, "chunk": CHUNK},
        "roofline": roofline,
        "mfma": {"achieved_TFLOPs": round(mfma_tflops, 2), "peak_TFLOPs": MFMA_BF16_PEAK_TFLOPS,
                 "frac": round(mfma_tflops / MFMA_BF16_PEAK_TFLOPS, 5)},
        "hbm_step": {"algorithmic_GBps": round(io_bytes / (ms_per_step * 1e-3) / 1e9, 1),
                     "frac": round(io_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)},
        "calls": call_out,
        "stages": stage_out,
    }

    # ---- what this machine sustains: a plain copy and a loop of bf16 matrix instructions ----
    src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).random_(0, 255)
    dst = torch.empty_like(src)
    for _ in range(2):
        binding.hgrn2_probe_copy(dst, src)
    t_copy = timed(lambda i: binding.hgrn2_probe_copy(dst, src), reps=10)
    del src, dst
    mf_flops, mf_out = binding.hgrn2_probe_mfma(2000)
    t_mfma = timed(lambda i: binding.hgrn2_probe_mfma(2000, mf_out), reps=5)
    result["empirical_peaks"] = {
        "copy_GBps": round(2 * (1 << 30) / t_copy / 1e9, 1), "copy_frac_of_published": round(2 * (1 << 30) / t_copy / 1e9 / HBM_PEAK_GBS, 4),
        "mfma_bf16_TFLOPs": round(mf_flops / t_mfma / 1e12, 1),
        "mfma_frac_of_published": round(mf_flops / t_mfma / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
        "what": "hgrn2_probe_copy of 1 GiB (2 GiB of traffic); hgrn2_probe_mfma: 8192 waves x 2000 x 4 independent 32x32x16 bf16 MFMAs",
        "published": {"hbm_GBps": HBM_PEAK_GBS, "mfma_bf16_TFLOPs": MFMA_BF16_PEAK_TFLOPS, "header": "include/mi355x_peaks.h"}}
    result["roofline"]["frac_of_copy_rate"] = round(result["roofline"]["achieved"] / result["empirical_peaks"]["copy_GBps"], 4)

    # ---- the three layers configs[2] names (gates of layers 0, 12, 23 of the 24-layer stack) ----
    layers = {}
    for layer in ((args.layer,) if args.no_layers else (0, 12, 23)):
        a = sets[0] if layer == args.layer else tuple(to_dev(x) for x in (lambda wl: (wl.q, wl.f, wl.v, wl.dO))(synth.config2(layer)))
        b = tuple(t.clone() for t in a)          # the same data at other addresses: no step finds its inputs in cache
        pair = (a, b)

        def layer_step(i):
            q, f, v, dO = pair[i % 2]
            binding.hgrn2_fwd_saving(q, f, v, None, o=o, hT=hT, saved_states=saved[i % 2], workspace=ws)
            binding.hgrn2_bwd_saved(q, f, v, saved[i % 2], dO, None, workspace=ws, grad_q=gq, grad_f=gf, grad_v=gv)

        # the host spent seconds drawing this layer's inputs: bring the clocks back up first
        _, warm_out = binding.hgrn2_probe_mfma(2000)
        for i in range(20):
            binding.hgrn2_probe_mfma(2000, warm_out)
            layer_step(i)
        torch.cuda.synchronize()
        del warm_out
        tl = timed_run(layer_step, reps=50)
        layers["layer_%d" % layer] = {"lower_bound": round(synth.layer_lower_bound(layer), 4), "ms_per_step": round(tl * 1e3, 4),
                                      "tokens_per_s": round(tokens / tl, 1)}
        del pair, a, b
    result["layers"] = layers

    # ---- the layer around the recurrence (Eq. 1 -> Eq. 2 -> Eq. 3): the three input projections of the
    # token mixer as one bf16 MFMA product with bias + activation, the recurrence on its token-major
    # outputs with the gate formed in the kernels, and the whole reverse mode ----
    if not args.no_layer:
        dm = H * D
        gen = torch.Generator(device=dev).manual_seed(synth.BASE_SEED + 12)
        xs = [torch.randn((B, N, dm), generator=gen, device=dev).to(torch.bfloat16) for _ in range(2)]
        w3 = (torch.randn((3 * dm, dm), generator=gen, device=dev) / dm ** 0.5).to(torch.bfloat16)
        b3 = 0.5 * torch.randn((3 * dm,), generator=gen, device=dev)
        betal = torch.full((H, D), float(synth.layer_lower_bound(args.layer)), dtype=torch.float32, device=dev)
        dys = [torch.randn((B, N, H, D), generator=gen, device=dev).to(torch.bfloat16) for _ in range(2)]
        zl, vl2, ql, avl = (torch.empty((B, N, H, D), dtype=torch.bfloat16, device=dev) for _ in range(4))
        yl = torch.empty_like(zl)
        glq, glz, glv = (torch.empty_like(zl) for _ in range(3))
        glx = torch.empty_like(xs[0])
        glw = torch.empty((3 * dm, dm), dtype=torch.float32, device=dev)
        glb = torch.empty((3 * dm,), dtype=torch.float32, device=dev)
        shl = binding.make_shape(ql, vl2, zl, 0, binding.HGRN2_LAYOUT_BNHD)
        wsl = torch.empty(max(binding.hgrn2_fwd_workspace_bytes(shl), binding.hgrn2_bwd_saved_workspace_bytes(shl, True)),
                          dtype=torch.uint8, device=dev)
        wsp = torch.empty(int(binding.lib().hgru2_proj_bwd_workspace_bytes(B * N, dm)), dtype=torch.uint8, device=dev)
        BNHD = binding.HGRN2_LAYOUT_BNHD

        def proj_fwd(i):
            binding.hgru2_proj_fwd(xs[i % 2], w3, b3, z=zl.view(B, N, dm), v=vl2.view(B, N, dm), q=ql.view(B, N, dm),
                                   av=avl.view(B, N, dm))

        def proj_bwd(i):
            binding.hgru2_proj_bwd(xs[i % 2], w3, ql.view(B, N, dm), avl.view(B, N, dm), glz.view(B, N, dm), glv.view(B, N, dm),
                                   glq.view(B, N, dm), workspace=wsp, grad_x=glx, grad_w3=glw, grad_b3=glb)

        def layer_step(i):
            proj_fwd(i)
            binding.hgrn2_fwd_saving(ql, zl, vl2, None, beta=betal, o=yl, hT=hT, saved_states=saved[0], workspace=wsl, layout=BNHD)
            binding.hgrn2_bwd_saved(ql, zl, vl2, saved[0], dys[i % 2], None, beta=betal, workspace=wsl, grad_q=glq, grad_f=glz,
                                    grad_v=glv, layout=BNHD)
            proj_bwd(i)

        for i in range(4):
            layer_step(i)
        t_pf, t_pb, t_layer = timed(proj_fwd, reps=20), timed(proj_bwd, reps=10), timed(layer_step, reps=10)
        fl_f = 2.0 * B * N * dm * 3 * dm
        result["layer"] = {
            "workload": "Eq. 1 -> Eq. 2 -> Eq. 3 at B=%d N=%d width %d (H=%d, head %d), bf16: projections (one [%d, %d] x [%d, %d] "
                        "product, bias + activation fused), recurrence with the gate formed in the kernels, reverse mode of both"
                        % (B, N, dm, H, D, B * N, dm, dm, 3 * dm),
            "proj_fwd_us": round(t_pf * 1e6, 1), "proj_bwd_us": round(t_pb * 1e6, 1), "ms_per_step": round(t_layer * 1e3, 4),
            "tokens_per_s": round(tokens / t_layer, 1),
            "roofline_proj_fwd": {"bound": "mfma", "achieved": round(fl_f / t_pf / 1e12, 1), "peak": MFMA_BF16_PEAK_TFLOPS,
                                  "unit": "TFLOP/s", "frac": round(fl_f / t_pf / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
                                  "traffic": MEASURED_TRAFFIC_BYTES.get("proj_fwd_gemm")},
            "proj_bwd_TFLOPs": round(2 * fl_f / t_pb / 1e12, 1)}
        del xs, w3, dys, zl, vl2, ql, avl, yl, glq, glz, glv, glx, glw, wsl, wsp

    # ---- the same step with the gate of Eq. 2 formed inside the kernels (z and beta instead of f) ----
    if not args.no_gated:
        rng = np.random.default_rng(synth.BASE_SEED + 7)
        beta = torch.full((H, D), float(synth.layer_lower_bound(args.layer)), dtype=torch.float32, device=dev)
        zs = [to_dev(synth.bf16_round(rng.standard_normal((B, H, N, D), dtype=np.float32))) for _ in range(2)]
        wsg = torch.empty(binding.hgrn2_bwd_gated_workspace_bytes(shape), dtype=torch.uint8, device=dev)
        gb = torch.empty_like(beta)

        def gated_step(i):
            q, _, v, dO = sets[i % 2]
            binding.hgrn2_fwd_gated(q, zs[i % 2], beta, v, None, o=o, hT=hT, workspace=wsg)
            binding.hgrn2_bwd_gated(q, zs[i % 2], beta, v, dO, None, None, workspace=wsg, grad_q=gq, grad_z=gf,
                                    grad_beta=gb, grad_v=gv)

        for i in range(10):
            gated_step(i)
        dtg = timed(gated_step, reps=50)
        result["gated"] = {"workload": "the same shape with z ~ N(0,1) (bf16) and beta = %.4f in place of f"
                                       % synth.layer_lower_bound(args.layer),
                           "ms_per_step": round(dtg * 1e3, 4), "tokens_per_s": round(tokens / dtg, 1)}
        # ... and on token-major [B][N][H][d] tensors, the layout the layer's projections write
        BNHD = binding.HGRN2_LAYOUT_BNHD
        tm = lambda t: t.view(B, N, H, D)          # timing only: the same bytes read as [B][N][H][d]

        def gated_step_token_major(i):
            q, _, v, dO = sets[i % 2]
            binding.hgrn2_fwd_gated(tm(q), tm(zs[i % 2]), beta, tm(v), None, o=tm(o), hT=hT, workspace=wsg, layout=BNHD)
            binding.hgrn2_bwd_gated(tm(q), tm(zs[i % 2]), beta, tm(v), tm(dO), None, None, workspace=wsg, grad_q=tm(gq),
                                    grad_z=tm(gf), grad_beta=gb, grad_v=tm(gv), layout=BNHD)

        for i in range(10):
            gated_step_token_major(i)
        dtm = timed(gated_step_token_major, reps=50)
        result["gated"]["token_major_ms_per_step"] = round(dtm * 1e3, 4)
        result["gated"]["token_major_tokens_per_s"] = round(tokens / dtm, 1)

        def gated_pair_token_major(i):     # ... and as a training pair (the forward pass keeps the states), as the layer uses it
            q, _, v, dO = sets[i % 2]
            binding.hgrn2_fwd_saving(tm(q), tm(zs[i % 2]), tm(v), None, beta=beta, o=tm(o), hT=hT, saved_states=saved[0],
                                     workspace=wsg, layout=BNHD)
            binding.hgrn2_bwd_saved(tm(q), tm(zs[i % 2]), tm(v), saved[0], tm(dO), None, beta=beta, workspace=wsg,
                                    grad_q=tm(gq), grad_f=tm(gf), grad_v=tm(gv), layout=BNHD)

        for i in range(10):
            gated_pair_token_major(i)
        dtp = timed(gated_pair_token_major, reps=50)
        result["gated"]["token_major_training_pair_ms_per_step"] = round(dtp * 1e3, 4)
        result["gated"]["token_major_training_pair_tokens_per_s"] = round(tokens / dtp, 1)
        del zs, wsg

    # ---- the same step in the small-gate modes: reference rows every 32 and every 16 tokens ----
    if not args.no_small_gates:
        fine = {}
        for ck in (32, 16):
            shf = binding.make_shape(sets[0][0], sets[0][2], sets[0][1], ck)
            wsf = torch.empty(binding.hgrn2_bwd_workspace_bytes(shf), dtype=torch.uint8, device=dev)

            def fine_step(i):
                q, f, v, dO = sets[i % 2]
                binding.hgrn2_fwd(q, f, v, None, o=o, hT=hT, workspace=wsf, chunk=ck)
                binding.hgrn2_bwd(q, f, v, dO, None, None, workspace=wsf, grad_q=gq, grad_f=gf, grad_v=gv, chunk=ck)

            savedf = torch.empty(binding.hgrn2_saved_states_bytes(shf), dtype=torch.uint8, device=dev)

            def fine_pair(i):         # the training pair in the same mode
                q, f, v, dO = sets[i % 2]
                binding.hgrn2_fwd_saving(q, f, v, None, o=o, hT=hT, saved_states=savedf, workspace=wsf, chunk=ck)
                binding.hgrn2_bwd_saved(q, f, v, savedf, dO, None, workspace=wsf, grad_q=gq, grad_f=gf, grad_v=gv, chunk=ck)

            for i in range(4):
                fine_step(i); fine_pair(i)
            dtf = timed(fine_step, reps=20)
            dtp = timed(fine_pair, reps=20)
            fine["chunk_%d" % ck] = {"ms_per_step": round(dtf * 1e3, 4), "tokens_per_s": round(tokens / dtf, 1),
                                     "training_pair_ms_per_step": round(dtp * 1e3, 4),
                                     "training_pair_tokens_per_s": round(tokens / dtp, 1),
                                     "workspace_MB": round(wsf.numel() / 1e6, 1),
                                     "saved_states_MB": round(savedf.numel() / 1e6, 1)}
            del wsf, savedf
        # chunk length chosen on the device (HGRN2_CHUNK_AUTO): the headline's training pair with ordinary
        # gates, for which the passes for 32 and 16 tokens per chunk are enqueued and return at once
        sha = binding.make_shape(sets[0][0], sets[0][2], sets[0][1], -1)
        wsa = torch.empty(binding.hgrn2_bwd_workspace_bytes(sha), dtype=torch.uint8, device=dev)
        saveda = torch.empty(binding.hgrn2_saved_states_bytes(sha), dtype=torch.uint8, device=dev)

        def auto_pair(i):
            q, f, v, dO = sets[i % 2]
            binding.hgrn2_fwd_saving(q, f, v, None, o=o, hT=hT, saved_states=saveda, workspace=wsa, chunk=-1)
            binding.hgrn2_bwd_saved(q, f, v, saveda, dO, None, workspace=wsa, grad_q=gq, grad_f=gf, grad_v=gv, chunk=-1)

        for i in range(10):
            auto_pair(i)
        dta = timed(auto_pair, reps=40)
        fine["chunk_chosen_on_device"] = {"training_pair_ms_per_step": round(dta * 1e3, 4),
                                          "training_pair_tokens_per_s": round(tokens / dta, 1),
                                          "workspace_MB": round(wsa.numel() / 1e6, 1),
                                          "saved_states_MB": round(saveda.numel() / 1e6, 1)}
        del wsa, saveda
        fine["workload"] = ("the main shape and gates with a reference row every 32 (16) tokens: chunks that hold 32 (16) "
                            "tokens in their middle rows")
        result["small_gate_modes"] = fine

    # ---- long sequences in a small batch: twice the tokens of the main shape in 32 sequences ----
    if not args.no_long:
        Bl, Nl = 2, 16384
        gen = torch.Generator(device=dev).manual_seed(synth.BASE_SEED + 11)
        rnd = lambda: torch.randn((Bl, H, Nl, D), generator=gen, device=dev).to(torch.bfloat16)
        ql, vl_, dOl = rnd(), rnd(), rnd()
        fl = (0.99 + 0.01 * torch.rand((Bl, H, Nl, D), generator=gen, device=dev)).to(torch.bfloat16)   # long-range layer: gates in [0.99, 1]
        shl = binding.make_shape(ql, vl_, fl, 0, binding.HGRN2_LAYOUT_BHND)
        wsl = torch.empty(binding.hgrn2_bwd_workspace_bytes(shl), dtype=torch.uint8, device=dev)
        ol, gql, gfl, gvl = (torch.empty_like(ql) for _ in range(4))
        hTl = torch.empty((Bl, H, D, D), dtype=torch.float32, device=dev)

        savedl = torch.empty(binding.hgrn2_saved_states_bytes(shl), dtype=torch.uint8, device=dev)

        def long_fwd(i):          # the training pair, as in the headline
            binding.hgrn2_fwd_saving(ql, fl, vl_, None, o=ol, hT=hTl, saved_states=savedl, workspace=wsl)

        def long_bwd(i):
            binding.hgrn2_bwd_saved(ql, fl, vl_, savedl, dOl, None, workspace=wsl, grad_q=gql, grad_f=gfl, grad_v=gvl)

        def long_bwd_stateless(i):
            binding.hgrn2_bwd(ql, fl, vl_, dOl, None, None, workspace=wsl, grad_q=gql, grad_f=gfl, grad_v=gvl)

        for i in range(5):
            long_fwd(i); long_bwd(i)
        tf, tb = timed(long_fwd, reps=30), timed(long_bwd, reps=30)
        io_long = 11 * Bl * H * Nl * D * 2          # q, f, v, o; q, f, v, dO, dq, df, dv
        result["long_sequence"] = {"workload": "B=%d, H=%d, N=%d, d=%d, bf16, gates in [0.99, 1]; each sequence walked in runs"
                                               % (Bl, H, Nl, D),
                                   "fwd_ms": round(tf * 1e3, 4), "bwd_ms": round(tb * 1e3, 4),
                                   "ms_per_step": round((tf + tb) * 1e3, 4),
                                   "tokens_per_s": round(Bl * Nl / (tf + tb), 1),
                                   "algorithmic_GBps": round(io_long / (tf + tb) / 1e9, 1),
                                   "stateless_bwd_ms": round(timed(long_bwd_stateless, reps=20) * 1e3, 4)}
        # bf16 has three values in [0.99, 1]; the same gates kept in fp32 (4 bytes per gate)
        fl32 = 0.99 + 0.01 * torch.rand((Bl, H, Nl, D), generator=gen, device=dev)
        fl = fl32
        for i in range(3):
            long_fwd(i); long_bwd(i)
        tf32, tb32 = timed(long_fwd, reps=20), timed(long_bwd, reps=20)
        result["long_sequence"]["fp32_gates"] = {"fwd_ms": round(tf32 * 1e3, 4), "bwd_ms": round(tb32 * 1e3, 4),
                                                 "tokens_per_s": round(Bl * Nl / (tf32 + tb32), 1)}
        del ql, vl_, dOl, fl, fl32, wsl, ol, gql, gfl, gvl, savedl
        # the same number of tokens as two documents of unequal length packed along the token axis
        docs = [20000, 12768]
        Tl = sum(docs)
        rndp = lambda: torch.randn((Tl, H, D), generator=gen, device=dev).to(torch.bfloat16)
        qp, vp, dOp = rndp(), rndp(), rndp()
        fp = (0.99 + 0.01 * torch.rand((Tl, H, D), generator=gen, device=dev)).to(torch.bfloat16)
        cup = torch.tensor(np.concatenate([[0], np.cumsum(docs)]).astype(np.int32), device=dev)
        shp = binding.make_shape_varlen(qp, vp, fp, len(docs))
        wsp = torch.empty(binding.hgrn2_bwd_varlen_workspace_bytes(shp), dtype=torch.uint8, device=dev)
        op, gqp, gfp, gvp = (torch.empty_like(qp) for _ in range(4))
        hTp = torch.empty((len(docs), H, D, D), dtype=torch.float32, device=dev)

        def packed_fwd(i):
            binding.hgrn2_fwd_varlen(qp, fp, vp, cup, None, o=op, hT=hTp, workspace=wsp)

        def packed_bwd(i):
            binding.hgrn2_bwd_varlen(qp, fp, vp, dOp, cup, None, None, workspace=wsp, grad_q=gqp, grad_f=gfp, grad_v=gvp)

        keptp = torch.empty(binding.hgrn2_saved_states_varlen_bytes(shp), dtype=torch.uint8, device=dev)

        def packed_fwd_saving(i):
            binding.hgrn2_fwd_varlen(qp, fp, vp, cup, None, o=op, hT=hTp, workspace=wsp, saved_states=keptp)

        def packed_bwd_saved(i):
            binding.hgrn2_bwd_varlen(qp, fp, vp, dOp, cup, None, None, workspace=wsp, grad_q=gqp, grad_f=gfp, grad_v=gvp,
                                     saved_states=keptp)

        for i in range(5):
            packed_fwd(i); packed_bwd(i); packed_fwd_saving(i); packed_bwd_saved(i)
        tpf, tpb = timed(packed_fwd, reps=30), timed(packed_bwd, reps=30)
        tpfs, tpbs = timed(packed_fwd_saving, reps=30), timed(packed_bwd_saved, reps=30)
        result["long_sequence"]["packed"] = {"workload": "documents of %s tokens packed as [T][H][d]" % docs,
                                             "fwd_ms": round(tpf * 1e3, 4), "bwd_ms": round(tpb * 1e3, 4),
                                             "tokens_per_s": round(Tl / (tpf + tpb), 1),
                                             "training_pair_fwd_ms": round(tpfs * 1e3, 4), "training_pair_bwd_ms": round(tpbs * 1e3, 4),
                                             "training_pair_tokens_per_s": round(Tl / (tpfs + tpbs), 1)}
        del qp, vp, dOp, fp, wsp, op, gqp, gfp, gvp, keptp

    # ---- second workload: the element-wise HGRN1 recurrence at the same layer (width 2048) ----
    if not args.no_hgrn1:
        d1 = H * D
        rng = np.random.default_rng(synth.BASE_SEED + 8)
        mk = lambda: to_dev(synth.bf16_round(rng.standard_normal((B, N, d1), dtype=np.float32)))
        lb1 = float(synth.layer_lower_bound(args.layer))
        sets1 = []
        for _ in range(2):
            g = 1.0 / (1.0 + np.exp(-rng.standard_normal((B, N, d1), dtype=np.float32)))
            sets1.append((to_dev(synth.bf16_round((lb1 + (1.0 - lb1) * g).astype(np.float32))), mk(),
                          to_dev(synth.bf16_round(g.astype(np.float32))), mk()))      # f, i, o, dy
        ws1 = torch.empty(binding.hgrn1_workspace_bytes(B, N, d1), dtype=torch.uint8, device=dev)
        y1 = torch.empty_like(sets1[0][1])

        def h1_fwd(i):
            f1, i1, o1, _ = sets1[i % 2]
            binding.hgrn1_fwd(f1, i1, o1, None, y=y1, want_hN=False, workspace=ws1)

        def h1_bwd(i):
            f1, i1, o1, dy1 = sets1[i % 2]
            binding.hgrn1_bwd(f1, i1, o1, dy1, None, None, workspace=ws1)

        ws1p = [torch.empty_like(ws1) for _ in range(2)]     # training pair: one workspace per input set, as a step keeps it

        def h1_fwd_keep(i):
            f1, i1, o1, _ = sets1[i % 2]
            binding.hgrn1_fwd(f1, i1, o1, None, y=y1, want_hN=False, workspace=ws1p[i % 2])

        def h1_bwd_saved(i):
            f1, i1, o1, dy1 = sets1[i % 2]
            binding.hgrn1_bwd(f1, i1, o1, dy1, None, None, workspace=ws1p[i % 2], saved=True)

        for i in range(6):
            h1_fwd(i); h1_bwd(i); h1_fwd_keep(i); h1_bwd_saved(i)
        tf, tb = timed(h1_fwd, reps=50), timed(h1_bwd, reps=50)
        tbs = timed(h1_bwd_saved, reps=50)
        # the same layer from its pre-activations (Eq. 1 activations and the Eq. 2 bound formed in the kernels);
        # the N(0,1) tensors stand in for zf, zi, zo
        beta1 = torch.full((d1,), lb1, dtype=torch.float32, device=dev)

        def h1_fwd_act(i):
            _, a, o1, c = sets1[i % 2]
            binding.hgrn1_fwd_act(c, a, o1, beta1, None, y=y1, want_hN=False, workspace=ws1)

        def h1_bwd_act(i):
            f1, a, o1, c = sets1[i % 2]
            binding.hgrn1_bwd_act(c, a, o1, beta1, f1, None, None, workspace=ws1)

        for i in range(6):
            h1_fwd_act(i); h1_bwd_act(i)
        tfa, tba = timed(h1_fwd_act, reps=50), timed(h1_bwd_act, reps=50)
        e1 = B * N * d1 * el
        result["hgrn1"] = {
            "workload": "element-wise recurrence (Eq. 1), B=%d N=%d d=%d bf16, same gate statistics" % (B, N, d1),
            "fwd_us": round(tf * 1e6, 1), "bwd_us": round(tb * 1e6, 1), "bwd_saved_us": round(tbs * 1e6, 1),
            "fwd_act_us": round(tfa * 1e6, 1), "bwd_act_us": round(tba * 1e6, 1),
            "tokens_per_s_fwd_bwd": round(tokens / (tf + tbs), 1),
            "roofline_fwd": {"bound": "hbm", "achieved": round(4 * e1 / tf / 1e9, 1), "peak": HBM_PEAK_GBS,
                             "unit": "GB/s", "frac": round(4 * e1 / tf / 1e9 / HBM_PEAK_GBS, 4),
                             "traffic": MEASURED_TRAFFIC_BYTES.get("hgrn1_fwd_kernel")},
            "roofline_bwd": {"bound": "hbm", "achieved": round(7 * e1 / tbs / 1e9, 1), "peak": HBM_PEAK_GBS,
                             "unit": "GB/s", "frac": round(7 * e1 / tbs / 1e9 / HBM_PEAK_GBS, 4),
                             "kernel": "hgrn1_bwd_kernel (hgrn1_bwd_saved: the forward pass of the step kept the segment states)",
                             "traffic": MEASURED_TRAFFIC_BYTES.get("hgrn1_bwd_saved_kernel")}}
        del sets1, ws1, y1, ws1p

    # ---- variable-length batch: the same 16384 tokens per head, packed as documents of mixed length ----
    if not args.no_varlen:
        T = B * N
        rng = np.random.default_rng(synth.BASE_SEED + 9)
        lens = []
        while sum(lens) < T:
            lens.append(int(min(T - sum(lens), max(1, rng.lognormal(6.0, 1.0)))))
        pack = lambda t: t.permute(0, 2, 1, 3).reshape(T, H, D).contiguous()          # [B][H][N][d] -> [B N][H][d]
        vsets = [tuple(pack(t) for t in st_) for st_ in sets]

        def run_varlen(cu_list, pair=False, chunk=0):
            # pair: the forward pass keeps the chunk states for the backward pass (hgrn2_fwd_varlen_saving /
            # hgrn2_bwd_varlen_saved) instead of the backward pass recomputing them
            cu = torch.tensor(cu_list, dtype=torch.int32, device=dev)
            shp = binding.make_shape_varlen(vsets[0][0], vsets[0][2], vsets[0][1], len(cu_list) - 1, chunk)
            wsv = torch.empty(binding.hgrn2_bwd_varlen_workspace_bytes(shp), dtype=torch.uint8, device=dev)
            kept = torch.empty(binding.hgrn2_saved_states_varlen_bytes(shp), dtype=torch.uint8, device=dev) if pair else None
            ov, gqv, gfv, gvv = (torch.empty_like(vsets[0][0]) for _ in range(4))

            def fn(i):
                q, f, v, dO = vsets[i % 2]
                binding.hgrn2_fwd_varlen(q, f, v, cu, None, want_hT=False, o=ov, workspace=wsv, saved_states=kept, chunk=chunk)
                binding.hgrn2_bwd_varlen(q, f, v, dO, cu, None, None, workspace=wsv, grad_q=gqv, grad_f=gfv, grad_v=gvv,
                                         saved_states=kept, chunk=chunk)
            for i in range(6):
                fn(i)
            return timed(fn, reps=30)
        cu_mix = [0] + list(np.cumsum(lens))
        t_mix = run_varlen(cu_mix)
        t_eq = run_varlen([N * b for b in range(B + 1)])
        # short documents: 1024, 256 and 64 tokens each (the walks then take groups of documents)
        t_short = {L: run_varlen(list(range(0, T + 1, L))) for L in (1024, 256, 64)}
        t_pair = {"document_mix": run_varlen(cu_mix, True), "8_equal_sequences": run_varlen([N * b for b in range(B + 1)], True)}
        t_pair.update({str(L): run_varlen(list(range(0, T + 1, L)), True) for L in (1024, 256, 64)})
        # the document mix as a training pair with 32 tokens per chunk, and with the chunk length chosen on the device
        t_pair["document_mix_chunk_32"] = run_varlen(cu_mix, True, 32)
        t_pair["document_mix_chunk_chosen_on_device"] = run_varlen(cu_mix, True, -1)

        def fixed_bnhd(i):          # the same packing seen as an equal-length [B][N][H][d] batch
            q, f, v, dO = (t.view(B, N, H, D) for t in vsets[i % 2])
            binding.hgrn2_fwd(q, f, v, None, o=o.view(B, N, H, D), hT=hT, workspace=ws, layout=binding.HGRN2_LAYOUT_BNHD)
            binding.hgrn2_bwd(q, f, v, dO, None, None, workspace=ws, grad_q=gq.view(B, N, H, D), grad_f=gf.view(B, N, H, D),
                              grad_v=gv.view(B, N, H, D), layout=binding.HGRN2_LAYOUT_BNHD)
        for i in range(6):
            fixed_bnhd(i)
        t_fix = timed(fixed_bnhd, reps=30)
        result["varlen"] = {
            "workload": "T=%d tokens, H=%d, d=%d packed [T][H][d]; %d documents, lengths lognormal(6, 1) "
                        "(median %d, longest %d)" % (T, H, D, len(lens), int(np.median(lens)), max(lens)),
            "fwd_bwd_us_document_mix": round(t_mix * 1e6, 1), "tokens_per_s_document_mix": round(T / t_mix, 1),
            "fwd_bwd_us_8_equal_sequences": round(t_eq * 1e6, 1), "tokens_per_s_8_equal_sequences": round(T / t_eq, 1),
            "fwd_bwd_us_same_data_equal_length_entry_points": round(t_fix * 1e6, 1),
            "fwd_bwd_us_equal_documents_of": {str(L): round(t * 1e6, 1) for L, t in t_short.items()},
            "training_pair_fwd_bwd_us": {k: round(t * 1e6, 1) for k, t in t_pair.items()}}
        del vsets

    # ---- prefill -> decode hand-off: the chunkwise forward leaves the state the decode step continues from ----
    if not args.no_handoff:
        Bp, Np, n_dec = 32, 2048, 64
        wp = synth.make_sequence(synth.BASE_SEED + 10, Bp, H, Np, D, D, io_dtype="bf16",
                                 lb=float(synth.layer_lower_bound(args.layer)))
        qp, fp, vp = (to_dev(x) for x in (wp.q, wp.f, wp.v))
        wdn = synth.config4(T=n_dec, B=Bp, H=H, d=D)
        qn, fn_, vn = (to_dev(x) for x in (wdn.q, wdn.f, wdn.v))
        shp = binding.make_shape(qp, vp, fp)
        wsp = torch.empty(binding.hgrn2_fwd_workspace_bytes(shp), dtype=torch.uint8, device=dev)
        op = torch.empty_like(vp)
        state = torch.empty((Bp, H, D, D), dtype=torch.float32, device=dev)
        on = torch.empty((Bp, H, D), dtype=torch.bfloat16, device=dev)

        def prefill(i):
            binding.hgrn2_fwd(qp, fp, vp, None, o=op, hT=state, workspace=wsp)

        def decode(i):
            for t in range(n_dec):
                binding.hgrn2_step(qn[t], fn_[t], vn[t], state, on)
        for i in range(3):
            prefill(i); decode(i)
        tp, td = timed(prefill, reps=10), timed(decode, reps=5)
        # the same decode steps captured once into a HIP graph (the entry points only enqueue kernels)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            decode(0)
        graph.replay()
        tg = timed(lambda i: graph.replay(), reps=5)
        result["handoff"] = {
            "workload": "prefill B=%d H=%d N=%d d=%d, then %d decode steps in place on the state it returns "
                        "(fp32 [B][H][dk][dv], no copy or conversion between the two)" % (Bp, H, Np, D, n_dec),
            "prefill_us": round(tp * 1e6, 1), "prefill_tokens_per_s": round(Bp * Np / tp, 1),
            "decode_us_per_step": round(td / n_dec * 1e6, 2), "decode_tokens_per_s": round(Bp * n_dec / td, 1),
            "decode_us_per_step_hip_graph": round(tg / n_dec * 1e6, 2)}
        del qp, fp, vp, op, state

    # ---- decode: 512 consecutive in-place steps at B=256, H=16, d=128 ----
    if not args.no_decode:
        Bd, Hd, T_distinct = 256, 16, args.decode_steps          # a distinct token per step
        wd = synth.config4(T=T_distinct, B=Bd, H=Hd, d=D)
        qd, fd, vd = (to_dev(x) for x in (wd.q, wd.f, wd.v))
        st = to_dev(wd.state, torch.float32)
        od = torch.empty((Bd, Hd, D), dtype=torch.bfloat16, device=dev)
        for t in range(8):
            binding.hgrn2_step(qd[t], fd[t], vd[t], st, od)
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for t in range(args.decode_steps):
            k = t % T_distinct
            binding.hgrn2_step(qd[k], fd[k], vd[k], st, od)
        b.record()
        torch.cuda.synchronize()
        dt = a.elapsed_time(b) * 1e-3 / args.decode_steps
        step_bytes = 2 * Bd * Hd * D * D * 4 + 4 * Bd * Hd * D * el
        result["decode"] = {"workload": "configs[4]: B=256 H=16 dk=dv=128, %d in-place steps, a distinct token per step"
                                        % args.decode_steps,
                            "us_per_step": round(dt * 1e6, 2), "GBps": round(step_bytes / dt / 1e9, 1),
                            "roofline": {"bound": "hbm", "achieved": round(step_bytes / dt / 1e9, 1),
                                         "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                         "frac": round(step_bytes / dt / 1e9 / HBM_PEAK_GBS, 4),
                                         "algorithmic_bytes": step_bytes,
                                         "traffic": MEASURED_TRAFFIC_BYTES.get("step_kernel")}}

    # ---- CPU baseline: the fp64 oracle as it stands, on the same seeded inputs ----
    if not args.no_cpu_baseline:
        import oracle
        w = hosts[0]
        train_fwd(0)
        train_bwd(0)
        torch.cuda.synchronize()
        gpu_out = [x.float().cpu().numpy() for x in (o, gq, gf, gv)]
        reps, t_cpu = 0, 0.0
        while t_cpu < 10.0 and reps < 16:       # about ten seconds of CPU work
            c0 = time.perf_counter()
            o_ref, _ = oracle.fwd(w.q, w.f, w.v, None, want_hT=False)
            g_ref = oracle.bwd(w.q, w.f, w.v, w.dO, None, None, want_dh0=False)
            t_cpu += time.perf_counter() - c0
            reps += 1
        refs = [o_ref, g_ref[0], g_ref[1], g_ref[2]]
        errs = {}
        for name, x, r in zip(("o", "dq", "df", "dv"), gpu_out, refs):
            errs[name] = float("%.3e" % (np.max(np.abs(x - r)) / np.max(np.abs(r))))
        result["cpu_baseline"] = {"value": round(tokens * reps / t_cpu, 1), "unit": "tokens/s",
                                  "cores": oracle.threads(), "kind": "oracle",
                                  "sample": "the full benchmark workload (B=8,H=16,N=2048,d=128), fwd+bwd in fp64, "
                                            "%d repetition(s), %.1f s" % (reps, t_cpu)}
        result["parity_vs_oracle_full_size"] = errs
    torch.cuda.synchronize()
    result["gate_domain_flag"] = int(domain_flag.item())       # 0: every step of the headline ran inside the gate domain
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
