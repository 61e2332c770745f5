"""Seeded synthetic inputs with the shapes and gate statistics of the paper's workloads.

This module holds NO arithmetic of the method: it only draws random tensors and rounds them
to the storage type once, so that the HIP path and the CPU oracle (which never import each
other) can be fed bit-identical values.  Gates follow the lower-bounded construction of the
paper's Eq. 2, f = lb + (1 - lb) * sigmoid(z) with z ~ N(0, 1).

Draw order for every workload is fixed: q, z_f, v, [lb], [h0], [dO]; everything is drawn in
fp32 from numpy.random.default_rng(seed) and then rounded once to the storage dtype.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional

import numpy as np

BASE_SEED = 20240407


def bf16_round(x: np.ndarray) -> np.ndarray:
    """Round fp32 -> bf16 (round-to-nearest-even) and widen back to fp32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    bias = ((u >> 16) & 1) + np.uint32(0x7FFF)
    r = ((u + bias) & np.uint32(0xFFFF0000)).astype(np.uint32)
    return r.view(np.float32)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """The 16-bit patterns of fp32 values that are already bf16-representable."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    return (x.view(np.uint32) >> 16).astype(np.uint16)


def _sigmoid(z):
    return (1.0 / (1.0 + np.exp(-z.astype(np.float64)))).astype(np.float32)


@dataclass
class Workload:
    """One seeded input set.  All arrays are fp32 holding values exactly representable in the
    storage dtypes named by io_dtype / gate_dtype ("f32" or "bf16")."""
    name: str
    io_dtype: str
    gate_dtype: str
    q: np.ndarray
    f: np.ndarray
    v: np.ndarray
    h0: Optional[np.ndarray] = None
    dO: Optional[np.ndarray] = None
    dhT: Optional[np.ndarray] = None
    state: Optional[np.ndarray] = None          # decode workloads: initial state [B,H,dk,dv]
    chunk: int = 64
    meta: dict = field(default_factory=dict)


def _round(x, dtype):
    return bf16_round(x) if dtype == "bf16" else np.ascontiguousarray(x, dtype=np.float32)


def make_sequence(seed, B, H, N, dk, dv, *, io_dtype="bf16", gate_dtype=None, lb=0.0,
                  lb_per_head=None, with_h0=False, with_dO=False, with_dhT=False,
                  h0_std=0.1, name="custom", chunk=64) -> Workload:
    """q, v ~ N(0,1); f = lb + (1-lb)*sigmoid(N(0,1)).

    lb is a scalar, or lb_per_head=(lo, hi) draws one lower bound per head from U(lo, hi).
    """
    gate_dtype = gate_dtype or io_dtype
    rng = np.random.default_rng(seed)
    q = rng.standard_normal((B, H, N, dk), dtype=np.float32)
    z = rng.standard_normal((B, H, N, dk), dtype=np.float32)
    v = rng.standard_normal((B, H, N, dv), dtype=np.float32)
    if lb_per_head is not None:
        lbh = rng.uniform(lb_per_head[0], lb_per_head[1], size=(H,)).astype(np.float32)
        lbv = lbh.reshape(1, H, 1, 1)
    else:
        lbh = None
        lbv = np.float32(lb)
    f = (lbv + (np.float32(1.0) - lbv) * _sigmoid(z)).astype(np.float32)
    h0 = (h0_std * rng.standard_normal((B, H, dk, dv), dtype=np.float32)).astype(np.float32) \
        if with_h0 else None
    dO = rng.standard_normal((B, H, N, dv), dtype=np.float32) if with_dO else None
    dhT = (h0_std * rng.standard_normal((B, H, dk, dv), dtype=np.float32)).astype(np.float32) \
        if with_dhT else None
    f = _round(f, gate_dtype)
    f = np.minimum(f, np.float32(1.0))
    return Workload(name=name, io_dtype=io_dtype, gate_dtype=gate_dtype,
                    q=_round(q, io_dtype), f=f, v=_round(v, io_dtype), h0=h0,
                    dO=None if dO is None else _round(dO, io_dtype), dhT=dhT, chunk=chunk,
                    meta={"seed": seed, "B": B, "H": H, "N": N, "dk": dk, "dv": dv,
                          "lb": None if lbh is not None else float(lb),
                          "lb_per_head": None if lbh is None else lbh.tolist()})


def config0(scale=1) -> Workload:
    """Tiny forward, fp32: B=1, H=1, N=256, dk=dv=64, chunk 64, f = 0.5 + 0.5*sigmoid, h0 = 0."""
    return make_sequence(BASE_SEED + 0, 1, 1, 256 * scale, 64, 64, io_dtype="f32", lb=0.5,
                         name="config0_tiny_f32")


def config1() -> Workload:
    """Forward, bf16: B=4, H=8, N=1024, dk=dv=64, lb per head ~ U(0, 0.9), h0 ~ N(0, 0.1) fp32."""
    return make_sequence(BASE_SEED + 1, 4, 8, 1024, 64, 64, io_dtype="bf16", lb_per_head=(0.0, 0.9),
                         with_h0=True, name="config1_fwd_bf16")


def layer_lower_bound(layer: int, n_layers: int = 24) -> float:
    """Lower bound of layer `layer` in an n_layers stack at uniform initialisation of the
    lower-bound parameters: cumulative softmax gives l / L (the paper's cumax, shifted so
    that the first layer has bound zero and the last stays below one)."""
    return float(layer) / float(n_layers)


def config2(layer: int = 0, B=8, H=16, N=2048, d=128) -> Workload:
    """Layer-shaped forward+backward, bf16: B=8, H=16, N=2048, dk=dv=128; lb of the given layer
    of a 24-layer stack (layers 0, 12 and 23 are the ones measured); dO ~ N(0,1)."""
    w = make_sequence(BASE_SEED + 2 + 100 * layer, B, H, N, d, d, io_dtype="bf16",
                      lb=layer_lower_bound(layer), with_dO=True,
                      name="config2_layer%d_fwdbwd_bf16" % layer)
    w.meta["layer"] = layer
    return w


def config3(gate_dtype="bf16", B=2, H=16, N=16384, d=128) -> Workload:
    """Long sequence forward+backward, bf16: B=2, H=16, N=16384, f = 0.99 + 0.01*sigmoid."""
    return make_sequence(BASE_SEED + 3, B, H, N, d, d, io_dtype="bf16", gate_dtype=gate_dtype,
                         lb=0.99, with_dO=True, name="config3_long_fwdbwd_%sgate" % gate_dtype)


def config4(T=512, B=256, H=16, d=128, gate_dtype="bf16") -> Workload:
    """Decode: state [B,H,d,d] ~ N(0, 0.1) fp32; T tokens q, v ~ N(0,1) bf16,
    f = 0.9 + 0.1*sigmoid(N(0,1)); token tensors are [T,B,H,d], a distinct token per step."""
    rng = np.random.default_rng(BASE_SEED + 4)
    q = rng.standard_normal((T, B, H, d), dtype=np.float32)
    z = rng.standard_normal((T, B, H, d), dtype=np.float32)
    v = rng.standard_normal((T, B, H, d), dtype=np.float32)
    f = (np.float32(0.9) + np.float32(0.1) * _sigmoid(z)).astype(np.float32)
    state = (np.float32(0.1) * rng.standard_normal((B, H, d, d), dtype=np.float32)).astype(np.float32)
    f = np.minimum(_round(f, gate_dtype), np.float32(1.0))
    return Workload(name="config4_decode", io_dtype="bf16", gate_dtype=gate_dtype,
                    q=bf16_round(q), f=f, v=bf16_round(v), state=state,
                    meta={"seed": BASE_SEED + 4, "T": T, "B": B, "H": H, "dk": d, "dv": d})
