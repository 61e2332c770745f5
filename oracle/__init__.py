"""fp64 CPU oracle for the HGRN2 recurrence (paper Section 3.2, Eq. 3).

TEST INFRASTRUCTURE ONLY.  Nothing in the product package imports this; only the tests,
the smoke check and the CPU-baseline leg of the benchmark do.  The arithmetic lives in
``hgrn2_oracle.c`` (plain C, one token at a time); this module only compiles it with gcc,
marshals numpy arrays through ctypes and returns numpy arrays.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "hgrn2_oracle.c")
_LIB = os.path.join(_HERE, "libhgrn2_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle into a shared library next to its source."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
             "-ffp-contract=off", "-o", tmp, _SRC])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
    return _lib


_D = ctypes.POINTER(ctypes.c_double)


def _p(a):
    return None if a is None else a.ctypes.data_as(_D)


def _c(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.float64)


def threads() -> int:
    """Number of OpenMP threads the oracle will use."""
    return int(_load().hgrn2_oracle_threads())


def _check(rc):
    if rc != 0:
        raise RuntimeError("hgrn2 oracle returned status %d" % rc)


def fwd(q, f, v, h0=None, want_hT=True):
    """Eq. 3 over a whole sequence.  q, f: [B,H,N,dk]; v: [B,H,N,dv]; h0: [B,H,dk,dv] or None.

    Returns (o [B,H,N,dv], hT [B,H,dk,dv]); the input gate is tied, k = 1 - f.
    """
    q, f, v, h0 = _c(q), _c(f), _c(v), _c(h0)
    B, H, N, dk = q.shape
    dv = v.shape[-1]
    assert f.shape == q.shape and v.shape == (B, H, N, dv)
    assert h0 is None or h0.shape == (B, H, dk, dv)
    o = np.empty((B, H, N, dv), np.float64)
    hT = np.empty((B, H, dk, dv), np.float64) if want_hT else None
    _check(_load().hgrn2_oracle_fwd(B, H, N, dk, dv, _p(q), _p(f), _p(v), _p(h0), _p(o), _p(hT)))
    return o, hT


def fwd_untied(q, k, f, v, h0=None):
    """The same loop with a free key vector (GLA column of Table 4); for the f == 1 pin."""
    q, k, f, v, h0 = _c(q), _c(k), _c(f), _c(v), _c(h0)
    B, H, N, dk = q.shape
    dv = v.shape[-1]
    assert k.shape == q.shape and f.shape == q.shape
    o = np.empty((B, H, N, dv), np.float64)
    hT = np.empty((B, H, dk, dv), np.float64)
    _check(_load().hgrn2_oracle_fwd_untied(B, H, N, dk, dv, _p(q), _p(k), _p(f), _p(v), _p(h0),
                                           _p(o), _p(hT)))
    return o, hT


def step(q, f, v, state):
    """One token of Eq. 3.  q, f: [B,H,dk]; v: [B,H,dv]; state [B,H,dk,dv] is updated IN PLACE
    (must be a C-contiguous float64 array).  Returns o [B,H,dv]."""
    assert state.dtype == np.float64 and state.flags["C_CONTIGUOUS"]
    q, f, v = _c(q), _c(f), _c(v)
    B, H, dk = q.shape
    dv = v.shape[-1]
    assert state.shape == (B, H, dk, dv)
    o = np.empty((B, H, dv), np.float64)
    _check(_load().hgrn2_oracle_step(B, H, dk, dv, _p(q), _p(f), _p(v), _p(state), _p(o)))
    return o


def steps(q, f, v, state):
    """T consecutive single-token steps.  q, f: [T,B,H,dk]; v: [T,B,H,dv]; state updated in place.
    Returns o [T,B,H,dv]."""
    assert state.dtype == np.float64 and state.flags["C_CONTIGUOUS"]
    q, f, v = _c(q), _c(f), _c(v)
    T, B, H, dk = q.shape
    dv = v.shape[-1]
    assert state.shape == (B, H, dk, dv)
    o = np.empty((T, B, H, dv), np.float64)
    _check(_load().hgrn2_oracle_steps(T, B, H, dk, dv, _p(q), _p(f), _p(v), _p(state), _p(o)))
    return o


def bwd(q, f, v, dO, h0=None, dhT=None, want_dh0=True):
    """Reverse-mode gradients of L = sum(o * dO) + sum(hT * dhT).

    Returns (dq, df, dv, dh0); df already contains the tied path k = 1 - f.
    """
    q, f, v, dO, h0, dhT = _c(q), _c(f), _c(v), _c(dO), _c(h0), _c(dhT)
    B, H, N, dk = q.shape
    dv = v.shape[-1]
    assert dO.shape == v.shape
    dq = np.empty_like(q)
    df = np.empty_like(f)
    dvv = np.empty_like(v)
    dh0 = np.empty((B, H, dk, dv), np.float64) if want_dh0 else None
    _check(_load().hgrn2_oracle_bwd(B, H, N, dk, dv, _p(q), _p(f), _p(v), _p(h0), _p(dO), _p(dhT),
                                    _p(dq), _p(df), _p(dvv), _p(dh0)))
    return dq, df, dvv, dh0


# ---------------------------------------------------------------------------------------------
# Lower-bounded forget gate (paper Section 2, Eq. 2) and the cumulative-softmax lower bounds.
# Plain numpy in fp64, written from the definitions:
#     beta = cumsum(softmax(Gamma, over layers), over layers) - (its first row)
#     f    = beta + (1 - beta) * g,   g = sigmoid(z)
# Layouts: z, f: [B,H,N,dk]; beta: [H,dk] (one lower bound per channel of the layer, shared by
# batch and time); Gamma, the bounds of all layers: [L, d].
# ---------------------------------------------------------------------------------------------
def cumax(gamma):
    """Lower bounds of all layers from the learnable matrix Gamma [L, d]: softmax over the layer
    axis, cumulative sum over the layer axis, minus the first layer's row (so that the first
    layer has bound zero and the last stays below one)."""
    gamma = np.asarray(gamma, dtype=np.float64)
    e = np.exp(gamma - gamma.max(axis=0, keepdims=True))
    p = e / e.sum(axis=0, keepdims=True)
    c = np.cumsum(p, axis=0)
    return c - c[0:1]


def gate(z, beta):
    """f = beta + (1 - beta) * sigmoid(z), Eq. 2.  z: [B,H,N,dk]; beta: [H,dk]."""
    z = np.asarray(z, dtype=np.float64)
    b = np.asarray(beta, dtype=np.float64)[None, :, None, :]
    g = 1.0 / (1.0 + np.exp(-z))
    return b + (1.0 - b) * g


def fwd_gated(q, z, beta, v, h0=None, want_hT=True):
    """Eq. 3 with the gate of Eq. 2 formed from its pre-activation z."""
    return fwd(q, gate(z, beta), v, h0, want_hT)


def bwd_gated(q, z, beta, v, dO, h0=None, dhT=None, want_dh0=True):
    """Gradients of L = sum(o * dO) + sum(hT * dhT) w.r.t. q, z, beta, v, h0 (chain rule through
    Eq. 2: df/dz = (1 - beta) g (1 - g), df/dbeta = 1 - g, summed over batch and time for beta)."""
    z = np.asarray(z, dtype=np.float64)
    b = np.asarray(beta, dtype=np.float64)[None, :, None, :]
    g = 1.0 / (1.0 + np.exp(-z))
    dq, df, dv, dh0 = bwd(q, b + (1.0 - b) * g, v, dO, h0, dhT, want_dh0)
    dz = df * (1.0 - b) * g * (1.0 - g)
    dbeta = (df * (1.0 - g)).sum(axis=(0, 2))
    return dq, dz, dbeta, dv, dh0


# ---------------------------------------------------------------------------------------------
# HGRN1: the element-wise gated linear recurrence the paper starts from (Section 2, Eq. 1 with
# the gate of Eq. 2 already formed):   h_t = f_t * h_{t-1} + (1 - f_t) * i_t,   y_t = h_t * o_t
# per channel.  Plain numpy in fp64, one token at a time.  f, i, o: [B,N,d]; h0: [B,d] or None.
# ---------------------------------------------------------------------------------------------
def hgrn1_fwd(f, i, o, h0=None):
    f, i, o = (np.asarray(x, dtype=np.float64) for x in (f, i, o))
    B, N, d = f.shape
    h = np.zeros((B, d)) if h0 is None else np.array(h0, dtype=np.float64)
    y = np.empty((B, N, d))
    for t in range(N):
        h = f[:, t] * h + (1.0 - f[:, t]) * i[:, t]
        y[:, t] = h * o[:, t]
    return y, h


def hgrn1_bwd(f, i, o, dy, h0=None, dhN=None):
    """Reverse mode of the loop above for L = sum(y * dy) + sum(h_N * dhN).
    Returns (df, di, do, dh0); df includes the tied input gate 1 - f."""
    f, i, o, dy = (np.asarray(x, dtype=np.float64) for x in (f, i, o, dy))
    B, N, d = f.shape
    hs = np.empty((B, N + 1, d))
    hs[:, 0] = 0.0 if h0 is None else np.asarray(h0, dtype=np.float64)
    for t in range(N):
        hs[:, t + 1] = f[:, t] * hs[:, t] + (1.0 - f[:, t]) * i[:, t]
    dh = np.zeros((B, d)) if dhN is None else np.array(dhN, dtype=np.float64)
    df, di, do = np.empty_like(f), np.empty_like(f), np.empty_like(f)
    for t in range(N - 1, -1, -1):
        dh = dh + dy[:, t] * o[:, t]                 # dL/dh_t
        do[:, t] = dy[:, t] * hs[:, t + 1]
        df[:, t] = dh * (hs[:, t] - i[:, t])
        di[:, t] = dh * (1.0 - f[:, t])
        dh = dh * f[:, t]                            # dL/dh_{t-1} through the recurrence
    return df, di, do, dh


# ---------------------------------------------------------------------------------------------
# The HGRN1 layer's element-wise part as the paper writes it (Section 2): the three vectors of
# Eq. 1 come from pre-activations (the projections' outputs, biases included) through
#     g = sigmoid(zf),   i = tau(zi) with tau = SiLU,   o = sigmoid(zo),
# and the forget gate gets its lower bound by Eq. 2,  f = beta + (1 - beta) g,  beta: [d] per layer.
# ---------------------------------------------------------------------------------------------
def _sigmoid(z):
    return 1.0 / (1.0 + np.exp(-np.asarray(z, dtype=np.float64)))


def hgrn1_activations(zf, zi, zo, beta):
    b = np.asarray(beta, dtype=np.float64)[None, None, :]
    zi = np.asarray(zi, dtype=np.float64)
    return b + (1.0 - b) * _sigmoid(zf), zi * _sigmoid(zi), _sigmoid(zo)


def hgrn1_fwd_act(zf, zi, zo, beta, h0=None):
    return hgrn1_fwd(*hgrn1_activations(zf, zi, zo, beta), h0)


def hgrn1_bwd_act(zf, zi, zo, beta, dy, h0=None, dhN=None):
    """Gradients of L = sum(y * dy) + sum(h_N * dhN) w.r.t. zf, zi, zo, beta, h0: the chain rule
    through the activations, d sigmoid = s (1 - s), d SiLU(z) = s (1 + z (1 - s)), and
    df/dbeta = 1 - g summed over batch and time."""
    f, i, o = hgrn1_activations(zf, zi, zo, beta)
    df, di, do, dh0 = hgrn1_bwd(f, i, o, dy, h0, dhN)
    b = np.asarray(beta, dtype=np.float64)[None, None, :]
    g, si = _sigmoid(zf), _sigmoid(zi)
    zi = np.asarray(zi, dtype=np.float64)
    dzf = df * (1.0 - b) * g * (1.0 - g)
    dzi = di * si * (1.0 + zi * (1.0 - si))
    dzo = do * o * (1.0 - o)
    dbeta = (df * (1.0 - g)).sum(axis=(0, 1))
    return dzf, dzi, dzo, dbeta, dh0


# ---------------------------------------------------------------------------------------------
# What the exactness of a chunkwise evaluation with one reference row per chunk half depends on:
# the smallest product of one channel's gates over a half chunk (tokens [C n, C n + C/2) and
# [C n + C/2, C n + C) of every sequence; a ragged last piece counts with the tokens it has).
# ---------------------------------------------------------------------------------------------
# ---- input side of the HGRU2 token mixer (paper Section 2, Eq. 1, feeding Eq. 2 and Eq. 3) --------
# Three affine maps of the layer input x_t and their activations,
#     g_t = sigmoid(U x_t + b_u),   i_t = SiLU(V x_t + b_v),   o_t = sigmoid(W x_t + b_w),
# written out with numpy matmuls in fp64.  The forget gate's pre-activation z = U x + b_u is
# returned instead of g, because the lower bound of Eq. 2 is applied to g inside `gate`.
# Weights are [d_out, d_in] (row = output channel), x is [B, N, d].
def hgru2_proj(x, U, V, W, bu, bv, bw):
    x, U, V, W = (np.asarray(a, dtype=np.float64) for a in (x, U, V, W))
    bu, bv, bw = (np.asarray(a, dtype=np.float64) for a in (bu, bv, bw))
    z = x @ U.T + bu
    av = x @ V.T + bv
    aw = x @ W.T + bw
    return z, av * _sigmoid(av), _sigmoid(aw)


def hgru2_proj_bwd(x, U, V, W, bu, bv, bw, dz, di, do):
    """Reverse mode of hgru2_proj for L = sum(z dz) + sum(i di) + sum(o do): dx, dU, dV, dW, dbu, dbv, dbw."""
    x, U, V, W = (np.asarray(a, dtype=np.float64) for a in (x, U, V, W))
    bv, bw = np.asarray(bv, dtype=np.float64), np.asarray(bw, dtype=np.float64)
    dz, di, do = (np.asarray(a, dtype=np.float64) for a in (dz, di, do))
    av = x @ V.T + bv
    sv = _sigmoid(av)
    o = _sigmoid(x @ W.T + bw)
    dav = di * sv * (1.0 + av * (1.0 - sv))          # d SiLU(a) / da
    daw = do * o * (1.0 - o)                          # d sigmoid(a) / da
    d = x.shape[-1]
    x2 = x.reshape(-1, d)
    flat = lambda a: a.reshape(-1, a.shape[-1])
    dx = dz @ U + dav @ V + daw @ W
    return (dx, flat(dz).T @ x2, flat(dav).T @ x2, flat(daw).T @ x2,
            flat(dz).sum(axis=0), flat(dav).sum(axis=0), flat(daw).sum(axis=0))


def _split_heads(a, H):          # [B, N, H * dh] -> [B, H, N, dh]
    B, N, d = a.shape
    return np.ascontiguousarray(a.reshape(B, N, H, d // H).transpose(0, 2, 1, 3))


def _merge_heads(a):             # [B, H, N, dh] -> [B, N, H * dh]
    B, H, N, dh = a.shape
    return np.ascontiguousarray(a.transpose(0, 2, 1, 3).reshape(B, N, H * dh))


def hgru2_layer_fwd(x, U, V, W, bu, bv, bw, beta, H, h0=None):
    """Eq. 1 -> Eq. 2 -> Eq. 3 with H heads: y [B, N, d] and the final states [B, H, dh, dh].
    beta: the layer's lower bounds, [d] (viewed as [H][dh]).  Table 4's naming: q = o, v = i."""
    z, i, o = hgru2_proj(x, U, V, W, bu, bv, bw)
    d = z.shape[-1]
    y, hT = fwd_gated(_split_heads(o, H), _split_heads(z, H), np.asarray(beta, dtype=np.float64).reshape(H, d // H),
                      _split_heads(i, H), h0)
    return _merge_heads(y), hT


def hgru2_layer_bwd(x, U, V, W, bu, bv, bw, beta, H, dy, h0=None, dhT=None):
    """Reverse mode of hgru2_layer_fwd for L = sum(y dy) + sum(hT dhT):
    dx, dU, dV, dW, dbu, dbv, dbw, dbeta [d], dh0."""
    z, i, o = hgru2_proj(x, U, V, W, bu, bv, bw)
    d = z.shape[-1]
    b2 = np.asarray(beta, dtype=np.float64).reshape(H, d // H)
    dq, dz, dbeta, dv, dh0 = bwd_gated(_split_heads(o, H), _split_heads(z, H), b2, _split_heads(i, H),
                                       _split_heads(np.asarray(dy, dtype=np.float64), H), h0, dhT)
    g = hgru2_proj_bwd(x, U, V, W, bu, bv, bw, _merge_heads(dz), _merge_heads(dv), _merge_heads(dq))
    return g + (dbeta.reshape(-1), dh0)


def min_gate_product(f, chunk=64):
    """f: [B,H,N,dk] -> float (1.0 for an empty input)."""
    f = np.asarray(f, dtype=np.float64)
    N = f.shape[2]
    half = chunk // 2
    best = 1.0
    for s in range(0, N, half):
        best = min(best, float(np.prod(f[:, :, s:s + half, :], axis=2).min()))
    return best
