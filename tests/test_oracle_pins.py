"""Pins for the fp64 CPU oracle: every check compares it with something OTHER than its own loop.

P1  brute-force quadratic ("attention") form with the per-channel decay mask
P2  f == 1: tied gate -> state frozen at h0; untied key -> cumulative linear attention
P3  f == 0: o_t = (sum_a q_t[a]) v_t
P4  constant gate closed form 1 - c^t
P5  split / hand-off (hT -> h0), N x step == fwd, and the backward hand-off (dh0 -> dhT)
P6  convexity invariant of the tied gate (key and forget gate sum to one)
P7  chunkwise regrouping (the algebra the GPU kernels use), any chunk length
P8  linearity in v (+h0) and in q
P9  fp64 central finite differences, torch autograd, and the gate-gradient suffix identity
A two-token example in exact rational arithmetic closes the list (the paper prints no numeric
values of Eq. 3, so tests/golden/ holds no fixture for it).
"""
import os

import numpy as np
import pytest

import oracle

RNG = np.random.default_rng(12345)
HERE = os.path.dirname(os.path.abspath(__file__))


def rand_inputs(B, H, N, dk, dv, lo=0.05, hi=1.0, rng=RNG, h0=True):
    q = rng.standard_normal((B, H, N, dk))
    f = rng.uniform(lo, hi, size=(B, H, N, dk))
    v = rng.standard_normal((B, H, N, dv))
    h = 0.3 * rng.standard_normal((B, H, dk, dv)) if h0 else None
    return q, f, v, h


# ----------------------------------------------------------------------------- P1
def quadratic_form(q, f, v, h0):
    """O = A V + (Q * prod_{s<=i} f_s) h0, A_ij = sum_a q_i[a] k_j[a] prod_{s=j+1..i} f_s[a], j<=i.

    Written with explicit products over the gate (no recurrence, no logs): O(N^2 dk)."""
    B, H, N, dk = q.shape
    dv = v.shape[-1]
    o = np.zeros((B, H, N, dv))
    k = 1.0 - f
    for b in range(B):
        for h in range(H):
            for i in range(N):
                acc = np.zeros(dv)
                for j in range(i + 1):
                    decay = np.prod(f[b, h, j + 1:i + 1, :], axis=0)        # empty product = 1
                    acc += np.sum(q[b, h, i] * k[b, h, j] * decay) * v[b, h, j]
                if h0 is not None:
                    acc += (q[b, h, i] * np.prod(f[b, h, :i + 1, :], axis=0)) @ h0[b, h]
                o[b, h, i] = acc
    return o


@pytest.mark.parametrize("N,dk,dv,use_h0", [(1, 3, 2, True), (7, 4, 5, True), (48, 8, 6, False),
                                            (96, 16, 16, True)])
def test_p1_bruteforce_quadratic_form(N, dk, dv, use_h0):
    q, f, v, h0 = rand_inputs(2, 2, N, dk, dv, h0=use_h0)
    o, hT = oracle.fwd(q, f, v, h0)
    ref = quadratic_form(q, f, v, h0)
    assert np.max(np.abs(o - ref)) <= 1e-12 * max(1.0, np.max(np.abs(ref)))
    # final state from the unrolled sum: S_N = sum_j Diag(prod_{s>j} f) k_j^T v_j + Diag(prod f) h0
    k = 1.0 - f
    S = np.zeros_like(hT)
    for j in range(N):
        decay = np.prod(f[:, :, j + 1:, :], axis=2)
        S += (decay * k[:, :, j])[..., None] * v[:, :, j][..., None, :]
    if h0 is not None:
        S += np.prod(f, axis=2)[..., None] * h0
    assert np.max(np.abs(hT - S)) <= 1e-12


# ----------------------------------------------------------------------------- P2
def test_p2_f_one_tied_freezes_state():
    q, f, v, h0 = rand_inputs(2, 3, 20, 5, 4)
    f = np.ones_like(f)
    o, hT = oracle.fwd(q, f, v, h0)
    assert np.array_equal(hT, h0)
    assert np.allclose(o, np.einsum("bhna,bhac->bhnc", q, h0), rtol=0, atol=1e-13)
    o0, hT0 = oracle.fwd(q, f, v, None)
    assert np.all(o0 == 0) and np.all(hT0 == 0)


def test_p2_f_one_untied_is_cumulative_linear_attention():
    q, f, v, _ = rand_inputs(2, 2, 33, 6, 7, h0=False)
    k = RNG.standard_normal(q.shape)
    f = np.ones_like(f)
    o, hT = oracle.fwd_untied(q, k, f, v)
    A = np.tril(np.einsum("bhia,bhja->bhij", q, k))          # causal mask, diagonal kept
    assert np.allclose(o, A @ v, rtol=0, atol=1e-12)
    assert np.allclose(hT, np.einsum("bhna,bhnc->bhac", k, v), rtol=0, atol=1e-12)


def test_untied_with_tied_key_equals_tied():
    q, f, v, h0 = rand_inputs(1, 2, 17, 4, 3)
    o1, h1 = oracle.fwd(q, f, v, h0)
    o2, h2 = oracle.fwd_untied(q, 1.0 - f, f, v, h0)
    assert np.array_equal(o1, o2) and np.array_equal(h1, h2)


# ----------------------------------------------------------------------------- P3
def test_p3_f_zero():
    q, f, v, h0 = rand_inputs(2, 2, 11, 5, 6)
    f = np.zeros_like(f)
    o, hT = oracle.fwd(q, f, v, h0)
    assert np.allclose(o, q.sum(-1, keepdims=True) * v, rtol=0, atol=1e-13)
    assert np.allclose(hT, np.broadcast_to(v[:, :, -1][:, :, None, :], hT.shape))


# ----------------------------------------------------------------------------- P4
@pytest.mark.parametrize("c", [0.0, 0.3, 0.9, 0.999, 1.0])
def test_p4_constant_gate_closed_form(c):
    B, H, N, dk, dv = 1, 2, 200, 6, 5
    q = np.ones((B, H, N, dk))
    v = np.ones((B, H, N, dv))
    f = np.full((B, H, N, dk), c)
    o, hT = oracle.fwd(q, f, v, None)
    t = np.arange(1, N + 1, dtype=np.float64)
    want = dk * (1.0 - c ** t)
    assert np.allclose(o, want[None, None, :, None], rtol=1e-12, atol=1e-13)
    assert np.allclose(hT, 1.0 - c ** N, rtol=1e-12, atol=1e-13)


# ----------------------------------------------------------------------------- P5
def test_p5_split_handoff_forward_and_steps():
    q, f, v, h0 = rand_inputs(2, 2, 70, 6, 5)
    o, hT = oracle.fwd(q, f, v, h0)
    m = 29
    o1, h1 = oracle.fwd(q[:, :, :m], f[:, :, :m], v[:, :, :m], h0)
    o2, h2 = oracle.fwd(q[:, :, m:], f[:, :, m:], v[:, :, m:], h1)
    assert np.array_equal(np.concatenate([o1, o2], 2), o) and np.array_equal(h2, hT)
    st = h0.copy()
    for t in range(q.shape[2]):
        ot = oracle.step(q[:, :, t], f[:, :, t], v[:, :, t], st)
        assert np.array_equal(ot, o[:, :, t])
    assert np.array_equal(st, hT)
    st2 = h0.copy()
    tok = lambda x: np.ascontiguousarray(np.moveaxis(x, 2, 0))
    o_s = oracle.steps(tok(q), tok(f), tok(v), st2)
    assert np.array_equal(np.moveaxis(o_s, 0, 2), o) and np.array_equal(st2, hT)


def test_p5_split_handoff_backward():
    q, f, v, h0 = rand_inputs(1, 2, 50, 5, 4)
    dO = RNG.standard_normal(v.shape)
    dhT = RNG.standard_normal(h0.shape)
    dq, df, dv, dh0 = oracle.bwd(q, f, v, dO, h0, dhT)
    m = 21
    _, h1 = oracle.fwd(q[:, :, :m], f[:, :, :m], v[:, :, :m], h0)
    dq2, df2, dv2, dh1 = oracle.bwd(q[:, :, m:], f[:, :, m:], v[:, :, m:], dO[:, :, m:], h1, dhT)
    dq1, df1, dv1, dh0b = oracle.bwd(q[:, :, :m], f[:, :, :m], v[:, :, :m], dO[:, :, :m], h0, dh1)
    for whole, a, b in ((dq, dq1, dq2), (df, df1, df2), (dv, dv1, dv2)):
        assert np.allclose(whole, np.concatenate([a, b], 2), rtol=1e-12, atol=1e-12)
    assert np.allclose(dh0, dh0b, rtol=1e-12, atol=1e-12)


# ----------------------------------------------------------------------------- P6
def test_p6_convexity_invariant():
    B, H, N, dk, dv = 2, 2, 40, 5, 4
    q, f, v, _ = rand_inputs(B, H, N, dk, dv, lo=0.0, hi=1.0, h0=False)
    vbar = RNG.standard_normal((B, H, 1, dv))
    v_const = np.broadcast_to(vbar, v.shape).copy()
    h0 = np.broadcast_to(vbar, (B, H, dk, dv)).copy()
    _, hT = oracle.fwd(q, f, v_const, h0)
    assert np.allclose(hT, h0, rtol=0, atol=1e-13)        # convex combination of equal rows
    h0r = RNG.standard_normal((B, H, dk, dv))
    st = h0r.copy()
    lo = h0r.copy()                                  # running per-entry bounds
    hi = h0r.copy()
    for t in range(N):
        oracle.step(q[:, :, t], f[:, :, t], v[:, :, t], st)
        lo = np.minimum(lo, v[:, :, t][:, :, None, :])
        hi = np.maximum(hi, v[:, :, t][:, :, None, :])
        assert np.all(st >= lo - 1e-13) and np.all(st <= hi + 1e-13)


# ----------------------------------------------------------------------------- P7
def chunkwise_fwd(q, f, v, h0, C):
    """fp64 regrouping into chunks of C: O = tril(Q~ K~^T) V + Q~ S_n, S_{n+1} = Diag(g) S_n + K^^T V,
    with chunk-local cumulative gate products (no logs, so f = 0 inside a chunk is avoided by
    the caller)."""
    B, H, N, dk = q.shape
    dv = v.shape[-1]
    S = np.zeros((B, H, dk, dv)) if h0 is None else h0.copy()
    o = np.zeros((B, H, N, dv))
    for s in range(0, N, C):
        e = min(N, s + C)
        Q, F, V = q[:, :, s:e], f[:, :, s:e], v[:, :, s:e]
        K = 1.0 - F
        G = np.cumprod(F, axis=2)                     # Gamma_r, inclusive
        g = G[:, :, -1]                               # whole-chunk decay
        Qs, Ks, Kh = Q * G, K / G, K * (g[:, :, None] / G)
        P = np.tril(np.einsum("bhia,bhja->bhij", Qs, Ks))
        o[:, :, s:e] = P @ V + np.einsum("bhia,bhac->bhic", Qs, S)
        S = g[..., None] * S + np.einsum("bhja,bhjc->bhac", Kh, V)
    return o, S


@pytest.mark.parametrize("C", [1, 16, 64, 100])
def test_p7_chunk_invariance(C):
    q, f, v, h0 = rand_inputs(1, 2, 100, 8, 6, lo=0.4)
    o, hT = oracle.fwd(q, f, v, h0)
    oc, hc = chunkwise_fwd(q, f, v, h0, C)
    assert np.allclose(o, oc, rtol=1e-9, atol=1e-9) and np.allclose(hT, hc, rtol=1e-9, atol=1e-9)


# ----------------------------------------------------------------------------- P8
def test_p8_linearity():
    q, f, v, h0 = rand_inputs(1, 2, 25, 5, 4)
    q2, _, v2, h02 = rand_inputs(1, 2, 25, 5, 4)
    a, b = 0.7, -1.9
    o1, h1 = oracle.fwd(q, f, v, h0)
    o2, h2 = oracle.fwd(q, f, v2, h02)
    o12, h12 = oracle.fwd(q, f, a * v + b * v2, a * h0 + b * h02)
    assert np.allclose(o12, a * o1 + b * o2, atol=1e-12) and np.allclose(h12, a * h1 + b * h2, atol=1e-12)
    o3, _ = oracle.fwd(q2, f, v, h0)
    o13, _ = oracle.fwd(a * q + b * q2, f, v, h0)
    assert np.allclose(o13, a * o1 + b * o3, atol=1e-12)


# ----------------------------------------------------------------------------- P9
def loss(q, f, v, h0, dO, dhT):
    o, hT = oracle.fwd(q, f, v, h0)
    return float(np.sum(o * dO) + np.sum(hT * dhT))


@pytest.mark.parametrize("N", [1, 5, 70])      # 70 crosses the oracle's checkpoint interval of 64
def test_p9_finite_differences(N):
    rng = np.random.default_rng(99 + N)
    B, H, dk, dv = 1, 2, 4, 3
    q, f, v, h0 = rand_inputs(B, H, N, dk, dv, lo=0.2, hi=0.95, rng=rng)
    dO = rng.standard_normal(v.shape)
    dhT = rng.standard_normal(h0.shape)
    grads = oracle.bwd(q, f, v, dO, h0, dhT)
    eps = 1e-6
    args = [q, f, v, h0]
    for which, g in zip(range(4), grads):
        x = args[which]
        flat = x.reshape(-1)
        idx = rng.choice(flat.size, size=min(flat.size, 60), replace=False)
        for i in idx:
            old = flat[i]
            flat[i] = old + eps
            lp = loss(q, f, v, h0, dO, dhT)
            flat[i] = old - eps
            lm = loss(q, f, v, h0, dO, dhT)
            flat[i] = old
            fd = (lp - lm) / (2 * eps)
            assert abs(fd - g.reshape(-1)[i]) <= 1e-7 * max(1.0, abs(fd)), (which, i, fd, g.reshape(-1)[i])


def test_p9_torch_autograd():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(7)
    B, H, N, dk, dv = 2, 2, 37, 5, 6
    q, f, v, h0 = rand_inputs(B, H, N, dk, dv, lo=0.1, hi=1.0, rng=rng)
    dO = rng.standard_normal(v.shape)
    dhT = rng.standard_normal(h0.shape)
    tq, tf, tv, th = (torch.tensor(x, dtype=torch.float64, requires_grad=True) for x in (q, f, v, h0))
    S = th
    outs = []
    for t in range(N):
        S = tf[:, :, t, :, None] * S + (1 - tf[:, :, t, :, None]) * tv[:, :, t, None, :]
        outs.append(torch.einsum("bha,bhac->bhc", tq[:, :, t], S))
    L = (torch.stack(outs, 2) * torch.tensor(dO)).sum() + (S * torch.tensor(dhT)).sum()
    L.backward()
    dq, df, dv_, dh0 = oracle.bwd(q, f, v, dO, h0, dhT)
    for mine, ref in ((dq, tq.grad), (df, tf.grad), (dv_, tv.grad), (dh0, th.grad)):
        assert np.allclose(mine, ref.numpy(), rtol=1e-11, atol=1e-11)


def test_p9_gate_gradient_suffix_identity():
    """f * (decay-path gradient) at step s equals sum_{t>=s}(q_t dq_t - k_t dk_t) + rowsum(dhT * hT);
    dk is recovered from the untied split: df = dd - dk and dk_t = sum_b dS_t[a,b] v_t[b]."""
    rng = np.random.default_rng(3)
    B, H, N, dk, dv = 1, 2, 45, 4, 5
    q, f, v, h0 = rand_inputs(B, H, N, dk, dv, lo=0.2, rng=rng)
    dO = rng.standard_normal(v.shape)
    dhT = rng.standard_normal(h0.shape)
    dq, df, dv_, _ = oracle.bwd(q, f, v, dO, h0, dhT)
    _, hT = oracle.fwd(q, f, v, h0)
    # dk via finite differences of the untied loop (independent of oracle.bwd)
    k = 1.0 - f
    eps = 1e-6
    dk_fd = np.zeros_like(k)
    for idx in np.ndindex(*k.shape):
        old = k[idx]
        k[idx] = old + eps
        op, hp = oracle.fwd_untied(q, k, f, v, h0)
        k[idx] = old - eps
        om, hm = oracle.fwd_untied(q, k, f, v, h0)
        k[idx] = old
        dk_fd[idx] = (np.sum((op - om) * dO) + np.sum((hp - hm) * dhT)) / (2 * eps)
    dd = df + dk_fd                                   # decay-path gradient
    terms = q * dq - (1.0 - f) * dk_fd
    suffix = np.flip(np.cumsum(np.flip(terms, 2), 2), 2) + np.sum(dhT * hT, -1)[:, :, None, :]
    assert np.allclose(f * dd, suffix, rtol=1e-6, atol=1e-6)


# ----------------------------------------------------------------------------- two-token closed form
def test_two_token_closed_form_exact():
    """N = 2, dk = 2, dv = 1 written out term by term in exact rational arithmetic (all inputs
    dyadic, so the fp64 oracle must reproduce every value exactly)."""
    from fractions import Fraction as Fr
    q1, q2 = (Fr(1), Fr(2)), (Fr(-1), Fr(1))
    f1, f2 = (Fr(1, 2), Fr(1, 4)), (Fr(3, 4), Fr(1, 2))
    v1, v2 = Fr(2), Fr(-4)
    h0 = (Fr(1), Fr(-2))
    g1, g2 = Fr(1), Fr(3)                                    # upstream gradients of o_1, o_2
    S1 = tuple(f1[a] * h0[a] + (1 - f1[a]) * v1 for a in range(2))
    S2 = tuple(f2[a] * S1[a] + (1 - f2[a]) * v2 for a in range(2))
    o1 = q1[0] * S1[0] + q1[1] * S1[1]
    o2 = q2[0] * S2[0] + q2[1] * S2[1]
    # L = g1 o1 + g2 o2, differentiated by hand
    dS2 = tuple(q2[a] * g2 for a in range(2))
    dS1 = tuple(q1[a] * g1 + f2[a] * dS2[a] for a in range(2))
    want = {
        "o": [o1, o2], "hT": list(S2),
        "dq": [g1 * S1[0], g1 * S1[1], g2 * S2[0], g2 * S2[1]],
        "df": [dS1[0] * (h0[0] - v1), dS1[1] * (h0[1] - v1), dS2[0] * (S1[0] - v2), dS2[1] * (S1[1] - v2)],
        "dv": [sum((1 - f1[a]) * dS1[a] for a in range(2)), sum((1 - f2[a]) * dS2[a] for a in range(2))],
        "dh0": [f1[0] * dS1[0], f1[1] * dS1[1]],
    }
    assert (o1, o2) == (Fr(7, 2), Fr(-13, 8)) and want["dv"] == [Fr(2), Fr(3, 4)]   # by hand
    arr = lambda xs, shape: np.array([float(x) for x in xs], dtype=np.float64).reshape(shape)
    q = arr(q1 + q2, (1, 1, 2, 2)); f = arr(f1 + f2, (1, 1, 2, 2)); v = arr([v1, v2], (1, 1, 2, 1))
    h = arr(h0, (1, 1, 2, 1)); dO = arr([g1, g2], (1, 1, 2, 1))
    o, hT = oracle.fwd(q, f, v, h)
    dq, df, dv, dh0 = oracle.bwd(q, f, v, dO, h, None)
    assert np.array_equal(o.reshape(-1), arr(want["o"], -1))
    assert np.array_equal(hT.reshape(-1), arr(want["hT"], -1))
    assert np.array_equal(dq.reshape(-1), arr(want["dq"], -1))
    assert np.array_equal(df.reshape(-1), arr(want["df"], -1))
    assert np.array_equal(dv.reshape(-1), arr(want["dv"], -1))
    assert np.array_equal(dh0.reshape(-1), arr(want["dh0"], -1))


# ----------------------------------------------------------------------------- planted mistakes
def test_pins_detect_planted_mistakes():
    """A dropped tie, a stale-state read-out or a transposed state would each break a pin."""
    q, f, v, h0 = rand_inputs(1, 1, 12, 4, 4)
    o, _ = oracle.fwd(q, f, v, h0)
    ref = quadratic_form(q, f, v, h0)
    # read-out from S_{t-1} instead of S_t
    stale = np.zeros_like(o)
    S = h0[0, 0].copy()
    for t in range(12):
        stale[0, 0, t] = q[0, 0, t] @ S
        S = f[0, 0, t][:, None] * S + (1 - f[0, 0, t])[:, None] * v[0, 0, t][None, :]
    assert np.max(np.abs(stale - ref)) > 1e-3 and np.max(np.abs(o - ref)) < 1e-12
    # untied key k = 1 would violate the convexity pin
    o_bad, h_bad = oracle.fwd_untied(q, np.ones_like(q), f, np.ones_like(v), np.ones_like(h0))
    assert np.max(np.abs(h_bad - 1.0)) > 1e-3


# ------------------------------------------------------------------ lower-bounded gate (Eq. 2)
def test_gate_closed_forms_and_library_sigmoid():
    """z = 0 gives (1 + beta)/2; z -> +-inf gives 1 and beta; beta = 0 reduces to the logistic
    function, checked against scipy's."""
    from scipy.special import expit
    rng = np.random.default_rng(5)
    beta = rng.uniform(0.0, 0.95, size=(3, 8))
    z0 = np.zeros((2, 3, 5, 8))
    assert np.allclose(oracle.gate(z0, beta), (1.0 + beta)[None, :, None, :] / 2.0, rtol=0, atol=1e-15)
    assert np.allclose(oracle.gate(z0 + 50.0, beta), 1.0, rtol=0, atol=1e-15)
    assert np.allclose(oracle.gate(z0 - 50.0, beta), np.broadcast_to(beta[None, :, None, :], z0.shape), rtol=0, atol=1e-15)
    z = rng.standard_normal((2, 3, 5, 8)) * 3.0
    assert np.allclose(oracle.gate(z, np.zeros((3, 8))), expit(z), rtol=1e-14, atol=0)
    f = oracle.gate(z, beta)
    b = np.broadcast_to(beta[None, :, None, :], z.shape)
    assert np.all(f > b) and np.all(f < 1.0)                     # the bound is a bound
    assert np.all(oracle.gate(z + 0.1, beta) > f)                # increasing in z
    assert np.allclose((f - b) / (1.0 - b), expit(z), rtol=1e-13)  # the residual is the plain gate


def test_cumax_properties_and_uniform_case():
    """Rows increase with the layer, the first is zero, the last is 1 - softmax_0 < 1; a constant
    Gamma gives l / L (the bounds the layer-shaped workload uses); softmax/cumsum against scipy/numpy."""
    from scipy.special import softmax
    rng = np.random.default_rng(6)
    gamma = rng.standard_normal((24, 16))
    beta = oracle.cumax(gamma)
    assert np.all(beta[0] == 0.0)
    assert np.all(np.diff(beta, axis=0) > 0.0)
    p = softmax(gamma, axis=0)
    assert np.allclose(beta[-1], 1.0 - p[0], rtol=1e-13)
    assert np.allclose(beta, np.cumsum(p, axis=0) - p[0], rtol=1e-13, atol=1e-15)
    uni = oracle.cumax(np.full((24, 4), 0.37))
    assert np.allclose(uni, (np.arange(24) / 24.0)[:, None], rtol=1e-13, atol=1e-15)
    from paper_2404_07904_amd import synth
    assert abs(uni[12, 0] - synth.layer_lower_bound(12)) < 1e-15


def test_bwd_gated_finite_differences():
    """Central differences of L w.r.t. every entry of z and beta (and a sample of q, v) on a tiny case."""
    rng = np.random.default_rng(8)
    B, H, N, dk, dv = 2, 2, 9, 3, 4
    q, v = rng.standard_normal((B, H, N, dk)), rng.standard_normal((B, H, N, dv))
    z = rng.standard_normal((B, H, N, dk))
    beta = rng.uniform(0.0, 0.9, size=(H, dk))
    h0 = 0.3 * rng.standard_normal((B, H, dk, dv))
    dO, dhT = rng.standard_normal((B, H, N, dv)), rng.standard_normal((B, H, dk, dv))

    def loss(z_, beta_, q_=q, v_=v):
        o, hT = oracle.fwd_gated(q_, z_, beta_, v_, h0)
        return float((o * dO).sum() + (hT * dhT).sum())

    dq, dz, dbeta, dvv, _ = oracle.bwd_gated(q, z, beta, v, dO, h0, dhT)
    eps = 1e-6
    num = np.zeros_like(z)
    for idx in np.ndindex(*z.shape):
        zp, zm = z.copy(), z.copy()
        zp[idx] += eps; zm[idx] -= eps
        num[idx] = (loss(zp, beta) - loss(zm, beta)) / (2 * eps)
    assert np.max(np.abs(num - dz)) <= 1e-7 * max(1.0, np.max(np.abs(dz)))
    numb = np.zeros_like(beta)
    for idx in np.ndindex(*beta.shape):
        bp, bm = beta.copy(), beta.copy()
        bp[idx] += eps; bm[idx] -= eps
        numb[idx] = (loss(z, bp) - loss(z, bm)) / (2 * eps)
    assert np.max(np.abs(numb - dbeta)) <= 1e-7 * max(1.0, np.max(np.abs(dbeta)))
    # planted mistake: dropping the (1 - beta) factor of dz must be caught by the same check
    g = 1.0 / (1.0 + np.exp(-z))
    wrong = dz / (1.0 - beta[None, :, None, :])
    assert np.max(np.abs(num - wrong)) > 1e-3 * np.max(np.abs(dz))
    assert g.shape == z.shape


# ------------------------------------------------------------------ HGRN1 element-wise recurrence (Eq. 1)
def test_hgrn1_brute_force_closed_forms_and_hgrn2_with_unit_state():
    """h_t = sum_j (prod_{j<s<=t} f_s)(1 - f_j) i_j + (prod_{s<=t} f_s) h0 written out; constant gate
    gives the geometric closed form; f = 0 copies the input, f = 1 freezes h0; and a 1 x 1 state of
    the HGRN2 recurrence (q = output gate, v = input) is the same thing, computed by the C oracle."""
    rng = np.random.default_rng(21)
    B, N, d = 2, 17, 5
    f = rng.uniform(0.05, 0.98, (B, N, d)); i = rng.standard_normal((B, N, d)); o = rng.uniform(0, 1, (B, N, d))
    h0 = rng.standard_normal((B, d))
    y, hN = oracle.hgrn1_fwd(f, i, o, h0)
    ref = np.empty_like(y)
    for t in range(N):
        acc = np.prod(f[:, :t + 1], axis=1) * h0
        for j in range(t + 1):
            acc = acc + np.prod(f[:, j + 1:t + 1], axis=1) * (1.0 - f[:, j]) * i[:, j]
        ref[:, t] = acc * o[:, t]
    assert np.max(np.abs(y - ref)) <= 1e-13
    c = 0.7
    yc, hc = oracle.hgrn1_fwd(np.full((1, 9, 3), c), np.ones((1, 9, 3)), np.ones((1, 9, 3)))
    assert np.allclose(yc[0, :, 0], 1.0 - c ** np.arange(1, 10), rtol=1e-13)
    y0, _ = oracle.hgrn1_fwd(np.zeros_like(f), i, o, h0)
    assert np.array_equal(y0, i * o)
    y1, h1 = oracle.hgrn1_fwd(np.ones_like(f), i, o, h0)
    assert np.array_equal(y1, h0[:, None, :] * o) and np.array_equal(h1, h0)
    # HGRN2 with dk = dv = 1: one "head" per channel
    q2 = o.transpose(0, 2, 1)[..., None]; f2 = f.transpose(0, 2, 1)[..., None]; v2 = i.transpose(0, 2, 1)[..., None]
    o2, hT2 = oracle.fwd(q2, f2, v2, h0[..., None, None])
    assert np.max(np.abs(o2[..., 0].transpose(0, 2, 1) - y)) <= 1e-13
    assert np.max(np.abs(hT2[..., 0, 0] - hN)) <= 1e-13


def test_hgrn1_bwd_finite_differences_and_hgrn2_unit_state():
    rng = np.random.default_rng(22)
    B, N, d = 2, 11, 3
    f = rng.uniform(0.1, 0.95, (B, N, d)); i = rng.standard_normal((B, N, d)); o = rng.uniform(0, 1, (B, N, d))
    h0 = rng.standard_normal((B, d)); dy = rng.standard_normal((B, N, d)); dhN = rng.standard_normal((B, d))

    def loss(f_, i_, o_, h0_):
        y, hN = oracle.hgrn1_fwd(f_, i_, o_, h0_)
        return float((y * dy).sum() + (hN * dhN).sum())

    df, di, do, dh0 = oracle.hgrn1_bwd(f, i, o, dy, h0, dhN)
    eps = 1e-6
    for name, x, g in (("f", f, df), ("i", i, di), ("o", o, do), ("h0", h0, dh0)):
        num = np.zeros_like(x)
        for idx in np.ndindex(*x.shape):
            xp, xm = x.copy(), x.copy()
            xp[idx] += eps; xm[idx] -= eps
            args = {"f": f, "i": i, "o": o, "h0": h0}
            ap, am = dict(args), dict(args)
            ap[name], am[name] = xp, xm
            num[idx] = (loss(ap["f"], ap["i"], ap["o"], ap["h0"]) - loss(am["f"], am["i"], am["o"], am["h0"])) / (2 * eps)
        assert np.max(np.abs(num - g)) <= 1e-7 * max(1.0, np.max(np.abs(g))), name
    # the same gradients from the HGRN2 oracle with a 1 x 1 state per channel
    tr = lambda x: x.transpose(0, 2, 1)[..., None]
    dq2, df2, dv2, dh02 = oracle.bwd(tr(o), tr(f), tr(i), tr(dy), h0[..., None, None], dhN[..., None, None])
    back = lambda x: x[..., 0].transpose(0, 2, 1)
    assert np.max(np.abs(back(df2) - df)) <= 1e-12 and np.max(np.abs(back(dv2) - di)) <= 1e-12
    assert np.max(np.abs(back(dq2) - do)) <= 1e-12 and np.max(np.abs(dh02[..., 0, 0] - dh0)) <= 1e-12


# ------------------------------------------------------------------ HGRN1 with its activations (Eq. 1 + Eq. 2)
def test_hgrn1_activations_special_values_and_limits():
    """Pins of the activation step that do not re-type its formulas: known values of sigmoid and
    SiLU (sigmoid(0) = 1/2, sigmoid(ln 3) = 3/4, SiLU(0) = 0, SiLU(z) - SiLU(-z) = z), the range of
    the bounded gate (beta <= f <= 1, f = beta at zf -> -inf, f = 1 at zf -> +inf, beta = 0 leaves
    the plain sigmoid), and math.tanh as an independent evaluation of the sigmoid."""
    import math
    z = np.array([[[0.0, math.log(3.0), -math.log(3.0), 40.0, -40.0]]])
    beta = np.array([0.25, 0.0, 0.5, 0.9, 0.9])
    f, i, o = oracle.hgrn1_activations(z, z, z, beta)
    assert np.allclose(f[0, 0], [0.25 + 0.75 * 0.5, 0.75, 0.5 + 0.5 * 0.25, 1.0, 0.9], atol=1e-15)
    assert np.allclose(o[0, 0, :3], [0.5, 0.75, 0.25], atol=1e-15)
    assert i[0, 0, 0] == 0.0 and abs(i[0, 0, 1] - 0.75 * math.log(3.0)) <= 1e-15
    zz = np.linspace(-6, 6, 25)[None, None, :]
    _, ip, _ = oracle.hgrn1_activations(zz, zz, zz, np.zeros(25))
    _, im, _ = oracle.hgrn1_activations(zz, -zz, zz, np.zeros(25))
    assert np.max(np.abs(ip - im - zz)) <= 1e-14                      # SiLU(z) - SiLU(-z) = z
    f0, _, o0 = oracle.hgrn1_activations(zz, zz, zz, np.zeros(25))
    th = np.array([0.5 * (1.0 + math.tanh(0.5 * x)) for x in zz[0, 0]])
    assert np.max(np.abs(f0[0, 0] - th)) <= 1e-15 and np.max(np.abs(o0[0, 0] - th)) <= 1e-15
    rng = np.random.default_rng(31)
    b = rng.uniform(0, 0.95, 7)
    fz, _, _ = oracle.hgrn1_activations(rng.standard_normal((3, 9, 7)) * 4, np.zeros((3, 9, 7)), np.zeros((3, 9, 7)), b)
    assert np.all(fz >= b[None, None, :]) and np.all(fz <= 1.0)


def test_hgrn1_act_bwd_finite_differences():
    """Central differences of L = sum(y dy) + sum(h_N dhN) through the activations, for every input
    including the per-channel lower bound; and a planted mistake (dropping the factor 1 - beta from
    dzf, or the z (1 - s) term from the SiLU derivative) is far outside the bound."""
    rng = np.random.default_rng(32)
    B, N, d = 2, 9, 3
    zf, zi, zo = (rng.standard_normal((B, N, d)) * 1.5 for _ in range(3))
    beta = rng.uniform(0.05, 0.8, d)
    h0 = rng.standard_normal((B, d)); dy = rng.standard_normal((B, N, d)); dhN = rng.standard_normal((B, d))

    def loss(a):
        y, hN = oracle.hgrn1_fwd_act(a["zf"], a["zi"], a["zo"], a["beta"], a["h0"])
        return float((y * dy).sum() + (hN * dhN).sum())

    dzf, dzi, dzo, dbeta, dh0 = oracle.hgrn1_bwd_act(zf, zi, zo, beta, dy, h0, dhN)
    args = {"zf": zf, "zi": zi, "zo": zo, "beta": beta, "h0": h0}
    eps = 1e-6
    nums = {}
    for name, g in (("zf", dzf), ("zi", dzi), ("zo", dzo), ("beta", dbeta), ("h0", dh0)):
        x = args[name]
        num = np.zeros_like(x)
        for idx in np.ndindex(*x.shape):
            ap, am = dict(args), dict(args)
            xp, xm = x.copy(), x.copy()
            xp[idx] += eps; xm[idx] -= eps
            ap[name], am[name] = xp, xm
            num[idx] = (loss(ap) - loss(am)) / (2 * eps)
        nums[name] = num
        assert np.max(np.abs(num - g)) <= 2e-7 * max(1.0, np.max(np.abs(g))), name
    assert np.max(np.abs(nums["zf"] - dzf / (1.0 - beta)[None, None, :])) > 1e-3 * np.max(np.abs(dzf))
    s = 1.0 / (1.0 + np.exp(-zi))
    di_only = dzi / (s * (1.0 + zi * (1.0 - s))) * s
    assert np.max(np.abs(nums["zi"] - di_only)) > 1e-3 * np.max(np.abs(dzi))


# ------------------------------------------------------------------ gate-domain probe
def test_min_gate_product_constant_gate_and_brute_force():
    """A constant gate c gives c^32 (c^r for a ragged last piece of r tokens is larger); a single
    small gate shows up in exactly its own half chunk; token-by-token brute force on random gates."""
    assert abs(oracle.min_gate_product(np.full((1, 1, 128, 4), 0.5)) - 0.5 ** 32) <= 1e-24
    assert abs(oracle.min_gate_product(np.full((2, 1, 40, 4), 0.9)) - 0.9 ** 32) <= 1e-15      # pieces of 32 and 8 tokens
    assert oracle.min_gate_product(np.zeros((1, 1, 0, 4))) == 1.0
    f = np.ones((1, 2, 200, 3)); f[0, 1, 70, 2] = 1e-3
    assert abs(oracle.min_gate_product(f) - 1e-3) <= 1e-18
    rng = np.random.default_rng(41)
    f = rng.uniform(0.3, 1.0, (2, 2, 77, 3))
    best = 1.0
    for b in range(2):
        for h in range(2):
            for a in range(3):
                for s in range(0, 77, 32):
                    p = 1.0
                    for t in range(s, min(s + 32, 77)):
                        p *= f[b, h, t, a]
                    best = min(best, p)
    assert abs(oracle.min_gate_product(f) - best) <= 1e-15 * best


# ------------------------------------------------------------------ input side of the token mixer (Eq. 1)
def test_hgru2_proj_special_weights_and_written_out_sums():
    """Identity weights and zero biases leave the three activations of x itself (SciPy's logistic
    function and the HGRN1 oracle's activations as outside references); general weights against the
    affine maps written out as explicit sums; a weight that only reads channel 0 against a scalar
    closed form."""
    from scipy.special import expit
    rng = np.random.default_rng(51)
    B, N, d = 2, 5, 6
    x = rng.standard_normal((B, N, d))
    I, zero = np.eye(d), np.zeros(d)
    z, i, o = oracle.hgru2_proj(x, I, I, I, zero, zero, zero)
    assert np.max(np.abs(z - x)) == 0.0
    assert np.max(np.abs(i - x * expit(x))) <= 1e-15 and np.max(np.abs(o - expit(x))) <= 1e-15
    f1, i1, o1 = oracle.hgrn1_activations(x, x, x, np.zeros(d))
    assert np.max(np.abs(i1 - i)) <= 1e-15 and np.max(np.abs(o1 - o)) <= 1e-15 and np.max(np.abs(f1 - expit(z))) <= 1e-15
    U, V, W = (rng.standard_normal((d, d)) for _ in range(3))
    bu, bv, bw = (rng.standard_normal(d) for _ in range(3))
    z, i, o = oracle.hgru2_proj(x, U, V, W, bu, bv, bw)
    for b in range(B):
        for t in range(N):
            for c in range(d):
                au = bu[c] + sum(U[c, k] * x[b, t, k] for k in range(d))
                av = bv[c] + sum(V[c, k] * x[b, t, k] for k in range(d))
                aw = bw[c] + sum(W[c, k] * x[b, t, k] for k in range(d))
                assert abs(z[b, t, c] - au) <= 1e-13
                assert abs(i[b, t, c] - av / (1.0 + np.exp(-av))) <= 1e-13
                assert abs(o[b, t, c] - 1.0 / (1.0 + np.exp(-aw))) <= 1e-13
    # transposed weights would pass the identity case: a weight with a single non-zero entry tells them apart
    E = np.zeros((d, d)); E[2, 0] = 3.0                 # output channel 2 reads input channel 0
    z, _, _ = oracle.hgru2_proj(x, E, I, I, zero, zero, zero)
    assert np.max(np.abs(z[..., 2] - 3.0 * x[..., 0])) <= 1e-15 and np.max(np.abs(z[..., 0])) == 0.0


def _fd(fun, args, name, eps=1e-6):
    x = args[name]
    num = np.zeros_like(x)
    for idx in np.ndindex(*x.shape):
        ap, am = dict(args), dict(args)
        xp, xm = x.copy(), x.copy()
        xp[idx] += eps; xm[idx] -= eps
        ap[name], am[name] = xp, xm
        num[idx] = (fun(ap) - fun(am)) / (2 * eps)
    return num


def test_hgru2_proj_bwd_finite_differences():
    rng = np.random.default_rng(52)
    B, N, d = 2, 3, 4
    args = {"x": rng.standard_normal((B, N, d)), "U": rng.standard_normal((d, d)), "V": rng.standard_normal((d, d)),
            "W": rng.standard_normal((d, d)), "bu": rng.standard_normal(d), "bv": rng.standard_normal(d),
            "bw": rng.standard_normal(d)}
    dz, di, do = (rng.standard_normal((B, N, d)) for _ in range(3))

    def loss(a):
        z, i, o = oracle.hgru2_proj(a["x"], a["U"], a["V"], a["W"], a["bu"], a["bv"], a["bw"])
        return float((z * dz).sum() + (i * di).sum() + (o * do).sum())
    grads = oracle.hgru2_proj_bwd(args["x"], args["U"], args["V"], args["W"], args["bu"], args["bv"], args["bw"], dz, di, do)
    for name, g in zip(("x", "U", "V", "W", "bu", "bv", "bw"), grads):
        num = _fd(loss, args, name)
        assert num.shape == g.shape, name
        assert np.max(np.abs(num - g)) <= 3e-7 * max(1.0, np.max(np.abs(g))), name
    # planted mistakes that the differences must catch: the SiLU derivative without its second term, a transposed weight gradient
    num_v = _fd(loss, args, "V")
    av = args["x"] @ args["V"].T + args["bv"]
    s = 1.0 / (1.0 + np.exp(-av))
    wrong = (di * s).reshape(-1, d).T @ args["x"].reshape(-1, d)
    assert np.max(np.abs(num_v - wrong)) > 1e-2 * np.max(np.abs(num_v))
    assert np.max(np.abs(num_v - grads[2].T)) > 1e-2 * np.max(np.abs(num_v))


def test_hgru2_layer_reduces_to_the_gated_recurrence_and_finite_differences():
    """With one head, identity weights and zero biases the layer IS fwd_gated on (sigmoid(x), x,
    SiLU(x)); with two heads, every head sees its own slice of the channels; reverse mode against
    finite differences through Eq. 1 -> Eq. 2 -> Eq. 3 for every parameter."""
    from scipy.special import expit
    rng = np.random.default_rng(53)
    B, N, d = 1, 4, 4
    x = rng.standard_normal((B, N, d))
    I, zero = np.eye(d), np.zeros(d)
    beta = rng.uniform(0.0, 0.8, d)
    y, hT = oracle.hgru2_layer_fwd(x, I, I, I, zero, zero, zero, beta, 1)
    y1, hT1 = oracle.fwd_gated(expit(x)[:, None], x[:, None], beta[None, :], (x * expit(x))[:, None])
    assert np.max(np.abs(y - y1[:, 0])) <= 1e-14 and np.max(np.abs(hT - hT1)) <= 1e-14
    H = 2
    y2, hT2 = oracle.hgru2_layer_fwd(x, I, I, I, zero, zero, zero, beta, H)
    for h in range(H):
        sl = slice(h * d // H, (h + 1) * d // H)
        yh, hTh = oracle.fwd_gated(expit(x[..., sl])[:, None], x[..., sl][:, None], beta[None, sl], (x * expit(x))[..., sl][:, None])
        assert np.max(np.abs(y2[..., sl] - yh[:, 0])) <= 1e-14 and np.max(np.abs(hT2[:, h] - hTh[:, 0])) <= 1e-14
    args = {"x": x, "U": 0.5 * rng.standard_normal((d, d)), "V": rng.standard_normal((d, d)), "W": rng.standard_normal((d, d)),
            "bu": rng.standard_normal(d), "bv": rng.standard_normal(d), "bw": rng.standard_normal(d), "beta": beta,
            "h0": 0.1 * rng.standard_normal((B, H, d // H, d // H))}
    dy = rng.standard_normal((B, N, d))
    dhT = rng.standard_normal((B, H, d // H, d // H))

    def loss(a):
        yy, hh = oracle.hgru2_layer_fwd(a["x"], a["U"], a["V"], a["W"], a["bu"], a["bv"], a["bw"], a["beta"], H, a["h0"])
        return float((yy * dy).sum() + (hh * dhT).sum())
    grads = oracle.hgru2_layer_bwd(args["x"], args["U"], args["V"], args["W"], args["bu"], args["bv"], args["bw"], beta, H, dy,
                                   args["h0"], dhT)
    for name, g in zip(("x", "U", "V", "W", "bu", "bv", "bw", "beta", "h0"), grads):
        num = _fd(loss, args, name)
        assert np.max(np.abs(num - g)) <= 5e-7 * max(1.0, np.max(np.abs(g))), name
