"""torch.autograd entry points over the C-ABI binding, for callers that train with PyTorch.

Argument marshalling only: every forward and backward below is one call into the library
(`binding.hgrn2_fwd` / `hgrn2_bwd` and their gated, variable-length and element-wise forms); no
arithmetic of the method happens here.  The backward passes are stateless, as the library's are:
they take the saved inputs and recompute what they need.

    o, hT = hgrn2_recurrence(q, f, v, h0)                      # Eq. 3, gates given
    o, hT = hgrn2_recurrence_gated(q, z, beta, v, h0)          # gate of Eq. 2 formed in the kernels
    o, hT = hgrn2_recurrence_varlen(q, f, v, cu_seqlens, h0)   # packed sequences (beta= optional)
    y, hN = hgrn1_recurrence(f, i, o, h0)                      # Eq. 1, f, i, o given
    y, hN = hgrn1_layer(zf, zi, zo, beta, h0)                  # Eq. 1 + Eq. 2 from pre-activations

Gradients flow to every floating-point tensor argument, including the initial state and the lower
bounds; the final state is differentiable too (its gradient enters the backward as grad_hT).
"""
import torch

from . import binding


def _c(t):
    return None if t is None else t.contiguous()


class _Hgrn2(torch.autograd.Function):
    @staticmethod
    def forward(ctx, q, f, v, h0, layout, chunk):
        o, hT = binding.hgrn2_fwd(q, f, v, h0, layout=layout, chunk=chunk)
        ctx.save_for_backward(q, f, v, h0)
        ctx.layout, ctx.chunk = layout, chunk
        ctx.set_materialize_grads(False)
        return o, hT

    @staticmethod
    def backward(ctx, grad_o, grad_hT):
        q, f, v, h0 = ctx.saved_tensors
        if grad_o is None:
            grad_o = torch.zeros_like(v)
        want_h0 = h0 is not None and ctx.needs_input_grad[3]
        gq, gf, gv, gh0 = binding.hgrn2_bwd(q, f, v, _c(grad_o), h0, _c(grad_hT), want_grad_h0=want_h0,
                                            layout=ctx.layout, chunk=ctx.chunk)
        return gq, gf.to(f.dtype), gv, gh0, None, None


class _Hgrn2Gated(torch.autograd.Function):
    @staticmethod
    def forward(ctx, q, z, beta, v, h0, layout, chunk):
        o, hT = binding.hgrn2_fwd_gated(q, z, beta, v, h0, layout=layout, chunk=chunk)
        ctx.save_for_backward(q, z, beta, v, h0)
        ctx.layout, ctx.chunk = layout, chunk
        ctx.set_materialize_grads(False)
        return o, hT

    @staticmethod
    def backward(ctx, grad_o, grad_hT):
        q, z, beta, v, h0 = ctx.saved_tensors
        if grad_o is None:
            grad_o = torch.zeros_like(v)
        want_h0 = h0 is not None and ctx.needs_input_grad[4]
        gq, gz, gb, gv, gh0 = binding.hgrn2_bwd_gated(q, z, beta, v, _c(grad_o), h0, _c(grad_hT),
                                                      want_grad_h0=want_h0, layout=ctx.layout, chunk=ctx.chunk)
        return gq, gz.to(z.dtype), gb, gv, gh0, None, None


class _Hgrn2Varlen(torch.autograd.Function):
    @staticmethod
    def forward(ctx, q, f, v, cu_seqlens, h0, beta, chunk):
        o, hT = binding.hgrn2_fwd_varlen(q, f, v, cu_seqlens, h0, beta=beta, chunk=chunk)
        ctx.save_for_backward(q, f, v, cu_seqlens, h0, beta)
        ctx.chunk = chunk
        ctx.set_materialize_grads(False)
        return o, hT

    @staticmethod
    def backward(ctx, grad_o, grad_hT):
        q, f, v, cu, h0, beta = ctx.saved_tensors
        if grad_o is None:
            grad_o = torch.zeros_like(v)
        want_h0 = h0 is not None and ctx.needs_input_grad[4]
        res = binding.hgrn2_bwd_varlen(q, f, v, _c(grad_o), cu, h0, _c(grad_hT), beta=beta, want_grad_h0=want_h0,
                                       chunk=ctx.chunk)
        gq, gf, gv, gh0 = res[:4]
        gb = res[4] if beta is not None else None
        return gq, gf.to(f.dtype), gv, None, gh0, gb, None


class _Hgrn1(torch.autograd.Function):
    @staticmethod
    def forward(ctx, f, i, o, h0):
        y, hN = binding.hgrn1_fwd(f, i, o, h0)
        ctx.save_for_backward(f, i, o, h0)
        ctx.set_materialize_grads(False)
        return y, hN

    @staticmethod
    def backward(ctx, grad_y, grad_hN):
        f, i, o, h0 = ctx.saved_tensors
        if grad_y is None:
            grad_y = torch.zeros_like(i)
        want_h0 = h0 is not None and ctx.needs_input_grad[3]
        gf, gi, go, gh0 = binding.hgrn1_bwd(f, i, o, _c(grad_y), h0, _c(grad_hN), want_grad_h0=want_h0)
        return gf.to(f.dtype), gi, go, gh0


class _Hgrn1Layer(torch.autograd.Function):
    @staticmethod
    def forward(ctx, zf, zi, zo, beta, h0):
        y, hN = binding.hgrn1_fwd_act(zf, zi, zo, beta, h0)
        ctx.save_for_backward(zf, zi, zo, beta, h0)
        ctx.set_materialize_grads(False)
        return y, hN

    @staticmethod
    def backward(ctx, grad_y, grad_hN):
        zf, zi, zo, beta, h0 = ctx.saved_tensors
        if grad_y is None:
            grad_y = torch.zeros_like(zi)
        want_h0 = h0 is not None and ctx.needs_input_grad[4]
        gf, gi, go, gb, gh0 = binding.hgrn1_bwd_act(zf, zi, zo, beta, _c(grad_y), h0, _c(grad_hN),
                                                    want_grad_h0=want_h0)
        return gf.to(zf.dtype), gi, go, gb, gh0


def hgrn2_recurrence(q, f, v, h0=None, layout=binding.HGRN2_LAYOUT_BHND, chunk=0):
    """o, hT of Eq. 3 with the gates given.  q, f: [B,H,N,dk], v: [B,H,N,dv] (or [B,N,H,d] with
    layout=HGRN2_LAYOUT_BNHD), contiguous; h0: fp32 [B,H,dk,dv] or None.  chunk=16 selects the
    small-gate mode of the library (reference rows every 16 tokens, four times the work)."""
    return _Hgrn2.apply(q, f, v, h0, layout, chunk)


def hgrn2_recurrence_gated(q, z, beta, v, h0=None, layout=binding.HGRN2_LAYOUT_BHND, chunk=0):
    """o, hT of Eq. 3 with f = beta + (1 - beta) sigmoid(z) (Eq. 2) formed in the kernels;
    beta: fp32 [H,dk]; chunk=16: the small-gate mode."""
    return _Hgrn2Gated.apply(q, z, beta, v, h0, layout, chunk)


def hgrn2_recurrence_varlen(q, f, v, cu_seqlens, h0=None, beta=None, chunk=0):
    """o, hT for sequences packed along the token axis: q, f [T,H,dk], v [T,H,dv], cu_seqlens int32
    [n_seq + 1] on the device, h0 / hT fp32 [n_seq,H,dk,dv]; with beta, f holds pre-activations."""
    return _Hgrn2Varlen.apply(q, f, v, cu_seqlens, h0, beta, chunk)


def hgrn1_recurrence(f, i, o, h0=None):
    """y, hN of Eq. 1 with f, i, o given.  [B,N,d] bf16 (f may be fp32); h0: fp32 [B,d] or None."""
    return _Hgrn1.apply(f, i, o, h0)


def hgrn1_layer(zf, zi, zo, beta, h0=None):
    """y, hN of Eq. 1 from the pre-activations, with the lower bound of Eq. 2; beta: fp32 [d]."""
    return _Hgrn1Layer.apply(zf, zi, zo, beta, h0)
