"""Thin ctypes binding of libhgrn2.so: same entry-point names as include/hgrn2.h, argument
marshalling only.  PyTorch is used for device memory and the current stream, nothing else; every
step of the computation runs in the HIP kernels.  There is no fallback: if the library is missing
or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libhgrn2.so")

HGRN2_F32, HGRN2_BF16 = 0, 1
HGRN2_LAYOUT_BHND, HGRN2_LAYOUT_BNHD = 0, 1
STATUS = {0: "HGRN2_OK", 1: "HGRN2_ERR_NULL", 2: "HGRN2_ERR_SHAPE", 3: "HGRN2_ERR_UNSUPPORTED",
          4: "HGRN2_ERR_WORKSPACE", 5: "HGRN2_ERR_HIP"}
EXPORTS = ["hgrn2_fwd_workspace_bytes", "hgrn2_bwd_workspace_bytes", "hgrn2_fwd", "hgrn2_bwd",
           "hgrn2_step", "hgrn2_step_gated", "hgrn1_workspace_bytes", "hgrn1_fwd", "hgrn1_bwd", "hgrn1_fwd_act", "hgrn1_bwd_act", "hgrn1_bwd_saved", "hgrn1_bwd_act_saved", "hgrn2_bwd_gated_workspace_bytes", "hgrn2_fwd_gated", "hgrn2_bwd_gated", "hgrn2_cumax", "hgrn2_min_gate_product",
           "hgrn2_fwd_varlen_workspace_bytes", "hgrn2_bwd_varlen_workspace_bytes", "hgrn2_fwd_varlen", "hgrn2_bwd_varlen", "hgrn2_saved_states_varlen_bytes", "hgrn2_fwd_varlen_saving", "hgrn2_bwd_varlen_saved", "hgrn2_state_sweep", "hgrn2_fwd_readout", "hgrn2_bwd_chunk_grads",
           "hgrn2_min_gate_product_varlen_workspace_bytes", "hgrn2_min_gate_product_varlen", "hgrn2_status_string",
           "hgrn2_noalloc_workspace_limit", "hgrn2_noalloc_init", "hgrn2_bwd_noalloc",
           "hgrn2_saved_states_bytes", "hgrn2_bwd_saved_workspace_bytes", "hgrn2_fwd_saving", "hgrn2_bwd_saved",
           "hgrn2_probe_copy", "hgrn2_probe_mfma_out_floats", "hgrn2_probe_mfma",
           "hgru2_proj_bwd_workspace_bytes", "hgru2_proj_fwd", "hgru2_proj_bwd"]
SWEEP_STATE_FWD, SWEEP_STATE_BWD, SWEEP_STATE_GRAD = 0, 1, 2


class hgrn2_shape(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("H", ctypes.c_int32), ("N", ctypes.c_int32),
                ("dk", ctypes.c_int32), ("dv", ctypes.c_int32), ("chunk", ctypes.c_int32),
                ("io_dtype", ctypes.c_int32), ("gate_dtype", ctypes.c_int32), ("layout", ctypes.c_int32),
                ("gate_domain_flag", ctypes.c_void_p)]


class Hgrn2Error(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s failed: %s (%s)" % (where, STATUS.get(status, status), status_string(status)))


_lib = None


def lib() -> ctypes.CDLL:
    """Load the native library (built in-tree by paper_2404_07904_amd.build); fail loudly if absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("native library %s is missing: run `python -m paper_2404_07904_amd.build`"
                               % LIB_PATH)
        L = ctypes.CDLL(LIB_PATH)
        vp, sz, i32 = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int32
        sp = ctypes.POINTER(hgrn2_shape)
        L.hgrn2_fwd_workspace_bytes.restype = sz
        L.hgrn2_fwd_workspace_bytes.argtypes = [sp]
        L.hgrn2_bwd_workspace_bytes.restype = sz
        L.hgrn2_bwd_workspace_bytes.argtypes = [sp]
        L.hgrn2_fwd.restype = ctypes.c_int
        L.hgrn2_fwd.argtypes = [sp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.hgrn2_bwd.restype = ctypes.c_int
        L.hgrn2_bwd.argtypes = [sp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.hgrn2_bwd_gated_workspace_bytes.restype = sz
        L.hgrn2_bwd_gated_workspace_bytes.argtypes = [sp]
        L.hgrn2_fwd_gated.restype = ctypes.c_int
        L.hgrn2_fwd_gated.argtypes = [sp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.hgrn2_bwd_gated.restype = ctypes.c_int
        L.hgrn2_bwd_gated.argtypes = [sp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.hgrn2_fwd_varlen_workspace_bytes.restype = sz
        L.hgrn2_fwd_varlen_workspace_bytes.argtypes = [sp]
        L.hgrn2_bwd_varlen_workspace_bytes.restype = sz
        L.hgrn2_bwd_varlen_workspace_bytes.argtypes = [sp]
        L.hgrn2_fwd_varlen.restype = ctypes.c_int
        L.hgrn2_fwd_varlen.argtypes = [sp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.hgrn2_bwd_varlen.restype = ctypes.c_int
        L.hgrn2_bwd_varlen.argtypes = [sp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.hgrn2_saved_states_varlen_bytes.restype = sz
        L.hgrn2_saved_states_varlen_bytes.argtypes = [sp]
        L.hgrn2_fwd_varlen_saving.restype = ctypes.c_int
        L.hgrn2_fwd_varlen_saving.argtypes = [sp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp, sz, vp]
        L.hgrn2_bwd_varlen_saved.restype = ctypes.c_int
        L.hgrn2_bwd_varlen_saved.argtypes = [sp, vp, vp, vp, vp, vp, vp, vp, sz, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.hgrn2_min_gate_product.restype = ctypes.c_int
        L.hgrn2_min_gate_product.argtypes = [sp, vp, vp, vp, vp]
        L.hgrn2_min_gate_product_varlen_workspace_bytes.restype = sz
        L.hgrn2_min_gate_product_varlen_workspace_bytes.argtypes = [sp]
        L.hgrn2_min_gate_product_varlen.restype = ctypes.c_int
        L.hgrn2_min_gate_product_varlen.argtypes = [sp, vp, vp, vp, vp, vp, sz, vp]
        L.hgrn2_cumax.restype = ctypes.c_int
        L.hgrn2_cumax.argtypes = [i32, i32, vp, vp, vp]
        L.hgrn1_workspace_bytes.restype = sz
        L.hgrn1_workspace_bytes.argtypes = [i32, i32, i32]
        L.hgrn1_fwd.restype = ctypes.c_int
        L.hgrn1_fwd.argtypes = [i32, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.hgrn1_bwd.restype = ctypes.c_int
        L.hgrn1_bwd.argtypes = [i32, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.hgrn1_fwd_act.restype = ctypes.c_int
        L.hgrn1_fwd_act.argtypes = [i32, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.hgrn1_bwd_act.restype = ctypes.c_int
        L.hgrn1_bwd_act.argtypes = [i32, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.hgrn1_bwd_saved.restype = ctypes.c_int
        L.hgrn1_bwd_saved.argtypes = L.hgrn1_bwd.argtypes
        L.hgrn1_bwd_act_saved.restype = ctypes.c_int
        L.hgrn1_bwd_act_saved.argtypes = L.hgrn1_bwd_act.argtypes
        L.hgrn2_step.restype = ctypes.c_int
        L.hgrn2_step.argtypes = [i32, i32, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp]
        L.hgrn2_step_gated.restype = ctypes.c_int
        L.hgrn2_step_gated.argtypes = [i32, i32, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp]
        L.hgrn2_state_sweep.restype = ctypes.c_int
        L.hgrn2_state_sweep.argtypes = [sp, i32, vp, vp, vp, vp, vp, vp, sz, vp]
        L.hgrn2_fwd_readout.restype = ctypes.c_int
        L.hgrn2_fwd_readout.argtypes = [sp, vp, vp, vp, vp, vp, vp]
        L.hgrn2_bwd_chunk_grads.restype = ctypes.c_int
        L.hgrn2_bwd_chunk_grads.argtypes = [sp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp]
        L.hgru2_proj_bwd_workspace_bytes.restype = sz
        L.hgru2_proj_bwd_workspace_bytes.argtypes = [i32, i32]
        L.hgru2_proj_fwd.restype = ctypes.c_int
        L.hgru2_proj_fwd.argtypes = [i32, i32, vp, vp, vp, vp, vp, vp, vp, vp]
        L.hgru2_proj_bwd.restype = ctypes.c_int
        L.hgru2_proj_bwd.argtypes = [i32, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.hgrn2_probe_copy.restype = ctypes.c_int
        L.hgrn2_probe_copy.argtypes = [vp, vp, sz, vp]
        L.hgrn2_probe_mfma_out_floats.restype = sz
        L.hgrn2_probe_mfma_out_floats.argtypes = []
        L.hgrn2_probe_mfma.restype = ctypes.c_int
        L.hgrn2_probe_mfma.argtypes = [i32, vp, ctypes.POINTER(ctypes.c_double), vp]
        L.hgrn2_saved_states_bytes.restype = sz
        L.hgrn2_saved_states_bytes.argtypes = [sp]
        L.hgrn2_bwd_saved_workspace_bytes.restype = sz
        L.hgrn2_bwd_saved_workspace_bytes.argtypes = [sp, i32]
        L.hgrn2_fwd_saving.restype = ctypes.c_int
        L.hgrn2_fwd_saving.argtypes = [sp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp, sz, vp]
        L.hgrn2_bwd_saved.restype = ctypes.c_int
        L.hgrn2_bwd_saved.argtypes = [sp, vp, vp, vp, vp, vp, sz, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.hgrn2_noalloc_workspace_limit.restype = sz
        L.hgrn2_noalloc_workspace_limit.argtypes = []
        L.hgrn2_noalloc_init.restype = ctypes.c_int
        L.hgrn2_noalloc_init.argtypes = []
        L.hgrn2_bwd_noalloc.restype = ctypes.c_int
        L.hgrn2_bwd_noalloc.argtypes = [sp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp]
        L.hgrn2_status_string.restype = ctypes.c_char_p
        L.hgrn2_status_string.argtypes = [ctypes.c_int]
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().hgrn2_status_string(int(status)).decode()


def _dt(t: torch.Tensor) -> int:
    if t.dtype == torch.bfloat16:
        return HGRN2_BF16
    if t.dtype == torch.float32:
        return HGRN2_F32
    raise TypeError("unsupported dtype %s" % t.dtype)


def _ptr(t):
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "tensors must be contiguous device tensors"
    return ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def make_shape(q, v, f, chunk=0, layout=HGRN2_LAYOUT_BHND) -> hgrn2_shape:
    """Shape descriptor of contiguous tensors q, f [B,H,N,dk], v [B,H,N,dv] (or [B,N,H,d] with
    layout=HGRN2_LAYOUT_BNHD)."""
    if layout == HGRN2_LAYOUT_BNHD:
        B, N, H, dk = q.shape
    else:
        B, H, N, dk = q.shape
    return hgrn2_shape(B, H, N, dk, v.shape[-1], chunk, _dt(q), _dt(f), layout)


def _flagged(shape: hgrn2_shape, domain_flag) -> hgrn2_shape:
    """Point the shape at the caller's gate-domain flag (a one-element int32 device tensor the
    kernels set to 1 when the gates leave the domain of the chunkwise kernels), if one is given."""
    if domain_flag is not None:
        assert domain_flag.dtype == torch.int32 and domain_flag.is_cuda and domain_flag.numel() >= 1
        shape.gate_domain_flag = domain_flag.data_ptr()
    return shape


def hgrn2_fwd_workspace_bytes(shape: hgrn2_shape) -> int:
    return int(lib().hgrn2_fwd_workspace_bytes(ctypes.byref(shape)))


def hgrn2_bwd_workspace_bytes(shape: hgrn2_shape) -> int:
    return int(lib().hgrn2_bwd_workspace_bytes(ctypes.byref(shape)))


def _workspace(nbytes, device, workspace):
    if workspace is not None:
        return workspace
    return torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)


def hgrn2_fwd(q, f, v, h0=None, *, want_hT=True, chunk=0, o=None, hT=None, workspace=None,
              layout=HGRN2_LAYOUT_BHND, domain_flag=None):
    """o, hT = chunkwise forward of the recurrence.  q, f: [B,H,N,dk]; v: [B,H,N,dv]; h0 fp32."""
    shape = _flagged(make_shape(q, v, f, chunk, layout), domain_flag)
    assert v.dtype == q.dtype and f.shape == q.shape
    if o is None:
        o = torch.empty_like(v)
    if hT is None and want_hT:
        hT = torch.empty((shape.B, shape.H, shape.dk, shape.dv), dtype=torch.float32, device=q.device)
    nbytes = hgrn2_fwd_workspace_bytes(shape)
    ws = _workspace(nbytes, q.device, workspace)
    rc = lib().hgrn2_fwd(ctypes.byref(shape), _ptr(q), _ptr(f), _ptr(v), _ptr(h0), _ptr(o), _ptr(hT),
                         _ptr(ws), ws.numel(), _stream())
    if rc != 0:
        raise Hgrn2Error(rc, "hgrn2_fwd")
    return o, hT


def hgrn2_bwd(q, f, v, grad_o, h0=None, grad_hT=None, *, want_grad_h0=False, chunk=0, workspace=None,
              grad_q=None, grad_f=None, grad_v=None, grad_h0=None, layout=HGRN2_LAYOUT_BHND, domain_flag=None):
    """grad_q, grad_f, grad_v, grad_h0 of L = sum(o*grad_o) + sum(hT*grad_hT)."""
    shape = _flagged(make_shape(q, v, f, chunk, layout), domain_flag)
    grad_q = torch.empty_like(q) if grad_q is None else grad_q
    grad_f = torch.empty_like(q) if grad_f is None else grad_f
    grad_v = torch.empty_like(v) if grad_v is None else grad_v
    if grad_h0 is None and want_grad_h0:
        grad_h0 = torch.empty((shape.B, shape.H, shape.dk, shape.dv), dtype=torch.float32, device=q.device)
    nbytes = hgrn2_bwd_workspace_bytes(shape)
    ws = _workspace(nbytes, q.device, workspace)
    rc = lib().hgrn2_bwd(ctypes.byref(shape), _ptr(q), _ptr(f), _ptr(v), _ptr(h0), _ptr(grad_o),
                         _ptr(grad_hT), _ptr(grad_q), _ptr(grad_f), _ptr(grad_v), _ptr(grad_h0),
                         _ptr(ws), ws.numel(), _stream())
    if rc != 0:
        raise Hgrn2Error(rc, "hgrn2_bwd")
    return grad_q, grad_f, grad_v, grad_h0


def hgru2_proj_fwd(x, w3, b3, *, keep_av=True, z=None, v=None, q=None, av=None):
    """z, v, q (and av) of the three input projections of the HGRU2 token mixer (Eq. 1).  x: bf16
    [..., d] (any leading shape, contiguous); w3: bf16 [3d, d] (rows of U, V, W); b3: fp32 [3d]."""
    d = x.shape[-1]
    M = x.numel() // d if d else 0
    assert tuple(w3.shape) == (3 * d, d) and w3.dtype == torch.bfloat16 and x.dtype == torch.bfloat16
    assert b3.dtype == torch.float32 and b3.numel() == 3 * d
    z = torch.empty_like(x) if z is None else z
    v = torch.empty_like(x) if v is None else v
    q = torch.empty_like(x) if q is None else q
    if av is None and keep_av:
        av = torch.empty_like(x)
    rc = lib().hgru2_proj_fwd(M, d, _ptr(x), _ptr(w3), _ptr(b3), _ptr(z), _ptr(v), _ptr(q), _ptr(av), _stream())
    if rc != 0:
        raise Hgrn2Error(rc, "hgru2_proj_fwd")
    return z, v, q, av


def hgru2_proj_bwd(x, w3, q, av, grad_z, grad_v, grad_q, *, workspace=None, grad_x=None, grad_w3=None, grad_b3=None):
    """grad_x (bf16), grad_w3 (fp32 [3d, d]), grad_b3 (fp32 [3d]) of the three projections."""
    d = x.shape[-1]
    M = x.numel() // d if d else 0
    grad_x = torch.empty_like(x) if grad_x is None else grad_x
    grad_w3 = torch.empty((3 * d, d), dtype=torch.float32, device=x.device) if grad_w3 is None else grad_w3
    grad_b3 = torch.empty((3 * d,), dtype=torch.float32, device=x.device) if grad_b3 is None else grad_b3
    ws = _workspace(int(lib().hgru2_proj_bwd_workspace_bytes(M, d)), x.device, workspace)
    rc = lib().hgru2_proj_bwd(M, d, _ptr(x), _ptr(w3), _ptr(q), _ptr(av), _ptr(grad_z), _ptr(grad_v), _ptr(grad_q),
                              _ptr(grad_x), _ptr(grad_w3), _ptr(grad_b3), _ptr(ws), ws.numel(), _stream())
    if rc != 0:
        raise Hgrn2Error(rc, "hgru2_proj_bwd")
    return grad_x, grad_w3, grad_b3


def hgrn2_probe_copy(dst, src):
    """Plain device copy of src into dst (uint8 tensors of equal size, a multiple of 16 bytes)."""
    assert dst.numel() == src.numel() and dst.dtype == torch.uint8 and src.dtype == torch.uint8
    rc = lib().hgrn2_probe_copy(_ptr(dst), _ptr(src), src.numel(), _stream())
    if rc != 0:
        raise Hgrn2Error(rc, "hgrn2_probe_copy")


def hgrn2_probe_mfma(iters, out=None):
    """A launch of nothing but bf16 matrix instructions; returns (flops of the launch, out)."""
    if out is None:
        out = torch.empty(int(lib().hgrn2_probe_mfma_out_floats()), dtype=torch.float32, device="cuda")
    flops = ctypes.c_double(0.0)
    rc = lib().hgrn2_probe_mfma(int(iters), _ptr(out), ctypes.byref(flops), _stream())
    if rc != 0:
        raise Hgrn2Error(rc, "hgrn2_probe_mfma")
    return flops.value, out


def hgrn2_saved_states_bytes(shape: hgrn2_shape) -> int:
    return int(lib().hgrn2_saved_states_bytes(ctypes.byref(shape)))


def hgrn2_bwd_saved_workspace_bytes(shape: hgrn2_shape, gated: bool) -> int:
    return int(lib().hgrn2_bwd_saved_workspace_bytes(ctypes.byref(shape), 1 if gated else 0))


def hgrn2_fwd_saving(q, f, v, h0=None, *, beta=None, want_hT=True, o=None, hT=None, saved_states=None, workspace=None,
                     layout=HGRN2_LAYOUT_BHND, domain_flag=None, chunk=0):
    """hgrn2_fwd (or hgrn2_fwd_gated when beta is given) that also keeps the per-chunk states for
    hgrn2_bwd_saved.  Returns o, hT, saved_states (a uint8 device buffer)."""
    shape = _flagged(make_shape(q, v, f, chunk, layout), domain_flag)
    if o is None:
        o = torch.empty_like(v)
    if hT is None and want_hT:
        hT = torch.empty((shape.B, shape.H, shape.dk, shape.dv), dtype=torch.float32, device=q.device)
    if saved_states is None:
        saved_states = torch.empty(max(hgrn2_saved_states_bytes(shape), 256), dtype=torch.uint8, device=q.device)
    ws = _workspace(hgrn2_fwd_workspace_bytes(shape), q.device, workspace)
    rc = lib().hgrn2_fwd_saving(ctypes.byref(shape), _ptr(q), _ptr(f), _ptr(beta), _ptr(v), _ptr(h0), _ptr(o), _ptr(hT),
                                _ptr(saved_states), saved_states.numel(), _ptr(ws), ws.numel(), _stream())
    if rc != 0:
        raise Hgrn2Error(rc, "hgrn2_fwd_saving")
    return o, hT, saved_states


def hgrn2_bwd_saved(q, f, v, saved_states, grad_o, grad_hT=None, *, beta=None, want_grad_h0=False, workspace=None,
                    grad_q=None, grad_f=None, grad_v=None, grad_h0=None, layout=HGRN2_LAYOUT_BHND, domain_flag=None,
                    chunk=0):
    """hgrn2_bwd (hgrn2_bwd_gated when beta is given) from the states hgrn2_fwd_saving kept.  Returns
    grad_q, grad_f, grad_v, grad_h0 and, with beta, grad_beta as a fifth value."""
    shape = _flagged(make_shape(q, v, f, chunk, layout), domain_flag)
    grad_q = torch.empty_like(q) if grad_q is None else grad_q
    grad_f = torch.empty_like(q) if grad_f is None else grad_f
    grad_v = torch.empty_like(v) if grad_v is None else grad_v
    if grad_h0 is None and want_grad_h0:
        grad_h0 = torch.empty((shape.B, shape.H, shape.dk, shape.dv), dtype=torch.float32, device=q.device)
    gb = torch.empty_like(beta) if beta is not None else None
    ws = _workspace(hgrn2_bwd_saved_workspace_bytes(shape, beta is not None), q.device, workspace)
    rc = lib().hgrn2_bwd_saved(ctypes.byref(shape), _ptr(q), _ptr(f), _ptr(beta), _ptr(v), _ptr(saved_states),
                               saved_states.numel(), _ptr(grad_o), _ptr(grad_hT), _ptr(grad_q), _ptr(grad_f), _ptr(gb),
                               _ptr(grad_v), _ptr(grad_h0), _ptr(ws), ws.numel(), _stream())
    if rc != 0:
        raise Hgrn2Error(rc, "hgrn2_bwd_saved")
    return (grad_q, grad_f, grad_v, grad_h0) if beta is None else (grad_q, grad_f, grad_v, grad_h0, gb)


def hgrn2_noalloc_workspace_limit() -> int:
    return int(lib().hgrn2_noalloc_workspace_limit())


def hgrn2_bwd_noalloc(q, f, v, grad_o, h0, grad_hT, grad_q, grad_f, grad_v, grad_h0=None, *, chunk=0,
                      layout=HGRN2_LAYOUT_BHND, domain_flag=None):
    """hgrn2_bwd on the library's built-in scratch array: every output is the caller's, nothing is
    allocated here or in the library."""
    shape = _flagged(make_shape(q, v, f, chunk, layout), domain_flag)
    rc = lib().hgrn2_bwd_noalloc(ctypes.byref(shape), _ptr(q), _ptr(f), _ptr(v), _ptr(h0), _ptr(grad_o),
                                 _ptr(grad_hT), _ptr(grad_q), _ptr(grad_f), _ptr(grad_v), _ptr(grad_h0), _stream())
    if rc != 0:
        raise Hgrn2Error(rc, "hgrn2_bwd_noalloc")
    return grad_q, grad_f, grad_v, grad_h0


def hgrn2_bwd_gated_workspace_bytes(shape: hgrn2_shape) -> int:
    return int(lib().hgrn2_bwd_gated_workspace_bytes(ctypes.byref(shape)))


def hgrn2_fwd_gated(q, z, beta, v, h0=None, *, want_hT=True, o=None, hT=None, workspace=None,
                    layout=HGRN2_LAYOUT_BHND, chunk=0, domain_flag=None):
    """hgrn2_fwd with the gate f = beta + (1 - beta) sigmoid(z) formed inside the kernels.
    z: [B,H,N,dk]; beta: fp32 [H,dk]."""
    shape = _flagged(make_shape(q, v, z, chunk, layout), domain_flag)
    assert beta.dtype == torch.float32 and tuple(beta.shape) == (shape.H, shape.dk)
    if o is None:
        o = torch.empty_like(v)
    if hT is None and want_hT:
        hT = torch.empty((shape.B, shape.H, shape.dk, shape.dv), dtype=torch.float32, device=q.device)
    ws = _workspace(hgrn2_fwd_workspace_bytes(shape), q.device, workspace)
    rc = lib().hgrn2_fwd_gated(ctypes.byref(shape), _ptr(q), _ptr(z), _ptr(beta), _ptr(v), _ptr(h0), _ptr(o),
                               _ptr(hT), _ptr(ws), ws.numel(), _stream())
    if rc != 0:
        raise Hgrn2Error(rc, "hgrn2_fwd_gated")
    return o, hT


def hgrn2_bwd_gated(q, z, beta, v, grad_o, h0=None, grad_hT=None, *, want_grad_h0=False, workspace=None,
                    grad_q=None, grad_z=None, grad_beta=None, grad_v=None, grad_h0=None,
                    layout=HGRN2_LAYOUT_BHND, chunk=0, domain_flag=None):
    """grad_q, grad_z, grad_beta, grad_v, grad_h0 of L = sum(o*grad_o) + sum(hT*grad_hT)."""
    shape = _flagged(make_shape(q, v, z, chunk, layout), domain_flag)
    grad_q = torch.empty_like(q) if grad_q is None else grad_q
    grad_z = torch.empty_like(q) if grad_z is None else grad_z
    grad_v = torch.empty_like(v) if grad_v is None else grad_v
    grad_beta = torch.empty_like(beta) if grad_beta is None else grad_beta
    if grad_h0 is None and want_grad_h0:
        grad_h0 = torch.empty((shape.B, shape.H, shape.dk, shape.dv), dtype=torch.float32, device=q.device)
    ws = _workspace(hgrn2_bwd_gated_workspace_bytes(shape), q.device, workspace)
    rc = lib().hgrn2_bwd_gated(ctypes.byref(shape), _ptr(q), _ptr(z), _ptr(beta), _ptr(v), _ptr(h0), _ptr(grad_o),
                               _ptr(grad_hT), _ptr(grad_q), _ptr(grad_z), _ptr(grad_beta), _ptr(grad_v),
                               _ptr(grad_h0), _ptr(ws), ws.numel(), _stream())
    if rc != 0:
        raise Hgrn2Error(rc, "hgrn2_bwd_gated")
    return grad_q, grad_z, grad_beta, grad_v, grad_h0


def make_shape_varlen(q, v, f, n_seq, chunk=0) -> hgrn2_shape:
    """Shape descriptor of packed tensors q, f [T,H,dk], v [T,H,dv] holding n_seq sequences."""
    T, H, dk = q.shape
    return hgrn2_shape(n_seq, H, T, dk, v.shape[-1], chunk, _dt(q), _dt(f), HGRN2_LAYOUT_BNHD)


def hgrn2_fwd_varlen_workspace_bytes(shape: hgrn2_shape) -> int:
    return int(lib().hgrn2_fwd_varlen_workspace_bytes(ctypes.byref(shape)))


def hgrn2_bwd_varlen_workspace_bytes(shape: hgrn2_shape) -> int:
    return int(lib().hgrn2_bwd_varlen_workspace_bytes(ctypes.byref(shape)))


def hgrn2_saved_states_varlen_bytes(shape: hgrn2_shape) -> int:
    return int(lib().hgrn2_saved_states_varlen_bytes(ctypes.byref(shape)))


def hgrn2_fwd_varlen(q, f, v, cu_seqlens, h0=None, *, beta=None, want_hT=True, o=None, hT=None, workspace=None,
                     chunk=0, domain_flag=None, saved_states=None):
    """o, hT for sequences packed along the token axis.  q, f: [T,H,dk]; v: [T,H,dv]; cu_seqlens:
    int32 device tensor [n_seq + 1]; h0, hT: fp32 [n_seq,H,dk,dv].  With beta [H,dk] fp32, f holds the
    gates' pre-activations (Eq. 2).  With saved_states (a uint8 device tensor of
    hgrn2_saved_states_varlen_bytes bytes) the call is hgrn2_fwd_varlen_saving."""
    assert cu_seqlens.dtype == torch.int32 and cu_seqlens.is_contiguous()
    shape = _flagged(make_shape_varlen(q, v, f, cu_seqlens.numel() - 1, chunk), domain_flag)
    if o is None:
        o = torch.empty_like(v)
    if hT is None and want_hT:
        hT = torch.empty((shape.B, shape.H, shape.dk, shape.dv), dtype=torch.float32, device=q.device)
    ws = _workspace(hgrn2_fwd_varlen_workspace_bytes(shape), q.device, workspace)
    if saved_states is not None:
        rc = lib().hgrn2_fwd_varlen_saving(ctypes.byref(shape), _ptr(cu_seqlens), _ptr(q), _ptr(f), _ptr(beta), _ptr(v),
                                           _ptr(h0), _ptr(o), _ptr(hT), _ptr(saved_states), saved_states.numel(),
                                           _ptr(ws), ws.numel(), _stream())
        if rc != 0:
            raise Hgrn2Error(rc, "hgrn2_fwd_varlen_saving")
        return o, hT
    rc = lib().hgrn2_fwd_varlen(ctypes.byref(shape), _ptr(cu_seqlens), _ptr(q), _ptr(f), _ptr(beta), _ptr(v), _ptr(h0),
                                _ptr(o), _ptr(hT), _ptr(ws), ws.numel(), _stream())
    if rc != 0:
        raise Hgrn2Error(rc, "hgrn2_fwd_varlen")
    return o, hT


def hgrn2_bwd_varlen(q, f, v, grad_o, cu_seqlens, h0=None, grad_hT=None, *, beta=None, want_grad_h0=False,
                     workspace=None, grad_q=None, grad_f=None, grad_v=None, chunk=0, domain_flag=None, saved_states=None):
    """grad_q, grad_f, grad_v, grad_h0 for sequences packed along the token axis; with beta also
    grad_beta (returned as a fifth value), and grad_f is then the gradient of the pre-activations.
    With saved_states (filled by hgrn2_fwd_varlen of the same arguments) the call is hgrn2_bwd_varlen_saved."""
    assert cu_seqlens.dtype == torch.int32 and cu_seqlens.is_contiguous()
    shape = _flagged(make_shape_varlen(q, v, f, cu_seqlens.numel() - 1, chunk), domain_flag)
    gq = torch.empty_like(q) if grad_q is None else grad_q
    gf = torch.empty_like(q) if grad_f is None else grad_f
    gv = torch.empty_like(v) if grad_v is None else grad_v
    gh0 = (torch.empty((shape.B, shape.H, shape.dk, shape.dv), dtype=torch.float32, device=q.device)
           if want_grad_h0 else None)
    gb = torch.empty((shape.H, shape.dk), dtype=torch.float32, device=q.device) if beta is not None else None
    ws = _workspace(hgrn2_bwd_varlen_workspace_bytes(shape), q.device, workspace)
    if saved_states is not None:
        rc = lib().hgrn2_bwd_varlen_saved(ctypes.byref(shape), _ptr(cu_seqlens), _ptr(q), _ptr(f), _ptr(beta), _ptr(v),
                                          _ptr(h0), _ptr(saved_states), saved_states.numel(), _ptr(grad_o), _ptr(grad_hT),
                                          _ptr(gq), _ptr(gf), _ptr(gb), _ptr(gv), _ptr(gh0), _ptr(ws), ws.numel(), _stream())
        name = "hgrn2_bwd_varlen_saved"
    else:
        rc = lib().hgrn2_bwd_varlen(ctypes.byref(shape), _ptr(cu_seqlens), _ptr(q), _ptr(f), _ptr(beta), _ptr(v), _ptr(h0),
                                    _ptr(grad_o), _ptr(grad_hT), _ptr(gq), _ptr(gf), _ptr(gb), _ptr(gv), _ptr(gh0), _ptr(ws),
                                    ws.numel(), _stream())
        name = "hgrn2_bwd_varlen"
    if rc != 0:
        raise Hgrn2Error(rc, name)
    return (gq, gf, gv, gh0) if beta is None else (gq, gf, gv, gh0, gb)


def hgrn2_min_gate_product(f, beta=None, layout=HGRN2_LAYOUT_BHND, chunk=0):
    """Smallest product of one channel's gates over a half chunk (32 tokens; 8 with chunk=16, the
    small-gate mode) in f [B,H,N,dk] (or [B,N,H,dk]); a one-element fp32 device tensor.  The
    chunkwise passes are exact while it exceeds 2**-100.  With beta [H,dk], f holds
    pre-activations (Eq. 2)."""
    shape = make_shape(f, f, f, chunk, layout)
    out = torch.empty((1,), dtype=torch.float32, device=f.device)
    rc = lib().hgrn2_min_gate_product(ctypes.byref(shape), _ptr(f), _ptr(beta), _ptr(out), _stream())
    if rc != 0:
        raise Hgrn2Error(rc, "hgrn2_min_gate_product")
    return out


def hgrn2_min_gate_product_varlen(f, cu_seqlens, beta=None, chunk=0):
    """hgrn2_min_gate_product for sequences packed along the token axis: f [T,H,dk], cu_seqlens int32
    [n_seq + 1] on the device; the windows start anew with every sequence."""
    assert cu_seqlens.dtype == torch.int32 and cu_seqlens.is_contiguous()
    shape = make_shape_varlen(f, f, f, cu_seqlens.numel() - 1, chunk)
    out = torch.empty((1,), dtype=torch.float32, device=f.device)
    ws = _workspace(int(lib().hgrn2_min_gate_product_varlen_workspace_bytes(ctypes.byref(shape))), f.device, None)
    rc = lib().hgrn2_min_gate_product_varlen(ctypes.byref(shape), _ptr(cu_seqlens), _ptr(f), _ptr(beta), _ptr(out),
                                             _ptr(ws), ws.numel(), _stream())
    if rc != 0:
        raise Hgrn2Error(rc, "hgrn2_min_gate_product_varlen")
    return out


def hgrn2_cumax(gamma):
    """beta [L,d] = cumulative softmax of gamma [L,d] over the layer axis, minus its first row."""
    assert gamma.dtype == torch.float32 and gamma.dim() == 2
    beta = torch.empty_like(gamma)
    rc = lib().hgrn2_cumax(gamma.shape[0], gamma.shape[1], _ptr(gamma), _ptr(beta), _stream())
    if rc != 0:
        raise Hgrn2Error(rc, "hgrn2_cumax")
    return beta


def hgrn1_workspace_bytes(B, N, d) -> int:
    return int(lib().hgrn1_workspace_bytes(B, N, d))


def hgrn1_fwd(f, i, o, h0=None, *, want_hN=True, y=None, hN=None, workspace=None):
    """y, hN of the element-wise recurrence h_t = f_t h_{t-1} + (1 - f_t) i_t, y_t = h_t o_t.
    f, i, o: [B,N,d] (i, o bf16; f bf16 or fp32); h0: fp32 [B,d] or None."""
    B, N, d = i.shape
    y = torch.empty_like(i) if y is None else y
    if hN is None and want_hN:
        hN = torch.empty((B, d), dtype=torch.float32, device=i.device)
    ws = _workspace(hgrn1_workspace_bytes(B, N, d), i.device, workspace)
    rc = lib().hgrn1_fwd(B, N, d, _dt(i), _dt(f), _ptr(f), _ptr(i), _ptr(o), _ptr(h0), _ptr(y), _ptr(hN), _ptr(ws),
                         ws.numel(), _stream())
    if rc != 0:
        raise Hgrn2Error(rc, "hgrn1_fwd")
    return y, hN


def hgrn1_bwd(f, i, o, grad_y, h0=None, grad_hN=None, *, want_grad_h0=False, workspace=None, saved=False):
    """grad_f, grad_i, grad_o, grad_h0 of L = sum(y*grad_y) + sum(hN*grad_hN).  saved=True calls
    hgrn1_bwd_saved: `workspace` is then the one hgrn1_fwd of the same inputs was given."""
    B, N, d = i.shape
    gf, gi, go = torch.empty_like(i), torch.empty_like(i), torch.empty_like(i)
    gh0 = torch.empty((B, d), dtype=torch.float32, device=i.device) if want_grad_h0 else None
    assert workspace is not None or not saved
    ws = _workspace(hgrn1_workspace_bytes(B, N, d), i.device, workspace)
    fn = lib().hgrn1_bwd_saved if saved else lib().hgrn1_bwd
    rc = fn(B, N, d, _dt(i), _dt(f), _ptr(f), _ptr(i), _ptr(o), _ptr(h0), _ptr(grad_y), _ptr(grad_hN),
            _ptr(gf), _ptr(gi), _ptr(go), _ptr(gh0), _ptr(ws), ws.numel(), _stream())
    if rc != 0:
        raise Hgrn2Error(rc, "hgrn1_bwd_saved" if saved else "hgrn1_bwd")
    return gf, gi, go, gh0


def hgrn1_fwd_act(zf, zi, zo, beta, h0=None, *, want_hN=True, y=None, hN=None, workspace=None):
    """y, hN of the element-wise recurrence from the pre-activations of Eq. 1 and the lower bounds
    beta [d] of Eq. 2.  zf, zi, zo: [B,N,d]."""
    B, N, d = zf.shape
    assert zi.shape == zf.shape and zo.shape == zf.shape and beta.dtype == torch.float32 and beta.numel() == d
    if y is None:
        y = torch.empty_like(zi)
    if hN is None and want_hN:
        hN = torch.empty((B, d), dtype=torch.float32, device=zf.device)
    ws = _workspace(hgrn1_workspace_bytes(B, N, d), zf.device, workspace)
    rc = lib().hgrn1_fwd_act(B, N, d, _dt(zi), _dt(zf), _ptr(zf), _ptr(zi), _ptr(zo), _ptr(beta), _ptr(h0), _ptr(y),
                             _ptr(hN), _ptr(ws), ws.numel(), _stream())
    if rc != 0:
        raise Hgrn2Error(rc, "hgrn1_fwd_act")
    return y, hN


def hgrn1_bwd_act(zf, zi, zo, beta, grad_y, h0=None, grad_hN=None, *, want_grad_h0=False, workspace=None, saved=False):
    """grad_zf, grad_zi, grad_zo, grad_beta, grad_h0 of L = sum(y*grad_y) + sum(hN*grad_hN).  saved=True
    calls hgrn1_bwd_act_saved: `workspace` is then the one hgrn1_fwd_act of the same inputs was given."""
    B, N, d = zf.shape
    assert workspace is not None or not saved
    gf, gi, go = torch.empty_like(zi), torch.empty_like(zi), torch.empty_like(zi)
    gb = torch.empty((d,), dtype=torch.float32, device=zf.device)
    gh0 = torch.empty((B, d), dtype=torch.float32, device=zf.device) if want_grad_h0 else None
    ws = _workspace(hgrn1_workspace_bytes(B, N, d), zf.device, workspace)
    fn = lib().hgrn1_bwd_act_saved if saved else lib().hgrn1_bwd_act
    rc = fn(B, N, d, _dt(zi), _dt(zf), _ptr(zf), _ptr(zi), _ptr(zo), _ptr(beta), _ptr(h0),
            _ptr(grad_y), _ptr(grad_hN), _ptr(gf), _ptr(gi), _ptr(go), _ptr(gb), _ptr(gh0), _ptr(ws),
            ws.numel(), _stream())
    if rc != 0:
        raise Hgrn2Error(rc, "hgrn1_bwd_act_saved" if saved else "hgrn1_bwd_act")
    return gf, gi, go, gb, gh0


def hgrn2_step(q_t, f_t, v_t, state, o_t=None):
    """One decode step; `state` [B,H,dk,dv] fp32 is updated in place.  Returns o_t [B,H,dv]."""
    B, H, dk = q_t.shape
    dv = v_t.shape[-1]
    assert state.dtype == torch.float32 and tuple(state.shape) == (B, H, dk, dv)
    if o_t is None:
        o_t = torch.empty_like(v_t)
    rc = lib().hgrn2_step(B, H, dk, dv, _dt(q_t), _dt(f_t), _ptr(q_t), _ptr(f_t), _ptr(v_t), _ptr(state),
                          _ptr(o_t), _stream())
    if rc != 0:
        raise Hgrn2Error(rc, "hgrn2_step")
    return o_t


def hgrn2_step_gated(q_t, z_t, beta, v_t, state, o_t=None):
    """One decode step from the gate's pre-activations z_t [B,H,dk] and the layer's lower bounds
    beta [H,dk] fp32 (Eq. 2); `state` is updated in place.  Returns o_t [B,H,dv]."""
    B, H, dk = q_t.shape
    dv = v_t.shape[-1]
    assert state.dtype == torch.float32 and tuple(state.shape) == (B, H, dk, dv)
    assert beta.dtype == torch.float32 and tuple(beta.shape) == (H, dk)
    if o_t is None:
        o_t = torch.empty_like(v_t)
    rc = lib().hgrn2_step_gated(B, H, dk, dv, _dt(q_t), _dt(z_t), _ptr(q_t), _ptr(z_t), _ptr(beta), _ptr(v_t),
                                _ptr(state), _ptr(o_t), _stream())
    if rc != 0:
        raise Hgrn2Error(rc, "hgrn2_step_gated")
    return o_t


def hgrn2_state_sweep(shape, mode, q, f, b_src, chunk_states, init_state=None, final_state=None):
    """Stage entry point: chunk-to-chunk recurrence; fills `chunk_states` (uint8 device buffer)."""
    rc = lib().hgrn2_state_sweep(ctypes.byref(shape), mode, _ptr(q), _ptr(f), _ptr(b_src), _ptr(init_state),
                                 _ptr(final_state), _ptr(chunk_states), chunk_states.numel(), _stream())
    if rc != 0:
        raise Hgrn2Error(rc, "hgrn2_state_sweep")


def hgrn2_fwd_readout(shape, q, f, v, chunk_states, o):
    rc = lib().hgrn2_fwd_readout(ctypes.byref(shape), _ptr(q), _ptr(f), _ptr(v), _ptr(chunk_states), _ptr(o),
                                 _stream())
    if rc != 0:
        raise Hgrn2Error(rc, "hgrn2_fwd_readout")


def hgrn2_bwd_chunk_grads(shape, q, f, v, grad_o, chunk_states, chunk_state_grads, grad_q, grad_f, grad_v):
    rc = lib().hgrn2_bwd_chunk_grads(ctypes.byref(shape), _ptr(q), _ptr(f), _ptr(v), _ptr(grad_o),
                                     _ptr(chunk_states), _ptr(chunk_state_grads), _ptr(grad_q), _ptr(grad_f),
                                     _ptr(grad_v), _stream())
    if rc != 0:
        raise Hgrn2Error(rc, "hgrn2_bwd_chunk_grads")
