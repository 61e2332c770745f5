"""Helpers shared by the GPU parity tests: move seeded inputs to the device in their storage
dtype, run the oracle on the same (already rounded) values, and compare with the error measure
the tolerances are stated in:  max|x - y| / max|y|  per output tensor."""
import numpy as np
import torch

TOL = {"f32": 1e-4, "bf16": 2e-2}
TORCH_DT = {"f32": torch.float32, "bf16": torch.bfloat16}


def dev(x, dtype="f32"):
    if x is None:
        return None
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to("cuda").to(TORCH_DT[dtype]).contiguous()


def host(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


def rel_err(x, ref):
    ref = np.asarray(ref, dtype=np.float64)
    x = np.asarray(x, dtype=np.float64)
    assert x.shape == ref.shape, (x.shape, ref.shape)
    if ref.size == 0:
        return 0.0
    assert np.all(np.isfinite(x)), "non-finite values in the GPU result"
    den = max(float(np.max(np.abs(ref))), 1e-30)
    return float(np.max(np.abs(x - ref))) / den


def check(name, x, ref, tol):
    e = rel_err(x, ref)
    print("    %-8s max|x-y|/max|y| = %.3e (tol %.1e)" % (name, e, tol), flush=True)
    assert e <= tol, "%s: error %.3e exceeds %.1e" % (name, e, tol)
    return e
