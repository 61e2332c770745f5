"""Helpers shared by the GPU parity tests: move seeded inputs to the device in their storage
dtype, run the oracle on the same (already rounded) values, and compare with the error measure
the tolerances are stated in:  max|x - y| / max|y|  per output tensor (plus two logged figures, one
of them bounded as well: see check)."""
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


# Next to the max-norm measure the tolerances are stated in, two more figures are logged for every
# tensor: the relative L2 error, and the worst element-wise relative error over the entries that
# matter, |y| >= 1e-2 max|y| (a localised mistake -- one row, one channel -- shows there long
# before it moves the global maximum).  The latter is bounded too: an entry of size s max|y|,
# s >= 1e-2, can be off by at most tol max|y| under the max-norm bound, i.e. by tol / s of itself;
# the parity bar here is a quarter of that worst case, 25 tol (0.5 for bf16 storage, 2.5e-3 for fp32).
SIGNIFICANT = 1e-2
ELEMENTWISE_FACTOR = 25.0


def error_figures(x, ref):
    ref = np.asarray(ref, dtype=np.float64)
    x = np.asarray(x, dtype=np.float64)
    if ref.size == 0:
        return 0.0, 0.0, 0.0
    top = max(float(np.max(np.abs(ref))), 1e-30)
    diff = np.abs(x - ref)
    l2 = float(np.sqrt(np.sum(diff * diff)) / max(float(np.sqrt(np.sum(ref * ref))), 1e-30))
    big = np.abs(ref) >= SIGNIFICANT * top
    worst = float(np.max(diff[big] / np.abs(ref[big]))) if np.any(big) else 0.0
    return float(np.max(diff)) / top, l2, worst


def check(name, x, ref, tol):
    e = rel_err(x, ref)
    _, l2, worst = error_figures(x, ref)
    print("    %-8s max|x-y|/max|y| = %.3e (tol %.1e)   rel L2 = %.3e   worst element-wise (|y| >= 1e-2 max) = %.3e"
          % (name, e, tol, l2, worst), flush=True)
    assert e <= tol, "%s: error %.3e exceeds %.1e" % (name, e, tol)
    assert worst <= ELEMENTWISE_FACTOR * tol, "%s: element-wise relative error %.3e exceeds %.1e" % (name, worst, ELEMENTWISE_FACTOR * tol)
    return e
