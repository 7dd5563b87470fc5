"""Shared comparison helper for the tests (no method arithmetic)."""
import numpy as np


def rel_err(x, ref):
    """max |x - ref| / max(|ref|, rms(ref)) over a tensor: relative error that
    stays defined where values cross zero."""
    x = np.asarray(x, np.float64)
    ref = np.asarray(ref, np.float64)
    assert x.shape == ref.shape, (x.shape, ref.shape)
    if ref.size == 0:
        return 0.0
    scale = np.maximum(np.abs(ref), np.sqrt(np.mean(ref * ref)))
    scale = np.where(scale == 0.0, 1.0, scale)
    return float(np.max(np.abs(x - ref) / scale))


def assert_close(x, ref, tol, what=""):
    e = rel_err(x, ref)
    assert e <= tol, f"{what}: relative error {e:.3e} > {tol:.1e}"
