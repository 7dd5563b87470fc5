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


def l2_rel_err(x, ref):
    """||x - ref||_2 / ||ref||_2 over a tensor."""
    x = np.asarray(x, np.float64)
    ref = np.asarray(ref, np.float64)
    assert x.shape == ref.shape, (x.shape, ref.shape)
    den = np.linalg.norm(ref)
    return float(np.linalg.norm(x - ref) / (den if den > 0 else 1.0))


def assert_close_bf16(x, ref, what=""):
    """Bar for the bf16-operand LSTM path: 2e-2 relative per tensor, taken in
    the 2-norm (each bf16 operand carries a relative rounding error of up to
    2^-9, and the largest of millions of such elementwise errors is an
    extreme-value statistic, not a measure of the arithmetic), plus an
    elementwise sanity bound of 1e-1 on the error relative to
    max(|ref|, rms(ref))."""
    e2, em = l2_rel_err(x, ref), rel_err(x, ref)
    assert e2 <= 2e-2, f"{what}: relative 2-norm error {e2:.3e} > 2.0e-02"
    assert em <= 1e-1, f"{what}: elementwise relative error {em:.3e} > 1.0e-01"


def assert_close_update(x, ref, what=""):
    """Bar for the CHANGE of a weight tensor over a few optimiser steps of the fp32 path: 1e-3 relative in the
    2-norm (measured 1e-5 .. 2e-4), plus an elementwise sanity bound of 1e-1 relative to max(|ref|, rms(ref)).
    Adam's step m / (sqrt(v) + eps) does not depend on the size of the gradient: an element whose gradient is at
    the level of fp32 rounding noise still takes a step of full size, in a direction that noise decides, so the
    largest elementwise error of a big tensor (measured up to 3e-2 on one element of 16384) says nothing about
    the arithmetic."""
    e2, em = l2_rel_err(x, ref), rel_err(x, ref)
    assert e2 <= 1e-3, f"{what}: relative 2-norm error {e2:.3e} > 1.0e-03"
    assert em <= 1e-1, f"{what}: elementwise relative error {em:.3e} > 1.0e-01"
