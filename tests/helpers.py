"""Shared comparison helpers for the test-suite."""
import numpy as np


def tol_ok(got, ref, rtol):
    """Tolerance used for every floating-point comparison:
    |got - ref| <= rtol * (|ref| + rms(ref row)).  Pure element-wise relative error is undefined at
    zeros, and the rounding error of an accumulated element scales with the size of the operands that
    went into it, which the elements of one row (last axis) share; so the row's RMS sets the floor.
    Vectors use the RMS of the whole vector."""
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    if ref.size == 0:
        return True, 0.0
    if ref.ndim >= 2:
        rms = np.sqrt(np.mean(ref * ref, axis=-1, keepdims=True))
    else:
        rms = float(np.sqrt(np.mean(ref * ref)))
    err = np.abs(got - ref)
    bound = rtol * (np.abs(ref) + rms)
    worst = float((err / np.maximum(bound, 1e-300)).max())
    return bool((err <= bound).all()), worst


def tol_stats(got, ref, rtol, per_tensor=False):
    """(worst |err|/bound, number of elements above the bound) with the tol_ok bound; per_tensor=True takes one
    RMS over the whole tensor instead of one per row (the other reading of "rel" at zero outputs)."""
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    if ref.size == 0:
        return 0.0, 0
    if ref.ndim >= 2 and not per_tensor:
        rms = np.sqrt(np.mean(ref * ref, axis=-1, keepdims=True))
    else:
        rms = float(np.sqrt(np.mean(ref * ref)))
    ratio = np.abs(got - ref) / np.maximum(rtol * (np.abs(ref) + rms), 1e-300)
    return float(ratio.max()), int((ratio > 1.0).sum())


def assert_close(got, ref, rtol, what=""):
    ok, worst = tol_ok(got, ref, rtol)
    assert ok, f"{what}: worst |err|/bound = {worst:.3g} at rtol={rtol}"
