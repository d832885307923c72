"""Shared comparison helpers for the test-suite."""
import numpy as np


def tol_ok(got, ref, rtol):
    """Per-tensor tolerance used for every floating-point comparison:
    |got - ref| <= rtol * (|ref| + rms(ref)).  Pure element-wise relative error
    is undefined at zeros, so the tensor's RMS sets the floor."""
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    if ref.size == 0:
        return True, 0.0
    rms = float(np.sqrt(np.mean(ref * ref)))
    err = np.abs(got - ref)
    bound = rtol * (np.abs(ref) + rms)
    worst = float((err / np.maximum(bound, 1e-300)).max())
    return bool((err <= bound).all()), worst


def assert_close(got, ref, rtol, what=""):
    ok, worst = tol_ok(got, ref, rtol)
    assert ok, f"{what}: worst |err|/bound = {worst:.3g} at rtol={rtol}"
