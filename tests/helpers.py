"""Shared checks for the GPU parity tests (comparison logic only)."""
import numpy as np

TOL = 1e-4     # |y_gpu - y_oracle| <= TOL * sum|w||x| per output element (fp32 path)


def assert_within_bound(y_gpu: np.ndarray, y_ref: np.ndarray, bound: np.ndarray, what: str = ""):
    """Element-wise acceptance test; where bound == 0 the values must be identical."""
    assert y_gpu.shape == y_ref.shape, (what, y_gpu.shape, y_ref.shape)
    assert np.isfinite(y_gpu).all(), what
    err = np.abs(y_gpu.astype(np.float64) - y_ref.astype(np.float64))
    # the oracle rounds its fp64 sum once to fp32: allow that half-ulp on top of the bound
    slack = np.abs(y_ref.astype(np.float64)) * 2.0 ** -23
    bad = err > TOL * bound + slack
    if bad.any():
        i = np.unravel_index(np.argmax(err - TOL * bound), err.shape)
        raise AssertionError(f"{what}: {int(bad.sum())} of {bad.size} outputs outside the bound; worst at {i}: "
                             f"gpu={y_gpu[i]!r} ref={y_ref[i]!r} bound={bound[i]!r}")
    zero = bound == 0
    if zero.any():
        assert np.array_equal(y_gpu[zero], y_ref[zero]), f"{what}: outputs with no contributing weight differ"
    rel = float((err / np.maximum(bound, 1e-30)).max()) if err.size else 0.0
    return rel
