"""Shared test helpers: tolerance check and host<->device shuttling."""
import numpy as np

TOL = 1e-5   # |gpu - exact| <= TOL * sum|x*w| per output element


def assert_within_bound(gpu: np.ndarray, acc: np.ndarray, mag: np.ndarray, what: str = ""):
    """The acceptance bound: per element, error at most 1e-5 of the sum of |products|."""
    gpu = np.asarray(gpu, dtype=np.float64)
    assert gpu.shape == acc.shape, f"{what}: shape {gpu.shape} vs {acc.shape}"
    assert np.all(np.isfinite(gpu)), f"{what}: non-finite values (unwritten or corrupted output)"
    err = np.abs(gpu - acc)
    bad = err > TOL * mag
    if bad.any():
        i = np.unravel_index(np.argmax(err - TOL * mag), err.shape)
        raise AssertionError(
            f"{what}: {bad.sum()} of {bad.size} elements outside the bound; worst at {i}: "
            f"gpu={gpu[i]!r} exact={acc[i]!r} mag={mag[i]!r} err/mag={err[i] / max(mag[i], 1e-300):.3e}")
    return float((err / np.maximum(mag, 1e-300)).max())
