"""Shared helpers of the GPU parity tests (comparison against the float64 oracle)."""
import numpy as np

# element-wise bound of the fp32 path against the float64 oracle: |a - b| <= ATOL + RTOL*|b|
RTOL, ATOL = 1e-4, 1e-5


def assert_close(got, want, what, rtol=RTOL, atol=ATOL):
    got = np.asarray(got, np.float64)
    want = np.asarray(want, np.float64)
    assert got.shape == want.shape, f"{what}: shape {got.shape} vs {want.shape}"
    err = np.abs(got - want)
    tol = atol + rtol * np.abs(want)
    bad = err > tol
    if bad.any():
        i = np.unravel_index(np.argmax(err / tol), err.shape)
        rel = np.linalg.norm(got - want) / max(np.linalg.norm(want), 1e-30)
        raise AssertionError(f"{what}: {int(bad.sum())}/{bad.size} outside tolerance; worst at {i}: "
                             f"got {got[i]:.8g} want {want[i]:.8g}; ||diff||/||want|| = {rel:.3e}")


def compare_trees(got, want, what, names=None, **kw):
    """got/want: {key: {name: array}}; compares every tensor present in `want`."""
    for key, tensors in want.items():
        for name, w in tensors.items():
            if names is not None and not names(name):
                continue
            assert name in got[key], f"{what}: block {key} lacks {name}"
            assert_close(got[key][name], w, f"{what} block {key} {name}", **kw)
