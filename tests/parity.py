"""Shared parity criterion for GPU-vs-oracle comparisons.

Floating-point bar (bf16 inputs, fp32 accumulation): for every output row (one head vector,
or one activation row) both
    max |g - o| <= tol * max |o|      and      ||g - o||_2 <= tol * ||o||_2
with tol = 2e-2.  The oracle consumes exactly the bf16-rounded inputs the GPU consumes
(widened exactly to fp64), so the budget covers fp32 accumulation order, the bf16 rounding of
the softmax weights fed to the matrix cores, and the bf16 rounding of the result.
"""
import numpy as np

TOL = 2e-2

# every comparison made through assert_rows_close in this process: (what, tol, worst max-norm error, worst l2 error);
# tests/conftest.py writes the worst case per label to gpurun_out/parity_observed.json when the session ends
OBSERVED = []


def row_errors(got, want):
    got = np.asarray(got, np.float64).reshape(-1, got.shape[-1])
    want = np.asarray(want, np.float64).reshape(-1, want.shape[-1])
    diff = got - want
    amax = np.abs(want).max(axis=1)
    l2 = np.linalg.norm(want, axis=1)
    tiny = 1e-30
    e_inf = np.abs(diff).max(axis=1) / np.maximum(amax, tiny)
    e_l2 = np.linalg.norm(diff, axis=1) / np.maximum(l2, tiny)
    return e_inf, e_l2


def assert_rows_close(got, want, tol=TOL, what=""):
    assert got.shape == want.shape, (got.shape, want.shape)
    assert np.isfinite(np.asarray(got, np.float64)).all(), f"{what}: non-finite values in the GPU result"
    e_inf, e_l2 = row_errors(got, want)
    OBSERVED.append((what, float(tol), float(e_inf.max()), float(e_l2.max())))
    worst = int(np.argmax(e_inf))
    assert e_inf.max() <= tol, f"{what}: row {worst} max-norm relative error {e_inf.max():.3e} > {tol}"
    assert e_l2.max() <= tol, f"{what}: l2 relative error {e_l2.max():.3e} > {tol}"
    return float(e_inf.max()), float(e_l2.max())
