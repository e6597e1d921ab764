"""Error measures shared by the GPU parity tests.

max-norm relative error (the workload's tolerance applies to it):
    max|got - want| / max|want|, per sample, worst sample;
element-wise check with an absolute floor, so that a large relative error on one element cannot hide
behind the largest element of the field:
    |got - want| <= tol * (|want| + rms(want))   for every element;
and, reported only, the worst element-wise relative error with the floor 1e-3 * max|want|."""
import numpy as np

TOL_F32 = 1e-4
TOL_BF16 = 2e-2


def relerr(got, want, scale=None):
    """worst per-sample max-norm relative error; scale: max|want| of the whole field when `want` is a sample of it"""
    got, want = np.asarray(got, np.float64), np.asarray(want, np.float64)
    g, w = got.reshape(got.shape[0], -1), want.reshape(want.shape[0], -1)
    den = np.abs(w).max(axis=1) if scale is None else scale
    return float((np.abs(g - w).max(axis=1) / den).max())


def elementwise(got, want, rms=None, vmax=None):
    """(worst |d| / (|want| + rms), worst |d| / max(|want|, 1e-3 max|want|)) over all elements; rms / vmax of the
    whole field may be passed when `want` is a sample of it"""
    got, want = np.asarray(got, np.float64).ravel(), np.asarray(want, np.float64).ravel()
    d = np.abs(got - want)
    rms = float(np.sqrt((want * want).mean())) if rms is None else rms
    vmax = float(np.abs(want).max()) if vmax is None else vmax
    return float((d / (np.abs(want) + rms)).max()), float((d / np.maximum(np.abs(want), 1e-3 * vmax)).max())


def check(got, want, tol, what="", scale=None, rms=None):
    """Asserts both measures against `tol`; returns them (max-norm, element-wise with rms floor, element-wise
    with the 1e-3 max floor) for the test's report."""
    got, want = np.asarray(got, np.float64), np.asarray(want, np.float64)
    if got.ndim == 1:
        got, want = got[None], want[None]
    e_max = relerr(got, want, scale)
    e_el, e_floor = 0.0, 0.0
    for g, w in zip(got, want):
        a, b = elementwise(g, w, rms, scale)
        e_el, e_floor = max(e_el, a), max(e_floor, b)
    print("%s: max-norm rel %.3e, element-wise (rms floor) %.3e, element-wise (1e-3 max floor) %.3e, tol %.0e"
          % (what, e_max, e_el, e_floor, tol), flush=True)
    assert np.isfinite(e_max) and e_max < tol, (what, "max-norm", e_max)
    assert np.isfinite(e_el) and e_el < tol, (what, "element-wise", e_el)
    return e_max, e_el, e_floor
