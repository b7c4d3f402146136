"""The two parity measures of a layer output against the CPU oracle.

1. ``max_rel``: max |y - y_ref| / max |y_ref| over the tensor -- the gated "max relative error"
   (an element-wise ratio is undefined where a LayerNorm output crosses zero).
2. ``violations``: fraction of elements with |y - y_ref| > tol * |y_ref| + tol * rms(y_ref), a mixed
   absolute / relative bound per element, so that a small element cannot hide behind the tensor's
   largest one.  Expected to be exactly 0.
"""
import numpy as np


def parity(got, want, tol):
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    assert got.shape == want.shape, (got.shape, want.shape)
    if want.size == 0:
        return {"max_rel": 0.0, "violations": 0.0}
    delta = np.abs(got - want)
    rms = float(np.sqrt(np.mean(want * want)))
    bad = delta > tol * np.abs(want) + tol * rms
    bad |= ~np.isfinite(got)
    return {"max_rel": float(np.max(delta) / max(np.max(np.abs(want)), 1e-30)),
            "violations": float(np.mean(bad))}


def assert_parity(got, want, tol, label=None, max_violations=0.0):
    """max_violations: only for stress inputs far outside the configurations' recipe, where a
    per-feature gain of almost 2 scales a few elements' error past a bound tied to the tensor's rms."""
    p = parity(got, want, tol)
    assert p["max_rel"] <= tol and p["violations"] <= max_violations, (p, tol, label)
    return p
