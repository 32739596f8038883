"""Error measure used by every parity test.

Per group, an output passes iff for all i, j
    |Y - Yref| <= tol * max(|Yref|, rms(Yref))
i.e. a relative error whose floor is the group's own scale, so exact zeros (ReLU)
and cancelling sums do not make the ratio meaningless.  tol: 1e-5 for fp32,
2e-2 for bf16 inputs with fp32 accumulation, 6e-2 for fp8 E4M3.
"""
import numpy as np

TOL = {"f32": 1e-5, "bf16": 2e-2, "fp8": 6e-2}


def rel_err(Y, Yref, rms=None):
    Y = np.asarray(Y, dtype=np.float64)
    Yref = np.asarray(Yref, dtype=np.float64)
    if Yref.size == 0:
        return 0.0
    if rms is None:
        rms = float(np.sqrt(np.mean(Yref * Yref)))
    floor = np.maximum(np.abs(Yref), rms if rms > 0 else 1.0)
    return float(np.max(np.abs(Y - Yref) / floor))


def assert_close(Y, Yref, tol, what="", rms=None):
    assert np.asarray(Y).shape == np.asarray(Yref).shape, (what, np.asarray(Y).shape, np.asarray(Yref).shape)
    assert np.all(np.isfinite(np.asarray(Y, dtype=np.float64))), what + ": non-finite output"
    e = rel_err(Y, Yref, rms)
    assert e <= tol, "%s: max relative error %.3e exceeds %.1e" % (what, e, tol)
    return e
