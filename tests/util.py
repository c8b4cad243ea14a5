"""Error metrics shared by the tests (no method arithmetic)."""
import numpy as np


def relerr(a, b):
    """max_i |a_i - b_i| / max(|b_i|, rms(b)): element-wise relative error whose
    denominator is floored at the reference tensor's RMS.  An entry far below the
    RMS is the result of cancellation between RMS-sized terms, so its absolute error
    scales with the RMS, not with the entry."""
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    assert a.shape == b.shape, (a.shape, b.shape)
    if b.size == 0:
        return 0.0
    rms = float(np.sqrt(np.mean(b * b)))
    if rms == 0.0:
        return float(np.max(np.abs(a)))  # reference is exactly zero: absolute error
    den = np.maximum(np.abs(b), rms)
    return float(np.max(np.abs(a - b) / den))


TOL = {"f32": 1e-5, "bf16": 2e-2, "adam": 1e-6}
