"""Error metrics shared by the tests (no method arithmetic).

Three measures of a result `a` against the oracle's `b`:

relerr_max   max_i |a_i - b_i| / max_j |b_j|, taken per group (a group is a whole
             tensor, or one class's matrix for class gradients) and maximised over
             groups.  This is the "max relative error" the float tolerances (1e-5 for
             the fp32 path, 2e-2 for the bf16 path) are asserted on: the largest error
             relative to the scale of the tensor it sits in.
relerr_l2    ||a - b||_2 / ||b||_2 per group, maximised over groups: catches systematic
             errors (a dropped reduction tile, a wrong scale) that a max-normalised
             bound at bf16 precision could let through.  Bound: half the max tolerance.
relerr_elem  max_i |a_i - b_i| / max(|b_i|, rms(b)): strict element-wise measure, used
             where every output is an element-wise function of its inputs (gates, Adam
             state) and reported, not asserted, for the bf16 reductions: there an output
             is a sum of K terms each carrying ~3 bf16 roundings (unit roundoff 2^-8), so
             correct arithmetic has error of std ~3e-3 * rms and a maximum over 1e7
             elements of ~5.7 sigma ~ 2e-2 * rms: a 2e-2 bound relative to the rms would
             fail by chance.
"""
import numpy as np


def _groups(a, b, group_axis):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    assert a.shape == b.shape, (a.shape, b.shape)
    if group_axis is None or a.ndim == 0:
        return [(a.ravel(), b.ravel())]
    a = np.moveaxis(a, group_axis, 0).reshape(a.shape[group_axis], -1)
    b = np.moveaxis(b, group_axis, 0).reshape(b.shape[group_axis], -1)
    return list(zip(a, b))


def relerr_max(a, b, group_axis=None):
    worst = 0.0
    for ga, gb in _groups(a, b, group_axis):
        if gb.size == 0:
            continue
        scale = float(np.max(np.abs(gb)))
        err = float(np.max(np.abs(ga - gb)))
        worst = max(worst, err if scale == 0.0 else err / scale)
    return worst


def relerr_l2(a, b, group_axis=None):
    worst = 0.0
    for ga, gb in _groups(a, b, group_axis):
        if gb.size == 0:
            continue
        scale = float(np.sqrt(np.sum(gb * gb)))
        err = float(np.sqrt(np.sum((ga - gb) ** 2)))
        worst = max(worst, err if scale == 0.0 else err / scale)
    return worst


def relerr_elem(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    assert a.shape == b.shape, (a.shape, b.shape)
    if b.size == 0:
        return 0.0
    rms = float(np.sqrt(np.mean(b * b)))
    if rms == 0.0:
        return float(np.max(np.abs(a)))
    return float(np.max(np.abs(a - b) / np.maximum(np.abs(b), rms)))


relerr = relerr_elem

TOL = {"f32": 1e-5, "bf16": 2e-2, "adam": 1e-6}


def check_close(name, a, b, dtype, group_axis=None, log=None):
    """Asserts the float tolerance of the path `dtype` on (a, b); returns the measures."""
    e_max = relerr_max(a, b, group_axis)
    e_l2 = relerr_l2(a, b, group_axis)
    e_el = relerr_elem(a, b)
    if log is not None:
        log[name] = dict(max=e_max, l2=e_l2, elem=e_el)
    tol = TOL[dtype]
    assert e_max <= tol, f"{name}: max-normalised error {e_max:.3e} > {tol:g}"
    assert e_l2 <= tol / 2, f"{name}: relative L2 error {e_l2:.3e} > {tol / 2:g}"
    return e_max, e_l2, e_el
