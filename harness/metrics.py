"""Error metrics shared by the tests, the smoke check and the benchmark (no method arithmetic).

Measures of a result `a` against the oracle's `b`:

relerr_max   max_i |a_i - b_i| / max_j |b_j|, taken per group (a group is a whole
             tensor, or one class's matrix for class gradients) and maximised over
             groups.  This is the "max relative error" the float tolerances (1e-5 for
             the fp32 path, 2e-2 for the bf16 path) are asserted on: the largest error
             relative to the scale of the tensor it sits in.
relerr_l2    ||a - b||_2 / ||b||_2 per group, maximised over groups: catches systematic
             errors (a dropped reduction tile, a wrong scale) that a max-normalised
             bound at bf16 precision could let through.  Bound: half the max tolerance.
relerr_elem  max_i |a_i - b_i| / max(|b_i|, rms(b)), per group, rms over the entries of b that
             are not exactly zero: the strict element-wise measure.  Asserted at 1e-5 on every output of the fp32 path, at 1e-5 / 1e-6 where
             an output is an element-wise function of its inputs (gates, Adam state).
relerr_axis  max_i |a_i - b_i| / max(|b_i|, rms of b along `axis` through i): the element-wise
             measure for bf16 reductions.  An output there is a sum of K terms each carrying up
             to 4 bf16 roundings, so its error has standard deviation ~3.1e-3 times the root of
             the sum of its squared terms; along an axis on which the outputs share that root it
             equals the rms of the outputs themselves, which makes it the right floor:
               Y, dX [T,d]     a token's row (the rounded operand, h or du|dv, belongs to the row);
               dW2 [E,d,f]     the d outputs of a hidden unit (errors of dYp and h are relative
                               to the values themselves);
               dW1 [E,2,f,d]   the f hidden units of one input column, gate and up halves apart:
                               du = dh*v*s'(u) inherits from dh (a d-term sum) an error relative
                               to the row's typical |dh|, not to |dh[r,h]| itself, so a hidden
                               unit whose dh is nearly zero on a class's few rows has a large
                               error relative to its OWN row of dW1 but not relative to the
                               column's rms over all hidden units.
             `axis` may be a tuple: the floor is then the largest of the rms values (used where
             only a few positions along the proper axis are sampled and its rms is noisy).
             Bound: elem_bound_bf16(n).
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
    nz = b != 0.0         # exact zeros (dropped tokens, classes without rows) do not dilute the floor
    if not nz.any():
        return float(np.max(np.abs(a)))
    rms = float(np.sqrt(np.mean(b[nz] * b[nz])))
    return float(np.max(np.abs(a - b) / np.maximum(np.abs(b), rms)))


def relerr_elem_groups(a, b, group_axis=None):
    return max([relerr_elem(ga, gb) for ga, gb in _groups(a, b, group_axis)] + [0.0])


def relerr_axis(a, b, axis):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    assert a.shape == b.shape, (a.shape, b.shape)
    if b.size == 0:
        return 0.0
    den = np.abs(b)
    for ax in (axis if isinstance(axis, tuple) else (axis,)):
        den = np.maximum(den, np.sqrt(np.mean(b * b, axis=ax, keepdims=True)))
    err = np.abs(a - b)
    ok = den > 0
    worst = float(np.max(err[ok] / den[ok])) if ok.any() else 0.0
    if (err[~ok] > 0).any():              # b is zero along the whole axis: a must be as well
        return float("inf")
    return worst


def elem_bound_bf16(n, K=1):
    """Largest element-wise error (relative to max(|b_i|, axis rms)) that correct bf16
    arithmetic produces among n outputs of a K-term reduction, with a 2x margin (the terms are
    products of rounded factors with data of unequal scale -- gates between 0 and 1, rows of
    different norms -- so the error is heavier-tailed than the normal law used here):
      * every term carries up to 4 roundings to bf16 (relative rms error of one rounding
        2^-7 / sqrt(12) / 1.44 = 1.57e-3, so 3.1e-3 for four) -> the error of an output is
        close to normal with sigma = 3.1e-3 x (root of the sum of squared terms);
      * the largest of n such errors is sigma x sqrt(2 ln 2n);
      * a bf16 output is rounded once more (2^-8 relative);
      * the fp32 accumulation adds at most sqrt(K) x 2^-24 on the same scale."""
    sigma = 4 ** 0.5 * 2.0 ** -7 / 12 ** 0.5 / 1.44
    return 2.0 * (sigma * (2.0 * np.log(2.0 * max(n, 1))) ** 0.5 + 2.0 ** -8 + K ** 0.5 * 2.0 ** -24)

TOL = {"f32": 1e-5, "bf16": 2e-2, "adam": 1e-6}


def check_close(name, a, b, dtype, group_axis=None, log=None, iid_axis=None, K=1):
    """Asserts the float tolerances of the path `dtype` on (a, b); returns the measures.

    fp32 path: max-normalised, L2 and the strict element-wise measure per group, all at 1e-5.
    bf16 path: max-normalised at 2e-2, L2 at 1e-2 and, where `iid_axis` names the axis along
    which the outputs share their term scale, the element-wise measure relerr_axis at
    elem_bound_bf16(number of elements, K)."""
    e_max = relerr_max(a, b, group_axis)
    e_l2 = relerr_l2(a, b, group_axis)
    e_el = relerr_elem_groups(a, b, group_axis)
    entry = dict(max=e_max, l2=e_l2, elem=e_el)
    tol = TOL[dtype]
    assert e_max <= tol, f"{name}: max-normalised error {e_max:.3e} > {tol:g}"
    assert e_l2 <= tol / 2, f"{name}: relative L2 error {e_l2:.3e} > {tol / 2:g}"
    if dtype == "f32":
        assert e_el <= tol, f"{name}: element-wise error {e_el:.3e} > {tol:g}"
    elif iid_axis is not None:
        e_ax = relerr_axis(a, b, iid_axis)
        bound = elem_bound_bf16(np.asarray(b).size, K)
        entry.update(axis=e_ax, axis_bound=bound)
        assert e_ax <= bound, f"{name}: element-wise error {e_ax:.3e} (floor: rms along axis {iid_axis}) > {bound:.3e}"
    if log is not None:
        log[name] = entry
    return e_max, e_l2, e_el
