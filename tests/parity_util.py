"""Helpers shared by the GPU parity tests.  Everything here runs on the CPU and calls only the oracle.

Comparison rule.  An fp32 sum of n products carries a rounding error of at most about n 2^-24 times the sum of
the MAGNITUDES of its terms, whatever the value of the sum itself is; so besides the two tensor-wide checks
(largest error against the largest oracle magnitude, and the 2-norm of the error against the 2-norm of the
oracle's tensor) every element is held to  |gpu - oracle| <= tol * (sum of |terms| of that element), which is
what "relative 1e-4" can mean for an element that is small because its terms cancel.  The magnitude sums come
from the oracle's own routines run on absolute values.

The kink of eq. (3).  f' jumps at z = 0.  The oracle adds a row in double, the kernel in fp32 in another order,
so a pre-activation whose exact value lies within the kernel's worst-case rounding error of zero,
|z_jb| < (n_j + 2) 2^-24 (|b_j| + sum_i |w_ji| |x_ib|) (plus what the same error in the layers before
contributes through x), may take either branch and both results are correct evaluations of the method.  Such a
pre-activation is "in the band" (decided from oracle values alone).  The other branch changes that neuron's
delta for that sample by at most (1 + alpha) |dLoss/da|, and the change flows back along the stored connections
like any delta.  kink_allowance() bounds, per element, how far a correct result may therefore lie from the
oracle's; close() takes that allowance off the element's error before any check.
"""
import numpy as np

U24 = 2.0 ** -24


def close(got, ref, tol, what="", mag=None, rows=None, allow=None, tally=None):
    """Tensor-wide checks (largest error against tol * the largest oracle magnitude, and 2-norm of the error
    against tol * the 2-norm of the oracle's tensor); with `mag` also the element-wise check
    |got - ref| <= tol * mag.  `allow` (per element, >= 0: see kink_delta) is subtracted from every element's
    error first.  `rows` (bool mask over axis 0) restricts everything.  Returns the largest error as a fraction of
    what was allowed.  `tally` (dict) counts the elements checked and those that needed their allowance, i.e. lay
    beyond tol * mag before it was taken off."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, what
    if rows is not None:
        got, ref = got[rows], ref[rows]
        mag = None if mag is None else np.asarray(mag)[rows]
        allow = None if allow is None else np.asarray(allow)[rows]
    assert np.all(np.isfinite(got)), what
    if ref.size == 0:
        return 0.0
    diff = np.abs(got - ref)
    if tally is not None:
        tally["checked"] = tally.get("checked", 0) + diff.size
        if allow is not None and mag is not None:
            tally["needed"] = tally.get("needed", 0) + int((diff > tol * np.asarray(mag, dtype=np.float64)).sum())
    if allow is not None:
        diff = np.maximum(diff - np.asarray(allow, dtype=np.float64), 0.0)
    scale = np.abs(ref).max()
    if scale == 0:
        assert diff.max() == 0, what
        return 0.0
    err = diff.max()
    if err > tol * scale:
        at = np.unravel_index(np.argmax(diff), diff.shape)
        raise AssertionError(f"{what}: max abs err {err:.3e} > {tol} * {scale:.3e} at {at}: got {got[at]!r} ref {ref[at]!r}"
                             + (f" sum|terms| {np.asarray(mag)[at]!r}" if mag is not None else "")
                             + (f" kink allowance {np.asarray(allow)[at]!r}" if allow is not None else ""))
    nrm = np.linalg.norm(diff) / np.linalg.norm(ref)
    assert nrm <= tol, f"{what}: normwise err {nrm:.3e} > {tol}"
    worst = err / scale / tol
    if mag is not None:
        mag = np.asarray(mag, dtype=np.float64)
        assert mag.shape == ref.shape, what
        bound = tol * np.maximum(mag, np.finfo(np.float32).tiny)
        bad = diff > bound
        if bad.any():
            at = np.unravel_index(np.argmax(diff / bound), diff.shape)
            raise AssertionError(f"{what}: {int(bad.sum())} elements beyond {tol} * sum|terms|; worst at {at}: "
                                 f"got {got[at]!r} ref {ref[at]!r} sum|terms| {mag[at]!r}")
        worst = max(worst, float((diff / bound).max()))
    return worst


def abs_forward(orc, O, x, with_bias=True):
    """[n_out, B] float32: |b_j| + sum_i |w_ji| x_ib for a non-negative x (the oracle's forward routine run on
    absolute values); without the bias term if with_bias is False."""
    x = np.ascontiguousarray(np.abs(x), dtype=np.float32)
    B = x.shape[1]
    m = np.zeros((O.n_out, B), dtype=np.float32)
    a = np.zeros((O.n_out, B), dtype=np.float32)
    bias = np.abs(O.bias) if with_bias else np.zeros(O.n_out, np.float32)
    val = np.abs(O.val) if O.nnz else np.zeros(1, np.float32)
    orc.lib().or_forward(O.n_out, O.rowptr, O.colidx, val, bias, x, B, B, 0, 0, np.float32(0), m, a, B)
    return m


def abs_backward(orc, O, x, dz, need_input_grad=True, val=None):
    """Magnitude sums of the backward pass: (sum_b |dz_jb||x_ib| per stored connection, sum_b |dz_jb| per neuron,
    sum_j |w_ji||dz_jb| per input element or None), by the oracle's backward routine on absolute values.  `val`:
    the weights to use when O.val no longer holds the ones the backward pass saw (after an update)."""
    x = np.ascontiguousarray(np.abs(x), dtype=np.float32)
    d = np.ascontiguousarray(np.abs(dz), dtype=np.float32)
    B = x.shape[1]
    scratch = np.zeros_like(d)
    g = np.zeros(max(O.nnz, 1), dtype=np.float32)
    gb = np.zeros(O.n_out, dtype=np.float32)
    gx = np.zeros((O.n_in, B), dtype=np.float32) if need_input_grad else None
    w = np.abs(O.val if val is None else val) if O.nnz else np.zeros(1, np.float32)
    rc = orc.lib().or_backward(O.n_in, O.n_out, O.rowptr, O.colidx, np.ascontiguousarray(w, dtype=np.float32),
                               x, B, d, d, B, B, 0, 0, np.float32(0), scratch, g, gb,
                               gx.ctypes.data if gx is not None else None, B)
    assert rc == 0
    return g[: O.nnz], gb, gx


def forward_bounds(orc, O, mag_in, err_in):
    """For layer O fed with an input whose elements are bounded by mag_in and which the kernel knows to within
    err_in: (mag_z, err_z) = (|b_j| + sum_i |w_ji| mag_in, (n_j + 2) 2^-24 mag_z + sum_i |w_ji| err_in): the sum of
    magnitudes behind every pre-activation, and the most by which an fp32 evaluation in any order, of inputs
    that are themselves off by err_in, can differ from the exact value.  Since |f(z)| <= |z| and f is
    1-Lipschitz (alpha <= 1), both also bound the activation."""
    mag_z = abs_forward(orc, O, mag_in)
    n_j = np.diff(O.rowptr).astype(np.float32)
    err_z = ((n_j + 2.0) * np.float32(U24))[:, None] * mag_z
    if err_in is not None:
        err_z = err_z + abs_forward(orc, O, err_in, with_bias=False)
    return mag_z, err_z


def band(O, err_z):
    """bool [n_out, B]: pre-activations of layer O (after O.forward) that lie within err_z of the kink.  All False
    for an identity (output) layer."""
    if not O.act_kind:
        return np.zeros(O.z.shape, dtype=bool)
    return np.abs(O.z) < err_z


def slope_magnitude(O):
    """|f'(z)| of layer O's last forward: 1 above the kink, alpha at or below it (1 for an identity layer)."""
    if not O.act_kind:
        return np.ones(O.z.shape, np.float32)
    return np.where(O.z > 0, np.float32(1.0), np.float32(abs(float(O.alpha)))).astype(np.float32)


def entry_rows(O):
    return np.repeat(np.arange(O.n_out), np.diff(O.rowptr))


def kink_delta(O, in_band, mag_ga, allow_ga):
    """Bound on how far dz of layer O may lie from the oracle's, per element: the incoming gradient dLoss/da is
    itself uncertain by allow_ga (flips in the layers after this one) and bounded by mag_ga; an element in
    the band may in addition have taken the other branch of eq. (3)."""
    slope = slope_magnitude(O)
    allow = slope * allow_ga
    if O.act_kind and in_band.any():
        a = np.float32(1.0 + abs(float(O.alpha)))
        allow = np.where(in_band, a * (mag_ga + allow_ga) + allow_ga, allow).astype(np.float32)
    return allow
