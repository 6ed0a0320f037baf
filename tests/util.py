"""Helpers shared by the GPU parity tests (no arithmetic of the method).

A comparison with the oracle is three bounds at once, all scaled by the tolerance `tol` of the
configuration's precision (1e-4 fp32, 2e-2 bf16 storage with fp32 accumulation):

  tensor    ||got - want||_2 <= tol * ||want||_2                       (the bar the workload states)
  row       ||got_r - want_r||_2 <= C_ROW * tol * max(||want_r||_2, rms row norm)   for every row r of a matrix
  element   |got_ij - want_ij| <= C_ELEM * tol * (s_ij + |want_ij|)                 for every element,
            s_ij = max(rms(want), rms(row i) * rms(column j) / rms(want)) for a matrix, rms(want) for a vector

The tensor norm alone lets a single wrong row or tile through (one bad row of 4096 moves it by
1/64); the row and element bounds do not: a wrong row has an error of the order of its own norm, a
wrong element an error of the order of the tensor's rms, both an order of magnitude above the bounds.
The element scale s_ij is the size an element of the matrix has where it sits: an element of a product
X^T dY sums terms whose size goes with the norm of row i of X^T and of column j of dY, and its rounding
error goes with the size of those terms, not with the value they happen to sum to (the value gradients
of an attention block are ten times the key gradients next to them in the same matrix); in the quiet
parts of a matrix the scale stays the global rms.
The constants leave room for what rounding really does: storage rounding is relative to the element
(|want_ij| term), accumulated rounding through a stack of layers is spread evenly (rms term), and the
largest of millions of such errors sits five to six standard deviations out -- a result whose tensor
error is just at `tol` has element errors up to about 6 x tol x rms, so C_ELEM = 8 is the smallest
constant that cannot fail a result the tensor bound accepts, and rows of such a result err by up to
about 1.3 x tol of their norm (C_ROW = 2).
"""
import numpy as np

from oracle import layer as L
from paper_2204_12013_amd import synth

TOL = {synth.DTYPE_FP32: 1e-4, synth.DTYPE_BF16: 2e-2}
C_ROW = 2.0
C_ELEM = 8.0

# worst observed fraction of each bound, per label prefix: printed at the end of a GPU test session
WORST = {}


def rel_l2(got, want):
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    denom = np.linalg.norm(want.ravel())
    return float(np.linalg.norm((got - want).ravel()) / (denom if denom > 0 else 1.0))


def closeness(got, want, tol, elem_tol=None, floor=0.0):
    """(tensor, row, element) errors, each as a fraction of its bound (<= 1 passes).  elem_tol: a tolerance
    of its own for the element bound (default: tol).  floor: the size of the terms the elements sum, where the
    expected values themselves say nothing about it (a slice that is exactly zero by cancellation: the query
    gradient of a one-token sequence is P (dP - delta) with dP = delta); the scales of the row and element
    bounds are then at least this."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    assert got.shape == want.shape, (got.shape, want.shape)
    err = got - want
    if not np.all(np.isfinite(err)):
        return float("inf"), float("inf"), float("inf")
    if floor > 0:
        t = float(np.linalg.norm(err.ravel()) / max(np.linalg.norm(want.ravel()), floor * np.sqrt(want.size))) / tol
    else:
        t = rel_l2(got, want) / tol
    rms = float(np.sqrt(np.mean(want * want))) if want.size else 0.0
    scale = max(rms, floor)
    if want.ndim == 2 and rms > 0:
        row = np.sqrt(np.mean(want * want, axis=1, keepdims=True))
        col = np.sqrt(np.mean(want * want, axis=0, keepdims=True))
        scale = np.maximum(max(rms, floor), row * col / rms)
    bound = C_ELEM * (tol if elem_tol is None else elem_tol) * (scale + np.abs(want))
    with np.errstate(divide="ignore", invalid="ignore"):
        frac = np.where(bound > 0, np.abs(err) / bound, np.where(err == 0, 0.0, np.inf))
    e = float(frac.max()) if frac.size else 0.0
    closeness.where = np.unravel_index(int(np.argmax(frac)), frac.shape) if frac.size else ()
    r = 0.0
    if want.ndim == 2 and want.shape[0] > 1:
        wn = np.linalg.norm(want, axis=1)
        row_floor = max(float(np.sqrt(np.mean(wn * wn))), floor * np.sqrt(want.shape[1]))
        den = C_ROW * tol * np.maximum(wn, row_floor)
        en = np.linalg.norm(err, axis=1)
        with np.errstate(divide="ignore", invalid="ignore"):
            rf = np.where(den > 0, en / den, np.where(en == 0, 0.0, np.inf))
        r = float(rf.max())
    return t, r, e


def assert_close(got, want, tol, label="", elem_tol=None, floor=0.0):
    """The three bounds of the module docstring; returns the tensor-level relative L2 error."""
    t, r, e = closeness(got, want, tol, elem_tol, floor)
    key = str(label).split(":")[0] if label else "unlabelled"
    w = WORST.setdefault(key, [0.0, 0.0, 0.0])
    w[0], w[1], w[2] = max(w[0], t), max(w[1], r), max(w[2], e)
    assert t <= 1.0, "%s: rel L2 %.3e > %.1e" % (label, t * tol, tol)
    assert r <= 1.0, "%s: worst row error is %.2f of its bound (%.1f x %.1e x row norm)" % (label, r, C_ROW, tol)
    if e > 1.0:
        i = closeness.where
        g, w_ = np.asarray(got, dtype=np.float64)[i], np.asarray(want, dtype=np.float64)[i]
        rms = float(np.sqrt(np.mean(np.asarray(want, dtype=np.float64) ** 2)))
        raise AssertionError("%s: worst element error is %.2f of its bound (%.1f x %.1e x (scale + |value|)): element %s got %.6g "
                             "want %.6g, tensor rms %.4g" % (label, e, C_ELEM, tol if elem_tol is None else elem_tol,
                                                              tuple(int(v) for v in i), g, w_, rms))
    return t * tol


def oracle_layers(flat_layers, H, F):
    """[n, layer_params] float32 -> list of named float64 parameter dicts."""
    return [L.unpack_layer(np.asarray(row, dtype=np.float64), H, F) for row in flat_layers]


def check_grads(got_flat, want_named_list, H, F, tol, label):
    """Every named tensor of every layer on its own (not one global norm), with all three bounds."""
    got_flat = np.asarray(got_flat, dtype=np.float64).reshape(len(want_named_list), -1)
    worst = 0.0
    for l, want in enumerate(want_named_list):
        got = L.unpack_layer(got_flat[l], H, F)
        for n in L.PARAM_NAMES:
            worst = max(worst, assert_close(got[n], want[n], tol, "%s gradient: layer %d %s" % (label, l, n)))
    return worst
