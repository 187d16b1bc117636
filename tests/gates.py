"""The two error gates every layer output is held to, and the references they need.

A layer computes y_i = act(sum_j W'_ij x_j + v_i) in fp32; the oracle gives the same
sum in fp64.  "Maximum relative error 1e-5" needs a scale to be relative to, and a
bare max|dy| / max|y| is not enough (a wrong small output passes) and not always
fair (after a ReLU, or when the bias cancels the sum, every output can be small
against the terms that were added).  So an output is checked twice:

* condition-aware, per component:  |y_i - ref_i| <= (n + 4) 2^-24 (sum_j |W'_ij| |x_j| + |v_i|)
  with n the largest number of non-zero weights in a row - the first-order bound
  of n products added in fp32 in any order (a rounding per addition, one for a
  product that is not fused into its addition, the bias, the final store).  A dropped, doubled or misplaced term
  is off by about 1/n of that sum, thousands of times the bound.  Where the sum is
  zero (a row without weights, no bias) the output must be exactly zero.
* normwise:  max|y - ref| <= 1e-5 max|pre-activation ref|.  The scale is taken
  before the activation: a ReLU only clips, it does not change what the error is
  relative to.
"""
from dataclasses import dataclass

import numpy as np

import oracle

TOL = 1e-5
U32 = 2.0 ** -24


@dataclass
class Ref:
    pre: np.ndarray        # fp64, before the activation
    absum: np.ndarray      # sum_j |W'_ij| |x_j| + |v_i|, same shape
    terms: int             # most non-zero weights in one row


def fc_ref(oW, X, bias=None, nthreads=8) -> Ref:
    pre = oracle.fc_forward(oW, X, bias, False, nthreads)
    absum = oracle.fc_forward(np.abs(oW), np.abs(X), None if bias is None else np.abs(bias), False, nthreads)
    return Ref(pre, absum, int((oW != 0).sum(axis=1).max()) if oW.size else 0)


def conv_ref(oW, X, geom, bias=None, nthreads=8) -> Ref:
    pre = oracle.conv_forward(oW, X, geom, bias, False, nthreads)
    absum = oracle.conv_forward(np.abs(oW), np.abs(X), geom, None if bias is None else np.abs(bias), False, nthreads)
    return Ref(pre, absum, int((oW != 0).sum(axis=1).max()) if oW.size else 0)


def errors(Y, ref: Ref, relu: bool):
    """(normwise error, componentwise error in units of 2^-24, largest absolute
    error where the condition sum is zero)."""
    want = np.maximum(ref.pre, 0.0) if relu else ref.pre
    err = np.abs(np.asarray(Y, dtype=np.float64) - want)
    scale = max(float(np.abs(ref.pre).max()), 1e-300) if err.size else 1.0
    live = ref.absum > 0
    comp = float((err[live] / ref.absum[live]).max()) / U32 if live.any() else 0.0
    dead = float(err[~live].max()) if (~live).any() else 0.0
    return (float(err.max()) / scale if err.size else 0.0), comp, dead


def assert_close(Y, ref: Ref, relu: bool, tol=TOL, product_rel=0.0, what=None):
    """Both gates.  product_rel is the relative error each product may carry on top of
    the fp32 accumulation (0 for exact fp32 products; 3 * 2^-16 for the three-term
    bf16 split), in which case the normwise gate widens by the same amount times the
    condition sum."""
    assert Y.shape == ref.pre.shape, (Y.shape, ref.pre.shape, what)
    nw, comp, dead = errors(Y, ref, relu)
    assert dead == 0.0, ("output without terms is not zero", dead, what)
    bound = ref.terms + 4 + product_rel / U32
    assert comp <= bound, ("componentwise", comp, bound, what)
    scale = max(float(np.abs(ref.pre).max()), 1e-300)
    nw_tol = tol + product_rel * float(ref.absum.max()) / scale if product_rel else tol
    assert nw <= nw_tol, ("normwise", nw, nw_tol, what)
    return nw, comp
