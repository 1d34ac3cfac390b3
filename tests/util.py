"""Helpers shared by the parity tests.

Tolerance.  The stated bar is a maximum
relative error of 1e-4 for fp32 outputs and 1e-2 for the fp16-storage variant.  It is
enforced in two ways:

  E_inf = max|got - ref| / max|ref|  <=  tol                      (whole tensor)

and element by element against the magnitude of what was summed,

  |got_i - ref_i|  <=  1e-4 * A_i  +  out_ulp * |ref_i|

where A_i = sum |w||x| + |bias| + |residual| is the same layer evaluated by the oracle on
absolute values (the condition denominator of the sum: any fp32 summation order obeys
|error| <= (n+2) * 2^-24 * A_i, which stays below 1e-4 * A_i up to n ~ 1600 terms in the
worst case and far beyond that in practice), and out_ulp is the rounding of the stored
result (0 for fp32 against the oracle's correctly rounded fp32, 2^-10 for fp16).
A plain element-wise relative error is ill-conditioned wherever terms cancel (it is not
bounded by any summation order), so it is reported but gated only on elements that are not
small: E_el over |ref_i| >= 1e-2 * max|ref|.
"""
import numpy as np

import oracle

TOL_F32 = 1e-4
TOL_F16 = 1e-2
SUM_TOL = 1e-4          # accumulation is fp32 in both variants
F16_ULP = 2.0 ** -10


def rel_errors(got, ref, floor=1e-2):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    scale = np.abs(ref).max() if ref.size else 0.0
    d = np.abs(got - ref)
    if scale == 0.0:
        return (d.max() if d.size else 0.0), 0.0
    big = np.abs(ref) >= floor * scale
    e_el = (d[big] / np.abs(ref[big])).max() if big.any() else 0.0
    return d.max() / scale, e_el


def assert_close(got, ref, tol, what=""):
    """Whole-tensor gate (used for chained networks where no per-element condition
    number is available): E_inf and E_el over the not-small elements."""
    assert np.isfinite(np.asarray(got, dtype=np.float64)).all(), f"{what}: non-finite output"
    e_inf, e_el = rel_errors(got, ref)
    assert e_inf <= tol and e_el <= tol, f"{what}: E_inf={e_inf:.3e} E_el={e_el:.3e} tol={tol}"
    return e_inf, e_el


def cond_conv(x, w, bias, residual, stride, pad):
    ab = lambda a: None if a is None else np.abs(np.asarray(a, dtype=np.float32))
    return oracle.conv2d_f64(ab(x), ab(w), ab(bias), ab(residual), stride, pad, False)


def cond_depthwise(x, w, bias, stride, pad):
    ab = lambda a: None if a is None else np.abs(np.asarray(a, dtype=np.float32))
    return oracle.depthwise_conv2d_f64(ab(x), ab(w), ab(bias), stride, pad, False)


def cond_fc(x, w, bias):
    ab = lambda a: None if a is None else np.abs(np.asarray(a, dtype=np.float32))
    return oracle.fc_f64(ab(x), ab(w), ab(bias), False)


def assert_layer_close(got, ref, cond, tol, what="", f16=False):
    """Single-layer gate: E_inf <= tol and the element-wise bound described above."""
    g = np.asarray(got, dtype=np.float64)
    r = np.asarray(ref, dtype=np.float64)
    assert g.shape == r.shape == cond.shape, (g.shape, r.shape, cond.shape)
    assert np.isfinite(g).all(), f"{what}: non-finite output"
    d = np.abs(g - r)
    bound = SUM_TOL * cond + (F16_ULP if f16 else 0.0) * np.abs(r) + 1e-30
    bad = d > bound
    assert not bad.any(), (f"{what}: {bad.sum()} elements beyond the bound, worst ratio "
                           f"{(d / bound).max():.3f}")
    e_inf, e_el = rel_errors(g, r)
    assert e_inf <= tol, f"{what}: E_inf={e_inf:.3e} tol={tol}"
    return e_inf, e_el, float((d / bound).max())


def assert_chain_close(got, ref, cond_last, tol, what=""):
    """End-to-end gate for a chained network: E_inf <= tol, and every output within
    tol * max(A_i, 0.01 * max|ref|), where A_i is the condition sum of the LAST layer on the
    oracle's input to it.  Perturbations inherited from earlier layers are relative to the
    scale of the activations rather than to each activation, hence the floor."""
    g = np.asarray(got, dtype=np.float64)
    r = np.asarray(ref, dtype=np.float64)
    c = np.asarray(cond_last, dtype=np.float64).reshape(r.shape)
    assert g.shape == r.shape
    assert np.isfinite(g).all(), f"{what}: non-finite output"
    d = np.abs(g - r)
    e_inf, e_el = rel_errors(g, r)
    scale = np.maximum(c, 0.01 * np.abs(r).max())
    worst = float((d / (tol * scale + 1e-30)).max())
    assert e_inf <= tol and worst <= 1.0, f"{what}: E_inf={e_inf:.3e} worst |d|/(tol*scale)={worst:.3f}"
    return e_inf, e_el, worst
