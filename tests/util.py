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

Tensors behind SEVERAL layers (the output of a chained network, a map read back from inside
one) are gated on the stated bar itself, E_inf <= tol on the whole tensor, with exactly the
stated tol and no multiplier (assert_net_close), or -- where the condition sum of the last
layer is at hand -- on assert_chain_close.  An element there inherits the perturbations of
its inputs, which are relative to the scale of the activations and not to the element, so
no element-wise relative figure is bounded by the summation order any more; it is returned
for the log only.
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


def assert_net_close(got, ref, tol, what=""):
    """Gate for a tensor behind several layers: finite, and E_inf = max|got - ref| / max|ref|
    within the stated bar.  Returns (E_inf, E_el); E_el is informative only (see above)."""
    assert np.isfinite(np.asarray(got, dtype=np.float64)).all(), f"{what}: non-finite output"
    e_inf, e_el = rel_errors(got, ref)
    assert e_inf <= tol, f"{what}: E_inf={e_inf:.3e} tol={tol}"
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


CHAIN_SIGMAS = 8.0      # standard deviations the statistical bound allows


def chain_bounds(ops, ins, outs, ws, bs, f16):
    """Element-wise bound on |got - ref| for the output of EVERY op of a chained network: a
    forward error analysis run by the oracle on magnitudes, no tolerance chosen by hand.
    Two bounds are propagated and the smaller one is used.

    Worst case (every perturbation aligned).  With B_in the bound on the op's input (zero for
    the net input) a fused layer obeys

        e   = sum |w| B_in  (+ B_residual)  +  SUM_TOL * A        (A as in assert_layer_close)
        B   = e + out_ulp * (|ref| + e)

    (ReLU and the maximum are 1-Lipschitz; a mean averages the bounds; both sides round to the
    storage type, hence one full step out_ulp of the larger of the two values; in fp16 storage
    a residual the runner computes inside the layer -- a fused projection shortcut -- skips
    the rounding the separate layer applies: one more step of |residual|).  This bound is
    rigorous but grows with the product of the layers' absolute row sums, so a few layers deep
    it says nothing.

    Statistical (rounding errors as independent zero-mean variables, the usual probabilistic
    model of rounding error analysis): variances propagate through a layer with the SQUARED
    weights,

        s2  = sum w^2 s2_in  (+ s2_residual)  +  (SUM_TOL * A / CHAIN_SIGMAS)^2
                                               +  2 * (out_ulp * |ref|)^2 / 12

    (two roundings of a uniform error of one step each), and the bound is CHAIN_SIGMAS
    standard deviations.  Returns a list aligned with `ops` (float64 arrays like outs[i])."""
    npdt = np.float16 if f16 else np.float32
    ulp = F16_ULP if f16 else 0.0
    f32 = lambda a: np.ascontiguousarray(np.asarray(a, dtype=np.float64) * (1.0 + 1e-6), dtype=np.float32)
    first = ins[0]
    zero = np.zeros(first.shape, dtype=np.float64)
    bound_of, var_of = {ops[0].src: zero}, {ops[0].src: zero}
    ref_of = {ops[0].src: np.asarray(first, dtype=np.float64)}
    result = []
    for i, op in enumerate(ops):
        b_in, v_in = bound_of[op.src], var_of[op.src]
        ref = np.asarray(outs[i], dtype=np.float64)
        own = np.zeros(ref.shape)          # this op's own summation error, worst case
        if op.kind in ("conv", "dwconv", "fc"):
            w = np.asarray(ws[i]).astype(npdt)
            aw = np.abs(w.astype(np.float32))
            w2 = aw.astype(np.float64) ** 2
            if op.kind == "conv":
                res = ref_of[op.res] if op.res >= 0 else None
                e = oracle.conv2d_f64(f32(b_in), aw, None, f32(bound_of[op.res]) if op.res >= 0 else None, op.stride, op.pad, False)
                v = oracle.conv2d_f64(f32(v_in), f32(w2), None, f32(var_of[op.res]) if op.res >= 0 else None, op.stride, op.pad, False)
                own = SUM_TOL * cond_conv(ins[i], w, bs[i], None if res is None else res.astype(np.float32), op.stride, op.pad)
                if res is not None:
                    own = own + ulp * np.abs(res)
            elif op.kind == "dwconv":
                e = oracle.depthwise_conv2d_f64(f32(b_in), aw, None, op.stride, op.pad, False)
                v = oracle.depthwise_conv2d_f64(f32(v_in), f32(w2), None, op.stride, op.pad, False)
                own = SUM_TOL * cond_depthwise(ins[i], w, bs[i], op.stride, op.pad)
            else:
                e = oracle.fc_f64(f32(b_in), aw, None, False).reshape(ref.shape)
                v = oracle.fc_f64(f32(v_in), f32(w2), None, False).reshape(ref.shape)
                own = SUM_TOL * cond_fc(ins[i], w, bs[i]).reshape(ref.shape)
        elif op.kind == "maxpool":
            e = oracle.maxpool(f32(b_in), op.k, op.stride, op.pad, dtype=np.float64)
            v = oracle.maxpool(f32(v_in), op.k, op.stride, op.pad, dtype=np.float64)
        elif op.kind in ("avgpool2d", "avgpool"):
            mean = (lambda a: oracle.avgpool(a, op.k, op.stride, op.pad, dtype=np.float64)) if op.kind == "avgpool2d" \
                else (lambda a: oracle.global_avgpool(a, dtype=np.float64))
            e = mean(f32(b_in))
            v = mean(f32(v_in))           # (an upper bound: the mean of n independent errors has 1/n of it)
            own = 2e-6 * mean(np.abs(np.asarray(ins[i], dtype=np.float32)))
        elif op.kind == "concat":
            e = np.concatenate([bound_of[b] for b in op.srcs], axis=1)
            v = np.concatenate([var_of[b] for b in op.srcs], axis=1)
        else:
            raise ValueError(op.kind)
        if op.kind in ("maxpool", "concat"):          # values are passed on, not rounded again
            b_worst, var = e, v
        else:
            e = e + own
            b_worst = e + ulp * (np.abs(ref) + e) + (2.0 ** -24 if f16 else 0.0)
            var = v + (own / CHAIN_SIGMAS) ** 2 + 2.0 * (ulp * np.abs(ref)) ** 2 / 12.0 + ((2.0 ** -24) ** 2 if f16 else 0.0)
        b = np.minimum(b_worst, CHAIN_SIGMAS * np.sqrt(var))
        # (what is carried on: the worst-case recursion may start again from the smaller bound)
        bound_of[op.dst] = b
        var_of[op.dst] = np.minimum(var, (b_worst / CHAIN_SIGMAS) ** 2) if b_worst.size else var
        ref_of[op.dst] = ref
        result.append(b)
    return result


def assert_within_bound(got, ref, bound, what=""):
    g = np.asarray(got, dtype=np.float64)
    r = np.asarray(ref, dtype=np.float64)
    assert g.shape == r.shape == bound.shape, (g.shape, r.shape, bound.shape)
    assert np.isfinite(g).all(), f"{what}: non-finite output"
    d = np.abs(g - r)
    lim = bound * 1.001 + 1e-30
    assert (d <= lim).all(), f"{what}: {int((d > lim).sum())} elements beyond the propagated bound, worst ratio {(d / lim).max():.3f}"
    return float((d / lim).max())
