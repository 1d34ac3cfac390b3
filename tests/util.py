"""Helpers shared by the parity tests."""
import numpy as np

TOL_F32 = 1e-4   # max relative error stated for fp32 outputs
TOL_F16 = 1e-2   # and for the fp16-storage variant


def rel_errors(got, ref):
    """(E_inf, E_el): max|d|/max|ref| and the largest element-wise relative error over the
    elements with |ref| >= 1e-3 * max|ref| (relative error on near-zero outputs is
    ill-conditioned by cancellation and is covered by E_inf instead)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    scale = np.abs(ref).max() if ref.size else 0.0
    d = np.abs(got - ref)
    if scale == 0.0:
        return (d.max() if d.size else 0.0), 0.0
    big = np.abs(ref) >= 1e-3 * scale
    e_el = (d[big] / np.abs(ref[big])).max() if big.any() else 0.0
    return d.max() / scale, e_el


def assert_close(got, ref, tol, what=""):
    assert np.isfinite(np.asarray(got, dtype=np.float64)).all(), f"{what}: non-finite output"
    e_inf, e_el = rel_errors(got, ref)
    assert e_inf <= tol and e_el <= tol, f"{what}: E_inf={e_inf:.3e} E_el={e_el:.3e} tol={tol}"
    return e_inf, e_el
