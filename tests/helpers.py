"""Shared test utilities: the error metric used for every floating-point comparison."""
import os

import numpy as np


def err_report(got, ref):
    """Mixed tolerance metric.

    Returns (elementwise, normwise): elementwise = max_i |got_i - ref_i| / max(rms(ref), |ref_i|),
    normwise = ||got - ref||_2 / ||ref||_2.  A tensor passes at tolerance tol when both are <= tol
    (i.e. rtol = tol with atol = tol * rms(ref), plus a norm bound).
    """
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    assert np.isfinite(got).all(), "non-finite value in result"
    if ref.size == 0:
        return 0.0, 0.0
    rms = np.sqrt(np.mean(ref * ref))
    nrm = np.sqrt(np.sum(ref * ref))
    diff = np.abs(got - ref)
    if rms == 0.0:
        return (0.0, 0.0) if diff.max() == 0.0 else (np.inf, np.inf)
    elem = float(np.max(diff / np.maximum(rms, np.abs(ref))))
    norm = float(np.sqrt(np.sum(diff * diff)) / nrm)
    return elem, norm


def err_report_rows(got, ref):
    """The same metric with one scale per row: elementwise = max_ij |got_ij - ref_ij| / max(rms(ref_i), |ref_ij|),
    normwise = max_i ||got_i - ref_i|| / ||ref_i||.  For tensors whose rows differ in scale by construction
    (a token's attention output is an average over all earlier tokens, so row norms fall with the position)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape and got.ndim == 2, (got.shape, ref.shape)
    assert np.isfinite(got).all(), "non-finite value in result"
    if ref.size == 0:
        return 0.0, 0.0
    rms = np.sqrt(np.mean(ref * ref, axis=1, keepdims=True))
    diff = np.abs(got - ref)
    zero = rms[:, 0] == 0.0
    if zero.any() and diff[zero].max() != 0.0:
        return np.inf, np.inf
    rms = np.where(rms == 0.0, 1.0, rms)
    elem = float(np.max(diff / np.maximum(rms, np.abs(ref))))
    norm = float(np.max(np.sqrt(np.mean(diff * diff, axis=1, keepdims=True)) / rms))
    return elem, norm


def assert_close_rows(got, ref, tol, what=""):
    elem, norm = err_report_rows(got, ref)
    if os.environ.get("SDP_TEST_VERBOSE"):
        print(f"[err] {what}: per-row elementwise {elem:.3e} normwise {norm:.3e} (tol {tol:.0e})", flush=True)
    assert elem <= tol and norm <= tol, f"{what}: per-row elementwise {elem:.3e}, normwise {norm:.3e} > tol {tol:.1e}"
    return elem, norm


def assert_close(got, ref, tol, what="", elem_tol=None):
    """Both figures of err_report within tol; elem_tol, when given, replaces tol for the elementwise figure."""
    elem, norm = err_report(got, ref)
    et = tol if elem_tol is None else elem_tol
    if os.environ.get("SDP_TEST_VERBOSE"):
        print(f"[err] {what}: elementwise {elem:.3e} normwise {norm:.3e} (tol {et:.0e} / {tol:.0e})", flush=True)
    assert elem <= et and norm <= tol, f"{what}: elementwise {elem:.3e} > {et:.1e} or normwise {norm:.3e} > {tol:.1e}"
    return elem, norm


def assert_close_with_model(got, model, ref, tol, what="", elem_allow=None, rows=False, slack_elem=1.5, slack_norm=1.1):
    """bf16 results whose distance from the exact result is set by the storage format.  `ref` is the oracle, `model`
    the same arithmetic in fp64 with only the bf16 rounding points of the GPU path switched on
    (tests/rounding_model.py).  Individual roundings of the two cannot be expected to coincide (an upstream
    difference far below one bf16 ulp flips a later rounding), so the comparison is between error figures:

      - `got` is no further from `ref` than the rounding points alone put `model`, up to slack_norm on the
        normwise figure and slack_elem on the elementwise maximum (an extreme value over 10^4 - 10^6 elements);
        the floor of both allowances is a quarter of tol, for tensors the model reproduces almost exactly;
      - and within the fixed bounds: tol normwise, elem_allow (default tol) elementwise.

    rows=True takes one scale per row."""
    rep = err_report_rows if rows else err_report
    eo, no = rep(got, ref)
    e3, n3 = rep(model, ref)
    ea = tol if elem_allow is None else elem_allow
    if os.environ.get("SDP_TEST_VERBOSE"):
        print(f"[err] {what}: vs oracle {eo:.2e} / {no:.2e} (bounds {ea:.0e} / {tol:.0e}); rounding model vs oracle "
              f"{e3:.2e} / {n3:.2e}", flush=True)
    assert eo <= max(slack_elem * e3, tol / 4) and no <= max(slack_norm * n3, tol / 4), (
        f"{what}: {eo:.3e} / {no:.3e} from the oracle, but the bf16 rounding points alone give {e3:.3e} / {n3:.3e}")
    assert eo <= ea and no <= tol, f"{what}: elementwise {eo:.3e} > {ea:.1e} or normwise {no:.3e} > {tol:.1e} from the oracle"
    return eo, no
