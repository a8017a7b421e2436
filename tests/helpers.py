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


def assert_close(got, ref, tol, what=""):
    elem, norm = err_report(got, ref)
    if os.environ.get("SDP_TEST_VERBOSE"):
        print(f"[err] {what}: elementwise {elem:.3e} normwise {norm:.3e} (tol {tol:.0e})", flush=True)
    assert elem <= tol and norm <= tol, f"{what}: elementwise {elem:.3e}, normwise {norm:.3e} > tol {tol:.1e}"
    return elem, norm
