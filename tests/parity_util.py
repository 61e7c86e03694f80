"""Tolerances and comparison helpers for the GPU-vs-oracle parity tests.

fp32 path: log Z within 1e-5 relative; every gradient tensor within 1e-4 relative, read per tensor as
|x - y| <= 1e-4 |y| + 1e-4 mean|y| elementwise and a relative L2 error <= 1e-4.
"""
import numpy as np

LOGZ_RTOL_FP32 = 1e-5
GRAD_RTOL_FP32 = 1e-4


def check_logZ(got, ref, rtol=LOGZ_RTOL_FP32):
    got, ref = np.asarray(got, np.float64), np.asarray(ref, np.float64)
    fin = np.isfinite(ref)
    assert np.array_equal(np.isfinite(got), fin), f"finite pattern differs: {got} vs {ref}"
    assert np.all(got[~fin] == ref[~fin])
    err = np.abs(got[fin] - ref[fin])
    tol = rtol * np.abs(ref[fin])
    assert np.all(err <= tol), f"logZ max rel err {np.max(err / np.abs(ref[fin])):.3e} (tol {rtol})\n{got}\n{ref}"
    return float(np.max(err / np.abs(ref[fin]))) if fin.any() else 0.0


def check_grad(name, got, ref, rtol=GRAD_RTOL_FP32):
    got, ref = np.asarray(got, np.float64), np.asarray(ref, np.float64)
    assert got.shape == ref.shape, f"{name}: shape {got.shape} vs {ref.shape}"
    assert np.all(np.isfinite(got)), f"{name}: non-finite entries"
    scale = np.mean(np.abs(ref))
    err = np.abs(got - ref)
    tol = rtol * np.abs(ref) + rtol * scale
    worst = np.unravel_index(np.argmax(err - tol), err.shape)
    l2 = np.linalg.norm(got - ref) / max(np.linalg.norm(ref), 1e-300)
    assert np.all(err <= tol), (f"{name}: elementwise tolerance exceeded at {worst}: got {got[worst]:.8e} ref "
                                f"{ref[worst]:.8e} (mean|ref| {scale:.3e}, rel L2 {l2:.3e})")
    assert l2 <= rtol, f"{name}: relative L2 error {l2:.3e} > {rtol}"
    return float(l2)


def check_all(got, ref, logz_rtol=LOGZ_RTOL_FP32, grad_rtol=GRAD_RTOL_FP32):
    stats = {"logZ": check_logZ(got["logZ"], ref["logZ"], logz_rtol)}
    for k in ("grad_log_root", "grad_log_emit", "grad_L", "grad_R"):
        stats[k] = check_grad(k, got[k], ref[k], grad_rtol)
    return stats
