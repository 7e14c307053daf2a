"""Fit of the profiled prefill-delay model that the run-time choice of the re-computation configuration uses
(App. B: the estimate's parameters come from the profiling phase).  Host code; no step of the hot path.

Model (the one dsk_estimate_prefill_ms evaluates), for R recomputed of L layers over T tokens, in ms:

    t(T, R) = c0 + R * (c1 * T + c2 * T^2) + (L - R) * c3 * T

A recomputed layer costs projections and MLP (linear in T) plus causal attention (quadratic), a reused layer the
transfer of its KV (linear).  The coefficients are costs, so the fit is a non-negative least-squares problem; every
measurement is weighted by 1/t, so that it is the relative misfit that is minimised (the SLO comparison the
estimate feeds is a relative one).
"""
from __future__ import annotations

import numpy as np
from scipy.optimize import nnls


def fit_latency_model(points, n_layers: int):
    """points: iterable of (n_tokens, n_recomputed, measured_ms).  Returns ((c0, c1, c2, c3), max_rel_residual)."""
    pts = [(float(t), float(r), float(ms)) for t, r, ms in points]
    if len(pts) < 4 or any(ms <= 0.0 for _, _, ms in pts):
        raise ValueError("need at least four measurements with positive durations")
    A = np.array([[1.0, r * t, r * t * t, (n_layers - r) * t] for t, r, _ in pts])
    y = np.array([ms for _, _, ms in pts])
    Aw = A / y[:, None]                      # rows scaled by 1/t: relative residuals
    scale = np.maximum(Aw.max(axis=0), 1e-300)   # columns scaled: a well-conditioned problem
    coef = nnls(Aw / scale, np.ones(len(y)))[0] / scale
    resid = float(np.max(np.abs(A @ coef - y) / y))
    return tuple(float(c) for c in coef), resid
