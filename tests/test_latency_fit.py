"""The latency-model fit (App. B: parameters obtained by profiling) recovers known coefficients from exact and
from noisy synthetic measurements, and never returns a negative cost."""
import numpy as np
import pytest

from oracle import policy_oracle as P
from paper_2411_02820_amd.latency_fit import fit_latency_model

L = 32
TRUE = (0.4, 3.5e-4, 3.3e-9, 2.0e-5)
GRID = [(T, R) for T in (2048, 4096, 8192, 16384) for R in (2, 4, 8, 16)]


def test_exact_measurements_give_back_the_coefficients():
    pts = [(T, R, P.estimate_prefill_ms(TRUE, L, R, T)) for T, R in GRID]
    lat, resid = fit_latency_model(pts, L)
    assert resid <= 1e-9
    assert lat == pytest.approx(TRUE, rel=1e-6)


def test_noisy_measurements_stay_within_the_noise():
    rng = np.random.default_rng(3)
    pts = [(T, R, P.estimate_prefill_ms(TRUE, L, R, T) * (1.0 + 0.03 * rng.uniform(-1, 1))) for T, R in GRID]
    lat, resid = fit_latency_model(pts, L)
    assert resid <= 0.06 and all(c >= 0.0 for c in lat)
    for T, R in ((3000, 3), (12000, 12), (16384, 32)):
        assert P.estimate_prefill_ms(lat, L, R, T) == pytest.approx(P.estimate_prefill_ms(TRUE, L, R, T), rel=0.08)


def test_costs_are_never_negative_and_bad_input_is_refused():
    # measurements that a free fit would explain with a negative constant
    pts = [(T, R, 1e-3 * R * T) for T, R in GRID]
    lat, _ = fit_latency_model(pts, L)
    assert all(c >= 0.0 for c in lat)
    with pytest.raises(ValueError):
        fit_latency_model(pts[:3], L)
    with pytest.raises(ValueError):
        fit_latency_model([(1, 1, 0.0)] * 5, L)
