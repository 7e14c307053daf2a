"""The library's run-time choice of the re-computation configuration (host code, no GPU) against the oracle:
the worked example and a few thousand seeded random frontiers, every answer identical."""
import numpy as np
import pytest

from oracle import policy_oracle as P
from tests.test_oracle_policy import FRONTIER, L, LAT


def test_worked_example_through_the_c_abi():
    from paper_2411_02820_amd import binding as B
    assert B.dsk_estimate_prefill_ms(LAT, L, 4, 1000) == pytest.approx(12.2)
    for slo, target, waiting in ((300.0, 0.75, 0), (200.0, 0.75, 0), (1000.0, 0.75, 0), (10.0, 0.75, 0),
                                 (1000.0, 0.75, 3), (1000.0, 0.5, 1), (1000.0, 0.99, 1)):
        assert B.dsk_select_recompute(FRONTIER, L, 8000, LAT, slo, target, waiting) == \
            P.select_recompute(FRONTIER, L, 8000, LAT, slo, target, waiting)


def test_random_frontiers_match_the_oracle():
    from paper_2411_02820_amd import binding as B
    rng = np.random.default_rng(11)
    for _ in range(3000):
        n_layers = int(rng.integers(1, 81))
        n = int(rng.integers(1, 9))
        frontier = []
        for _ in range(n):
            lo = int(rng.integers(0, n_layers + 1))
            hi = int(rng.integers(lo, n_layers + 1))
            frontier.append((lo, hi, float(rng.integers(0, 6)) / 5.0))   # coarse qualities: ties occur
        lat = (float(rng.uniform(0, 2)), float(rng.uniform(0, 4e-3)), float(rng.uniform(0, 2e-7)), float(rng.uniform(0, 2e-4)))
        T = int(rng.integers(0, 40000))
        slo = float(rng.uniform(0, 800))
        target = float(rng.integers(0, 7)) / 5.0
        waiting = int(rng.integers(0, 3))
        got = B.dsk_select_recompute(frontier, n_layers, T, lat, slo, target, waiting)
        assert got == P.select_recompute(frontier, n_layers, T, lat, slo, target, waiting)
        for lo, hi, _ in frontier:
            assert B.dsk_estimate_prefill_ms(lat, n_layers, hi - lo, T) == pytest.approx(
                P.estimate_prefill_ms(lat, n_layers, hi - lo, T), rel=1e-12, abs=1e-12)


def test_bad_input_rejected():
    from paper_2411_02820_amd import binding as B
    for frontier in ([], [(3, 40, 0.5)], [(5, 4, 0.5)]):
        with pytest.raises(B.DskError) as e:
            B.dsk_select_recompute(frontier, L, 10, LAT, 1.0, 0.5, 0)
        assert e.value.status == B.DSK_EINVAL
