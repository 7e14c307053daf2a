"""Pins for the run-time choice of the re-computation configuration (App. B): a worked example by hand, the two
regimes the appendix describes, and properties any correct implementation has."""
import itertools

import pytest

from oracle import policy_oracle as P

L = 32
# a frontier in the shape of Sec. 4.2's example: quality grows with the number of recomputed layers
FRONTIER = [(16, 16, 0.30), (14, 18, 0.55), (12, 20, 0.70), (10, 21, 0.78), (6, 22, 0.80), (0, 32, 0.82)]
# 1 ms fixed, 2 us per token per recomputed layer, 1e-4 us per token^2 per recomputed layer, 0.1 us per token per reused layer
LAT = (1.0, 2e-3, 1e-7, 1e-4)


def test_latency_model_by_hand():
    # T = 1000, R = 4: 1 + 4 * (2 + 0.1) + 28 * 0.1 = 12.2 ms
    assert P.estimate_prefill_ms(LAT, L, 4, 1000) == pytest.approx(12.2)
    # no recompute: only the constant and the transfers; full prefill: no transfers
    assert P.estimate_prefill_ms(LAT, L, 0, 1000) == pytest.approx(1.0 + 32 * 0.1)
    assert P.estimate_prefill_ms(LAT, L, 32, 1000) == pytest.approx(1.0 + 32 * 2.1)


def test_worked_example():
    T = 8000
    # per recomputed layer 16 + 6.4 = 22.4 ms, per reused layer 0.8 ms
    est = [P.estimate_prefill_ms(LAT, L, hi - lo, T) for lo, hi, _ in FRONTIER]
    assert est == pytest.approx([26.6, 113.0, 199.4, 264.2, 372.2, 717.8])
    # idle engine: the most layers that fit the SLO
    assert P.select_recompute(FRONTIER, L, T, LAT, 300.0, 0.75, 0) == 3
    assert P.select_recompute(FRONTIER, L, T, LAT, 200.0, 0.75, 0) == 2
    assert P.select_recompute(FRONTIER, L, T, LAT, 1000.0, 0.75, 0) == 5
    # nothing fits: the cheapest point
    assert P.select_recompute(FRONTIER, L, T, LAT, 10.0, 0.75, 0) == 0
    # requests are waiting: the fewest layers above the accuracy target, whatever the SLO
    assert P.select_recompute(FRONTIER, L, T, LAT, 1000.0, 0.75, 3) == 3
    assert P.select_recompute(FRONTIER, L, T, LAT, 1000.0, 0.50, 1) == 1
    # target out of reach: the cheapest point
    assert P.select_recompute(FRONTIER, L, T, LAT, 1000.0, 0.99, 1) == 0


def test_properties():
    tokens = (500, 4000, 16000)
    slos = (5.0, 50.0, 150.0, 400.0, 2000.0)
    for T in tokens:
        picked = [P.select_recompute(FRONTIER, L, T, LAT, s, 0.7, 0) for s in slos]
        n_layers = [FRONTIER[i][1] - FRONTIER[i][0] for i in picked]
        assert n_layers == sorted(n_layers), "a looser SLO never recomputes fewer layers"
        for s, i in zip(slos, picked):
            lo, hi, _ = FRONTIER[i]
            fits = [j for j, (a, b, _) in enumerate(FRONTIER) if P.estimate_prefill_ms(LAT, L, b - a, T) <= s]
            if fits:
                assert i in fits and all(FRONTIER[j][1] - FRONTIER[j][0] <= hi - lo for j in fits)
    for s in slos:   # more tokens never allow more layers
        n = [FRONTIER[P.select_recompute(FRONTIER, L, T, LAT, s, 0.7, 0)] for T in tokens]
        n = [hi - lo for lo, hi, _ in n]
        assert n == sorted(n, reverse=True)
    # under load the choice ignores tokens and SLO
    for T, s in itertools.product(tokens, slos):
        assert P.select_recompute(FRONTIER, L, T, LAT, s, 0.7, 2) == 2


def test_order_independence_and_ties():
    T = 8000
    for perm in itertools.permutations(range(len(FRONTIER)), len(FRONTIER)):
        if perm[0] > 2:   # a sample of the orders is enough
            continue
        fr = [FRONTIER[i] for i in perm]
        assert fr[P.select_recompute(fr, L, T, LAT, 300.0, 0.75, 0)] == FRONTIER[3]
        assert fr[P.select_recompute(fr, L, T, LAT, 300.0, 0.75, 1)] == FRONTIER[3]
    # equal layer counts: the better quality wins
    fr = [(0, 4, 0.5), (8, 12, 0.6), (20, 24, 0.55)]
    assert P.select_recompute(fr, L, T, LAT, 1e9, 0.0, 0) == 1
    assert P.select_recompute(fr, L, T, LAT, 1e9, 0.0, 1) == 1


def test_bad_input_rejected():
    with pytest.raises(ValueError):
        P.select_recompute([], L, 10, LAT, 1.0, 0.5, 0)
    with pytest.raises(ValueError):
        P.select_recompute([(3, 40, 0.5)], L, 10, LAT, 1.0, 0.5, 0)
    with pytest.raises(ValueError):
        P.select_recompute([(5, 4, 0.5)], L, 10, LAT, 1.0, 0.5, 0)
