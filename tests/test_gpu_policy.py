"""App. B on the GPU side: the latency model is fitted from measured dsk_partial_prefill calls (the profiling
phase), and the library's choice of the re-computation configuration with those coefficients is checked
against the oracle's, through the C ABI."""
import numpy as np
import pytest
import torch

from oracle import policy_oracle as P
from paper_2411_02820_amd import synth
from paper_2411_02820_amd.latency_fit import fit_latency_model

pytestmark = pytest.mark.gpu

# wide enough that a layer is compute-bound from 4096 tokens on (the regime the model describes), small enough to
# profile in a second
SHAPE = synth.ModelShape(8, 2048, 16, 4, 128, 8192, 500000.0, 1e-5, "bf16")
TOKENS = (4096, 8192, 16384)
DEPTHS = (2, 4, 8)


def test_latency_model_fitted_from_measured_calls_drives_the_policy():
    from paper_2411_02820_amd import binding as B
    from tests import gpu_util as G
    L, Tmax = SHAPE.n_layers, max(TOKENS)
    with G.GpuModel(SHAPE, Tmax) as m:
        m.init_random(synth.SEED_RECEIVER)
        hidden = torch.empty((Tmax, SHAPE.hidden), dtype=torch.bfloat16, device="cuda")
        B.dsk_fill_normal(hidden, hidden.numel(), synth.SEED_HIDDEN, 0, 1.0, 0.0, 0, B.DSK_BF16)
        kv_r, kv_out = m.new_cache(Tmax, fill=0.5), m.new_cache(Tmax, fill=0.0)

        def measure(T, R, reps=4):
            batch = B.Batch(synth.cu_seqlens([T]), synth.packed_positions([T]))
            lo = min(2, L - R)
            best = float("inf")
            for i in range(reps + 1):   # the first call is a warm-up
                s, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                torch.cuda.synchronize()
                s.record()
                B.dsk_partial_prefill(m.handle, hidden, lo, lo + R, B.kv_desc(kv_r), B.kv_desc(kv_out), batch.desc, None)
                e.record()
                torch.cuda.synchronize()
                if i:
                    best = min(best, s.elapsed_time(e))
            return best

        points = [(T, R, measure(T, R)) for T in TOKENS for R in DEPTHS]
        lat, resid = fit_latency_model(points, L)
        print("measured (T, R, ms):", [(t, r, round(ms, 3)) for t, r, ms in points])
        print("fitted (c0, c1, c2, c3):", lat, "max relative residual:", round(resid, 4))
        assert resid <= 0.10, f"the profiled delays do not follow c0 + R(c1 T + c2 T^2) + (L-R) c3 T: {resid:.3f}"
        # a point that was not part of the fit
        T_new, R_new = 12288, 6
        got, est = measure(T_new, R_new), B.dsk_estimate_prefill_ms(lat, L, R_new, T_new)
        print(f"held-out point T={T_new} R={R_new}: measured {got:.3f} ms, estimated {est:.3f} ms")
        assert est == pytest.approx(got, rel=0.2)

    # the library's estimate and choice with the fitted coefficients, against the oracle
    frontier = [(2, 2, 0.30), (2, 4, 0.55), (1, 5, 0.70), (0, 6, 0.74), (0, 8, 0.80)]
    full_ms = P.estimate_prefill_ms(lat, L, L, Tmax)
    for T in (3000, 8192, 16384):
        for lo, hi, _ in frontier:
            assert B.dsk_estimate_prefill_ms(lat, L, hi - lo, T) == pytest.approx(
                P.estimate_prefill_ms(lat, L, hi - lo, T), rel=1e-12, abs=1e-12)
        picks = []
        for frac in (0.0, 0.1, 0.3, 0.5, 0.7, 0.9, 1.2):
            for waiting in (0, 2):
                for target in (0.5, 0.72, 0.99):
                    got = B.dsk_select_recompute(frontier, L, T, lat, frac * full_ms, target, waiting)
                    assert got == P.select_recompute(frontier, L, T, lat, frac * full_ms, target, waiting)
                    picks.append(got)
        assert len(set(picks)) >= 3, "the sweep must exercise several frontier points"
