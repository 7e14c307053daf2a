"""Choice of the re-computation configuration at run time (App. B, "Dynamic Re-computation Configuration
Adaptation"), as a plain function.

TEST INFRASTRUCTURE ONLY (like everything under oracle/); shares no code with the library.

The offline profile is a list of frontier points (lo, hi, quality): for some numbers of recomputed layers the
contiguous group [lo, hi) with the best quality found (Sec. 4.2, the Pareto frontier).  At run time, in the
paper's order:

  1. If requests are waiting in the engine the load is high: take the point with the fewest recomputed layers
     whose quality still reaches the accuracy target.
  2. Otherwise estimate each point's prefill latency from the request's token count with the profiled latency
     model and take the point with the most recomputed layers (the highest re-computation ratio, hence the best
     accuracy) that meets the latency SLO.

Readings where the appendix is silent: if no point reaches the accuracy target in step 1, or none meets the SLO
in step 2, the point with the fewest recomputed layers is taken (the cheapest one); ties in the number of layers
go to the higher quality, then to the lower index.  The latency model is the one a profile of this library
supports: a constant, a per-recomputed-layer term linear in the tokens (projections, MLP) plus one quadratic in
them (causal attention), and a per-reused-layer term linear in the tokens (its KV transfer):

  t(T, R) = c0 + R * (c1 * T + c2 * T^2) + (L - R) * c3 * T
"""


def estimate_prefill_ms(lat, n_layers, n_recomputed, n_tokens):
    c0, c1, c2, c3 = lat
    return c0 + n_recomputed * (c1 * n_tokens + c2 * n_tokens * n_tokens) + (n_layers - n_recomputed) * c3 * n_tokens


def select_recompute(frontier, n_layers, n_tokens, lat, slo_ms, quality_target, n_waiting):
    """frontier: list of (lo, hi, quality).  Returns the index of the chosen point."""
    if not frontier:
        raise ValueError("empty frontier")
    for lo, hi, _ in frontier:
        if not (0 <= lo <= hi <= n_layers):
            raise ValueError("frontier point outside the model")

    def layers(i):
        return frontier[i][1] - frontier[i][0]

    def fewest(candidates):
        best = None
        for i in candidates:
            if best is None or layers(i) < layers(best) or (layers(i) == layers(best) and frontier[i][2] > frontier[best][2]):
                best = i
        return best

    everything = range(len(frontier))
    if n_waiting > 0:
        good = [i for i in everything if frontier[i][2] >= quality_target]
        return fewest(good if good else everything)
    in_time = [i for i in everything if estimate_prefill_ms(lat, n_layers, layers(i), n_tokens) <= slo_ms]
    if not in_time:
        return fewest(everything)
    best = None
    for i in in_time:
        if best is None or layers(i) > layers(best) or (layers(i) == layers(best) and frontier[i][2] > frontier[best][2]):
            best = i
    return best
