"""Unit-cost schedule model of the three KV-loading strategies (Sec. 4.3, Fig. 13).

TEST INFRASTRUCTURE ONLY (like everything under oracle/).  The paper's worked example: two receiver
models with ten layers each share one link and one GPU; recomputing one layer and transferring one
layer's KV or one E cache each cost one time unit; A recomputes layers 4-10 (reuses 1-3, needs the E
cache of layer 4), B recomputes layers 1-3 (reuses 4-10; its transition layer is the first layer, so it
needs no E cache); A arrives at t=0, B at t=2.  The figure's totals are reproduced by this reading:

  (a) load everything, then compute: jobs are served one after the other; a job costs
      [E] + L transfers + R recomputed layers.
  (b) load only the reused layers, then compute: as (a) with L-R transfers.
  (c) pipelined: the link and the GPU are separate FIFO resources.  A job's E cache goes first on the
      link; its recompute may start once the E cache has arrived (at arrival if none is needed) and the
      GPU is free; its reused-layer transfers follow on the link in parallel; the job ends when both its
      transfers and its recompute have ended.

TTFT of a job = end - arrival; the figure quotes the sum over the two jobs.
"""
from dataclasses import dataclass


@dataclass(frozen=True)
class Job:
    arrival: float
    n_layers: int
    n_recompute: int
    needs_e: bool      # transition layer is not the first layer


def total_ttft(jobs, strategy, unit_load=1.0, unit_compute=1.0):
    """strategy: 'all_then_compute' (a), 'reused_then_compute' (b), 'pipelined' (c)."""
    jobs = sorted(jobs, key=lambda j: j.arrival)
    total = 0.0
    if strategy in ("all_then_compute", "reused_then_compute"):
        t = 0.0
        for j in jobs:
            n_load = j.n_layers if strategy == "all_then_compute" else j.n_layers - j.n_recompute
            t = max(t, j.arrival) + (unit_load if j.needs_e else 0.0) + n_load * unit_load + j.n_recompute * unit_compute
            total += t - j.arrival
        return total
    if strategy != "pipelined":
        raise ValueError(strategy)
    link = gpu = 0.0
    for j in jobs:
        link = max(link, j.arrival)
        e_done = j.arrival
        if j.needs_e:
            link += unit_load
            e_done = link
        link += (j.n_layers - j.n_recompute) * unit_load
        gpu = max(gpu, e_done) + j.n_recompute * unit_compute
        total += max(link, gpu) - j.arrival
    return total
