"""The schedule model of the three loading strategies against the totals the paper prints (Sec. 4.3)."""
import os

from oracle.schedule_model import Job, total_ttft

HERE = os.path.dirname(os.path.abspath(__file__))


def golden():
    out = {}
    for line in open(os.path.join(HERE, "golden", "fig13_loading_strategies.txt")):
        if line.strip() and not line.startswith("#"):
            k, v = line.split()
            out[k] = float(v)
    return out


def paper_example():
    return [Job(0.0, 10, 7, True), Job(2.0, 10, 3, False)]


def test_totals_of_the_worked_example():
    for strategy, expected in golden().items():
        assert total_ttft(paper_example(), strategy) == expected, strategy


def test_pipelining_never_loses_and_degenerate_cases():
    jobs = paper_example()
    assert total_ttft(jobs, "pipelined") <= total_ttft(jobs, "reused_then_compute") <= total_ttft(jobs, "all_then_compute")
    # full prefill (nothing reused, no E cache): no transfers in (b) and (c)
    full = [Job(0.0, 10, 10, False)]
    assert total_ttft(full, "reused_then_compute") == total_ttft(full, "pipelined") == 10
    assert total_ttft(full, "all_then_compute") == 20
    # full reuse: only transfers
    reuse = [Job(0.0, 10, 0, False)]
    assert total_ttft(reuse, "pipelined") == total_ttft(reuse, "reused_then_compute") == 10
    # a faster link shrinks the pipelined total towards the compute time
    assert total_ttft([Job(0.0, 10, 7, True)], "pipelined", unit_load=0.01) < 7.1
