"""bench.py's command line, as far as it can be checked without a GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, cwd=ROOT)
    assert r.returncode != 0 and "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_workloads_name_known_shapes_and_flop_count_covers_experts():
    sys.path.insert(0, ROOT)
    import bench
    from paper_2411_02820_amd import synth
    for name, (shape_name, lens, lo, hi, s1, host) in bench.WORKLOADS.items():
        shape = getattr(synth, shape_name)
        assert lens is None or all(n > 0 for n in lens)
        assert lo is None or 0 <= lo < hi <= shape.n_layers, name
    # per token and layer: 2 flops per weight of the projections a token goes through (+ the router), + attention
    d, F = 4096, 14336
    dense = bench.recompute_flops(synth.LLAMA_8B, [1], 1)
    moe = bench.recompute_flops(synth.MIXTRAL_8X7B, [1], 1)
    assert dense == 2.0 * (d * 6144 + d * d + 3 * d * F) + 2.0 * 32 * 128 * 2
    assert moe - dense == 2.0 * (3 * d * F + d * 8)
