"""The seeded input generator: determinism, statistics, bf16 rounding."""
import numpy as np

from paper_2411_02820_amd import synth


def test_generator_is_counter_based():
    a = synth.normal_f32(1000, 7, 3, 0.02)
    b = synth.normal_f32(400, 7, 3, 0.02, idx0=600)
    assert np.array_equal(a[600:], b)
    assert not np.array_equal(a, synth.normal_f32(1000, 8, 3, 0.02))
    assert not np.array_equal(a, synth.normal_f32(1000, 7, 4, 0.02))


def test_generator_known_values():
    # element 0 of (seed 0, stream 0) from the definition, evaluated with Python integers
    key = synth.stream_key(0, 0)
    a = synth._mix64_int(key)
    b = synth._mix64_int(key + synth._G)
    s = sum((a >> (16 * i)) & 0xFFFF for i in range(4)) + sum((b >> (16 * i)) & 0xFFFF for i in range(4))
    assert synth.lane_sums(0, 0, 0, 1)[0] == s - 262140


def test_moments():
    v = synth.normal_f32(1 << 20, 1, 2, 0.02)
    assert abs(v.mean()) < 1e-4
    assert abs(v.std() / 0.02 - 1) < 5e-3
    g = synth.normal_f32(1 << 16, 1, 2, 0.02, offset=1.0)
    assert abs(g.mean() - 1) < 1e-3


def test_threaded_matches_serial():
    n = (1 << 20) * 5 + 17
    a = synth.normal_f32(n, 3, 1, 1.0)
    b = synth.normal_f32(n, 3, 1, 1.0, chunk=n + 1)
    assert np.array_equal(a, b)


def test_bf16_round_to_nearest_even():
    x = np.array([1.0, 1.0 + 2**-8, 1.0 + 2**-7, 1.0 + 3 * 2**-8, -1.0 - 2**-8 - 2**-20], dtype=np.float32)
    got = synth.bf16_bits_to_f32(synth.f32_to_bf16_bits(x))
    # ties go to the even mantissa; above-tie rounds away
    assert np.array_equal(got, np.array([1.0, 1.0, 1.0 + 2**-7, 1.0 + 2**-6, -1.0 - 2**-7], dtype=np.float32))


def test_shapes_and_ratios():
    # E cache is 2x one layer's KV for the 8B shape and 4x for the 70B shape (Sec. 4.1)
    for shape, ratio in ((synth.LLAMA_8B, 2), (synth.LLAMA_70B, 4)):
        assert shape.hidden == ratio * 2 * shape.kv_width
    lens = synth.ragged_lengths(8, 1024, 8192)
    assert lens.min() >= 1024 and lens.max() <= 8192
    cu = synth.cu_seqlens(lens)
    assert cu[-1] == lens.sum()
    pos = synth.packed_positions(lens)
    assert pos[cu[1]] == 0 and pos[cu[1] - 1] == lens[0] - 1


def test_expert_tensor_streams_do_not_collide_with_layer_streams():
    # every tensor of a model is its own generator stream: layer tensors below 2^20, expert tensors from 2^20 on
    streams = set()
    for layer in range(80):
        for kind in range(10):
            streams.add(synth.weight_stream(layer, kind))
        for e in range(64):
            for kind in (synth.WG, synth.WU, synth.WD):
                streams.add(synth.expert_stream(layer, e, kind))
    assert len(streams) == 80 * 10 + 80 * 64 * 3
    assert max(synth.weight_stream(l, k) for l in range(80) for k in range(10)) < synth.EXPERT_STREAM0


def test_expert_layer_weights_have_the_declared_shapes():
    shape = synth.TINY_MOE
    w = synth.layer_weights(shape, synth.SEED_RECEIVER, 1)
    assert w["router"].shape == (shape.n_experts, shape.hidden) and len(w["experts"]) == shape.n_experts
    assert "wg" not in w
    for e in w["experts"]:
        assert e["wg"].shape == (shape.ffn, shape.hidden) and e["wu"].shape == (shape.ffn, shape.hidden)
        assert e["wd"].shape == (shape.hidden, shape.ffn)
    # different experts draw different numbers
    assert not (w["experts"][0]["wg"] == w["experts"][1]["wg"]).all()
