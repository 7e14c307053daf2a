"""Pins for the oracle's mixture-of-experts MLP (the Mixtral receiver of Sec. 5.4): hand-worked values, the dense
special cases, invariants, the router written the other way round (softmax over all experts, then renormalised over
the chosen ones) with torch routines, and a whole layer stack against the `transformers` Mixtral model in float64."""
import math

import numpy as np
import pytest
import torch

from oracle import dsk_oracle as O
from paper_2411_02820_amd import synth
from tests.helpers import oracle_config, weights_fn

rng = np.random.default_rng(77)
SILU1 = 0.7310585786300049  # 1 / (1 + e^-1)


def random_experts(E, d, F, scale=1.0):
    return [{"wg": scale * rng.standard_normal((F, d)), "wu": scale * rng.standard_normal((F, d)),
             "wd": scale * rng.standard_normal((d, F))} for _ in range(E)]


def test_hand_example_top1_and_top2():
    # d = 2, F = 1, two experts; y = (1, 0): router logits (1, 2)
    y = np.array([[1.0, 0.0]])
    router = np.array([[1.0, 0.0], [2.0, 0.0]])
    e0 = {"wg": np.array([[2.0, 0.0]]), "wu": np.array([[1.0, 0.0]]), "wd": np.array([[1.0], [0.0]])}
    e1 = {"wg": np.array([[1.0, 0.0]]), "wu": np.array([[3.0, 0.0]]), "wd": np.array([[1.0], [2.0]])}
    # expert 1 alone: silu(1) * 3 = 2.19317..., times wd = (1, 2)
    out = O.moe_mlp(y, router, [e0, e1], 1)
    assert np.allclose(out, [[3 * SILU1, 6 * SILU1]], atol=1e-15)
    # both: gates softmax(2, 1) = (sigmoid(1), 1 - sigmoid(1)); expert 0 gives silu(2) * 1 on the first coordinate
    silu2 = 2.0 / (1.0 + math.exp(-2.0))
    g1, g0 = SILU1, 1.0 - SILU1
    out = O.moe_mlp(y, router, [e0, e1], 2)
    assert np.allclose(out, [[g1 * 3 * SILU1 + g0 * silu2, g1 * 6 * SILU1]], atol=1e-15)
    logits, experts, gates = O.moe_route(y, router, 2)
    assert np.array_equal(experts, [[1, 0]]) and np.allclose(gates, [[g1, g0]], atol=1e-15)
    assert np.allclose(logits, [[1.0, 2.0]])


def test_one_expert_is_the_dense_mlp():
    d, F, n = 12, 20, 5
    y = rng.standard_normal((n, d))
    ex = random_experts(1, d, F)
    ref = O.swiglu_mlp(y, ex[0]["wg"], ex[0]["wu"], ex[0]["wd"])
    assert np.allclose(O.moe_mlp(y, rng.standard_normal((1, d)), ex, 1), ref, atol=1e-12)
    # the dense MLP itself against torch routines
    t = torch.from_numpy
    lib = (torch.nn.functional.silu(t(y) @ t(ex[0]["wg"]).T) * (t(y) @ t(ex[0]["wu"]).T)) @ t(ex[0]["wd"]).T
    assert np.allclose(ref, lib.numpy(), atol=1e-12)


@pytest.mark.parametrize("top_k", [1, 2, 3])
def test_identical_experts_make_the_router_irrelevant(top_k):
    d, F, n, E = 10, 14, 6, 4
    y = rng.standard_normal((n, d))
    ex = random_experts(1, d, F) * E
    ref = O.swiglu_mlp(y, ex[0]["wg"], ex[0]["wu"], ex[0]["wd"])
    assert np.allclose(O.moe_mlp(y, rng.standard_normal((E, d)), ex, top_k), ref, atol=1e-12)


def test_gates_sum_to_one_and_order_is_descending():
    y = rng.standard_normal((40, 16))
    router = rng.standard_normal((8, 16))
    logits, experts, gates = O.moe_route(y, router, 3)
    assert np.allclose(gates.sum(-1), 1.0, atol=1e-14)
    assert np.all(np.diff(gates, axis=-1) <= 0)
    picked = np.take_along_axis(logits, experts, axis=1)
    assert np.all(np.diff(picked, axis=-1) <= 0)
    rest = np.sort(logits, axis=1)[:, :-3]
    assert np.all(rest.max(-1) <= picked[:, -1])


def test_router_against_softmax_over_all_experts_then_renormalised():
    # the formulation of the Mixtral reference code, with library routines
    y = rng.standard_normal((33, 24))
    router = rng.standard_normal((8, 24))
    _, experts, gates = O.moe_route(y, router, 2)
    p = torch.softmax(torch.from_numpy(y @ router.T), dim=-1)
    top_p, top_i = torch.topk(p, 2, dim=-1)
    top_p = top_p / top_p.sum(-1, keepdim=True)
    assert np.array_equal(experts, top_i.numpy())
    assert np.allclose(gates, top_p.numpy(), atol=1e-14)


def test_ties_go_to_the_lower_expert_index():
    y = np.array([[1.0, 1.0]])
    router = np.array([[0.5, 0.5], [2.0, -1.0], [0.25, 0.75], [1.0, 0.0]])  # logits (1, 1, 1, 1)
    _, experts, gates = O.moe_route(y, router, 2)
    assert np.array_equal(experts, [[0, 1]]) and np.allclose(gates, 0.5)


def test_invariances():
    d, F, n, E = 12, 9, 7, 5
    y = rng.standard_normal((n, d))
    router = rng.standard_normal((E, d))
    ex = random_experts(E, d, F)
    ref = O.moe_mlp(y, router, ex, 2)
    # relabelling the experts changes nothing
    perm = np.array([3, 0, 4, 1, 2])
    assert np.allclose(O.moe_mlp(y, router[perm], [ex[i] for i in perm], 2), ref, atol=1e-12)
    # an expert nobody picks can hold anything: with positive inputs a router row of -5 is never among the top two
    yp = np.abs(y)
    router2 = router.copy()
    router2[4] = -5.0
    _, experts, _ = O.moe_route(yp, router2, 2)
    assert 4 not in set(experts.ravel())
    ex2 = list(ex)
    ex2[4] = random_experts(1, d, F, 50.0)[0]
    assert np.array_equal(O.moe_mlp(yp, router2, ex2, 2), O.moe_mlp(yp, router2, ex, 2))
    # each token is routed on its own
    assert np.allclose(O.moe_mlp(y[2:5], router, ex, 2), ref[2:5], atol=1e-12)


def test_mlp_output_is_the_gate_weighted_sum_of_the_chosen_experts():
    d, F, n, E = 8, 6, 9, 6
    y = rng.standard_normal((n, d))
    router = rng.standard_normal((E, d))
    ex = random_experts(E, d, F)
    dense = np.stack([O.swiglu_mlp(y, e["wg"], e["wu"], e["wd"]) for e in ex])  # [E, n, d]
    logits = y @ router.T
    for i in range(n):
        top = np.argsort(-logits[i], kind="stable")[:2]
        z = np.exp(logits[i, top])
        want = (z[0] * dense[top[0], i] + z[1] * dense[top[1], i]) / z.sum()
        assert np.allclose(O.moe_mlp(y[i:i + 1], router, ex, 2)[0], want, atol=1e-12)


# ---- whole layers against the transformers Mixtral model ----
SHAPE = synth.ModelShape(n_layers=3, hidden=48, n_q_heads=4, n_kv_heads=2, head_dim=16, ffn=40,
                         rope_base=10000.0, rms_eps=1e-5, dtype="f32", n_experts=4, top_k=2)
CFG = oracle_config(SHAPE)
W_SCALE = 12.0  # std 0.02 weights give a nearly linear network and a nearly flat router


def scaled_weights(seed):
    base = weights_fn(SHAPE, seed)

    def get(l):
        w = dict(base(l))
        for k in ("wq", "wk", "wv", "wo", "router"):
            w[k] = w[k] * W_SCALE
        w["experts"] = [{k: v.astype(np.float64) * W_SCALE for k, v in e.items()} for e in w["experts"]]
        return w
    return get


def hf_mixtral(weights):
    from transformers import MixtralConfig, MixtralModel
    cfg = MixtralConfig(hidden_size=SHAPE.hidden, intermediate_size=SHAPE.ffn, num_hidden_layers=SHAPE.n_layers,
                        num_attention_heads=SHAPE.n_q_heads, num_key_value_heads=SHAPE.n_kv_heads,
                        head_dim=SHAPE.head_dim, rms_norm_eps=SHAPE.rms_eps, vocab_size=8, rope_theta=SHAPE.rope_base,
                        max_position_embeddings=512, num_local_experts=SHAPE.n_experts,
                        num_experts_per_tok=SHAPE.top_k, attn_implementation="eager", experts_implementation="eager",
                        sliding_window=None)
    m = MixtralModel(cfg).double().eval()
    names = {"g1": "input_layernorm.weight", "wq": "self_attn.q_proj.weight", "wk": "self_attn.k_proj.weight",
             "wv": "self_attn.v_proj.weight", "wo": "self_attn.o_proj.weight", "g2": "post_attention_layernorm.weight",
             "router": "mlp.gate.weight"}
    sd = m.state_dict()
    for l in range(SHAPE.n_layers):
        w = weights(l)
        for k, n in names.items():
            sd[f"layers.{l}.{n}"].copy_(torch.from_numpy(np.asarray(w[k], dtype=np.float64)))
        gate_up = np.stack([np.concatenate([e["wg"], e["wu"]], axis=0) for e in w["experts"]])
        sd[f"layers.{l}.mlp.experts.gate_up_proj"].copy_(torch.from_numpy(gate_up))
        sd[f"layers.{l}.mlp.experts.down_proj"].copy_(torch.from_numpy(np.stack([e["wd"] for e in w["experts"]])))
    return m


def test_layer_stack_matches_the_library_mixtral():
    T = 21
    w = scaled_weights(synth.SEED_RECEIVER)
    x = synth.hidden_states(SHAPE, T).astype(np.float64)
    m = hf_mixtral(w)
    with torch.no_grad():
        out = m(inputs_embeds=torch.from_numpy(x)[None], use_cache=True, output_hidden_states=True)
    dummy = [(None, None)] * SHAPE.n_layers
    for hi in range(1, SHAPE.n_layers):  # the state entering layer hi (the last hidden state of the library is normed)
        kv, h = O.partial_prefill(CFG, w, x, 0, hi, dummy, np.arange(T), np.array([0, T]))
        assert np.allclose(h, out.hidden_states[hi][0].numpy(), atol=2e-5), hi
    kv, _ = O.partial_prefill(CFG, w, x, 0, SHAPE.n_layers, dummy, np.arange(T), np.array([0, T]))
    for l in range(SHAPE.n_layers):
        K = out.past_key_values.layers[l].keys[0].permute(1, 0, 2).numpy()
        V = out.past_key_values.layers[l].values[0].permute(1, 0, 2).numpy()
        assert np.allclose(kv[l][0], K, atol=2e-5) and np.allclose(kv[l][1], V, atol=2e-5), l
    # the experts matter in this comparison: every expert is used, and swapping two of them breaks it
    y = O.rmsnorm(x, w(0)["g2"], CFG.rms_eps)
    _, experts, _ = O.moe_route(y, w(0)["router"], 2)
    assert len(set(experts.ravel())) == SHAPE.n_experts


def test_selective_prefill_composes_with_expert_layers():
    T = 13
    w = scaled_weights(synth.SEED_RECEIVER)
    x = synth.hidden_states(SHAPE, T).astype(np.float64)
    dummy = [(None, None)] * SHAPE.n_layers
    pos, cu = np.arange(T), np.array([0, T])
    kv_full, h_full = O.partial_prefill(CFG, w, x, 0, 3, dummy, pos, cu)
    kv_a, h1 = O.partial_prefill(CFG, w, x, 0, 1, dummy, pos, cu)
    kv_b, h3 = O.partial_prefill(CFG, w, h1, 1, 3, kv_a, pos, cu)
    assert np.array_equal(h3, h_full)
    for l in range(3):
        assert np.array_equal(kv_b[l][0], kv_full[l][0]) and np.array_equal(kv_b[l][1], kv_full[l][1])
