"""Mixture-of-experts receiver (Sec. 5.4, Mixtral) on the HIP path against the CPU oracle, through the C ABI.

The router decides an integer (which experts a token visits) from floating-point logits.  Where the oracle's logits
separate the k-th from the (k+1)-th expert by less than the rounding of the device's inputs, both choices are correct
outcomes of the method at that precision: such tokens are checked for a valid choice at the component level and left
out of the element-wise comparison at the model level (their share is asserted to stay small); every other token
must agree with the oracle to the usual bar (1e-3 fp32, 2e-2 bf16)."""
import numpy as np
import pytest
import torch

from oracle import dsk_oracle as O
from paper_2411_02820_amd import synth
from tests.helpers import kv_list, oracle_config, weights_fn

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-3, "bf16": 2e-2}
# gap between the last chosen and the first rejected logit, in units of the standard deviation of the top_k + 1
# highest logits of all tokens, below which a
# token's routing counts as undecided at the path's precision (fp32: accumulation order; bf16: the normalised
# activations are rounded to 2^-9 relative and the states entering a layer carry up to 1e-2 from the layers before)
MARGIN = {"f32": 1e-4, "bf16": 5e-2}

SMALL_MOE_BF16 = synth.ModelShape(2, 512, 8, 2, 128, 512, 500000.0, 1e-5, "bf16", 4, 2)
SMALL_MOE_BF16_E8 = synth.ModelShape(2, 512, 8, 2, 128, 256, 500000.0, 1e-5, "bf16", 8, 2)


@pytest.fixture(scope="module")
def G():
    from tests import gpu_util
    return gpu_util


def scaled_weights(shape, seed, scale):
    base = weights_fn(shape, seed)

    def get(l):
        w = dict(base(l))
        for k in ("wq", "wk", "wv", "wo", "router"):
            w[k] = (w[k].astype(np.float32) * np.float32(scale)).astype(np.float64)
        w["experts"] = [{k: (v.astype(np.float32) * np.float32(scale)).astype(np.float64) for k, v in e.items()}
                        for e in w["experts"]]
        return w
    return get


class RouteRecorder:
    """Wraps the oracle's router to note, per call, which token rows were undecided (see MARGIN)."""

    def __init__(self, monkeypatch, top_k, margin):
        self.calls = []
        orig = O.moe_route

        def wrapped(y, router, k):
            logits, experts, gates = orig(y, router, k)
            srt = -np.sort(-logits, axis=1)
            gap = srt[:, top_k - 1] - srt[:, top_k] if logits.shape[1] > top_k else np.full(len(logits), np.inf)
            self.calls.append(gap < margin * srt[:, :top_k + 1].std())  # spread of the logits that compete
            return logits, experts, gates
        monkeypatch.setattr(O, "moe_route", wrapped)


# ---------------------------------------------------------------- router alone
@pytest.mark.parametrize("dtype,n,d,E,k", [("f32", 133, 256, 4, 2), ("bf16", 1000, 512, 8, 2), ("bf16", 77, 4096, 8, 2),
                                            ("bf16", 65, 512, 16, 4), ("f32", 9, 64, 3, 1), ("bf16", 40, 256, 5, 5)])
def test_router_against_oracle(G, dtype, n, d, E, k):
    from paper_2411_02820_amd import binding as B
    shape = synth.ModelShape(1, d, 1, 1, 64, 64, 1e4, 1e-5, dtype)
    x = synth.normal(n * d, 11, 0, 1.0, 0.0, dtype).reshape(n, d)
    wr = synth.normal(E * d, 11, 1, 0.1, 0.0, dtype).reshape(E, d)
    ex = torch.empty((n, k), dtype=torch.int32, device="cuda")
    ga = torch.empty((n, k), dtype=torch.float32, device="cuda")
    B.dsk_moe_route(B.DSK_F32 if dtype == "f32" else B.DSK_BF16, G.to_dev(x, shape), G.to_dev(wr, shape), n, d, E, k, ex, ga)
    torch.cuda.synchronize()
    ex, ga = ex.cpu().numpy(), ga.cpu().numpy()
    logits, ex_ref, ga_ref = O.moe_route(x.astype(np.float64), wr.astype(np.float64), k)  # same (representable) inputs
    thr = 1e-5 * np.abs(logits).max()  # fp32 accumulation of d products
    srt = -np.sort(-logits, axis=1)
    gaps = np.diff(-srt[:, :k + 1] if E > k else -srt, axis=1)  # gaps between consecutive logits down to the first rejected
    decided = (gaps > thr).all(axis=1) if gaps.size else np.ones(n, bool)
    assert decided.mean() > 0.9
    assert np.array_equal(ex[decided], ex_ref[decided])
    assert np.allclose(ga[decided], ga_ref[decided], atol=2e-5)
    # the rest: a valid choice (distinct experts, none worse than the k-th logit by more than thr) and gates that sum to one
    for i in np.where(~decided)[0]:
        assert len(set(ex[i])) == k and (logits[i, ex[i]] >= srt[i, k - 1] - thr).all()
    assert np.allclose(ga.sum(-1), 1.0, atol=1e-5) and (ga >= 0).all()
    assert (np.diff(ga, axis=1) <= 1e-6).all(), "highest logit first"


def test_router_ties_go_to_the_lower_index(G):
    from paper_2411_02820_amd import binding as B
    shape = synth.ModelShape(1, 256, 1, 1, 64, 64, 1e4, 1e-5, "bf16")
    n, d = 50, 256
    x = synth.normal(n * d, 12, 0, 1.0, 0.0, "bf16").reshape(n, d)
    row = synth.normal(d, 12, 1, 0.1, 0.0, "bf16")
    wr = np.stack([row, row, row, row])  # four identical experts: all logits equal
    ex = torch.empty((n, 2), dtype=torch.int32, device="cuda")
    ga = torch.empty((n, 2), dtype=torch.float32, device="cuda")
    B.dsk_moe_route(B.DSK_BF16, G.to_dev(x, shape), G.to_dev(wr, shape), n, d, 4, 2, ex, ga)
    torch.cuda.synchronize()
    assert np.array_equal(ex.cpu().numpy(), np.tile([0, 1], (n, 1)))
    assert np.array_equal(ga.cpu().numpy(), np.full((n, 2), 0.5, dtype=np.float32))
    _, ex_ref, _ = O.moe_route(x.astype(np.float64), wr.astype(np.float64), 2)
    assert np.array_equal(ex_ref, np.tile([0, 1], (n, 1)))


def test_router_rejects_bad_shapes(G):
    from paper_2411_02820_amd import binding as B
    x = torch.zeros((4, 64), dtype=torch.float32, device="cuda")
    ex = torch.empty((4, 2), dtype=torch.int32, device="cuda")
    ga = torch.empty((4, 2), dtype=torch.float32, device="cuda")
    for E, k in ((2, 3), (65, 2), (4, 0), (16, 9)):
        with pytest.raises(B.DskError) as err:
            B.dsk_moe_route(B.DSK_F32, x, x, 4, 64, E, k, ex, ga)
        assert err.value.status == B.DSK_ESHAPE


# ---------------------------------------------------------------- whole path
def run_moe_case(G, monkeypatch, shape, lens, lo, hi, slens, scale, max_undecided=0.25):
    tol = TOL[shape.dtype]
    cfg = oracle_config(shape)
    cu = synth.cu_seqlens(lens)
    T = int(cu[-1])
    S = int(sum(slens)) if slens else 0
    pos = synth.packed_positions(lens)
    hidden_in = synth.hidden_states(shape, T)
    kv_r = synth.kv_cache(shape, T)
    w = scaled_weights(shape, synth.SEED_RECEIVER, scale)
    if shape.dtype == "bf16" and scale > 2.0 and hi > lo:
        # strong weights: the bound follows the spread of the attention scores, as for the dense model
        from tests.test_gpu_parity import bf16_tolerance
        tol = bf16_tolerance(cfg, w(lo), hidden_in.astype(np.float64), pos)
        print(f"weight scale {scale}: tolerance {tol:.3e}")
    rec = RouteRecorder(monkeypatch, shape.top_k, MARGIN[shape.dtype])

    with G.GpuModel(shape, max(T, S, 1), T + S) as m:
        m.load_from_generator(synth.SEED_RECEIVER, scale=scale)
        kv_out, h_out = m.partial(G.to_dev(hidden_in, shape), lo, hi, G.to_dev(kv_r, shape), lens, n_rows=T + S)
        torch.cuda.synchronize()
        kv_gpu, h_gpu = G.to_np(kv_out), G.to_np(h_out)

        kv_ref, h_ref = O.partial_prefill(cfg, w, hidden_in.astype(np.float64), lo, hi, kv_list(kv_r), pos, cu)
        assert len(rec.calls) == hi - lo
        # a token undecided in layer l may differ from that layer's output on: its rows are skipped from there
        bad = np.zeros(T, bool)
        for l in range(shape.n_layers):
            if lo <= l < hi:
                ok = ~bad
                assert O.max_rel_err(kv_gpu[l, 0, :T][ok], kv_ref[l][0][ok]) <= tol, f"K layer {l}"
                assert O.max_rel_err(kv_gpu[l, 1, :T][ok], kv_ref[l][1][ok]) <= tol, f"V layer {l}"
                bad |= rec.calls[l - lo]
            else:
                assert np.array_equal(kv_gpu[l, :, :T], kv_r[l]), f"splice layer {l}"
            assert np.isnan(kv_gpu[l, :, T:]).all()
        print(f"undecided routings: {bad.mean():.3f} of {T} prefix tokens")
        assert bad.mean() <= max_undecided
        assert O.max_rel_err(h_gpu[~bad], h_ref[~bad]) <= tol, "hidden_out"

        if S:
            rec.calls.clear()
            xs = synth.hidden_states(shape, S, seed=synth.SEED_SUFFIX)
            hs_out = m.suffix(G.to_dev(xs, shape), kv_out, lens, slens)
            torch.cuda.synchronize()
            kv_gpu2, hs_gpu = G.to_np(kv_out), G.to_np(hs_out)
            spos = synth.packed_positions(slens, start=lens)
            kv_s, hs_ref = O.suffix_prefill(cfg, w, xs.astype(np.float64), kv_ref, spos, cu, synth.cu_seqlens(slens))
            assert np.array_equal(kv_gpu2[:, :, :T], kv_gpu[:, :, :T])
            sbad = np.zeros(S, bool)
            for l in range(shape.n_layers):
                ok = ~sbad
                assert O.max_rel_err(kv_gpu2[l, 0, T:][ok], kv_s[l][0][ok]) <= tol, f"suffix K layer {l}"
                assert O.max_rel_err(kv_gpu2[l, 1, T:][ok], kv_s[l][1][ok]) <= tol, f"suffix V layer {l}"
                sbad |= rec.calls[l]
            print(f"undecided routings: {sbad.mean():.3f} of {S} suffix tokens")
            assert sbad.mean() <= max(max_undecided, 2.0 / S)
            assert O.max_rel_err(hs_gpu[~sbad], hs_ref[~sbad]) <= tol, "suffix hidden_out"


def test_tiny_fp32_experts(G, monkeypatch):
    # 3 layers, d 256, 4/2 heads, dh 64, 4 experts of width 320, top 2; every expert runs over all rows (fp32 path)
    run_moe_case(G, monkeypatch, synth.TINY_MOE, [128], 1, 3, [16], 8.0, max_undecided=0.02)


def test_tiny_fp32_experts_ragged_whole_model(G, monkeypatch):
    run_moe_case(G, monkeypatch, synth.TINY_MOE, [70, 1, 129, 37], 0, 3, [3, 1, 16, 5], 8.0, max_undecided=0.02)


def test_small_bf16_experts_grouped_rows(G, monkeypatch):
    # prefix rows grouped by expert on the tensor-core path (333 tokens, 666 expert rows over 4 experts), suffix rows
    # through every expert
    run_moe_case(G, monkeypatch, SMALL_MOE_BF16, [333], 0, 2, [17], 2.0)


def test_small_bf16_eight_experts_ragged(G, monkeypatch):
    run_moe_case(G, monkeypatch, SMALL_MOE_BF16_E8, [200, 1, 77, 300], 0, 2, [9, 1, 33, 2], 2.0)


def test_small_bf16_just_above_the_few_row_path(G, monkeypatch):
    # 65 tokens: grouped, every expert's rows a fraction of one 256-row tile
    run_moe_case(G, monkeypatch, SMALL_MOE_BF16_E8, [65], 0, 2, None, 2.0)


def test_expert_weights_round_trip_and_generator(G):
    # set/get of router and expert tensors, and the device generator against the host generator, bit for bit
    shape = SMALL_MOE_BF16
    with G.GpuModel(shape, 8) as m:
        m.init_random(synth.SEED_RECEIVER)
        for l in (0, 1):
            assert np.array_equal(G.to_np(m.get_tensor(l, synth.WR)), synth.layer_tensor(shape, synth.SEED_RECEIVER, l, synth.WR))
            for e in (0, 3):
                for kind in (synth.WG, synth.WU, synth.WD):
                    assert np.array_equal(G.to_np(m.get_tensor(l, kind, expert=e)),
                                          synth.expert_tensor(shape, synth.SEED_RECEIVER, l, e, kind)), (l, e, kind)
        from paper_2411_02820_amd import binding as B
        t = torch.zeros((shape.ffn, shape.hidden), dtype=torch.bfloat16, device="cuda")
        for bad in (synth.WG, B.DSK_EXPERT(4, synth.WG), B.DSK_EXPERT(0, synth.WQ)):
            with pytest.raises(B.DskError) as err:
                B.dsk_model_set_tensor(m.handle, 0, bad, t)
            assert err.value.status == B.DSK_EINVAL


def test_expert_with_no_tokens(G, monkeypatch):
    # one expert's router row pushed far down: it receives no rows, its tiles do not exist, the result is unchanged
    shape = SMALL_MOE_BF16
    cfg = oracle_config(shape)
    T = 300
    lens = [T]
    cu, pos = synth.cu_seqlens(lens), synth.packed_positions(lens)
    hidden_in = np.abs(synth.hidden_states(shape, T))  # positive states: after the norm (gains near 1) still positive
    base = scaled_weights(shape, synth.SEED_RECEIVER, 2.0)

    def w(l):
        ww = dict(base(l))
        r = ww["router"].copy()
        r[2] = -1.0
        ww["router"] = r
        return ww
    rec = RouteRecorder(monkeypatch, shape.top_k, MARGIN["bf16"])
    kv_ref, h_ref = O.partial_prefill(cfg, w, hidden_in.astype(np.float64), 0, 1, [(None, None)] * 2, pos, cu)
    y = O.rmsnorm(hidden_in.astype(np.float64), w(0)["g1"], cfg.rms_eps)
    with G.GpuModel(shape, T) as m:
        m.load_from_generator(synth.SEED_RECEIVER, scale=2.0)
        from paper_2411_02820_amd import binding as B
        r = synth.layer_tensor(shape, synth.SEED_RECEIVER, 0, synth.WR) * np.float32(2.0)
        r[2] = -1.0
        B.dsk_model_set_tensor(m.handle, 0, synth.WR, G.to_dev(r, shape))
        kv_r = synth.kv_cache(shape, T)
        kv_out, h_out = m.partial(G.to_dev(hidden_in, shape), 0, 1, G.to_dev(kv_r, shape), lens)
        torch.cuda.synchronize()
        ok = ~rec.calls[0]
        assert ok.mean() > 0.75
        assert O.max_rel_err(G.to_np(h_out)[ok], h_ref[ok]) <= TOL["bf16"]


# ---------------------------------------------------------------- at the width of Mixtral 8x7B
def host_moe_layer(shape, seed, layer):
    print(f"[host] generating layer {layer} of the {shape.hidden}-wide model with {shape.n_experts} experts", flush=True)
    w = synth.layer_weights(shape, seed, layer)
    return {k: ([{n: t.astype(np.float64) for n, t in e.items()} for e in v] if k == "experts" else v.astype(np.float64))
            for k, v in w.items()}


def test_mixtral_width_layer_over_4096_tokens_and_suffix_pass(G, monkeypatch):
    # Two layers of the Mixtral 8x7B layer shape (d 4096, 32/8 heads, 8 experts of width 14336, top 2), weights from the
    # device generator (bit-identical to the host's).  (a) Layer 0 over 4096 tokens: 8192 expert rows grouped on the
    # device, about four 256-row tiles per expert, both expert projections in one grouped launch each: K/V of every
    # row and the state leaving the layer at sampled rows against the oracle.  (b) The suffix pass of 64 tokens through
    # both layers against seeded N(0,1) prefix rows: every expert streamed over the 64 rows on the few-row tiles.
    from paper_2411_02820_amd import binding as B
    from tests.test_gpu_fullsize import device_kv_cache, device_normal, host_kv_rows
    base = synth.MIXTRAL_8X7B
    shape = synth.ModelShape(2, base.hidden, base.n_q_heads, base.n_kv_heads, base.head_dim, base.ffn, base.rope_base,
                             base.rms_eps, "bf16", base.n_experts, base.top_k)
    cfg = oracle_config(shape)
    T, S = 4096, 64
    rows = sorted({0, 1, 63, 64, 255, 256, 1000, 2047, 2048, 3000, 4000, 4094, 4095})
    hidden_host = synth.hidden_states(shape, T)
    w0 = host_moe_layer(shape, synth.SEED_RECEIVER, 0)
    rec = RouteRecorder(monkeypatch, shape.top_k, MARGIN["bf16"])
    with G.GpuModel(shape, T, T + S) as m:
        m.init_random(synth.SEED_RECEIVER)
        B.dsk_set_option("reset_stats", 0)
        hidden_dev = device_normal(B, (T, shape.hidden), synth.SEED_HIDDEN, 0)
        assert np.array_equal(G.to_np(hidden_dev[:2]), hidden_host[:2])
        kv_1, h_1 = m.partial(hidden_dev, 0, 1, device_kv_cache(B, shape, T, T), [T])
        torch.cuda.synchronize()
        assert B.dsk_get_stat("gemm_generic_launches") == 0 and B.dsk_get_stat("gemm_mfma_launches") == 4
        h_ref, K, V = O.prefix_layer(cfg, w0, hidden_host.astype(np.float64), synth.packed_positions([T]),
                                     synth.cu_seqlens([T]), rows=rows)
        ok = ~rec.calls[0]
        errs = {"K": O.max_rel_err(G.to_np(kv_1[0, 0, :T]), K), "V": O.max_rel_err(G.to_np(kv_1[0, 1, :T]), V),
                "hidden_rows": O.max_rel_err(G.to_np(h_1)[rows][ok], h_ref[ok])}
        print(f"layer 0 over {T} tokens: {ok.sum()} of {len(rows)} sampled rows decided; max-rel-err:",
              {k: f"{v:.2e}" for k, v in errs.items()}, flush=True)
        assert ok.sum() >= len(rows) - 4 and max(errs.values()) <= TOL["bf16"], errs

        # (b) suffix pass
        rec.calls.clear()
        cu, cus = synth.cu_seqlens([T]), synth.cu_seqlens([S])
        spos = synth.packed_positions([S], start=[T])
        xs_host = synth.hidden_states(shape, S, seed=synth.SEED_SUFFIX)
        kv = device_kv_cache(B, shape, T + S, T)
        B.dsk_set_option("reset_stats", 0)
        hs = m.suffix(G.to_dev(xs_host, shape), kv, [T], [S])
        torch.cuda.synchronize()
        assert B.dsk_get_stat("gemm_generic_launches") == 0 and B.dsk_get_stat("attn_generic_launches") == 0
        weights = {0: w0}

        def wfn(l):
            if l not in weights:
                weights.clear()
                weights[l] = host_moe_layer(shape, synth.SEED_RECEIVER, l)
            return weights[l]
        del w0
        kv_s, hs_ref = O.suffix_prefill(cfg, wfn, xs_host.astype(np.float64), [host_kv_rows(shape, l, T) for l in range(2)],
                                        spos, cu, cus)
        bad0, bad1 = rec.calls[0], rec.calls[0] | rec.calls[1]
        errs = {"sK0": O.max_rel_err(G.to_np(kv[0, 0, T:]), kv_s[0][0]), "sV0": O.max_rel_err(G.to_np(kv[0, 1, T:]), kv_s[0][1]),
                "sK1": O.max_rel_err(G.to_np(kv[1, 0, T:])[~bad0], kv_s[1][0][~bad0]),
                "sV1": O.max_rel_err(G.to_np(kv[1, 1, T:])[~bad0], kv_s[1][1][~bad0]),
                "suffix_hidden": O.max_rel_err(G.to_np(hs)[~bad1], hs_ref[~bad1])}
        print(f"suffix pass: undecided routings {bad0.sum()} + {(bad1 & ~bad0).sum()} of {S}; max-rel-err:",
              {k: f"{v:.2e}" for k, v in errs.items()}, flush=True)
        assert bad1.mean() <= 0.35 and max(errs.values()) <= TOL["bf16"], errs


def test_bf16_experts_on_the_plain_kernels_agree_with_the_tensor_core_path(G, monkeypatch):
    # the "force_generic" hook sends a bf16 model through the plain-ALU kernels, every expert over all rows, for any
    # number of rows: the same oracle bar, and the same tokens decided
    from paper_2411_02820_amd import binding as B
    B.dsk_set_option("force_generic", 1)
    try:
        run_moe_case(G, monkeypatch, SMALL_MOE_BF16, [150], 0, 2, [5], 2.0)
    finally:
        B.dsk_set_option("force_generic", 0)


def test_model_create_rejects_bad_expert_configurations(G):
    from paper_2411_02820_amd import binding as B
    import dataclasses
    for E, k in ((4, 0), (4, 5), (65, 2), (0, 2), (16, 9)):
        shape = dataclasses.replace(synth.TINY_MOE, n_experts=E, top_k=k)
        with pytest.raises(B.DskError) as err:
            B.dsk_model_create(B.config_from_shape(shape), 8, 8)
        assert err.value.status == B.DSK_ESHAPE, (E, k)


def test_two_recompute_groups_with_experts(G, monkeypatch):
    # the several-groups call on an expert model: bit-identical to chained single-group calls (Sec. 4.1)
    shape = SMALL_MOE_BF16
    T = 200
    hidden = synth.hidden_states(shape, T)
    kv_r = synth.kv_cache(shape, T)
    with G.GpuModel(shape, T) as m:
        m.load_from_generator(synth.SEED_RECEIVER, scale=2.0)
        h_dev, kv_dev = G.to_dev(hidden, shape), G.to_dev(kv_r, shape)
        kv_g, outs = m.partial_groups([(0, 1, h_dev), (1, 2, h_dev)], kv_dev, [T])
        kv_a, h_a = m.partial(h_dev, 0, 1, kv_dev, [T])
        kv_b, h_b = m.partial(h_dev, 1, 2, kv_a, [T])
        torch.cuda.synchronize()
        assert torch.equal(kv_g[:, :, :T], kv_b[:, :, :T])
        assert torch.equal(outs[0], h_a) and torch.equal(outs[1], h_b)


def test_other_expert_counts(G, monkeypatch):
    # one expert per token of three (fp32), and four of sixteen on the grouped tensor-core path
    run_moe_case(G, monkeypatch, synth.ModelShape(2, 256, 4, 2, 64, 192, 10000.0, 1e-5, "f32", 3, 1), [90, 41], 0, 2, [6, 2], 8.0,
                 max_undecided=0.02)
    run_moe_case(G, monkeypatch, synth.ModelShape(2, 512, 8, 2, 128, 128, 500000.0, 1e-5, "bf16", 16, 4), [200], 0, 2, [40], 2.0,
                 max_undecided=0.5)
