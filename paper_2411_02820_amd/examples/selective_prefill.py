"""The three interfaces of Sec. 4.4 end to end, on a small model: a sender LLM prefills a context and stores its KV
cache and the E cache of the transition layer; a receiver LLM of the same architecture fetches them, recomputes
layers [lo, hi) from the E cache while the other layers' KV is loaded on the side stream (Sec. 4.1, 4.3), and
prefills its new tokens against the mixed cache.  The recompute configuration is chosen at run time from a frontier
table, a latency model and an SLO (App. B).

    python -m paper_2411_02820_amd.examples.selective_prefill

Everything that computes runs in libdsk (HIP, gfx950); torch only owns device memory.  Weights and inputs are
synthetic (seeded), and the frontier's quality numbers are placeholders: quality needs trained model pairs."""
import time

import torch

from paper_2411_02820_amd import binding as B
from paper_2411_02820_amd import synth

SHAPE = synth.ModelShape(n_layers=8, hidden=1024, n_q_heads=8, n_kv_heads=2, head_dim=128, ffn=2816,
                         rope_base=500000.0, rms_eps=1e-5, dtype="bf16")
T, S = 2048, 32            # context tokens, new tokens
SENDER, RECEIVER = 1, 0    # model ids (also the weight seeds)


def main():
    cfg = B.config_from_shape(SHAPE)
    L, d = SHAPE.n_layers, SHAPE.hidden
    row_bytes = SHAPE.kv_width * SHAPE.elem_bytes
    bf16 = torch.bfloat16

    def cache(rows):
        return torch.empty((L, 2, rows, SHAPE.n_kv_heads, SHAPE.head_dim), dtype=bf16, device="cuda")

    context = B.dsk_hash_context(b"a long document both agents read")
    prefix = B.Batch(synth.cu_seqlens([T]), synth.packed_positions([T]))
    suffix = B.Batch(synth.cu_seqlens([S]), synth.packed_positions([S], start=[T]))
    embeddings = torch.empty((T, d), dtype=bf16, device="cuda")
    B.dsk_fill_normal(embeddings, embeddings.numel(), synth.SEED_HIDDEN, 0, 1.0, 0.0, 0, B.DSK_BF16)

    # ---- choose the recompute configuration (App. B): most layers whose estimated delay meets the SLO ----
    frontier = [(3, 3, 0.30), (3, 5, 0.62), (2, 6, 0.74), (0, L, 0.80)]   # (lo, hi, quality): placeholders
    latency = (0.05, 1.5e-4, 2.0e-9, 1.0e-5)                               # ms: c0, per layer-token, per layer-token^2, per reused token
    pick = B.dsk_select_recompute(frontier, L, T, latency, slo_ms=2.0, quality_target=0.7, n_waiting=0)
    lo, hi, _ = frontier[pick]
    print(f"recompute layers [{lo},{hi}) of {L} (estimated {B.dsk_estimate_prefill_ms(latency, L, hi - lo, T):.2f} ms)")

    store = B.dsk_store_create(1 << 30, 1 << 30)
    sender = B.dsk_model_create(cfg, T, T)
    receiver = B.dsk_model_create(cfg, T, T + S)
    try:
        B.dsk_model_init_random(sender, SENDER, synth.WEIGHT_STD)
        B.dsk_model_init_random(receiver, RECEIVER, synth.WEIGHT_STD)

        # ---- sender: full prefill, then store(KV) and store(E at layer lo) ----
        kv_sender = cache(T)
        B.dsk_partial_prefill(sender, embeddings, 0, L, None, B.kv_desc(kv_sender), prefix.desc)
        e_lo = torch.empty((T, d), dtype=bf16, device="cuda")
        if lo > 0:   # the state entering layer lo: layers [0, lo) once more (the path is deterministic)
            B.dsk_partial_prefill(sender, embeddings, 0, lo, B.kv_desc(kv_sender), B.kv_desc(kv_sender), prefix.desc, e_lo)
        else:
            e_lo.copy_(embeddings)
        B.dsk_store_put_kv(store, context, SENDER, B.kv_desc(kv_sender), L, T, row_bytes)   # GPU memory while it fits (Sec. 4.4)
        B.dsk_store_put_e(store, context, SENDER, lo, e_lo)
        torch.cuda.synchronize()

        # ---- receiver: fetch, selective prefill (loads pipelined under the recompute), suffix ----
        kv_fetched, _ = B.dsk_store_fetch_kv(store, context, SENDER)
        e_ptr, e_mem, _ = B.dsk_store_fetch_e(store, context, SENDER, lo)
        kv_mixed = cache(T + S)
        new_tokens = torch.empty((S, d), dtype=bf16, device="cuda")
        B.dsk_fill_normal(new_tokens, new_tokens.numel(), synth.SEED_SUFFIX, 0, 1.0, 0.0, 0, B.DSK_BF16)
        out = torch.empty_like(new_tokens)

        def selective():
            B.dsk_partial_prefill(receiver, (e_ptr, e_mem), lo, hi, kv_fetched, B.kv_desc(kv_mixed), prefix.desc, None,
                                  B.DSK_DEFER_JOIN)
            B.dsk_suffix_prefill(receiver, new_tokens, B.kv_desc(kv_mixed), prefix.desc, suffix.desc, T, out)

        def full():
            B.dsk_partial_prefill(receiver, embeddings, 0, L, None, B.kv_desc(kv_mixed), prefix.desc)
            B.dsk_suffix_prefill(receiver, new_tokens, B.kv_desc(kv_mixed), prefix.desc, suffix.desc, T, out)

        times = {}
        for name, fn in (("full prefill", full), ("selective prefill", selective)):
            fn()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(5):
                fn()
            torch.cuda.synchronize()
            times[name] = (time.perf_counter() - t0) / 5 * 1e3
            print(f"{name}: {times[name]:.2f} ms to the first new token's state")
        # reused layers are the sender's, bit for bit; recomputed ones are the receiver's own
        same = torch.equal(kv_mixed[0, :, :T].view(torch.int16), kv_sender[0, :, :T].view(torch.int16)) if lo > 0 else True
        fresh = not torch.equal(kv_mixed[lo, :, :T].view(torch.int16), kv_sender[lo, :, :T].view(torch.int16))
        finite = bool(torch.isfinite(out.float()).all())
        print(f"reused layer identical: {same}; recomputed layer differs from the sender's: {fresh}; output finite: {finite}")
        assert same and fresh and finite
        print("ok")
    finally:
        B.dsk_model_destroy(sender)
        B.dsk_model_destroy(receiver)
        B.dsk_store_destroy(store)


if __name__ == "__main__":
    main()
