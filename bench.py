#!/usr/bin/env python3
"""Benchmark of the selective-layer prefill hot path on one MI355X.

One step = one pass of the whole path on one batch: dsk_partial_prefill (recompute layers [lo,hi)
from the sender's E cache while the other layers' KV is spliced in on the side stream) followed by
dsk_suffix_prefill (the new tokens through all layers against the mixed cache).  Inputs are
synthetic and resident in HBM before the timed region.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload 8b-8k|8b-4k|8b-ragged|8b-16k-hostkv|8b-32k|70b-8k|mixtral-8k|tiny]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0  # MI355X dense bf16 MFMA

WORKLOADS = {
    # name: (shape name, prefix lengths (None: seeded ragged batch), lo, hi, suffix tokens per sequence, KV/E in pinned host memory)
    "8b-8k": ("LLAMA_8B", [8192], 8, 16, 64, False),         # the point the headline metric is quoted on
    "8b-4k": ("LLAMA_8B", [4096], 8, 16, 64, False),         # workload 2
    "8b-ragged": ("LLAMA_8B", None, None, None, 128, False),  # workload 3: 8 prefixes U[1024,8192], 4 layers
    "8b-16k-hostkv": ("LLAMA_8B", [16384], 4, 12, 64, True),  # workload 4: reused KV + E cache in pinned host memory
    "70b-8k": ("LLAMA_70B", [8192], 20, 36, 64, False),      # workload 5
    "tiny": ("TINY", [128], 1, 3, 16, False),                # workload 1
    "8b-32k": ("LLAMA_8B", [32768], 8, 16, 64, False),       # the long end of the paper's contexts (App. A: P95 about 30k)
    "mixtral-8k": ("MIXTRAL_8X7B", [8192], 8, 16, 64, False),  # the mixture-of-experts receiver of Sec. 5.4
}


def recompute_flops(shape, lens, n_layers):
    """Algorithmic flops of recomputing n_layers over the packed prefixes (MAC = 2, attention causal)."""
    d, hq, hkv, dh, f = shape.hidden, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.ffn
    mlps = shape.top_k if shape.n_experts else 1  # expert MLPs a token goes through (+ the router)
    gemm = 2.0 * sum(lens) * (d * (hq + 2 * hkv) * dh + hq * dh * d + mlps * 3 * d * f + d * shape.n_experts)
    attn = sum(2.0 * hq * dh * t * (t + 1) for t in lens)
    return n_layers * (gemm + attn)


def kernel_source_sha256(name="gemm_mfma.hip"):
    import hashlib
    with open(os.path.join(ROOT, "paper_2411_02820_amd", "csrc", name), "rb") as f:
        return hashlib.sha256(f.read()).hexdigest()


def measured_traffic(workload):
    """Fabric-side bytes per launch of the dominant kernel, from the committed rocprofv3 --pmc summary (FETCH_SIZE
    and WRITE_SIZE runs scaled by a known-size copy).  The counters cannot be read from inside this process, so the
    figure belongs to the kernel source the profile was taken with: the summary records that file's SHA-256, and a
    figure whose hash is not the current source's is dropped (None), as is a workload with no summary."""
    path = os.path.join(ROOT, "profiles", f"bench_{workload}_gemm_pmc_traffic.txt")
    try:
        fields = dict(line.split()[:2] for line in open(path) if line[:1].isalpha() and len(line.split()) >= 2)
    except OSError:
        return None
    if fields.get("kernel_source_sha256") != kernel_source_sha256():
        return None
    return float(fields["traffic_bytes_per_launch"]) if "traffic_bytes_per_launch" in fields else None


PHASE_TIMES = {}


def time_region(torch, fn, reps, name=None):
    """Mean duration of fn in ms over reps back-to-back calls (HIP events on the current stream); with a name,
    the per-call median and minimum are kept for the output line as well."""
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(reps + 1)]
    torch.cuda.synchronize()
    ev[0].record()
    for i in range(reps):
        fn()
        ev[i + 1].record()
    torch.cuda.synchronize()
    if name:
        each = sorted(ev[i].elapsed_time(ev[i + 1]) for i in range(reps))
        PHASE_TIMES[name] = {"median_ms": round(each[len(each) // 2], 3), "min_ms": round(each[0], 3), "reps": reps}
    return ev[0].elapsed_time(ev[reps]) / reps


def cpu_baseline(shape, lens, lo, hi):
    """The oracle, as it stands, on a bounded sample of the workload itself: ONE decoder layer over the workload's
    own packed prefixes, with K and V projected for every token and the rest of the layer (attention over all
    earlier tokens of the sequence, MLP) for token rows taken at a fixed stride through the batch, the last row
    included, so that short and long attention spans appear in their true proportion.  The layer's time is the K/V
    time plus the sampled rows' time scaled to all rows; tokens/s = tokens / (that time x (hi - lo) layers)."""
    import numpy as np
    from oracle import dsk_oracle as O
    from paper_2411_02820_amd import synth
    T = sum(lens)
    n_rows = min(T, 768 if shape.hidden <= 4096 else 256)   # about 10-30 s of host work
    rows = sorted(set(int(r) for r in np.linspace(0, T - 1, n_rows).round()))
    cfg = O.Config(shape.n_layers, shape.hidden, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.ffn,
                   shape.rope_base, shape.rms_eps, shape.n_experts, shape.top_k)
    w = synth.layer_weights(shape, synth.SEED_RECEIVER, lo)
    w = {k: ([{n: t.astype(np.float64) for n, t in e.items()} for e in v] if k == "experts" else v.astype(np.float64))
         for k, v in w.items()}
    x = synth.hidden_states(shape, T).astype(np.float64)
    pos, cu = synth.packed_positions(lens), synth.cu_seqlens(lens)
    t0 = time.perf_counter()
    O.project_kv(cfg, w, x, pos)
    t_kv = time.perf_counter() - t0
    t0 = time.perf_counter()
    O.prefix_layer(cfg, w, x, pos, cu, rows=rows)   # projects K/V again, then the sampled rows
    t_rows = max(time.perf_counter() - t0 - t_kv, 1e-9)
    t_layer = t_kv + t_rows * T / len(rows)
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    return {"value": T / (t_layer * (hi - lo)), "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"fp64 numpy oracle, one {shape.hidden}-wide decoder layer over the workload's {T} prefix tokens: K/V of all "
                      f"rows {t_kv:.2f} s, attention + MLP of {len(rows)} rows at a fixed stride {t_rows:.2f} s, scaled to all rows "
                      f"-> {t_layer:.1f} s per layer, x {hi - lo} layers; cores = BLAS threads (the per-row attention loop is "
                      f"sequential Python around BLAS calls)"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="8b-8k", choices=sorted(WORKLOADS))
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-full-prefill", action="store_true")
    ap.add_argument("--load-sweep", action="store_true",
                    help="host-KV workloads: time the three loading strategies over emulated links of several rates")
    ap.add_argument("--fit-latency", action="store_true",
                    help="profile partial-prefill delay over token counts and recompute depths, fit the App. B latency model "
                         "and show the configuration the policy picks for a synthetic frontier at several SLOs")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="also run one plain 1 GiB device copy, the known-size kernel that scales FETCH_SIZE/WRITE_SIZE")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (no sharding or collectives); use --gpus 1")

    import torch
    from paper_2411_02820_amd import binding as B
    from paper_2411_02820_amd import synth

    shape_name, lens, lo, hi, S1, host_kv = WORKLOADS[args.workload]
    shape = getattr(synth, shape_name)
    L = shape.n_layers
    if lens is None:  # workload 3: seeded ragged batch and start layer
        lens = [int(x) for x in synth.ragged_lengths(8, 1024, 8192)]
        lo = int(synth.uniform_ints(1, 0, 28, synth.SEED_LENGTHS, 1)[0])
        hi = lo + 4
    slens = [S1] * len(lens)
    T, S = sum(lens), sum(slens)
    tdt = torch.float32 if shape.dtype == "f32" else torch.bfloat16
    code = B.DSK_F32 if shape.dtype == "f32" else B.DSK_BF16
    dev = "cuda"
    cfg = B.config_from_shape(shape)
    rows = T + S

    def new_cache(n_rows=rows):
        return torch.empty((L, 2, n_rows, shape.n_kv_heads, shape.head_dim), dtype=tdt, device=dev)

    prefix = B.Batch(synth.cu_seqlens(lens), synth.packed_positions(lens))
    suffix = B.Batch(synth.cu_seqlens(slens), synth.packed_positions(slens, start=lens))
    hidden_in = torch.empty((T, shape.hidden), dtype=tdt, device=dev)
    kv_sender = new_cache(T)

    # ---- sender (seed 1): its KV for all layers and its hidden state entering layer lo (Sec. 4.1) ----
    sender_fits = shape.hidden <= 4096
    if sender_fits:
        sender = B.dsk_model_create(cfg, T, T)
        B.dsk_model_init_random(sender, synth.SEED_SENDER, synth.WEIGHT_STD)
        x0 = torch.empty((T, shape.hidden), dtype=tdt, device=dev)
        B.dsk_fill_normal(x0, x0.numel(), synth.SEED_HIDDEN, 0, 1.0, 0.0, 0, code)
        B.dsk_partial_prefill(sender, x0, 0, L, None, B.kv_desc(kv_sender), prefix.desc, None)
        if lo > 0:
            # layers [0, lo) again, in place (the path is deterministic), to obtain the state entering layer lo
            B.dsk_partial_prefill(sender, x0, 0, lo, B.kv_desc(kv_sender), B.kv_desc(kv_sender), prefix.desc, hidden_in)
        else:
            hidden_in.copy_(x0)
        torch.cuda.synchronize()
        B.dsk_model_destroy(sender)
        del x0
        data = "synthetic: random-init receiver (seed 0); reused KV and E cache from a random-init sender (seed 1) prefill"
    else:  # two 137 GB models do not fit: N(0,1) tensors stand in for the sender's caches
        B.dsk_fill_normal(hidden_in, hidden_in.numel(), synth.SEED_HIDDEN, 0, 1.0, 0.0, 0, code)
        B.dsk_fill_normal(kv_sender, kv_sender.numel(), synth.SEED_KV, 0, 1.0, 0.0, 0, code)
        data = "synthetic: random-init receiver (seed 0); reused KV and E cache ~N(0,1)"
    torch.cuda.empty_cache()

    model = B.dsk_model_create(cfg, T, rows)
    B.dsk_model_init_random(model, synth.SEED_RECEIVER, synth.WEIGHT_STD)
    weights_gb = B.dsk_model_weight_bytes(model) / 1e9
    kv_out = new_cache()
    xs = torch.empty((S, shape.hidden), dtype=tdt, device=dev)
    B.dsk_fill_normal(xs, xs.numel(), synth.SEED_SUFFIX, 0, 1.0, 0.0, 0, code)
    hs_out = torch.empty_like(xs)
    kv_dev_desc = B.kv_desc(kv_sender)
    hidden_dev = hidden_in
    if host_kv:  # workload 4: the sender's KV and E cache wait in pinned host memory
        kv_host = torch.empty(kv_sender.shape, dtype=tdt, pin_memory=True)
        kv_host.copy_(kv_sender)
        e_host = torch.empty(hidden_in.shape, dtype=tdt, pin_memory=True)
        e_host.copy_(hidden_in)
        torch.cuda.synchronize()
        kv_r, hidden_in = B.kv_desc(kv_host), e_host
        data += "; reused KV and E cache staged in pinned host memory (loads timed, PCIe-inclusive)"
    else:
        kv_r = kv_dev_desc
    kv_o = B.kv_desc(kv_out)
    kv_out.fill_(float("nan"))
    torch.cuda.synchronize()

    def partial(a=lo, b=hi):
        B.dsk_partial_prefill(model, hidden_in, a, b, kv_r, kv_o, prefix.desc, None, B.DSK_DEFER_JOIN)

    def suffix_pass():
        B.dsk_suffix_prefill(model, xs, kv_o, prefix.desc, suffix.desc, T, hs_out)

    def step():
        partial()
        suffix_pass()

    if args.pmc_calibration:
        cal_src = torch.empty(1 << 28, dtype=torch.float32, device=dev)
        cal_src.fill_(1.0)
        cal_dst = torch.empty_like(cal_src)
        cal_dst.copy_(cal_src)  # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del cal_src, cal_dst

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    # ---- timed region: exactly K steps; the library brackets its prefill GEMM launches with HIP events ----
    B.dsk_set_option("reset_stats", 0)
    B.dsk_set_option("time_gemm", 1)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    B.dsk_set_option("time_gemm", 0)
    ms_per_step = wall * 1e3 / args.steps
    gemm_ms = B.dsk_get_stat("timed_gemm_ms")
    gemm_n = B.dsk_get_stat("timed_gemm_launches")
    gemm_flops = B.dsk_get_stat("timed_gemm_flops")
    attn_ms, attn_n, attn_flops = (B.dsk_get_stat("timed_attn_" + k) for k in ("ms", "launches", "flops"))

    # ---- phase split, full-prefill comparison (outside the timed region) ----
    def partial_joined():
        partial()
        B.dsk_join_loads(model)
    t_partial = time_region(torch, partial_joined, max(2, args.steps // 2), "partial_prefill")
    t_suffix = time_region(torch, suffix_pass, max(2, args.steps // 2), "suffix_prefill")
    # the timed steps really wrote the cache: a reused layer is the sender's, bit for bit, in a cache that was
    # filled with NaN before the first step
    chk = lo - 1 if lo > 0 else (hi if hi < L else None)
    splice_ok = None if chk is None else bool(torch.equal(kv_out[chk, :, :T].view(torch.int16 if tdt == torch.bfloat16 else torch.int32),
                                                            kv_sender[chk, :, :T].view(torch.int16 if tdt == torch.bfloat16 else torch.int32)))
    extra = {}
    if not args.no_full_prefill:
        def full():
            B.dsk_partial_prefill(model, hidden_in, 0, L, None, kv_o, prefix.desc, None, 0)
        full()
        t_full = time_region(torch, full, 2, "full_prefill")
        extra["full_prefill_ms"] = round(t_full, 3)
        extra["speedup_vs_full_prefill"] = round((t_full + t_suffix) / (t_partial + t_suffix), 3)
        extra["full_prefill_tokens_per_s"] = round(T / (t_full / 1e3), 1)
    if host_kv:
        # overlap of the per-layer loads with the recompute: device-resident inputs, sequential (load, then
        # compute) and pipelined runs of the same call
        def run_mode(mode, kv_desc, e):
            B.dsk_set_load_mode(model, mode)
            def f():
                B.dsk_partial_prefill(model, e, lo, hi, kv_desc, kv_o, prefix.desc, None, 0)
            f()
            return time_region(torch, f, 3)
        t_dev = run_mode(B.DSK_LOAD_PIPELINED, kv_dev_desc, hidden_dev)
        t_seq = run_mode(B.DSK_LOAD_REUSED_FIRST, kv_r, hidden_in)
        t_pipe = run_mode(B.DSK_LOAD_PIPELINED, kv_r, hidden_in)
        load_ms = max(t_seq - t_dev, 1e-6)
        reused_bytes = (L - (hi - lo)) * 2 * T * shape.kv_width * shape.elem_bytes + T * shape.hidden * shape.elem_bytes
        extra["host_kv"] = {"partial_ms_device_resident": round(t_dev, 3), "partial_ms_load_then_compute": round(t_seq, 3),
                            "partial_ms_pipelined": round(t_pipe, 3), "exposed_load_ms": round(t_pipe - t_dev, 3),
                            "overlap_efficiency": round(1.0 - (t_pipe - t_dev) / load_ms, 4),
                            "h2d_gb_per_s": round(reused_bytes / (load_ms * 1e-3) / 1e9, 1),
                            "loaded_bytes": int(reused_bytes)}
        if args.load_sweep:
            # Sec. 4.3 Fig. 13 / Sec. 5.5 Fig. 20 on this machine: prefill delay (selective prefill of the prefix, joined)
            # of the three strategies against the link rate; 0 = the native host link.  "model" is the unit-cost
            # schedule of Fig. 13 fed with this run's per-layer recompute time and the layer/E-cache bytes at that rate.
            layer_bytes = 2 * T * shape.kv_width * shape.elem_bytes
            e_bytes = T * shape.hidden * shape.elem_bytes
            t_layer = t_dev / (hi - lo)
            native = reused_bytes / (load_ms * 1e-3) / 1e9
            sweep = []
            for gbps in (2.0, 5.0, 10.0, 20.0, 0.0):
                B.dsk_set_load_throttle(model, gbps)
                rate = (gbps if gbps > 0 else native) * 1e9
                tl, te = layer_bytes / rate * 1e3, e_bytes / rate * 1e3
                n_reused = L - (hi - lo)
                row = {"link_gb_per_s": gbps if gbps > 0 else round(native, 1)}
                for name, mode, model_ms in (
                        ("all_then_compute", B.DSK_LOAD_ALL_FIRST, te + L * tl + (hi - lo) * t_layer),
                        ("reused_then_compute", B.DSK_LOAD_REUSED_FIRST, te + n_reused * tl + (hi - lo) * t_layer),
                        ("pipelined", B.DSK_LOAD_PIPELINED, max(te + n_reused * tl, te + (hi - lo) * t_layer))):
                    row[name + "_ms"] = round(run_mode(mode, kv_r, hidden_in), 2)
                    row[name + "_model_ms"] = round(model_ms, 2)
                sweep.append(row)
            B.dsk_set_load_throttle(model, 0.0)
            B.dsk_set_load_mode(model, B.DSK_LOAD_PIPELINED)
            extra["load_sweep"] = sweep
    if args.fit_latency and len(lens) == 1:
        # App. B takes the estimate's parameters from the profiling phase.  Profile the joined
        # selective prefill at three token counts x three depths, least-squares fit of
        # t = c0 + R (c1 T + c2 T^2) + (L - R) c3 T, then ask the library's policy for a synthetic frontier.
        from paper_2411_02820_amd.latency_fit import fit_latency_model
        points = []
        for Tn in (T // 4, T // 2, T):
            pb = B.Batch(synth.cu_seqlens([Tn]), synth.packed_positions([Tn]))
            for R in sorted({min(2, L), min(4, L), min(8, L)}):
                a = min(lo, L - R)
                def f():
                    B.dsk_partial_prefill(model, hidden_in, a, a + R, kv_r, kv_o, pb.desc, None, 0)
                f()
                points.append((Tn, R, time_region(torch, f, 2)))
        lat, resid = fit_latency_model(points, L)
        t_fit = points
        frontier = [(lo, min(lo + r, L), q) for r, q in ((0, 0.30), (2, 0.55), (4, 0.70), (8, 0.78))] + [(0, L, 0.82)]
        full_ms = B.dsk_estimate_prefill_ms(lat, L, L, T)
        picks = []
        for frac in (0.05, 0.15, 0.3, 0.6, 1.1):
            i = B.dsk_select_recompute(frontier, L, T, lat, frac * full_ms, 0.7, 0)
            picks.append({"slo_ms": round(frac * full_ms, 2), "recompute": list(frontier[i][:2]),
                          "estimate_ms": round(B.dsk_estimate_prefill_ms(lat, L, frontier[i][1] - frontier[i][0], T), 2)})
        i_busy = B.dsk_select_recompute(frontier, L, T, lat, full_ms, 0.7, 4)
        extra["latency_model"] = {"c0_ms": lat[0], "c_layer_token_ms": lat[1], "c_layer_token2_ms": lat[2],
                                  "c_reused_token_ms": lat[3], "max_rel_residual": round(resid, 4),
                                  "points": len(t_fit), "policy_idle": picks,
                                  "policy_4_waiting_target_0.7": list(frontier[i_busy][:2]),
                                  "frontier": "synthetic (quality values are placeholders)"}
    flops = recompute_flops(shape, lens, hi - lo)
    # what the matrix cores of this machine sustain in a register-only loop (bf16), right after the measurements
    from paper_2411_02820_amd import diag
    peak_measured = diag.dsk_diag_mfma_peak()
    extra.update({
        "partial_prefill_ms": round(t_partial, 3), "suffix_prefill_ms": round(t_suffix, 3),
        "ttft_ms": round(t_partial + t_suffix, 3), "phase_timing": PHASE_TIMES,
        "reused_layer_bit_exact_after_timed_steps": splice_ok,
        "recompute_tflops_algorithmic": round(flops / 1e12, 2),
        "mfma_util_recompute_phase": round(flops / (t_partial * 1e-3) / (PEAK_BF16_TFLOPS * 1e12), 4),
        "mfma_peak_measured_tflops": round(peak_measured, 1),
        "mfma_util_recompute_phase_vs_measured_peak": round(flops / (t_partial * 1e-3) / (peak_measured * 1e12), 4),
        "reused_kv_bytes": int((L - (hi - lo)) * 2 * T * shape.kv_width * shape.elem_bytes),
        "weights_gb": round(weights_gb, 2),
        "kernel_launch_mix": {k: int(B.dsk_get_stat(k)) for k in
                              ("gemm_mfma_launches", "gemm_generic_launches", "attn_mfma_launches", "attn_generic_launches")},
    })

    out = {
        "metric": "selective_prefill_tokens_per_s", "value": round(T / (ms_per_step / 1e3), 1), "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 3),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if shape.dtype == "bf16" else "f32", "data": data,
        "config": {"workload": f"{shape_name} shape, {len(lens)} prefix(es) of {lens if len(lens) > 1 else lens[0]} tokens, "
                               f"recompute layers [{lo},{hi}) of {L}, suffix {S1} tokens per sequence; "
                               f"step = dsk_partial_prefill + dsk_suffix_prefill",
                   "prefix_tokens": T, "lo": lo, "hi": hi, "suffix_tokens": S},
    }
    if shape.dtype == "bf16" and gemm_n > 0:
        achieved = gemm_flops / (gemm_ms * 1e-3) / 1e12
        out["roofline"] = {"bound": "mfma", "achieved": round(achieved, 1), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                           "frac": round(achieved / PEAK_BF16_TFLOPS, 4), "traffic": measured_traffic(args.workload),
                           "traffic_unit": "bytes per launch (L2<->fabric reads + writes, rocprofv3 --pmc, see profiles/)",
                           "kernel": "gemm16_bf16_kernel<256,256,2,4> (prefill GEMMs: QKV, O, gate/up, down"
                                     + ("; the expert projections are its grouped instantiation, one launch over all experts)" if shape.n_experts else ")"),
                           "launches": int(gemm_n), "avg_launch_ms": round(gemm_ms / gemm_n, 4),
                           "flops_per_launch": round(gemm_flops / gemm_n / 1e9, 1), "flops_unit": "GFLOP"}
    else:
        out["roofline"] = {"bound": "alu", "achieved": round(flops / (t_partial * 1e-3) / 1e12, 3), "peak": 157.3,
                           "unit": "TFLOP/s", "frac": round(flops / (t_partial * 1e-3) / 157.3e12, 5), "traffic": None,
                           "kernel": "fp32 plain-ALU path (latency bound at this size)"}
    if shape.dtype == "bf16" and attn_n > 0:
        a_tf = attn_flops / (attn_ms * 1e-3) / 1e12
        out["roofline_attention"] = {"bound": "mfma", "achieved": round(a_tf, 1), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                                     "frac": round(a_tf / PEAK_BF16_TFLOPS, 4), "traffic": None,
                                     "kernel": "attn_bf16_kernel<128,false,4> (causal attention over the prefix; HIP events in the timed steps)",
                                     "launches": int(attn_n), "avg_launch_ms": round(attn_ms / attn_n, 4),
                                     "flops_per_launch": round(attn_flops / attn_n / 1e9, 1), "flops_unit": "GFLOP (causal)"}
    # The suffix pass streams every weight once and reads the prefix K/V of every layer: HBM-bound (few rows).
    kv_layer_bytes = 2 * T * shape.kv_width * shape.elem_bytes
    suffix_bytes = B.dsk_model_weight_bytes(model) + L * kv_layer_bytes
    out["roofline_suffix"] = {"bound": "hbm", "achieved": round(suffix_bytes / (t_suffix * 1e-3) / 1e9, 1), "peak": 8000.0,
                              "unit": "GB/s", "frac": round(suffix_bytes / (t_suffix * 1e-3) / 8e12, 4), "traffic": None,
                              "kernel": "dsk_suffix_prefill as a whole (all launches of the pass; HIP events on its stream)",
                              "algorithmic_bytes": int(suffix_bytes), "ms": round(t_suffix, 3),
                              "bytes_are": "all weights once + prefix K/V of every layer once"}
    # The splice / load of the reused layers: device-resident caches are copied HBM to HBM (every byte read and
    # written), host-resident ones cross the host link.
    def pure_splice():
        B.dsk_partial_prefill(model, hidden_in, lo, lo, kv_r, kv_o, prefix.desc, None, 0)
    pure_splice()
    t_splice = time_region(torch, pure_splice, 3)
    moved = L * kv_layer_bytes + (T * shape.hidden * shape.elem_bytes if host_kv else 0)
    if host_kv:
        out["roofline_load"] = {"bound": "pcie", "achieved": round(moved / (t_splice * 1e-3) / 1e9, 1), "peak": 64.0,
                                "unit": "GB/s", "frac": round(moved / (t_splice * 1e-3) / 64e9, 4), "traffic": None,
                                "kernel": "hipMemcpyAsync host to device, all layers + E cache, nothing else running",
                                "algorithmic_bytes": int(moved), "ms": round(t_splice, 3),
                                "peak_is": "PCIe Gen5 x16, one direction"}
    else:
        out["roofline_load"] = {"bound": "hbm", "achieved": round(2 * moved / (t_splice * 1e-3) / 1e9, 1), "peak": 8000.0,
                                "unit": "GB/s", "frac": round(2 * moved / (t_splice * 1e-3) / 8e12, 4), "traffic": None,
                                "kernel": "hipMemcpyAsync device to device, all layers, nothing else running",
                                "algorithmic_bytes": int(2 * moved), "ms": round(t_splice, 3),
                                "bytes_are": "every spliced byte read once and written once"}
    out.update(extra)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(shape, lens, lo, hi)
    B.dsk_model_destroy(model)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
