"""CPU oracle for selective-layer prefill (DroidSpeak, arxiv 2411.02820).

TEST INFRASTRUCTURE ONLY.  Nothing in the product path may import this file; it is used
by tests/, by __graft_entry__.smoke() and by the cpu_baseline leg of bench.py.  It shares
no code with the HIP library and imports nothing from it.

What it computes.  The paper's method (Sec. 4.1) changes *which* decoder layers run and
what is copied, never the layer arithmetic: a contiguous group of layers [lo, hi) is
recomputed over the whole context starting from the sender's E cache (the hidden state
entering layer lo, Sec. 2.1 "Query, Key, Value, and Embedding"), every other layer keeps
the sender's KV unchanged, and the first new tokens are then prefilled against that
mixed cache.  The result therefore has a plain definition - run the receiver's ordinary
Llama-style decoder layers - and this file is that definition written out in numpy,
float64 by default, one readable statement per step, no blocking or fusion.

The paper is silent on the layer itself ("same architecture"); the readings taken are:
pre-norm residual blocks, RMSNorm with eps inside the square root, half-split RoPE
pairing (i, i+dh/2) with theta_i = base^(-2i/dh), K cached after RoPE and V as projected,
contiguous GQA groups (kv head = q head // (Hq/Hkv)), softmax scale 1/sqrt(dh), SwiGLU
MLP, no biases.  For the mixture-of-experts receiver of Sec. 5.4 (Mixtral) the MLP is a
router over E expert SwiGLU MLPs: top-k experts by router logit, gate weights = softmax
over the chosen logits, ties to the lower expert index; attention and KV are unchanged.

Every function here is pinned by tests/test_oracle_*.py against something that is not
this file: hand-worked values, closed forms, invariants, an explicit T x T brute-force
attention, torch CPU library routines and an independent Llama implementation.

Layouts: hidden states [T, d]; K and V of a layer [rows, Hkv, dh]; weights in their
logical [out, in] shape; tokens of several sequences packed back to back, sequence b
owning rows cu_seqlens[b] .. cu_seqlens[b+1]-1, causal order = packed order.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np


@dataclass(frozen=True)
class Config:
    n_layers: int
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ffn: int
    rope_base: float
    rms_eps: float = 1e-5
    n_experts: int = 0  # 0: dense SwiGLU MLP; > 0: that many expert MLPs behind a router
    top_k: int = 0      # experts per token


def rmsnorm(x, g, eps):
    """y = x / sqrt(mean(x^2) + eps) * g over the last axis."""
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * g


def rope(x, positions, base):
    """Rotary embedding on x [T, H, dh]: pair (i, i+dh/2) is rotated by positions*base^(-2i/dh)."""
    dh = x.shape[-1]
    half = dh // 2
    theta = np.asarray(base, dtype=np.float64) ** (-2.0 * np.arange(half, dtype=np.float64) / dh)
    ang = np.asarray(positions, dtype=np.float64)[:, None] * theta[None, :]
    c = np.cos(ang)[:, None, :].astype(x.dtype)
    s = np.sin(ang)[:, None, :].astype(x.dtype)
    x1, x2 = x[..., :half], x[..., half:]
    return np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1)


def silu(z):
    return z / (1.0 + np.exp(-z))


def swiglu_mlp(y, wg, wu, wd):
    """(silu(y Wg^T) * (y Wu^T)) Wd^T for token rows y [n, d]."""
    return (silu(y @ wg.T) * (y @ wu.T)) @ wd.T


def moe_route(y, router, top_k):
    """Expert choice of every token (Sec. 5.4, the mixture-of-experts receiver; routing as in Mixtral).

    y [n, d] normalised hidden states, router [E, d].  Returns (logits [n, E], experts [n, top_k], gates
    [n, top_k]): the top_k experts of a token by router logit, highest first, equal logits going to the lower
    expert index, and the softmax of those top_k logits (the same numbers as a softmax over all E logits
    renormalised over the chosen ones)."""
    logits = y @ router.T
    n, E = logits.shape
    experts = np.empty((n, top_k), dtype=np.int64)
    gates = np.empty((n, top_k), dtype=logits.dtype)
    for i in range(n):
        order = sorted(range(E), key=lambda e: (-logits[i, e], e))[:top_k]
        chosen = logits[i, order]
        p = np.exp(chosen - chosen.max())
        experts[i] = order
        gates[i] = p / p.sum()
    return logits, experts, gates


def moe_mlp(y, router, experts_w, top_k):
    """Sparse mixture-of-experts MLP: every token goes through its top_k experts' SwiGLU MLPs and the results are
    added with the gate weights.  experts_w[e] = dict(wg, wu, wd) of expert e.  Returns [n, d].
    Written expert by expert (the tokens that chose expert e go through its MLP together), which is the same sum."""
    _, experts, gates = moe_route(y, router, top_k)
    out = np.zeros((y.shape[0], experts_w[0]["wd"].shape[0]), dtype=y.dtype)
    for e, ew in enumerate(experts_w):
        rows, place = np.nonzero(experts == e)  # a token lists an expert at most once: rows are distinct
        if len(rows):
            out[rows] += gates[rows, place][:, None] * swiglu_mlp(y[rows], ew["wg"], ew["wu"], ew["wd"])
    return out


def attend_row(q_t, K, V):
    """One query token against the keys it may see.

    q_t [Hq, dh]; K, V [n, Hkv, dh] are exactly the visible rows.  Query head a uses kv
    head a // (Hq/Hkv).  Returns [Hq, dh]."""
    Hq, dh = q_t.shape
    Hkv = K.shape[1]
    group = Hq // Hkv
    out = np.empty_like(q_t)
    for a in range(Hq):
        c = a // group
        s = K[:, c, :] @ q_t[a] / np.sqrt(dh)
        p = np.exp(s - s.max())
        p = p / p.sum()
        out[a] = p @ V[:, c, :]
    return out


def project_kv(cfg, w, h, positions):
    """K (after RoPE) and V of one layer for every token of h [T, d]."""
    T = h.shape[0]
    x = rmsnorm(h, w["g1"], cfg.rms_eps)
    k = (x @ w["wk"].T).reshape(T, cfg.n_kv_heads, cfg.head_dim)
    v = (x @ w["wv"].T).reshape(T, cfg.n_kv_heads, cfg.head_dim)
    return rope(k, positions, cfg.rope_base), v


def layer_rows(cfg, w, h_rows, pos_rows, visible):
    """Decoder layer output for a set of tokens whose visible K/V rows are given.

    h_rows [n, d] are the tokens' hidden states entering the layer, pos_rows their
    positions, visible(i) -> (K_i, V_i) the keys/values token i attends to (its own row
    included).  Returns the hidden states leaving the layer, [n, d]."""
    n = h_rows.shape[0]
    x = rmsnorm(h_rows, w["g1"], cfg.rms_eps)
    q = rope((x @ w["wq"].T).reshape(n, cfg.n_q_heads, cfg.head_dim), pos_rows, cfg.rope_base)
    attn = np.empty((n, cfg.n_q_heads * cfg.head_dim), dtype=h_rows.dtype)
    for i in range(n):
        K_i, V_i = visible(i)
        attn[i] = attend_row(q[i], K_i, V_i).reshape(-1)
    h1 = h_rows + attn @ w["wo"].T
    y = rmsnorm(h1, w["g2"], cfg.rms_eps)
    if "router" in w:
        return h1 + moe_mlp(y, w["router"], w["experts"], cfg.top_k)
    return h1 + swiglu_mlp(y, w["wg"], w["wu"], w["wd"])


def _seq_of_rows(cu_seqlens, T):
    seq = np.empty(T, dtype=np.int64)
    for b in range(len(cu_seqlens) - 1):
        seq[cu_seqlens[b]:cu_seqlens[b + 1]] = b
    return seq


def prefix_layer(cfg, w, h, positions, cu_seqlens, rows=None):
    """One decoder layer over packed prefix tokens h [T, d].

    Returns (h_next, K, V).  With rows given (sorted token indices), K and V are still
    computed for every token but h_next only for those rows (shape [len(rows), d])."""
    T = h.shape[0]
    K, V = project_kv(cfg, w, h, positions)
    seq = _seq_of_rows(cu_seqlens, T)
    sel = np.arange(T) if rows is None else np.asarray(rows, dtype=np.int64)

    def visible(i):
        t = sel[i]
        start = cu_seqlens[seq[t]]
        return K[start:t + 1], V[start:t + 1]

    h_next = layer_rows(cfg, w, h[sel], np.asarray(positions)[sel], visible)
    return h_next, K, V


def partial_prefill(cfg, weights, hidden_in, lo, hi, kv_reused, positions, cu_seqlens):
    """Selective-layer prefill (Sec. 4.1; the partial_prefill interface of Sec. 4.4).

    weights(l) -> dict of layer l's tensors; hidden_in [T, d] is the E cache at the
    transition layer lo; kv_reused[l] = (K, V) of the sender for every layer.
    Returns (kv_out, hidden_out): kv_out[l] is the fresh (K, V) for lo <= l < hi and the
    very same arrays as kv_reused[l] otherwise; hidden_out is the state leaving layer hi-1
    (hidden_in itself when lo == hi)."""
    if not (0 <= lo <= hi <= cfg.n_layers):
        raise ValueError("need 0 <= lo <= hi <= n_layers")
    kv_out = [kv_reused[l] for l in range(cfg.n_layers)]
    h = hidden_in
    for l in range(lo, hi):
        h, K, V = prefix_layer(cfg, weights(l), h, positions, cu_seqlens)
        kv_out[l] = (K, V)
    return kv_out, h


def partial_prefill_groups(cfg, weights, groups, kv_reused, positions, cu_seqlens):
    """Selective-layer prefill with several recomputed layer groups (Sec. 4.1, "critical
    layer groups": the layers worth recomputing need not be one contiguous run).

    groups: list of (lo, hi, hidden_in), ascending and disjoint; each group restarts from
    the sender's E cache at its own transition layer lo, exactly as a single group does,
    and what a group leaves in the residual stream is discarded.  Layers outside every
    group keep the sender's KV.  Returns (kv_out, [hidden_out of each group])."""
    prev_hi = 0
    for lo, hi, _ in groups:
        if not (prev_hi <= lo <= hi <= cfg.n_layers):
            raise ValueError("groups must be ascending, disjoint and inside [0, n_layers]")
        prev_hi = hi
    kv_out = [kv_reused[l] for l in range(cfg.n_layers)]
    hidden_outs = []
    for lo, hi, hidden_in in groups:
        h = hidden_in
        for l in range(lo, hi):
            h, K, V = prefix_layer(cfg, weights(l), h, positions, cu_seqlens)
            kv_out[l] = (K, V)
        hidden_outs.append(h)
    return kv_out, hidden_outs


def suffix_prefill(cfg, weights, suffix_hidden_in, kv, suffix_positions, cu_prefix, cu_suffix):
    """Prefill of the new tokens against the mixed cache, through all layers (Sec. 4.1:
    in a layer whose KV is reused only the new tokens' states flow).

    suffix_hidden_in [S_total, d]; kv[l] = (K, V) holding the prefix rows of every
    sequence (packed by cu_prefix); suffix token j of sequence b sees that sequence's
    prefix rows and suffix rows 0..j.  Returns (kv_suffix, hidden_out) with
    kv_suffix[l] = (K, V) of the suffix tokens, [S_total, Hkv, dh]."""
    S = suffix_hidden_in.shape[0]
    seq = _seq_of_rows(cu_suffix, S)
    h = suffix_hidden_in
    kv_suffix = []
    for l in range(cfg.n_layers):
        w = weights(l)
        Kp, Vp = kv[l]
        Ks, Vs = project_kv(cfg, w, h, suffix_positions)

        def visible(j, Kp=Kp, Vp=Vp, Ks=Ks, Vs=Vs):
            b = seq[j]
            p0, p1, s0 = cu_prefix[b], cu_prefix[b + 1], cu_suffix[b]
            return (np.concatenate([Kp[p0:p1], Ks[s0:j + 1]]).astype(h.dtype),
                    np.concatenate([Vp[p0:p1], Vs[s0:j + 1]]).astype(h.dtype))

        h = layer_rows(cfg, w, h, suffix_positions, visible)
        kv_suffix.append((Ks, Vs))
    return kv_suffix, h


def max_rel_err(got, ref):
    """max|got - ref| / max|ref| over a tensor: the error measure of the parity tests."""
    ref = np.asarray(ref, dtype=np.float64)
    got = np.asarray(got, dtype=np.float64)
    denom = np.max(np.abs(ref))
    if denom == 0.0:
        return float(np.max(np.abs(got)))
    return float(np.max(np.abs(got - ref)) / denom)
