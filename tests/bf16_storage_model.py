"""What the bf16 number format alone costs: the oracle's decoder layer with every tensor that a bf16 data path has to
store as a matrix-core operand rounded to bf16 (round to nearest even), all arithmetic still in fp64.

Test infrastructure.  It implements no kernel's blocking or order of summation: it answers the question "how far from
the fp64 oracle does ANY implementation land that feeds bf16 operands to its GEMMs", which is what bounds the parity of
a deep recomputed group (the errors of successive layers add).  Rounded, because they are GEMM / attention operands:
the normalised activations, the projected q, k, v (k and q again after the rotation, as a cache in bf16 holds them),
the attention probabilities, the attention output, the SwiGLU output.  Not rounded: the residual stream (the library
keeps it in fp32 between the layers of a call), sums and softmax statistics.

With rounding switched off the function is the oracle's prefix_layer (tests/test_bf16_storage_model.py pins that).
"""
import numpy as np

from oracle import dsk_oracle as O
from paper_2411_02820_amd import synth


def to_bf16(x):
    return synth.bf16_bits_to_f32(synth.f32_to_bf16_bits(np.asarray(x, dtype=np.float32))).astype(np.float64)


def prefix_layer(cfg, w, h, positions, cu_seqlens, rounded=True):
    """One decoder layer over packed prefix tokens h [T, d] (fp64).  Returns (h_next, K, V) like the oracle."""
    R = to_bf16 if rounded else (lambda x: x)
    T = h.shape[0]
    Hq, Hkv, dh = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    x = R(O.rmsnorm(h, w["g1"], cfg.rms_eps))
    q = R(O.rope(R(x @ w["wq"].T).reshape(T, Hq, dh), positions, cfg.rope_base))
    k = R(O.rope(R(x @ w["wk"].T).reshape(T, Hkv, dh), positions, cfg.rope_base))
    v = R(x @ w["wv"].T).reshape(T, Hkv, dh)
    attn = np.zeros((T, Hq, dh))
    for b in range(len(cu_seqlens) - 1):
        s0, s1 = int(cu_seqlens[b]), int(cu_seqlens[b + 1])
        n = s1 - s0
        causal = np.tril(np.ones((n, n), dtype=bool))
        for a in range(Hq):
            c = a // (Hq // Hkv)
            s = q[s0:s1, a, :] @ k[s0:s1, c, :].T / np.sqrt(dh)
            s = np.where(causal, s, -np.inf)
            p = np.exp(s - s.max(axis=1, keepdims=True))
            den = p.sum(axis=1, keepdims=True)
            attn[s0:s1, a, :] = (R(p) @ v[s0:s1, c, :]) / den
    h1 = h + R(attn.reshape(T, Hq * dh)) @ w["wo"].T
    y = R(O.rmsnorm(h1, w["g2"], cfg.rms_eps))
    act = R(O.silu(y @ w["wg"].T) * (y @ w["wu"].T))
    return h1 + act @ w["wd"].T, k, v
