"""Shared test helpers: glue between the seeded input generator and the oracle.

No arithmetic of the method lives here; only shape conversion and config mapping."""
import numpy as np

from oracle import dsk_oracle as O
from paper_2411_02820_amd import synth


def oracle_config(shape: synth.ModelShape) -> O.Config:
    return O.Config(shape.n_layers, shape.hidden, shape.n_q_heads, shape.n_kv_heads,
                    shape.head_dim, shape.ffn, shape.rope_base, shape.rms_eps, shape.n_experts, shape.top_k)


def weights_fn(shape: synth.ModelShape, seed: int, dtype=np.float64, cache=None):
    """Callable l -> dict of layer tensors as `dtype` arrays, generated from the seed."""
    cache = {} if cache is None else cache

    def get(l):
        if l not in cache:
            w = synth.layer_weights(shape, seed, l)
            cache[l] = {k: v.astype(dtype) for k, v in w.items() if k != "experts"}
            if "experts" in w:
                cache[l]["experts"] = [{k: v.astype(dtype) for k, v in e.items()} for e in w["experts"]]
        return cache[l]
    return get


def kv_list(kv: np.ndarray, dtype=np.float64):
    """[L, 2, rows, Hkv, dh] array -> list of (K, V)."""
    return [(kv[l, 0].astype(dtype), kv[l, 1].astype(dtype)) for l in range(kv.shape[0])]
