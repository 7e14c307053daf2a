"""Seeded synthetic inputs (weights, hidden states, KV caches, ragged lengths).

This module holds no transformer arithmetic.  It only draws numbers, and it is the
single source of inputs for both the CPU oracle's tests and the HIP path's tests and
benchmark.  The HIP library carries its own implementation of the same counter-based
generator (needed to fill 137 GB of 70B-shaped weights on the device); a test checks
that the two agree bit for bit.

Generator ("ih8"): element `idx` of stream `stream` under `seed` is

    key = mix64(seed*G + stream*H + C)                       (all mod 2^64)
    a   = mix64(key + (2*idx)*G),  b = mix64(key + (2*idx+1)*G)
    s   = sum of the eight 16-bit lanes of a and b           (0 .. 524280)
    z   = s - 262140                                          (exact integer, mean 0)
    val = fl32(fl32(z) * scale) (+ offset, one more fp32 rounding, when offset != 0)

with mix64 the SplitMix64 output function, G its golden-ratio increment, and
scale = fl32(std / sqrt(8*(2^32-1)/12)) so that `val` has standard deviation `std`
(an Irwin-Hall sum of 8 uniforms: approximately normal, excess kurtosis -0.15, support
+-4.9 std).  Only integer operations and one or two IEEE fp32 roundings are involved, so
any two implementations agree exactly, with no dependence on a math library.
bf16 values are the fp32 values rounded to nearest-even on their upper 16 bits.
"""
from __future__ import annotations

import math
import os
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass

import numpy as np

_M64 = (1 << 64) - 1
_G = 0x9E3779B97F4A7C15
_H = 0xD1342543DE82EF95
_C = 0x632BE59BD9B4E019
_M1 = 0xBF58476D1CE4E5B9
_M2 = 0x94D049BB133111EB

LANE_MEAN_SUM = 262140  # 8 * 32767.5
LANE_SUM_STD = math.sqrt(8.0 * (2.0**32 - 1.0) / 12.0)

# tensor kinds inside one decoder layer; weight stream id = layer*16 + kind
G1, WQ, WK, WV, WO, G2, WG, WU, WD = range(9)
WR = 9  # router of a mixture-of-experts layer
TENSOR_NAMES = ("g1", "wq", "wk", "wv", "wo", "g2", "wg", "wu", "wd")
EXPERT_STREAM0 = 1 << 20  # expert tensors: stream EXPERT_STREAM0 + (layer*64 + expert)*4 + {0: wg, 1: wu, 2: wd}

# seed plan for the synthetic workloads
SEED_RECEIVER = 0
SEED_SENDER = 1
SEED_HIDDEN = 2
SEED_KV = 3
SEED_SUFFIX = 4
SEED_LENGTHS = 5


def _mix64_int(z: int) -> int:
    z &= _M64
    z = ((z ^ (z >> 30)) * _M1) & _M64
    z = ((z ^ (z >> 27)) * _M2) & _M64
    return z ^ (z >> 31)


def stream_key(seed: int, stream: int) -> int:
    return _mix64_int(seed * _G + stream * _H + _C)


def scale_for_std(std: float) -> np.float32:
    # std enters as an fp32 value (the C ABI takes a float), the division is done in double
    return np.float32(float(np.float32(std)) / LANE_SUM_STD)


def _mix64(z: np.ndarray) -> np.ndarray:
    z = (z ^ (z >> np.uint64(30))) * np.uint64(_M1)
    z = (z ^ (z >> np.uint64(27))) * np.uint64(_M2)
    return z ^ (z >> np.uint64(31))


def lane_sums(seed: int, stream: int, idx0: int, n: int) -> np.ndarray:
    """Centred integer lane sums z for elements idx0 .. idx0+n-1 (int32)."""
    key = np.uint64(stream_key(seed, stream))
    with np.errstate(over="ignore"):
        idx = np.arange(idx0, idx0 + n, dtype=np.uint64)
        c = key + (idx * np.uint64(2)) * np.uint64(_G)
        a = _mix64(c)
        b = _mix64(c + np.uint64(_G))
    s = a.view(np.uint16).reshape(n, 4).sum(axis=1, dtype=np.int32)
    s += b.view(np.uint16).reshape(n, 4).sum(axis=1, dtype=np.int32)
    return s - np.int32(LANE_MEAN_SUM)


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16, returned as uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (r >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _n_workers() -> int:
    return max(1, min(16, os.cpu_count() or 1))


def _generate(n: int, seed: int, stream: int, std: float, offset: float, idx0: int, bf16: bool,
              chunk: int = 1 << 20) -> np.ndarray:
    out = np.empty(n, dtype=np.float32)
    scale = scale_for_std(std)
    off = np.float32(offset)

    def work(s):
        m = min(chunk, n - s)
        v = lane_sums(seed, stream, idx0 + s, m).astype(np.float32) * scale
        if offset != 0.0:
            v = v + off
        if bf16:
            v = bf16_bits_to_f32(f32_to_bf16_bits(v))
        out[s:s + m] = v

    starts = range(0, n, chunk)
    if n <= 4 * chunk:
        for s in starts:
            work(s)
    else:  # numpy releases the GIL inside its loops, so plain threads scale
        with ThreadPoolExecutor(_n_workers()) as ex:
            list(ex.map(work, starts))
    return out


def normal_f32(n: int, seed: int, stream: int, std: float, offset: float = 0.0,
               idx0: int = 0, chunk: int = 1 << 20) -> np.ndarray:
    """n fp32 values offset + std*z of the ih8 generator, elements idx0.."""
    return _generate(n, seed, stream, std, offset, idx0, False, chunk)


def normal(n: int, seed: int, stream: int, std: float, offset: float = 0.0,
           dtype: str = "f32", idx0: int = 0) -> np.ndarray:
    """fp32 array of generated values; for dtype 'bf16' each value is bf16-representable."""
    if dtype not in ("f32", "bf16"):
        raise ValueError(dtype)
    return _generate(n, seed, stream, std, offset, idx0, dtype == "bf16")


@dataclass(frozen=True)
class ModelShape:
    """Llama-style decoder shape (names follow the usual notation: L, d, Hq, Hkv, dh, F)."""
    n_layers: int
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ffn: int
    rope_base: float
    rms_eps: float = 1e-5
    dtype: str = "bf16"  # "f32" or "bf16"
    n_experts: int = 0   # 0: dense MLP; E > 0: E expert MLPs of width F behind a router [E, d]
    top_k: int = 0       # experts per token

    def tensor_shape(self, kind: int) -> tuple:
        d, hq, hkv, dh, f = self.hidden, self.n_q_heads, self.n_kv_heads, self.head_dim, self.ffn
        return {
            G1: (d,), G2: (d,),
            WQ: (hq * dh, d), WK: (hkv * dh, d), WV: (hkv * dh, d),
            WO: (d, hq * dh), WG: (f, d), WU: (f, d), WD: (d, f), WR: (self.n_experts, d),
        }[kind]

    @property
    def kv_width(self) -> int:
        return self.n_kv_heads * self.head_dim

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == "f32" else 2


TINY = ModelShape(4, 256, 4, 2, 64, 688, 10000.0, 1e-5, "f32")
LLAMA_8B = ModelShape(32, 4096, 32, 8, 128, 14336, 500000.0, 1e-5, "bf16")
LLAMA_70B = ModelShape(80, 8192, 64, 8, 128, 28672, 500000.0, 1e-5, "bf16")
TINY_MOE = ModelShape(3, 256, 4, 2, 64, 320, 10000.0, 1e-5, "f32", 4, 2)
MIXTRAL_8X7B = ModelShape(32, 4096, 32, 8, 128, 14336, 1000000.0, 1e-5, "bf16", 8, 2)

WEIGHT_STD = 0.02


def weight_stream(layer: int, kind: int) -> int:
    return layer * 16 + kind


def layer_tensor(shape: ModelShape, seed: int, layer: int, kind: int) -> np.ndarray:
    """One weight tensor in its logical [out, in] row-major shape, as fp32 values.

    Projection matrices are N(0, 0.02); norm gains are 1 + N(0, 0.02)."""
    tshape = shape.tensor_shape(kind)
    n = int(np.prod(tshape))
    offset = 1.0 if kind in (G1, G2) else 0.0
    return normal(n, seed, weight_stream(layer, kind), WEIGHT_STD, offset, shape.dtype).reshape(tshape)


def expert_stream(layer: int, expert: int, kind: int) -> int:
    return EXPERT_STREAM0 + (layer * 64 + expert) * 4 + {WG: 0, WU: 1, WD: 2}[kind]


def expert_tensor(shape: ModelShape, seed: int, layer: int, expert: int, kind: int) -> np.ndarray:
    """WG, WU or WD of one expert of a mixture-of-experts layer, [out, in] row-major, N(0, 0.02)."""
    tshape = shape.tensor_shape(kind)
    return normal(int(np.prod(tshape)), seed, expert_stream(layer, expert, kind), WEIGHT_STD, 0.0,
                  shape.dtype).reshape(tshape)


def layer_weights(shape: ModelShape, seed: int, layer: int) -> dict:
    if shape.n_experts == 0:
        return {TENSOR_NAMES[k]: layer_tensor(shape, seed, layer, k) for k in range(9)}
    w = {TENSOR_NAMES[k]: layer_tensor(shape, seed, layer, k) for k in (G1, WQ, WK, WV, WO, G2)}
    w["router"] = layer_tensor(shape, seed, layer, WR)
    w["experts"] = [{TENSOR_NAMES[k]: expert_tensor(shape, seed, layer, e, k) for k in (WG, WU, WD)}
                    for e in range(shape.n_experts)]
    return w


def hidden_states(shape: ModelShape, n_tokens: int, seed: int = SEED_HIDDEN, stream: int = 0) -> np.ndarray:
    """[n_tokens, d] ~ N(0,1)."""
    return normal(n_tokens * shape.hidden, seed, stream, 1.0, 0.0, shape.dtype).reshape(n_tokens, shape.hidden)


def kv_cache(shape: ModelShape, n_rows: int, seed: int = SEED_KV) -> np.ndarray:
    """[L, 2, n_rows, Hkv, dh] ~ N(0,1); index 1 selects K (0) or V (1)."""
    out = np.empty((shape.n_layers, 2, n_rows, shape.n_kv_heads, shape.head_dim), dtype=np.float32)
    per = n_rows * shape.kv_width
    for l in range(shape.n_layers):
        for j in range(2):
            out[l, j] = normal(per, seed, l * 2 + j, 1.0, 0.0, shape.dtype).reshape(out.shape[2:])
    return out


def uniform_ints(n: int, lo: int, hi: int, seed: int, stream: int = 0) -> np.ndarray:
    """n integers uniform in [lo, hi] (inclusive) from the same counter generator."""
    key = np.uint64(stream_key(seed, stream))
    with np.errstate(over="ignore"):
        idx = np.arange(n, dtype=np.uint64)
        a = _mix64(key + (idx * np.uint64(2)) * np.uint64(_G))
    span = np.uint64(hi - lo + 1)
    return (lo + ((a >> np.uint64(11)) % span).astype(np.int64)).astype(np.int64)


def ragged_lengths(batch: int, lo: int, hi: int, seed: int = SEED_LENGTHS) -> np.ndarray:
    return uniform_ints(batch, lo, hi, seed, 0)


def cu_seqlens(lengths) -> np.ndarray:
    cu = np.zeros(len(lengths) + 1, dtype=np.int32)
    cu[1:] = np.cumsum(np.asarray(lengths, dtype=np.int64))
    return cu


def packed_positions(lengths, start=None) -> np.ndarray:
    """Positions start_i .. start_i+len_i-1 of every sequence, packed in order (int32)."""
    parts = []
    for i, n in enumerate(lengths):
        s0 = 0 if start is None else int(start[i])
        parts.append(np.arange(s0, s0 + int(n), dtype=np.int32))
    return np.concatenate(parts) if parts else np.zeros(0, dtype=np.int32)
