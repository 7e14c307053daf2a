"""ctypes binding of libdsk.so: the same entry points as include/dsk.h, argument marshalling only.

Every step of the path runs inside the library's HIP kernels.  There is no fallback: if the
shared library has not been built, importing this module raises.  torch is used by callers
for device memory and streams; this file only turns tensors into raw pointers.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
# PyTorch first: it brings its own copy of the HIP runtime, and the process must end up with ONE runtime.  Loaded
# after torch, libdsk.so binds to that copy; loaded before, it would pull in the system's runtime, and torch would
# then find no GPU.
import torch  # noqa: F401

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdsk.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: build it first (python -m paper_2411_02820_amd.build "
                      "or __graft_entry__.build()); there is no non-HIP fallback")

lib = C.CDLL(LIB_PATH)

# ---- enums (include/dsk.h) ----
DSK_OK, DSK_EINVAL, DSK_ESHAPE, DSK_EDTYPE, DSK_ENOMEM, DSK_EHIP = 0, -1, -2, -3, -4, -5
DSK_F32, DSK_BF16 = 0, 1
DSK_MEM_DEVICE, DSK_MEM_HOST_PINNED = 0, 1
DSK_G1, DSK_WQ, DSK_WK, DSK_WV, DSK_WO, DSK_G2, DSK_WG, DSK_WU, DSK_WD = range(9)
DSK_DEFER_JOIN = 1
DSK_LOAD_PIPELINED, DSK_LOAD_REUSED_FIRST, DSK_LOAD_ALL_FIRST = 0, 1, 2

EXPORTS = (
    "dsk_model_create", "dsk_model_destroy", "dsk_model_set_tensor", "dsk_model_get_tensor",
    "dsk_model_init_random", "dsk_fill_normal", "dsk_partial_prefill", "dsk_partial_prefill_groups",
    "dsk_suffix_prefill",
    "dsk_join_loads", "dsk_set_load_mode", "dsk_set_load_throttle", "dsk_model_weight_bytes", "dsk_model_workspace_bytes",
    "dsk_strerror", "dsk_last_hip_error", "dsk_hash_context", "dsk_store_create", "dsk_store_destroy",
    "dsk_store_put_kv", "dsk_store_put_e", "dsk_store_fetch_kv_layer", "dsk_store_fetch_kv", "dsk_store_fetch_e",
    "dsk_store_erase", "dsk_store_usage", "dsk_estimate_prefill_ms", "dsk_select_recompute", "dsk_linear", "dsk_linear_static", "dsk_attention", "dsk_set_option", "dsk_get_stat",
    "dsk_moe_route",
)


class dsk_group_t(C.Structure):
    _fields_ = [("lo", C.c_int32), ("hi", C.c_int32), ("hidden_in", C.c_void_p), ("hidden_in_mem", C.c_int32),
                ("hidden_out", C.c_void_p)]


class dsk_frontier_point_t(C.Structure):
    _fields_ = [("lo", C.c_int32), ("hi", C.c_int32), ("quality", C.c_double)]


class dsk_latency_model_t(C.Structure):
    _fields_ = [("c0", C.c_double), ("c_layer_token", C.c_double), ("c_layer_token2", C.c_double),
                ("c_reused_token", C.c_double)]


class dsk_config_t(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("hidden", C.c_int32), ("n_q_heads", C.c_int32),
                ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32), ("ffn", C.c_int32),
                ("rope_base", C.c_double), ("rms_eps", C.c_double), ("dtype", C.c_int32),
                ("n_experts", C.c_int32), ("top_k", C.c_int32)]


class dsk_kv_t(C.Structure):
    _fields_ = [("base", C.c_void_p), ("mem", C.c_int32), ("layer_stride", C.c_int64),
                ("v_offset", C.c_int64), ("n_rows", C.c_int64)]


class dsk_batch_t(C.Structure):
    _fields_ = [("n_seqs", C.c_int32), ("n_tokens", C.c_int32),
                ("cu_seqlens_host", C.POINTER(C.c_int32)), ("cu_seqlens_dev", C.c_void_p),
                ("positions_dev", C.c_void_p)]


_P = C.c_void_p
lib.dsk_model_create.argtypes = [C.POINTER(dsk_config_t), C.c_int64, C.c_int64, C.POINTER(_P)]
lib.dsk_model_destroy.argtypes = [_P]
lib.dsk_model_set_tensor.argtypes = [_P, C.c_int, C.c_int, _P, C.c_int, _P]
lib.dsk_model_get_tensor.argtypes = [_P, C.c_int, C.c_int, _P, _P]
lib.dsk_model_init_random.argtypes = [_P, C.c_uint64, C.c_float, _P]
lib.dsk_fill_normal.argtypes = [_P, C.c_int64, C.c_uint64, C.c_uint64, C.c_float, C.c_float, C.c_int64, C.c_int, _P]
lib.dsk_partial_prefill.argtypes = [_P, _P, C.c_int, C.c_int, C.c_int, C.POINTER(dsk_kv_t), C.POINTER(dsk_kv_t),
                                    C.POINTER(dsk_batch_t), _P, C.c_uint32, _P]
lib.dsk_partial_prefill_groups.argtypes = [_P, C.POINTER(dsk_group_t), C.c_int, C.POINTER(dsk_kv_t), C.POINTER(dsk_kv_t),
                                           C.POINTER(dsk_batch_t), C.c_uint32, _P]
lib.dsk_suffix_prefill.argtypes = [_P, _P, C.POINTER(dsk_kv_t), C.POINTER(dsk_batch_t), C.POINTER(dsk_batch_t),
                                   C.c_int64, _P, _P]
lib.dsk_linear.argtypes = [C.c_int, _P, _P, _P, _P, C.c_int, C.c_int, C.c_int, _P]
lib.dsk_linear_static.argtypes = [C.c_int, _P, _P, _P, _P, C.c_int, C.c_int, C.c_int, _P]
lib.dsk_attention.argtypes = [C.c_int, _P, _P, _P, _P, C.POINTER(dsk_batch_t), C.POINTER(dsk_batch_t), C.c_int64,
                              C.c_int, C.c_int, C.c_int, _P, C.c_int64, _P]
lib.dsk_moe_route.argtypes = [C.c_int, _P, _P, C.c_int, C.c_int, C.c_int, C.c_int, _P, _P, _P]
lib.dsk_set_option.argtypes = [C.c_char_p, C.c_int]
lib.dsk_get_stat.argtypes = [C.c_char_p, C.POINTER(C.c_double)]
lib.dsk_join_loads.argtypes = [_P, _P]
lib.dsk_set_load_mode.argtypes = [_P, C.c_int]
lib.dsk_hash_context.argtypes = [C.c_char_p, C.c_int64]
lib.dsk_hash_context.restype = C.c_uint64
lib.dsk_store_create.argtypes = [C.c_int64, C.c_int64, C.POINTER(_P)]
lib.dsk_store_destroy.argtypes = [_P]
lib.dsk_store_put_kv.argtypes = [_P, C.c_uint64, C.c_uint64, C.POINTER(dsk_kv_t), C.c_int, C.c_int64, C.c_int64, C.c_int, _P,
                                 C.POINTER(C.c_int)]
lib.dsk_store_put_e.argtypes = [_P, C.c_uint64, C.c_uint64, C.c_int, _P, C.c_int, C.c_int64, C.c_int, _P, C.POINTER(C.c_int)]
lib.dsk_store_fetch_kv_layer.argtypes = [_P, C.c_uint64, C.c_uint64, C.c_int, C.POINTER(_P), C.POINTER(_P), C.POINTER(C.c_int),
                                         C.POINTER(C.c_int64)]
lib.dsk_store_fetch_kv.argtypes = [_P, C.c_uint64, C.c_uint64, C.POINTER(dsk_kv_t), C.POINTER(C.c_int)]
lib.dsk_store_fetch_e.argtypes = [_P, C.c_uint64, C.c_uint64, C.c_int, C.POINTER(_P), C.POINTER(C.c_int), C.POINTER(C.c_int64)]
lib.dsk_store_erase.argtypes = [_P, C.c_uint64, C.c_uint64]
lib.dsk_store_usage.argtypes = [_P, C.POINTER(C.c_int64), C.POINTER(C.c_int64), C.POINTER(C.c_int64)]
lib.dsk_estimate_prefill_ms.argtypes = [C.POINTER(dsk_latency_model_t), C.c_int, C.c_int, C.c_int64]
lib.dsk_estimate_prefill_ms.restype = C.c_double
lib.dsk_select_recompute.argtypes = [C.POINTER(dsk_frontier_point_t), C.c_int, C.c_int, C.c_int64, C.POINTER(dsk_latency_model_t),
                                     C.c_double, C.c_double, C.c_int, C.POINTER(C.c_int)]
lib.dsk_set_load_throttle.argtypes = [_P, C.c_double]
lib.dsk_model_weight_bytes.argtypes = [_P]
lib.dsk_model_weight_bytes.restype = C.c_int64
lib.dsk_model_workspace_bytes.argtypes = [_P]
lib.dsk_model_workspace_bytes.restype = C.c_int64
lib.dsk_strerror.argtypes = [C.c_int]
lib.dsk_strerror.restype = C.c_char_p
lib.dsk_last_hip_error.argtypes = []
for _n in EXPORTS:
    if _n not in ("dsk_model_weight_bytes", "dsk_model_workspace_bytes", "dsk_strerror", "dsk_estimate_prefill_ms",
                  "dsk_hash_context"):
        getattr(lib, _n).restype = C.c_int


class DskError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = lib.dsk_strerror(status).decode()
        if status == DSK_EHIP:
            msg += f" (hipError_t {lib.dsk_last_hip_error()})"
        super().__init__(f"{where}: {msg} [{status}]")


def _check(status: int, where: str):
    if status != DSK_OK:
        raise DskError(status, where)


def _ptr(x):
    """Raw address of a torch tensor / int / (address, dsk_mem) pair / None."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    if isinstance(x, tuple):
        return x[0]
    return x.data_ptr()


def _stream(stream):
    if stream is None:
        return None
    return stream if isinstance(stream, int) else stream.cuda_stream


def _mem_of(t) -> int:
    if isinstance(t, tuple):   # (address, dsk_mem), e.g. what the cache store hands out
        return t[1]
    return DSK_MEM_DEVICE if t.is_cuda else DSK_MEM_HOST_PINNED


# ---- the entry points, same names as the header ----
def dsk_model_create(cfg: dsk_config_t, max_tokens: int, max_kv_rows: int) -> int:
    out = _P()
    _check(lib.dsk_model_create(C.byref(cfg), max_tokens, max_kv_rows, C.byref(out)), "dsk_model_create")
    return out.value


def dsk_model_destroy(model: int):
    _check(lib.dsk_model_destroy(model), "dsk_model_destroy")


def dsk_model_set_tensor(model: int, layer: int, tensor: int, src, stream=None):
    _check(lib.dsk_model_set_tensor(model, layer, tensor, _ptr(src), _mem_of(src), _stream(stream)),
           "dsk_model_set_tensor")


def dsk_model_get_tensor(model: int, layer: int, tensor: int, dst, stream=None):
    _check(lib.dsk_model_get_tensor(model, layer, tensor, _ptr(dst), _stream(stream)), "dsk_model_get_tensor")


def dsk_model_init_random(model: int, seed: int, std: float, stream=None):
    _check(lib.dsk_model_init_random(model, seed, std, _stream(stream)), "dsk_model_init_random")


def dsk_fill_normal(dst, n: int, seed: int, stream_id: int, std: float, offset: float, idx0: int, dtype: int,
                    stream=None):
    _check(lib.dsk_fill_normal(_ptr(dst), n, seed, stream_id, std, offset, idx0, dtype, _stream(stream)),
           "dsk_fill_normal")


def dsk_partial_prefill(model: int, hidden_in, lo: int, hi: int, kv_reused, kv_out: dsk_kv_t, batch: dsk_batch_t,
                        hidden_out=None, flags: int = 0, stream=None):
    _check(lib.dsk_partial_prefill(model, _ptr(hidden_in), _mem_of(hidden_in), lo, hi,
                                   None if kv_reused is None else C.byref(kv_reused), C.byref(kv_out),
                                   C.byref(batch), _ptr(hidden_out), flags, _stream(stream)),
           "dsk_partial_prefill")


def dsk_partial_prefill_groups(model: int, groups, kv_reused, kv_out: dsk_kv_t, batch: dsk_batch_t, flags: int = 0,
                               stream=None):
    """groups: sequence of (lo, hi, hidden_in, hidden_out or None)."""
    arr = (dsk_group_t * max(1, len(groups)))()
    for i, (lo, hi, hidden_in, hidden_out) in enumerate(groups):
        arr[i].lo, arr[i].hi = lo, hi
        arr[i].hidden_in, arr[i].hidden_in_mem = _ptr(hidden_in), _mem_of(hidden_in)
        arr[i].hidden_out = _ptr(hidden_out)
    _check(lib.dsk_partial_prefill_groups(model, arr, len(groups), None if kv_reused is None else C.byref(kv_reused),
                                          C.byref(kv_out), C.byref(batch), flags, _stream(stream)),
           "dsk_partial_prefill_groups")


def dsk_suffix_prefill(model: int, suffix_hidden_in, kv: dsk_kv_t, prefix: dsk_batch_t, suffix: dsk_batch_t,
                       suffix_row0: int, hidden_out, stream=None):
    _check(lib.dsk_suffix_prefill(model, _ptr(suffix_hidden_in), C.byref(kv), C.byref(prefix), C.byref(suffix),
                                  suffix_row0, _ptr(hidden_out), _stream(stream)), "dsk_suffix_prefill")


def dsk_linear(dtype: int, x, w, y, r, M: int, N: int, K: int, stream=None):
    _check(lib.dsk_linear(dtype, _ptr(x), _ptr(w), _ptr(y), _ptr(r), M, N, K, _stream(stream)), "dsk_linear")


def dsk_linear_static(dtype: int, x, w, y, r, M: int, N: int, K: int, stream=None):
    _check(lib.dsk_linear_static(dtype, _ptr(x), _ptr(w), _ptr(y), _ptr(r), M, N, K, _stream(stream)), "dsk_linear_static")


def dsk_attention(dtype: int, q, k_rows, v_rows, out, queries: dsk_batch_t, prefix, own_row0: int, n_q_heads: int,
                  n_kv_heads: int, head_dim: int, scratch=None, stream=None):
    nbytes = 0 if scratch is None else scratch.numel() * scratch.element_size()
    _check(lib.dsk_attention(dtype, _ptr(q), _ptr(k_rows), _ptr(v_rows), _ptr(out), C.byref(queries),
                             None if prefix is None else C.byref(prefix), own_row0, n_q_heads, n_kv_heads, head_dim,
                             _ptr(scratch), nbytes, _stream(stream)), "dsk_attention")


def dsk_moe_route(dtype: int, x, wr, n: int, d: int, n_experts: int, top_k: int, experts_out, gates_out, stream=None):
    _check(lib.dsk_moe_route(dtype, _ptr(x), _ptr(wr), n, d, n_experts, top_k, _ptr(experts_out), _ptr(gates_out),
                             _stream(stream)), "dsk_moe_route")


def DSK_EXPERT(e: int, t: int) -> int:
    return 16 + e * 16 + t


def dsk_set_option(name: str, value: int):
    _check(lib.dsk_set_option(name.encode(), value), "dsk_set_option")


def dsk_get_stat(name: str) -> float:
    v = C.c_double()
    _check(lib.dsk_get_stat(name.encode(), C.byref(v)), "dsk_get_stat")
    return v.value


def dsk_join_loads(model: int, stream=None):
    _check(lib.dsk_join_loads(model, _stream(stream)), "dsk_join_loads")


def dsk_set_load_mode(model: int, mode: int):
    _check(lib.dsk_set_load_mode(model, mode), "dsk_set_load_mode")


def dsk_set_load_throttle(model: int, gb_per_s: float):
    _check(lib.dsk_set_load_throttle(model, gb_per_s), "dsk_set_load_throttle")


DSK_ENOENT = -6
DSK_ELIMIT = -7
DSK_STATIC_MAX_M, DSK_STATIC_MAX_N = 64, 65536
DSK_TIER_AUTO, DSK_TIER_DEVICE, DSK_TIER_HOST = 0, 1, 2


def dsk_hash_context(data: bytes) -> int:
    return lib.dsk_hash_context(data, len(data))


def dsk_store_create(device_capacity_bytes: int, host_capacity_bytes: int) -> int:
    out = _P()
    _check(lib.dsk_store_create(device_capacity_bytes, host_capacity_bytes, C.byref(out)), "dsk_store_create")
    return out.value


def dsk_store_destroy(store: int):
    _check(lib.dsk_store_destroy(store), "dsk_store_destroy")


def dsk_store_put_kv(store: int, context: int, model_id: int, kv: dsk_kv_t, n_layers: int, n_rows: int, row_bytes: int,
                     tier: int = DSK_TIER_AUTO, stream=None) -> bool:
    ins = C.c_int(0)
    _check(lib.dsk_store_put_kv(store, context, model_id, C.byref(kv), n_layers, n_rows, row_bytes, tier, _stream(stream),
                                C.byref(ins)), "dsk_store_put_kv")
    return bool(ins.value)


def dsk_store_put_e(store: int, context: int, model_id: int, layer: int, e_cache, tier: int = DSK_TIER_AUTO,
                    stream=None) -> bool:
    ins = C.c_int(0)
    nbytes = e_cache.numel() * e_cache.element_size()
    _check(lib.dsk_store_put_e(store, context, model_id, layer, _ptr(e_cache), _mem_of(e_cache), nbytes, tier,
                               _stream(stream), C.byref(ins)), "dsk_store_put_e")
    return bool(ins.value)


def dsk_store_fetch_kv_layer(store: int, context: int, model_id: int, layer: int):
    """-> (k_ptr, v_ptr, mem, bytes_each)"""
    k, v, mem, n = _P(), _P(), C.c_int(), C.c_int64()
    _check(lib.dsk_store_fetch_kv_layer(store, context, model_id, layer, C.byref(k), C.byref(v), C.byref(mem), C.byref(n)),
           "dsk_store_fetch_kv_layer")
    return k.value, v.value, mem.value, n.value


def dsk_store_fetch_kv(store: int, context: int, model_id: int):
    """-> (dsk_kv_t, n_layers)"""
    d, n = dsk_kv_t(), C.c_int()
    _check(lib.dsk_store_fetch_kv(store, context, model_id, C.byref(d), C.byref(n)), "dsk_store_fetch_kv")
    return d, n.value


def dsk_store_fetch_e(store: int, context: int, model_id: int, layer: int):
    """-> (ptr, mem, bytes)"""
    p, mem, n = _P(), C.c_int(), C.c_int64()
    _check(lib.dsk_store_fetch_e(store, context, model_id, layer, C.byref(p), C.byref(mem), C.byref(n)), "dsk_store_fetch_e")
    return p.value, mem.value, n.value


def dsk_store_erase(store: int, context: int, model_id: int):
    _check(lib.dsk_store_erase(store, context, model_id), "dsk_store_erase")


def dsk_store_usage(store: int):
    """-> (device_bytes, host_bytes, n_entries)"""
    a, b, c = C.c_int64(), C.c_int64(), C.c_int64()
    _check(lib.dsk_store_usage(store, C.byref(a), C.byref(b), C.byref(c)), "dsk_store_usage")
    return a.value, b.value, c.value


def dsk_estimate_prefill_ms(lat, n_layers: int, n_recomputed: int, n_tokens: int) -> float:
    """lat: (c0, c_layer_token, c_layer_token2, c_reused_token)."""
    return lib.dsk_estimate_prefill_ms(C.byref(dsk_latency_model_t(*lat)), n_layers, n_recomputed, n_tokens)


def dsk_select_recompute(frontier, n_layers: int, n_tokens: int, lat, slo_ms: float, quality_target: float,
                         n_waiting: int) -> int:
    """frontier: sequence of (lo, hi, quality); returns the index of the chosen point."""
    arr = (dsk_frontier_point_t * max(1, len(frontier)))(*[dsk_frontier_point_t(*p) for p in frontier])
    chosen = C.c_int(-1)
    _check(lib.dsk_select_recompute(arr, len(frontier), n_layers, n_tokens, C.byref(dsk_latency_model_t(*lat)), slo_ms,
                                    quality_target, n_waiting, C.byref(chosen)), "dsk_select_recompute")
    return chosen.value


def dsk_model_weight_bytes(model: int) -> int:
    return lib.dsk_model_weight_bytes(model)


def dsk_model_workspace_bytes(model: int) -> int:
    return lib.dsk_model_workspace_bytes(model)


# ---- descriptor helpers (marshalling only) ----
def config_from_shape(shape) -> dsk_config_t:
    """shape: an object with n_layers, hidden, n_q_heads, n_kv_heads, head_dim, ffn, rope_base, rms_eps, dtype."""
    return dsk_config_t(shape.n_layers, shape.hidden, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.ffn,
                        float(shape.rope_base), float(shape.rms_eps), DSK_F32 if shape.dtype == "f32" else DSK_BF16,
                        getattr(shape, "n_experts", 0), getattr(shape, "top_k", 0))


def kv_desc(t) -> dsk_kv_t:
    """Descriptor of a cache tensor laid out [L, 2, n_rows, Hkv, dh] (contiguous; device or pinned host)."""
    assert t.dim() == 5 and t.shape[1] == 2 and t.is_contiguous()
    es = t.element_size()
    row = t.shape[3] * t.shape[4] * es
    return dsk_kv_t(t.data_ptr(), _mem_of(t), 2 * t.shape[2] * row, t.shape[2] * row, t.shape[2])


class Batch:
    """Owns the host and device arrays a dsk_batch_t points to (keeps them alive)."""

    def __init__(self, cu_seqlens, positions=None, device="cuda"):
        import torch
        self.cu_host = np.ascontiguousarray(cu_seqlens, dtype=np.int32)
        self.cu_dev = torch.from_numpy(self.cu_host).to(device)
        self.pos_dev = None if positions is None else torch.from_numpy(
            np.ascontiguousarray(positions, dtype=np.int32)).to(device)
        self.desc = dsk_batch_t(len(self.cu_host) - 1, int(self.cu_host[-1]),
                                self.cu_host.ctypes.data_as(C.POINTER(C.c_int32)), self.cu_dev.data_ptr(),
                                None if self.pos_dev is None else self.pos_dev.data_ptr())
