"""store / fetch / partial_prefill (Sec. 4.4) on the GPU: what the store returns is byte-identical to what was
stored, per layer and per tier, and a selective prefill fed from the store equals one fed directly."""
import numpy as np
import pytest
import torch

from paper_2411_02820_amd import synth

pytestmark = pytest.mark.gpu

SHAPE = synth.TINY


def view(ptr, mem, nbytes, shape):
    """Bytes behind a pointer the store handed out, as a uint8 numpy array (copy)."""
    import ctypes
    from paper_2411_02820_amd import binding as B
    if mem == B.DSK_MEM_HOST_PINNED:
        return np.ctypeslib.as_array((ctypes.c_uint8 * nbytes).from_address(ptr)).copy()
    hip = ctypes.CDLL("libamdhip64.so")
    hip.hipMemcpy.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int]
    out = np.empty(nbytes, dtype=np.uint8)
    assert hip.hipMemcpy(out.ctypes.data, ptr, nbytes, 2) == 0   # hipMemcpyDeviceToHost
    return out


def test_store_fetch_partial_prefill():
    from paper_2411_02820_amd import binding as B
    from tests import gpu_util as G
    T = 96
    L = SHAPE.n_layers
    ctx = B.dsk_hash_context(b"the shared context of two fine-tuned models")
    sender, receiver = 1, 0
    kv_np = synth.kv_cache(SHAPE, T)
    e_np = synth.hidden_states(SHAPE, T)
    kv_dev = G.to_dev(kv_np, SHAPE)
    e_dev = G.to_dev(e_np, SHAPE)
    row_bytes = SHAPE.kv_width * 4
    layer_bytes = 2 * T * row_bytes
    st = B.dsk_store_create(2 * L * layer_bytes, 8 * L * layer_bytes)
    try:
        # device tier takes the first cache, a second context overflows to pinned host memory
        assert B.dsk_store_put_kv(st, ctx, sender, B.kv_desc(kv_dev), L, T, row_bytes) is True
        assert B.dsk_store_put_kv(st, ctx, sender, B.kv_desc(kv_dev), L, T, row_bytes) is False   # already there
        assert B.dsk_store_put_e(st, ctx, sender, 1, e_dev) is True
        ctx2 = B.dsk_hash_context(b"another context")
        assert B.dsk_store_put_kv(st, ctx2, sender, B.kv_desc(kv_dev), L, T, row_bytes) is True
        torch.cuda.synchronize()
        dev_b, host_b, n = B.dsk_store_usage(st)
        assert n == 3 and dev_b == L * layer_bytes + e_np.nbytes and host_b == L * layer_bytes
        for c, want_mem in ((ctx, B.DSK_MEM_DEVICE), (ctx2, B.DSK_MEM_HOST_PINNED)):
            for l in range(L):
                k, v, mem, each = B.dsk_store_fetch_kv_layer(st, c, sender, l)
                assert mem == want_mem and each == T * row_bytes
                assert np.array_equal(view(k, mem, each, None).view(np.float32), kv_np[l, 0].ravel())
                assert np.array_equal(view(v, mem, each, None).view(np.float32), kv_np[l, 1].ravel())
        ep, emem, ebytes = B.dsk_store_fetch_e(st, ctx, sender, 1)
        assert ebytes == e_np.nbytes and np.array_equal(view(ep, emem, ebytes, None).view(np.float32), e_np.ravel())

        # partial_prefill from the store (both tiers) == partial_prefill from the original tensors
        with G.GpuModel(SHAPE, T) as m:
            m.load_from_generator(synth.SEED_RECEIVER, scale=8.0)
            kv_ref, h_ref = m.partial(e_dev, 1, 3, kv_dev, [T])
            batch = B.Batch(synth.cu_seqlens([T]), synth.packed_positions([T]))
            for c in (ctx, ctx2):
                desc, n_layers = B.dsk_store_fetch_kv(st, c, sender)
                assert n_layers == L
                kv_out = m.new_cache(T, fill=float("nan"))
                h_out = torch.empty_like(h_ref)
                B.dsk_partial_prefill(m.handle, (ep, emem), 1, 3, desc, B.kv_desc(kv_out), batch.desc, h_out)
                torch.cuda.synchronize()
                assert torch.equal(kv_out, kv_ref) and torch.equal(h_out, h_ref)

        B.dsk_store_erase(st, ctx2, sender)
        assert B.dsk_store_usage(st)[1] == 0
        with pytest.raises(B.DskError) as e:
            B.dsk_store_fetch_kv(st, ctx2, sender)
        assert e.value.status == B.DSK_ENOENT
        # nothing fits any more on the device tier alone
        with pytest.raises(B.DskError) as e:
            B.dsk_store_put_kv(st, 77, sender, B.kv_desc(kv_dev), L, T, row_bytes, B.DSK_TIER_DEVICE)
        assert e.value.status == B.DSK_ENOMEM
    finally:
        B.dsk_store_destroy(st)
