"""Host side of the cache store (no GPU): the context hash against the published FNV-1a test vectors, and the
store's bookkeeping paths that touch no device memory."""
import pytest


def test_context_hash_is_fnv1a_64():
    from paper_2411_02820_amd import binding as B
    # test vectors of the FNV reference distribution (FNV-1a, 64 bit)
    assert B.dsk_hash_context(b"") == 0xcbf29ce484222325
    assert B.dsk_hash_context(b"a") == 0xaf63dc4c8601ec8c
    assert B.dsk_hash_context(b"foobar") == 0x85944171f73967e8
    assert B.dsk_hash_context(b"a long context") != B.dsk_hash_context(b"a long contexT")


def test_empty_store_and_bad_arguments():
    from paper_2411_02820_amd import binding as B
    st = B.dsk_store_create(1 << 20, 1 << 20)
    try:
        assert B.dsk_store_usage(st) == (0, 0, 0)
        for fn, args in ((B.dsk_store_fetch_kv, (st, 1, 2)), (B.dsk_store_fetch_kv_layer, (st, 1, 2, 0)),
                         (B.dsk_store_fetch_e, (st, 1, 2, 0)), (B.dsk_store_erase, (st, 1, 2))):
            with pytest.raises(B.DskError) as e:
                fn(*args)
            assert e.value.status == B.DSK_ENOENT
        assert B.lib.dsk_store_put_kv(st, 1, 2, None, 1, 1, 16, 0, None, None) == B.DSK_EINVAL
        assert B.lib.dsk_store_put_e(st, 1, 2, 0, None, 0, 16, 0, None, None) == B.DSK_EINVAL
    finally:
        B.dsk_store_destroy(st)
    with pytest.raises(B.DskError):
        B.dsk_store_create(-1, 0)
    assert B.lib.dsk_strerror(B.DSK_ENOENT) == b"no such entry in the cache store"
