"""epd_store_hash_noalloc (the entry point for callers that cannot allocate: its scratch is a
static device array inside the library) against epd_store_hash (scratch in the caller's pool)
through the C ABI: the keys must be bit-identical, on two calls in a row, the second with a
smaller input -- the array keeps the first call's contents and nothing may leak from them."""

import ctypes as C

import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def both(store, data, offsets, salts):
    import torch
    from paper_2601_11590_amd import binding as B
    n = len(salts)
    want = store.hash(data, offsets, salts)                                   # existing entry point (waits for its keys)
    keys_dev = torch.full((n, 2), -1, dtype=torch.int64, device="cuda:0")     # output buffer: the caller's
    free_before = torch.cuda.mem_get_info()[0]
    B.epd_store_hash_noalloc(data.data_ptr(), offsets, salts, keys_dev.data_ptr(), torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    assert torch.cuda.mem_get_info()[0] == free_before, "device memory in use changed across the call"
    got = keys_dev.cpu().numpy().view(np.uint64)
    return want, got


def test_noalloc_keys_equal_the_pool_variant_on_two_calls_the_second_smaller():
    import torch
    from paper_2601_11590_amd import binding as B
    store = B.MMStore(4 << 20)
    try:
        rng = np.random.default_rng(21)
        big = torch.from_numpy(rng.integers(0, 256, size=48 << 20, dtype=np.uint8)).to("cuda:0")
        # call 1: 32 ranges (the maximum), ragged lengths and start alignments, the largest 24 MiB
        # (many blocks per range: the scratch array fills up), one empty range
        lens = [24 << 20, 0, 1, 3, 4, 5, 64 * 256 * 4, 64 * 256 * 4 + 1, 100003, 7 << 20] + [int(v) for v in rng.integers(1, 300000, size=22)]
        offs = np.concatenate([[0], np.cumsum(lens)]).astype(np.uint64)
        salts = rng.integers(0, 2 ** 63, size=len(lens), dtype=np.uint64)
        want, got = both(store, big, offs, salts)
        assert np.array_equal(want, got), "first call"
        assert len(np.unique(want[:, 0])) == len(lens)
        # call 2, right behind it: three short ranges of the same buffer -- far fewer blocks, so most
        # of the array still holds call 1's partial hashes
        offs2 = np.array([5, 5 + 70001, 5 + 70001 + 12, 5 + 70001 + 12 + 4096], dtype=np.uint64)
        salts2 = np.array([1, 2, 3], dtype=np.uint64)
        want2, got2 = both(store, big, offs2, salts2)
        assert np.array_equal(want2, got2), "second, smaller call"
        # and the first input once more: same keys as before
        want3, got3 = both(store, big, offs, salts)
        assert np.array_equal(want3, want) and np.array_equal(got3, want)
        # sizes beyond the array's capacity are refused with nothing launched
        offs33 = np.arange(34, dtype=np.uint64) * 16
        keys_dev = torch.zeros((33, 2), dtype=torch.int64, device="cuda:0")
        with pytest.raises(B.StoreError) as ei:
            B.epd_store_hash_noalloc(big.data_ptr(), offs33, np.ones(33, np.uint64), keys_dev.data_ptr(), 0)
        assert ei.value.status == B.EPD_ERR_SHAPE and "at most 32" in str(ei.value)
        torch.cuda.synchronize()
        assert int(keys_dev.abs().sum()) == 0
        U64P = C.POINTER(C.c_uint64)
        assert B.lib.epd_store_hash_noalloc(None, offs2.ctypes.data_as(U64P), salts2.ctypes.data_as(U64P), 3, keys_dev.data_ptr(), None) \
            == B.EPD_ERR_INVALID_ARG
    finally:
        store.close()
