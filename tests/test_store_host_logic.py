"""Host logic of the MM-Store stand-in (paper section 3.2): the library's pool bookkeeping
against the oracle's model, on the CPU -- create / lookup / insert / stats never touch device
memory, so a made-up pool address serves."""

import numpy as np
import pytest

from oracle import mm_store as S
from paper_2601_11590_amd import binding as B

FAKE_POOL = 0x7F0000000000          # never dereferenced
SCRATCH = 1 << 20


def test_create_rejects_bad_pools():
    with pytest.raises(B.StoreError) as e:
        B.epd_store_create(FAKE_POOL + 8, 4 << 20)
    assert e.value.status == B.EPD_ERR_INVALID_ARG and "aligned" in str(e.value)
    with pytest.raises(B.StoreError) as e:
        B.epd_store_create(FAKE_POOL, SCRATCH)
    assert e.value.status == B.EPD_ERR_WORKSPACE
    with pytest.raises(B.StoreError):
        B.epd_store_create(0, 4 << 20)


def test_hand_derived_replacement_sequence_through_the_c_abi():
    st = B.epd_store_create(FAKE_POOL, SCRATCH + 1024)
    base = FAKE_POOL + SCRATCH
    A, Bk, Ck, D, E = [(i, i) for i in range(5)]
    assert B.epd_store_insert(st, A, 300) == base
    assert B.epd_store_insert(st, Bk, 200) == base + 512
    assert B.epd_store_insert(st, Ck, 256) == base + 768
    assert B.epd_store_lookup(st, A) == (base, 300)
    assert B.epd_store_lookup(st, D) is None
    assert B.epd_store_insert(st, D, 256) == base + 512            # B was least recently used
    assert B.epd_store_lookup(st, Bk) is None
    assert B.epd_store_insert(st, E, 600) == base                   # C, A and D all have to go
    assert B.epd_store_stats(st) == dict(hits=1, misses=2, evictions=4, entries=1)
    with pytest.raises(B.StoreError) as e:
        B.epd_store_insert(st, (9, 9), 2000)
    assert e.value.status == B.EPD_ERR_WORKSPACE
    assert B.epd_store_stats(st)["entries"] == 1                    # nothing dropped for an impossible entry
    B.epd_store_destroy(st)


@pytest.mark.parametrize("seed", range(4))
def test_random_traffic_matches_the_oracle_model(seed):
    rng = np.random.default_rng(seed)
    arena = int(rng.integers(8, 64)) * 256
    st = B.epd_store_create(FAKE_POOL, SCRATCH + arena + int(rng.integers(0, 256)))   # a ragged tail is not used
    model = S.Store(arena)
    base = FAKE_POOL + SCRATCH
    keys = [(int(rng.integers(1, 2 ** 61)), int(rng.integers(1, 2 ** 61))) for _ in range(24)]
    for step in range(600):
        k = keys[int(rng.integers(0, len(keys)))]
        if rng.random() < 0.5:
            got = B.epd_store_lookup(st, k)
            want = model.lookup(k)
            assert (got is None) == (want is None), step
            if got is not None:
                assert got == (base + want[0], want[1]), step
        else:
            n = int(rng.integers(1, arena // 2))
            assert B.epd_store_insert(st, k, n) == base + model.insert(k, n), step
    assert B.epd_store_stats(st) == dict(hits=model.hits, misses=model.misses, evictions=model.evictions,
                                         entries=len(model.entries))
    B.epd_store_destroy(st)
