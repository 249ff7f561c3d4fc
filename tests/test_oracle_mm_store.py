"""Pins of the MM-Store oracle (hash of the multimodal input as the key of the feature pool,
paper section 3.2): closed forms and algebraic laws of the polynomial hash evaluated in a
second, different order, and hand-derived replacement sequences for the pool."""

import numpy as np

from oracle import mm_store as S

P, (R0, R1) = S.P, S.BASES


def horner(words, r):
    h = 0
    for w in words:
        h = (h + w + 1) * r % P
    return h


def test_bases_and_modulus():
    assert P == 2305843009213693951 and 1 < R0 < P and 1 < R1 < P and R0 != R1


def test_empty_input_closed_form():
    # four header words, all zero: (0 + 1) * (R^4 + R^3 + R^2 + R)
    assert S.words_of(b"", 0) == [0, 0, 0, 0]
    assert S.hash128(b"", 0) == tuple((r ** 4 + r ** 3 + r ** 2 + r) % P for r in (R0, R1))


def test_one_word_closed_form_and_padding():
    # bytes 01 00 00 00: length 4, salt 0, data word 1 -> 5 R^5 + R^4 + R^3 + R^2 + 2 R
    want = tuple((5 * r ** 5 + r ** 4 + r ** 3 + r ** 2 + 2 * r) % P for r in (R0, R1))
    assert S.hash128(b"\x01\x00\x00\x00") == want
    # three bytes are padded with one zero: same data word 1, but the length word is 3
    want3 = tuple((4 * r ** 5 + r ** 4 + r ** 3 + r ** 2 + 2 * r) % P for r in (R0, R1))
    assert S.hash128(b"\x01\x00\x00") == want3
    assert S.words_of(b"\x01\x02\x03\x04\x05", 0)[4:] == [0x04030201, 0x05]      # little-endian words


def test_salt_enters_as_two_header_words():
    salt = 0x1122334455667788
    assert S.words_of(b"ab", salt)[:4] == [2, 0, 0x55667788, 0x11223344]
    assert S.hash128(b"ab", salt) != S.hash128(b"ab", salt + 1) != S.hash128(b"ab", 0)


def test_power_sum_equals_horner_on_random_inputs():
    rng = np.random.default_rng(1)
    for n in (0, 1, 3, 4, 5, 63, 64, 65, 1000, 4099):
        data = rng.integers(0, 256, size=n, dtype=np.uint8).tobytes()
        salt = int(rng.integers(0, 2 ** 62))
        w = S.words_of(data, salt)
        assert S.hash128(data, salt) == (horner(w, R0), horner(w, R1))
        assert all(0 <= h < P for h in S.hash128(data, salt))


def test_concatenation_law_of_the_word_polynomial():
    # H(s1 + s2) = H(s1) * R^len(s2) + H(s2): what lets chunks be hashed independently
    rng = np.random.default_rng(2)
    s = [int(v) for v in rng.integers(0, 2 ** 32, size=300)]
    for cut in (0, 1, 150, 299, 300):
        for r in (R0, R1):
            assert horner(s, r) == (horner(s[:cut], r) * pow(r, len(s) - cut, P) + horner(s[cut:], r)) % P


def test_every_single_byte_change_moves_both_hashes():
    rng = np.random.default_rng(3)
    data = bytearray(rng.integers(0, 256, size=101, dtype=np.uint8).tobytes())
    base = S.hash128(bytes(data), 7)
    for i in range(len(data)):
        for delta in (1, 128, 255):
            d = bytearray(data)
            d[i] = (d[i] + delta) % 256
            h = S.hash128(bytes(d), 7)
            assert h[0] != base[0] and h[1] != base[1]
    # trailing zero bytes and swapped words are different inputs
    assert S.hash128(b"abc") != S.hash128(b"abc\0") != S.hash128(b"abc\0\0")
    assert S.hash128(b"aaaabbbb") != S.hash128(b"bbbbaaaa")


def test_pool_first_fit_and_least_recently_used_replacement_by_hand():
    st = S.Store(1024)
    A, B, C, D, E, F = [(i, i) for i in range(6)]
    assert st.insert(A, 300) == 0            # occupies [0, 512)
    assert st.insert(B, 200) == 512          # [512, 768)
    assert st.insert(C, 256) == 768          # [768, 1024): pool full
    assert st.lookup(A) == (0, 300) and st.hits == 1          # A becomes the most recent
    assert st.lookup(D) is None and st.misses == 1
    assert st.insert(D, 256) == 512 and st.evictions == 1     # B was least recent
    assert st.lookup(B) is None
    # 600 bytes need 768 contiguous: C goes (free 256 at the top), A goes (free [0, 512)),
    # still split by D, D goes -> offset 0
    assert st.insert(E, 600) == 0 and st.evictions == 4
    assert list(st.entries) == [E]
    assert st.insert(F, 100) == 768          # first fit behind E's 768 bytes
    assert st.insert(F, 200) == 768          # same key: replaced in place, no eviction
    assert st.evictions == 4 and st.entries[F] == (768, 200)
    assert st.insert((9, 9), 2000) is None and st.insert((9, 9), 0) is None
    assert list(st.entries) == [E, F]        # an impossible insert drops nothing


def test_pool_reuses_a_hole_in_the_middle():
    st = S.Store(2048)
    for i, n in enumerate((256, 512, 256, 512)):            # [0,256) [256,768) [768,1024) [1024,1536)
        st.insert((i, 0), n)
    st.lookup((0, 0)); st.lookup((2, 0)); st.lookup((3, 0))  # entry 1 is now least recent
    assert st.insert((7, 0), 600) is not None                # needs 768: tail has 512 -> evict entry 1 -> hole of 512 -> evict entry 0 -> [0, 768)
    assert st.entries[(7, 0)] == (0, 600) and st.evictions == 2
    assert st.insert((8, 0), 512) == 1536                    # the tail was free all along
