"""CPU oracle of the single-node stand-in for the paper's MM Store (section 3.2, "Multimodal
Cache Pooling" and "Fault-Tolerant and Recomputation"): encoded features are kept under the hash
of the multimodal input; a hit returns the stored rows, a miss (never stored, or evicted)
recomputes them.

TEST INFRASTRUCTURE ONLY.  Imported by the tests; shares no code with the HIP library.

The paper names neither the hash nor the pool's replacement rule.  Readings taken here:

  * key = two polynomial hashes modulo the Mersenne prime P = 2^61 - 1 over the input taken as
    32-bit little-endian words (the last word zero-padded), preceded by four header words: the
    byte length (low, high) and a caller's 64-bit salt (low, high) -- the salt carries what the
    bytes alone do not say (frame size, grid, model).  With s_0 .. s_{L-1} the header and data
    words and R_k the base of hash k,
        H_k = sum_j (s_j + 1) * R_k^(L - j)   (mod P),   k = 0, 1.
    The "+ 1" keeps zero words from vanishing, so inputs that differ only in trailing zeros
    differ in every term position as well as in the length word.
  * the pool is a byte arena; an entry occupies one contiguous, 256-byte aligned range; on
    insert the least recently used entries are dropped until a free range (first fit, lowest
    address) holds the new entry; a lookup that hits makes the entry the most recent one.

Plain Python integers, one term at a time; nothing is blocked or reordered.
"""

from __future__ import annotations

from collections import OrderedDict
from typing import Dict, List, Optional, Tuple

P = (1 << 61) - 1
BASES = (0x1D4E2C1B3A596877 % P, 0x0F1E2D3C4B5A6978 % P)     # fixed, arbitrary, below P
ALIGN = 256


def words_of(data: bytes, salt: int) -> List[int]:
    """Header (length low/high, salt low/high) followed by the little-endian data words."""
    n = len(data)
    pad = (-n) % 4
    body = data + b"\0" * pad
    out = [n & 0xFFFFFFFF, n >> 32, salt & 0xFFFFFFFF, (salt >> 32) & 0xFFFFFFFF]
    out.extend(int.from_bytes(body[i:i + 4], "little") for i in range(0, len(body), 4))
    return out


def hash128(data: bytes, salt: int = 0) -> Tuple[int, int]:
    """(H_0, H_1) of the definition above, each term evaluated with its own power."""
    s = words_of(bytes(data), salt)
    L = len(s)
    return tuple(sum((w + 1) * pow(r, L - j, P) for j, w in enumerate(s)) % P for r in BASES)


class Store:
    """Bookkeeping model of the pool: key -> (offset, bytes), least recently used first."""

    def __init__(self, pool_bytes: int):
        self.pool_bytes = pool_bytes - pool_bytes % ALIGN
        self.entries: "OrderedDict[Tuple[int, int], Tuple[int, int]]" = OrderedDict()
        self.hits = self.misses = self.evictions = 0

    @staticmethod
    def _round(n: int) -> int:
        return (n + ALIGN - 1) // ALIGN * ALIGN

    def lookup(self, key) -> Optional[Tuple[int, int]]:
        if key in self.entries:
            self.entries.move_to_end(key)
            self.hits += 1
            return self.entries[key]
        self.misses += 1
        return None

    def _first_fit(self, need: int) -> Optional[int]:
        pos = 0
        for off, size in sorted(self.entries.values()):
            if off - pos >= need:
                return pos
            pos = off + self._round(size)
        return pos if self.pool_bytes - pos >= need else None

    def insert(self, key, nbytes: int) -> Optional[int]:
        """Offset of the new entry, or None when it can never fit.  An existing key is replaced."""
        need = self._round(nbytes)
        if nbytes <= 0 or need > self.pool_bytes:
            return None
        self.entries.pop(key, None)
        while True:
            off = self._first_fit(need)
            if off is not None:
                break
            self.entries.popitem(last=False)
            self.evictions += 1
        self.entries[key] = (off, nbytes)
        return off
