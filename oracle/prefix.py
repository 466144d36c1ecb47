"""Oracle: chunk-prefix keys and the longest stored prefix (App. A, step 2: hash every chunk
prefix, find the last one the storage backend holds, that fixes how many tokens can be loaded;
App. B: the store "hashes token chunks into keys").  Test infrastructure only.

The paper names no hash.  Reading taken: the key of chunk i covers the whole prefix up to and
including chunk i by chaining,
    key_i = FNV-1a-64( 8 bytes of key_{i-1}, little-endian  ||  the chunk's token ids as
                       little-endian 32-bit integers ),      key_{-1} = the FNV offset basis,
over full chunks only (a ragged tail is never a stored chunk).  FNV-1a is the published
Fowler-Noll-Vo function: h = basis; for each byte: h = (h xor byte) * prime mod 2^64.
"""
from __future__ import annotations

from typing import Iterable, List, Sequence

import numpy as np

FNV64_BASIS = 0xCBF29CE484222325
FNV64_PRIME = 0x100000001B3
_MASK = (1 << 64) - 1


def fnv1a64(data: bytes, h: int = FNV64_BASIS) -> int:
    for byte in data:
        h = ((h ^ byte) * FNV64_PRIME) & _MASK
    return h


def prefix_keys(tokens: Sequence[int], chunk: int) -> List[int]:
    """One key per full chunk; key i identifies tokens [0, (i+1)*chunk)."""
    toks = np.asarray(tokens, dtype="<i4")
    keys, prev = [], FNV64_BASIS
    for i in range(len(toks) // chunk):
        prev = fnv1a64(int(prev).to_bytes(8, "little") + toks[i * chunk:(i + 1) * chunk].tobytes())
        keys.append(prev)
    return keys


def longest_stored_prefix(keys: Sequence[int], stored: Iterable[int]) -> int:
    """Number of leading chunks whose key the store holds (the paper's total_tokens / chunk)."""
    have = set(int(k) for k in stored)
    n = 0
    for k in keys:
        if int(k) not in have:
            break
        n += 1
    return n
