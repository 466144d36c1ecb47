"""Pins of the chunk-prefix keys: the published FNV-1a test vectors, the chaining property,
and the longest-prefix rule of App. A step 2."""
import numpy as np

from oracle import prefix as opx


def test_fnv1a64_published_vectors():
    # vectors from the FNV reference test suite
    assert opx.fnv1a64(b"") == 0xCBF29CE484222325
    assert opx.fnv1a64(b"a") == 0xAF63DC4C8601EC8C
    assert opx.fnv1a64(b"b") == 0xAF63DF4C8601F1A5
    assert opx.fnv1a64(b"foobar") == 0x85944171F73967E8


def test_prefix_keys_chain():
    rng = np.random.default_rng(0)
    toks = rng.integers(0, 32000, 1000).astype(np.int32)
    keys = opx.prefix_keys(toks, 128)
    assert len(keys) == 7 and len(set(keys)) == 7                      # full chunks only; the ragged tail has no key
    # a key is a function of the whole prefix, not of its chunk alone
    same_chunk_elsewhere = np.concatenate([toks[128:256], toks[128:256]])
    assert opx.prefix_keys(same_chunk_elsewhere, 128)[1] != keys[1]
    assert opx.prefix_keys(same_chunk_elsewhere, 128)[0] != keys[1]
    # changing one token changes that chunk's key and every later one, none before
    t2 = toks.copy()
    t2[300] += 1
    k2 = opx.prefix_keys(t2, 128)
    assert k2[:2] == keys[:2] and all(a != b for a, b in zip(k2[2:], keys[2:]))
    # first key written out by hand: basis bytes then the ids, little-endian
    data = (0xCBF29CE484222325).to_bytes(8, "little") + toks[:128].astype("<i4").tobytes()
    assert keys[0] == opx.fnv1a64(data)
    # a longer prompt with the same beginning shares the keys of the common chunks
    assert opx.prefix_keys(np.concatenate([toks, toks]), 128)[:7] == keys


def test_longest_stored_prefix():
    keys = [11, 22, 33, 44]
    assert opx.longest_stored_prefix(keys, [11, 22, 33, 44, 55]) == 4
    assert opx.longest_stored_prefix(keys, [11, 22, 44]) == 2          # a later hit behind a gap does not count
    assert opx.longest_stored_prefix(keys, [22, 33]) == 0
    assert opx.longest_stored_prefix([], [1]) == 0
