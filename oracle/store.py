"""Oracle: byte images of the stored KV ("we precompute and store all requests'
KV in advance", Sec. 5.1 "Datasets").  Test infrastructure only.

The storage tier holds one image per logical page of ``page_tokens`` tokens.
An image is, for every layer, the layer's K block followed by its V block:

    image[layer][0][kv_head][token_in_page][hd]      K, rotated, as cached
    image[layer][1][kv_head][hd][token_in_page]      V, stored transposed

in the cache's element type.  Token slots past the end of the prompt are zero.
This is an interface format, restated here from its description; the oracle
does no arithmetic on the values beyond the storage rounding already applied
by ``transformer.round_storage``.
"""
from __future__ import annotations

import numpy as np

from .transformer import KVCache


def _encode(x: np.ndarray, dtype: str) -> np.ndarray:
    """fp64 values (already representable in ``dtype``) -> raw storage words."""
    x32 = np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "f32":
        return x32.view(np.uint32)
    if dtype == "bf16":
        return (x32.view(np.uint32) >> np.uint32(16)).astype(np.uint16)
    raise ValueError(dtype)


def decode_words(words: np.ndarray, dtype: str) -> np.ndarray:
    """Raw storage words -> float64 values (a reinterpretation, no rounding)."""
    if dtype == "f32":
        return words.view(np.float32).astype(np.float64)
    if dtype == "bf16":
        return (words.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    raise ValueError(dtype)


def page_image_words(n_layers: int, n_kv: int, hd: int, page_tokens: int) -> int:
    return n_layers * 2 * n_kv * page_tokens * hd


def pack_store(cache: KVCache, page_tokens: int, dtype: str) -> np.ndarray:
    """[n_logical_pages, L, 2, n_kv * page_tokens * hd] storage words."""
    L, T, n_kv, hd = cache.k.shape
    n_pages = (T + page_tokens - 1) // page_tokens
    wdt = np.uint32 if dtype == "f32" else np.uint16
    out = np.zeros((n_pages, L, 2, n_kv * page_tokens * hd), dtype=wdt)
    for p in range(n_pages):
        t0, t1 = p * page_tokens, min((p + 1) * page_tokens, T)
        n = t1 - t0
        for l in range(L):
            kblk = np.zeros((n_kv, page_tokens, hd), dtype=np.float64)
            vblk = np.zeros((n_kv, hd, page_tokens), dtype=np.float64)
            kblk[:, :n, :] = np.transpose(cache.k[l, t0:t1], (1, 0, 2))   # [kv, tok, hd]
            vblk[:, :, :n] = np.transpose(cache.v[l, t0:t1], (1, 2, 0))   # [kv, hd, tok]
            out[p, l, 0] = _encode(kblk, dtype).reshape(-1)
            out[p, l, 1] = _encode(vblk, dtype).reshape(-1)
    return out


def unpack_store(images: np.ndarray, n_tokens: int, n_kv: int, hd: int,
                 page_tokens: int, dtype: str) -> KVCache:
    """Inverse of ``pack_store``."""
    n_pages, L = images.shape[0], images.shape[1]
    cache = KVCache(L, n_tokens, n_kv, hd)
    for p in range(n_pages):
        t0, t1 = p * page_tokens, min((p + 1) * page_tokens, n_tokens)
        n = t1 - t0
        for l in range(L):
            kblk = decode_words(images[p, l, 0], dtype).reshape(n_kv, page_tokens, hd)
            vblk = decode_words(images[p, l, 1], dtype).reshape(n_kv, hd, page_tokens)
            cache.k[l, t0:t1] = np.transpose(kblk[:, :n, :], (1, 0, 2))
            cache.v[l, t0:t1] = np.transpose(vblk[:, :, :n], (2, 0, 1))
    cache.filled = n_tokens
    return cache


# --------------------------------------------------------------------------- #
# 8-bit stored KV (Sec. 5.5: KV compression combined with the method, "the most common
# 8-bit quantization"; the paper names no scheme)
# --------------------------------------------------------------------------- #
# Reading taken here: symmetric absmax quantisation of every (token, KV head) row of head_dim
# values, for K (as cached, rotated) and V alike:
#     scale = max|x| / 127            code = round_half_even(x / scale), clipped to [-127, 127]
#     x'    = storage_round(code * scale)
# with scale and both products / quotients in float32 (the GPU's precision; these steps decide
# integers and stored bit patterns, so the oracle takes them in that precision too).  A row of
# zeros has scale 0 and codes 0.  An image of one page, per layer and per K|V:
#     int8   codes [kv_head][token_in_page][hd]      (V is NOT transposed in this format)
#     float32 scales [kv_head][token_in_page]
# i.e. n_kv * page_tokens * (hd + 4) bytes against 2 * n_kv * page_tokens * hd for bf16.

def quantize_rows_int8(x: np.ndarray):
    """x [..., hd] (values exactly representable in float32) -> (int8 codes, float32 scales [...])."""
    x32 = np.ascontiguousarray(x, dtype=np.float32)
    scale = (np.abs(x32).max(axis=-1) / np.float32(127.0)).astype(np.float32)
    safe = np.where(scale > 0, scale, np.float32(1.0)).astype(np.float32)
    q = np.rint((x32 / safe[..., None]).astype(np.float32))
    q = np.clip(q, -127, 127).astype(np.int8)
    q[scale == 0] = 0
    return q, scale


def dequantize_rows_int8(codes: np.ndarray, scale: np.ndarray, dtype: str) -> np.ndarray:
    """code * scale in float32, then the storage rounding of ``dtype``; returned as float64."""
    from .transformer import round_storage
    x32 = (codes.astype(np.float32) * scale[..., None].astype(np.float32)).astype(np.float32)
    return round_storage(x32.astype(np.float64), dtype)


def int8_image_bytes(n_layers: int, n_kv: int, hd: int, page_tokens: int) -> int:
    return n_layers * 2 * n_kv * page_tokens * (hd + 4)


def pack_store_int8(cache: KVCache, page_tokens: int) -> np.ndarray:
    """[n_logical_pages, L, 2, n_kv * page_tokens * (hd + 4)] bytes (uint8)."""
    L, T, n_kv, hd = cache.k.shape
    n_pages = (T + page_tokens - 1) // page_tokens
    nc = n_kv * page_tokens * hd
    out = np.zeros((n_pages, L, 2, n_kv * page_tokens * (hd + 4)), dtype=np.uint8)
    for p in range(n_pages):
        t0, t1 = p * page_tokens, min((p + 1) * page_tokens, T)
        n = t1 - t0
        for l in range(L):
            for which, src in ((0, cache.k), (1, cache.v)):
                blk = np.zeros((n_kv, page_tokens, hd), dtype=np.float64)
                blk[:, :n, :] = np.transpose(src[l, t0:t1], (1, 0, 2))        # [kv, tok, hd]
                q, sc = quantize_rows_int8(blk)
                out[p, l, which, :nc] = q.reshape(-1).view(np.uint8)
                out[p, l, which, nc:] = sc.reshape(-1).view(np.uint8)
    return out


def unpack_store_int8(images: np.ndarray, n_tokens: int, n_kv: int, hd: int,
                      page_tokens: int, dtype: str) -> KVCache:
    """The cache a loader must produce from int8 images: dequantised and storage-rounded."""
    n_pages, L = images.shape[0], images.shape[1]
    nc = n_kv * page_tokens * hd
    cache = KVCache(L, n_tokens, n_kv, hd)
    for p in range(n_pages):
        t0, t1 = p * page_tokens, min((p + 1) * page_tokens, n_tokens)
        n = t1 - t0
        for l in range(L):
            for which, dst in ((0, cache.k), (1, cache.v)):
                q = images[p, l, which, :nc].view(np.int8).reshape(n_kv, page_tokens, hd)
                sc = np.ascontiguousarray(images[p, l, which, nc:]).view(np.float32).reshape(n_kv, page_tokens)
                x = dequantize_rows_int8(q, sc, dtype)
                dst[l, t0:t1] = np.transpose(x[:, :n, :], (1, 0, 2))
    cache.filled = n_tokens
    return cache


# --------------------------------------------------------------------------- #
# 4-bit stored KV (Sec. 5.5 / Table 6 pair the method with a second, stronger compression level;
# the paper takes a published 3-bit scheme that needs calibration data, so it is not reproduced)
# --------------------------------------------------------------------------- #
# Reading taken here: the 8-bit scheme above with 15 levels instead of 255:
#     scale = max|x| / 7             code = round_half_even(x / scale), clipped to [-7, 7]
# again in float32, one scale per (token, KV head) row.  Two codes share a byte: element 2i in the
# low nibble, element 2i+1 in the high nibble, each as a 4-bit two's complement number.  An image
# of one page, per layer and per K|V:
#     uint8  packed codes [kv_head][token_in_page][hd / 2]
#     float32 scales      [kv_head][token_in_page]
# i.e. n_kv * page_tokens * (hd / 2 + 4) bytes.

def quantize_rows_int4(x: np.ndarray):
    """x [..., hd] -> (int8 codes in [-7, 7], float32 scales [...])."""
    x32 = np.ascontiguousarray(x, dtype=np.float32)
    scale = (np.abs(x32).max(axis=-1) / np.float32(7.0)).astype(np.float32)
    safe = np.where(scale > 0, scale, np.float32(1.0)).astype(np.float32)
    q = np.rint((x32 / safe[..., None]).astype(np.float32))
    q = np.clip(q, -7, 7).astype(np.int8)
    q[scale == 0] = 0
    return q, scale


def pack_nibbles(codes: np.ndarray) -> np.ndarray:
    """int8 codes [..., hd] in [-8, 7] -> uint8 [..., hd / 2]; even element low, odd element high."""
    u = codes.astype(np.int16) & 0xF
    return (u[..., 0::2] | (u[..., 1::2] << 4)).astype(np.uint8)


def unpack_nibbles(packed: np.ndarray) -> np.ndarray:
    """Inverse of pack_nibbles: uint8 [..., n] -> int8 [..., 2 n] (sign-extended nibbles)."""
    lo = (packed & 0xF).astype(np.int16)
    hi = (packed >> 4).astype(np.int16)
    lo = np.where(lo >= 8, lo - 16, lo)
    hi = np.where(hi >= 8, hi - 16, hi)
    out = np.empty(packed.shape[:-1] + (packed.shape[-1] * 2,), dtype=np.int8)
    out[..., 0::2] = lo
    out[..., 1::2] = hi
    return out


def int4_image_bytes(n_layers: int, n_kv: int, hd: int, page_tokens: int) -> int:
    return n_layers * 2 * n_kv * page_tokens * (hd // 2 + 4)


def pack_store_int4(cache: KVCache, page_tokens: int) -> np.ndarray:
    """[n_logical_pages, L, 2, n_kv * page_tokens * (hd / 2 + 4)] bytes (uint8)."""
    L, T, n_kv, hd = cache.k.shape
    n_pages = (T + page_tokens - 1) // page_tokens
    nc = n_kv * page_tokens * (hd // 2)
    out = np.zeros((n_pages, L, 2, n_kv * page_tokens * (hd // 2 + 4)), dtype=np.uint8)
    for p in range(n_pages):
        t0, t1 = p * page_tokens, min((p + 1) * page_tokens, T)
        n = t1 - t0
        for l in range(L):
            for which, src in ((0, cache.k), (1, cache.v)):
                blk = np.zeros((n_kv, page_tokens, hd), dtype=np.float64)
                blk[:, :n, :] = np.transpose(src[l, t0:t1], (1, 0, 2))        # [kv, tok, hd]
                q, sc = quantize_rows_int4(blk)
                out[p, l, which, :nc] = pack_nibbles(q).reshape(-1)
                out[p, l, which, nc:] = sc.reshape(-1).view(np.uint8)
    return out


def unpack_store_int4(images: np.ndarray, n_tokens: int, n_kv: int, hd: int,
                      page_tokens: int, dtype: str) -> KVCache:
    """The cache a loader must produce from 4-bit images: dequantised and storage-rounded."""
    n_pages, L = images.shape[0], images.shape[1]
    nc = n_kv * page_tokens * (hd // 2)
    cache = KVCache(L, n_tokens, n_kv, hd)
    for p in range(n_pages):
        t0, t1 = p * page_tokens, min((p + 1) * page_tokens, n_tokens)
        n = t1 - t0
        for l in range(L):
            for which, dst in ((0, cache.k), (1, cache.v)):
                q = unpack_nibbles(images[p, l, which, :nc].reshape(n_kv, page_tokens, hd // 2))
                sc = np.ascontiguousarray(images[p, l, which, nc:]).view(np.float32).reshape(n_kv, page_tokens)
                x = dequantize_rows_int8(q, sc, dtype)      # code * scale, storage-rounded: same rule for both widths
                dst[l, t0:t1] = np.transpose(x[:, :n, :], (1, 0, 2))
    cache.filled = n_tokens
    return cache
