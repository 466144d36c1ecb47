"""Oracle: the KV cache of a decoder-only prompt, in fp64 NumPy.  Test infrastructure only.

What is computed (paper Sec. 3, "Attention and KV cache"): for every layer the
keys K = X W_K and values V = X W_V of every prompt token, where X is the
layer's input produced by ordinary causal self-attention
softmax(Q K^T / sqrt(d_k)) V over all earlier tokens.  Sec. 3 "Chunk Prefill"
and Sec. 4 Part 2 only change *when* and *by whom* a token's K/V are produced,
never their values, so the oracle is the plain definition written three ways:

* ``prefill_monolithic``      all T tokens at once under a causal mask;
* ``prefill_chunked``         chunk by chunk against the cached earlier K/V;
* ``prefill_token_by_token``  one token at a time (the decode recurrence).

The paper fixes none of the block internals (it runs "LLaMA 2 / LLaMA 3.1"
models through an inference engine, Sec. 5.1 "Models"); the block below is the
Llama block the benchmark configurations name: pre-RMSNorm, rotary position
embedding on q and k with adjacent-pair rotation (2i, 2i+1), grouped-query
attention (query head j reads KV head j // (n_q / n_kv)), SwiGLU feed-forward,
no biases.  K is cached after the rotation.

Precision: everything is float64.  ``kv_dtype`` says in which type the cache
*stores* K and V ("f32", "bf16" or None = keep fp64): values are rounded once
at the cache write and attention then reads the cached (rounded) values, as a
real KV cache does (Sec. 5.1: BF16 is the default KV-cache type).

Weights use the paper's orientation Q = X W_Q: every matrix is [in, out].
"""
from __future__ import annotations

from typing import Dict, List, Optional, Tuple

import numpy as np

F64 = np.float64


# --------------------------------------------------------------------------- #
# storage rounding
# --------------------------------------------------------------------------- #
def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round to the nearest bfloat16 (ties to even); result returned as float64."""
    x32 = np.asarray(x, dtype=np.float32)
    u = x32.view(np.uint32).astype(np.uint64)
    lsb = (u >> np.uint64(16)) & np.uint64(1)
    u = (u + np.uint64(0x7FFF) + lsb) & np.uint64(0xFFFF0000)
    return u.astype(np.uint32).view(np.float32).astype(F64)


def round_storage(x: np.ndarray, kv_dtype: Optional[str]) -> np.ndarray:
    if kv_dtype is None:
        return np.asarray(x, dtype=F64)
    if kv_dtype == "f32":
        return np.asarray(x, dtype=np.float32).astype(F64)
    if kv_dtype == "bf16":
        return round_to_bf16(x)
    raise ValueError(f"unknown kv_dtype {kv_dtype!r}")


# --------------------------------------------------------------------------- #
# block pieces
# --------------------------------------------------------------------------- #
def rmsnorm(x: np.ndarray, gain: np.ndarray, eps: float) -> np.ndarray:
    """y = x / sqrt(mean(x^2) + eps) * gain, per row."""
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * gain


def rope(x: np.ndarray, pos: np.ndarray, theta: float) -> np.ndarray:
    """Rotary embedding.  x: [T, heads, hd]; pos: [T] absolute positions.

    Pair i = (x[2i], x[2i+1]) is rotated by the angle pos * theta**(-2i/hd).
    """
    T, H, hd = x.shape
    half = hd // 2
    inv_freq = theta ** (-(2.0 * np.arange(half, dtype=F64)) / hd)          # [half]
    ang = np.asarray(pos, dtype=F64)[:, None] * inv_freq[None, :]            # [T, half]
    c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    xe, xo = x[..., 0::2], x[..., 1::2]
    out = np.empty_like(x, dtype=F64)
    out[..., 0::2] = xe * c - xo * s
    out[..., 1::2] = xe * s + xo * c
    return out


def softmax(s: np.ndarray) -> np.ndarray:
    """Row softmax over the last axis; -inf entries get weight 0."""
    m = np.max(s, axis=-1, keepdims=True)
    e = np.exp(s - m)
    return e / np.sum(e, axis=-1, keepdims=True)


def silu(x: np.ndarray) -> np.ndarray:
    return x / (1.0 + np.exp(-x))


def attention(q: np.ndarray, k: np.ndarray, v: np.ndarray,
              q_pos: np.ndarray, k_pos: np.ndarray) -> np.ndarray:
    """Causal grouped-query attention.

    q: [Tq, n_q, hd]; k, v: [Tk, n_kv, hd]; a query at position p sees the keys
    whose position is <= p.  Returns [Tq, n_q, hd].
    """
    Tq, n_q, hd = q.shape
    n_kv = k.shape[1]
    group = n_q // n_kv
    visible = np.asarray(k_pos)[None, :] <= np.asarray(q_pos)[:, None]       # [Tq, Tk]
    out = np.empty((Tq, n_q, hd), dtype=F64)
    for j in range(n_q):
        g = j // group
        scores = (q[:, j, :] @ k[:, g, :].T) / np.sqrt(F64(hd))
        scores = np.where(visible, scores, -np.inf)
        out[:, j, :] = softmax(scores) @ v[:, g, :]
    return out


def swiglu_ffn(h: np.ndarray, w_gate: np.ndarray, w_up: np.ndarray, w_down: np.ndarray) -> np.ndarray:
    return (silu(h @ w_gate) * (h @ w_up)) @ w_down


# --------------------------------------------------------------------------- #
# prefill
# --------------------------------------------------------------------------- #
def _as64(w: Dict[str, np.ndarray]) -> Dict[str, np.ndarray]:
    return {k: np.asarray(a, dtype=F64) for k, a in w.items()}


class KVCache:
    """K, V of shape [n_layers, T, n_kv, hd] (float64 holding storage-rounded values)."""

    def __init__(self, n_layers: int, n_tokens: int, n_kv: int, hd: int):
        self.k = np.zeros((n_layers, n_tokens, n_kv, hd), dtype=F64)
        self.v = np.zeros((n_layers, n_tokens, n_kv, hd), dtype=F64)
        self.filled = 0


def _block_forward(x: np.ndarray, pos: np.ndarray, lw: Dict[str, np.ndarray], shape,
                   cache: KVCache, layer: int, kv_dtype: Optional[str]) -> np.ndarray:
    """One decoder block on rows x (positions ``pos``, contiguous, starting where the
    cache ends); writes their K/V into the cache and returns the block output."""
    n_q, n_kv, hd = shape.n_q, shape.n_kv, shape.head_dim
    T = x.shape[0]
    t0, t1 = int(pos[0]), int(pos[0]) + T
    h = rmsnorm(x, lw["attn_norm"], shape.rms_eps)
    q = (h @ lw["wq"]).reshape(T, n_q, hd)
    k = (h @ lw["wk"]).reshape(T, n_kv, hd)
    v = (h @ lw["wv"]).reshape(T, n_kv, hd)
    q = rope(q, pos, shape.rope_theta)
    k = rope(k, pos, shape.rope_theta)
    cache.k[layer, t0:t1] = round_storage(k, kv_dtype)
    cache.v[layer, t0:t1] = round_storage(v, kv_dtype)
    a = attention(q, cache.k[layer, :t1], cache.v[layer, :t1], pos, np.arange(t1))
    x = x + a.reshape(T, n_q * hd) @ lw["wo"]
    x = x + swiglu_ffn(rmsnorm(x, lw["ffn_norm"], shape.rms_eps),
                       lw["w_gate"], lw["w_up"], lw["w_down"])
    return x


def prefill_chunked(weights, shape, tokens: np.ndarray, chunk: int,
                    kv_dtype: Optional[str] = None, cache: Optional[KVCache] = None,
                    tok_begin: int = 0, tok_end: Optional[int] = None,
                    return_hidden: bool = False,
                    layer_inputs: Optional[Dict[int, List[np.ndarray]]] = None):
    """Chunk prefill (Sec. 3): tokens [tok_begin, tok_end) in pieces of ``chunk``
    tokens (the last may be shorter), each attending to everything cached before it.
    ``cache`` must already hold [0, tok_begin).  ``layer_inputs``, if given, maps a layer
    index to a list that receives a copy of that layer's input rows for every chunk, in
    order (index ``n_layers`` = the output of the last layer); nothing is computed for it."""
    tokens = np.asarray(tokens)
    T = len(tokens)
    tok_end = T if tok_end is None else tok_end
    layers = [_as64(lw) for lw in weights["layers"]]
    embed = weights["embed"]
    if cache is None:
        cache = KVCache(len(layers), T, shape.n_kv, shape.head_dim)
    hidden = None
    for t0 in range(tok_begin, tok_end, chunk):
        t1 = min(t0 + chunk, tok_end)
        pos = np.arange(t0, t1)
        x = np.asarray(embed[tokens[t0:t1]], dtype=F64)
        for l, lw in enumerate(layers):
            if layer_inputs is not None and l in layer_inputs:
                layer_inputs[l].append(x.copy())
            x = _block_forward(x, pos, lw, shape, cache, l, kv_dtype)
        if layer_inputs is not None and len(layers) in layer_inputs:
            layer_inputs[len(layers)].append(x.copy())
        cache.filled = t1
        hidden = x
    return (cache, hidden) if return_hidden else cache


def prefill_monolithic(weights, shape, tokens: np.ndarray,
                       kv_dtype: Optional[str] = None) -> KVCache:
    """The whole prompt in one pass, attention as one masked T x T matrix per head."""
    tokens = np.asarray(tokens)
    T = len(tokens)
    n_q, n_kv, hd = shape.n_q, shape.n_kv, shape.head_dim
    group = n_q // n_kv
    layers = [_as64(lw) for lw in weights["layers"]]
    cache = KVCache(len(layers), T, n_kv, hd)
    pos = np.arange(T)
    mask = np.tril(np.ones((T, T), dtype=bool))
    x = np.asarray(weights["embed"][tokens], dtype=F64)
    for l, lw in enumerate(layers):
        h = rmsnorm(x, lw["attn_norm"], shape.rms_eps)
        q = rope((h @ lw["wq"]).reshape(T, n_q, hd), pos, shape.rope_theta)
        k = rope((h @ lw["wk"]).reshape(T, n_kv, hd), pos, shape.rope_theta)
        v = (h @ lw["wv"]).reshape(T, n_kv, hd)
        k = round_storage(k, kv_dtype)
        v = round_storage(v, kv_dtype)
        cache.k[l], cache.v[l] = k, v
        a = np.empty((T, n_q, hd), dtype=F64)
        for j in range(n_q):
            s = np.einsum("td,sd->ts", q[:, j], k[:, j // group]) / np.sqrt(F64(hd))
            s = np.where(mask, s, -np.inf)
            a[:, j] = softmax(s) @ v[:, j // group]
        x = x + a.reshape(T, n_q * hd) @ lw["wo"]
        x = x + swiglu_ffn(rmsnorm(x, lw["ffn_norm"], shape.rms_eps),
                           lw["w_gate"], lw["w_up"], lw["w_down"])
    cache.filled = T
    return cache


def prefill_token_by_token(weights, shape, tokens: np.ndarray,
                           kv_dtype: Optional[str] = None) -> KVCache:
    """The decode recurrence: token t computes q_t, k_t, v_t, appends (k_t, v_t) to the
    cache and attends to cache[0..t] with plain vector arithmetic."""
    tokens = np.asarray(tokens)
    T = len(tokens)
    n_q, n_kv, hd = shape.n_q, shape.n_kv, shape.head_dim
    group = n_q // n_kv
    layers = [_as64(lw) for lw in weights["layers"]]
    cache = KVCache(len(layers), T, n_kv, hd)
    for t in range(T):
        x = np.asarray(weights["embed"][tokens[t]], dtype=F64)
        for l, lw in enumerate(layers):
            h = rmsnorm(x[None, :], lw["attn_norm"], shape.rms_eps)
            p = np.array([t])
            q = rope((h @ lw["wq"]).reshape(1, n_q, hd), p, shape.rope_theta)[0]
            k = rope((h @ lw["wk"]).reshape(1, n_kv, hd), p, shape.rope_theta)[0]
            v = (h @ lw["wv"]).reshape(n_kv, hd)
            cache.k[l, t] = round_storage(k, kv_dtype)
            cache.v[l, t] = round_storage(v, kv_dtype)
            a = np.empty((n_q, hd), dtype=F64)
            for j in range(n_q):
                ks, vs = cache.k[l, :t + 1, j // group], cache.v[l, :t + 1, j // group]
                w = ks @ q[j] / np.sqrt(F64(hd))
                w = np.exp(w - w.max())
                a[j] = (w / w.sum()) @ vs
            x = x + a.reshape(-1) @ lw["wo"]
            hf = rmsnorm(x[None, :], lw["ffn_norm"], shape.rms_eps)[0]
            x = x + (silu(hf @ lw["w_gate"]) * (hf @ lw["w_up"])) @ lw["w_down"]
    cache.filled = T
    return cache


# --------------------------------------------------------------------------- #
# the first output token (Sec. 3: prefill ends with it; Sec. 5.1: TTFT is measured up to it)
# --------------------------------------------------------------------------- #
def lm_logits(weights, shape, hidden: np.ndarray) -> np.ndarray:
    """Final RMSNorm and the vocabulary projection of hidden rows [..., d] -> [..., vocab]."""
    h = rmsnorm(np.asarray(hidden, dtype=F64), np.asarray(weights["final_norm"], dtype=F64), shape.rms_eps)
    return h @ np.asarray(weights["lm_head"], dtype=F64)


def first_token_logits(weights, shape, tokens: np.ndarray, cache: KVCache) -> np.ndarray:
    """Logits of the token that follows the prompt, from a COMPLETE cache that is only read:
    the prompt's last token is embedded and taken through every block; in block l its rotated
    query attends to cache.k[l, :T], cache.v[l, :T] exactly as they are (its own position
    included -- after a bidirectional prefill that entry may be a loaded one)."""
    tokens = np.asarray(tokens)
    T = len(tokens)
    n_q, hd = shape.n_q, shape.head_dim
    pos = np.array([T - 1])
    x = np.asarray(weights["embed"][tokens[T - 1]], dtype=F64)[None, :]
    for l, lw in enumerate(weights["layers"]):
        lw = _as64(lw)
        h = rmsnorm(x, lw["attn_norm"], shape.rms_eps)
        q = rope((h @ lw["wq"]).reshape(1, n_q, hd), pos, shape.rope_theta)
        a = attention(q, cache.k[l, :T], cache.v[l, :T], pos, np.arange(T))
        x = x + a.reshape(1, n_q * hd) @ lw["wo"]
        x = x + swiglu_ffn(rmsnorm(x, lw["ffn_norm"], shape.rms_eps), lw["w_gate"], lw["w_up"], lw["w_down"])
    return lm_logits(weights, shape, x[0])


def greedy_token(logits: np.ndarray) -> int:
    """Index of the largest logit; the lowest index among equal ones."""
    return int(np.argmax(logits))


# --------------------------------------------------------------------------- #
# the bidirectional result (Sec. 4 Part 2; App. A steps 4-7)
# --------------------------------------------------------------------------- #
def bidirectional_kv(weights, shape, tokens, chunk: int, meet_chunk: int,
                     stored: KVCache, kv_dtype: Optional[str] = None) -> KVCache:
    """KV cache when chunks [0, meet_chunk) are computed front-to-back and chunks
    [meet_chunk, N) are taken from ``stored`` as they are.  The computed part never
    reads a loaded chunk (a token attends only to earlier ones)."""
    T = len(tokens)
    split_tok = min(meet_chunk * chunk, T)
    out = KVCache(len(weights["layers"]), T, shape.n_kv, shape.head_dim)
    if split_tok > 0:
        prefill_chunked(weights, shape, tokens, chunk, kv_dtype, cache=out,
                        tok_begin=0, tok_end=split_tok)
    out.k[:, split_tok:] = stored.k[:, split_tok:]
    out.v[:, split_tok:] = stored.v[:, split_tok:]
    out.filled = T
    return out


# --------------------------------------------------------------------------- #
# sizes and work (Table 1; Sec. 4 Part 2 insight)
# --------------------------------------------------------------------------- #
def kv_bytes_per_token(n_layers: int, n_kv: int, head_dim: int, elem_bytes: int = 2) -> int:
    """K and V, every layer, every KV head (Table 1, "KV-size/Token")."""
    return 2 * n_layers * n_kv * head_dim * elem_bytes


def chunk_flops(shape, chunk_index: int, chunk: int) -> int:
    """Multiply-add work of prefilling one full chunk: projections (constant per chunk)
    plus causal attention against (chunk_index + 1) chunks (grows with the index --
    the insight of Sec. 4 Part 2).  The masked half of the diagonal block is not counted."""
    d, hd = shape.d_model, shape.head_dim
    hq, hkv, ff, L = shape.n_q * hd, shape.n_kv * hd, shape.ffn, shape.n_layers
    p_lin = L * (d * hq + 2 * d * hkv + hq * d + 3 * d * ff)
    pairs = chunk_index * chunk * chunk + chunk * (chunk + 1) // 2
    return 2 * p_lin * chunk + L * 4 * hq * pairs
