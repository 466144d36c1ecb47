"""Pins for oracle/transformer.py: values the paper prints, hand-worked models, closed
forms, special cases and invariants.  None of these re-use the oracle's own formulas as
the expected value; a dropped term, wrong sign/index or transposed operand in the oracle
fails at least one of them."""
import math

import numpy as np
import pytest

import synth_inputs as si
from oracle import transformer as otf
from oracle import store as ostore


# ----------------------------------------------------------------------------- Table 1
def test_kv_bytes_per_token_matches_table1(golden):
    for model, layers, kvh, hd, kb in golden("table1_kv_size.txt"):
        got = otf.kv_bytes_per_token(int(layers), int(kvh), int(hd), elem_bytes=2)
        assert got == int(kb) * 1024, model


def test_kv_bytes_of_benchmark_shapes():
    # the three bf16 benchmark shapes are Table 1's 7B / 8B / 70B rows
    for shape, kb in ((si.LLAMA2_7B, 512), (si.LLAMA3_8B, 128), (si.LLAMA2_70B, 320)):
        assert otf.kv_bytes_per_token(shape.n_layers, shape.n_kv, shape.head_dim, 2) == kb * 1024
    cache = otf.KVCache(si.TINY.n_layers, 3, si.TINY.n_kv, si.TINY.head_dim)
    assert (cache.k[:, 0].size + cache.v[:, 0].size) * 4 == 4096     # 4 KiB / token, fp32


# ----------------------------------------------------------------------------- pieces
def test_rmsnorm_hand_values():
    # x = (3, 4): mean square 12.5, so y = x / sqrt(12.5) times the gain
    y = otf.rmsnorm(np.array([[3.0, 4.0]]), np.array([2.0, 0.5]), 0.0)
    np.testing.assert_allclose(y, [[2 * 3 / math.sqrt(12.5), 0.5 * 4 / math.sqrt(12.5)]], rtol=1e-15)
    # eps enters under the root: x = (1, 1), eps = 3 -> 1 / sqrt(1 + 3) = 1/2
    y = otf.rmsnorm(np.array([[1.0, 1.0]]), np.ones(2), 3.0)
    np.testing.assert_allclose(y, [[0.5, 0.5]], rtol=1e-15)


def test_rope_hand_values_and_properties():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((5, 3, 8))
    # position 0 is the identity
    np.testing.assert_array_equal(otf.rope(x, np.zeros(5), 10000.0), x)
    # head_dim 2, position 1: a plain rotation by one radian; (1,0) -> (cos 1, sin 1)
    y = otf.rope(np.array([[[1.0, 0.0]]]), np.array([1]), 10000.0)
    np.testing.assert_allclose(y[0, 0], [0.5403023058681398, 0.8414709848078965], rtol=1e-15)
    # pair i turns by pos * theta^(-2i/hd): hd 4, theta 100 -> second pair by pos/10
    y = otf.rope(np.array([[[0.0, 0.0, 1.0, 0.0]]]), np.array([5]), 100.0)
    np.testing.assert_allclose(y[0, 0], [0, 0, math.cos(0.5), math.sin(0.5)], atol=1e-15)
    # rotations keep every pair's length
    pos = np.array([0, 1, 7, 100, 4095])
    y = otf.rope(x, pos, 10000.0)
    np.testing.assert_allclose(y[..., 0::2] ** 2 + y[..., 1::2] ** 2,
                               x[..., 0::2] ** 2 + x[..., 1::2] ** 2, rtol=1e-12)
    # q.k depends on the position difference only
    q, k = rng.standard_normal((1, 1, 8)), rng.standard_normal((1, 1, 8))
    d1 = np.sum(otf.rope(q, [13], 1e4) * otf.rope(k, [4], 1e4))
    d2 = np.sum(otf.rope(q, [109], 1e4) * otf.rope(k, [100], 1e4))
    assert abs(d1 - d2) < 1e-12


def test_softmax_and_silu():
    s = np.array([[0.0, math.log(2.0), -np.inf], [1000.0, 1000.0, 1000.0]])
    p = otf.softmax(s)
    np.testing.assert_allclose(p, [[1 / 3, 2 / 3, 0.0], [1 / 3, 1 / 3, 1 / 3]], rtol=1e-15)
    # silu(ln 3) = ln 3 * 3/4 ; silu(0) = 0 ; silu(-ln 3) = -ln 3 / 4
    np.testing.assert_allclose(otf.silu(np.array([math.log(3), 0.0, -math.log(3)])),
                               [0.75 * math.log(3), 0.0, -0.25 * math.log(3)], rtol=1e-15)


def test_attention_special_cases():
    rng = np.random.default_rng(1)
    T, hd = 6, 4
    v = rng.standard_normal((T, 1, hd))
    k = rng.standard_normal((T, 1, hd))
    pos = np.arange(T)
    # zero queries -> uniform weights over the visible keys -> running mean of V
    out = otf.attention(np.zeros((T, 1, hd)), k, v, pos, pos)
    want = np.cumsum(v[:, 0], axis=0) / np.arange(1, T + 1)[:, None]
    np.testing.assert_allclose(out[:, 0], want, rtol=1e-13)
    # the 1/sqrt(hd) scale: q.k = 2 ln 2 with hd = 4 gives logits (0, ln 2) -> weights 1/3, 2/3
    q = np.zeros((2, 1, 4)); q[1, 0, 0] = 1.0
    k2 = np.zeros((2, 1, 4)); k2[1, 0, 0] = 2 * math.log(2.0)
    v2 = np.array([[[3.0, 0, 0, 0]], [[0.0, 3.0, 0, 0]]])
    out = otf.attention(q, k2, v2, np.arange(2), np.arange(2))
    np.testing.assert_allclose(out[1, 0], [1.0, 2.0, 0, 0], rtol=1e-14)
    np.testing.assert_allclose(out[0, 0], [3.0, 0, 0, 0], rtol=1e-14)      # token 0 sees itself only
    # a chunk of queries at positions 4..5 against 6 cached keys = rows 4..5 of the full result
    qf = rng.standard_normal((T, 1, hd))
    full = otf.attention(qf, k, v, pos, pos)
    part = otf.attention(qf[4:], k, v, pos[4:], pos)
    np.testing.assert_array_equal(full[4:], part)


def test_gqa_equals_mha_with_repeated_kv():
    rng = np.random.default_rng(2)
    T, n_q, n_kv, hd = 5, 6, 2, 4
    q = rng.standard_normal((T, n_q, hd))
    k = rng.standard_normal((T, n_kv, hd))
    v = rng.standard_normal((T, n_kv, hd))
    pos = np.arange(T)
    g = otf.attention(q, k, v, pos, pos)
    # query heads 0,1,2 read KV head 0 and 3,4,5 read KV head 1
    m = otf.attention(q, np.repeat(k, 3, axis=1), np.repeat(v, 3, axis=1), pos, pos)
    np.testing.assert_allclose(g, m, rtol=1e-14)
    single = otf.attention(q[:, 4:5], k[:, 1:2], v[:, 1:2], pos, pos)
    np.testing.assert_allclose(g[:, 4:5], single, rtol=1e-14)


# ----------------------------------------------------------------------------- hand model
def _hand_shape(n_layers):
    return si.ModelShape("hand", n_layers, 2, 1, 1, 2, 1, 2, "f32", rms_eps=0.0, rope_theta=10000.0)


def _hand_layer1():
    return dict(attn_norm=np.array([2.0, 3.0]),
                wq=np.array([[1.0, 2.0], [0.0, 1.0]]),
                wk=np.array([[0.0, 1.0], [1.0, 0.0]]),
                wv=np.array([[1.0, 0.0], [1.0, 1.0]]),
                wo=np.array([[1.0, 1.0], [0.0, 2.0]]),
                ffn_norm=np.array([math.sqrt(90.0) / 6.0, math.sqrt(90.0) / 12.0]),
                w_gate=np.array([[math.log(3.0)], [0.0]]),
                w_up=np.array([[2.0], [1.0]]),
                w_down=np.array([[1.0, -1.0]]))


def test_hand_worked_two_token_layer():
    """d = hd = 2, one head.  Embeddings (1,1) and (1,-1) have unit mean square, so with
    gain (2,3) the normed rows are (2,3) and (2,-3).  K = h W_K swaps the entries:
    (3,2), (-3,2); V = h W_V = (h0+h1, h1): (5,3), (-1,-3).  Token 1 sits at position 1,
    its single pair turns by one radian: k1 = (-3c-2s, -3s+2c) with c=cos 1, s=sin 1."""
    shape = _hand_shape(1)
    w = {"embed": np.array([[1.0, 1.0], [1.0, -1.0]]), "layers": [_hand_layer1()]}
    for fn in (lambda: otf.prefill_monolithic(w, shape, [0, 1]),
               lambda: otf.prefill_chunked(w, shape, [0, 1], 1),
               lambda: otf.prefill_chunked(w, shape, [0, 1], 2),
               lambda: otf.prefill_token_by_token(w, shape, [0, 1])):
        c = fn()
        np.testing.assert_allclose(c.k[0, 0, 0], [3.0, 2.0], rtol=1e-14)
        np.testing.assert_allclose(c.k[0, 1, 0], [-3.3038488872202123, -1.4438083426874098], rtol=1e-14)
        np.testing.assert_allclose(c.v[0, 0, 0], [5.0, 3.0], rtol=1e-14)
        np.testing.assert_allclose(c.v[0, 1, 0], [-1.0, -3.0], rtol=1e-14)


def test_hand_worked_single_token_two_layers():
    """One token: attention returns v.  Layer 1: v = (5,3); a W_O = (5, 5+6) = (5,11);
    x = (1,1)+(5,11) = (6,12), mean square 90; the FFN gain is chosen so the normed row is
    (1,1); gate = ln 3 -> silu = 0.75 ln 3; up = 3; down (1,-1) -> +-2.25 ln 3;
    x' = (6 + 2.25 ln 3, 12 - 2.25 ln 3) = (8.4718776495, 9.5281223505).
    Layer 2 (gain 1): h = x'/rms(x') = (0.93970325475, 1.05686223938);
    K = h [[2,0],[1,1]] = (2h0+h1, h1); V = h [[0,1],[1,0]] = (h1, h0)."""
    shape = _hand_shape(2)
    l2 = dict(_hand_layer1())
    l2.update(attn_norm=np.ones(2), wk=np.array([[2.0, 0.0], [1.0, 1.0]]),
              wv=np.array([[0.0, 1.0], [1.0, 0.0]]))
    w = {"embed": np.array([[1.0, 1.0], [1.0, -1.0]]), "layers": [_hand_layer1(), l2]}
    for fn in (lambda: otf.prefill_monolithic(w, shape, [0]),
               lambda: otf.prefill_chunked(w, shape, [0], 4),
               lambda: otf.prefill_token_by_token(w, shape, [0])):
        c = fn()
        np.testing.assert_allclose(c.k[1, 0, 0], [2.9362687488682573, 1.0568622393765779], rtol=1e-13)
        np.testing.assert_allclose(c.v[1, 0, 0], [1.0568622393765779, 0.9397032547458398], rtol=1e-13)


# ----------------------------------------------------------------------------- invariants
SMALL = si.ModelShape("small", 3, 32, 4, 2, 8, 48, 50, "f32")


def _small_weights(seed=3):
    return si.make_weights(SMALL, seed=seed, std=0.3, gain_jitter=0.2)


def test_three_prefills_agree():
    """Chunk prefill is exact (Sec. 3): any chunking, down to one token, gives the KV of
    the monolithic pass.  Large weights (std 0.3) make attention far from uniform."""
    w = _small_weights()
    toks = si.make_tokens(37, SMALL.vocab, seed=5)
    mono = otf.prefill_monolithic(w, SMALL, toks)
    tbt = otf.prefill_token_by_token(w, SMALL, toks)
    np.testing.assert_allclose(tbt.k, mono.k, rtol=0, atol=1e-11)
    np.testing.assert_allclose(tbt.v, mono.v, rtol=0, atol=1e-11)
    for chunk in (1, 5, 8, 16, 37, 64):           # 5 and 8 and 16 do not divide 37
        ch = otf.prefill_chunked(w, SMALL, toks, chunk)
        np.testing.assert_allclose(ch.k, mono.k, rtol=0, atol=1e-11)
        np.testing.assert_allclose(ch.v, mono.v, rtol=0, atol=1e-11)
    assert np.abs(mono.k[2]).max() > 0.1 and np.abs(mono.v[2]).max() > 0.1


def test_causality_and_dependence():
    w = _small_weights()
    toks = si.make_tokens(20, SMALL.vocab, seed=6)
    base = otf.prefill_monolithic(w, SMALL, toks)
    t2 = toks.copy(); t2[12] = (t2[12] + 1) % SMALL.vocab
    alt = otf.prefill_monolithic(w, SMALL, t2)
    np.testing.assert_array_equal(alt.k[:, :12], base.k[:, :12])      # earlier tokens unaffected
    np.testing.assert_array_equal(alt.v[:, :12], base.v[:, :12])
    # later tokens of deeper layers do depend on it (attention really mixes tokens)
    assert np.abs(alt.k[1:, 13:] - base.k[1:, 13:]).max() > 1e-6
    # layer 0 K/V of later tokens depend only on their own token
    np.testing.assert_array_equal(alt.k[0, 13:], base.k[0, 13:])


def test_every_weight_matters():
    """Zeroing any one tensor of layer 0 changes the KV of layer 1 (nothing is dropped)."""
    w = _small_weights()
    toks = si.make_tokens(9, SMALL.vocab, seed=7)
    base = otf.prefill_monolithic(w, SMALL, toks)
    for name in ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down"):
        w2 = {"embed": w["embed"], "layers": [dict(l) for l in w["layers"]]}
        w2["layers"][0][name] = np.zeros_like(w["layers"][0][name])
        alt = otf.prefill_monolithic(w2, SMALL, toks)
        assert np.abs(alt.k[1] - base.k[1]).max() > 1e-9, name
    for name in ("attn_norm", "ffn_norm"):
        w2 = {"embed": w["embed"], "layers": [dict(l) for l in w["layers"]]}
        w2["layers"][0][name] = w["layers"][0][name] * 1.5
        alt = otf.prefill_monolithic(w2, SMALL, toks)
        assert np.abs(alt.k[1] - base.k[1]).max() > 1e-9, name


def test_residual_only_block_is_identity():
    """With W_O = 0 and W_down = 0 a block passes x through, so layer 1 sees the raw
    embeddings: its V is then rmsnorm(embedding) W_V, checked against a direct product."""
    w = _small_weights()
    for l in w["layers"]:
        l["wo"] = np.zeros_like(l["wo"]); l["w_down"] = np.zeros_like(l["w_down"])
    toks = si.make_tokens(7, SMALL.vocab, seed=8)
    c = otf.prefill_monolithic(w, SMALL, toks)
    x = w["embed"][toks].astype(np.float64)
    for l in range(SMALL.n_layers):
        g = w["layers"][l]["attn_norm"].astype(np.float64)
        h = x / np.sqrt((x * x).mean(-1, keepdims=True) + SMALL.rms_eps) * g
        want = (h @ w["layers"][l]["wv"].astype(np.float64)).reshape(7, SMALL.n_kv, SMALL.head_dim)
        np.testing.assert_allclose(c.v[l], want, rtol=1e-12, atol=1e-14)


def test_split_invariance_of_bidirectional_result():
    """Sec. 4 Part 2 / App. A step 7: whatever the meet point, chunk i of the result is the
    computed KV for i < m and the stored KV for i >= m; computed chunks do not depend on m."""
    w = _small_weights()
    toks = si.make_tokens(40, SMALL.vocab, seed=9)
    chunk, n = 8, 5
    stored = otf.prefill_monolithic(w, SMALL, toks, kv_dtype="bf16")
    marked = otf.KVCache(SMALL.n_layers, 40, SMALL.n_kv, SMALL.head_dim)
    marked.k[:] = stored.k + 1000.0          # make "stored" recognisable
    marked.v[:] = stored.v - 1000.0
    results = [otf.bidirectional_kv(w, SMALL, toks, chunk, m, marked, kv_dtype="bf16")
               for m in range(n + 1)]
    for m, r in enumerate(results):
        s = m * chunk
        np.testing.assert_array_equal(r.k[:, s:], marked.k[:, s:])
        np.testing.assert_array_equal(r.v[:, s:], marked.v[:, s:])
        np.testing.assert_array_equal(r.k[:, :s], results[n].k[:, :s])
        np.testing.assert_array_equal(r.v[:, :s], results[n].v[:, :s])
    # compute-only equals a plain chunked prefill; load-only equals the store
    np.testing.assert_allclose(results[n].k, stored.k, rtol=0, atol=1e-12)
    np.testing.assert_array_equal(results[0].v, marked.v)


# ----------------------------------------------------------------------------- storage rounding
def test_bf16_rounding():
    # 1 + 2^-8 is a tie between 1 and 1 + 2^-7 -> even mantissa (1.0); 1 + 3*2^-8 ties up to 1+2^-6
    x = np.array([1.0, 1.0 + 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -20, 1.0 + 3 * 2.0 ** -8, -2.5, 3.0e-5])
    y = otf.round_to_bf16(x)
    np.testing.assert_array_equal(y[:4], [1.0, 1.0, 1.0 + 2.0 ** -7, 1.0 + 2.0 ** -6])
    assert y[4] == -2.5
    assert abs(y[5] - 3.0e-5) <= 3.0e-5 * 2.0 ** -8
    # every result has at most 8 significant bits
    r = np.random.default_rng(0).standard_normal(1000)
    m, _ = np.frexp(otf.round_to_bf16(r))
    assert np.all(m * 256 == np.round(m * 256))
    assert np.all(np.abs(otf.round_to_bf16(r) - r) <= np.abs(r) * 2.0 ** -8)


def test_kv_dtype_rounds_once_and_attention_reads_cache():
    w = _small_weights()
    toks = si.make_tokens(24, SMALL.vocab, seed=10)
    exact = otf.prefill_monolithic(w, SMALL, toks)
    mono = otf.prefill_monolithic(w, SMALL, toks, kv_dtype="bf16")
    ch = otf.prefill_chunked(w, SMALL, toks, 8, kv_dtype="bf16")
    tbt = otf.prefill_token_by_token(w, SMALL, toks, kv_dtype="bf16")
    # layer 0 sees no attention: its cache is exactly the rounded exact K/V
    np.testing.assert_array_equal(mono.k[0], otf.round_to_bf16(exact.k[0]))
    np.testing.assert_array_equal(mono.k, otf.round_to_bf16(mono.k))     # stored values are bf16
    # the three routines agree up to rounding-boundary flips of single values
    for other in (ch, tbt):
        assert np.abs(other.k - mono.k).max() <= np.abs(mono.k).max() * 2.0 ** -7
        assert np.mean(other.k != mono.k) < 0.02
    assert np.abs(mono.k - exact.k).max() <= np.abs(exact.k).max() * 2.0 ** -6


# ----------------------------------------------------------------------------- store images
def test_store_layout_and_roundtrip():
    L, T, n_kv, hd, pt = 2, 11, 2, 4, 4
    cache = otf.KVCache(L, T, n_kv, hd)
    # value encodes its own coordinates: 1000*layer + 100*kv + 10*token(+0.5 for V) ... small ints are bf16-exact
    for l in range(L):
        for t in range(T):
            for g in range(n_kv):
                for e in range(hd):
                    cache.k[l, t, g, e] = l * 64 + g * 32 + t * 2 + (e == 3)
                    cache.v[l, t, g, e] = -(l * 64 + g * 32 + t * 2 + (e == 3))
    for dtype in ("f32", "bf16"):
        img = ostore.pack_store(cache, pt, dtype)
        assert img.shape == (3, L, 2, n_kv * pt * hd)
        vals = ostore.decode_words(img, dtype)
        # K of (page 1, layer 1, kv 1, token-in-page 2 -> token 6, e 3) at [kv][tok][hd]
        assert vals[1, 1, 0, (1 * pt + 2) * hd + 3] == 1 * 64 + 32 + 6 * 2 + 1
        # V of the same element sits transposed at [kv][hd][tok]
        assert vals[1, 1, 1, (1 * hd + 3) * pt + 2] == -(1 * 64 + 32 + 6 * 2 + 1)
        # ragged tail: page 2 holds tokens 8..10, slot 3 is zero
        assert vals[2, 0, 0, (0 * pt + 3) * hd + 0] == 0
        back = ostore.unpack_store(img, T, n_kv, hd, pt, dtype)
        np.testing.assert_array_equal(back.k, cache.k)
        np.testing.assert_array_equal(back.v, cache.v)
    assert ostore.page_image_words(L, n_kv, hd, pt) * 2 == pt * otf.kv_bytes_per_token(L, n_kv, hd, 2)


def test_chunk_flops_grows_linearly():
    """Sec. 4 Part 2 insight: work per chunk is affine in the chunk index; totals match a
    direct count of multiply-adds for a tiny case."""
    s = si.LLAMA3_8B
    f = [otf.chunk_flops(s, i, 1024) for i in range(5)]
    d = [f[i + 1] - f[i] for i in range(4)]
    assert len(set(d)) == 1 and d[0] == s.n_layers * 4 * s.n_q * s.head_dim * 1024 * 1024
    # direct count, tiny shape: per token 2*params; per (query,key) visible pair 4*hd per head
    t = si.ModelShape("t", 2, 8, 2, 1, 4, 12, 10, "f32")
    C, i = 3, 2
    params = t.n_layers * (8 * 8 + 2 * 8 * 4 + 8 * 8 + 3 * 8 * 12)
    pairs = sum(q + 1 for q in range(i * C, (i + 1) * C))
    assert otf.chunk_flops(t, i, C) == 2 * params * C + t.n_layers * t.n_q * 4 * t.head_dim * pairs


# --------------------------------------------------------------------------- first token
def test_first_token_equals_last_row_of_full_forward():
    """Decode-step identity: re-running the last token against the finished cache gives the
    hidden state the full forward had at that position, hence the same logits."""
    shape = si.TINY.with_(vocab=97, n_layers=3)
    w = si.make_weights(shape, seed=4, with_head=True)
    toks = si.make_tokens(50, shape.vocab, seed=5)
    cache, hidden = otf.prefill_chunked(w, shape, toks, 16, return_hidden=True)
    want = otf.lm_logits(w, shape, hidden[-1])
    got = otf.first_token_logits(w, shape, toks, cache)
    assert np.abs(got - want).max() < 1e-10 * np.abs(want).max()
    # and against the textbook definition written out: softmax-free check of the head itself
    h = hidden[-1] / np.sqrt(np.mean(hidden[-1] ** 2) + shape.rms_eps) * np.asarray(w["final_norm"], dtype=np.float64)
    np.testing.assert_allclose(want, h @ np.asarray(w["lm_head"], dtype=np.float64), rtol=1e-12)


def test_first_token_reads_the_cache_as_it_is():
    """The cache is authoritative, the last position included (it may hold loaded bytes)."""
    shape = si.TINY.with_(vocab=97)
    w = si.make_weights(shape, seed=6, with_head=True)
    toks = si.make_tokens(40, shape.vocab, seed=7)
    cache = otf.prefill_chunked(w, shape, toks, 16)
    base = otf.first_token_logits(w, shape, toks, cache)
    k0, v0 = cache.k.copy(), cache.v.copy()
    for t in (0, 39):                                   # an early entry and the token's own
        cache.v[1, t] += 0.5
        bumped = cache.v.copy()
        assert np.abs(otf.first_token_logits(w, shape, toks, cache) - base).max() > 1e-6
        np.testing.assert_array_equal(cache.v, bumped)  # read-only
        np.testing.assert_array_equal(cache.k, k0)
        cache.v[:] = v0
    # earlier prompt tokens enter only through the cache
    toks2 = toks.copy()
    toks2[:39] = (toks2[:39] + 1) % shape.vocab
    np.testing.assert_array_equal(otf.first_token_logits(w, shape, toks2, cache), base)


def test_greedy_token_lowest_index_on_ties():
    assert otf.greedy_token(np.array([1.0, 3.0, 3.0, 2.0])) == 1
    assert otf.greedy_token(np.array([-np.inf, -5.0])) == 1


# --------------------------------------------------------------------------- 8-bit stored KV
def test_int8_rows_hand_worked():
    from oracle import store as ostore
    x = np.array([[127.0, -63.5, 1.0, 0.49, -0.51, 0.0, 2.5, -127.0],      # scale 1: ties to even, clipping at the ends
                  [0.0] * 8,                                              # zero row: scale 0, codes 0
                  [0.5, -0.25, 0.125, 0.0, 0.0, 0.0, 0.0, 0.0]])          # scale 0.5/127
    q, sc = ostore.quantize_rows_int8(x)
    assert sc[0] == 1.0 and q[0].tolist() == [127, -64, 1, 0, -1, 0, 2, -127]     # -63.5 -> -64 (even), 2.5 -> 2 (even)
    assert sc[1] == 0.0 and not q[1].any()
    assert sc[2] == np.float32(0.5) / np.float32(127) and q[2].tolist()[:3] == [127, -64, 32]   # 63.5 -> 64, 31.75 -> 32
    d = ostore.dequantize_rows_int8(q, sc, "f32")
    assert d[0].tolist() == [127.0, -64.0, 1.0, 0.0, -1.0, 0.0, 2.0, -127.0] and not d[1].any()
    assert abs(d[2][0] - 0.5) < 1e-7


def test_int8_store_properties():
    from oracle import store as ostore
    rng = np.random.default_rng(3)
    L, T, n_kv, hd, pt = 2, 150, 2, 64, 64
    cache = otf.KVCache(L, T, n_kv, hd)
    cache.k[:] = otf.round_storage(rng.standard_normal(cache.k.shape) * 3, "bf16")
    cache.v[:] = otf.round_storage(rng.standard_normal(cache.v.shape), "bf16")
    img = ostore.pack_store_int8(cache, pt)
    assert img.shape == (3, L, 2, n_kv * pt * (hd + 4)) and img[0].size == ostore.int8_image_bytes(L, n_kv, hd, pt)
    assert ostore.int8_image_bytes(32, 8, 128, 256) * 2 * 128 == 32 * 2 * 8 * 256 * 128 * 2 * 132    # (hd+4)/(2 hd) of the bf16 image
    back = ostore.unpack_store_int8(img, T, n_kv, hd, pt, "bf16")
    for a, b in ((cache.k, back.k), (cache.v, back.v)):
        amax = np.abs(a).max(axis=-1, keepdims=True)
        # half a quantisation step plus the bf16 rounding of the result
        assert np.all(np.abs(a - b) <= amax / 254 * (1 + 1e-6) + np.abs(b) * 2.0 ** -8)
        hit = np.abs(a) == amax                                           # the row's largest element is code +-127: exact up to rounding
        assert np.all(np.abs(a[hit] - b[hit]) <= np.abs(a[hit]) * 2.0 ** -7)
    codes = img[..., :n_kv * pt * hd].view(np.int8)
    assert codes.min() >= -127 and codes.max() <= 127 and np.abs(codes).max() == 127
    # slots past the prompt are zeros with scale 0
    tail = img[2, :, :, :n_kv * pt * hd].view(np.int8).reshape(L, 2, n_kv, pt, hd)[:, :, :, T - 2 * pt:, :]
    assert not tail.any()
    # quantising what was dequantised (before storage rounding) reproduces the codes
    q, sc = ostore.quantize_rows_int8(cache.k[0])
    q2, _ = ostore.quantize_rows_int8(q.astype(np.float32) * sc[..., None])
    np.testing.assert_array_equal(q, q2)


def test_int4_rows_hand_worked():
    from oracle import store as ostore
    x = np.array([[7.0, -3.5, 1.0, 0.49, -0.51, 0.0, 2.5, -7.0],           # scale 1: ties to even, clipping at the ends
                  [0.0] * 8,                                               # zero row: scale 0, codes 0
                  [0.5, -0.25, 0.125, 0.0, 14.0, -14.0, 1.0, 3.0]])        # scale 2: 0.25 -> 0, -0.125 -> -0, 0.5 -> 0 (even), 1.5 -> 2
    q, sc = ostore.quantize_rows_int4(x)
    assert sc[0] == 1.0 and q[0].tolist() == [7, -4, 1, 0, -1, 0, 2, -7]          # -3.5 -> -4 (even), 2.5 -> 2 (even)
    assert sc[1] == 0.0 and not q[1].any()
    assert sc[2] == 2.0 and q[2].tolist() == [0, 0, 0, 0, 7, -7, 0, 2]
    # two codes per byte: even element low nibble, odd element high nibble, two's complement
    packed = ostore.pack_nibbles(q)
    assert packed[0].tolist() == [0x07 | (0xC << 4), 0x01 | (0x0 << 4), 0xF | (0x0 << 4), 0x2 | (0x9 << 4)]
    np.testing.assert_array_equal(ostore.unpack_nibbles(packed), q)
    every = np.arange(-8, 8, dtype=np.int8).reshape(1, 16)
    np.testing.assert_array_equal(ostore.unpack_nibbles(ostore.pack_nibbles(every)), every)
    d = ostore.dequantize_rows_int8(q, sc, "f32")
    assert d[0].tolist() == [7.0, -4.0, 1.0, 0.0, -1.0, 0.0, 2.0, -7.0] and d[2].tolist()[4:] == [14.0, -14.0, 0.0, 4.0]


def test_int4_store_properties():
    from oracle import store as ostore
    rng = np.random.default_rng(4)
    L, T, n_kv, hd, pt = 2, 150, 2, 64, 64
    cache = otf.KVCache(L, T, n_kv, hd)
    cache.k[:] = otf.round_storage(rng.standard_normal(cache.k.shape) * 3, "bf16")
    cache.v[:] = otf.round_storage(rng.standard_normal(cache.v.shape), "bf16")
    img = ostore.pack_store_int4(cache, pt)
    assert img.shape == (3, L, 2, n_kv * pt * (hd // 2 + 4)) and img[0].size == ostore.int4_image_bytes(L, n_kv, hd, pt)
    # 68 / 256 of the bf16 image and 68 / 132 of the 8-bit image at head_dim 128
    assert ostore.int4_image_bytes(32, 8, 128, 256) * 132 == ostore.int8_image_bytes(32, 8, 128, 256) * 68
    back = ostore.unpack_store_int4(img, T, n_kv, hd, pt, "bf16")
    for a, b in ((cache.k, back.k), (cache.v, back.v)):
        amax = np.abs(a).max(axis=-1, keepdims=True)
        # half a quantisation step (1/14 of the row's maximum) plus the bf16 rounding of the result
        assert np.all(np.abs(a - b) <= amax / 14 * (1 + 1e-6) + np.abs(b) * 2.0 ** -8)
        hit = np.abs(a) == amax
        assert np.all(np.abs(a[hit] - b[hit]) <= np.abs(a[hit]) * 2.0 ** -7)
        # coarser than the 8-bit store on the same data, and not trivially exact
        b8 = ostore.unpack_store_int8(ostore.pack_store_int8(cache, pt), T, n_kv, hd, pt, "bf16")
        assert np.abs(a - b).max() > 4 * np.abs(a - (b8.k if a is cache.k else b8.v)).max()
    codes = ostore.unpack_nibbles(img[..., :n_kv * pt * (hd // 2)])
    assert codes.min() == -7 and codes.max() == 7
    tail = codes[2].reshape(L, 2, n_kv, pt, hd)[:, :, :, T - 2 * pt:, :]
    assert not tail.any()
    # quantising what was dequantised (before storage rounding) reproduces the codes
    q, sc = ostore.quantize_rows_int4(cache.k[0])
    q2, _ = ostore.quantize_rows_int4(q.astype(np.float32) * sc[..., None])
    np.testing.assert_array_equal(q, q2)
