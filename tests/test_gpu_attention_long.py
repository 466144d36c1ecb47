"""Prefill attention against the oracle at the prefix lengths the benchmark configurations end on
(Sec. 3 "Chunk Prefill": the last chunk of a 32K / 64K / 72K prompt attends to every earlier key),
through the C ABI, for each MFMA attention kernel.

A workgroup there walks 512 to 1152 key tiles and 128 to 288 page-table entries, the two key halves
of the eight-wave kernels are merged after hundreds of tiles each, and with the wider score
distribution the lazy move of the softmax reference fires far from the first tile.

Tolerance.  Q, K and V are bf16 values, so the only roundings are the kernel's own, each at most 2^-9
of the rounded quantity: the output once; every probability where it enters the second product; and,
in the eight-wave kernels, Q once more after the softmax scale has been folded into it.  The last one
acts in the exponent: it turns the query by up to 2^-9 per element, which moves a score s by about
2^-9 |s| / sqrt(3) and the weight of that key by the same relative amount, a few 1e-3 for the keys with
scores of 5 to 7 that carry a peaked row.  Rows whose weight sits on few keys are also the rows with
the largest outputs, so this does not average out against the tensor's largest value: repeating
exactly these three roundings in float64 on the inputs below gives 4.5e-3 to 6.2e-3 of the largest
value (2.8e-3 without the second rounding of Q).  The bound is 2^-7 = 7.8e-3; per row, the
root-mean-square error must stay under half of that.  One 64-key tile dropped or read from the wrong
page changes a row of the flat-score cases (a mean over ~10^4 effective keys) by a few percent of the
row's own spread in every element, which the per-row bound catches.
"""
import functools

import numpy as np
import pytest

import synth_inputs as si
from oracle import store as ostore
from oracle import transformer as otf

pytestmark = pytest.mark.gpu

PT = 256
ROWS = 1024
TOL = 2.0 ** -7
HEADS = (0, 3, 4, 7)          # first and last query head of each KV group at GQA 4; a spread at GQA 8


def _shape(n_kv):
    return si.ModelShape("attn-long", 1, 256, 8, n_kv, 128, 512, 64, "bf16", rope_theta=500000.0)


@functools.lru_cache(maxsize=2)
def _case(tok_begin, n_kv, q_scale):
    """Inputs and the oracle's output for the checked heads (cached: the kernels share them)."""
    T = tok_begin + ROWS
    rng = np.random.default_rng([tok_begin, n_kv])
    cache = otf.KVCache(1, T, n_kv, 128)
    cache.k[0] = otf.round_to_bf16(rng.standard_normal((T, n_kv, 128)) * 1.5)
    cache.v[0] = otf.round_to_bf16(rng.standard_normal((T, n_kv, 128)))
    q = otf.round_to_bf16(rng.standard_normal((ROWS, 8, 128)) * q_scale)
    group = 8 // n_kv
    want = {}
    for j in HEADS:
        g = j // group
        want[j] = otf.attention(q[:, j:j + 1], cache.k[0][:, g:g + 1], cache.v[0][:, g:g + 1],
                                np.arange(tok_begin, T), np.arange(T))[:, 0]
    images = ostore.pack_store(cache, PT, "bf16")
    return q, images, want


@pytest.mark.parametrize("variant", [2, 3, 1], ids=["eight-wave-128q", "eight-wave-64q", "four-wave"])
@pytest.mark.parametrize("tok_begin,n_kv,q_scale", [
    (31744, 2, 1.0),      # last chunk of the 32K prompt, GQA 4, flat scores: every tile carries weight
    (64512, 2, 1.0),      # last chunk of the 64K prompt
    (72704, 1, 2.0),      # last chunk of the 72K prompt, GQA 8, wide scores: the reference moves late
    (72704, 2, 1.0),
])
def test_prefill_attention_last_chunk_of_long_prompts(tok_begin, n_kv, q_scale, variant):
    import torch
    import paper_2410_03065_amd as cake
    shape = _shape(n_kv)
    T = tok_begin + ROWS
    n_log = T // PT
    q, images, want = _case(tok_begin, n_kv, q_scale)
    bt = np.random.default_rng(7).permutation(n_log).astype(np.int32)       # scattered physical pages
    w = si.make_weights(shape, seed=0)
    eng = cake.Engine(shape, w, max_tokens=T, max_chunk=ROWS, page_tokens=PT, block_table=bt)
    eng.set_tuning(attn_variant=variant)
    eng.set_store(images)
    eng.load_chunk(0, T)
    Q = torch.from_numpy(q.transpose(1, 0, 2).astype(np.float32).copy()).cuda().to(torch.bfloat16)
    got = eng.op_attention(Q, 0, tok_begin).float().cpu().numpy().astype(np.float64).reshape(ROWS, 8, 128)
    eng.close()
    seen = []
    for j in HEADS:
        scale = np.abs(want[j]).max()
        err = np.abs(got[:, j] - want[j]).max() / scale
        # no row may be off as a whole (a lost tile shifts a row, rounding does not): rms per row,
        # against the largest value and against the row's own spread
        row_rms = np.sqrt(((got[:, j] - want[j]) ** 2).mean(axis=1))
        row_rel = (row_rms / np.sqrt((want[j] ** 2).mean(axis=1))).max()
        seen.append((j, round(float(err), 5), round(float(row_rms.max() / scale), 5), round(float(row_rel), 5)))
        assert err < TOL, seen
        assert row_rms.max() / scale < TOL / 2, seen
        assert row_rel < 2 * TOL * q_scale, seen          # the second rounding of Q grows with the scores
    print("attention errors (head, max/max, worst row rms/max, worst row rms/row rms):", seen)
