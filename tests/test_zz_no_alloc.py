"""The entry point that allocates nothing (cake_op_decode_attention_static) against the entry point it
is a variant of (cake_op_decode_attention), through the C ABI: same kernels, so the same bits, on
two calls in a row that share the library's static buffer, the second with a smaller input."""
import numpy as np
import pytest

import synth_inputs as si
from oracle import store as ostore
from oracle import transformer as otf

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("kind,n_q,n_kv,hd,pt", [("bf16", 8, 2, 128, 256), ("f32", 4, 2, 64, 64)])
def test_static_scratch_entry_point_matches_the_allocating_one(kind, n_q, n_kv, hd, pt):
    import torch
    import paper_2410_03065_amd as cake
    shape = si.ModelShape("no-alloc", 1, 256, n_q, n_kv, hd, 512, 64, kind, rope_theta=500000.0)
    w = si.make_weights(shape, seed=0, with_head=True)
    T_big, T_small = 20000, 1337
    n_log = (T_big + pt - 1) // pt
    bt = np.random.default_rng(5).permutation(n_log).astype(np.int32)
    eng = cake.Engine(shape, w, max_tokens=n_log * pt, max_chunk=256, page_tokens=pt, block_table=bt)
    rng = np.random.default_rng(T_big)
    cache = otf.KVCache(1, T_big, n_kv, hd)
    cache.k[0] = otf.round_storage(rng.standard_normal((T_big, n_kv, hd)) * 1.5, kind)
    cache.v[0] = otf.round_storage(rng.standard_normal((T_big, n_kv, hd)), kind)
    eng.set_store(ostore.pack_store(cache, pt, kind))
    eng.load_chunk(0, T_big)
    qs = [torch.from_numpy((rng.standard_normal((n_q, hd)) * 2).astype(np.float32)).cuda() for _ in range(2)]
    want = [eng.op_decode_attention(q, 0, T).cpu().numpy() for q, T in zip(qs, (T_big, T_small))]
    outs = [torch.empty_like(q) for q in qs]                      # made before the calls under test
    # two calls in a row on the shared static buffer, the second over fewer key ranges
    got = [eng.op_decode_attention(q, 0, T, out=o, static=True).cpu().numpy()
           for q, o, T in zip(qs, outs, (T_big, T_small))]
    for g, w_, q, T in zip(got, want, qs, (T_big, T_small)):
        np.testing.assert_array_equal(g, w_)                      # same kernels, same launch shape: same bits
        ref = otf.attention(q.cpu().numpy().astype(np.float64)[None], cache.k[0][:T], cache.v[0][:T],
                            np.array([T - 1]), np.arange(T))[0]
        assert np.abs(g - ref).max() / np.abs(ref).max() < (1.2e-2 if kind == "bf16" else 2e-5)
    # the big case again after the small one: entries the small call left untouched are not relied on
    again = eng.op_decode_attention(qs[0], 0, T_big, out=outs[0], static=True).cpu().numpy()
    np.testing.assert_array_equal(again, want[0])
    eng.close()


def test_static_scratch_entry_point_works_without_head_weights_and_rejects_oversize():
    import torch
    import paper_2410_03065_amd as cake
    shape = si.ModelShape("no-alloc-nohead", 1, 256, 8, 2, 128, 512, 64, "bf16")
    eng = cake.Engine(shape, si.make_weights(shape, seed=0), max_tokens=512, max_chunk=256, page_tokens=64)
    q = torch.zeros((8, 128), dtype=torch.float32, device="cuda")
    with pytest.raises(cake.CakeError):                    # the allocating variant needs the head workspace
        eng.op_decode_attention(q, 0, 100)
    out = eng.op_decode_attention(q, 0, 100, static=True)  # zero queries over a zero cache: finite zeros
    assert torch.isfinite(out).all() and float(out.abs().max()) == 0.0
    eng.close()
    big = si.ModelShape("no-alloc-big", 1, 256, 128, 8, 128, 512, 64, "bf16")      # 128 query heads: beyond the buffer
    eng = cake.Engine(big, si.make_weights(big, seed=0), max_tokens=512, max_chunk=256, page_tokens=64)
    q = torch.zeros((128, 128), dtype=torch.float32, device="cuda")
    with pytest.raises(cake.CakeError) as ei:
        eng.op_decode_attention(q, 0, 100, static=True)
    assert ei.value.code == cake.E_INVAL
    eng.close()
