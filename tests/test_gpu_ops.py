"""GPU parity of the single kernels against the oracle's pieces, through the C ABI."""
import numpy as np
import pytest

import synth_inputs as si
from oracle import transformer as otf
from oracle import store as ostore

pytestmark = pytest.mark.gpu


def _engine(shape, T, C, pt, **kw):
    import paper_2410_03065_amd as cake
    w = si.make_weights(shape.with_(vocab=64, n_layers=1), seed=0)
    return cake.Engine(shape.with_(vocab=64, n_layers=1), w, max_tokens=T, max_chunk=min(C, T), page_tokens=pt, **kw)


def _bf16_vals(rng, shape, scale=1.0):
    a = (rng.standard_normal(shape) * scale).astype(np.float32)
    a.view(np.uint32)[...] &= np.uint32(0xFFFF0000)
    return a


def _rel(got, want):
    return float(np.abs(got - want).max() / np.abs(want).max())


SHAPE_BF = si.ModelShape("op-bf16", 1, 256, 8, 2, 128, 512, 64, "bf16", rope_theta=500000.0)
SHAPE_F32 = si.ModelShape("op-f32", 1, 256, 4, 4, 64, 688, 64, "f32")


@pytest.mark.parametrize("kind", ["f32", "bf16"])
@pytest.mark.parametrize("rows,d", [(37, 1000), (37, 4096), (5, 8192), (3, 1024), (2, 9216)])
def test_rmsnorm(kind, rows, d):
    import torch
    shape = SHAPE_F32 if kind == "f32" else SHAPE_BF
    eng = _engine(shape, 256, 256, 64)
    rng = np.random.default_rng(0)
    x = rng.standard_normal((rows, d)).astype(np.float32) * 3
    g = (1 + 0.3 * rng.standard_normal(d)).astype(np.float32)
    got = eng.op_rmsnorm(torch.from_numpy(x).cuda(), torch.from_numpy(g).cuda()).float().cpu().numpy()
    want = otf.rmsnorm(x.astype(np.float64), g.astype(np.float64), shape.rms_eps)
    assert _rel(got, want) < (1e-6 if kind == "f32" else 2.0 ** -8)


@pytest.mark.parametrize("kind,path,M,N,K,cfg", [
    ("f32", 0, 130, 100, 72, 0), ("f32", 0, 256, 688, 256, 0),
    ("bf16", 1, 130, 100, 72, 0),                      # generic kernel on bf16
    ("bf16", 0, 300, 256, 512, 0), ("bf16", 0, 1024, 384, 4096, 0), ("bf16", 0, 1, 128, 64, 0),
    ("bf16", 0, 700, 512, 96, 1), ("bf16", 0, 700, 512, 96, 2), ("bf16", 0, 700, 512, 96, 3),   # each tile shape,
    ("bf16", 0, 257, 256, 32, 1), ("bf16", 0, 257, 256, 64, 2), ("bf16", 0, 129, 256, 160, 3),  # short K, ragged M
    ("bf16", 0, 1024, 2048, 1024, 1),
    ("bf16", 0, 700, 384, 96, 4), ("bf16", 0, 129, 768, 160, 4), ("bf16", 0, 1024, 6144, 512, 0),   # 128x192 tiles
    ("bf16", 0, 300, 192, 96, 5), ("bf16", 0, 512, 4096, 1024, 0), ("bf16", 0, 129, 64, 192, 5),   # 128x64 tiles
    ("bf16", 0, 300, 256, 512, 6), ("bf16", 0, 129, 384, 64, 6), ("bf16", 0, 1024, 4096, 1024, 6),  # 128x128, two waves per half along K
    # the persistent four-wave kernel: one slice; ragged M over three slices; many slices; more tiles than
    # workgroups (260 plain tiles = 2 rounds of 130 workgroups, 520 SwiGLU tiles = 3 rounds, the last one short)
    ("bf16", 0, 257, 256, 64, 7), ("bf16", 0, 300, 768, 192, 7), ("bf16", 0, 1024, 512, 4096, 7), ("bf16", 0, 1000, 16640, 128, 7),
    # its column panels of mixed width: 256- and 192-wide in one round (plain) and in consecutive rounds of the same
    # workgroups (SwiGLU: 64 + 64 panels x 4 row bands = 512 items); 192- and 128-wide likewise
    ("bf16", 0, 1024, 14336, 128, 7), ("bf16", 0, 1024, 10240, 192, 7),
])
def test_gemm_variants(kind, path, M, N, K, cfg):
    import torch
    shape = SHAPE_F32 if kind == "f32" else SHAPE_BF
    eng = _engine(shape, 256, 256, 64)
    eng.set_tuning(kernel_path=path, gemm_config=cfg)
    rng = np.random.default_rng(M + N + K)
    mk = (lambda s, sc=1.0: _bf16_vals(rng, s, sc)) if kind == "bf16" else (lambda s, sc=1.0: (rng.standard_normal(s) * sc).astype(np.float32))
    a, w, w2 = mk((M, K)), mk((N, K), 0.05), mk((N, K), 0.05)
    x0 = rng.standard_normal((M, N)).astype(np.float32)
    td = torch.float32 if kind == "f32" else torch.bfloat16
    A, W, W2 = (torch.from_numpy(t).cuda().to(td) for t in (a, w, w2))
    a64, w64, w264 = a.astype(np.float64), w.astype(np.float64), w2.astype(np.float64)
    want = a64 @ w64.T
    got = eng.op_gemm(A, W).cpu().numpy()
    assert _rel(got, want) < 2e-6 * max(1, K / 256)
    X = torch.from_numpy(x0.copy()).cuda()
    got = eng.op_gemm_residual(A, W, X).cpu().numpy()
    assert _rel(got, x0 + want) < 2e-6 * max(1, K / 256)
    want = otf.silu(want) * (a64 @ w264.T)
    got = eng.op_gemm_swiglu(A, W, W2).float().cpu().numpy()
    tol = 1e-5 if kind == "f32" else 2.0 ** -8 * 1.01
    assert np.all(np.abs(got - want) <= tol * np.abs(want) + 1e-6 * np.abs(want).max())


@pytest.mark.parametrize("M,N,K,cfg,ks,tile", [
    (1024, 1024, 4096, 1, 2, (256, 256)), (1024, 1024, 4096, 1, 4, (256, 256)), (1024, 1024, 4096, 1, 8, (256, 256)),
    (700, 512, 2048, 2, 4, (256, 128)),      # ragged M
    (300, 768, 1024, 3, 2, (128, 128)),
    (129, 768, 2048, 4, 2, (128, 192)),
    (200, 512, 1024, 5, 2, (128, 64)),
    (300, 768, 2048, 6, 4, (128, 128)),      # split over workgroups and, inside each, over two waves
    (1024, 1024, 4096, 7, 4, (256, 256)), (700, 512, 2048, 7, 2, (256, 256)), (1024, 2048, 4096, 7, 8, (256, 256)),  # persistent kernel
    (512, 4096, 11008, 0, 0, None),          # down projection with 512-token chunks: the cost model splits it
])
def test_gemm_split_k(M, N, K, cfg, ks, tile):
    """K of one tile spread over several workgroups: same result as the fp64 product, the same bits on
    every launch (the parts are summed in K order whoever finishes last), counters back at zero."""
    import torch
    eng = _engine(SHAPE_BF.with_(d_model=4096), 1024, 1024, 64)
    eng.set_tuning(gemm_config=cfg, gemm_ksplit=ks)
    plan = eng.op_gemm_plan(M, N, K, residual=True)
    if tile is not None:
        assert plan == (tile[0], tile[1], ks), plan          # the forced split is really what runs
    else:
        assert plan[2] > 1, plan                              # too few large tiles: the model splits
        assert eng.op_gemm_plan(1024, 8192, 28672) == (256, 256, 2)      # the widest model's down projection
        assert eng.op_gemm_plan(1024, 4096, 14336) == (128, 128, 1)      # 256 tiles of 128 x 128 fill the chip: unsplit
        assert eng.op_gemm_plan(1024, 6144, 4096, residual=False) == (128, 192, 1)
    rng = np.random.default_rng(M + N + K + ks)
    x0 = rng.standard_normal((M, N)).astype(np.float32)
    tol = 2e-6 * max(1, K / 256)
    # two different products take turns, so a part left over from the launch before would show
    ops = []
    for _ in range(2):
        a, w = _bf16_vals(rng, (M, K)), _bf16_vals(rng, (N, K), 0.05)
        A, W = (torch.from_numpy(t).cuda().to(torch.bfloat16) for t in (a, w))
        ops.append((A, W, a.astype(np.float64) @ w.astype(np.float64).T))
    first = [None, None]
    for turn in range(6):
        A, W, want = ops[turn % 2]
        if turn < 2:
            assert _rel(eng.op_gemm(A, W).cpu().numpy(), want) < tol
        X = torch.from_numpy(x0.copy()).cuda()
        got = eng.op_gemm_residual(A, W, X).cpu().numpy()
        if first[turn % 2] is None:
            assert _rel(got, x0 + want) < tol
            first[turn % 2] = got
        else:
            np.testing.assert_array_equal(got, first[turn % 2])
    # unsplit, the same kernel agrees to rounding
    eng.set_tuning(gemm_config=cfg, gemm_ksplit=1)
    assert eng.op_gemm_plan(M, N, K)[2] == 1
    A, W, want = ops[0]
    X = torch.from_numpy(x0.copy()).cuda()
    assert _rel(eng.op_gemm_residual(A, W, X).cpu().numpy(), first[0]) < tol


@pytest.mark.parametrize("kind", ["f32", "bf16"])
@pytest.mark.parametrize("tok_begin,rows", [(0, 200), (192, 100), (100, 157), (65400, 136)])
def test_rope_and_page_write(kind, tok_begin, rows):
    import torch
    shape = SHAPE_F32 if kind == "f32" else SHAPE_BF
    pt, T = 128, tok_begin + rows
    n_log = (T + pt - 1) // pt
    bt = np.random.default_rng(1).permutation(n_log).astype(np.int32)      # scattered physical pages
    eng = _engine(shape, n_log * pt, 256, pt, block_table=bt)
    rng = np.random.default_rng(2)
    nq, nkv, hd = shape.n_q, shape.n_kv, shape.head_dim
    qkv = rng.standard_normal((rows, (nq + 2 * nkv) * hd)).astype(np.float32)
    q = eng.op_rope_kv_write(torch.from_numpy(qkv).cuda(), 0, tok_begin).float().cpu().numpy()   # [nq][rows][hd]
    pos = np.arange(tok_begin, tok_begin + rows)
    q64 = qkv[:, :nq * hd].astype(np.float64).reshape(rows, nq, hd)
    k64 = qkv[:, nq * hd:(nq + nkv) * hd].astype(np.float64).reshape(rows, nkv, hd)
    v64 = qkv[:, (nq + nkv) * hd:].astype(np.float64).reshape(rows, nkv, hd)
    want_q = otf.rope(q64, pos, shape.rope_theta).transpose(1, 0, 2)
    tol = 2e-6 if kind == "f32" else 2.0 ** -8 * 1.01
    assert np.all(np.abs(q - want_q) <= tol * np.abs(want_q) + 1e-6)
    cache = otf.KVCache(1, T, nkv, hd)
    cache.k[0, tok_begin:] = otf.rope(k64, pos, shape.rope_theta)
    cache.v[0, tok_begin:] = v64
    want = ostore.decode_words(ostore.pack_store(_rounded(cache, kind), pt, kind), kind)
    got = eng.pool_images(T)
    assert np.all(np.abs(got - want) <= tol * np.abs(want) + 1e-6)
    # V is a pure copy: exact after storage rounding; untouched slots stay zero
    np.testing.assert_array_equal(got[:, :, 1], want[:, :, 1])
    assert np.all(got[want == 0] == 0)


def _rounded(cache, kind):
    out = otf.KVCache(*cache.k.shape[:1], cache.k.shape[1], cache.k.shape[2], cache.k.shape[3])
    out.k[:] = otf.round_storage(cache.k, kind)
    out.v[:] = otf.round_storage(cache.v, kind)
    return out


@pytest.mark.parametrize("kind,path,variant", [("f32", 0, 0), ("bf16", 1, 0), ("bf16", 0, 0), ("bf16", 0, 1), ("bf16", 0, 2),
                                               ("bf16", 0, 3)])
@pytest.mark.parametrize("tok_begin,rows", [(0, 130), (256, 256), (448, 77), (1, 1), (0, 64), (64, 1), (960, 200)])
def test_attention(kind, path, variant, tok_begin, rows):
    import torch
    shape = SHAPE_F32 if kind == "f32" else SHAPE_BF
    pt, T = 128, tok_begin + rows
    n_log = (T + pt - 1) // pt
    bt = np.random.default_rng(3).permutation(n_log).astype(np.int32)
    eng = _engine(shape, n_log * pt, 256, pt, block_table=bt)
    eng.set_tuning(kernel_path=path, attn_variant=variant)
    rng = np.random.default_rng(4 + rows)
    nq, nkv, hd = shape.n_q, shape.n_kv, shape.head_dim
    cache = otf.KVCache(1, T, nkv, hd)
    cache.k[0] = rng.standard_normal((T, nkv, hd)) * 1.5          # peaked softmax rows
    cache.v[0] = rng.standard_normal((T, nkv, hd))
    cache = _rounded(cache, kind)
    images = ostore.pack_store(cache, pt, kind)
    eng.set_store(images)
    eng.load_chunk(0, T)
    q = otf.round_storage(rng.standard_normal((rows, nq, hd)), kind)
    td = torch.float32 if kind == "f32" else torch.bfloat16
    Q = torch.from_numpy(q.transpose(1, 0, 2).astype(np.float32).copy()).cuda().to(td)
    got = eng.op_attention(Q, 0, tok_begin).float().cpu().numpy().reshape(rows, nq, hd)
    want = otf.attention(q, cache.k[0], cache.v[0], np.arange(tok_begin, T), np.arange(T))
    # bf16: the output (2^-9), each probability where it enters P.V (2^-9) and, in the eight-wave kernels, Q once more
    # after the softmax scale has been folded into it (2^-9, acting in the exponent: it dominates on these peaked
    # rows).  The same three roundings repeated in float64 give up to 6.2e-3 of the largest value on inputs of this
    # distribution (tests/test_gpu_attention_long.py has the derivation); the bound is 2^-7, and no row may be off
    # as a whole (a tile dropped or read from the wrong page shifts a row; rounding does not).
    tol = 2e-5 if kind == "f32" else 2.0 ** -7
    err = _rel(got, want)
    row_rms = np.sqrt(((got - want) ** 2).mean(axis=2)).max() / np.abs(want).max()
    print("attention error: largest %.2e, worst row rms %.2e (of the largest value)" % (err, row_rms))
    assert err < tol, err
    assert row_rms < tol / 2, row_rms


def test_attention_and_page_write_above_2_and_4_gib():
    """Physical pages whose byte offset in the pool has bit 31 / bit 32 set (a 4 GiB pool is what
    the 32K-token benchmark uses): offsets must be formed in unsigned 64-bit arithmetic."""
    import torch
    import paper_2410_03065_amd as cake
    shape = si.ModelShape("op-bf16-big", 1, 256, 32, 8, 128, 512, 64, "bf16", rope_theta=500000.0)
    pt, T = 256, 1024
    n_phys = 4200                                         # 1 MiB per page and layer -> 4.1 GiB pool
    bt = np.array([2047, 2048, 4199, 3], dtype=np.int32)  # just below / above 2 GiB, above 4 GiB, low
    w = si.make_weights(shape, seed=0)
    eng = cake.Engine(shape, w, max_tokens=T, max_chunk=T, page_tokens=pt, block_table=bt, n_physical_pages=n_phys)
    rng = np.random.default_rng(11)
    nq, nkv, hd = shape.n_q, shape.n_kv, shape.head_dim
    qkv = rng.standard_normal((T, (nq + 2 * nkv) * hd)).astype(np.float32)
    q_dev = eng.op_rope_kv_write(torch.from_numpy(qkv).cuda(), 0, 0)
    pos = np.arange(T)
    cache = otf.KVCache(1, T, nkv, hd)
    cache.k[0] = otf.rope(qkv[:, nq * hd:(nq + nkv) * hd].astype(np.float64).reshape(T, nkv, hd), pos, shape.rope_theta)
    cache.v[0] = qkv[:, (nq + nkv) * hd:].astype(np.float64).reshape(T, nkv, hd)
    cache = _rounded(cache, "bf16")
    want_img = ostore.decode_words(ostore.pack_store(cache, pt, "bf16"), "bf16")
    got_img = eng.pool_images(T)
    assert np.abs(got_img - want_img).max() <= 2.0 ** -7 * np.abs(want_img).max()
    got = eng.op_attention(q_dev, 0, 0).float().cpu().numpy().reshape(T, nq, hd)
    q64 = q_dev.float().cpu().numpy().astype(np.float64).transpose(1, 0, 2)
    # attention over what the pages actually hold (already checked against the oracle above)
    held = ostore.unpack_store(eng.pool_raw(T).view(np.uint16), T, nkv, hd, pt, "bf16")
    want = otf.attention(q64, held.k[0], held.v[0], pos, pos)
    assert _rel(got, want) < 2.0 ** -7


@pytest.mark.parametrize("kind,path,shape_kw,T,pt", [
    ("bf16", 0, dict(n_q=8, n_kv=2), 40000, 256),     # GQA 4:1, 625 key tiles: several tiles per wave, ragged tail
    ("bf16", 0, dict(n_q=8, n_kv=1), 9001, 64),       # GQA 8:1, small pages
    ("bf16", 0, dict(n_q=4, n_kv=4), 70, 128),        # MHA, two tiles
    ("bf16", 1, dict(n_q=8, n_kv=2), 5000, 256),      # vector-ALU kernel on the same layout
    ("f32", 0, dict(n_q=4, n_kv=4), 3000, 128),       # float32 pages, head_dim 64
    ("f32", 0, dict(n_q=4, n_kv=2), 130, 64),
])
def test_decode_attention(kind, path, shape_kw, T, pt):
    """One query per head against T cached keys (first-token step), both kernels."""
    import torch
    import paper_2410_03065_amd as cake
    base = SHAPE_F32 if kind == "f32" else SHAPE_BF
    shape = base.with_(vocab=64, n_layers=1, **shape_kw)
    w = si.make_weights(shape, seed=0, with_head=True)
    n_log = (T + pt - 1) // pt
    bt = np.random.default_rng(5).permutation(n_log).astype(np.int32)
    eng = cake.Engine(shape, w, max_tokens=n_log * pt, max_chunk=min(256, n_log * pt), page_tokens=pt, block_table=bt)
    eng.set_tuning(kernel_path=path)
    rng = np.random.default_rng(T)
    nq, nkv, hd = shape.n_q, shape.n_kv, shape.head_dim
    cache = otf.KVCache(1, T, nkv, hd)
    cache.k[0] = rng.standard_normal((T, nkv, hd)) * 1.5
    cache.v[0] = rng.standard_normal((T, nkv, hd))
    cache = _rounded(cache, kind)
    eng.set_store(ostore.pack_store(cache, pt, kind))
    eng.load_chunk(0, T)
    q = rng.standard_normal((nq, hd)).astype(np.float32) * 2
    got = eng.op_decode_attention(torch.from_numpy(q).cuda(), 0, T).cpu().numpy()
    want = otf.attention(q.astype(np.float64)[None], cache.k[0], cache.v[0], np.array([T - 1]), np.arange(T))[0]
    # MFMA path: q and the probabilities are rounded to bf16 (2^-9 each); others are float32 throughout
    tol = 1.2e-2 if (kind == "bf16" and path == 0) else 2e-5
    assert _rel(got, want) < tol, _rel(got, want)


def test_mfma_rate_yardstick():
    """The MFMA-only kernel reports a rate between a quarter of the nominal bf16 peak and the peak itself,
    and refuses sizes beyond its workspace."""
    import paper_2410_03065_amd as cake
    eng = _engine(SHAPE_BF, 256, 256, 128)
    r = eng.mfma_rate(512, 2048)
    assert 600.0 < r < 2600.0, r
    with pytest.raises(cake.CakeError):
        eng.mfma_rate(60000, 16)
    with pytest.raises(cake.CakeError):
        eng.mfma_rate(0, 16)
