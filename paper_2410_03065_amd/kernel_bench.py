"""The kernels of one decoder layer of the chunked prefill (Sec. 3 "Chunk Prefill"), each run alone at the
shape it has in a configured workload, through the C ABI's op calls.

    python -m paper_2410_03065_amd.kernel_bench                       # Llama3-8B shape, 1024 rows, last chunk of 32K
    python -m paper_2410_03065_amd.kernel_bench --ops gateup --iters 8 --weight-sets 1 --vendor
    python -m paper_2410_03065_amd.kernel_bench --shape llama2-7b-shape --rows 512 --tok-begin 15872

Per op it prints the mean launch time (HIP events on the compute stream around `--iters` launches) and the
TFLOP/s that follow from the op's algorithmic FLOP count.  `--weight-sets n` cycles the GEMMs through n copies of
the weights so that, as in the prefill, a launch finds its weights in HBM and not in the caches (n = 1: the same
operands every time).  `--vendor` runs the same products through torch.matmul (the vendor's GEMM library) right
after ours: it is there so that a counter run (rocprofv3 --pmc) over this command holds both kernels side by
side, and is not used by anything else in the package.
"""
from __future__ import annotations

import argparse
import ctypes as C
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

OPS = ("qkv", "attention", "o", "gateup", "down", "mfma")


def main(argv=None):
    ap = argparse.ArgumentParser(description=__doc__.split("\n\n")[0])
    ap.add_argument("--shape", default="llama3-8b-shape")
    ap.add_argument("--rows", type=int, default=1024, help="tokens of the chunk (M of the GEMMs)")
    ap.add_argument("--tok-begin", type=int, default=31744, help="position of the chunk's first token (attention)")
    ap.add_argument("--iters", type=int, default=20)
    ap.add_argument("--warm", type=int, default=3)
    ap.add_argument("--weight-sets", type=int, default=8)
    ap.add_argument("--ops", default="qkv,attention,o,gateup,down",
                    help="comma-separated: qkv, attention, o, gateup, down, and mfma (the MFMA-only yardstick, cake_op_mfma_rate)")
    ap.add_argument("--gemm-config", type=int, default=0, help="0 = the library's choice, 1..7 = force a kernel")
    ap.add_argument("--gemm-ksplit", type=int, default=0, help="0 = the library's choice, n = K in n ranges where the kernel allows")
    ap.add_argument("--attn-variant", type=int, default=0)
    ap.add_argument("--vendor", action="store_true", help="also run the GEMMs through torch.matmul")
    args = ap.parse_args(argv)

    import torch
    import synth_inputs as si
    import paper_2410_03065_amd as cake

    full = si.SHAPES[args.shape]
    if full.dtype != "bf16":
        sys.exit("kernel_bench: bf16 shapes only")
    shape = full.with_(n_layers=1, vocab=1024)
    M, d, hd = args.rows, shape.d_model, shape.head_dim
    hq, hkv, ff = shape.n_q * hd, shape.n_kv * hd, shape.ffn
    T = args.tok_begin + M
    ops = [o for o in args.ops.split(",") if o]
    for o in ops:
        if o not in OPS:
            sys.exit("kernel_bench: unknown op %r (known: %s)" % (o, ", ".join(OPS)))
    eng = cake.Engine(shape, None, max_tokens=T, max_chunk=M, page_tokens=256, seed=0)
    eng.set_tuning(gemm_config=args.gemm_config, gemm_ksplit=args.gemm_ksplit, attn_variant=args.attn_variant)
    lib, ctx = eng.lib, eng.ctx
    g = torch.Generator(device="cuda").manual_seed(1)

    def rnd(rows, cols, std):
        return (torch.randn(rows, cols, device="cuda", generator=g) * std).to(torch.bfloat16)

    ws = max(1, args.weight_sets)
    bf, f32 = torch.bfloat16, torch.float32
    cases = {}   # op -> (flop, launch(i), vendor(i) or None)

    def gemm_case(N, K, residual):
        a, w = rnd(M, K, 1.0), [rnd(N, K, 0.02) for _ in range(ws)]
        out = torch.zeros(M, N, device="cuda", dtype=f32)
        call = lib.cake_op_gemm_residual if residual else lib.cake_op_gemm
        return (2.0 * M * N * K,
                lambda i: call(ctx, a.data_ptr(), w[i % ws].data_ptr(), out.data_ptr(), M, N, K),
                lambda i: torch.matmul(a, w[i % ws].t()))

    def gateup_case():
        a = rnd(M, d, 1.0)
        wg, wu = [rnd(ff, d, 0.02) for _ in range(ws)], [rnd(ff, d, 0.02) for _ in range(ws)]
        wgu = [torch.cat([wg[i], wu[i]]) for i in range(ws)] if args.vendor else None
        out = torch.empty(M, ff, device="cuda", dtype=bf)
        return (2.0 * M * d * 2 * ff,
                lambda i: lib.cake_op_gemm_swiglu(ctx, a.data_ptr(), wg[i % ws].data_ptr(), wu[i % ws].data_ptr(),
                                                  out.data_ptr(), M, ff, d),
                (lambda i: torch.matmul(a, wgu[i % ws].t())) if args.vendor else None)

    def attention_case():
        eng.pool.normal_(0.0, 1.0)
        q = torch.randn(shape.n_q, M, hd, device="cuda", generator=g).to(bf)
        ao = torch.empty(M, hq, device="cuda", dtype=bf)
        keys = args.tok_begin * M + M * (M + 1) // 2
        return (4.0 * shape.n_q * hd * keys,
                lambda i: lib.cake_op_attention(ctx, q.data_ptr(), ao.data_ptr(), 0, args.tok_begin, M, C.byref(eng.kv)),
                None)

    make = {"qkv": lambda: gemm_case(hq + 2 * hkv, d, False), "attention": attention_case,
            "o": lambda: gemm_case(d, hq, True), "gateup": gateup_case, "down": lambda: gemm_case(d, ff, True)}
    for o in ops:
        if o != "mfma":
            cases[o] = make[o]()

    def timed(fn, check):
        for i in range(args.warm):
            rc = fn(i)
            if check and rc != 0:
                raise cake.CakeError(rc, "kernel_bench")
        eng.sync()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        with torch.cuda.stream(eng.compute_stream):
            e0.record()
            for i in range(args.iters):
                fn(i)
            e1.record()
        e1.synchronize()
        return e0.elapsed_time(e1) * 1e3 / args.iters

    print("# %s, %d rows, chunk begins at token %d, %d weight set(s), %d launches each"
          % (full.name, M, args.tok_begin, ws, args.iters))
    print("# %-10s %10s %10s %12s %12s" % ("op", "us", "TFLOP/s", "vendor us", "vendor TFLOP/s"))
    for o in ops:
        if o == "mfma":   # 2048 workgroups x 8 waves x 4096 rounds of eight 32x32x16 MFMAs on register operands
            rates = sorted(eng.mfma_rate(2048, 4096) for _ in range(3))
            print("  %-10s %10s %10.1f   (median of three 10 ms launches; min %.1f, max %.1f)" % (o, "-", rates[1], rates[0], rates[2]), flush=True)
            continue
        flop, ours, vendor = cases[o]
        us = timed(ours, True)
        line = "  %-10s %10.1f %10.1f" % (o, us, flop / us / 1e6)
        if args.vendor and vendor is not None:
            vus = timed(vendor, False)
            line += " %12.1f %12.1f" % (vus, flop / vus / 1e6)
        print(line, flush=True)
    eng.close()


if __name__ == "__main__":
    main()
