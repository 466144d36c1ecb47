#!/usr/bin/env python3
"""Benchmark of the bidirectional KV-cache producer on one MI355X.

Workload (default): Llama3-8B-shaped decoder (32 layers, d 4096, 32 query / 8 KV heads x 128,
FFN 14336, vocab 128256), bf16, random weights N(0, 0.02); one 32768-token uniform-random
prompt, chunk 1024; stored KV for every chunk in pinned host memory acting as the storage
tier, throttled to 4 GB/s.  A "step" is one whole bidirectional prefill (every chunk of the
prompt either computed on the compute stream or loaded on the copy stream, planner running).
All inputs (weights, token ids, stored KV, KV pool) are resident before the timed region.

Prints ONE JSON line.  `value` is the mean time-to-first-token of the timed bidirectional
steps in seconds (entry of cake_bidirectional_prefill -> every chunk's KV resident).

After the headline workload the same measurement runs on the other configured workloads and is
appended under "configs" (tiny fp32 model at 1 GB/s; Llama2-7B shape, 16K tokens, chunk 512, 4 GB/s;
Llama3-8B shape, 64K tokens at 2, 8 and 25 GB/s; Llama2-70B shape, 72K tokens, 8 GB/s; about a
minute and a half together); `--headline-only` skips them, the headline keys are the same either way.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA, the published figure
PEAK_HBM_GBS = 8000.0
# One 32x32x16 bf16 MFMA is 32768 FLOP and occupies a SIMD's matrix pipe for 8 passes of 4 clocks,
# i.e. 1024 FLOP per clock per SIMD, 4 SIMDs per compute unit.
BF16_FLOP_PER_CU_PER_CLOCK = 4096
TRAFFIC_SUMMARY = os.path.join("profiles", "hbm_traffic_llama3_8b_32k.md")


def derived_peak(eng):
    """The bf16 MFMA peak from what the device reports: compute units x clock x FLOP per CU per clock."""
    cus, khz, mem = eng.device_info()
    return {"compute_units": cus, "clock_mhz": round(khz / 1e3, 1), "flop_per_cu_per_clock": BF16_FLOP_PER_CU_PER_CLOCK,
            "tflops": round(cus * khz * 1e3 * BF16_FLOP_PER_CU_PER_CLOCK / 1e12, 1), "hbm_gib": round(mem / 2.0 ** 30, 1)}


def cpu_baseline(shape, chunk, n_tokens, total_flops):
    """Times the oracle (as it stands) on a bounded sample: the first 4 chunks of the prompt
    through 4 layers of the same widths (10-20 s of host work), scaled to the whole job by FLOP count."""
    import numpy as np
    import synth_inputs as si
    from oracle import transformer as otf
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count()
    n_s = max(1, min(4, n_tokens // chunk))
    small = shape.with_(n_layers=min(4, shape.n_layers), vocab=4096)
    w = si.make_weights(small, seed=0)
    toks = si.make_tokens(n_s * chunk, small.vocab, seed=1)
    t0 = time.perf_counter()
    otf.prefill_chunked(w, small, toks, chunk, kv_dtype="bf16")
    dt = time.perf_counter() - t0
    fl = sum(otf.chunk_flops(small, i, chunk) for i in range(n_s))
    return {
        "value": dt * total_flops / fl, "unit": "s (TTFT, compute-only, extrapolated by FLOPs)",
        "cores": int(threads), "blas_threads": int(threads), "host_cpus": os.cpu_count(), "kind": "oracle",
        "sample": "oracle.prefill_chunked: first %d chunks of %d tokens through %d of %d layers at full width, "
                  "%.1f s measured, %.3f TFLOP; scaled x%.0f to the %d-token, %d-layer job"
                  % (n_s, chunk, small.n_layers, shape.n_layers, dt, fl / 1e12, total_flops / fl, n_tokens, shape.n_layers),
        "measured_s": dt, "measured_tflops": fl / dt / 1e12,
        "tiny_config": cpu_baseline_tiny(int(threads)),
    }


def cpu_baseline_tiny(threads):
    """The smallest configured workload run whole by the oracle: the full chunked prefill of the tiny
    fp32 model (2 layers, d 256, 2048 tokens, chunk 256) and the exhaustive meet-point search
    (Sec. 3.1) over its 8 chunks and over a 4096-chunk instance, each timed on the host."""
    import numpy as np
    import synth_inputs as si
    from oracle import transformer as otf
    from oracle import meet_point as omp
    shape, T, C = si.TINY, 2048, 256
    w = si.make_weights(shape, seed=0)
    toks = si.make_tokens(T, shape.vocab, seed=1)
    t0 = time.perf_counter()
    otf.prefill_chunked(w, shape, toks, C, kv_dtype="f32")
    dt = time.perf_counter() - t0
    n = T // C
    fl = [otf.chunk_flops(shape, i, C) for i in range(n)]
    c = [int(f / 1e3) for f in fl]                           # ns at 1 TFLOP/s
    l = [C * otf.kv_bytes_per_token(shape.n_layers, shape.n_kv, shape.head_dim, 4)] * n   # ns at 1 GB/s
    t0 = time.perf_counter()
    for _ in range(1000):
        m = omp.brute_force_meet_point(c, l)
    dt_plan = (time.perf_counter() - t0) / 1000
    rng = np.random.default_rng(0)
    big_c = np.cumsum(rng.integers(1, 1000, 4096)).tolist()
    big_l = rng.integers(1000, 2000000, 4096).tolist()
    t0 = time.perf_counter()
    omp.brute_force_meet_point(big_c, big_l)
    dt_big = time.perf_counter() - t0
    return {"workload": "tiny-f32, 2048 tokens, chunk 256, float64 oracle", "prefill_s": round(dt, 4),
            "prefill_gflops": round(sum(fl) / dt / 1e9, 2), "meet_point_search_8_chunks_s": round(dt_plan, 8),
            "meet_point_8_chunks_at_1tflops_1gbs": m if isinstance(m, int) else list(m),
            "meet_point_search_4096_chunks_s": round(dt_big, 4), "cores": threads, "blas_threads": threads}


def recorded_traffic(kernel_class, default_workload):
    """HBM bytes per launch of a kernel class as measured with rocprofv3 --pmc FETCH_SIZE /
    WRITE_SIZE on the default workload (summary kept under profiles/); None if not recorded."""
    if not default_workload:
        return None
    path = os.path.join(ROOT, TRAFFIC_SUMMARY)
    try:
        for line in open(path):
            f = line.split()
            if len(f) == 3 and f[0] == "traffic_bytes_per_launch" and f[1] == kernel_class:
                return int(f[2])
    except OSError:
        pass
    return None


def measure_config(cake, si, torch, name, T, C, pt, gbps_list, steps, warmup):
    """TTFT of one configured workload under the three regimes (compute-only, load-only at each tier
    bandwidth, bidirectional at each), with the per-class kernel rates of one bracketed compute-only pass."""
    import numpy as np
    shape = si.SHAPES[name]
    n = (T + C - 1) // C
    step = max(C, 1024) if shape.dtype == "bf16" else C    # compute step of the wide-step leg below
    eng = cake.Engine(shape, None, max_tokens=T, max_chunk=step, page_tokens=pt, seed=0, with_head=False)
    toks = si.make_tokens(T, shape.vocab, seed=1)
    # the pass that produces the stored KV is also the one with every kernel class bracketed by events
    eng.profile_enable(True)
    eng.bidirectional_prefill(toks, C, gbps_list[0], mode="compute_only", log=False)
    stats = eng.profile_read()
    eng.profile_enable(False)
    eng.store_from_pool(T)
    r_c = eng.bidirectional_prefill(toks, C, gbps_list[0], mode="compute_only")
    kernels = {k: {"avg_us": round(v["total_ns"] / v["launches"] / 1e3, 2),
                   "tflops": round(v["flops"] / v["total_ns"] / 1e3, 1) if v["flops"] else None}
               for k, v in stats.items() if v["launches"]}
    tiers = {}
    for gbps in gbps_list:
        for _ in range(warmup):
            eng.bidirectional_prefill(toks, C, gbps, mode="bidir", log=False)
        runs = [eng.bidirectional_prefill(toks, C, gbps, mode="bidir") for _ in range(steps)]
        r_l = eng.bidirectional_prefill(toks, C, gbps, mode="load_only")
        ttft = float(np.mean([r.ttft_ns for r in runs])) / 1e9
        load_bytes = sum(r.load_bytes for r in runs)
        load_ns = sum(r.load_busy_ns for r in runs)
        tiers["%g_gbs" % gbps] = {
            "bidirectional": round(ttft, 5), "load_only": round(r_l.ttft_ns / 1e9, 5),
            "meet_point": [r.meet_point for r in runs],
            "speedup_over_load_only": round(r_l.ttft_ns / 1e9 / ttft, 3),
            "speedup_over_compute_only": round(r_c.ttft_ns / 1e9 / ttft, 3),
            "achieved_gbps_bidirectional": round(load_bytes / load_ns, 4) if load_ns else None,
            "achieved_gbps_load_only": round(r_l.achieved_gbps, 4)}
    # Chunks shorter than 1024 tokens halve the GEMMs' M.  The engine's compute step and its fetch unit are separate
    # (Sec. 5.1 "Implementation": 128-token fetch chunks under 512/1024-token compute chunks), so the same request
    # also runs with 1024-token compute steps over fetch units of one chunk: two chunks' rows per pass over the weights.
    wide = None
    if step > C:
        reqs = [dict(tokens=toks, arrival_ns=0, prefix=True)]
        wide = {}
        for gbps in gbps_list:
            eng.adaptive_serve(reqs, step, C, gbps)
            fr = [eng.adaptive_serve(reqs, step, C, gbps) for _ in range(steps)]
            wide["%g_gbs" % gbps] = {"compute_step_tokens": step, "fetch_unit_tokens": C,
                                     "ttft_s": round(float(np.mean([f[0].ttft_ns for f in fr])) / 1e9, 5),
                                     "tokens_computed": [f[1][0]["tokens_computed"] for f in fr],
                                     "tokens_loaded": [f[1][0]["tokens_loaded"] for f in fr]}
        r_w = eng.bidirectional_prefill(toks, step, gbps_list[0], mode="compute_only")
        wide["compute_only_s"] = round(r_w.ttft_ns / 1e9, 5)
        wide["prefill_tflops_compute_only"] = round(r_w.compute_tflops, 1)
    out = {"workload": "%s, %d random tokens, chunk %d, page %d, stored KV in pinned host memory at %s GB/s"
                       % (shape.name, T, C, pt, "/".join("%g" % g for g in gbps_list)),
           "dtype": "bf16" if shape.dtype == "bf16" else "f32", "n_chunks": n, "steps": steps, "warmup": warmup,
           "compute_only_s": round(r_c.ttft_ns / 1e9, 5), "prefill_tflops_compute_only": round(r_c.compute_tflops, 1),
           "tiers": tiers, "kernels": kernels}
    if shape.dtype == "bf16":
        out["mfma_util_compute_only"] = round(r_c.compute_tflops / PEAK_BF16_TFLOPS, 4)
    if wide:
        out["wide_compute_steps"] = wide
    eng.close()
    del eng
    torch.cuda.empty_cache()
    return out


# the configured workloads besides the headline one: (key, shape, tokens, chunk, tier bandwidths in GB/s)
OTHER_CONFIGS = [
    ("tiny_f32_2k", "tiny-f32", 2048, 256, [1.0]),
    ("llama2_7b_16k_chunk512", "llama2-7b-shape", 16384, 512, [4.0]),
    ("llama3_8b_64k", "llama3-8b-shape", 65536, 1024, [2.0, 8.0, 25.0]),
    ("llama2_70b_72k", "llama2-70b-shape", 73728, 1024, [8.0]),
]


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--shape", default="llama3-8b-shape")
    ap.add_argument("--tokens", type=int, default=32768)
    ap.add_argument("--chunk", type=int, default=1024)
    ap.add_argument("--page-tokens", type=int, default=256)
    ap.add_argument("--gbps", type=float, default=4.0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-profile", action="store_true", help="do not bracket kernels with events in the timed region")
    ap.add_argument("--all-configs", action="store_true",
                    help="after the headline workload, also measure the other configured workloads (key \"configs\"); "
                         "this is the default, the flag is accepted for clarity")
    ap.add_argument("--headline-only", action="store_true", help="skip the other configured workloads")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one 1 GiB device-to-device copy, so a counter run has a kernel of known traffic")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
              "--gpus %d is not supported. Run with --gpus 1." % args.gpus, file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import synth_inputs as si
    import paper_2410_03065_amd as cake

    shape = si.SHAPES[args.shape]
    T, C, pt = args.tokens, args.chunk, args.page_tokens
    n = (T + C - 1) // C
    eng = cake.Engine(shape, None, max_tokens=T, max_chunk=C, page_tokens=pt, seed=0, with_head=True)
    toks = si.make_tokens(T, shape.vocab, seed=1)
    total_flops = sum(cake.range_flops(shape, i * C, min(C, T - i * C)) for i in range(n))
    kv_bytes = n * (C // pt) * cake.page_image_bytes(shape, pt)

    if args.calibrate_copy:   # 2^28 float32 read + written once: 1 GiB each way
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # stored KV = our own compute-only pass, copied into pinned host memory (the storage tier)
    eng.bidirectional_prefill(toks, C, args.gbps, mode="compute_only", log=False)
    eng.store_from_pool(T)

    for _ in range(args.warmup):
        eng.bidirectional_prefill(toks, C, args.gbps, mode="bidir", log=False)
    # One untimed pass with every kernel class bracketed by HIP events: the per-class table, and which
    # class has the largest share of GPU time on this workload (gate/up GEMM on the benchmark workload).
    stats, dominant = {}, None
    if not args.no_profile:
        eng.profile_enable(True)
        eng.bidirectional_prefill(toks, C, args.gbps, mode="bidir", log=False)
        stats = eng.profile_read()
        dominant = max((k for k in stats if stats[k]["launches"]), key=lambda k: stats[k]["total_ns"])
    # Timed region: only the dominant class is bracketed (one pair per layer; bracketing all eight
    # classes stretches a chunk by 10 % and the TTFT by 4 %).
    if not args.no_profile:
        eng.profile_enable(True, classes=[dominant])
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    runs = [eng.bidirectional_prefill(toks, C, args.gbps, mode="bidir") for _ in range(args.steps)]
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    dom_stats = eng.profile_read() if not args.no_profile else {}
    eng.profile_enable(False)

    # yardstick: bf16 MFMAs on register operands only, every CU busy for ~10 ms (median of three)
    mfma_only = sorted(eng.mfma_rate(2048, 4096) for _ in range(3))[1]

    # first-token step on the complete cache (reported beside the headline value, not inside it)
    eng.first_token(toks)
    if not args.no_profile:
        eng.profile_enable(True)
    t1 = time.perf_counter()
    ft = [eng.first_token(toks) for _ in range(3)]
    ft_wall = (time.perf_counter() - t1) / 3
    ft_stats = eng.profile_read() if not args.no_profile else {}
    eng.profile_enable(False)
    first_token = {"token": ft[-1][0], "wall_ms": round(ft_wall * 1e3, 3),
                   "device_ms": round(float(np.mean([f[1] for f in ft])) / 1e6, 3), "bound": "hbm", "peak_gbs": PEAK_HBM_GBS}
    for name in ("gemv", "decode_attention"):
        st = ft_stats.get(name)
        if st and st["launches"]:
            first_token[name] = {"launches": st["launches"], "total_ms": round(st["total_ns"] / 3e6, 3),
                                 "gbs": round(st["bytes"] / st["total_ns"], 1),
                                 "frac_of_hbm_peak": round(st["bytes"] / st["total_ns"] / PEAK_HBM_GBS, 3)}

    # fetch unit of one page (finer than the compute chunk): the adaptive engine with this request alone
    fine = None
    if pt < C:
        reqs = [dict(tokens=toks, arrival_ns=0, prefix=True)]
        eng.adaptive_serve(reqs, C, pt, args.gbps)
        fr = [eng.adaptive_serve(reqs, C, pt, args.gbps) for _ in range(2)]
        fine = {"fetch_unit_tokens": pt, "compute_step_tokens": C,
                "ttft_s": round(float(np.mean([f[0].ttft_ns for f in fr])) / 1e9, 5),
                "tokens_computed": [f[1][0]["tokens_computed"] for f in fr],
                "tokens_loaded": [f[1][0]["tokens_loaded"] for f in fr]}

    r_c = eng.bidirectional_prefill(toks, C, args.gbps, mode="compute_only")
    r_l = eng.bidirectional_prefill(toks, C, args.gbps, mode="load_only")

    # the same tier with an 8-bit store written from the pool (which the compute-only pass just filled)
    eng.bidirectional_prefill(toks, C, args.gbps, mode="compute_only", log=False)
    eng.write_store(T, cake.STORE_INT8)
    eng.bidirectional_prefill(toks, C, args.gbps, mode="bidir", log=False)
    r8 = [eng.bidirectional_prefill(toks, C, args.gbps, mode="bidir") for _ in range(2)]
    r8_l = eng.bidirectional_prefill(toks, C, args.gbps, mode="load_only")
    int8_store = {"ttft_s": round(float(np.mean([r.ttft_ns for r in r8])) / 1e9, 5), "meet_point": [r.meet_point for r in r8],
                  "load_only_s": round(r8_l.ttft_ns / 1e9, 5), "store_bytes": int(r8_l.load_bytes),
                  "achieved_gbps_load_only": round(r8_l.achieved_gbps, 4)}

    # and with the 4-bit store (two codes per byte)
    eng.bidirectional_prefill(toks, C, args.gbps, mode="compute_only", log=False)
    eng.write_store(T, cake.STORE_INT4)
    eng.bidirectional_prefill(toks, C, args.gbps, mode="bidir", log=False)
    r4 = [eng.bidirectional_prefill(toks, C, args.gbps, mode="bidir") for _ in range(2)]
    r4_l = eng.bidirectional_prefill(toks, C, args.gbps, mode="load_only")
    int4_store = {"ttft_s": round(float(np.mean([r.ttft_ns for r in r4])) / 1e9, 5), "meet_point": [r.meet_point for r in r4],
                  "load_only_s": round(r4_l.ttft_ns / 1e9, 5), "store_bytes": int(r4_l.load_bytes),
                  "achieved_gbps_load_only": round(r4_l.achieved_gbps, 4)}

    ttft = float(np.mean([r.ttft_ns for r in runs])) / 1e9
    comp_flops = sum(r.compute_flops for r in runs)
    comp_dev_ns = sum(r.compute_device_ns for r in runs)
    load_bytes = sum(r.load_bytes for r in runs)
    load_ns = sum(r.load_busy_ns for r in runs)
    prefill_tflops = comp_flops / comp_dev_ns / 1e3 if comp_dev_ns else 0.0

    kernels = {}
    roofline = None
    if stats:
        for name, s in stats.items():
            if not s["launches"]:
                continue
            avg_us = s["total_ns"] / s["launches"] / 1e3
            k = {"launches": s["launches"], "avg_us": round(avg_us, 2), "share": 0.0}
            if s["flops"]:
                k["tflops"] = round(s["flops"] / s["total_ns"] / 1e3, 1)
            k["gbs"] = round(s["bytes"] / s["total_ns"], 1)
            kernels[name] = k
        tot = sum(s["total_ns"] for s in stats.values())
        for name in kernels:
            kernels[name]["share"] = round(stats[name]["total_ns"] / tot, 3)
        dom = dominant
        s = dom_stats[dom]                       # from the timed region itself
        achieved = s["flops"] / s["total_ns"] / 1e3
        traffic = recorded_traffic(dom, (args.shape, T, C, pt) == ("llama3-8b-shape", 32768, 1024, 256))
        roofline = {"kernel": dom, "bound": "mfma", "achieved": round(achieved, 1), "peak": PEAK_BF16_TFLOPS,
                    "unit": "TFLOP/s", "frac": round(achieved / PEAK_BF16_TFLOPS, 4),
                    "peak_source": "published dense bf16 figure; peak_derived is this device's compute units x "
                                   "clock x 4096 FLOP per CU per clock",
                    "peak_derived": derived_peak(eng),
                    "traffic": traffic,
                    "traffic_source": None if traffic is None else
                    "recorded, not measured in this run: %s (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE passes over "
                    "this command, scaled by a 1 GiB copy)" % TRAFFIC_SUMMARY,
                    "avg_launch_us": round(s["total_ns"] / s["launches"] / 1e3, 2), "launches": s["launches"],
                    "flops_per_launch": s["flops"] // s["launches"]}

    # what the race costs the compute side: the same chunks' device times in the bidirectional and the compute-only pass
    m_last = runs[-1].meet_point
    both = [(a["device_ns"], b["device_ns"]) for a, b in zip(runs[-1].chunks[:m_last], r_c.chunks[:m_last]) if a["device_ns"] and b["device_ns"]]
    chunk_time_ratio = round(sum(a for a, _ in both) / sum(b for _, b in both), 4) if both else None

    out = {
        "metric": "ttft_s_32k_prompt_bidirectional", "value": round(ttft, 5), "unit": "s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(wall / args.steps * 1e3, 3), "higher_is_better": False, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16" if shape.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": "%s, %d random tokens, chunk %d, page %d, stored KV in pinned host memory at %.3g GB/s"
                               % (shape.name, T, C, pt, args.gbps),
                   "global_batch": 1, "seq_len": T, "parallelism": "single-gpu"},
        "ttft_s": {"bidirectional": round(ttft, 5), "compute_only": round(r_c.ttft_ns / 1e9, 5),
                   "load_only": round(r_l.ttft_ns / 1e9, 5),
                   "bidirectional_median": round(float(np.median([r.ttft_ns for r in runs])) / 1e9, 5),
                   "bidirectional_min": round(min(r.ttft_ns for r in runs) / 1e9, 5)},
        "speedup": {"over_load_only": round(r_l.ttft_ns / 1e9 / ttft, 3),
                    "over_compute_only": round(r_c.ttft_ns / 1e9 / ttft, 3)},
        "sum_ttft_over_baselines": round(ttft / (r_c.ttft_ns / 1e9) + ttft / (r_l.ttft_ns / 1e9), 4),
        "meet_point": [r.meet_point for r in runs], "n_chunks": n,
        "computed_chunk_time_bidirectional_over_compute_only": chunk_time_ratio,
        "prefill_tflops": {"bidirectional_compute_side": round(prefill_tflops, 1),
                           "compute_only": round(r_c.compute_tflops, 1), "algorithmic_total_tflop": round(total_flops / 1e12, 1)},
        "mfma_util": {"bidirectional_compute_side": round(prefill_tflops / PEAK_BF16_TFLOPS, 4),
                      "compute_only": round(r_c.compute_tflops / PEAK_BF16_TFLOPS, 4), "peak_tflops": PEAK_BF16_TFLOPS},
        "load_gbps": {"configured": args.gbps, "achieved_bidirectional": round(load_bytes / load_ns, 4) if load_ns else None,
                      "achieved_load_only": round(r_l.achieved_gbps, 4), "kv_bytes": kv_bytes},
        "kernels": kernels, "kernels_note": "per-class table from one untimed pass with every class bracketed by events "
                                            "(that pass runs ~10 % slower); roofline.achieved is from the timed region",
        "first_token": dict(first_token, ttft_to_first_token_s=round(ttft + ft_wall, 5)),
        "fine_fetch_unit": fine,
        "mfma_only": {"tflops": round(mfma_only, 1), "frac_of_peak": round(mfma_only / PEAK_BF16_TFLOPS, 4),
                      "what": "bf16 32x32x16 MFMAs on register operands, no memory traffic, every CU busy for "
                              "about 10 ms: the rate the matrix pipes sustain at the clock the device holds "
                              "under that load (cake_op_mfma_rate)"},
        "int8_store": int8_store,
        "int4_store": int4_store,
        "roofline": roofline,
    }
    if not args.headline_only:
        eng.close()
        del eng
        torch.cuda.empty_cache()
        out["configs"] = {}
        for key, name, T2, C2, tiers in OTHER_CONFIGS:
            t_cfg = time.perf_counter()
            out["configs"][key] = measure_config(cake, si, torch, name, T2, C2, min(pt, C2), tiers, 2, 1)
            out["configs"][key]["wall_s"] = round(time.perf_counter() - t_cfg, 1)
            print("bench.py: %s done in %.0f s" % (key, time.perf_counter() - t_cfg), file=sys.stderr, flush=True)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(shape, C, T, total_flops)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
