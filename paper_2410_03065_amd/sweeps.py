#!/usr/bin/env python3
"""Utilisation x bandwidth grid and fluctuation trace of the paper's evaluation, on synthetic input.

    python -m paper_2410_03065_amd.sweeps --grid          # Sec. 5.2 / Table 3 layout
    python -m paper_2410_03065_amd.sweeps --fluctuation   # Sec. 5.6 / Fig. 5 layout
    python -m paper_2410_03065_amd.sweeps --mix           # prefix request + Poisson arrivals, bandwidth step
    python -m paper_2410_03065_amd.sweeps --burst         # Sec. 5.7 layout: prefix request + a burst of short requests
    python -m paper_2410_03065_amd.sweeps --compression   # Sec. 5.5 / Table 6 layout: bandwidth x stored-KV precision
    python -m paper_2410_03065_amd.sweeps --chunks        # Sec. 3.2 / Fig. 4 layout: per-chunk compute and load time
    python -m paper_2410_03065_amd.sweeps --lengths --shape longalpaca-13b-shape --tokens 16384 --budget 512
                                                          # Sec. 5.3 / Table 4 layout: prompt length x bandwidth

Grid: one prefix-cached prompt (default: Llama3-8B shape, 32768 random tokens) is produced by the
adaptive engine while other users hold 0 / 12.5 / 50 / 87.5 % of every step's token budget, at the
tier bandwidths the paper lists (7, 25, 32, 56, 100 Gbps).  Each cell prints TTFT and the speed-up
over load-only (KV bytes / bandwidth, measured) and over compute-only at the same utilisation
(measured with the tier made useless).  Prints a Markdown table; inputs are seeded and synthetic.
"""
from __future__ import annotations

import argparse
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--grid", action="store_true")
    ap.add_argument("--fluctuation", action="store_true")
    ap.add_argument("--mix", action="store_true", help="one prefix-cached request among Poisson arrivals of 4K-token requests, "
                    "bandwidth stepping 25 -> 2 GB/s when the loader has completed its 8th chunk")
    ap.add_argument("--burst", action="store_true", help="prefix request, then 22 requests of 32-448 tokens: finish time when the "
                    "prefix request runs to completion first against the adaptive mode")
    ap.add_argument("--compression", action="store_true", help="tier bandwidth x store format (16-bit, 8-bit, 4-bit): "
                    "speed-up over load-only and over compute-only, the request alone on the GPU")
    ap.add_argument("--chunks", action="store_true", help="time of every chunk when computed (grows with its position) "
                    "and when loaded (constant), at the first --gbit bandwidth")
    ap.add_argument("--lengths", action="store_true", help="prompt length (quarters of --tokens) x tier bandwidth: "
                    "speed-up over load-only and over compute-only, the request alone on the GPU")
    ap.add_argument("--rate", type=float, default=2.0, help="arrivals per second of the other requests (--mix)")
    ap.add_argument("--other-tokens", type=int, default=4096)
    ap.add_argument("--shape", default="llama3-8b-shape")
    ap.add_argument("--tokens", type=int, default=32768)
    ap.add_argument("--budget", type=int, default=1024, help="token budget of an engine step")
    ap.add_argument("--fetch-unit", type=int, default=256)
    ap.add_argument("--gbit", type=float, nargs="*", default=[7, 25, 32, 56, 100], help="tier bandwidths in Gbit/s")
    ap.add_argument("--shares", type=float, nargs="*", default=[0.125, 0.5, 0.875, 1.0])
    args = ap.parse_args()

    import numpy as np
    import synth_inputs as si
    import paper_2410_03065_amd as cake

    shape = si.SHAPES[args.shape]
    T, B, U = args.tokens, args.budget, args.fetch_unit
    eng = cake.Engine(shape, None, max_tokens=T, max_chunk=B, page_tokens=U, seed=0)
    toks = si.make_tokens(T, shape.vocab, seed=1)
    eng.bidirectional_prefill(toks, B, 4.0, mode="compute_only", log=False)     # stored KV = our own compute-only pass
    eng.store_from_pool(T)
    reqs = [dict(tokens=toks, arrival_ns=0, prefix=True)]

    def run(gbps, other=None, gbps_trace=None, interval_ns=0):
        if other is not None or gbps_trace is not None:
            eng.set_traces(other_tokens=other, gbps_trace=gbps_trace, gbps_interval_ns=interval_ns)
        return eng.adaptive_serve(reqs, B, U, gbps)

    run(4.0)   # warm-up
    print("workload: %s, %d random tokens, step budget %d, fetch unit %d, one MI355X" % (shape.name, T, B, U))
    if args.grid:
        load_only = {}
        for gb in args.gbit:
            r = eng.bidirectional_prefill(toks, B, gb / 8.0, mode="load_only", log=False)
            load_only[gb] = r.ttft_ns / 1e9
        print("\n| utilisation | compute-only s | " + " | ".join("%g Gbps: TTFT s (x load-only \\\\ x compute-only)" % g for g in args.gbit) + " |")
        print("|---|---|" + "---|" * len(args.gbit))
        for share in args.shares:
            other = int(round(B * (1 - share)))
            tr = [other] if other else None
            res_c, _, _ = run(1e-4, tr)                                      # tier too slow to be given anything
            t_c = res_c.ttft_ns / 1e9
            assert res_c.meet_point == res_c.n_chunks
            cells = []
            for gb in args.gbit:
                res, per_req, _ = run(gb / 8.0, tr)
                t = res.ttft_ns / 1e9
                cells.append("%.3f (%.2f \\\\ %.2f) m=%d" % (t, load_only[gb] / t, t_c / t, per_req[0]["tokens_computed"]))
            print("| %.1f %% | %.3f | %s |" % (share * 100, t_c, " | ".join(cells)))
        print("\nload-only s: " + ", ".join("%g Gbps %.5f" % (g, load_only[g]) for g in args.gbit))
    if args.compression:
        r_c = eng.bidirectional_prefill(toks, B, 4.0, mode="compute_only", log=False)     # also refills the pool for the writers
        t_c = r_c.ttft_ns / 1e9
        rows = {gb: [] for gb in args.gbit}
        sizes = []
        for name, fmt in (("16-bit", cake.STORE_RAW), ("8-bit", cake.STORE_INT8), ("4-bit", cake.STORE_INT4)):
            eng.bidirectional_prefill(toks, B, 4.0, mode="compute_only", log=False)
            eng.write_store(T, fmt)
            eng.bidirectional_prefill(toks, B, 4.0, mode="bidir", log=False)              # staging of this format set up
            for gb in args.gbit:
                r_l = eng.bidirectional_prefill(toks, B, gb / 8.0, mode="load_only", log=False)
                r_b = eng.bidirectional_prefill(toks, B, gb / 8.0, mode="bidir", log=False)
                t = r_b.ttft_ns / 1e9
                rows[gb].append("%.3f (%.2f \\\\ %.2f) m=%d" % (t, r_l.ttft_ns / 1e9 / t, t_c / t, r_b.meet_point))
            sizes.append("%s %.2f GB" % (name, r_l.load_bytes / 1e9))
        print("\ncompute-only %.3f s; store sizes: %s; cell = TTFT s (x load-only \\\\ x compute-only) meet point of %d chunks"
              % (t_c, ", ".join(sizes), r_c.n_chunks))
        print("| bandwidth | 16-bit | 8-bit | 4-bit |")
        print("|---|---|---|---|")
        for gb in args.gbit:
            print("| %g Gbps | %s |" % (gb, " | ".join(rows[gb])))
    if args.compression and (args.chunks or args.lengths):
        # the compression table left its last (4-bit) store in place: the tables below are about 16-bit KV
        eng.bidirectional_prefill(toks, B, 4.0, mode="compute_only", log=False)
        eng.store_from_pool(T)
    if args.chunks:
        gb = args.gbit[0]
        r_c = eng.bidirectional_prefill(toks, B, gb / 8.0, mode="compute_only")
        r_l = eng.bidirectional_prefill(toks, B, gb / 8.0, mode="load_only")
        print("\n| chunk (of %d tokens) | computed: ms on the GPU | PFLOP/s | loaded at %g Gbps: ms |" % (B, gb))
        print("|---|---|---|---|")
        for i, (cc, cl) in enumerate(zip(r_c.chunks, r_l.chunks)):
            ms_c = cc["device_ns"] / 1e6
            print("| %d | %.2f | %.2f | %.2f |" % (i, ms_c, cc["work"] / max(1, cc["device_ns"]) / 1e6, (cl["end_ns"] - cl["start_ns"]) / 1e6))
    if args.lengths:
        print("\ncell = TTFT s (x load-only \\\\ x compute-only) meet point / chunks; chunk %d" % B)
        print("| prompt tokens | compute-only s | " + " | ".join("%g Gbps" % g for g in args.gbit) + " |")
        print("|---|---|" + "---|" * len(args.gbit))
        for quarter in (1, 2, 3, 4):
            n = max(B, (T * quarter // 4) // U * U)
            part = toks[:n]                                  # the stored KV of a prefix is the prefix of the stored KV
            eng.bidirectional_prefill(part, B, 4.0, mode="compute_only", log=False)
            t_c = eng.bidirectional_prefill(part, B, 4.0, mode="compute_only", log=False).ttft_ns / 1e9
            cells = []
            for gb in args.gbit:
                r_l = eng.bidirectional_prefill(part, B, gb / 8.0, mode="load_only", log=False)
                r_b = eng.bidirectional_prefill(part, B, gb / 8.0, mode="bidir", log=False)
                t = r_b.ttft_ns / 1e9
                cells.append("%.3f (%.2f \\\\ %.2f) %d/%d" % (t, r_l.ttft_ns / 1e9 / t, t_c / t, r_b.meet_point, r_b.n_chunks))
            print("| %d | %.3f | %s |" % (n, t_c, " | ".join(cells)))
    if args.mix:
        # arrivals drawn from t = -2 s so the GPU is already shared when the prefix request comes in (t = 0 here = 2 s)
        rng = np.random.default_rng(2)
        t, arrivals = 0.0, []
        while True:
            t += rng.exponential(1.0 / args.rate)
            if t > 4.0:
                break
            arrivals.append(t)
        C = B
        others = []
        for j, ta in enumerate(arrivals):
            kv, pool = eng.new_kv(args.other_tokens)
            others.append(dict(tokens=si.make_tokens(args.other_tokens, shape.vocab, seed=100 + j), arrival_ns=int(ta * 1e9),
                               prefix=False, kv=kv, pool=pool))
        mix = others + [dict(tokens=toks, arrival_ns=int(2.0e9), prefix=True)]
        for label, step_after in (("constant 4 GB/s", None), ("25 GB/s, then 2 GB/s after the loader's 8th chunk", 8)):
            gb = 4.0 if step_after is None else 25.0
            if step_after is not None:
                eng.schedule_bandwidth_step(step_after, 2.0)
            res, per_req, steps = eng.adaptive_serve(mix, B, C, gb)
            print("\nmix, %s: %d requests of %d tokens at %.1f /s (Poisson, seed 2) + the %d-token prefix request at t = 2 s"
                  % (label, len(others), args.other_tokens, args.rate, T))
            print("prefix request: TTFT %.3f s, %d tokens computed, %d loaded (meet point chunk %d of %d), %d engine steps"
                  % (per_req[-1]["ttft_ns"] / 1e9, per_req[-1]["tokens_computed"], per_req[-1]["tokens_loaded"], res.meet_point,
                     res.n_chunks, len(steps)))
            print("other requests: TTFT ms " + ", ".join("%.0f" % (p["ttft_ns"] / 1e6) for p in per_req[:-1]))
            seen, line = -1, []
            for d in res.decisions:
                if d["m_star"] != seen:
                    seen = d["m_star"]
                    line.append("%d@%.0fms" % (seen, d["now_ns"] / 1e6 - 2000.0))
            print("planned meet point over time (chunk @ ms after the prefix request arrived): " + " ".join(line))
    if args.burst:
        import time
        rng = np.random.default_rng(4)
        lens = np.clip(rng.gamma(2.0, 60.0, 22).astype(int) + 32, 32, 448)        # spiked towards short prompts
        arr = np.sort(rng.uniform(0.02, 0.30, 22))                                  # all arrive while the prefix request is in flight
        burst = []
        for j, (n_tok, ta) in enumerate(zip(lens, arr)):
            kv, pool = eng.new_kv(int(n_tok))
            burst.append(dict(tokens=si.make_tokens(int(n_tok), shape.vocab, seed=200 + j), arrival_ns=int(ta * 1e9), prefix=False,
                              kv=kv, pool=pool))
        pre = dict(tokens=toks, arrival_ns=0, prefix=True)
        eng.adaptive_serve(burst + [pre], B, U, 4.0)                                # warm-up of the small shapes
        # (a) the prefix request first, to completion; the burst waits for it
        t0 = time.perf_counter()
        r_first, _, _ = eng.adaptive_serve([pre], B, U, 4.0)
        waited = [dict(b, arrival_ns=0) for b in burst]
        eng.adaptive_serve(waited, B, U, 4.0)
        t_seq = time.perf_counter() - t0
        # (b) adaptive mode: the burst is served as it arrives, the prefix request takes what is left of each step
        t0 = time.perf_counter()
        r_ad, per_req, steps = eng.adaptive_serve(burst + [pre], B, U, 4.0)
        t_ad = time.perf_counter() - t0
        print("\nburst: %d-token prefix request at t = 0, then 22 requests of %d..%d tokens (total %d) arriving within 0.3 s, 4 GB/s"
              % (T, lens.min(), lens.max(), lens.sum()))
        print("prefix request first, burst after it: all done after %.3f s (prefix TTFT %.3f s; a burst request waits up to %.3f s)"
              % (t_seq, r_first.ttft_ns / 1e9, r_first.ttft_ns / 1e9 - arr.min()))
        print("adaptive mode: all done after %.3f s (prefix TTFT %.3f s, %d tokens computed; burst TTFT ms: median %.1f, max %.1f)"
              % (t_ad, per_req[-1]["ttft_ns"] / 1e9, per_req[-1]["tokens_computed"],
                 float(np.median([p["ttft_ns"] for p in per_req[:-1]])) / 1e6, max(p["ttft_ns"] for p in per_req[:-1]) / 1e6))
    if args.fluctuation:
        rng = np.random.default_rng(3)
        other = (B - rng.integers(0, B // 2 // 64 + 1, 64) * 64).astype(np.int32)      # the request gets 0 .. B/2 tokens a step
        gbps = rng.uniform(0.0, 25.0 / 8.0, 64)                                        # 0 .. 25 Gbit/s
        res, per_req, steps = run(25.0 / 16.0, other, gbps, 20_000_000)
        t = res.ttft_ns / 1e9
        print("\nfluctuation: budget for the request uniform in [0, %d] tokens per step, bandwidth uniform in [0, 25] Gbps "
              "re-drawn every 20 ms: TTFT %.3f s, %d tokens computed, %d loaded, %d engine steps, %d planner looks"
              % (B // 2, t, per_req[0]["tokens_computed"], per_req[0]["tokens_loaded"], len(steps), len(res.decisions)))
        print("| t ms | planned meet point (fetch unit) | load estimate GB/s | compute estimate TFLOP/s |")
        print("|---|---|---|---|")
        last = -1
        for d in res.decisions:
            ms = int(d["now_ns"] / 1e6)
            if ms // 100 != last:
                last = ms // 100
                print("| %d | %d | %.2f | %.0f |" % (ms, d["m_star"], d["est_load_bytes"] / max(1, d["est_load_ns"]),
                                                    d["est_compute_flops"] / max(1, d["est_compute_ns"]) / 1e3))


if __name__ == "__main__":
    main()
