"""CPU tests of the C ABI's host side: every declared symbol is exported, the O(n) planner
returns the oracle's brute-force integers, and the library's claim protocol replays
bit-exactly in the oracle's independent discrete-event simulator.  No GPU is touched."""
import ctypes
import os
import re

import numpy as np
import pytest

import synth_inputs as si
from oracle import meet_point as mp
from oracle import transformer as otf
import paper_2410_03065_amd as cake

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "cake.h")).read()
    declared = set(re.findall(r"\b(cake_[a-z_0-9]+)\s*\(", header))
    declared -= {"cake_ctx"}
    assert declared == set(cake.EXPORTS)
    lib = ctypes.CDLL(cake.LIB_PATH)
    for name in declared:
        assert hasattr(lib, name), name


def test_struct_sizes_match_the_header_layout():
    assert ctypes.sizeof(cake.ChunkLog) == 48
    assert ctypes.sizeof(cake.DecisionLog) == 96
    assert ctypes.sizeof(cake.Request) == 64
    assert ctypes.sizeof(cake.StepLog) == 40
    assert ctypes.sizeof(cake.ModelDesc) == 40
    assert ctypes.sizeof(cake.Tuning) == 40
    assert ctypes.sizeof(cake.Kv) == 40
    assert ctypes.sizeof(cake.KvStore) == 48 and ctypes.sizeof(cake.Traces) == 56


def test_planner_equals_brute_force_bit_exactly():
    rng = np.random.default_rng(11)
    for trial in range(600):
        n = int(rng.integers(0, 13))
        hi = int(rng.choice([3, 50, 10**6, 10**12]))
        c = rng.integers(0, hi, size=n, dtype=np.uint64)
        l = rng.integers(0, hi, size=n, dtype=np.uint64)
        oc = int(rng.integers(0, hi)) if trial % 3 == 0 else 0
        ol = int(rng.integers(0, hi)) if trial % 5 == 0 else 0
        want = mp.brute_force_meet_point([int(x) for x in c], [int(x) for x in l], oc, ol)
        assert cake.plan_meet_point(c, l, oc, ol) == want, (c, l, oc, ol)
    # larger n, against the same definition
    for n in (64, 72, 257):
        c, l = si.make_costs(n, 77 + n, 1, 10**9)
        assert cake.plan_meet_point(c, l) == mp.brute_force_meet_point([int(x) for x in c], [int(x) for x in l])


def test_planner_extremes_and_errors():
    assert cake.plan_meet_point([], []) == (0, 0)
    assert cake.plan_meet_point([5], [5]) == (0, 5)          # tie -> fewest computed chunks
    assert cake.plan_meet_point([1, 1, 1], [100, 100, 100]) == (3, 3)     # compute-only
    assert cake.plan_meet_point([100, 100, 100], [1, 1, 1]) == (0, 3)     # load-only
    with pytest.raises(cake.CakeError):
        cake.plan_meet_point([1, 1], [2**63, 2**63])                      # sums beyond 2^63 are refused
    with pytest.raises(cake.CakeError):
        cake.plan_meet_point([1], [1], compute_offset_ns=2**63)


def _shape_costs(shape, T, C, page_tokens):
    n = (T + C - 1) // C
    flops = [mp.range_flops(shape.n_layers, shape.d_model, shape.n_q, shape.n_kv, shape.head_dim, shape.ffn,
                            i * C, min((i + 1) * C, T)) for i in range(n)]
    per_page = page_tokens * otf.kv_bytes_per_token(shape.n_layers, shape.n_kv, shape.head_dim, shape.elem_bytes)
    byts = [((min((i + 1) * C, T) - i * C + page_tokens - 1) // page_tokens) * per_page for i in range(n)]
    return n, flops, byts


def _same_log(lib_log, ora_log):
    assert len(lib_log) == len(ora_log)
    for a, b in zip(lib_log, ora_log):
        assert a["f_off"] == 0 and a["partial_ns"] == 0        # whole-chunk claims only
        assert (a["who"], a["now_ns"], a["f"], a["b"], a["o_c"], a["o_l"], a["est_compute_ns"],
                a["est_compute_flops"], a["est_load_ns"], a["est_load_bytes"], a["m_star"], a["claimed"]) == \
               (b.who, b.now, b.f, b.b, b.o_c, b.o_l, b.D, b.F, b.load_ns, b.load_bytes, b.m_star, b.claimed)


@pytest.mark.parametrize("mode", ["bidir", "compute_only", "load_only", "forced", "greedy"])
def test_claim_protocol_replays_bit_exactly(mode):
    """Scripted durations that differ from the estimates (noisy compute, a bandwidth step)."""
    rng = np.random.default_rng(5)
    for trial in range(40):
        shape = [si.LLAMA3_8B, si.LLAMA2_7B, si.TINY][trial % 3]
        C = [1024, 512, 256][trial % 3]
        n_chunks = int(rng.integers(1, 40))
        T = n_chunks * C - int(rng.integers(0, C)) * (trial % 2)
        n, flops, byts = _shape_costs(shape, T, C, 256)
        tput = float(rng.uniform(2e5, 2e6))                       # flops per ns
        ac = [max(1, int(f / tput * rng.uniform(0.8, 1.3))) for f in flops]
        bw = float(rng.uniform(0.5, 30.0))                        # bytes per ns
        al = [max(1, int(b / bw)) for b in byts]
        step = int(rng.integers(0, n + 1))
        for j in range(n - 1 - step, -1, -1):                     # rate changes after `step` loads
            al[j] = max(1, int(al[j] * 7.5))
        prior_c = (10**9, int(5e14))
        prior_l = (10**9, int(bw * 1e9))
        forced = int(rng.integers(0, n + 1))
        omode = {"bidir": mp.MODE_BIDIR, "compute_only": mp.MODE_COMPUTE_ONLY, "load_only": mp.MODE_LOAD_ONLY,
                 "forced": mp.MODE_FORCED, "greedy": mp.MODE_GREEDY}[mode]
        est = mp.Estimator(prior_c[0], prior_c[1], prior_l[0], prior_l[1])
        t_o, src_o, log_o = mp.simulate_claims(n, flops, byts, ac, al, est, omode, forced)
        t_l, src_l, log_l = cake.simulate_race(flops, byts, ac, al, prior_c, prior_l, mode, forced)
        assert (t_l, src_l) == (t_o, src_o)
        _same_log(log_l, log_o)
        m = src_l.count(cake.SRC_COMPUTE)
        assert src_l == [cake.SRC_COMPUTE] * m + [cake.SRC_LOAD] * (n - m)
        # every logged planner decision is the brute-force optimum of its own logged inputs
        if mode == "bidir":
            for d in log_l:
                e = mp.Estimator(d["est_compute_ns"], d["est_compute_flops"], d["est_load_ns"], d["est_load_bytes"])
                ce = [e.est_compute(flops[i]) for i in range(d["f"], d["b"] + 1)]
                le = [e.est_load(byts[i]) for i in range(d["f"], d["b"] + 1)]
                assert d["m_star"] == d["f"] + mp.brute_force_meet_point(ce, le, d["o_c"], d["o_l"])[0]


def test_claim_protocol_load_failure_replays():
    n, flops, byts = _shape_costs(si.LLAMA3_8B, 16 * 1024, 1024, 256)
    ac = [f // 10**6 for f in flops]
    al = [b // 4 for b in byts]
    for fail in (15, 12, 9):
        est = mp.Estimator(10**9, 10**15, 10**9, 4 * 10**9)
        t_o, src_o, log_o = mp.simulate_claims(n, flops, byts, ac, al, est, fail_load_chunk=fail)
        t_l, src_l, log_l = cake.simulate_race(flops, byts, ac, al, (10**9, 10**15), (10**9, 4 * 10**9),
                                               fail_load_chunk=fail)
        assert (t_l, src_l) == (t_o, src_o)
        _same_log(log_l, log_o)
        assert src_l[fail] == cake.SRC_COMPUTE and all(s == cake.SRC_COMPUTE for s in src_l[:fail])
    with pytest.raises(cake.CakeError):      # load-only cannot recover from a failed load
        cake.simulate_race(flops, byts, ac, al, mode="load_only", fail_load_chunk=3)


def test_bidir_never_loses_to_the_baselines_when_estimates_hold():
    """The paper's sub-1.0 cells (Sec. 5.3/5.4) come from racing without a plan; with a plan
    and costs that match the estimates the result equals the best split."""
    for seed in range(60):
        n = 2 + seed % 30
        c, l = si.make_costs(n, 900 + seed, 1, 10**6)
        c, l = [int(x) for x in c], [int(x) for x in l]
        t, src, _ = cake.simulate_race(c, l, c, l)
        assert t == mp.brute_force_meet_point(c, l)[1] <= min(sum(c), sum(l))
        t_lit, _, _ = mp.literal_race(c, l)
        assert t <= t_lit


def test_sizes():
    for shape, C in ((si.LLAMA3_8B, 1024), (si.LLAMA2_70B, 1024), (si.LLAMA2_7B, 512), (si.TINY, 256)):
        for i in (0, 1, 17):
            assert cake.range_flops(shape, i * C, C) == otf.chunk_flops(shape, i, C)
        assert cake.page_image_bytes(shape, 256) == 256 * otf.kv_bytes_per_token(
            shape.n_layers, shape.n_kv, shape.head_dim, shape.elem_bytes)
    assert cake.range_flops(si.LLAMA3_8B, 1000, 24) + cake.range_flops(si.LLAMA3_8B, 1024, 1000) == \
        cake.range_flops(si.LLAMA3_8B, 1000, 1024)
    # page image sizes of the three store formats, against the oracle's
    import ctypes
    from oracle import store as ostore
    lib = cake.load_library()
    for shape in (si.LLAMA3_8B, si.LLAMA2_70B, si.TINY):
        md = ctypes.byref(cake.model_desc(shape))
        a = (shape.n_layers, shape.n_kv, shape.head_dim, 256)
        assert lib.cake_store_image_bytes(md, 256, cake.STORE_RAW) == cake.page_image_bytes(shape, 256)
        assert lib.cake_store_image_bytes(md, 256, cake.STORE_INT8) == ostore.int8_image_bytes(*a)
        assert lib.cake_store_image_bytes(md, 256, cake.STORE_INT4) == ostore.int4_image_bytes(*a)
        assert lib.cake_store_image_bytes(md, 256, 3) == 0 and lib.cake_store_image_bytes(md, 0, cake.STORE_RAW) == 0


def test_engine_refuses_to_run_without_gpu():
    import torch
    if torch.cuda.is_available():
        pytest.skip("GPU present")
    with pytest.raises(cake.CakeError):
        cake.Engine(si.TINY.with_(vocab=64), None, max_tokens=64, max_chunk=64, page_tokens=64)


def test_threaded_executor_under_thread_sanitizer(tmp_path):
    """The two-worker executor with a fake backend (sleeps instead of GPU work), built with
    ThreadSanitizer: exclusive claims, prefix/suffix sources, a failed load recomputed, no data race."""
    import shutil
    import subprocess
    if shutil.which("g++") is None:
        pytest.skip("no g++")
    exe = str(tmp_path / "race_tsan")
    src = os.path.join(ROOT, "tests", "host", "race_tsan.cpp")
    subprocess.run(["g++", "-std=c++17", "-O1", "-g", "-fsanitize=thread", "-pthread", src, "-o", exe], check=True)
    env = dict(os.environ, TSAN_OPTIONS="halt_on_error=1")
    p = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert p.returncode == 0 and "ok" in p.stdout, p.stdout + p.stderr


def test_prefix_keys_and_lookup_match_the_oracle():
    from oracle import prefix as opx
    rng = np.random.default_rng(1)
    for n, chunk in ((0, 16), (15, 16), (16, 16), (1000, 128), (4096, 1024), (777, 1)):
        toks = rng.integers(0, 2 ** 31 - 1, n).astype(np.int32)
        keys = cake.prefix_keys(toks, chunk)
        assert keys == opx.prefix_keys(toks, chunk)
        for have in (0, len(keys) // 2, len(keys)):
            stored = sorted(keys[:have] + [int(k) for k in rng.integers(0, 2 ** 63, 5)])
            assert cake.prefix_lookup(stored, keys) == opx.longest_stored_prefix(keys, stored)
        if len(keys) > 2:                                    # a gap ends the prefix
            stored = sorted(keys[:1] + keys[2:])
            assert cake.prefix_lookup(stored, keys) == 1
    with pytest.raises(cake.CakeError):
        cake.prefix_lookup([3, 2, 1], [1])                   # index not ascending
    with pytest.raises(cake.CakeError):
        cake.prefix_keys(np.zeros(4, dtype=np.int32), 0)
