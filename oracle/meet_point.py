"""Oracle: where the forward (compute) and backward (load) sweeps should meet.
Test infrastructure only; exact Python integers throughout.

The paper gives the race (App. A; Alg. 1) and states its purpose: the merging
point shifts with resource availability "always ensuring minimal latency"
(Sec. 4 Part 3) and "minimize[s] TTFT" (Sec. 5.6).  The plain definition of
that purpose, used as the oracle:

    chunks 0..N-1, compute costs c_i, load costs l_j, both sides start at once
    (after offsets o_c, o_l if a side is still busy with earlier work);
    a split m in 0..N means chunks [0, m) are computed front-to-back and
    chunks [m, N) are loaded back-to-front, so

        TTFT(m) = max(o_c + sum_{i<m} c_i ,  o_l + sum_{j>=m} l_j)

    m* = the smallest m minimising TTFT(m).  m = 0 is load-only, m = N is
    compute-only (the two baselines of Sec. 5.1).

``brute_force_meet_point`` evaluates all N+1 splits.  ``literal_race`` is
Alg. 1 as printed (with half-open ranges, see below), ``simulate_claims`` is a
discrete-event replay of the claim protocol the library uses, written here
independently from its description.

Readings taken where Alg. 1 is ambiguous:
* ranges are half-open: the loader owns [io, T), the compute side [0, cp), the
  race ends when cp >= io (as printed, io starts at T-1 and one token can be
  left to nobody);
* ties between splits go to the smallest m.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Sequence, Tuple

COMPUTE, LOAD = 0, 1


def ttft_of_split(c: Sequence[int], l: Sequence[int], m: int, o_c: int = 0, o_l: int = 0) -> int:
    n = len(c)
    assert len(l) == n and 0 <= m <= n
    a = o_c + sum(int(x) for x in c[:m])
    b = o_l + sum(int(x) for x in l[m:])
    return max(a, b)


def brute_force_meet_point(c: Sequence[int], l: Sequence[int],
                           o_c: int = 0, o_l: int = 0) -> Tuple[int, int]:
    """(m*, TTFT(m*)) by trying every split; smallest m on ties."""
    best_m, best_t = 0, ttft_of_split(c, l, 0, o_c, o_l)
    for m in range(1, len(c) + 1):
        t = ttft_of_split(c, l, m, o_c, o_l)
        if t < best_t:
            best_m, best_t = m, t
    return best_m, best_t


# --------------------------------------------------------------------------- #
# Alg. 1 as printed: two loops that look only at the two pointers
# --------------------------------------------------------------------------- #
def literal_race(c: Sequence[int], l: Sequence[int]) -> Tuple[int, int, int]:
    """Alg. 1 with chunk-granular pointers.  Returns (ttft, n_computed, n_loaded).

    ComputeKV: while cp < io: stop if chunk cp is already resident (a *completed*
    fetch); else compute it, then cp += 1.  FetchKV: while cp < io: fetch the chunk
    ending at io, then io -= 1.  Pointers move only when a chunk completes, so the
    middle chunk can be produced by both sides at once; the procedure returns when
    both loops have ended.
    """
    n = len(c)
    cp, io = 0, n                      # compute owns [0,cp), loader owns [io,n)
    free_at = [0, 0]                   # when each loop next looks at the pointers
    done = [False, False]
    inflight: List[Optional[int]] = [None, None]
    count = [0, 0]
    resident = [False] * n
    while not (done[COMPUTE] and done[LOAD]):
        t = min(free_at[w] for w in (COMPUTE, LOAD) if not done[w])
        due = [w for w in (COMPUTE, LOAD) if not done[w] and free_at[w] == t]
        for w in due:                  # chunks completing at t update the pointers first
            i = inflight[w]
            if i is None:
                continue
            inflight[w] = None
            count[w] += 1
            if w == COMPUTE:
                cp = i + 1
            else:
                resident[i] = True
                io = i
        for w in due:                  # then each free loop tests its while-condition
            if w == COMPUTE and cp < io and not resident[cp]:
                inflight[w] = cp
                free_at[w] = t + int(c[cp])
            elif w == LOAD and cp < io:
                inflight[w] = io - 1
                free_at[w] = t + int(l[io - 1])
            else:
                done[w] = True
    return max(free_at), count[COMPUTE], count[LOAD]


# --------------------------------------------------------------------------- #
# cost estimates used by the claim protocol
# --------------------------------------------------------------------------- #
def range_flops(L: int, d: int, n_q: int, n_kv: int, hd: int, ff: int,
                t0: int, t1: int) -> int:
    """Work of prefilling tokens [t0, t1): projections + causal attention."""
    hq, hkv = n_q * hd, n_kv * hd
    p_lin = L * (d * hq + 2 * d * hkv + hq * d + 3 * d * ff)
    n = t1 - t0
    return 2 * p_lin * n + L * 4 * hq * (t0 * n + n * (n + 1) // 2)


@dataclass
class Estimator:
    """Integer running estimates.  Compute: the last <= 4 measured chunks give a
    throughput D/F (ns per unit of work); a chunk's estimate is floor(F_i * D / F).
    Load: the last measured chunk gives ns per byte."""
    prior_compute_ns: int
    prior_compute_flops: int
    prior_load_ns: int
    prior_load_bytes: int
    window: List[Tuple[int, int]] = field(default_factory=list)
    last_load: Optional[Tuple[int, int]] = None

    def compute_state(self) -> Tuple[int, int]:
        if not self.window:
            return self.prior_compute_ns, self.prior_compute_flops
        return sum(w[0] for w in self.window), sum(w[1] for w in self.window)

    def load_state(self) -> Tuple[int, int]:
        return self.last_load if self.last_load else (self.prior_load_ns, self.prior_load_bytes)

    def est_compute(self, flops: int) -> int:
        D, F = self.compute_state()
        return flops * D // F

    def est_load(self, nbytes: int) -> int:
        ns, b = self.load_state()
        return nbytes * ns // b

    def add_compute(self, ns: int, flops: int) -> None:
        self.window.append((ns, flops))
        if len(self.window) > 4:
            self.window.pop(0)

    def add_load(self, ns: int, nbytes: int) -> None:
        self.last_load = (ns, nbytes)


@dataclass
class Decision:
    who: int
    now: int
    f: int
    b: int
    o_c: int
    o_l: int
    D: int
    F: int
    load_ns: int
    load_bytes: int
    m_star: int
    claimed: int      # chunk index or -1


MODE_BIDIR, MODE_COMPUTE_ONLY, MODE_LOAD_ONLY, MODE_FORCED, MODE_GREEDY = 0, 1, 2, 3, 4


def simulate_claims(n_chunks: int, chunk_flops: Sequence[int], chunk_bytes: Sequence[int],
                    actual_compute_ns: Sequence[int], actual_load_ns: Sequence[int],
                    est: Estimator, mode: int = MODE_BIDIR, forced_m: int = 0,
                    fail_load_chunk: int = -1):
    """Discrete-event replay of the claim protocol in virtual time.

    Unclaimed chunks are the range [f, b].  A free worker looks at the range under
    a lock: it estimates every remaining chunk's compute and load cost, takes as
    offsets the predicted remaining time of the other side's chunk in flight, finds
    the best split m* of the range by ``brute_force_meet_point`` and claims its end
    of the range only if that end lies on its side of m* (compute: f < m*; load:
    b >= m*).  Otherwise it waits for the other side's next event.  Forced modes
    replace m* by a constant; the greedy mode always claims (Alg. 1 with exclusive
    claims).  A failing load returns its chunk to the range and retires the loader.

    Returns (ttft, sources, decisions) with sources[i] in {COMPUTE, LOAD}.
    """
    f, b = 0, n_chunks - 1
    busy = [False, False]
    until = [0, 0]
    pred_end = [0, 0]
    started = [0, 0]
    inflight = [-1, -1]
    retired = [False, False]
    sources = [-1] * n_chunks
    log: List[Decision] = []
    t = 0

    def decide(w: int) -> int:
        nonlocal f, b
        D, F = est.compute_state()
        lns, lby = est.load_state()
        o_c = max(0, pred_end[COMPUTE] - t) if busy[COMPUTE] else 0
        o_l = max(0, pred_end[LOAD] - t) if busy[LOAD] else 0
        if mode == MODE_COMPUTE_ONLY:
            m_star = n_chunks
        elif mode == MODE_LOAD_ONLY:
            m_star = 0
        elif mode == MODE_FORCED:
            m_star = forced_m
        elif mode == MODE_GREEDY:
            m_star = b + 1 if w == COMPUTE else f
        elif retired[1 - w]:
            m_star = b + 1 if w == COMPUTE else f
        else:
            ce = [est.est_compute(chunk_flops[i]) for i in range(f, b + 1)]
            le = [est.est_load(chunk_bytes[i]) for i in range(f, b + 1)]
            m_rel, _ = brute_force_meet_point(ce, le, o_c, o_l)
            m_star = f + m_rel
        f0, b0, claim = f, b, -1
        if w == COMPUTE and f < m_star:
            claim = f
            f += 1
        elif w == LOAD and b >= m_star:
            claim = b
            b -= 1
        log.append(Decision(w, t, f0, b0, o_c, o_l, D, F, lns, lby, m_star, claim))
        return claim

    while True:
        changed = True
        while changed:
            changed = False
            for w in (COMPUTE, LOAD):
                if busy[w] or retired[w] or f > b:
                    continue
                if mode == MODE_COMPUTE_ONLY and w == LOAD:
                    continue
                if mode == MODE_LOAD_ONLY and w == COMPUTE:
                    continue
                i = decide(w)
                if i >= 0:
                    busy[w], inflight[w], started[w] = True, i, t
                    if w == COMPUTE:
                        until[w] = t + int(actual_compute_ns[i])
                        pred_end[w] = t + est.est_compute(chunk_flops[i])
                    else:
                        until[w] = t + int(actual_load_ns[i])
                        pred_end[w] = t + est.est_load(chunk_bytes[i])
                    changed = True
        if not (busy[COMPUTE] or busy[LOAD]):
            break
        t = min(until[w] for w in (COMPUTE, LOAD) if busy[w])
        for w in (COMPUTE, LOAD):
            if busy[w] and until[w] == t:
                i = inflight[w]
                busy[w], inflight[w] = False, -1
                if w == LOAD and i == fail_load_chunk:
                    b = i                      # chunk goes back; loader is retired
                    retired[LOAD] = True
                    continue
                sources[i] = w
                if w == COMPUTE:
                    est.add_compute(t - started[w], chunk_flops[i])
                else:
                    est.add_load(t - started[w], chunk_bytes[i])
    if f <= b:
        raise RuntimeError("claim protocol stalled with chunks left")
    return t, sources, log


# --------------------------------------------------------------------------- #
# adaptive scheduling mode (Sec. 4 Part 3; evaluated in Sec. 5.7)
# --------------------------------------------------------------------------- #
def fill_token_budget(budget: int, n_decoding: int, nonprefix_remaining: Sequence[int],
                      prefix_offer: int):
    """One engine step of the adaptive mode.  The budget is dealt out in the paper's order:
    1. decoding requests (one token each), 2. chunked prefill of requests without a stored
    prefix, oldest first, 3. chunked prefill of the prefix-cached request with what is left.
    ``nonprefix_remaining`` lists the unprefilled tokens of the arrived non-prefix requests in
    arrival order; ``prefix_offer`` is how many tokens the prefix request could use.
    Returns (decode_tokens, [tokens per non-prefix request], prefix_tokens)."""
    left = budget
    dec = min(left, n_decoding)
    left -= dec
    grants = []
    for rem in nonprefix_remaining:
        g = min(left, rem)
        grants.append(g)
        left -= g
    return dec, grants, min(left, prefix_offer)


def front_claim(f: int, f_off: int, b: int, m_star: int, max_tokens: int, tok_count: Sequence[int]):
    """Token-granular claim of the compute side (adaptive mode, Sec. 4 Part 3, with fetch units
    smaller than a compute step, Sec. 5.1 "Implementation"): take consecutive tokens from token
    ``f_off`` of chunk ``f`` on, whole chunks and at last a part of one, until ``max_tokens`` are
    taken, the unclaimed range [f, b] ends, or the next chunk is at or past the meet point.
    Returns (tokens, f after, f_off after)."""
    got = 0
    while f <= b and f < m_star and got < max_tokens:
        take = min(tok_count[f] - f_off, max_tokens - got)
        got += take
        f_off += take
        if f_off < tok_count[f]:
            break
        f, f_off = f + 1, 0
    return got, f, f_off


def expected_meet_point(f: int, b: int, f_off: int, o_c: int, o_l: int, partial_ns: int,
                        est: Estimator, chunk_flops: Sequence[int], chunk_bytes: Sequence[int]) -> int:
    """The split a planned look at the range [f, b] must log.  When the compute side has
    already taken f_off tokens of chunk f, that chunk stays with it: the plan covers
    [f+1, b] and the estimate of the rest of chunk f counts as compute-side offset."""
    lo = f + 1 if f_off > 0 else f
    ce = [est.est_compute(chunk_flops[i]) for i in range(lo, b + 1)]
    le = [est.est_load(chunk_bytes[i]) for i in range(lo, b + 1)]
    extra = partial_ns if f_off > 0 else 0
    return lo + brute_force_meet_point(ce, le, o_c + extra, o_l)[0]
