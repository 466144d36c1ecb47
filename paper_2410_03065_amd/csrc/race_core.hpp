// Meet-point planner and the claim protocol of the two-ended race (host only).
//
// The paper's race (App. A; Alg. 1) lets both sides run until their pointers
// cross.  Here each free worker first re-plans where the sweeps should meet
// (Sec. 4 Part 3: the merge point must track resource availability and keep
// latency minimal) and claims its end of the unclaimed range only if that end
// lies on its side of the plan.  Claims are exclusive, so the middle chunk is
// never produced twice (Alg. 1 as printed allows that).
//
// Everything here is integer arithmetic on logged inputs, so every decision can
// be replayed exactly by an independent implementation.
#pragma once
#include <algorithm>
#include <cstddef>
#include <cstdint>
#include <vector>

#include "../../include/cake.h"

namespace cake {

constexpr uint64_t kCostCap = uint64_t(1) << 62;

inline uint64_t sat_add(uint64_t a, uint64_t b) {
    uint64_t s = a + b;
    return (s < a || s > kCostCap) ? kCostCap : s;
}

// TTFT(m) = max(oc + sum_{i<m} c_i, ol + sum_{j>=m} l_j); smallest minimiser.
// One backward pass for the load suffix sums, one forward pass for the scan.
inline int plan_meet_point(const uint64_t* c, const uint64_t* l, int n, uint64_t oc, uint64_t ol,
                           int* m_out, uint64_t* ttft_out, std::vector<uint64_t>& scratch) {
    if (n < 0 || (n > 0 && (!c || !l))) return CAKE_E_INVAL;
    scratch.resize(size_t(n) + 1);
    scratch[n] = ol;
    for (int j = n - 1; j >= 0; --j) {
        scratch[j] = scratch[j + 1] + l[j];
        if (scratch[j] < scratch[j + 1] || scratch[j] > (uint64_t(1) << 63)) return CAKE_E_INVAL;
    }
    uint64_t front = oc;
    int best_m = 0;
    uint64_t best = front > scratch[0] ? front : scratch[0];
    for (int m = 1; m <= n; ++m) {
        uint64_t nf = front + c[m - 1];
        if (nf < front || nf > (uint64_t(1) << 63)) return CAKE_E_INVAL;
        front = nf;
        uint64_t t = front > scratch[m] ? front : scratch[m];
        if (t < best) { best = t; best_m = m; }
        if (front >= best) break;  // the compute side alone already reaches the best: no later m wins
    }
    *m_out = best_m;
    *ttft_out = best;
    return CAKE_OK;
}

inline uint64_t muldiv(uint64_t a, uint64_t b, uint64_t d) {
    unsigned __int128 p = (unsigned __int128)a * b;
    unsigned __int128 q = d ? p / d : (unsigned __int128)kCostCap;
    return q > kCostCap ? kCostCap : uint64_t(q);
}

inline uint64_t range_flops(const cake_model_desc& m, int64_t t0, int64_t cnt) {
    unsigned __int128 hq = (unsigned __int128)m.n_q_heads * m.head_dim, hkv = (unsigned __int128)m.n_kv_heads * m.head_dim;
    unsigned __int128 d = m.d_model, ff = m.ffn_dim, L = m.n_layers;
    unsigned __int128 p_lin = L * (d * hq + 2 * d * hkv + hq * d + 3 * d * ff);
    unsigned __int128 n = cnt;
    unsigned __int128 pairs = (unsigned __int128)t0 * n + n * (n + 1) / 2;
    unsigned __int128 r = 2 * p_lin * n + L * 4 * hq * pairs;
    return r > kCostCap ? kCostCap : uint64_t(r);
}

inline uint64_t page_image_bytes(const cake_model_desc& m, int page_tokens) {
    uint64_t e = m.dtype == CAKE_F32 ? 4 : 2;
    return uint64_t(m.n_layers) * 2 * m.n_kv_heads * page_tokens * m.head_dim * e;
}

// Bytes of one page image in a store of the given format (cake_store_format).
inline uint64_t store_image_bytes(const cake_model_desc& m, int page_tokens, int format) {
    if (format == CAKE_STORE_INT8) return uint64_t(m.n_layers) * 2 * m.n_kv_heads * page_tokens * (uint64_t(m.head_dim) + 4);
    if (format == CAKE_STORE_INT4) return uint64_t(m.n_layers) * 2 * m.n_kv_heads * page_tokens * (uint64_t(m.head_dim) / 2 + 4);
    return page_image_bytes(m, page_tokens);
}

// Running integer estimates (rules stated at cake_decision_log in cake.h).
struct Estimator {
    uint64_t prior_c_ns = 1000000000ull, prior_c_flops = 500000000000000ull;
    uint64_t prior_l_ns = 1000000000ull, prior_l_bytes = 4000000000ull;
    uint64_t win_ns[4] = {0, 0, 0, 0}, win_flops[4] = {0, 0, 0, 0};
    int win_n = 0, win_pos = 0;
    bool have_load = false;
    uint64_t last_l_ns = 0, last_l_bytes = 0;

    void compute_state(uint64_t* ns, uint64_t* flops) const {
        if (win_n == 0) { *ns = prior_c_ns; *flops = prior_c_flops; return; }
        uint64_t a = 0, b = 0;
        for (int i = 0; i < win_n; ++i) { a += win_ns[i]; b += win_flops[i]; }
        *ns = a; *flops = b;
    }
    void load_state(uint64_t* ns, uint64_t* bytes) const {
        if (have_load) { *ns = last_l_ns; *bytes = last_l_bytes; }
        else { *ns = prior_l_ns; *bytes = prior_l_bytes; }
    }
    uint64_t est_compute(uint64_t flops) const {
        uint64_t D, F; compute_state(&D, &F); return muldiv(flops, D, F);
    }
    uint64_t est_load(uint64_t bytes) const {
        uint64_t D, B; load_state(&D, &B); return muldiv(bytes, D, B);
    }
    void add_compute(uint64_t ns, uint64_t flops) {
        win_ns[win_pos] = ns; win_flops[win_pos] = flops;
        win_pos = (win_pos + 1) & 3;
        if (win_n < 4) ++win_n;
    }
    void add_load(uint64_t ns, uint64_t bytes) { have_load = true; last_l_ns = ns; last_l_bytes = bytes; }
};

enum { W_COMPUTE = 0, W_LOAD = 1 };

// The claim protocol.  Not thread safe by itself: the threaded executor calls it
// under its mutex, the virtual-time driver below calls it from one thread.
struct RaceCore {
    int n = 0, f = 0, b = -1;
    int mode = CAKE_BIDIR, forced_m = 0;
    const uint64_t* flops = nullptr;  // per chunk
    const uint64_t* bytes = nullptr;  // per chunk
    // token-granular compute claims (adaptive mode): tokens of chunk f already claimed, and what is
    // needed to price a partial chunk
    int f_off = 0;
    const int32_t* tok_begin = nullptr;
    const int32_t* tok_count = nullptr;
    const cake_model_desc* model = nullptr;
    Estimator est;
    struct Worker {
        bool busy = false, retired = false;
        uint64_t started = 0, pred_end = 0;
        int inflight = -1;
    } w[2];
    // progress of the load in flight, if the executor can observe it (bytes the tier has delivered
    // so far and the time that took); 0 bytes = unknown
    uint64_t load_prog_ns = 0, load_prog_bytes = 0;
    // Adaptive mode: the compute side is free but gets no tokens of the step budget (higher priorities
    // take all of it) since `starved_since`.  Its offset in the plan is then the time it has gone without
    // tokens so far -- a starvation is expected to last about as long again as it already has -- so that
    // the loader takes over chunks the compute side would only reach much later.
    bool starved = false;
    uint64_t starved_since = 0;
    cake_decision_log* log = nullptr;
    int log_cap = 0, log_n = 0;
    bool log_overflow = false;
    std::vector<uint64_t> ce, le, scratch;

    void init(int n_chunks, const uint64_t* fl, const uint64_t* by, int md, int fm) {
        n = n_chunks; f = 0; b = n_chunks - 1; flops = fl; bytes = by; mode = md; forced_m = fm; f_off = 0;
        w[0] = Worker(); w[1] = Worker(); log_n = 0; log_overflow = false; starved = false; starved_since = 0;
        if (mode == CAKE_COMPUTE_ONLY) w[W_LOAD].retired = true;
        if (mode == CAKE_LOAD_ONLY) w[W_COMPUTE].retired = true;
    }
    bool range_empty() const { return f > b; }
    bool all_done() const { return f > b && !w[0].busy && !w[1].busy; }

    struct Plan { int m_star; uint64_t oc, ol, D, F, LN, LB, partial; };

    // Where should the sweeps meet, seen by worker `who` at `now`?  When compute has already taken
    // part of chunk f (f_off > 0) that chunk is compute's: the plan covers [f+1, b] and the rest of
    // chunk f is added to the compute side's offset.
    Plan plan(int who, uint64_t now) {
        Plan p{};
        est.compute_state(&p.D, &p.F);
        est.load_state(&p.LN, &p.LB);
        p.oc = (w[W_COMPUTE].busy && w[W_COMPUTE].pred_end > now) ? w[W_COMPUTE].pred_end - now : 0;
        if (!w[W_COMPUTE].busy && starved && now > starved_since) p.oc = now - starved_since;
        p.ol = (w[W_LOAD].busy && w[W_LOAD].pred_end > now) ? w[W_LOAD].pred_end - now : 0;
        if (w[W_LOAD].busy && load_prog_bytes > 0 && w[W_LOAD].inflight >= 0) {
            // the chunk in flight tells the tier's current rate sooner than its completion would
            p.LN = load_prog_ns; p.LB = load_prog_bytes;
            const uint64_t total = bytes[w[W_LOAD].inflight];
            p.ol = total > load_prog_bytes ? muldiv(total - load_prog_bytes, load_prog_ns, load_prog_bytes) : 0;
        }
        const int lo = f_off > 0 ? f + 1 : f;   // first chunk the loader could still take
        if (f_off > 0) p.partial = est.est_compute(range_flops(*model, tok_begin[f] + f_off, tok_count[f] - f_off));
        if (mode == CAKE_COMPUTE_ONLY) p.m_star = n;
        else if (mode == CAKE_LOAD_ONLY) p.m_star = lo;
        else if (mode == CAKE_FORCED_SPLIT) p.m_star = forced_m > lo ? forced_m : lo;
        else if (mode == CAKE_GREEDY || w[1 - who].retired) p.m_star = (who == W_COMPUTE) ? b + 1 : lo;
        else {
            int cnt = b - lo + 1;
            ce.resize(cnt > 0 ? cnt : 0); le.resize(cnt > 0 ? cnt : 0);
            for (int k = 0; k < cnt; ++k) {
                ce[k] = est.est_compute(flops[lo + k]);
                le[k] = muldiv(bytes[lo + k], p.LN, p.LB);
            }
            int m_rel = 0; uint64_t t = 0;
            if (cnt <= 0) m_rel = 0;
            else if (plan_meet_point(ce.data(), le.data(), cnt, sat_add(p.oc, p.partial), p.ol, &m_rel, &t, scratch) != CAKE_OK) {
                // sums beyond 2^63 ns: fall back to the greedy rule rather than fail the run
                m_rel = (who == W_COMPUTE) ? cnt : 0;
            }
            p.m_star = lo + m_rel;
        }
        return p;
    }

    void record(int who, uint64_t now, const Plan& p, int f0, int b0, int off0, int claim, int claim_tokens) {
        if (!log) return;
        if (log_n < log_cap) {
            cake_decision_log& d = log[log_n++];
            d.who = who; d.f = f0; d.b = b0; d.m_star = p.m_star; d.claimed = claim; d.f_off = off0;
            d.claimed_tokens = claim_tokens; d.pad_ = 0;
            d.now_ns = now; d.o_c = p.oc; d.o_l = p.ol;
            d.est_compute_ns = p.D; d.est_compute_flops = p.F; d.est_load_ns = p.LN; d.est_load_bytes = p.LB;
            d.partial_ns = p.partial;
        } else log_overflow = true;
    }

    // A free worker looks at the range.  Returns the claimed chunk or -1 (wait).  Compute claims
    // the whole (rest of) chunk f; see claim_front for smaller compute steps.
    int decide(int who, uint64_t now) {
        if (f > b || w[who].retired || w[who].busy) return -1;
        const Plan p = plan(who, now);
        int f0 = f, b0 = b, off0 = f_off, claim = -1, claim_tokens = 0;
        uint64_t cost = 0;
        if (who == W_COMPUTE && f < p.m_star) {
            cost = f_off > 0 ? p.partial : est.est_compute(flops[f]);
            if (tok_count) claim_tokens = tok_count[f] - f_off;
            claim = f++;
            f_off = 0;
        } else if (who == W_LOAD && b >= p.m_star && !(b == f && f_off > 0)) {
            cost = est.est_load(bytes[b]);
            if (tok_count) claim_tokens = tok_count[b];
            claim = b--;
        }
        record(who, now, p, f0, b0, off0, claim, claim_tokens);
        if (claim >= 0) {
            Worker& me = w[who];
            me.busy = true; me.inflight = claim; me.started = now;
            me.pred_end = sat_add(now, cost);
        }
        return claim;
    }

    // Compute side, token granular: claims up to max_tokens consecutive tokens from the front of the
    // range, over as many chunks as that takes (the chunks here may be fetch units much smaller than
    // a compute step) but never into a chunk at or past the planned meet point.  Returns the number
    // of tokens claimed (0 = wait) and their first token.  The compute worker is marked busy until
    // complete_front().
    int claim_front(uint64_t now, int max_tokens, int* first_token) {
        if (f > b || w[W_COMPUTE].retired || w[W_COMPUTE].busy || max_tokens <= 0) return 0;
        const Plan p = plan(W_COMPUTE, now);
        const int f0 = f, b0 = b, off0 = f_off;
        int got = 0;
        if (f < p.m_star) {
            *first_token = tok_begin[f] + f_off;
            while (f <= b && f < p.m_star && got < max_tokens) {
                const int take = std::min(tok_count[f] - f_off, max_tokens - got);
                got += take;
                f_off += take;
                if (f_off < tok_count[f]) break;
                ++f; f_off = 0;
            }
            Worker& me = w[W_COMPUTE];
            me.busy = true; me.inflight = f0; me.started = now;
            me.pred_end = sat_add(now, est.est_compute(range_flops(*model, *first_token, got)));
        }
        record(W_COMPUTE, now, p, f0, b0, off0, got > 0 ? f0 : -1, got);
        return got;
    }

    // The compute step holding a claim_front() part has ended; the sample is the wall time since
    // the request last got tokens against its FLOPs in this step (the rate it actually gets when
    // the GPU is shared).
    void complete_front(uint64_t step_ns, uint64_t prefix_flops) {
        w[W_COMPUTE].busy = false;
        w[W_COMPUTE].inflight = -1;
        est.add_compute(step_ns, prefix_flops);
    }

    // The worker's chunk in flight has ended at `now`.  A failed load gives the chunk
    // back to the range and retires the loader; a failed compute retires the compute side.
    void complete(int who, uint64_t now, bool failed) {
        Worker& me = w[who];
        if (who == W_LOAD) load_prog_ns = load_prog_bytes = 0;
        int i = me.inflight;
        me.busy = false; me.inflight = -1;
        if (i < 0) return;
        if (failed) {
            if (who == W_LOAD) b = i; else f = i;
            me.retired = true;
            return;
        }
        uint64_t dur = now - me.started;
        if (who == W_COMPUTE) est.add_compute(dur, flops[i]); else est.add_load(dur, bytes[i]);
    }
};

// Virtual-time driver: both workers free at t = 0; at every event time completions are
// applied first (compute before load), then free workers look at the range in the order
// compute, load, repeated until nobody claims.
inline int simulate_race(RaceCore& core, const uint64_t* actual_c, const uint64_t* actual_l,
                         int fail_load_chunk, int32_t* sources, uint64_t* ttft) {
    uint64_t t = 0, until[2] = {0, 0};
    for (int i = 0; i < core.n; ++i) sources[i] = CAKE_SRC_NONE;
    for (;;) {
        bool changed = true;
        while (changed) {
            changed = false;
            for (int who = 0; who < 2; ++who) {
                int c = core.decide(who, t);
                if (c >= 0) {
                    until[who] = t + (who == W_COMPUTE ? actual_c[c] : actual_l[c]);
                    changed = true;
                }
            }
        }
        if (!core.w[0].busy && !core.w[1].busy) break;
        uint64_t nt = ~uint64_t(0);
        for (int who = 0; who < 2; ++who)
            if (core.w[who].busy && until[who] < nt) nt = until[who];
        t = nt;
        for (int who = 0; who < 2; ++who) {
            if (core.w[who].busy && until[who] == t) {
                int i = core.w[who].inflight;
                bool fail = (who == W_LOAD && i == fail_load_chunk);
                core.complete(who, t, fail);
                if (!fail) sources[i] = who;
            }
        }
    }
    *ttft = t;
    return core.range_empty() ? CAKE_OK : CAKE_E_STATE;
}

}  // namespace cake
