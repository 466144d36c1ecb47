// Host-only entry points: the meet-point planner, the virtual-time race and size helpers.
#include <vector>

#include "race_core.hpp"

extern "C" {

int32_t cake_plan_meet_point(const uint64_t* compute_ns, const uint64_t* load_ns, int32_t n,
                             uint64_t compute_offset_ns, uint64_t load_offset_ns,
                             int32_t* m_out, uint64_t* ttft_ns_out) {
    if (!m_out || !ttft_ns_out) return CAKE_E_INVAL;
    if (compute_offset_ns > (uint64_t(1) << 62) || load_offset_ns > (uint64_t(1) << 62)) return CAKE_E_INVAL;
    std::vector<uint64_t> scratch;
    int m = 0;
    uint64_t t = 0;
    int rc = cake::plan_meet_point(compute_ns, load_ns, n, compute_offset_ns, load_offset_ns, &m, &t, scratch);
    if (rc != CAKE_OK) return rc;
    *m_out = m;
    *ttft_ns_out = t;
    return CAKE_OK;
}

int32_t cake_simulate_race(int32_t n_chunks, const uint64_t* chunk_flops, const uint64_t* chunk_bytes,
                           const uint64_t* actual_compute_ns, const uint64_t* actual_load_ns,
                           uint64_t prior_compute_ns, uint64_t prior_compute_flops,
                           uint64_t prior_load_ns, uint64_t prior_load_bytes, int32_t mode,
                           int32_t forced_m, int32_t fail_load_chunk, int32_t* sources_out,
                           uint64_t* ttft_ns_out, cake_decision_log* decisions, int32_t decisions_cap,
                           int32_t* n_decisions_out) {
    if (n_chunks < 0 || !ttft_ns_out) return CAKE_E_INVAL;
    if (n_chunks > 0 && (!chunk_flops || !chunk_bytes || !actual_compute_ns || !actual_load_ns || !sources_out))
        return CAKE_E_INVAL;
    if (mode < CAKE_BIDIR || mode > CAKE_GREEDY) return CAKE_E_INVAL;
    if (mode == CAKE_FORCED_SPLIT && (forced_m < 0 || forced_m > n_chunks)) return CAKE_E_INVAL;
    if (!prior_compute_flops || !prior_load_bytes) return CAKE_E_INVAL;
    cake::RaceCore core;
    core.est.prior_c_ns = prior_compute_ns;
    core.est.prior_c_flops = prior_compute_flops;
    core.est.prior_l_ns = prior_load_ns;
    core.est.prior_l_bytes = prior_load_bytes;
    core.init(n_chunks, chunk_flops, chunk_bytes, mode, forced_m);
    core.log = decisions;
    core.log_cap = decisions ? decisions_cap : 0;
    int rc = cake::simulate_race(core, actual_compute_ns, actual_load_ns, fail_load_chunk, sources_out, ttft_ns_out);
    if (n_decisions_out) *n_decisions_out = core.log_n;
    if (rc == CAKE_OK && core.log_overflow) rc = CAKE_E_CAPACITY;
    return rc;
}

uint64_t cake_range_flops(const cake_model_desc* model, int32_t tok_begin, int32_t tok_count) {
    if (!model || tok_begin < 0 || tok_count < 0) return 0;
    return cake::range_flops(*model, tok_begin, tok_count);
}

// FNV-1a, 64 bit: h = (h xor byte) * prime for every byte
static inline uint64_t fnv1a64_bytes(uint64_t h, const unsigned char* p, size_t n) {
    for (size_t i = 0; i < n; ++i) h = (h ^ p[i]) * 0x100000001B3ull;
    return h;
}

int32_t cake_prefix_keys(const int32_t* token_ids, int32_t n_tokens, int32_t chunk_tokens, uint64_t* keys_out,
                         int32_t keys_cap) {
    if (!token_ids || n_tokens < 0 || chunk_tokens <= 0 || (!keys_out && keys_cap > 0) || keys_cap < 0) return CAKE_E_INVAL;
    const int32_t n = n_tokens / chunk_tokens;
    uint64_t prev = 0xCBF29CE484222325ull;
    for (int32_t i = 0; i < n && i < keys_cap; ++i) {
        unsigned char kb[8];
        for (int b = 0; b < 8; ++b) kb[b] = (unsigned char)(prev >> (8 * b));
        uint64_t h = fnv1a64_bytes(0xCBF29CE484222325ull, kb, 8);
        for (int32_t t = 0; t < chunk_tokens; ++t) {
            const uint32_t id = (uint32_t)token_ids[size_t(i) * chunk_tokens + t];
            unsigned char tb[4] = {(unsigned char)id, (unsigned char)(id >> 8), (unsigned char)(id >> 16), (unsigned char)(id >> 24)};
            h = fnv1a64_bytes(h, tb, 4);
        }
        keys_out[i] = prev = h;
    }
    return n;
}

int32_t cake_prefix_lookup(const uint64_t* stored_sorted, int32_t n_stored, const uint64_t* keys, int32_t n_keys) {
    if (n_stored < 0 || n_keys < 0 || (n_stored > 0 && !stored_sorted) || (n_keys > 0 && !keys)) return CAKE_E_INVAL;
    for (int32_t i = 1; i < n_stored; ++i)
        if (stored_sorted[i - 1] > stored_sorted[i]) return CAKE_E_INVAL;
    int32_t hit = 0;
    for (; hit < n_keys; ++hit) {
        int32_t lo = 0, hi = n_stored;   // binary search for keys[hit]
        while (lo < hi) {
            const int32_t mid = lo + (hi - lo) / 2;
            if (stored_sorted[mid] < keys[hit]) lo = mid + 1; else hi = mid;
        }
        if (lo == n_stored || stored_sorted[lo] != keys[hit]) break;
    }
    return hit;
}

uint64_t cake_store_image_bytes(const cake_model_desc* model, int32_t page_tokens, int32_t format) {
    if (!model || page_tokens <= 0 || (format != CAKE_STORE_RAW && format != CAKE_STORE_INT8 && format != CAKE_STORE_INT4)) return 0;
    return cake::store_image_bytes(*model, page_tokens, format);
}

uint64_t cake_page_image_bytes(const cake_model_desc* model, int32_t page_tokens) {
    if (!model || page_tokens <= 0) return 0;
    return cake::page_image_bytes(*model, page_tokens);
}

}  // extern "C"
