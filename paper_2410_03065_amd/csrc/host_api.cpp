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

uint64_t cake_store_image_bytes(const cake_model_desc* model, int32_t page_tokens, int32_t format) {
    if (!model || page_tokens <= 0 || (format != CAKE_STORE_RAW && format != CAKE_STORE_INT8)) return 0;
    return cake::store_image_bytes(*model, page_tokens, format);
}

uint64_t cake_page_image_bytes(const cake_model_desc* model, int32_t page_tokens) {
    if (!model || page_tokens <= 0) return 0;
    return cake::page_image_bytes(*model, page_tokens);
}

}  // extern "C"
