// C ABI: context, chunk prefill, throttled chunk load, bidirectional prefill.
// See include/cake.h for the contract of every entry point.
#include <hip/hip_runtime.h>
#include <errno.h>
#include <sys/prctl.h>
#include <time.h>
#include <unistd.h>

#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <memory>
#include <mutex>
#include <string>
#include <thread>
#include <vector>

#include "executor.hpp"
#include "kernels.hpp"

using namespace cake;

struct cake_ctx {
    cake_model_desc m{};
    std::vector<cake_layer_weights> layers;
    const void* embed = nullptr;
    int device = 0;
    int max_tokens = 0, max_chunk = 0;
    hipStream_t cs = nullptr, ls = nullptr;
    // activation workspace (device)
    float* x = nullptr;       // [max_chunk][d]            residual stream, float32
    void* h = nullptr;        // [max_chunk][d]            normed activations, model dtype
    float* qkv = nullptr;     // [max_chunk][(n_q+2n_kv)hd] float32
    void* q = nullptr;        // [n_q][rows][hd]           rotated queries, model dtype
    void* ao = nullptr;       // [max_chunk][n_q*hd]       attention output, model dtype
    void* act = nullptr;      // [max_chunk][ffn]          SwiGLU output, model dtype
    float* rope_cs = nullptr; // [max_chunk][hd/2][2]
    int32_t* d_ids = nullptr; // [max_tokens]
    // first-token step (one row, float32 throughout); null unless the weights carry final_norm and lm_head
    const float* final_norm = nullptr;
    const void* lm_head = nullptr;
    float *t_h = nullptr, *t_q = nullptr, *t_qr = nullptr, *t_ao = nullptr, *t_act = nullptr, *t_logits = nullptr,
          *t_part = nullptr;
    int32_t* t_tok = nullptr;
    void* static_scratch = nullptr;   // this device's copy of the file-scope scratch array (set by cake_create)
    GemmSplitWs split{};       // parts and ticket counters of the split-K GEMMs (bf16 models; compute stream only)
    void* q_stage = nullptr;   // device staging for quantised page images: a ring of image slots (cake_create)
    size_t q_stage_bytes = 0;
    // second hop of a file-backed store: two pinned buffers of one DMA piece each
    void* f_stage[2] = {nullptr, nullptr};
    size_t f_stage_bytes = 0;
    int f_next = 0;
    hipEvent_t ev_a = nullptr, ev_b = nullptr;
    hipEvent_t ev_load = nullptr;   // blocking-sync event: the load worker sleeps until the copy stream has drained
    std::atomic<double> gbps{0.0};
    std::atomic<int> async_load_rc{0};   // first failure of a load queued by cake_load_chunk since the last cake_sync_load
    int step_after = -1;
    double step_gbps = 0.0;
    // traces for the next cake_adaptive_serve (copied by cake_set_traces)
    std::vector<int32_t> tr_other, tr_ids;
    std::vector<double> tr_gbps;
    uint64_t tr_interval_ns = 0;
    std::atomic<uint64_t> tr_t0{0};   // 0: no bandwidth trace running
    cake_kv tr_kv{};
    cake_tuning tun{1000000000ull, 500000000000000ull, 4ull << 20, 0, 0, 0, 0};  // gemm_config 0 = automatic
    std::mutex err_mu;
    std::string err;
    std::unique_ptr<std::atomic<int32_t>[]> status;
    int n_status = 0;
    // progress of the paced load in flight (written by the load thread, read by planners)
    std::atomic<uint64_t> load_start_ns{0}, load_bytes_done{0};
    // per-kernel-class timing (compute thread only)
    bool prof_on = false, prof_open = false;
    uint32_t prof_mask = 0xffffffffu;   // kernel classes that are bracketed while profiling is on
    struct ProfRec { int cls; uint64_t flops, bytes; };
    std::vector<hipEvent_t> prof_events;  // pairs: [2i] before, [2i+1] after
    std::vector<ProfRec> prof_recs;
    // the load worker of every race of this context (bound to the context's device when it starts)
    WorkerThread load_thread;
};

// Partial results of the one-token attention for callers that may not allocate device memory
// (cake_op_decode_attention_static): one array per GPU the library runs on, held until the process
// ends.  Sized for 64 query heads of head dimension 128 over the largest number of key ranges the
// kernels use (128): 64 * 128 * 130 floats.  In host code the array's name is only a handle for
// hipGetSymbolAddress; kernels get the address that call returned for the current device.
constexpr size_t STATIC_SCRATCH_BYTES = size_t(64) * 128 * (128 + 2) * sizeof(float);
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];
constexpr int STATIC_SCRATCH_MAX_DEVICES = 64;
static std::mutex g_scratch_mu;
static void* g_scratch_ptr[STATIC_SCRATCH_MAX_DEVICES] = {};

// Address of `scratch` on `device`, which must be the current device; looked up once per device.
static hipError_t static_scratch_for_device(int device, void** out) {
    if (device < 0 || device >= STATIC_SCRATCH_MAX_DEVICES) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> g(g_scratch_mu);
    if (!g_scratch_ptr[device]) {
        void* p = nullptr;
        hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_scratch_ptr[device] = p;
    }
    *out = g_scratch_ptr[device];
    return hipSuccess;
}

static int fail(cake_ctx* ctx, int code, const char* fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    if (ctx) {
        std::lock_guard<std::mutex> g(ctx->err_mu);
        ctx->err = buf;
    }
    return code;
}

#define HIP_TRY(ctx, expr)                                                                      \
    do {                                                                                        \
        hipError_t e_ = (expr);                                                                 \
        if (e_ != hipSuccess) return fail(ctx, CAKE_E_HIP, "%s: %s", #expr, hipGetErrorString(e_)); \
    } while (0)

static size_t esize(const cake_ctx* c) { return c->m.dtype == CAKE_F32 ? 4 : 2; }
static bool store_format_known(int f) { return f == CAKE_STORE_RAW || f == CAKE_STORE_INT8 || f == CAKE_STORE_INT4; }
// bits per stored code of a quantised format, 0 for the raw format
static int store_code_bits(int f) { return f == CAKE_STORE_INT8 ? 8 : f == CAKE_STORE_INT4 ? 4 : 0; }

static int check_store(cake_ctx* c, const cake_kv_store* st, const cake_kv* kv) {
    if (!st) return fail(c, CAKE_E_INVAL, "store: null");
    if (st->source == CAKE_STORE_PINNED ? !st->base : (st->source != CAKE_STORE_FILE || st->fd < 0))
        return fail(c, CAKE_E_INVAL, "store: no memory / file given (source %d)", st->source);
    if (!store_format_known(st->format)) return fail(c, CAKE_E_INVAL, "store: unknown format %d", st->format);
    if (st->n_pages < 0) return fail(c, CAKE_E_INVAL, "store: negative page count");
    if (st->page_tokens != kv->page_tokens) return fail(c, CAKE_E_INVAL, "store/page size mismatch");
    if (st->page_stride_bytes < cake::store_image_bytes(c->m, kv->page_tokens, st->format))
        return fail(c, CAKE_E_INVAL, "store: page stride smaller than a page image");
    return CAKE_OK;
}

static int check_kv(cake_ctx* ctx, const cake_kv* kv, int tok_end) {
    if (!kv || !kv->pool || !kv->block_table_host || !kv->block_table_dev) return fail(ctx, CAKE_E_INVAL, "kv: null pointer");
    if (kv->page_tokens <= 0 || kv->page_tokens % 64) return fail(ctx, CAKE_E_INVAL, "kv: page_tokens must be a positive multiple of 64");
    if (kv->n_physical_pages <= 0 || kv->n_logical_pages <= 0) return fail(ctx, CAKE_E_INVAL, "kv: no pages");
    int need = (tok_end + kv->page_tokens - 1) / kv->page_tokens;
    if (need > kv->n_logical_pages) return fail(ctx, CAKE_E_INVAL, "kv: block table has %d pages, %d needed", kv->n_logical_pages, need);
    for (int p = 0; p < need; ++p) {
        int pp = kv->block_table_host[p];
        if (pp < 0 || pp >= kv->n_physical_pages) return fail(ctx, CAKE_E_INVAL, "kv: block_table[%d] = %d outside the pool", p, pp);
    }
    return CAKE_OK;
}

static KvView make_view(const cake_ctx* c, const cake_kv* kv, int layer) {
    KvView v;
    v.pool = kv->pool;
    v.block_table = kv->block_table_dev;
    v.page_tokens = kv->page_tokens;
    v.n_physical_pages = kv->n_physical_pages;
    v.n_kv = c->m.n_kv_heads;
    v.head_dim = c->m.head_dim;
    v.layer = layer;
    return v;
}

// ------------------------------------------------------------------ kernel dispatch
static hipError_t gemm(cake_ctx* c, int epi, const void* a, const void* w, const void* w2, void* out, int M, int N, int K) {
    if (c->m.dtype == CAKE_BF16 && c->tun.kernel_path == 0 && gemm_mfma_supported(epi, M, N, K))
        return launch_gemm_mfma(epi, a, w, w2, out, M, N, K, c->cs, c->tun.gemm_config - 1, c->split.part ? &c->split : nullptr,
                                c->tun.gemm_ksplit);
    return launch_gemm_generic(c->m.dtype, epi, a, w, w2, out, M, N, K, c->cs);
}

static hipError_t attention(cake_ctx* c, const void* q, void* out, int tok_begin, int rows, const KvView& kv) {
    if (c->m.dtype == CAKE_BF16 && c->tun.kernel_path == 0 && attention_mfma_supported(kv.head_dim, kv.page_tokens))
        return launch_attention_mfma(q, out, c->m.n_q_heads, tok_begin, rows, kv, c->cs, c->tun.attn_variant);
    return launch_attention_generic(c->m.dtype, q, out, c->m.n_q_heads, tok_begin, rows, kv, c->cs);
}

static hipError_t prof_before(cake_ctx* c, int cls, uint64_t flops, uint64_t bytes) {
    c->prof_open = c->prof_on && ((c->prof_mask >> cls) & 1u);
    if (!c->prof_open) return hipSuccess;
    size_t i = c->prof_recs.size();
    while (c->prof_events.size() < 2 * (i + 1)) {
        hipEvent_t e;
        hipError_t rc = hipEventCreate(&e);
        if (rc != hipSuccess) return rc;
        c->prof_events.push_back(e);
    }
    c->prof_recs.push_back({cls, flops, bytes});
    return hipEventRecord(c->prof_events[2 * i], c->cs);
}
static hipError_t prof_after(cake_ctx* c) {
    if (!c->prof_open) return hipSuccess;
    return hipEventRecord(c->prof_events[2 * c->prof_recs.size() - 1], c->cs);
}
#define KLAUNCH(c, cls, fl, by, expr)                       \
    do {                                                    \
        HIP_TRY(c, prof_before(c, cls, fl, by));            \
        HIP_TRY(c, expr);                                   \
        HIP_TRY(c, prof_after(c));                          \
    } while (0)

// Enqueues the prefill of [tok_begin, tok_begin+rows); token ids already in c->d_ids.
static int enqueue_prefill(cake_ctx* c, int tok_begin, int rows, const cake_kv* kv) {
    const cake_model_desc& m = c->m;
    const uint64_t d = m.d_model, hq = uint64_t(m.n_q_heads) * m.head_dim, hkv = uint64_t(m.n_kv_heads) * m.head_dim;
    const uint64_t nqkv = hq + 2 * hkv, ff = m.ffn_dim, R = rows, e = esize(c);
    const uint64_t t0 = tok_begin;
    // algorithmic work per launch: flops of the contraction; bytes = operands once + result once
    const uint64_t attn_flops = 4 * hq * (t0 * R + R * (R + 1) / 2);
    const uint64_t attn_bytes = (2 * R * hq + 2 * hkv * (t0 + R)) * e;
    KLAUNCH(c, CAKE_K_EMBED, 0, R * d * (e + 4), launch_embed(m.dtype, c->embed, c->d_ids + tok_begin, c->x, rows, d, m.vocab, c->cs));
    HIP_TRY(c, launch_rope_table(c->rope_cs, tok_begin, rows, m.head_dim, m.rope_theta, c->cs));
    for (int l = 0; l < m.n_layers; ++l) {
        const cake_layer_weights& w = c->layers[l];
        KvView view = make_view(c, kv, l);
        KLAUNCH(c, CAKE_K_RMSNORM, 0, R * d * (4 + e), launch_rmsnorm(m.dtype, c->x, w.attn_norm, c->h, rows, d, m.rms_eps, c->cs));
        KLAUNCH(c, CAKE_K_GEMM_QKV, 2 * R * nqkv * d, (R * d + nqkv * d) * e + R * nqkv * 4,
                gemm(c, EPI_STORE_F32, c->h, w.wqkv, nullptr, c->qkv, rows, nqkv, d));
        KLAUNCH(c, CAKE_K_ROPE_KV, 0, R * nqkv * (4 + e),
                launch_rope_kv_write(m.dtype, c->qkv, c->rope_cs, c->q, m.n_q_heads, tok_begin, rows, view, c->cs));
        KLAUNCH(c, CAKE_K_ATTENTION, attn_flops, attn_bytes, attention(c, c->q, c->ao, tok_begin, rows, view));
        KLAUNCH(c, CAKE_K_GEMM_O, 2 * R * d * hq, (R * hq + d * hq) * e + 2 * R * d * 4,
                gemm(c, EPI_RESIDUAL_F32, c->ao, w.wo, nullptr, c->x, rows, d, hq));
        KLAUNCH(c, CAKE_K_RMSNORM, 0, R * d * (4 + e), launch_rmsnorm(m.dtype, c->x, w.ffn_norm, c->h, rows, d, m.rms_eps, c->cs));
        KLAUNCH(c, CAKE_K_GEMM_GATEUP, 4 * R * ff * d, (R * d + 2 * ff * d + R * ff) * e,
                gemm(c, EPI_SWIGLU, c->h, w.w_gate, w.w_up, c->act, rows, m.ffn_dim, d));
        KLAUNCH(c, CAKE_K_GEMM_DOWN, 2 * R * d * ff, (R * ff + d * ff) * e + 2 * R * d * 4,
                gemm(c, EPI_RESIDUAL_F32, c->act, w.w_down, nullptr, c->x, rows, d, m.ffn_dim));
    }
    return CAKE_OK;
}

// Enqueues the first-token step for a prompt of n_tokens whose KV is complete; the last token's id
// is already in c->d_ids[n_tokens-1].  The cache is read, never written.
static int enqueue_first_token(cake_ctx* c, int n_tokens, const cake_kv* kv) {
    const cake_model_desc& m = c->m;
    const uint64_t d = m.d_model, hq = uint64_t(m.n_q_heads) * m.head_dim, hkv = uint64_t(m.n_kv_heads) * m.head_dim;
    const uint64_t ff = m.ffn_dim, e = esize(c), T = n_tokens;
    const int pos = n_tokens - 1;
    HIP_TRY(c, launch_embed(m.dtype, c->embed, c->d_ids + pos, c->x, 1, d, m.vocab, c->cs));
    for (int l = 0; l < m.n_layers; ++l) {
        const cake_layer_weights& w = c->layers[l];
        KvView view = make_view(c, kv, l);
        HIP_TRY(c, launch_rmsnorm(CAKE_F32, c->x, w.attn_norm, c->t_h, 1, d, m.rms_eps, c->cs));
        KLAUNCH(c, CAKE_K_GEMV, 2 * hq * d, hq * d * e,                 // the W_Q rows only: K and V of the token are cached
                launch_gemv(m.dtype, 0, c->t_h, w.wqkv, nullptr, c->t_q, hq, d, c->cs));
        HIP_TRY(c, launch_rope_token(c->t_q, c->t_qr, m.n_q_heads, m.head_dim, pos, m.rope_theta, c->cs));
        KLAUNCH(c, CAKE_K_DECODE_ATTN, 4 * hq * T, 2 * hkv * T * e,
                launch_decode_attention(m.dtype, c->t_qr, c->t_ao, c->t_part, m.n_q_heads, n_tokens, view, c->cs,
                                        c->tun.kernel_path == 1));
        KLAUNCH(c, CAKE_K_GEMV, 2 * d * hq, d * hq * e, launch_gemv(m.dtype, 1, c->t_ao, w.wo, nullptr, c->x, d, hq, c->cs));
        HIP_TRY(c, launch_rmsnorm(CAKE_F32, c->x, w.ffn_norm, c->t_h, 1, d, m.rms_eps, c->cs));
        KLAUNCH(c, CAKE_K_GEMV, 4 * ff * d, 2 * ff * d * e, launch_gemv(m.dtype, 2, c->t_h, w.w_gate, w.w_up, c->t_act, ff, d, c->cs));
        KLAUNCH(c, CAKE_K_GEMV, 2 * d * ff, d * ff * e, launch_gemv(m.dtype, 1, c->t_act, w.w_down, nullptr, c->x, d, ff, c->cs));
    }
    HIP_TRY(c, launch_rmsnorm(CAKE_F32, c->x, c->final_norm, c->t_h, 1, d, m.rms_eps, c->cs));
    KLAUNCH(c, CAKE_K_GEMV, 2 * uint64_t(m.vocab) * d, uint64_t(m.vocab) * d * e,
            launch_gemv(m.dtype, 0, c->t_h, c->lm_head, nullptr, c->t_logits, m.vocab, d, c->cs));
    HIP_TRY(c, launch_argmax(c->t_logits, m.vocab, c->t_tok, c->cs));
    return CAKE_OK;
}

// ------------------------------------------------------------------ throttled load
// The load worker never spins: a spinning thread that the scheduler puts on the compute thread's core
// keeps that thread off it for a whole timeslice.  It sleeps to an absolute deadline on the monotonic
// clock (the worker thread runs with a timer slack of 1 us, so it wakes within a few us); what a wake-up
// is late by is made up at the next piece, because the pacing deadlines are cumulative.
static void wait_until_ns(uint64_t deadline) {
    timespec ts;
    ts.tv_sec = time_t(deadline / 1000000000ull);
    ts.tv_nsec = long(deadline % 1000000000ull);
    while (mono_ns() < deadline)
        if (clock_nanosleep(CLOCK_MONOTONIC, TIMER_ABSTIME, &ts, nullptr) != 0 && errno != EINTR) break;
}

// Waits until everything issued to the copy stream so far has completed.  The last DMA piece of a chunk
// is usually a fraction of a millisecond away: the event is polled for that long, offering the CPU to
// other runnable threads between polls (an interrupt-driven wake-up costs up to hundreds of us on a busy
// host); a longer wait sleeps on the blocking-sync event.
static hipError_t drain_copy_stream(cake_ctx* c) {
    hipError_t e = hipEventRecord(c->ev_load, c->ls);
    if (e != hipSuccess) return e;
    const uint64_t t0 = mono_ns();
    bool polled_not_ready = false;
    for (;;) {
        e = hipEventQuery(c->ev_load);
        if (e != hipErrorNotReady) break;
        polled_not_ready = true;
        if (mono_ns() - t0 > 300000) break;
        std::this_thread::yield();
    }
    // "not ready" is an answer, not a failure: it must not be what a later hipGetLastError() on this thread reports
    if (polled_not_ready) (void)hipGetLastError();
    return e == hipErrorNotReady ? hipEventSynchronize(c->ev_load) : e;
}

// The tier's rate right now: the bandwidth trace if one is running (never below 0.01 GB/s, so a
// sample of zero slows the load down without stalling it for good), else the configured rate.
static double live_rate(cake_ctx* c) {
    const uint64_t t0 = c->tr_t0.load(std::memory_order_relaxed);
    if (t0 && !c->tr_gbps.empty() && c->tr_interval_ns) {
        const uint64_t now = mono_ns();
        const size_t k = size_t(((now > t0 ? now - t0 : 0) / c->tr_interval_ns) % c->tr_gbps.size());
        return std::max(c->tr_gbps[k], 0.01);
    }
    return c->gbps.load(std::memory_order_relaxed);
}

static int ensure_stage(cake_ctx* c, uint64_t bytes) {
    if (c->q_stage_bytes >= bytes) return CAKE_OK;
    // the copy stream may still read the old buffer
    if (hipStreamSynchronize(c->ls) != hipSuccess) return fail(c, CAKE_E_HIP, "stream sync before staging growth");
    (void)hipFree(c->q_stage);
    c->q_stage = nullptr; c->q_stage_bytes = 0;
    if (hipMalloc(&c->q_stage, bytes) != hipSuccess) { (void)hipGetLastError(); return fail(c, CAKE_E_NOMEM, "staging buffer of %llu bytes", (unsigned long long)bytes); }
    c->q_stage_bytes = bytes;
    return CAKE_OK;
}

static int ensure_file_stage(cake_ctx* c, uint64_t bytes) {
    if (c->f_stage_bytes >= bytes) return CAKE_OK;
    if (hipStreamSynchronize(c->ls) != hipSuccess) return fail(c, CAKE_E_HIP, "stream sync before staging growth");
    for (int i = 0; i < 2; ++i) {
        if (c->f_stage[i]) (void)hipHostFree(c->f_stage[i]);
        c->f_stage[i] = nullptr;
    }
    c->f_stage_bytes = 0;
    for (int i = 0; i < 2; ++i)
        if (hipHostMalloc(&c->f_stage[i], bytes, hipHostMallocDefault) != hipSuccess) {
            (void)hipGetLastError();
            return fail(c, CAKE_E_NOMEM, "pinned staging buffer of %llu bytes", (unsigned long long)bytes);
        }
    c->f_stage_bytes = bytes;
    return CAKE_OK;
}

// Reads exactly n bytes at `off`; a short file or an I/O error is a store miss.
static int pread_all(cake_ctx* c, int fd, void* dst, uint64_t n, uint64_t off) {
    char* p = (char*)dst;
    while (n > 0) {
        ssize_t got = pread(fd, p, size_t(n), off_t(off));
        if (got < 0 && errno == EINTR) continue;
        if (got <= 0)
            return fail(c, CAKE_E_STORE_MISS, "store file: read of %llu bytes at %llu failed (%s)", (unsigned long long)n,
                        (unsigned long long)off, got == 0 ? "end of file" : strerror(errno));
        p += got; off += uint64_t(got); n -= uint64_t(got);
    }
    return CAKE_OK;
}

// fixed_gbps > 0: that rate; == 0: unthrottled; < 0: the context's live rate.
static int enqueue_load(cake_ctx* c, const cake_kv_store* st, int tok_begin, int tok_count, const cake_kv* kv,
                        double fixed_gbps) {
    const cake_model_desc& m = c->m;
    if (!st) return fail(c, CAKE_E_INVAL, "store: null");
    const bool from_file = st->source == CAKE_STORE_FILE;
    if (st->source != CAKE_STORE_PINNED && !from_file) return fail(c, CAKE_E_INVAL, "store: unknown source %d", st->source);
    if (from_file ? st->fd < 0 : !st->base) return fail(c, CAKE_E_INVAL, "store: no memory / file given");
    if (tok_count <= 0) return CAKE_OK;
    if (st->page_tokens != kv->page_tokens) return fail(c, CAKE_E_INVAL, "store/page size mismatch");
    const int pt = kv->page_tokens;
    if (tok_begin % pt) return fail(c, CAKE_E_INVAL, "load range must start on a page boundary");
    const int p0 = tok_begin / pt, p1 = (tok_begin + tok_count + pt - 1) / pt;
    if (!store_format_known(st->format)) return fail(c, CAKE_E_INVAL, "store: unknown format %d", st->format);
    const uint64_t layer_bytes = uint64_t(2) * m.n_kv_heads * pt * m.head_dim * esize(c);
    const uint64_t image_bytes = cake::store_image_bytes(m, pt, st->format);
    if (st->page_stride_bytes < image_bytes) return fail(c, CAKE_E_INVAL, "store: page stride smaller than a page image");
    if (p1 > st->n_pages) return fail(c, CAKE_E_STORE_MISS, "store holds %d pages, page %d requested", st->n_pages, p1 - 1);
    const uint64_t piece_max = c->tun.piece_bytes ? c->tun.piece_bytes : (4ull << 20);
    const int bits = store_code_bits(st->format);
    // Nothing is allocated on a load: both staging areas belong to the context (cake_create, cake_set_tuning).
    // Quantised images go through a ring of image slots; a slot is written again only after the dequantise
    // kernel that read it, because copies and kernels of a load share the one copy stream.
    const uint64_t n_slots = bits ? c->q_stage_bytes / image_bytes : 0;
    if (bits && n_slots == 0)
        return fail(c, CAKE_E_INVAL, "a quantised page image of %llu bytes exceeds the context's staging buffer (%llu): "
                    "page_tokens above max_chunk", (unsigned long long)image_bytes, (unsigned long long)c->q_stage_bytes);
    if (from_file && c->f_stage_bytes < piece_max) return fail(c, CAKE_E_STATE, "file staging smaller than a DMA piece");
    const uint64_t start = mono_ns();
    c->load_bytes_done.store(0);
    c->load_start_ns.store(start);
    double release = 0.0;  // ns after start at which the tier has delivered everything issued so far
    // src: address in pinned memory, or byte position in the file
    auto paced_copy = [&](char* dst, uint64_t src, uint64_t bytes) -> int {
        for (uint64_t off = 0; off < bytes; off += piece_max) {
            uint64_t n = std::min(piece_max, bytes - off);
            double rate = fixed_gbps < 0 ? live_rate(c) : fixed_gbps;
            if (rate > 0) {
                release += double(n) / rate;  // GB/s = bytes per ns
                wait_until_ns(start + uint64_t(release));
            }
            const void* from = (const void*)(uintptr_t)(src + off);
            if (from_file) {
                // two buffers: this piece is read from the file while the previous piece's DMA runs
                const int b = c->f_next;
                c->f_next ^= 1;
                int rc = pread_all(c, st->fd, c->f_stage[b], n, src + off);
                if (rc != CAKE_OK) return rc;
                // the copy stream is in order: once it has drained, the DMA out of the OTHER buffer (issued one
                // piece ago, running while this piece was read) is done and that buffer may be refilled next
                HIP_TRY(c, drain_copy_stream(c));
                from = c->f_stage[b];
                HIP_TRY(c, hipMemcpyAsync(dst + off, from, n, hipMemcpyHostToDevice, c->ls));
            } else {
                HIP_TRY(c, hipMemcpyAsync(dst + off, from, n, hipMemcpyHostToDevice, c->ls));
            }
            c->load_bytes_done.fetch_add(n, std::memory_order_relaxed);
        }
        return CAKE_OK;
    };
    for (int p = p0; p < p1; ++p) {
        const uint64_t img = (from_file ? st->file_offset : uint64_t((uintptr_t)st->base)) + uint64_t(p) * st->page_stride_bytes;
        const int pp = kv->block_table_host[p];
        if (bits) {
            // the whole image lands in the staging buffer, then one kernel on the copy stream
            // dequantises it into the page of every layer; stream order keeps the two apart
            char* stage = (char*)c->q_stage + (uint64_t(p - p0) % n_slots) * image_bytes;
            int rc = paced_copy(stage, img, image_bytes);
            if (rc != CAKE_OK) return rc;
            HIP_TRY(c, launch_dequant_page(m.dtype, stage, make_view(c, kv, 0), pp, m.n_layers, bits, c->ls));
            continue;
        }
        for (int l = 0; l < m.n_layers; ++l) {
            char* dst = (char*)kv->pool + (uint64_t(l) * kv->n_physical_pages + pp) * layer_bytes;
            int rc = paced_copy(dst, img + uint64_t(l) * layer_bytes, layer_bytes);
            if (rc != CAKE_OK) return rc;
        }
    }
    return CAKE_OK;
}

// ------------------------------------------------------------------ executor backend
namespace {
struct HipBackend : Backend {
    cake_ctx* c;
    const cake_kv_store* store;
    const cake_kv* kv;
    const int32_t *tb, *tc;
    int rc_hard = CAKE_OK;
    HipBackend(cake_ctx* c_, const cake_kv_store* s, const cake_kv* k, const int32_t* b, const int32_t* n)
        : c(c_), store(s), kv(k), tb(b), tc(n) {}
    int compute_chunk(int i, uint64_t* device_ns) override {
        if (hipEventRecord(c->ev_a, c->cs) != hipSuccess) return CAKE_E_HIP;
        int rc = enqueue_prefill(c, tb[i], tc[i], kv);
        if (rc != CAKE_OK) return rc;
        if (hipEventRecord(c->ev_b, c->cs) != hipSuccess) return CAKE_E_HIP;
        if (hipStreamSynchronize(c->cs) != hipSuccess) return fail(c, CAKE_E_HIP, "compute stream failed in chunk %d", i);
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, c->ev_a, c->ev_b) == hipSuccess) *device_ns = uint64_t(double(ms) * 1e6);
        return CAKE_OK;
    }
    int load_chunk(int i) override {
        int rc = enqueue_load(c, store, tb[i], tc[i], kv, -1.0);
        if (rc != CAKE_OK) {
            // pieces (and dequantise kernels) of this chunk that were already issued must have landed before
            // the chunk goes back to the range: the compute side may rewrite the same pages at once
            (void)hipStreamSynchronize(c->ls);
            return rc;
        }
        if (drain_copy_stream(c) != hipSuccess) return fail(c, CAKE_E_HIP, "copy stream failed in chunk %d", i);
        return CAKE_OK;
    }
    void on_load_completed(int n_loaded) override {
        if (c->step_after >= 0 && n_loaded == c->step_after) c->gbps.store(c->step_gbps);
    }
    bool load_progress(uint64_t* elapsed_ns, uint64_t* bytes_done) override {
        const uint64_t st = c->load_start_ns.load(), by = c->load_bytes_done.load(), now = mono_ns();
        if (!st || now <= st) return false;
        *elapsed_ns = now - st;
        *bytes_done = by;
        return by > 0;
    }
};
}  // namespace

extern "C" {

int32_t cake_create(cake_ctx** out, const cake_model_desc* model, const cake_weights* weights, int32_t max_tokens,
                    int32_t max_chunk, void* compute_stream, void* copy_stream) {
    if (!out || !model || !weights || !weights->layers || !weights->embed) return CAKE_E_INVAL;
    const cake_model_desc& m = *model;
    if (m.n_layers <= 0 || m.d_model <= 0 || m.n_q_heads <= 0 || m.n_kv_heads <= 0 || m.ffn_dim <= 0 || m.vocab <= 0)
        return CAKE_E_INVAL;
    if (m.head_dim != 64 && m.head_dim != 128) return CAKE_E_INVAL;
    if (m.n_q_heads % m.n_kv_heads) return CAKE_E_INVAL;
    if (m.dtype != CAKE_F32 && m.dtype != CAKE_BF16) return CAKE_E_INVAL;
    if ((m.d_model & 7) || (m.ffn_dim & 7)) return CAKE_E_INVAL;  // 16-byte vector loads of rows
    if (max_tokens <= 0 || max_chunk <= 0 || max_chunk > max_tokens) return CAKE_E_INVAL;
    for (int l = 0; l < m.n_layers; ++l) {
        const cake_layer_weights& w = weights->layers[l];
        if (!w.attn_norm || !w.wqkv || !w.wo || !w.ffn_norm || !w.w_gate || !w.w_up || !w.w_down) return CAKE_E_INVAL;
    }
    cake_ctx* c = new (std::nothrow) cake_ctx();
    if (!c) return CAKE_E_NOMEM;
    c->m = m;
    c->layers.assign(weights->layers, weights->layers + m.n_layers);
    c->embed = weights->embed;
    c->max_tokens = max_tokens;
    c->max_chunk = max_chunk;
    c->cs = (hipStream_t)compute_stream;
    c->ls = (hipStream_t)copy_stream;
    const size_t e = esize(c), R = size_t(max_chunk);
    const size_t hq = size_t(m.n_q_heads) * m.head_dim, nqkv = size_t(m.n_q_heads + 2 * m.n_kv_heads) * m.head_dim;
    bool ok = hipGetDevice(&c->device) == hipSuccess;
    ok = ok && static_scratch_for_device(c->device, &c->static_scratch) == hipSuccess;
    ok = ok && hipMalloc((void**)&c->x, R * m.d_model * 4) == hipSuccess;
    ok = ok && hipMalloc(&c->h, R * m.d_model * e) == hipSuccess;
    ok = ok && hipMalloc((void**)&c->qkv, R * nqkv * 4) == hipSuccess;
    ok = ok && hipMalloc(&c->q, R * hq * e) == hipSuccess;
    ok = ok && hipMalloc(&c->ao, R * hq * e) == hipSuccess;
    ok = ok && hipMalloc(&c->act, R * m.ffn_dim * e) == hipSuccess;
    ok = ok && hipMalloc((void**)&c->rope_cs, R * m.head_dim * 4) == hipSuccess;
    ok = ok && hipMalloc((void**)&c->d_ids, size_t(max_tokens) * 4) == hipSuccess;
    if (m.dtype == CAKE_BF16) {
        // room for 256 workgroups' float32 tiles of 256 x 256, less for a small model
        const size_t rows_up = (R + 255) / 256 * 256;
        c->split.part_bytes = std::min<size_t>(size_t(64) << 20, 8 * rows_up * std::max<size_t>(m.d_model, nqkv) * 4);
        c->split.n_counters = 1024;
        ok = ok && hipMalloc((void**)&c->split.part, c->split.part_bytes) == hipSuccess;
        ok = ok && hipMalloc((void**)&c->split.counters, size_t(c->split.n_counters) * 4) == hipSuccess;
        ok = ok && hipMemset(c->split.counters, 0, size_t(c->split.n_counters) * 4) == hipSuccess;
    }
    {
        // staging of the load path, so that no load allocates: device room for the 8-bit images (the largest
        // quantised format) of max_chunk tokens, and two pinned buffers of one DMA piece for file-backed stores
        const uint64_t per_token = cake::store_image_bytes(m, 64, CAKE_STORE_INT8) / 64;
        ok = ok && ensure_stage(c, per_token * uint64_t(max_chunk)) == CAKE_OK;
        ok = ok && ensure_file_stage(c, c->tun.piece_bytes) == CAKE_OK;
    }
    ok = ok && hipEventCreate(&c->ev_a) == hipSuccess && hipEventCreate(&c->ev_b) == hipSuccess;
    ok = ok && hipEventCreateWithFlags(&c->ev_load, hipEventBlockingSync | hipEventDisableTiming) == hipSuccess;
    if (weights->final_norm && weights->lm_head) {
        c->final_norm = weights->final_norm;
        c->lm_head = weights->lm_head;
        ok = ok && hipMalloc((void**)&c->t_h, size_t(m.d_model) * 4) == hipSuccess;
        ok = ok && hipMalloc((void**)&c->t_q, hq * 4) == hipSuccess;
        ok = ok && hipMalloc((void**)&c->t_qr, hq * 4) == hipSuccess;
        ok = ok && hipMalloc((void**)&c->t_ao, hq * 4) == hipSuccess;
        ok = ok && hipMalloc((void**)&c->t_act, size_t(m.ffn_dim) * 4) == hipSuccess;
        ok = ok && hipMalloc((void**)&c->t_logits, size_t(m.vocab) * 4) == hipSuccess;
        ok = ok && hipMalloc((void**)&c->t_part, decode_attention_workspace_bytes(m.n_q_heads, m.head_dim)) == hipSuccess;
        ok = ok && hipMalloc((void**)&c->t_tok, 4) == hipSuccess;
    }
    if (!ok) {
        (void)hipGetLastError();
        cake_destroy(c);
        return CAKE_E_NOMEM;
    }
    const int device = c->device;
    c->load_thread.start([device] {
        (void)hipSetDevice(device);
        (void)prctl(PR_SET_TIMERSLACK, 1000UL, 0UL, 0UL, 0UL);   // this thread's sleeps end within ~1 us of their deadline
    });
    *out = c;
    return CAKE_OK;
}

int32_t cake_destroy(cake_ctx* c) {
    if (!c) return CAKE_OK;
    c->load_thread.stop();
    if (c->cs || c->ls) (void)hipDeviceSynchronize();
    (void)hipFree(c->x); (void)hipFree(c->h); (void)hipFree(c->qkv); (void)hipFree(c->q);
    (void)hipFree(c->ao); (void)hipFree(c->act); (void)hipFree(c->rope_cs); (void)hipFree(c->d_ids);
    (void)hipFree(c->t_h); (void)hipFree(c->t_q); (void)hipFree(c->t_qr); (void)hipFree(c->t_ao);
    (void)hipFree(c->t_act); (void)hipFree(c->t_logits); (void)hipFree(c->t_part); (void)hipFree(c->t_tok);
    (void)hipFree(c->q_stage); (void)hipFree(c->split.part); (void)hipFree(c->split.counters);
    for (int i = 0; i < 2; ++i)
        if (c->f_stage[i]) (void)hipHostFree(c->f_stage[i]);
    for (hipEvent_t e : c->prof_events) (void)hipEventDestroy(e);
    if (c->ev_a) (void)hipEventDestroy(c->ev_a);
    if (c->ev_b) (void)hipEventDestroy(c->ev_b);
    if (c->ev_load) (void)hipEventDestroy(c->ev_load);
    delete c;
    return CAKE_OK;
}

const char* cake_last_error(const cake_ctx* c) { return c ? c->err.c_str() : "null context"; }

int32_t cake_set_tuning(cake_ctx* c, const cake_tuning* t) {
    if (!c || !t) return CAKE_E_INVAL;
    if (t->prior_compute_ns && t->prior_compute_flops) {
        c->tun.prior_compute_ns = t->prior_compute_ns;
        c->tun.prior_compute_flops = t->prior_compute_flops;
    }
    if (t->piece_bytes) {
        if (t->piece_bytes < 4096) return fail(c, CAKE_E_INVAL, "piece_bytes below 4096");
        c->tun.piece_bytes = t->piece_bytes;
        c->load_thread.wait();   // a queued load may be using the staging buffers this resizes
        int rc = ensure_file_stage(c, t->piece_bytes);
        if (rc != CAKE_OK) return rc;
    }
    if (t->kernel_path < 0 || t->kernel_path > 1) return fail(c, CAKE_E_INVAL, "kernel_path must be 0 or 1");
    c->tun.kernel_path = t->kernel_path;
    if (t->gemm_config < 0 || t->gemm_config > 7) return fail(c, CAKE_E_INVAL, "gemm_config must be 0..7");
    c->tun.gemm_config = t->gemm_config;
    if (t->attn_variant < 0 || t->attn_variant > 3) return fail(c, CAKE_E_INVAL, "attn_variant must be 0..3");
    c->tun.attn_variant = t->attn_variant;
    if (t->gemm_ksplit != 0 && t->gemm_ksplit != 1 && t->gemm_ksplit != 2 && t->gemm_ksplit != 4 && t->gemm_ksplit != 8)
        return fail(c, CAKE_E_INVAL, "gemm_ksplit must be 0, 1, 2, 4 or 8");
    c->tun.gemm_ksplit = t->gemm_ksplit;
    return CAKE_OK;
}

int32_t cake_prefill_chunk(cake_ctx* c, const int32_t* token_ids, int32_t tok_begin, int32_t tok_count,
                           const cake_kv* kv) {
    if (!c || !token_ids) return CAKE_E_INVAL;
    if (tok_begin < 0 || tok_count < 0 || tok_count > c->max_chunk || tok_begin + tok_count > c->max_tokens)
        return fail(c, CAKE_E_INVAL, "token range [%d,+%d) outside max_tokens %d / max_chunk %d", tok_begin, tok_count,
                    c->max_tokens, c->max_chunk);
    if (tok_count == 0) return CAKE_OK;
    int rc = check_kv(c, kv, tok_begin + tok_count);
    if (rc != CAKE_OK) return rc;
    for (int i = 0; i < tok_count; ++i) {
        int id = token_ids[tok_begin + i];
        if (id < 0 || id >= c->m.vocab) return fail(c, CAKE_E_INVAL, "token id %d at %d outside the vocabulary", id, tok_begin + i);
    }
    HIP_TRY(c, hipMemcpyAsync(c->d_ids + tok_begin, token_ids + tok_begin, size_t(tok_count) * 4, hipMemcpyHostToDevice, c->cs));
    return enqueue_prefill(c, tok_begin, tok_count, kv);
}

int32_t cake_load_chunk(cake_ctx* c, const cake_kv_store* store, int32_t tok_begin, int32_t tok_count,
                        const cake_kv* kv, double gbps) {
    if (!c) return CAKE_E_INVAL;
    if (tok_begin < 0 || tok_count < 0) return fail(c, CAKE_E_INVAL, "negative token range");
    int rc = check_kv(c, kv, tok_begin + tok_count);
    if (rc != CAKE_OK) return rc;
    rc = check_store(c, store, kv);
    if (rc != CAKE_OK) return rc;
    if (tok_begin % kv->page_tokens) return fail(c, CAKE_E_INVAL, "load range must start on a page boundary");
    if ((tok_begin + tok_count + kv->page_tokens - 1) / kv->page_tokens > store->n_pages)
        return fail(c, CAKE_E_STORE_MISS, "store holds %d pages, the range needs more", store->n_pages);
    // The range goes to the context's load worker, which paces the pieces onto the copy stream; this call
    // returns at once.  The two descriptors are copied, what they point to stays borrowed until cake_sync_load.
    const cake_kv_store st = *store;
    const cake_kv k = *kv;
    const double rate = gbps > 0 ? gbps : 0.0;
    c->load_thread.submit([c, st, k, tok_begin, tok_count, rate] {
        int r = enqueue_load(c, &st, tok_begin, tok_count, &k, rate);
        if (r != CAKE_OK) {
            int expected = CAKE_OK;
            c->async_load_rc.compare_exchange_strong(expected, r);   // the first failure is the one reported
        }
    });
    return CAKE_OK;
}

int32_t cake_bidirectional_prefill(cake_ctx* c, const int32_t* token_ids, int32_t n_tokens,
                                   const cake_kv_store* store, int32_t chunk, double gbps, int32_t mode,
                                   int32_t forced_m, const cake_kv* kv, cake_result* res) {
    if (!c || !token_ids || !res) return CAKE_E_INVAL;
    if (n_tokens <= 0 || n_tokens > c->max_tokens) return fail(c, CAKE_E_INVAL, "n_tokens %d outside (0, %d]", n_tokens, c->max_tokens);
    if (chunk <= 0 || chunk > c->max_chunk) return fail(c, CAKE_E_INVAL, "chunk %d outside (0, %d]", chunk, c->max_chunk);
    if (mode < CAKE_BIDIR || mode > CAKE_GREEDY) return fail(c, CAKE_E_INVAL, "unknown mode %d", mode);
    int rc = check_kv(c, kv, n_tokens);
    if (rc != CAKE_OK) return rc;
    if (chunk % kv->page_tokens) return fail(c, CAKE_E_INVAL, "chunk must be a multiple of page_tokens");
    const int n = (n_tokens + chunk - 1) / chunk;
    if (mode == CAKE_FORCED_SPLIT && (forced_m < 0 || forced_m > n)) return fail(c, CAKE_E_INVAL, "forced_m %d outside [0,%d]", forced_m, n);
    if (mode != CAKE_COMPUTE_ONLY) {
        rc = check_store(c, store, kv);
        if (rc != CAKE_OK) return rc;
        if (!(gbps > 0)) return fail(c, CAKE_E_INVAL, "gbps must be positive");
    }
    std::vector<int32_t> tb(n), tc(n);
    std::vector<uint64_t> flops(n), bytes(n);
    const uint64_t image = cake::store_image_bytes(c->m, kv->page_tokens, store ? store->format : CAKE_STORE_RAW);
    for (int i = 0; i < n; ++i) {
        tb[i] = i * chunk;
        tc[i] = std::min(chunk, n_tokens - tb[i]);
        flops[i] = cake::range_flops(c->m, tb[i], tc[i]);
        bytes[i] = uint64_t((tc[i] + kv->page_tokens - 1) / kv->page_tokens) * image;
    }
    // The store may hold only a prefix of the prompt (App. A step 2): the race covers the chunks
    // wholly inside it, the others are computed once the raced part is complete.
    int n_race = n;
    if (mode != CAKE_COMPUTE_ONLY) {
        const int64_t stored_tokens = std::min<int64_t>(n_tokens, int64_t(store->n_pages) * kv->page_tokens);
        n_race = 0;
        while (n_race < n && tb[n_race] + tc[n_race] <= stored_tokens) ++n_race;
    }
    if (mode == CAKE_FORCED_SPLIT && forced_m > n_race) return fail(c, CAKE_E_INVAL, "forced_m %d beyond the %d stored chunks", forced_m, n_race);
    const bool computes = mode != CAKE_LOAD_ONLY || n_race < n;
    if (computes)
        for (int i = 0; i < n_tokens; ++i)
            if (token_ids[i] < 0 || token_ids[i] >= c->m.vocab) return fail(c, CAKE_E_INVAL, "token id at %d outside the vocabulary", i);

    c->status.reset(new std::atomic<int32_t>[n]);
    c->n_status = n;
    for (int i = 0; i < n; ++i) c->status[i].store(CAKE_CHUNK_EMPTY);
    c->gbps.store(gbps > 0 ? gbps : 0.0);

    Executor ex;
    ex.core.est.prior_c_ns = c->tun.prior_compute_ns;
    ex.core.est.prior_c_flops = c->tun.prior_compute_flops;
    ex.core.est.prior_l_ns = 1000000000ull;
    ex.core.est.prior_l_bytes = gbps > 0 ? uint64_t(gbps * 1e9) : 4000000000ull;
    if (ex.core.est.prior_l_bytes == 0) ex.core.est.prior_l_bytes = 1;
    ex.core.init(n_race, flops.data(), bytes.data(), mode, forced_m);
    ex.core.tok_begin = tb.data(); ex.core.tok_count = tc.data(); ex.core.model = &c->m;
    ex.core.log = res->decisions;
    ex.core.log_cap = res->decisions ? res->decisions_cap : 0;
    ex.status = c->status.get();
    ex.tok_begin = tb.data();
    ex.tok_count = tc.data();

    HipBackend be(c, store, kv, tb.data(), tc.data());
    const uint64_t t_entry = mono_ns();
    if (computes) {
        HIP_TRY(c, hipMemcpyAsync(c->d_ids, token_ids, size_t(n_tokens) * 4, hipMemcpyHostToDevice, c->cs));
    }
    uint64_t race_ns = 0;
    rc = ex.run(be, &race_ns, &c->load_thread);
    // chunks beyond the stored prefix: they attend to everything before them, so they start after the join
    ex.chunk_log.resize(size_t(n), cake_chunk_log{CAKE_SRC_NONE, 0, 0, 0, 0, 0, 0});
    for (int i = n_race; i < n && rc == CAKE_OK; ++i) {
        c->status[i].store(CAKE_CHUNK_COMPUTING);
        cake_chunk_log& cl = ex.chunk_log[i];
        cl.start_ns = ex.now();
        rc = be.compute_chunk(i, &cl.device_ns);
        if (rc != CAKE_OK) break;
        cl.source = CAKE_SRC_COMPUTE; cl.tok_begin = tb[i]; cl.tok_count = tc[i]; cl.end_ns = ex.now(); cl.work = flops[i];
        c->status[i].store(CAKE_CHUNK_RESIDENT);
    }
    const uint64_t ttft = mono_ns() - t_entry;
    c->step_after = -1;  // a scheduled bandwidth step applies to one run

    res->n_chunks = n;
    res->n_decisions = ex.core.log_n;
    res->load_failed_chunk = ex.load_failed_chunk;
    res->ttft_ns = ttft;
    res->meet_point = 0;
    res->stored_chunks = n_race;
    res->pad_ = 0;
    res->compute_busy_ns = res->compute_device_ns = res->compute_flops = res->load_busy_ns = res->load_bytes = 0;
    for (int i = 0; i < n; ++i) {
        const cake_chunk_log& cl = ex.chunk_log[i];
        if (cl.source == CAKE_SRC_COMPUTE) {
            if (i < n_race) ++res->meet_point;
            res->compute_busy_ns += cl.end_ns - cl.start_ns;
            res->compute_device_ns += cl.device_ns;
            res->compute_flops += cl.work;
        } else if (cl.source == CAKE_SRC_LOAD) {
            res->load_busy_ns += cl.end_ns - cl.start_ns;
            res->load_bytes += cl.work;
        }
        if (res->chunks && i < res->chunks_cap) res->chunks[i] = cl;
    }
    if (rc != CAKE_OK) {
        if (c->err.empty()) fail(c, rc, "race ended with status %d", rc);
        return rc;
    }
    if ((res->chunks && res->chunks_cap < n) || ex.core.log_overflow) return CAKE_E_CAPACITY;
    return CAKE_OK;
}

int32_t cake_first_token(cake_ctx* c, const int32_t* token_ids, int32_t n_tokens, const cake_kv* kv, int32_t* token_out,
                         float* logits_out, uint64_t* device_ns_out) {
    if (!c || !token_ids || !token_out) return CAKE_E_INVAL;
    if (!c->final_norm || !c->lm_head) return fail(c, CAKE_E_STATE, "the context was created without final_norm / lm_head");
    if (n_tokens <= 0 || n_tokens > c->max_tokens) return fail(c, CAKE_E_INVAL, "n_tokens %d outside (0, %d]", n_tokens, c->max_tokens);
    int rc = check_kv(c, kv, n_tokens);
    if (rc != CAKE_OK) return rc;
    const int32_t last = token_ids[n_tokens - 1];
    if (last < 0 || last >= c->m.vocab) return fail(c, CAKE_E_INVAL, "last token id outside the vocabulary");
    HIP_TRY(c, hipMemcpyAsync(c->d_ids + (n_tokens - 1), &token_ids[n_tokens - 1], 4, hipMemcpyHostToDevice, c->cs));
    HIP_TRY(c, hipEventRecord(c->ev_a, c->cs));
    rc = enqueue_first_token(c, n_tokens, kv);
    if (rc != CAKE_OK) return rc;
    HIP_TRY(c, hipEventRecord(c->ev_b, c->cs));
    HIP_TRY(c, hipMemcpyAsync(token_out, c->t_tok, 4, hipMemcpyDeviceToHost, c->cs));
    if (logits_out)
        HIP_TRY(c, hipMemcpyAsync(logits_out, c->t_logits, size_t(c->m.vocab) * 4, hipMemcpyDeviceToHost, c->cs));
    HIP_TRY(c, hipStreamSynchronize(c->cs));
    if (device_ns_out) {
        float ms = 0.f;
        HIP_TRY(c, hipEventElapsedTime(&ms, c->ev_a, c->ev_b));
        *device_ns_out = uint64_t(double(ms) * 1e6);
    }
    return CAKE_OK;
}

int32_t cake_write_store(cake_ctx* c, const cake_kv* kv, int32_t n_tokens, const cake_kv_store* dst) {
    if (!c || !dst || !dst->base) return CAKE_E_INVAL;
    if (n_tokens <= 0 || n_tokens > c->max_tokens) return fail(c, CAKE_E_INVAL, "n_tokens %d outside (0, %d]", n_tokens, c->max_tokens);
    int rc = check_kv(c, kv, n_tokens);
    if (rc != CAKE_OK) return rc;
    if (!store_format_known(dst->format)) return fail(c, CAKE_E_INVAL, "store: unknown format %d", dst->format);
    const int pt = kv->page_tokens, n_pages = (n_tokens + pt - 1) / pt;
    const uint64_t image = cake::store_image_bytes(c->m, pt, dst->format);
    if (dst->page_tokens != pt || dst->page_stride_bytes < image || dst->n_pages < n_pages)
        return fail(c, CAKE_E_INVAL, "store does not fit %d pages of %llu bytes", n_pages, (unsigned long long)image);
    const uint64_t layer_bytes = uint64_t(2) * c->m.n_kv_heads * pt * c->m.head_dim * esize(c);
    const int bits = store_code_bits(dst->format);
    if (bits) {
        rc = ensure_stage(c, image);
        if (rc != CAKE_OK) return rc;
    }
    for (int p = 0; p < n_pages; ++p) {
        char* out = (char*)dst->base + uint64_t(p) * dst->page_stride_bytes;
        const int pp = kv->block_table_host[p];
        if (bits) {
            char* stage = (char*)c->q_stage;   // quantise, copy out, next page: one stream keeps them in order
            HIP_TRY(c, launch_quant_page(c->m.dtype, stage, make_view(c, kv, 0), pp, c->m.n_layers, bits, c->cs));
            HIP_TRY(c, hipMemcpyAsync(out, stage, image, hipMemcpyDeviceToHost, c->cs));
        } else {
            for (int l = 0; l < c->m.n_layers; ++l) {
                const char* src = (const char*)kv->pool + (uint64_t(l) * kv->n_physical_pages + pp) * layer_bytes;
                HIP_TRY(c, hipMemcpyAsync(out + uint64_t(l) * layer_bytes, src, layer_bytes, hipMemcpyDeviceToHost, c->cs));
            }
        }
    }
    HIP_TRY(c, hipStreamSynchronize(c->cs));
    return CAKE_OK;
}

int32_t cake_set_traces(cake_ctx* c, const cake_traces* t) {
    if (!c) return CAKE_E_INVAL;
    c->tr_other.clear(); c->tr_ids.clear(); c->tr_gbps.clear(); c->tr_interval_ns = 0;
    if (!t) return CAKE_OK;
    if (t->n_other_tokens < 0 || t->n_gbps < 0) return fail(c, CAKE_E_INVAL, "traces: negative length");
    if (t->n_other_tokens > 0) {
        if (!t->other_tokens || !t->scratch_kv || !t->scratch_token_ids || t->n_scratch_tokens <= 0)
            return fail(c, CAKE_E_INVAL, "traces: other_tokens needs scratch pages and token ids");
        int rc = check_kv(c, t->scratch_kv, t->n_scratch_tokens);
        if (rc != CAKE_OK) return rc;
        for (int i = 0; i < t->n_other_tokens; ++i)
            if (t->other_tokens[i] < 0 || t->other_tokens[i] > t->n_scratch_tokens || t->other_tokens[i] > c->max_chunk)
                return fail(c, CAKE_E_INVAL, "traces: other_tokens[%d] outside [0, min(scratch, max_chunk)]", i);
        for (int i = 0; i < t->n_scratch_tokens; ++i)
            if (t->scratch_token_ids[i] < 0 || t->scratch_token_ids[i] >= c->m.vocab)
                return fail(c, CAKE_E_INVAL, "traces: scratch token id outside the vocabulary");
        c->tr_other.assign(t->other_tokens, t->other_tokens + t->n_other_tokens);
        c->tr_ids.assign(t->scratch_token_ids, t->scratch_token_ids + t->n_scratch_tokens);
        c->tr_kv = *t->scratch_kv;
    }
    if (t->n_gbps > 0) {
        if (!t->gbps || t->gbps_interval_ns == 0) return fail(c, CAKE_E_INVAL, "traces: gbps needs samples and an interval");
        for (int i = 0; i < t->n_gbps; ++i)
            if (!(t->gbps[i] >= 0)) return fail(c, CAKE_E_INVAL, "traces: gbps[%d] negative", i);
        c->tr_gbps.assign(t->gbps, t->gbps + t->n_gbps);
        c->tr_interval_ns = t->gbps_interval_ns;
    }
    return CAKE_OK;
}

// Adaptive mode (Sec. 4 Part 3): the engine loop that deals a token budget out per step.
int32_t cake_adaptive_serve(cake_ctx* c, cake_request* reqs, int32_t n_reqs, int32_t token_budget, int32_t fetch_chunk,
                            double gbps, cake_result* res, cake_step_log* steps, int32_t steps_cap,
                            int32_t* n_steps_out) {
    if (!c || !reqs || n_reqs <= 0 || !res) return CAKE_E_INVAL;
    if (token_budget <= 0 || token_budget > c->max_chunk) return fail(c, CAKE_E_INVAL, "token_budget %d outside (0, %d]", token_budget, c->max_chunk);
    int P = -1;
    for (int i = 0; i < n_reqs; ++i) {
        cake_request& r = reqs[i];
        if (!r.token_ids || r.n_tokens <= 0 || r.n_tokens > c->max_tokens) return fail(c, CAKE_E_INVAL, "request %d: bad prompt", i);
        int rc = check_kv(c, r.kv, r.n_tokens);
        if (rc != CAKE_OK) return rc;
        for (int t = 0; t < r.n_tokens; ++t)
            if (r.token_ids[t] < 0 || r.token_ids[t] >= c->m.vocab) return fail(c, CAKE_E_INVAL, "request %d: token id outside the vocabulary", i);
        if (r.has_prefix_cache) {
            if (P >= 0) return fail(c, CAKE_E_INVAL, "more than one prefix-cached request");
            P = i;
        }
        if (r.want_first_token && !c->lm_head) return fail(c, CAKE_E_STATE, "request %d: the first token needs final_norm and lm_head", i);
        r.ttft_ns = 0; r.tokens_computed = 0; r.tokens_loaded = 0; r.first_token = -1;
    }
    std::vector<int32_t> tb, tc;
    std::vector<uint64_t> flops, bytes;
    Executor ex;
    int nc = 0;
    if (P >= 0) {
        const cake_request& r = reqs[P];
        {
            int rcs = check_store(c, r.store, r.kv);
            if (rcs != CAKE_OK) return rcs;
            if (int64_t(r.store->n_pages) * r.kv->page_tokens < r.n_tokens) return fail(c, CAKE_E_INVAL, "adaptive mode needs the whole prompt stored");
        }
        if (fetch_chunk <= 0 || fetch_chunk % r.kv->page_tokens) return fail(c, CAKE_E_INVAL, "fetch_chunk must be a multiple of page_tokens");
        if (!store_format_known(r.store->format)) return fail(c, CAKE_E_INVAL, "store: unknown format %d", r.store->format);
        if (r.store->page_tokens != r.kv->page_tokens ||
            r.store->page_stride_bytes < cake::store_image_bytes(c->m, r.kv->page_tokens, r.store->format))
            return fail(c, CAKE_E_INVAL, "store does not match the page layout");
        if (!(gbps > 0)) return fail(c, CAKE_E_INVAL, "gbps must be positive");
        nc = (r.n_tokens + fetch_chunk - 1) / fetch_chunk;
        tb.resize(nc); tc.resize(nc); flops.resize(nc); bytes.resize(nc);
        const uint64_t image = cake::store_image_bytes(c->m, r.kv->page_tokens, r.store->format);
        for (int i = 0; i < nc; ++i) {
            tb[i] = i * fetch_chunk;
            tc[i] = std::min(fetch_chunk, r.n_tokens - tb[i]);
            flops[i] = cake::range_flops(c->m, tb[i], tc[i]);
            bytes[i] = uint64_t((tc[i] + r.kv->page_tokens - 1) / r.kv->page_tokens) * image;
        }
    }
    c->status.reset(new std::atomic<int32_t>[std::max(nc, 1)]);
    c->n_status = nc;
    for (int i = 0; i < nc; ++i) c->status[i].store(CAKE_CHUNK_EMPTY);
    c->gbps.store(gbps > 0 ? gbps : 0.0);
    ex.core.est.prior_c_ns = c->tun.prior_compute_ns;
    ex.core.est.prior_c_flops = c->tun.prior_compute_flops;
    ex.core.est.prior_l_ns = 1000000000ull;
    ex.core.est.prior_l_bytes = gbps > 0 ? std::max<uint64_t>(1, uint64_t(gbps * 1e9)) : 4000000000ull;
    ex.core.init(nc, flops.data(), bytes.data(), CAKE_BIDIR, 0);
    ex.core.tok_begin = tb.data(); ex.core.tok_count = tc.data(); ex.core.model = &c->m;
    ex.core.log = res->decisions;
    ex.core.log_cap = res->decisions ? res->decisions_cap : 0;
    ex.status = c->status.get();
    ex.tok_begin = tb.data(); ex.tok_count = tc.data();
    ex.chunk_log.assign(size_t(nc), cake_chunk_log{CAKE_SRC_NONE, 0, 0, 0, 0, 0, 0});
    HipBackend be(c, P >= 0 ? reqs[P].store : nullptr, P >= 0 ? reqs[P].kv : nullptr, tb.data(), tc.data());

    // requests in arrival order (stable)
    std::vector<int> order(n_reqs);
    for (int i = 0; i < n_reqs; ++i) order[i] = i;
    std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return reqs[a].arrival_ns < reqs[b].arrival_ns; });
    std::vector<int32_t> next_tok(n_reqs, 0);
    std::vector<char> done(n_reqs, 0);
    // a request whose KV is complete either leaves, or waits for its decode step (the first token)
    std::vector<char> kv_complete(n_reqs, 0), ft_pending(n_reqs, 0);
    std::vector<int32_t> ft_tok(n_reqs, -1);
    auto finish_kv = [&](int i, uint64_t at_ns, int* n_done_p) {
        kv_complete[i] = 1;
        if (reqs[i].want_first_token) { ft_pending[i] = 1; return; }
        reqs[i].ttft_ns = at_ns - reqs[i].arrival_ns;
        done[i] = 1; ++*n_done_p;
    };
    int n_done = 0, n_steps = 0, hard = CAKE_OK;
    bool steps_overflow = false, loader_started = false;
    uint64_t prefix_compute_end = 0, starved_ns = 0;
    ex.t0 = mono_ns();

    struct Part { int req, first, count; bool decode; };   // req == -1: the other users' share of the step (trace)
    std::vector<Part> parts;
    if (!c->tr_gbps.empty()) c->tr_t0.store(mono_ns());
    while (n_done < n_reqs && hard == CAKE_OK) {
        uint64_t now = ex.now();
        if (P >= 0 && !loader_started && reqs[P].arrival_ns <= now) {
            c->load_thread.submit([&] { ex.worker(W_LOAD, be); });
            loader_started = true;
        }
        // The prefix-cached request's KV is complete as soon as nothing is left to claim and the loader's
        // last chunk has landed.  Looked at before every step, not only when the engine is idle: its
        // first-token step is priority 1 and must go into this very step even while other requests keep
        // the budget busy.
        if (P >= 0 && loader_started && !kv_complete[P]) {
            std::lock_guard<std::mutex> g(ex.mu);
            if (ex.core.range_empty() && !ex.core.w[W_LOAD].busy && ex.first_error == CAKE_OK) {
                uint64_t end = prefix_compute_end;
                for (int i = 0; i < nc; ++i) if (ex.chunk_log[i].source == CAKE_SRC_LOAD) end = std::max(end, ex.chunk_log[i].end_ns);
                finish_kv(P, end, &n_done);
                if (n_done >= n_reqs) break;
            }
        }
        // ---- deal the budget out: (1) decoding requests, one token each: here the first-token step
        // of a request whose KV is complete; (2) prefill of requests without a stored prefix, oldest
        // first; (3) the rest to the prefix-cached request, as far as the plan gives it to the compute side
        parts.clear();
        int left = token_budget, np_tokens = 0, first_np = -1, bg_tokens = 0, dec_tokens = 0;
        if (!c->tr_other.empty()) {
            bg_tokens = std::min(left, c->tr_other[size_t(n_steps) % c->tr_other.size()]);
            if (bg_tokens > 0) parts.push_back({-1, 0, bg_tokens, false});
            left -= bg_tokens;
        }
        for (int k = 0; k < n_reqs && left > 0; ++k) {
            int i = order[k];
            if (!ft_pending[i]) continue;
            parts.push_back({i, reqs[i].n_tokens - 1, 1, true});
            left -= 1; ++dec_tokens;
        }
        for (int k = 0; k < n_reqs && left > 0; ++k) {
            int i = order[k];
            if (i == P || done[i] || kv_complete[i] || reqs[i].arrival_ns > now) continue;
            int nt = std::min(left, reqs[i].n_tokens - next_tok[i]);
            parts.push_back({i, next_tok[i], nt, false});
            if (first_np < 0) first_np = i;
            left -= nt; np_tokens += nt;
        }
        int got = 0, first = -1;
        const bool prefix_live = P >= 0 && !kv_complete[P] && reqs[P].arrival_ns <= now;
        if (prefix_live) {
            std::lock_guard<std::mutex> g(ex.mu);
            // no budget left for the request: the plan must know that its compute side is not coming soon
            if (left <= 0 && !ex.core.starved) { ex.core.starved = true; ex.core.starved_since = now; }
            if (left > 0) ex.core.starved = false;
            if (left > 0) {
                ex.refresh_load_progress(be);
                got = ex.core.claim_front(now, left, &first);
                if (got > 0) { ++ex.gen; ex.cv.notify_all(); }
            }
        }
        if (got > 0) parts.push_back({P, first, got, false});

        const bool only_background = parts.size() == 1 && parts[0].req == -1;
        bool prefix_finished_by_loader = false;
        if (parts.empty() || only_background) {
            std::unique_lock<std::mutex> lk(ex.mu);
            prefix_finished_by_loader = prefix_live && ex.core.range_empty() && !ex.core.w[W_LOAD].busy;
        }
        if (parts.empty() || (only_background && prefix_finished_by_loader)) {
            // idle: the prefix request may be finished by the loader, or nothing has arrived yet
            std::unique_lock<std::mutex> lk(ex.mu);
            if (prefix_live && ex.core.range_empty() && !ex.core.w[W_LOAD].busy) {
                uint64_t end = prefix_compute_end;
                for (int i = 0; i < nc; ++i) if (ex.chunk_log[i].source == CAKE_SRC_LOAD) end = std::max(end, ex.chunk_log[i].end_ns);
                finish_kv(P, end, &n_done);
                continue;
            }
            if (ex.first_error != CAKE_OK) { hard = ex.first_error; break; }
            uint64_t wake = ~uint64_t(0);
            for (int i = 0; i < n_reqs; ++i)
                if (!done[i] && reqs[i].arrival_ns > now) wake = std::min(wake, reqs[i].arrival_ns);
            const uint64_t seen = ex.gen;
            if (wake == ~uint64_t(0)) ex.cv.wait(lk, [&] { return ex.gen != seen || ex.first_error != CAKE_OK; });
            else ex.cv.wait_for(lk, std::chrono::nanoseconds(wake - now), [&] { return ex.gen != seen || ex.first_error != CAKE_OK; });
            continue;
        }
        // ---- run the step
        const uint64_t t_start = ex.now();
        for (const Part& p : parts) {
            const int32_t* ids = p.req < 0 ? c->tr_ids.data() : reqs[p.req].token_ids + p.first;
            const cake_kv* pkv = p.req < 0 ? &c->tr_kv : reqs[p.req].kv;
            if (hipMemcpyAsync(c->d_ids + p.first, ids, size_t(p.count) * 4, hipMemcpyHostToDevice, c->cs) != hipSuccess) { hard = CAKE_E_HIP; break; }
            int rc = p.decode ? enqueue_first_token(c, reqs[p.req].n_tokens, pkv) : enqueue_prefill(c, p.first, p.count, pkv);
            if (rc != CAKE_OK) { hard = rc; break; }
            // the token leaves the device before the next decode part overwrites it (one stream)
            if (p.decode && hipMemcpyAsync(&ft_tok[p.req], c->t_tok, 4, hipMemcpyDeviceToHost, c->cs) != hipSuccess) { hard = CAKE_E_HIP; break; }
        }
        if (hard == CAKE_OK && hipStreamSynchronize(c->cs) != hipSuccess) hard = fail(c, CAKE_E_HIP, "compute stream failed in an adaptive step");
        const uint64_t t_end = ex.now();
        if (hard != CAKE_OK) break;
        for (const Part& p : parts) {
            if (p.decode) {   // the first token is out: the request leaves
                reqs[p.req].first_token = ft_tok[p.req];
                reqs[p.req].ttft_ns = t_end - reqs[p.req].arrival_ns;
                ft_pending[p.req] = 0;
                done[p.req] = 1; ++n_done;
                continue;
            }
            if (p.req == P || p.req < 0) continue;
            next_tok[p.req] += p.count;
            reqs[p.req].tokens_computed += p.count;
            if (next_tok[p.req] == reqs[p.req].n_tokens) finish_kv(p.req, t_end, &n_done);
        }
        if (prefix_live) {
            std::lock_guard<std::mutex> g(ex.mu);
            if (got > 0) {
                // the sample spans the steps since the request last got tokens: the rate it actually gets
                ex.core.complete_front(t_end - t_start + starved_ns, cake::range_flops(c->m, first, got));
                starved_ns = 0;
                reqs[P].tokens_computed += got;
                prefix_compute_end = t_end;
                // chunks the compute side has now finished
                for (int i = 0; i < nc; ++i) {
                    if (ex.chunk_log[i].source != CAKE_SRC_NONE) continue;
                    const bool finished = i < ex.core.f;
                    if (!finished) break;
                    cake_chunk_log& cl = ex.chunk_log[i];
                    cl.source = CAKE_SRC_COMPUTE; cl.tok_begin = tb[i]; cl.tok_count = tc[i];
                    cl.start_ns = t_start; cl.end_ns = t_end; cl.work = flops[i]; cl.device_ns = 0;
                    c->status[i].store(CAKE_CHUNK_RESIDENT);
                }
            } else {
                starved_ns += t_end - t_start;   // a step the prefix request got nothing of
            }
            ++ex.gen;
            ex.cv.notify_all();
        }
        if (steps) {
            if (n_steps < steps_cap) {
                cake_step_log& sl = steps[n_steps];
                sl.start_ns = now; sl.end_ns = t_end; sl.decode_tokens = dec_tokens; sl.nonprefix_tokens = np_tokens;
                sl.prefix_tokens = got; sl.prefix_tok_begin = got > 0 ? first : -1; sl.first_nonprefix_req = first_np; sl.other_tokens = bg_tokens;
            } else steps_overflow = true;
        }
        ++n_steps;
    }
    if (hard != CAKE_OK) {
        std::lock_guard<std::mutex> g(ex.mu);
        if (ex.first_error == CAKE_OK) ex.first_error = hard;
        ++ex.gen;
        ex.cv.notify_all();
    }
    if (loader_started) c->load_thread.wait();
    if (hard == CAKE_OK && ex.first_error != CAKE_OK) hard = ex.first_error;
    (void)hipStreamSynchronize(c->cs);
    c->step_after = -1;

    res->n_chunks = nc;
    res->n_decisions = ex.core.log_n;
    res->load_failed_chunk = ex.load_failed_chunk;
    res->ttft_ns = P >= 0 ? reqs[P].ttft_ns : 0;
    res->meet_point = 0;
    res->compute_busy_ns = res->compute_device_ns = res->compute_flops = res->load_busy_ns = res->load_bytes = 0;
    for (int i = 0; i < nc; ++i) {
        const cake_chunk_log& cl = ex.chunk_log[i];
        if (cl.source == CAKE_SRC_COMPUTE) { ++res->meet_point; res->compute_flops += cl.work; }
        else if (cl.source == CAKE_SRC_LOAD) {
            res->load_busy_ns += cl.end_ns - cl.start_ns; res->load_bytes += cl.work;
            reqs[P].tokens_loaded += tc[i];
        }
        if (res->chunks && i < res->chunks_cap) res->chunks[i] = cl;
    }
    c->tr_t0.store(0);   // traces apply to one run
    c->tr_other.clear(); c->tr_ids.clear(); c->tr_gbps.clear(); c->tr_interval_ns = 0;
    if (n_steps_out) *n_steps_out = std::min(n_steps, steps ? steps_cap : n_steps);
    if (hard != CAKE_OK) {
        if (c->err.empty()) fail(c, hard, "adaptive run ended with status %d", hard);
        return hard;
    }
    if ((res->chunks && res->chunks_cap < nc) || ex.core.log_overflow || steps_overflow) return CAKE_E_CAPACITY;
    return CAKE_OK;
}

int32_t cake_set_bandwidth(cake_ctx* c, double gbps) {
    if (!c || !(gbps > 0)) return CAKE_E_INVAL;
    c->gbps.store(gbps);
    return CAKE_OK;
}

int32_t cake_schedule_bandwidth_step(cake_ctx* c, int32_t after_loaded_chunks, double gbps) {
    if (!c) return CAKE_E_INVAL;
    if (after_loaded_chunks < 0) { c->step_after = -1; return CAKE_OK; }
    if (!(gbps > 0)) return CAKE_E_INVAL;
    c->step_after = after_loaded_chunks;
    c->step_gbps = gbps;
    return CAKE_OK;
}

int32_t cake_chunk_state(const cake_ctx* c, int32_t chunk) {
    if (!c || chunk < 0 || chunk >= c->n_status) return CAKE_E_INVAL;
    return c->status[chunk].load();
}

int32_t cake_sync_compute(cake_ctx* c) {
    if (!c) return CAKE_E_INVAL;
    HIP_TRY(c, hipStreamSynchronize(c->cs));
    return CAKE_OK;
}

int32_t cake_sync_load(cake_ctx* c) {
    if (!c) return CAKE_E_INVAL;
    c->load_thread.wait();                      // every queued load has issued its last piece
    HIP_TRY(c, hipStreamSynchronize(c->ls));    // ... and the pieces have landed
    return c->async_load_rc.exchange(CAKE_OK);  // first failure of a queued load since the last call (text in cake_last_error)
}

int32_t cake_profile_enable(cake_ctx* c, int32_t on) {
    if (!c) return CAKE_E_INVAL;
    HIP_TRY(c, hipStreamSynchronize(c->cs));
    c->prof_on = on != 0;
    c->prof_mask = on > 1 ? uint32_t(on) >> 1 : 0xffffffffu;
    c->prof_recs.clear();
    return CAKE_OK;
}

int32_t cake_profile_read(cake_ctx* c, cake_kernel_stats* out) {
    if (!c || !out) return CAKE_E_INVAL;
    HIP_TRY(c, hipStreamSynchronize(c->cs));
    for (int k = 0; k < CAKE_K_COUNT; ++k) out[k] = cake_kernel_stats{0, 0, 0, 0};
    for (size_t i = 0; i < c->prof_recs.size(); ++i) {
        float ms = 0.f;
        HIP_TRY(c, hipEventElapsedTime(&ms, c->prof_events[2 * i], c->prof_events[2 * i + 1]));
        cake_kernel_stats& s = out[c->prof_recs[i].cls];
        s.launches += 1;
        s.total_ns += uint64_t(double(ms) * 1e6);
        s.flops += c->prof_recs[i].flops;
        s.bytes += c->prof_recs[i].bytes;
    }
    c->prof_recs.clear();
    return CAKE_OK;
}

// ---- single kernels -------------------------------------------------------------------
int32_t cake_op_rmsnorm(cake_ctx* c, const float* x, const float* gain, void* out, int32_t rows, int32_t cols) {
    if (!c || !x || !gain || !out || rows < 0 || cols <= 0) return CAKE_E_INVAL;
    HIP_TRY(c, launch_rmsnorm(c->m.dtype, x, gain, out, rows, cols, c->m.rms_eps, c->cs));
    return CAKE_OK;
}

int32_t cake_op_gemm(cake_ctx* c, const void* a, const void* w, float* out, int32_t M, int32_t N, int32_t K) {
    if (!c || !a || !w || !out || M < 0 || N <= 0 || K <= 0 || (K & 7)) return CAKE_E_INVAL;
    HIP_TRY(c, gemm(c, EPI_STORE_F32, a, w, nullptr, out, M, N, K));
    return CAKE_OK;
}

int32_t cake_op_gemm_residual(cake_ctx* c, const void* a, const void* w, float* x, int32_t M, int32_t N, int32_t K) {
    if (!c || !a || !w || !x || M < 0 || N <= 0 || K <= 0 || (K & 7)) return CAKE_E_INVAL;
    HIP_TRY(c, gemm(c, EPI_RESIDUAL_F32, a, w, nullptr, x, M, N, K));
    return CAKE_OK;
}

int32_t cake_op_gemm_plan(cake_ctx* c, int32_t residual, int32_t M, int32_t N, int32_t K, int32_t tile[2], int32_t* ksplit) {
    if (!c || !tile || !ksplit || M < 0 || N <= 0 || K <= 0) return CAKE_E_INVAL;
    const int epi = residual ? EPI_RESIDUAL_F32 : EPI_STORE_F32;
    tile[0] = tile[1] = 0; *ksplit = 1;
    if (c->m.dtype == CAKE_BF16 && c->tun.kernel_path == 0 && gemm_mfma_supported(epi, M, N, K)) {
        int bm, bn, ks;
        gemm_mfma_plan(epi, M, N, K, c->tun.gemm_config - 1, c->split.part ? &c->split : nullptr, c->tun.gemm_ksplit, &bm, &bn, &ks);
        tile[0] = bm; tile[1] = bn; *ksplit = ks;
    }
    return CAKE_OK;
}

int32_t cake_op_mfma_rate(cake_ctx* c, int32_t workgroups, int32_t iters, double* tflops) {
    if (!c || !tflops || workgroups <= 0 || workgroups > 65536 || iters <= 0 || iters > (1 << 22)) return CAKE_E_INVAL;
    // one float per wave, written into the float32 qkv workspace (at least max_chunk * 3 * head_dim floats)
    const size_t room = size_t(c->max_chunk) * size_t(c->m.n_q_heads + 2 * c->m.n_kv_heads) * c->m.head_dim;
    if (size_t(workgroups) * 8 > room) return fail(c, CAKE_E_INVAL, "mfma_rate: %d workgroups need %zu floats of workspace", workgroups, size_t(workgroups) * 8);
    HIP_TRY(c, launch_mfma_rate(c->qkv, workgroups, std::max(1, iters / 8), c->cs));   // clocks up
    HIP_TRY(c, hipEventRecord(c->ev_a, c->cs));
    HIP_TRY(c, launch_mfma_rate(c->qkv, workgroups, iters, c->cs));
    HIP_TRY(c, hipEventRecord(c->ev_b, c->cs));
    HIP_TRY(c, hipStreamSynchronize(c->cs));
    float ms = 0.f;
    HIP_TRY(c, hipEventElapsedTime(&ms, c->ev_a, c->ev_b));
    *tflops = ms > 0.f ? double(workgroups) * 8.0 * iters * 8.0 * 32768.0 / (double(ms) * 1e-3) / 1e12 : 0.0;
    return CAKE_OK;
}

int32_t cake_device_info(cake_ctx* c, int32_t* compute_units, int32_t* clock_khz, uint64_t* hbm_bytes) {
    if (!c) return CAKE_E_INVAL;
    int v = 0;
    if (compute_units) {
        HIP_TRY(c, hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, c->device));
        *compute_units = v;
    }
    if (clock_khz) {
        HIP_TRY(c, hipDeviceGetAttribute(&v, hipDeviceAttributeClockRate, c->device));
        *clock_khz = v;
    }
    if (hbm_bytes) {
        size_t free_b = 0, total_b = 0;
        HIP_TRY(c, hipMemGetInfo(&free_b, &total_b));
        *hbm_bytes = total_b;
    }
    return CAKE_OK;
}

int32_t cake_op_gemm_swiglu(cake_ctx* c, const void* a, const void* wg, const void* wu, void* out, int32_t M,
                            int32_t N, int32_t K) {
    if (!c || !a || !wg || !wu || !out || M < 0 || N <= 0 || K <= 0 || (K & 7)) return CAKE_E_INVAL;
    HIP_TRY(c, gemm(c, EPI_SWIGLU, a, wg, wu, out, M, N, K));
    return CAKE_OK;
}

int32_t cake_op_rope_kv_write(cake_ctx* c, const float* qkv, void* q, int32_t layer, int32_t tok_begin, int32_t rows,
                              const cake_kv* kv) {
    if (!c || !qkv || !q || layer < 0 || layer >= c->m.n_layers || tok_begin < 0 || rows < 0 || rows > c->max_chunk)
        return CAKE_E_INVAL;
    int rc = check_kv(c, kv, tok_begin + rows);
    if (rc != CAKE_OK) return rc;
    HIP_TRY(c, launch_rope_table(c->rope_cs, tok_begin, rows, c->m.head_dim, c->m.rope_theta, c->cs));
    HIP_TRY(c, launch_rope_kv_write(c->m.dtype, qkv, c->rope_cs, q, c->m.n_q_heads, tok_begin, rows, make_view(c, kv, layer), c->cs));
    return CAKE_OK;
}

int32_t cake_op_attention(cake_ctx* c, const void* q, void* out, int32_t layer, int32_t tok_begin, int32_t rows,
                          const cake_kv* kv) {
    if (!c || !q || !out || layer < 0 || layer >= c->m.n_layers || tok_begin < 0 || rows < 0) return CAKE_E_INVAL;
    int rc = check_kv(c, kv, tok_begin + rows);
    if (rc != CAKE_OK) return rc;
    HIP_TRY(c, attention(c, q, out, tok_begin, rows, make_view(c, kv, layer)));
    return CAKE_OK;
}

int32_t cake_op_decode_attention(cake_ctx* c, const float* q, float* out, int32_t layer, int32_t n_keys, const cake_kv* kv) {
    if (!c || !q || !out || layer < 0 || layer >= c->m.n_layers || n_keys <= 0 || n_keys > c->max_tokens)
        return fail(c, CAKE_E_INVAL, "op_decode_attention: bad argument");
    if (!c->t_part) return fail(c, CAKE_E_STATE, "the context was created without final_norm / lm_head");
    int rc = check_kv(c, kv, n_keys);
    if (rc != CAKE_OK) return rc;
    HIP_TRY(c, launch_decode_attention(c->m.dtype, q, out, c->t_part, c->m.n_q_heads, n_keys, make_view(c, kv, layer), c->cs,
                                       c->tun.kernel_path == 1));
    return CAKE_OK;
}

int32_t cake_op_decode_attention_static(cake_ctx* c, const float* q, float* out, int32_t layer, int32_t n_keys,
                                        const cake_kv* kv) {
    if (!c || !q || !out || layer < 0 || layer >= c->m.n_layers || n_keys <= 0 || n_keys > c->max_tokens)
        return fail(c, CAKE_E_INVAL, "op_decode_attention_static: bad argument");
    const size_t need = decode_attention_workspace_bytes(c->m.n_q_heads, c->m.head_dim);
    if (need > STATIC_SCRATCH_BYTES)
        return fail(c, CAKE_E_INVAL, "op_decode_attention_static: %d query heads of head dimension %d need %zu bytes of "
                    "partial results, the static buffer holds %zu (64 heads of 128)", c->m.n_q_heads, c->m.head_dim, need,
                    STATIC_SCRATCH_BYTES);
    if (!c->static_scratch) return fail(c, CAKE_E_STATE, "op_decode_attention_static: no static buffer on this device");
    int rc = check_kv(c, kv, n_keys);
    if (rc != CAKE_OK) return rc;
    // every key range that the combine kernel reads is written by this launch first: nothing needs clearing
    HIP_TRY(c, launch_decode_attention(c->m.dtype, q, out, (float*)c->static_scratch, c->m.n_q_heads, n_keys,
                                       make_view(c, kv, layer), c->cs, c->tun.kernel_path == 1));
    return CAKE_OK;
}

}  // extern "C"
