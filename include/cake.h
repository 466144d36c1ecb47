/*
 * cake.h -- C ABI of the bidirectional KV-cache producer for one long prompt.
 *
 * Method: "Compute Or Load KV Cache? Why not Both?" (the Cake paper).  The KV
 * cache of a prompt whose KV is already held by a slow storage tier is
 * produced from both ends at once (Sec. 4 Part 2; App. A; Alg. 1): the GPU
 * prefills chunks front-to-back, each chunk attending to all earlier KV
 * (Sec. 3 "Chunk Prefill"), while stored chunks are fetched back-to-front at
 * the tier's bandwidth (Sec. 5.1 "I/O Bandwidth Control"), until the two
 * sweeps meet.  Where they meet is planned from measured per-chunk costs:
 * compute cost grows with position, load cost is flat (Sec. 4 Part 2
 * "Insight").
 *
 * Conventions
 *  - Every call returns 0 (CAKE_OK) or a negative cake_status.  Nothing is
 *    thrown across this boundary.  cake_last_error() gives the text of the
 *    last failure on a context (owned by the context, valid until the next
 *    failing call on it).
 *  - "host" / "device" / "pinned host" is stated for every pointer.  The
 *    caller owns weights, token ids, the KV pool, the block tables, the store
 *    and both streams; the library borrows them (cake_create: until
 *    cake_destroy; other calls: until the call returns, or for async calls
 *    until the stream work they queued has finished).  The library owns only
 *    what sits inside cake_ctx (activation workspace, events, a device copy of
 *    the token ids).  No call allocates memory the caller must free.
 *  - Streams are hipStream_t passed as void*.  All device pointers belong to
 *    the device that was current when cake_create ran.
 *  - 1 GB/s = 1e9 bytes per second.  Times are integer nanoseconds.
 *
 * Matrix layout.  Every projection matrix is stored [out_features][in_features]
 * row-major (the transpose of the paper's W in Q = X W_Q), in the model's
 * element type.  Norm gains are float32 [d_model].
 *
 * KV layout.  Tokens are grouped into logical pages of page_tokens tokens
 * (a multiple of 64).  block_table[logical_page] names the physical page.
 * Device pool, element type = model dtype:
 *     pool[layer][physical_page][0][kv_head][token_in_page][head_dim]   K (rotated)
 *     pool[layer][physical_page][1][kv_head][head_dim][token_in_page]   V (transposed)
 * The storage tier holds one image per logical page,
 *     image[layer][0|1][...as above...],   at base + logical_page * page_stride_bytes,
 * so loading a page is n_layers contiguous copies and the bytes land exactly
 * as stored.  A store may instead hold 8-bit images (cake_store_format), sit
 * in a file rather than in pinned memory (cake_store_source), and cover only
 * a prefix of the prompt (cake_kv_store.n_pages).
 */
#ifndef CAKE_H
#define CAKE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct cake_ctx cake_ctx;

typedef enum {
    CAKE_OK = 0,
    CAKE_E_INVAL = -1,      /* bad argument; nothing was enqueued */
    CAKE_E_NOMEM = -2,      /* workspace allocation failed (cake_create only) */
    CAKE_E_HIP = -3,        /* a HIP runtime call failed */
    CAKE_E_STORE_MISS = -4, /* the store does not hold the requested page */
    CAKE_E_STATE = -5,      /* call order violated (e.g. earlier KV not resident) */
    CAKE_E_CAPACITY = -6    /* a caller-provided log array was too small (result still valid) */
} cake_status;

typedef enum { CAKE_F32 = 0, CAKE_BF16 = 1 } cake_dtype;

typedef enum {
    CAKE_BIDIR = 0,        /* planned race from both ends (the method) */
    CAKE_COMPUTE_ONLY = 1, /* baseline: prefill every chunk (Sec. 5.1 "Baselines") */
    CAKE_LOAD_ONLY = 2,    /* baseline: load every chunk */
    CAKE_FORCED_SPLIT = 3, /* chunks [0,forced_m) computed, [forced_m,N) loaded */
    CAKE_GREEDY = 4        /* Alg. 1 without a plan: both sides claim whenever free */
} cake_mode;

typedef enum { CAKE_SRC_NONE = -1, CAKE_SRC_COMPUTE = 0, CAKE_SRC_LOAD = 1 } cake_source;

typedef enum {
    CAKE_CHUNK_EMPTY = 0, CAKE_CHUNK_COMPUTING = 1, CAKE_CHUNK_LOADING = 2, CAKE_CHUNK_RESIDENT = 3
} cake_chunk_status;

/* Llama-style decoder shape (pre-RMSNorm, rotary q/k with adjacent-pair rotation,
 * grouped-query attention, SwiGLU, no biases).  head_dim must be 64 or 128. */
typedef struct {
    int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, ffn_dim, vocab;
    int32_t dtype;          /* cake_dtype: element type of weights, activations fed to GEMMs, and KV */
    float rms_eps;
    float rope_theta;
} cake_model_desc;

typedef struct {
    const float* attn_norm; /* device, [d_model] */
    const void* wqkv;       /* device, [(n_q+2*n_kv)*head_dim][d_model]: W_Q rows, then W_K, then W_V */
    const void* wo;         /* device, [d_model][n_q*head_dim] */
    const float* ffn_norm;  /* device, [d_model] */
    const void* w_gate;     /* device, [ffn_dim][d_model] */
    const void* w_up;       /* device, [ffn_dim][d_model] */
    const void* w_down;     /* device, [d_model][ffn_dim] */
} cake_layer_weights;

typedef struct {
    const void* embed;                /* device, [vocab][d_model] */
    const cake_layer_weights* layers; /* host array of n_layers structs (copied by cake_create) */
    const float* final_norm;          /* device, [d_model]; NULL if cake_first_token is not used */
    const void* lm_head;              /* device, [vocab][d_model]; NULL likewise */
} cake_weights;

typedef struct {
    void* pool;                      /* device, layout above */
    const int32_t* block_table_host; /* host,   [n_logical_pages] */
    const int32_t* block_table_dev;  /* device, same contents */
    int32_t page_tokens;             /* multiple of 64 */
    int32_t n_physical_pages;        /* pages per layer in the pool */
    int32_t n_logical_pages;
} cake_kv;

/* How a store holds a page.  CAKE_STORE_RAW: the page's bytes as they are in HBM (layout above).
 * CAKE_STORE_INT8 (Sec. 5.5: compressed KV combined with the method): per layer and per K|V,
 *   int8 codes [kv_head][token][head_dim] then float32 scales [kv_head][token];
 *   value = code * scale, one scale per token and KV head (absmax / 127), V not transposed.
 *   n_layers*2*n_kv*page_tokens*(head_dim+4) bytes per page.  Loaded pages are dequantised on
 *   arrival (float32 product, rounded once to the KV element type).
 * CAKE_STORE_INT4 (the stronger compression level of Sec. 5.5 / Table 6; the paper's own 3-bit scheme
 *   needs calibration data and is not reproduced): as CAKE_STORE_INT8 with 15 levels, absmax / 7,
 *   codes in [-7, 7] as 4-bit two's complement, two per byte (element 2i low nibble, 2i+1 high
 *   nibble): uint8 [kv_head][token][head_dim/2] then the float32 scales;
 *   n_layers*2*n_kv*page_tokens*(head_dim/2+4) bytes per page. */
typedef enum { CAKE_STORE_RAW = 0, CAKE_STORE_INT8 = 1, CAKE_STORE_INT4 = 2 } cake_store_format;

/* Where a store's bytes are.  CAKE_STORE_PINNED: pinned host memory at `base` (one hop, DMA reads it
 * directly).  CAKE_STORE_FILE: a file open for reading (`fd`, page p at file_offset + p * stride):
 * the load worker preads each piece into one of two pinned staging buffers and the DMA out of one
 * runs while the other is filled (the paper's second hop: storage -> CPU memory -> GPU). */
typedef enum { CAKE_STORE_PINNED = 0, CAKE_STORE_FILE = 1 } cake_store_source;

typedef struct {
    const void* base;           /* CAKE_STORE_PINNED: pinned host; else ignored */
    uint64_t page_stride_bytes; /* >= the page image size of `format` */
    int32_t page_tokens;        /* must equal cake_kv.page_tokens */
    int32_t n_pages;            /* logical pages held, from page 0: the stored prefix.  It may be shorter
                                   than the prompt: chunks not wholly inside it are computed after the
                                   race over the stored part has ended (App. A step 2: total_tokens) */
    int32_t format;             /* cake_store_format */
    int32_t source;             /* cake_store_source */
    int32_t fd;                 /* CAKE_STORE_FILE: descriptor, stays the caller's */
    int32_t pad_;
    uint64_t file_offset;       /* CAKE_STORE_FILE: byte offset of page 0 */
} cake_kv_store;

/* One record per chunk, indexed by chunk number. */
typedef struct {
    int32_t source;     /* cake_source */
    int32_t tok_begin, tok_count;
    uint64_t start_ns, end_ns; /* since the call started; end = KV of the chunk resident */
    uint64_t work;             /* compute: algorithmic FLOPs of the chunk; load: bytes */
    uint64_t device_ns;        /* compute: HIP-event time of the chunk's kernels; load: 0 */
} cake_chunk_log;

/* One record per look at the unclaimed range [f,b] by a free worker.  The
 * estimates the planner used are reproducible from these integers:
 *   compute estimate of chunk i = floor(flops_i * est_compute_ns / est_compute_flops)
 *   load estimate of chunk j    = floor(bytes_j * est_load_ns    / est_load_bytes)
 * (est_load_*: the last loaded chunk, or the progress of the chunk in flight once its first piece
 * has been released, or the prior; with progress known, o_l = floor(bytes left * ns / bytes done)). */
typedef struct {
    int32_t who;     /* cake_source of the worker */
    int32_t f, b;    /* unclaimed chunks before the decision */
    int32_t m_star;  /* planned meet point (absolute chunk index) */
    int32_t claimed; /* chunk claimed, or -1 (wait) */
    int32_t f_off;   /* tokens of chunk f already claimed by compute before this look (0 unless steps are
                        smaller than a chunk); when > 0 chunk f is compute's and the plan covers [f+1, b]
                        with partial_ns added to the compute offset */
    int32_t claimed_tokens; /* tokens this claim covers (0 on a wait; 0 from cake_simulate_race, which has no
                               token ranges): a compute step may span several chunks when the chunks are
                               fetch units smaller than the step, starting at token f_off of chunk `claimed` */
    int32_t pad_;
    uint64_t now_ns;
    uint64_t o_c, o_l;                            /* predicted remaining ns of the work in flight on each side; o_c in the
                                                     adaptive mode while higher priorities leave the request none of the step
                                                     budget: the ns it has gone without tokens so far (expected to last as
                                                     long again) */
    uint64_t est_compute_ns, est_compute_flops;   /* throughput sample: last <= 4 computed chunks, or the prior */
    uint64_t est_load_ns, est_load_bytes;         /* last loaded chunk, or the prior */
    uint64_t partial_ns;                          /* estimate of the unclaimed rest of chunk f when f_off > 0, else 0 */
} cake_decision_log;

typedef struct {
    /* in: capacities of the two caller-provided arrays (may be 0 / NULL) */
    cake_chunk_log* chunks;
    int32_t chunks_cap;
    cake_decision_log* decisions;
    int32_t decisions_cap;
    /* out */
    int32_t n_chunks;
    int32_t n_decisions;       /* number recorded (<= cap) */
    int32_t meet_point;        /* chunks [0,meet_point) were computed, chunks [meet_point, stored_chunks) loaded */
    int32_t load_failed_chunk; /* -1, or the chunk whose load failed and was recomputed */
    uint64_t ttft_ns;          /* entry -> every chunk's KV resident */
    uint64_t compute_busy_ns;  /* sum of computed chunks' wall times */
    uint64_t compute_device_ns;/* sum of computed chunks' HIP-event times */
    uint64_t compute_flops;    /* algorithmic FLOPs of the computed chunks */
    uint64_t load_busy_ns;
    uint64_t load_bytes;
    int32_t stored_chunks;     /* chunks wholly inside the stored prefix (= n_chunks when the store covers the
                                  prompt); chunks [stored_chunks, n_chunks) were computed after the race */
    int32_t pad_;
} cake_result;

/* Priors used before the first measurement, and pacing granularity. 0 = default. */
typedef struct {
    uint64_t prior_compute_ns, prior_compute_flops; /* default 1e9 ns per 5e14 FLOP */
    uint64_t piece_bytes;                           /* largest single DMA; default 4 MiB */
    int32_t kernel_path; /* 0: MFMA kernels where the shape allows (bf16); 1: generic kernels only */
    int32_t gemm_config; /* 0: tile shape chosen per GEMM; 1..7: force 256x256 / 256x128 / 128x128 / 128x192 / 128x64 /
                            128x128 with the waves dividing K / the persistent four-wave 256x256 kernel (testing) */
    int32_t attn_variant; /* 0: eight-wave attention kernel, 128 or 64 queries per workgroup by grid size;
                             1: four-wave kernel; 2 / 3: eight-wave with 128 / 64 queries (testing) */
    int32_t gemm_ksplit; /* 0: K of the residual / plain GEMMs split over 2, 4 or 8 workgroups per tile where a cost
                            model says so (few large tiles); 1: never; 2 / 4 / 8: that many wherever legal (testing) */
} cake_tuning;

/* ---- life cycle ------------------------------------------------------- */

/* Creates a context on the current device: copies the layer table, allocates the
 * activation workspace for chunks of up to max_chunk tokens, a device buffer for
 * max_tokens token ids and the staging of the load path (device room for the 8-bit page
 * images of max_chunk tokens; two pinned buffers of one DMA piece for file-backed stores),
 * and starts the load worker.  Loads allocate nothing; a page of more than max_chunk tokens
 * cannot be loaded from a quantised store.  compute_stream / copy_stream: hipStream_t, default priority.
 * Errors: CAKE_E_INVAL (shape not supported), CAKE_E_NOMEM, CAKE_E_HIP. */
int32_t cake_create(cake_ctx** out, const cake_model_desc* model, const cake_weights* weights,
                    int32_t max_tokens, int32_t max_chunk, void* compute_stream, void* copy_stream);
int32_t cake_destroy(cake_ctx* ctx);
const char* cake_last_error(const cake_ctx* ctx);
int32_t cake_set_tuning(cake_ctx* ctx, const cake_tuning* t);

/* ---- the four calls of the method ------------------------------------- */

/* Sec. 3 "Chunk Prefill"; App. A step 4.  Enqueues, on the compute stream, the prefill of
 * tokens [tok_begin, tok_begin+tok_count) through every layer: their K/V are written into
 * kv's pages and they attend to the pages of [0, tok_begin+tok_count).  Asynchronous.
 * token_ids: host, the whole prompt (indexed absolutely).  tok_count <= max_chunk.
 * The KV of [0,tok_begin) must be resident before the stream reaches this work; the
 * library cannot check data it did not produce, the caller orders it.
 * Errors: CAKE_E_INVAL (range outside the block table / max_chunk), CAKE_E_HIP. */
int32_t cake_prefill_chunk(cake_ctx* ctx, const int32_t* token_ids, int32_t tok_begin,
                           int32_t tok_count, const cake_kv* kv);

/* Sec. 5.1 "I/O Bandwidth Control"; App. A step 5.  Copies the stored images of the logical
 * pages covering [tok_begin, tok_begin+tok_count) into their physical pages on the copy
 * stream, in pieces, releasing a piece only once the tier would have delivered it at `gbps`
 * (cumulative bytes issued <= gbps * elapsed).  Asynchronous: the arguments are checked, the
 * range is handed to the context's load worker (a thread that lives with the context) and the
 * call returns; the worker paces the pieces onto the copy stream.  Ranges queued by several
 * calls are loaded in call order.  The chunk is resident once cake_sync_load has returned
 * CAKE_OK; a failure that only shows while loading (a short read from a file-backed store) is
 * returned by that cake_sync_load.  The two descriptor structs are copied; the store's bytes,
 * the pool and the host block table stay borrowed until cake_sync_load returns.
 * tok_begin must be page aligned.  gbps <= 0 means unthrottled.  Nothing is allocated.
 * Errors (all before anything is queued): CAKE_E_INVAL, CAKE_E_STORE_MISS (the store holds
 * fewer pages than the range needs). */
int32_t cake_load_chunk(cake_ctx* ctx, const cake_kv_store* store, int32_t tok_begin,
                        int32_t tok_count, const cake_kv* kv, double gbps);

/* Sec. 4 Part 3 ("always ensuring minimal latency").  Pure host function, no context.
 * Chunks [0,m) computed front-to-back, [m,n) loaded back-to-front:
 *   TTFT(m) = max(compute_offset_ns + sum_{i<m} compute_ns[i],
 *                 load_offset_ns    + sum_{j>=m} load_ns[j]),   m in 0..n.
 * Returns the smallest m minimising TTFT(m) and that TTFT.  O(n).
 * Errors: CAKE_E_INVAL (n < 0, NULL with n > 0, an offset above 2^62, or a running sum the
 * scan needs exceeding 2^63). */
int32_t cake_plan_meet_point(const uint64_t* compute_ns, const uint64_t* load_ns, int32_t n,
                             uint64_t compute_offset_ns, uint64_t load_offset_ns,
                             int32_t* m_out, uint64_t* ttft_ns_out);

/* App. A; Alg. 1.  Produces the KV of the whole prompt.  Blocking.  Splits n_tokens into
 * chunks of `chunk` tokens (a multiple of page_tokens; the last may be short), then runs a
 * compute worker (caller's thread, compute stream) from chunk 0 upward and a load worker
 * (own thread, copy stream) from the last chunk downward; each claims its end of the
 * unclaimed range under a lock after re-planning the meet point from measured costs, so no
 * chunk is produced twice.  Returns when both have drained; ttft_ns covers entry to that
 * point.  A failed load returns its chunk to the range, retires the loader and is reported
 * in load_failed_chunk (the call still succeeds if compute can finish the range).
 * If the store holds fewer pages than the prompt needs (the stored prefix found by
 * cake_prefix_lookup, App. A step 2), the race covers the chunks wholly inside the stored
 * prefix and the remaining chunks are computed afterwards; res->stored_chunks tells which.
 * Errors: CAKE_E_INVAL, CAKE_E_STORE_MISS (load-only mode and the store lacks a page),
 * CAKE_E_HIP, CAKE_E_CAPACITY (logs truncated; KV and scalars valid). */
int32_t cake_bidirectional_prefill(cake_ctx* ctx, const int32_t* token_ids, int32_t n_tokens,
                                   const cake_kv_store* store, int32_t chunk, double gbps,
                                   int32_t mode, int32_t forced_m, const cake_kv* kv,
                                   cake_result* res);

/* ---- adaptive scheduling (Sec. 4 Part 3; Sec. 5.7) ---------------------- */

/* One request of a serving mix.  in: prompt, arrival, its own KV pages, and for a prefix-cached
 * request the store that holds its KV.  out: when all of its KV was resident. */
typedef struct {
    const int32_t* token_ids;   /* host */
    int32_t n_tokens;
    int32_t has_prefix_cache;   /* 1: KV stored in `store`; produced by the bidirectional race */
    uint64_t arrival_ns;        /* after the start of the call */
    const cake_kv* kv;          /* this request's pages (block table + pool) */
    const cake_kv_store* store; /* prefix-cached requests only */
    uint64_t ttft_ns;           /* out: arrival -> all KV resident */
    int32_t tokens_computed;    /* out */
    int32_t tokens_loaded;      /* out */
    int32_t want_first_token;   /* 1: once the KV is complete the request takes one decode step (the first-token
                                   step of cake_first_token) in the next engine step, at priority 1; ttft_ns then
                                   runs to the end of that step.  Needs final_norm and lm_head in the weights */
    int32_t first_token;        /* out: that token, or -1 */
} cake_request;

/* One engine step: how the token budget was dealt out. */
typedef struct {
    uint64_t start_ns, end_ns;  /* start = the instant the budget was dealt (requests with arrival <= start count) */
    int32_t decode_tokens;      /* priority 1: first-token steps of requests whose KV is complete (want_first_token) */
    int32_t nonprefix_tokens;   /* priority 2 */
    int32_t prefix_tokens;      /* priority 3: what was left for the prefix-cached request */
    int32_t prefix_tok_begin;   /* first token of the prefix request's part, or -1 */
    int32_t first_nonprefix_req; /* index of the first non-prefix request served, or -1 */
    int32_t other_tokens;       /* taken off the top by the other-users trace (cake_set_traces), else 0 */
} cake_step_log;

/* Resource traces for the NEXT cake_adaptive_serve (copied; cleared when that call returns).
 * other_tokens: the paper's measure of GPU utilisation (Sec. 5.1 "GPU Resource Utilization"): at
 *   engine step k, other_tokens[k % n_other_tokens] tokens of the budget belong to other users
 *   and the requests of the call share the rest (budget 512, other 256 = 50 % utilisation).  The
 *   other users' share is really computed, as a prefill of that many of scratch_token_ids into
 *   scratch_kv (pages of the same layout holding >= n_scratch_tokens tokens), so it costs the
 *   GPU time it stands for.  Each entry <= n_scratch_tokens and <= the context's max_chunk.
 * gbps: the tier's bandwidth over time (Sec. 5.6): sample gbps[(t / gbps_interval_ns) % n_gbps],
 *   t since the call started, overrides the call's rate; samples below 0.01 GB/s count as 0.01.
 * A NULL pointer / zero length leaves that resource constant.  traces == NULL clears both.
 * Errors: CAKE_E_INVAL. */
typedef struct {
    const int32_t* other_tokens;
    int32_t n_other_tokens;
    int32_t n_scratch_tokens;
    const cake_kv* scratch_kv;
    const int32_t* scratch_token_ids; /* host */
    const double* gbps;
    int32_t n_gbps;
    int32_t pad_;
    uint64_t gbps_interval_ns;
} cake_traces;
int32_t cake_set_traces(cake_ctx* ctx, const cake_traces* traces);

/* Serves a mix of requests on one GPU with the paper's adaptive mode: every engine step fills a
 * budget of `token_budget` tokens in the order decoding requests, chunked prefill of requests
 * without a stored prefix (arrival order), chunked prefill of the prefix-cached request with
 * whatever budget is left; meanwhile that request's stored chunks of `fetch_chunk` tokens are
 * loaded back-to-front at `gbps` and the two meet where the planner says, re-planned at every
 * step from the rate the request actually gets.  At most one request may have has_prefix_cache.
 * Blocking; returns when every request's KV is resident (and its first token produced, where asked).  `res` describes the prefix request's
 * race (decision log included); `steps`/`n_steps_out` may be NULL.
 * Errors: CAKE_E_INVAL, CAKE_E_HIP, CAKE_E_STORE_MISS, CAKE_E_CAPACITY (logs truncated). */
int32_t cake_adaptive_serve(cake_ctx* ctx, cake_request* requests, int32_t n_requests,
                            int32_t token_budget, int32_t fetch_chunk, double gbps,
                            cake_result* res, cake_step_log* steps, int32_t steps_cap,
                            int32_t* n_steps_out);

/* First output token.  The paper measures the time to first token up to "the generation of the
 * first token" (Sec. 5.1, Metrics); once every chunk's KV is resident -- whichever side produced
 * it -- that token needs one more pass: the prompt's LAST token runs through the decoder against
 * the complete cache (which is read, never written: a loaded last chunk keeps its stored bytes),
 * then the final norm, the LM head and an argmax (lowest index among equal logits).
 * Requires KV of [0, n_tokens) resident in `kv` and a context created with final_norm and
 * lm_head.  token_ids: host, n_tokens ids (only the last is read).  token_out: host.
 * logits_out: host, vocab float32, or NULL.  device_ns_out: HIP-event time of the step, or NULL.
 * Blocking; runs on the compute stream.
 * Errors: CAKE_E_INVAL, CAKE_E_STATE (no head weights), CAKE_E_HIP. */
int32_t cake_first_token(cake_ctx* ctx, const int32_t* token_ids, int32_t n_tokens,
                         const cake_kv* kv, int32_t* token_out, float* logits_out,
                         uint64_t* device_ns_out);

/* Chunk-prefix keys (App. A step 2; App. B: the store hashes token chunks into keys).  One key per
 * FULL chunk of chunk_tokens ids; key i identifies the whole prefix [0, (i+1)*chunk_tokens):
 *   key_i = FNV-1a-64(8 bytes of key_{i-1}, little-endian, then the chunk's ids as little-endian
 *   32-bit integers), key_{-1} = the FNV offset basis 0xcbf29ce484222325.
 * Writes min(n_tokens / chunk_tokens, keys_cap) keys to keys_out (host) and returns
 * n_tokens / chunk_tokens, or CAKE_E_INVAL.  Pure; no context, no GPU. */
int32_t cake_prefix_keys(const int32_t* token_ids, int32_t n_tokens, int32_t chunk_tokens,
                         uint64_t* keys_out, int32_t keys_cap);
/* How many LEADING keys of `keys` occur in `stored_sorted` (ascending): the number of chunks of the
 * prompt whose KV the store holds (the paper's total_tokens / chunk).  A key found behind a
 * missing one does not count.  Returns the count, or CAKE_E_INVAL (also when not sorted). */
int32_t cake_prefix_lookup(const uint64_t* stored_sorted, int32_t n_stored, const uint64_t* keys,
                           int32_t n_keys);

/* Bytes of one page image in a store of `format`. */
uint64_t cake_store_image_bytes(const cake_model_desc* model, int32_t page_tokens, int32_t format);
/* Writes the pages that hold tokens [0, n_tokens) of `kv` into `dst` (pinned host, writable
 * despite the const base) in dst->format: CAKE_STORE_RAW copies, CAKE_STORE_INT8 / CAKE_STORE_INT4
 * quantise on the GPU (scale = absmax / 127 resp. / 7 per token and KV head, codes rounded half to
 * even).  Blocking.
 * Errors: CAKE_E_INVAL, CAKE_E_NOMEM (staging), CAKE_E_HIP. */
int32_t cake_write_store(cake_ctx* ctx, const cake_kv* kv, int32_t n_tokens, const cake_kv_store* dst);

/* ---- small helpers ---------------------------------------------------- */

/* Bandwidth of the simulated tier; thread-safe; takes effect at the next paced piece
 * (Sec. 5.6: the I/O rate fluctuates while a request is in flight).  gbps must be > 0. */
int32_t cake_set_bandwidth(cake_ctx* ctx, double gbps);
/* Schedules cake_set_bandwidth(gbps) to happen by itself when the load worker of the next
 * cake_bidirectional_prefill has completed `after_loaded_chunks` chunks (a count trigger, so
 * runs are repeatable).  after_loaded_chunks < 0 clears it. */
int32_t cake_schedule_bandwidth_step(cake_ctx* ctx, int32_t after_loaded_chunks, double gbps);
/* The paper's is_resident (App. B.2 step 4): cake_chunk_status of a chunk of the running or
 * last cake_bidirectional_prefill; negative cake_status on a bad index. */
int32_t cake_chunk_state(const cake_ctx* ctx, int32_t chunk);
/* Blocks until the compute stream has drained. */
int32_t cake_sync_compute(cake_ctx* ctx);
/* Blocks until every range queued by cake_load_chunk has been issued and the copy stream has
 * drained.  Returns the first failure of such a load since the previous call (CAKE_E_STORE_MISS,
 * CAKE_E_HIP; text in cake_last_error), else CAKE_OK. */
int32_t cake_sync_load(cake_ctx* ctx);

/* Algorithmic FLOPs of prefilling tokens [tok_begin, tok_begin+tok_count): projections
 * 2*P_lin*n plus causal attention n_layers*4*n_q*head_dim*(tok_begin*n + n(n+1)/2). */
uint64_t cake_range_flops(const cake_model_desc* model, int32_t tok_begin, int32_t tok_count);
/* Bytes of one page image (all layers, K and V). */
uint64_t cake_page_image_bytes(const cake_model_desc* model, int32_t page_tokens);

/* Virtual-time run of the claim protocol (the same decision code the threaded executor
 * uses), for host-side testing: chunk i costs actual_compute_ns[i] if computed and
 * actual_load_ns[i] if loaded; estimates follow the rules documented at
 * cake_decision_log with the given priors.  fail_load_chunk >= 0 makes that load fail.
 * sources_out[n]: cake_source per chunk.  decisions may be NULL.  No GPU involved. */
int32_t cake_simulate_race(int32_t n_chunks, const uint64_t* chunk_flops,
                           const uint64_t* chunk_bytes, const uint64_t* actual_compute_ns,
                           const uint64_t* actual_load_ns, uint64_t prior_compute_ns,
                           uint64_t prior_compute_flops, uint64_t prior_load_ns,
                           uint64_t prior_load_bytes, int32_t mode, int32_t forced_m,
                           int32_t fail_load_chunk, int32_t* sources_out, uint64_t* ttft_ns_out,
                           cake_decision_log* decisions, int32_t decisions_cap,
                           int32_t* n_decisions_out);

/* Per-kernel-class timing of the compute stream, for roofline reports.  While enabled, every
 * kernel launch of cake_prefill_chunk / cake_bidirectional_prefill is bracketed by a pair of
 * HIP events on the compute stream.  cake_profile_read drains the stream, adds the elapsed
 * times of all pairs recorded since the last read into `out[CAKE_K_COUNT]` (overwritten) and
 * forgets them.  flops / bytes are the algorithmic work of the launches (bytes: operands read
 * once + results written once).  cake_profile_enable: on = 0 stops, on = 1 brackets every class,
 * on = 2 * mask brackets only the classes whose bit (1 << class) is set in mask -- an event pair
 * costs a few microseconds of stream time, so timing one class perturbs a run about a tenth as
 * much as timing all of them (measured: 10 % against 1 % on a 1024-token chunk). */
typedef enum {
    CAKE_K_EMBED = 0, CAKE_K_RMSNORM = 1, CAKE_K_GEMM_QKV = 2, CAKE_K_ROPE_KV = 3, CAKE_K_ATTENTION = 4,
    CAKE_K_GEMM_O = 5, CAKE_K_GEMM_GATEUP = 6, CAKE_K_GEMM_DOWN = 7,
    CAKE_K_GEMV = 8,          /* first-token step: matrix-vector products (bytes = the weights streamed) */
    CAKE_K_DECODE_ATTN = 9,   /* first-token step: one-token attention (bytes = the layer's K and V) */
    CAKE_K_COUNT = 10
} cake_kernel_class;
typedef struct { uint64_t launches, total_ns, flops, bytes; } cake_kernel_stats;
int32_t cake_profile_enable(cake_ctx* ctx, int32_t on);
int32_t cake_profile_read(cake_ctx* ctx, cake_kernel_stats* out);

/* Single kernels, exposed for parity tests and profiling.  All asynchronous on the compute
 * stream; all pointers device; element type = the context's dtype unless stated. */
int32_t cake_op_rmsnorm(cake_ctx* ctx, const float* x, const float* gain, void* out,
                        int32_t rows, int32_t cols);
/* out[M][N] (float32) = a[M][K] * w[N][K]^T */
int32_t cake_op_gemm(cake_ctx* ctx, const void* a, const void* w, float* out,
                     int32_t M, int32_t N, int32_t K);
/* x[M][N] (float32) += a[M][K] * w[N][K]^T */
int32_t cake_op_gemm_residual(cake_ctx* ctx, const void* a, const void* w, float* x,
                              int32_t M, int32_t N, int32_t K);
/* Which kernel cake_op_gemm (residual = 0) or cake_op_gemm_residual (residual = 1) would launch for this
 * shape with the context's tuning: tile[0] x tile[1] = workgroup tile (0 x 0: the generic kernel), *ksplit =
 * K ranges per tile.  Host pointers; pure.  Errors: CAKE_E_INVAL. */
int32_t cake_op_gemm_plan(cake_ctx* ctx, int32_t residual, int32_t M, int32_t N, int32_t K,
                          int32_t tile[2], int32_t* ksplit);
/* Yardstick, not part of the method: `workgroups` workgroups of eight waves each run `iters` rounds of
 * eight independent bf16 MFMAs on register operands (no memory traffic); *tflops = what the matrix pipes
 * of this GPU delivered for that (host).  Blocking; uses the context's activation workspace.
 * Errors: CAKE_E_INVAL (sizes), CAKE_E_HIP. */
int32_t cake_op_mfma_rate(cake_ctx* ctx, int32_t workgroups, int32_t iters, double* tflops);
/* What the context's device reports (hipDeviceGetAttribute): *compute_units, *clock_khz = its peak engine
 * clock, *hbm_bytes = total device memory; the dense bf16 MFMA peak follows as compute_units x clock x 4096
 * FLOP (one 32x32x16 MFMA = 32768 FLOP in 32 clocks on each of 4 SIMDs).  Host pointers, any may be NULL;
 * pure.  Errors: CAKE_E_INVAL (ctx NULL), CAKE_E_HIP. */
int32_t cake_device_info(cake_ctx* ctx, int32_t* compute_units, int32_t* clock_khz, uint64_t* hbm_bytes);
/* out[M][N] = silu(a*wg^T) .* (a*wu^T), element type out */
int32_t cake_op_gemm_swiglu(cake_ctx* ctx, const void* a, const void* wg, const void* wu,
                            void* out, int32_t M, int32_t N, int32_t K);
/* q[n_q][rows][hd] from qkv[rows][(n_q+2n_kv)*hd] (float32) rotated at positions
 * tok_begin+row; K (rotated) and V written into layer `layer` of kv's pages. */
int32_t cake_op_rope_kv_write(cake_ctx* ctx, const float* qkv, void* q, int32_t layer,
                              int32_t tok_begin, int32_t rows, const cake_kv* kv);
/* out[rows][n_q*hd] = causal attention of q[n_q][rows][hd] (positions tok_begin+row)
 * against layer `layer` of kv's pages, keys 0 .. tok_begin+rows-1. */
int32_t cake_op_attention(cake_ctx* ctx, const void* q, void* out, int32_t layer,
                          int32_t tok_begin, int32_t rows, const cake_kv* kv);
/* out[n_q][hd] (float32) = attention of ONE query per head, q[n_q][hd] (float32, already rotated),
 * against keys 0 .. n_keys-1 of layer `layer` (the first-token step's attention).  Needs a
 * context created with head weights (it owns the split workspace). */
int32_t cake_op_decode_attention(cake_ctx* ctx, const float* q, float* out, int32_t layer,
                                 int32_t n_keys, const cake_kv* kv);
/* cake_op_decode_attention for callers that cannot allocate device memory (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): same arguments, same kernels and
 * the same result, but the per-key-range partial results go to a buffer that is part of the
 * library's image on each GPU (4 259 840 bytes, held until the process ends) instead of one that
 * cake_create allocated, so the call makes no hipMalloc / hipFree and works on a context created
 * without head weights.  Limit: n_q_heads * (head_dim + 2) <= 64 * 130, i.e. up to 64 query heads
 * of head dimension 128; a larger model is refused with CAKE_E_INVAL.  Every call on a GPU shares
 * that GPU's one buffer (each launch writes every entry it later reads, so nothing is cleared
 * between calls): calls that overlap on one GPU, from different streams or contexts, race.
 * Asynchronous on the compute stream.  Errors: CAKE_E_INVAL, CAKE_E_STATE, CAKE_E_HIP. */
int32_t cake_op_decode_attention_static(cake_ctx* ctx, const float* q, float* out, int32_t layer,
                                        int32_t n_keys, const cake_kv* kv);

#ifdef __cplusplus
}
#endif
#endif /* CAKE_H */
