// Launchers of the device kernels.  Every launcher enqueues on `st` and returns the
// hipError_t of the launch.  Shapes are validated by the callers in cake_api.hip.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace cake {

typedef __bf16 bf16_t;

// Where a layer's K and V live: see the pool layout in cake.h.
struct KvView {
    void* pool;
    const int32_t* block_table;  // device
    int32_t page_tokens;
    int32_t n_physical_pages;
    int32_t n_kv;
    int32_t head_dim;
    int32_t layer;
    // elements per (layer, page): 2 * n_kv * page_tokens * head_dim
    __host__ __device__ size_t page_elems() const { return size_t(2) * n_kv * page_tokens * head_dim; }
};

enum GemmEpilogue { EPI_STORE_F32 = 0, EPI_RESIDUAL_F32 = 1, EPI_SWIGLU = 2 };

// ---- generic kernels (any supported shape; the only path for float32 models) ----
hipError_t launch_embed(int dtype, const void* table, const int32_t* ids, float* x, int rows,
                        int d, int vocab, hipStream_t st);
hipError_t launch_rmsnorm(int dtype, const float* x, const float* gain, void* out, int rows, int d,
                          float eps, hipStream_t st);
hipError_t launch_rope_table(float* cs, int tok_begin, int rows, int head_dim, float theta,
                             hipStream_t st);
hipError_t launch_rope_kv_write(int dtype, const float* qkv, const float* cs, void* q, int n_q,
                                int tok_begin, int rows, const KvView& kv, hipStream_t st);
hipError_t launch_gemm_generic(int dtype, int epi, const void* a, const void* w, const void* w2,
                               void* out, int M, int N, int K, hipStream_t st);
hipError_t launch_attention_generic(int dtype, const void* q, void* out, int n_q, int tok_begin,
                                    int rows, const KvView& kv, hipStream_t st);

// ---- MFMA kernels (bf16) ----
bool gemm_mfma_supported(int epi, int M, int N, int K);
// Workspace of the split-K GEMMs: float32 parts of the tiles in flight, and one ticket counter per
// tile (zero between launches: the kernel puts it back).  Launches sharing it must not overlap.
struct GemmSplitWs {
    float* part;
    size_t part_bytes;
    unsigned* counters;
    int n_counters;
};
// cfg_override: -1 = choose the tile configuration from the shape; 0..5 = force one, unsplit (testing).
// ws: nullptr = never split K.  ksplit_override: 0 = by the cost model, 1 = never, 2/4/8 = that
// many K ranges wherever the shape and the workspace allow it.
hipError_t launch_gemm_mfma(int epi, const void* a, const void* w, const void* w2, void* out,
                            int M, int N, int K, hipStream_t st, int cfg_override = -1,
                            const GemmSplitWs* ws = nullptr, int ksplit_override = 0);
// What launch_gemm_mfma would launch: tile rows / columns and K ranges per tile.
void gemm_mfma_plan(int epi, int M, int N, int K, int cfg_override, const GemmSplitWs* ws, int ksplit_override,
                    int* bm, int* bn, int* ksplit);
// MFMA-only yardstick kernel: out holds workgroups * 8 floats; see kernels_gemm.hip.
hipError_t launch_mfma_rate(float* out, int workgroups, int iters, hipStream_t st);
bool attention_mfma_supported(int head_dim, int page_tokens);
// variant: 0 = eight-wave kernel, 128 or 64 queries per workgroup by grid size; 1 = four-wave kernel;
// 2 / 3 = eight-wave kernel with 128 / 64 queries per workgroup (testing).
hipError_t launch_attention_mfma(const void* q, void* out, int n_q, int tok_begin, int rows,
                                 const KvView& kv, hipStream_t st, int variant = 0);

bool decode_attention_mfma_supported(int dtype, int head_dim, int page_tokens, int r);
hipError_t launch_decode_attention_mfma(const float* q, float* part, int n_q, int n_keys, int tiles_per_split,
                                        int n_splits, const KvView& kv, hipStream_t st);

// ---- quantised stored KV (bits = 8 or 4): one page image (all layers) <-> the layer pages of physical page phys_page ----
hipError_t launch_dequant_page(int dtype, const void* image, const KvView& kv, int phys_page, int n_layers, int bits,
                               hipStream_t st);
hipError_t launch_quant_page(int dtype, void* image, const KvView& kv, int phys_page, int n_layers, int bits,
                             hipStream_t st);

// ---- first-token step (one row of activations: matrix-vector products, one-token attention) ----
// out[n] (mode 0: =, 1: +=) sum_k x[k] w[n][k]; mode 2: out[n] = silu(x.w[n]) * (x.w2[n]).  x, out float32.
hipError_t launch_gemv(int dtype, int mode, const float* x, const void* w, const void* w2, float* out,
                       int N, int K, hipStream_t st);
hipError_t launch_rope_token(const float* qin, float* qout, int n_heads, int head_dim, int pos,
                             float theta, hipStream_t st);
size_t decode_attention_workspace_bytes(int n_q, int head_dim);
// generic_only: keep to the vector-ALU kernel (testing)
hipError_t launch_decode_attention(int dtype, const float* q, float* out, float* part, int n_q,
                                   int n_keys, const KvView& kv, hipStream_t st, bool generic_only = false);
hipError_t launch_argmax(const float* v, int n, int32_t* result, hipStream_t st);

}  // namespace cake
