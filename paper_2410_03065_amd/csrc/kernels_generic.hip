// Generic device kernels: embedding gather, RMSNorm, rotary + KV page write, a plain
// LDS-tiled GEMM and a plain chunk-vs-prefix attention.  They accept float32 and bf16
// element types and any supported shape; float32 models run on them entirely, bf16
// models use them for the element-wise steps (the contractions go to the MFMA kernels).
//
// Operations follow the decoder block the benchmark shapes name (the paper, Sec. 3,
// states only Q = X W_Q, K = X W_K, V = X W_V and softmax(Q K^T / sqrt(d_k)) V):
// pre-RMSNorm, rotary embedding on adjacent pairs, grouped-query attention, SwiGLU.
#include "kernels.hpp"

namespace cake {

template <typename T> __device__ __forceinline__ float to_f(T v);
template <> __device__ __forceinline__ float to_f<float>(float v) { return v; }
template <> __device__ __forceinline__ float to_f<bf16_t>(bf16_t v) { return float(v); }
template <typename T> __device__ __forceinline__ T from_f(float v);
template <> __device__ __forceinline__ float from_f<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16_t from_f<bf16_t>(float v) { return bf16_t(v); }

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

// ------------------------------------------------------------------ embedding
template <typename T>
__global__ void __launch_bounds__(256) embed_kernel(const T* __restrict__ table, const int32_t* __restrict__ ids,
                                                    float* __restrict__ x, int d, int vocab) {
    int row = blockIdx.x;
    int id = ids[row];
    id = id < 0 ? 0 : (id >= vocab ? vocab - 1 : id);
    const T* src = table + size_t(id) * d;
    float* dst = x + size_t(row) * d;
    for (int c = threadIdx.x; c < d; c += 256) dst[c] = to_f<T>(src[c]);
}

hipError_t launch_embed(int dtype, const void* table, const int32_t* ids, float* x, int rows, int d,
                        int vocab, hipStream_t st) {
    if (rows <= 0) return hipSuccess;
    if (dtype == 0) hipLaunchKernelGGL(embed_kernel<float>, dim3(rows), dim3(256), 0, st, (const float*)table, ids, x, d, vocab);
    else hipLaunchKernelGGL(embed_kernel<bf16_t>, dim3(rows), dim3(256), 0, st, (const bf16_t*)table, ids, x, d, vocab);
    return hipGetLastError();
}

// ------------------------------------------------------------------ RMSNorm
// y = x / sqrt(mean(x^2) + eps) * gain ; one 256-thread block per row.
template <typename T>
__global__ void __launch_bounds__(256) rmsnorm_kernel(const float* __restrict__ x, const float* __restrict__ gain,
                                                      T* __restrict__ out, int d, float eps) {
    __shared__ float part[4];
    const float* xr = x + size_t(blockIdx.x) * d;
    float s = 0.f;
    for (int c = threadIdx.x; c < d; c += 256) { float v = xr[c]; s += v * v; }
    s = wave_sum(s);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = s;
    __syncthreads();
    float tot = part[0] + part[1] + part[2] + part[3];
    float r = 1.0f / sqrtf(tot / float(d) + eps);
    T* o = out + size_t(blockIdx.x) * d;
    for (int c = threadIdx.x; c < d; c += 256) o[c] = from_f<T>(xr[c] * r * gain[c]);
}

// Rows whose length is a multiple of 1024: every thread keeps its NV float4 pieces of the row in
// registers (one 16-byte load each, all in flight together), so the row is read once.
template <typename T, int NV>
__global__ void __launch_bounds__(256) rmsnorm_vec_kernel(const float* __restrict__ x, const float* __restrict__ gain,
                                                          T* __restrict__ out, float eps) {
    __shared__ float part[4];
    constexpr int d = NV * 1024;
    const float4* xr = (const float4*)(x + size_t(blockIdx.x) * d);
    float4 v[NV];
#pragma unroll
    for (int i = 0; i < NV; ++i) v[i] = xr[threadIdx.x + 256 * i];
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < NV; ++i) s += v[i].x * v[i].x + v[i].y * v[i].y + v[i].z * v[i].z + v[i].w * v[i].w;
    s = wave_sum(s);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = s;
    __syncthreads();
    const float tot = part[0] + part[1] + part[2] + part[3];
    const float r = 1.0f / sqrtf(tot / float(d) + eps);
    T* o = out + size_t(blockIdx.x) * d;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int c4 = threadIdx.x + 256 * i;
        const float4 g = ((const float4*)gain)[c4];
        const float y0 = v[i].x * r * g.x, y1 = v[i].y * r * g.y, y2 = v[i].z * r * g.z, y3 = v[i].w * r * g.w;
        if constexpr (sizeof(T) == 4) {
            ((float4*)o)[c4] = make_float4(y0, y1, y2, y3);
        } else {
            typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4_t;
            bf16x4_t w = {from_f<T>(y0), from_f<T>(y1), from_f<T>(y2), from_f<T>(y3)};
            ((bf16x4_t*)o)[c4] = w;
        }
    }
}

template <typename T>
static bool launch_rmsnorm_vec(const float* x, const float* gain, T* out, int rows, int d, float eps, hipStream_t st) {
    if (d % 1024 != 0 || d > 8192 || ((uintptr_t(x) | uintptr_t(gain) | uintptr_t(out)) & 15)) return false;
    switch (d / 1024) {
#define CAKE_RMS_CASE(NV) \
    case NV: hipLaunchKernelGGL((rmsnorm_vec_kernel<T, NV>), dim3(rows), dim3(256), 0, st, x, gain, out, eps); return true;
        CAKE_RMS_CASE(1) CAKE_RMS_CASE(2) CAKE_RMS_CASE(3) CAKE_RMS_CASE(4) CAKE_RMS_CASE(5) CAKE_RMS_CASE(6) CAKE_RMS_CASE(7)
        CAKE_RMS_CASE(8)
#undef CAKE_RMS_CASE
    }
    return false;
}

hipError_t launch_rmsnorm(int dtype, const float* x, const float* gain, void* out, int rows, int d, float eps,
                          hipStream_t st) {
    if (rows <= 0) return hipSuccess;
    if (dtype == 0 ? launch_rmsnorm_vec(x, gain, (float*)out, rows, d, eps, st)
                   : launch_rmsnorm_vec(x, gain, (bf16_t*)out, rows, d, eps, st))
        return hipGetLastError();
    if (dtype == 0) hipLaunchKernelGGL(rmsnorm_kernel<float>, dim3(rows), dim3(256), 0, st, x, gain, (float*)out, d, eps);
    else hipLaunchKernelGGL(rmsnorm_kernel<bf16_t>, dim3(rows), dim3(256), 0, st, x, gain, (bf16_t*)out, d, eps);
    return hipGetLastError();
}

// ------------------------------------------------------------------ rotary table
// cs[row][pair] = (cos, sin) of (tok_begin + row) * theta^(-2*pair/head_dim).  The angle is
// formed in double precision: at position 65535 a float32 angle is off by ~4e-3 rad.
__global__ void rope_table_kernel(float2* __restrict__ cs, int tok_begin, int rows, int half, double log2_theta) {
    int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= rows * half) return;
    int row = idx / half, pair = idx % half;
    double inv_freq = exp2(-(double(pair) / double(half)) * log2_theta);
    double ang = double(tok_begin + row) * inv_freq;
    double s, c;
    sincos(ang, &s, &c);
    cs[idx] = make_float2(float(c), float(s));
}

hipError_t launch_rope_table(float* cs, int tok_begin, int rows, int head_dim, float theta, hipStream_t st) {
    if (rows <= 0) return hipSuccess;
    int half = head_dim / 2, n = rows * half;
    hipLaunchKernelGGL(rope_table_kernel, dim3((n + 255) / 256), dim3(256), 0, st, (float2*)cs, tok_begin, rows, half,
                       log2(double(theta)));
    return hipGetLastError();
}

// ------------------------------------------------------------------ rotary + KV page write
// grid.x: 64-token tiles aligned to absolute token index (so a tile never straddles a page);
// grid.y: head index in [0, n_q + 2 n_kv): query heads, then key heads, then value heads.
// K/V slots of the last tile that lie past the range are zeroed: attention reads whole
// 64-key tiles and masks by position, and 0 * NaN from stale memory would poison P V.
template <typename T, int HD>
__global__ void __launch_bounds__(256)
rope_kv_write_kernel(const float* __restrict__ qkv, const float2* __restrict__ cs, T* __restrict__ q, int n_q,
                     int tok_begin, int rows, KvView kv) {
    constexpr int HALF = HD / 2;
    __shared__ T vt[64][HD + 2];
    const int n_kv = kv.n_kv;
    const int ldq = (n_q + 2 * n_kv) * HD;
    const int head = blockIdx.y;
    const int tile_tok0 = (tok_begin / 64 + blockIdx.x) * 64;  // absolute
    const int lo = max(tile_tok0, tok_begin), hi = min(tile_tok0 + 64, tok_begin + rows);
    if (lo >= hi) return;
    const int lpage = tile_tok0 / kv.page_tokens;
    const int ppage = kv.block_table[lpage];
    const int in_page0 = tile_tok0 - lpage * kv.page_tokens;
    T* page = (T*)kv.pool + (size_t(kv.layer) * kv.n_physical_pages + ppage) * kv.page_elems();

    if (head < n_q + n_kv) {
        const bool is_q = head < n_q;
        for (int idx = threadIdx.x; idx < 64 * HALF; idx += 256) {
            int t = idx / HALF, pair = idx % HALF;
            int tok = tile_tok0 + t;
            if (tok < lo) continue;
            T* kdst = page + (size_t(head - n_q) * kv.page_tokens + in_page0 + t) * HD + 2 * pair;
            if (tok >= hi) {  // slots of this tile past the range: keep them finite for masked reads
                if (!is_q) { kdst[0] = from_f<T>(0.f); kdst[1] = from_f<T>(0.f); }
                continue;
            }
            int row = tok - tok_begin;
            float2 v = *(const float2*)(qkv + size_t(row) * ldq + head * HD + 2 * pair);
            float2 c = cs[row * HALF + pair];
            float o0 = v.x * c.x - v.y * c.y;
            float o1 = v.x * c.y + v.y * c.x;
            T* dst = is_q ? q + (size_t(head) * rows + row) * HD + 2 * pair : kdst;
            dst[0] = from_f<T>(o0);
            dst[1] = from_f<T>(o1);
        }
    } else {
        const int g = head - n_q - n_kv;
        for (int idx = threadIdx.x; idx < 64 * HD; idx += 256) {
            int t = idx / HD, e = idx % HD;
            int tok = tile_tok0 + t;
            float v = (tok >= lo && tok < hi) ? qkv[size_t(tok - tok_begin) * ldq + head * HD + e] : 0.f;
            vt[t][e] = from_f<T>(v);
        }
        __syncthreads();
        T* vpage = page + size_t(n_kv) * kv.page_tokens * HD + size_t(g) * HD * kv.page_tokens;
        for (int idx = threadIdx.x; idx < 64 * HD; idx += 256) {
            int e = idx / 64, t = idx % 64;
            int tok = tile_tok0 + t;
            if (tok >= lo) vpage[size_t(e) * kv.page_tokens + in_page0 + t] = vt[t][e];  // zeros past the range
        }
    }
}

// bf16, head_dim 128: same grid and semantics as above with 16-byte loads (4 consecutive elements =
// 2 rotary pairs per thread, 32 threads per token row) and 8-byte stores; V^T leaves the LDS
// transpose as 16-byte pieces of 8 consecutive tokens.
__global__ void __launch_bounds__(256)
rope_kv_write_bf16_hd128_kernel(const float* __restrict__ qkv, const float2* __restrict__ cs, bf16_t* __restrict__ q,
                                int n_q, int tok_begin, int rows, KvView kv) {
    constexpr int HD = 128, HALF = 64;
    typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4_t;
    typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
    __shared__ bf16_t vt[64][HD + 2];
    const int n_kv = kv.n_kv;
    const int ldq = (n_q + 2 * n_kv) * HD;
    const int head = blockIdx.y;
    const int tile_tok0 = (tok_begin / 64 + blockIdx.x) * 64;  // absolute
    const int lo = max(tile_tok0, tok_begin), hi = min(tile_tok0 + 64, tok_begin + rows);
    if (lo >= hi) return;
    const int lpage = tile_tok0 / kv.page_tokens;
    const int ppage = kv.block_table[lpage];
    const int in_page0 = tile_tok0 - lpage * kv.page_tokens;
    bf16_t* page = (bf16_t*)kv.pool + (size_t(kv.layer) * kv.n_physical_pages + ppage) * kv.page_elems();
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;   // 4 elements of a row; 8 rows per pass

    if (head < n_q + n_kv) {
        const bool is_q = head < n_q;
#pragma unroll
        for (int pass = 0; pass < 8; ++pass) {
            const int t = ty + 8 * pass, tok = tile_tok0 + t;
            if (tok < lo) continue;
            bf16_t* kdst = page + (size_t(head - n_q) * kv.page_tokens + in_page0 + t) * HD + 4 * tx;
            if (tok >= hi) {  // slots of this tile past the range: keep them finite for masked reads
                if (!is_q) *(bf16x4_t*)kdst = bf16x4_t{0, 0, 0, 0};
                continue;
            }
            const int row = tok - tok_begin;
            const float4 v = *(const float4*)(qkv + size_t(row) * ldq + head * HD + 4 * tx);
            const float4 c = *(const float4*)(cs + row * HALF + 2 * tx);   // (cos, sin) of pairs 2tx, 2tx+1
            bf16x4_t w = {bf16_t(v.x * c.x - v.y * c.y), bf16_t(v.x * c.y + v.y * c.x),
                          bf16_t(v.z * c.z - v.w * c.w), bf16_t(v.z * c.w + v.w * c.z)};
            bf16_t* dst = is_q ? q + (size_t(head) * rows + row) * HD + 4 * tx : kdst;
            *(bf16x4_t*)dst = w;
        }
    } else {
        const int g = head - n_q - n_kv;
#pragma unroll
        for (int pass = 0; pass < 8; ++pass) {
            const int t = ty + 8 * pass, tok = tile_tok0 + t;
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (tok >= lo && tok < hi) v = *(const float4*)(qkv + size_t(tok - tok_begin) * ldq + head * HD + 4 * tx);
            vt[t][4 * tx + 0] = bf16_t(v.x); vt[t][4 * tx + 1] = bf16_t(v.y);
            vt[t][4 * tx + 2] = bf16_t(v.z); vt[t][4 * tx + 3] = bf16_t(v.w);
        }
        __syncthreads();
        bf16_t* vpage = page + size_t(n_kv) * kv.page_tokens * HD + size_t(g) * HD * kv.page_tokens;
        // 128 rows (head-dim index) x 8 pieces of 8 tokens = 1024 pieces, 4 per thread
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int piece = threadIdx.x + 256 * i, e = piece >> 3, t0 = (piece & 7) * 8;
            bf16x8_t w;
#pragma unroll
            for (int k = 0; k < 8; ++k) w[k] = vt[t0 + k][e];
            bf16_t* dst = vpage + size_t(e) * kv.page_tokens + in_page0 + t0;
            if (tile_tok0 + t0 >= lo) {
                *(bf16x8_t*)dst = w;   // zeros past the range
            } else {                   // tokens before the range belong to an earlier call: leave them
#pragma unroll
                for (int k = 0; k < 8; ++k)
                    if (tile_tok0 + t0 + k >= lo) dst[k] = w[k];
            }
        }
    }
}

hipError_t launch_rope_kv_write(int dtype, const float* qkv, const float* cs, void* q, int n_q, int tok_begin,
                                int rows, const KvView& kv, hipStream_t st) {
    if (rows <= 0) return hipSuccess;
    int tiles = (tok_begin + rows - 1) / 64 - tok_begin / 64 + 1;
    dim3 grid(tiles, n_q + 2 * kv.n_kv), block(256);
    const float2* c2 = (const float2*)cs;
    const bool aligned = ((uintptr_t(qkv) | uintptr_t(cs) | uintptr_t(q) | uintptr_t(kv.pool)) & 15) == 0;
    if (dtype == 1 && kv.head_dim == 128 && aligned) {
        hipLaunchKernelGGL(rope_kv_write_bf16_hd128_kernel, grid, block, 0, st, qkv, c2, (bf16_t*)q, n_q, tok_begin, rows, kv);
        return hipGetLastError();
    }
    if (dtype == 0 && kv.head_dim == 64)
        hipLaunchKernelGGL((rope_kv_write_kernel<float, 64>), grid, block, 0, st, qkv, c2, (float*)q, n_q, tok_begin, rows, kv);
    else if (dtype == 0 && kv.head_dim == 128)
        hipLaunchKernelGGL((rope_kv_write_kernel<float, 128>), grid, block, 0, st, qkv, c2, (float*)q, n_q, tok_begin, rows, kv);
    else if (dtype == 1 && kv.head_dim == 64)
        hipLaunchKernelGGL((rope_kv_write_kernel<bf16_t, 64>), grid, block, 0, st, qkv, c2, (bf16_t*)q, n_q, tok_begin, rows, kv);
    else if (dtype == 1 && kv.head_dim == 128)
        hipLaunchKernelGGL((rope_kv_write_kernel<bf16_t, 128>), grid, block, 0, st, qkv, c2, (bf16_t*)q, n_q, tok_begin, rows, kv);
    else
        return hipErrorInvalidValue;
    return hipGetLastError();
}

// ------------------------------------------------------------------ plain GEMM
// out[M][N] = a[M][K] * w[N][K]^T with float32 accumulation.  64x64 tile, 16-deep slices
// through LDS, 4x4 outputs per thread.  K must be a multiple of 4.
template <typename T> struct Vec4;
template <> struct Vec4<float> { typedef float4 type; };
template <> struct Vec4<bf16_t> { typedef uint2 type; };

template <typename T>
__device__ __forceinline__ void load4(const T* p, float* o);
template <>
__device__ __forceinline__ void load4<float>(const float* p, float* o) {
    float4 v = *(const float4*)p;
    o[0] = v.x; o[1] = v.y; o[2] = v.z; o[3] = v.w;
}
template <>
__device__ __forceinline__ void load4<bf16_t>(const bf16_t* p, float* o) {
    uint2 v = *(const uint2*)p;
    o[0] = __uint_as_float(v.x << 16); o[1] = __uint_as_float(v.x & 0xFFFF0000u);
    o[2] = __uint_as_float(v.y << 16); o[3] = __uint_as_float(v.y & 0xFFFF0000u);
}

template <typename T, int EPI>
__global__ void __launch_bounds__(256)
gemm_generic_kernel(const T* __restrict__ a, const T* __restrict__ w, const T* __restrict__ w2, void* __restrict__ outv,
                    int M, int N, int K) {
    constexpr int BK = 16;
    __shared__ float As[BK][64 + 4];
    __shared__ float Ws[BK][64 + 4];
    __shared__ float W2s[EPI == EPI_SWIGLU ? BK : 1][64 + 4];
    const int tid = threadIdx.x;
    const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
    const int lr = tid >> 2, lk = (tid & 3) * 4;
    const int arow = min(m0 + lr, M - 1), wrow = min(n0 + lr, N - 1);
    const int ty = tid >> 4, tx = tid & 15;
    float acc[4][4] = {}, acc2[4][4] = {};
    for (int k0 = 0; k0 < K; k0 += BK) {
        float va[4] = {0, 0, 0, 0}, vw[4] = {0, 0, 0, 0}, vw2[4] = {0, 0, 0, 0};
        if (k0 + lk < K) {
            load4<T>(a + size_t(arow) * K + k0 + lk, va);
            load4<T>(w + size_t(wrow) * K + k0 + lk, vw);
            if (EPI == EPI_SWIGLU) load4<T>(w2 + size_t(wrow) * K + k0 + lk, vw2);
        }
        __syncthreads();
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            As[lk + i][lr] = va[i];
            Ws[lk + i][lr] = vw[i];
            if (EPI == EPI_SWIGLU) W2s[lk + i][lr] = vw2[i];
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < BK; ++k) {
            float ar[4], wr[4], w2r[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                ar[i] = As[k][ty * 4 + i];
                wr[i] = Ws[k][tx * 4 + i];
                if (EPI == EPI_SWIGLU) w2r[i] = W2s[k][tx * 4 + i];
            }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    acc[i][j] = fmaf(ar[i], wr[j], acc[i][j]);
                    if (EPI == EPI_SWIGLU) acc2[i][j] = fmaf(ar[i], w2r[j], acc2[i][j]);
                }
        }
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        int row = m0 + ty * 4 + i;
        if (row >= M) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            int col = n0 + tx * 4 + j;
            if (col >= N) continue;
            size_t o = size_t(row) * N + col;
            if (EPI == EPI_STORE_F32) ((float*)outv)[o] = acc[i][j];
            else if (EPI == EPI_RESIDUAL_F32) ((float*)outv)[o] += acc[i][j];
            else {
                float g = acc[i][j];
                ((T*)outv)[o] = from_f<T>(g / (1.0f + expf(-g)) * acc2[i][j]);
            }
        }
    }
}

template <typename T>
static hipError_t gemm_generic_t(int epi, const void* a, const void* w, const void* w2, void* out, int M, int N, int K,
                                 hipStream_t st) {
    dim3 grid((N + 63) / 64, (M + 63) / 64), block(256);
    const T *A = (const T*)a, *W = (const T*)w, *W2 = (const T*)w2;
    if (epi == EPI_STORE_F32) hipLaunchKernelGGL((gemm_generic_kernel<T, EPI_STORE_F32>), grid, block, 0, st, A, W, W2, out, M, N, K);
    else if (epi == EPI_RESIDUAL_F32) hipLaunchKernelGGL((gemm_generic_kernel<T, EPI_RESIDUAL_F32>), grid, block, 0, st, A, W, W2, out, M, N, K);
    else if (epi == EPI_SWIGLU) hipLaunchKernelGGL((gemm_generic_kernel<T, EPI_SWIGLU>), grid, block, 0, st, A, W, W2, out, M, N, K);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

hipError_t launch_gemm_generic(int dtype, int epi, const void* a, const void* w, const void* w2, void* out, int M,
                               int N, int K, hipStream_t st) {
    if (M <= 0 || N <= 0) return hipSuccess;
    if (K <= 0 || (K & 3)) return hipErrorInvalidValue;
    return dtype == 0 ? gemm_generic_t<float>(epi, a, w, w2, out, M, N, K, st)
                      : gemm_generic_t<bf16_t>(epi, a, w, w2, out, M, N, K, st);
}

// ------------------------------------------------------------------ plain attention
// One wavefront per (query row, query head).  Keys are visited in groups of 64 (one key per
// lane for the scores); the running max / sum of the online softmax are wave-uniform; each
// lane owns HD/64 output dimensions for the P V accumulation.
template <typename T, int HD>
__global__ void __launch_bounds__(64)
attention_generic_kernel(const T* __restrict__ q, T* __restrict__ out, int n_q, int tok_begin, int rows, KvView kv) {
    constexpr int EPL = HD / 64;  // output dims per lane
    const int row = blockIdx.x, h = blockIdx.y, lane = threadIdx.x;
    const int g = h / (n_q / kv.n_kv);
    const int qpos = tok_begin + row;
    const float scale = 1.0f / sqrtf(float(HD));
    float qr[HD];
    const T* qp = q + (size_t(h) * rows + row) * HD;
#pragma unroll
    for (int e = 0; e < HD; ++e) qr[e] = to_f<T>(qp[e]) * scale;
    float m_run = -INFINITY, l_run = 0.f, o[EPL];
#pragma unroll
    for (int i = 0; i < EPL; ++i) o[i] = 0.f;
    const int n_groups = qpos / 64 + 1;
    const int pt = kv.page_tokens;
    for (int grp = 0; grp < n_groups; ++grp) {
        const int key0 = grp * 64;
        const int lpage = key0 / pt;
        const int in_page0 = key0 - lpage * pt;
        const T* page = (const T*)kv.pool + (size_t(kv.layer) * kv.n_physical_pages + kv.block_table[lpage]) * kv.page_elems();
        const T* kp = page + (size_t(g) * pt + in_page0 + lane) * HD;
        const T* vp = page + size_t(kv.n_kv) * pt * HD + size_t(g) * HD * pt + in_page0;
        float s = -INFINITY;
        if (key0 + lane <= qpos) {
            float acc = 0.f;
#pragma unroll
            for (int e = 0; e < HD; ++e) acc = fmaf(qr[e], to_f<T>(kp[e]), acc);
            s = acc;
        }
        float m_new = fmaxf(m_run, wave_max(s));
        float p = (key0 + lane <= qpos) ? expf(s - m_new) : 0.f;
        float corr = expf(m_run - m_new);
        l_run = l_run * corr + wave_sum(p);
        m_run = m_new;
        const int n_valid = min(64, qpos - key0 + 1);
#pragma unroll
        for (int i = 0; i < EPL; ++i) {
            const T* vrow = vp + size_t(lane + 64 * i) * pt;
            float acc = o[i] * corr;
            for (int j = 0; j < n_valid; ++j) acc = fmaf(__shfl(p, j, 64), to_f<T>(vrow[j]), acc);
            o[i] = acc;
        }
    }
    T* op = out + size_t(row) * n_q * HD + h * HD;
#pragma unroll
    for (int i = 0; i < EPL; ++i) op[lane + 64 * i] = from_f<T>(o[i] / l_run);
}

hipError_t launch_attention_generic(int dtype, const void* q, void* out, int n_q, int tok_begin, int rows,
                                    const KvView& kv, hipStream_t st) {
    if (rows <= 0) return hipSuccess;
    dim3 grid(rows, n_q), block(64);
    if (dtype == 0 && kv.head_dim == 64)
        hipLaunchKernelGGL((attention_generic_kernel<float, 64>), grid, block, 0, st, (const float*)q, (float*)out, n_q, tok_begin, rows, kv);
    else if (dtype == 0 && kv.head_dim == 128)
        hipLaunchKernelGGL((attention_generic_kernel<float, 128>), grid, block, 0, st, (const float*)q, (float*)out, n_q, tok_begin, rows, kv);
    else if (dtype == 1 && kv.head_dim == 64)
        hipLaunchKernelGGL((attention_generic_kernel<bf16_t, 64>), grid, block, 0, st, (const bf16_t*)q, (bf16_t*)out, n_q, tok_begin, rows, kv);
    else if (dtype == 1 && kv.head_dim == 128)
        hipLaunchKernelGGL((attention_generic_kernel<bf16_t, 128>), grid, block, 0, st, (const bf16_t*)q, (bf16_t*)out, n_q, tok_begin, rows, kv);
    else
        return hipErrorInvalidValue;
    return hipGetLastError();
}

}  // namespace cake
