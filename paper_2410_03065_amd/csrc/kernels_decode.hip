// Kernels of the first-token step: one token (the prompt's last) goes through the decoder against
// the complete KV cache, then final norm, LM head and argmax.  With one row of activations every
// projection is a matrix-vector product that streams its weights once, and attention streams the
// layer's K and V once: the whole step is bound by HBM bandwidth, so these kernels are built
// around wide coalesced loads and plain fp32 vector arithmetic (no MFMA: there is no reuse).
//
// The paper counts the time to first token up to "the generation of the first token" (Sec. 5.1,
// Metrics); the prefill it describes (Sec. 3) ends with that token's logits.
#include <algorithm>

#include "kernels.hpp"

namespace cake {

namespace {

__device__ __forceinline__ float wsum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ float wmax(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

// Sum over aligned groups of W lanes (W = 8, 16 or 32), result in every lane of the group.  The
// steps inside a row of 16 lanes are DPP moves fused into the add (no LDS traffic): swap
// neighbours, swap pairs, mirror the half row, mirror the row.
template <int W>
__device__ __forceinline__ float group_sum(float v) {
    static_assert(W == 8 || W == 16 || W == 32, "group width");
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0xB1, 0xF, 0xF, true));   // quad_perm [1,0,3,2]
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x4E, 0xF, 0xF, true));   // quad_perm [2,3,0,1]
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x141, 0xF, 0xF, true));  // row_half_mirror
    if (W >= 16) v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x140, 0xF, 0xF, true));  // row_mirror
    if (W >= 32) v += __shfl_xor(v, 16, 64);
    return v;
}

// 16 bytes of T -> floats
template <typename T> struct Ld16;
template <> struct Ld16<float> {
    static constexpr int N = 4;
    static __device__ __forceinline__ uint4 raw(const float* p) { return *(const uint4*)p; }
    static __device__ __forceinline__ void unpack(const uint4& v, float* o) {
        o[0] = __uint_as_float(v.x); o[1] = __uint_as_float(v.y); o[2] = __uint_as_float(v.z); o[3] = __uint_as_float(v.w);
    }
    static __device__ __forceinline__ void load(const float* p, float* o) { unpack(raw(p), o); }
};
template <> struct Ld16<bf16_t> {
    static constexpr int N = 8;
    static __device__ __forceinline__ uint4 raw(const bf16_t* p) { return *(const uint4*)p; }
    static __device__ __forceinline__ void unpack(const uint4& v, float* o) {
        const unsigned w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            o[2 * i] = __uint_as_float(w[i] << 16);
            o[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u);
        }
    }
    static __device__ __forceinline__ void load(const bf16_t* p, float* o) { unpack(raw(p), o); }
};

}  // namespace

// ------------------------------------------------------------------ matrix-vector product
// out[n] (op)= sum_k x[k] * w[n][k]; one wave per output row, 16-byte loads, 1 KB of the row per
// wave-instruction.  MODE 0: store; 1: add into out (residual stream); 2: silu(x.w[n]) * (x.w2[n]).
template <typename T, int MODE>
__global__ void __launch_bounds__(256) gemv_kernel(const float* __restrict__ x, const T* __restrict__ w,
                                                   const T* __restrict__ w2, float* __restrict__ out, int N, int K) {
    constexpr int E = Ld16<T>::N;
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= N) return;
    const T* wr = w + size_t(row) * K;
    const T* wr2 = MODE == 2 ? w2 + size_t(row) * K : nullptr;
    float acc = 0.f, acc2 = 0.f;
#pragma unroll 4
    for (int k = lane * E; k + E <= K; k += 64 * E) {
        float wf[E], xf[E];
        Ld16<T>::load(wr + k, wf);
#pragma unroll
        for (int e = 0; e < E; e += 4) {
            const float4 xv = *(const float4*)(x + k + e);
            xf[e] = xv.x; xf[e + 1] = xv.y; xf[e + 2] = xv.z; xf[e + 3] = xv.w;
        }
#pragma unroll
        for (int e = 0; e < E; ++e) acc = __builtin_fmaf(wf[e], xf[e], acc);
        if (MODE == 2) {
            Ld16<T>::load(wr2 + k, wf);
#pragma unroll
            for (int e = 0; e < E; ++e) acc2 = __builtin_fmaf(wf[e], xf[e], acc2);
        }
    }
    acc = wsum(acc);
    if (MODE == 2) acc2 = wsum(acc2);
    if (lane == 0) {
        if (MODE == 0) out[row] = acc;
        else if (MODE == 1) out[row] += acc;
        else out[row] = acc / (1.0f + __expf(-acc)) * acc2;
    }
}

hipError_t launch_gemv(int dtype, int mode, const float* x, const void* w, const void* w2, float* out, int N, int K,
                       hipStream_t st) {
    if (N <= 0) return hipSuccess;
    if (K % (dtype == 0 ? 4 : 8) || mode < 0 || mode > 2) return hipErrorInvalidValue;
    dim3 grid((N + 3) / 4), block(256);
#define CAKE_GEMV(T, MODE) \
    hipLaunchKernelGGL((gemv_kernel<T, MODE>), grid, block, 0, st, x, (const T*)w, (const T*)w2, out, N, K)
    if (dtype == 0) {
        if (mode == 0) CAKE_GEMV(float, 0); else if (mode == 1) CAKE_GEMV(float, 1); else CAKE_GEMV(float, 2);
    } else {
        if (mode == 0) CAKE_GEMV(bf16_t, 0); else if (mode == 1) CAKE_GEMV(bf16_t, 1); else CAKE_GEMV(bf16_t, 2);
    }
#undef CAKE_GEMV
    return hipGetLastError();
}

// ------------------------------------------------------------------ rotary on one token's queries
// q[h][2i], q[h][2i+1] rotated by pos * theta^(-2i/hd); the angle is formed in double precision
// like the prefill's table.
__global__ void rope_token_kernel(const float* __restrict__ qin, float* __restrict__ qout, int n_pairs, int half,
                                  int pos, double log2_theta) {
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= n_pairs) return;
    const int pair = idx % half;
    const double inv_freq = exp2(-(double(pair) / double(half)) * log2_theta);
    double s, c;
    sincos(double(pos) * inv_freq, &s, &c);
    const float2 v = ((const float2*)qin)[idx];
    ((float2*)qout)[idx] = make_float2(float(v.x * c - v.y * s), float(v.x * s + v.y * c));
}

hipError_t launch_rope_token(const float* qin, float* qout, int n_heads, int head_dim, int pos, float theta,
                             hipStream_t st) {
    const int half = head_dim / 2, n = n_heads * half;
    hipLaunchKernelGGL(rope_token_kernel, dim3((n + 255) / 256), dim3(256), 0, st, qin, qout, n, half, pos,
                       log2(double(theta)));
    return hipGetLastError();
}

// ------------------------------------------------------------------ one-token attention, keys split
// Grid (KV head g, split s).  The workgroup's four waves take the split's 64-key tiles in turn.
// Per tile: scores of the R query heads of the group against 64 keys (K rows are contiguous:
// KL lanes x 16 B per row, partial dots reduced across those lanes), online softmax with lane =
// key, then P.V with V^T rows (64 keys = VL lanes x 16 B, reduced across those lanes).  The waves'
// and then the splits' partial (max, sum, O) are merged by the usual rescaling.
constexpr int DEC_MAX_SPLITS = 128;

template <typename T, int HD, int R>
__global__ void __launch_bounds__(256, 2)
decode_attention_kernel(const float* __restrict__ q, float* __restrict__ part, int n_keys, int tiles_per_split,
                        KvView kv) {
    constexpr int E = Ld16<T>::N;
    constexpr int KL = HD / E, KPI = 64 / KL, NQI = 64 / KPI;   // lanes per K row, keys per instruction, instructions
    constexpr int VL = 64 / E, RPI = 64 / VL, NVI = HD / RPI;   // lanes per V^T row piece, rows per instruction
    __shared__ float sc[4][R][64];
    __shared__ float wo[4][R][HD];
    __shared__ float wm[4][R], wl[4][R];
    const int g = blockIdx.x, split = blockIdx.y, n_splits = gridDim.y;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int n_tiles = (n_keys + 63) / 64;
    const int tile_lo = split * tiles_per_split, tile_hi = min(tile_lo + tiles_per_split, n_tiles);
    const float scale = rsqrtf(float(HD));
    const int pt = kv.page_tokens;
    const size_t layer_base = size_t(kv.layer) * kv.n_physical_pages;

    const int ksub = lane % KL, kq = lane / KL;
    const int vsub = lane % VL, vq = lane / VL;
    float o_acc[R][NVI];
    float m_run[R], l_run[R];
#pragma unroll
    for (int j = 0; j < R; ++j) {
        m_run[j] = -1.0e30f;   // finite: a tile with every key masked then leaves exp(-inf - m) = 0, not NaN
        l_run[j] = 0.f;
#pragma unroll
        for (int i = 0; i < NVI; ++i) o_acc[j][i] = 0.f;
    }

    // uniform trip count for the four waves (barriers inside); a wave without a tile skips the work
    for (int base = tile_lo; base < tile_hi; base += 4) {
        const int tile = base + wave;
        const bool have = tile < tile_hi;
        const int key0 = tile * 64;
        const T* page = nullptr;
        int in_page0 = 0;
        if (have) {
            const int lpage = key0 / pt;
            in_page0 = key0 - lpage * pt;
            page = (const T*)kv.pool + (layer_base + kv.block_table[lpage]) * kv.page_elems();
        }
        // every K load of the tile is issued before the first is used (16 KB in flight together, not
        // one 1 KB round trip after another); the V^T loads go out as soon as the scores are formed,
        // so they fly during the softmax.  Registers are kept under 256 so two waves share a SIMD.
        uint4 kraw[NQI], vraw[NVI];
        if (have) {
            const T* kp = page + (size_t(g) * pt + in_page0) * HD;
            const T* vp = page + size_t(kv.n_kv) * pt * HD + size_t(g) * HD * pt + in_page0;
#pragma unroll
            for (int it = 0; it < NQI; ++it) kraw[it] = Ld16<T>::raw(kp + size_t(it * KPI + kq) * HD + ksub * E);
            float qreg[R][E];   // this lane's slice of the group's queries (L1-resident after the first tile)
#pragma unroll
            for (int j = 0; j < R; ++j)
#pragma unroll
                for (int e = 0; e < E; ++e) qreg[j][e] = q[size_t(g * R + j) * HD + ksub * E + e] * scale;
#pragma unroll
            for (int it = 0; it < NQI; ++it) {
                const int kt = it * KPI + kq;
                float kf[E];
                Ld16<T>::unpack(kraw[it], kf);
#pragma unroll
                for (int j = 0; j < R; ++j) {
                    float d = 0.f;
#pragma unroll
                    for (int e = 0; e < E; ++e) d = __builtin_fmaf(kf[e], qreg[j][e], d);
                    d = group_sum<KL>(d);
                    if (ksub == 0) sc[wave][j][kt] = d;
                }
            }
#pragma unroll
            for (int it = 0; it < NVI; ++it) vraw[it] = Ld16<T>::raw(vp + size_t(it * RPI + vq) * pt + vsub * E);
        }
        __syncthreads();
        float corr[R], pl[R][E];
        if (have) {
            const bool valid = key0 + lane < n_keys;
#pragma unroll
            for (int j = 0; j < R; ++j) {
                const float s = valid ? sc[wave][j][lane] : -INFINITY;
                const float m_new = fmaxf(m_run[j], wmax(s));
                const float p = __expf(s - m_new);
                corr[j] = __expf(m_run[j] - m_new);
                l_run[j] = l_run[j] * corr[j] + wsum(p);
                m_run[j] = m_new;
                sc[wave][j][lane] = p;
            }
        }
        __syncthreads();
        if (have) {
#pragma unroll
            for (int j = 0; j < R; ++j)
#pragma unroll
                for (int e = 0; e < E; ++e) pl[j][e] = sc[wave][j][vsub * E + e];
#pragma unroll
            for (int it = 0; it < NVI; ++it) {
                float vf[E];
                Ld16<T>::unpack(vraw[it], vf);
#pragma unroll
                for (int j = 0; j < R; ++j) {
                    float d = 0.f;
#pragma unroll
                    for (int e = 0; e < E; ++e) d = __builtin_fmaf(vf[e], pl[j][e], d);
                    d = group_sum<VL>(d);
                    o_acc[j][it] = o_acc[j][it] * corr[j] + d;
                }
            }
        }
        __syncthreads();   // sc is rewritten by the next tile
    }

    // merge the four waves, then hand the split's partial result to the combine kernel
#pragma unroll
    for (int j = 0; j < R; ++j) {
        if (lane == 0) { wm[wave][j] = m_run[j]; wl[wave][j] = l_run[j]; }
        if (vsub == 0)
#pragma unroll
            for (int it = 0; it < NVI; ++it) wo[wave][j][it * RPI + vq] = o_acc[j][it];
    }
    __syncthreads();
    for (int idx = threadIdx.x; idx < R * HD; idx += 256) {
        const int j = idx / HD, d = idx % HD;
        float m = wm[0][j];
#pragma unroll
        for (int w = 1; w < 4; ++w) m = fmaxf(m, wm[w][j]);
        float num = 0.f, den = 0.f;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const float c = __expf(wm[w][j] - m);
            num += wo[w][j][d] * c;
            den += wl[w][j] * c;
        }
        float* dst = part + (size_t(g * R + j) * n_splits + split) * (HD + 2);
        dst[d] = num;
        if (d == 0) { dst[HD] = m; dst[HD + 1] = den; }
    }
}

// One workgroup per query head; thread d owns output element d.  The per-split (max, sum) pairs are
// read by one lane each and reduced across the wave, so no thread walks the splits one dependent
// load after another.
template <int HD>
__global__ void __launch_bounds__(HD) decode_combine_kernel(const float* __restrict__ part, float* __restrict__ out,
                                                            int n_splits) {
    __shared__ float coef[DEC_MAX_SPLITS];
    __shared__ float den_s;
    const int h = blockIdx.x, d = threadIdx.x;
    const float* p = part + size_t(h) * n_splits * (HD + 2);
    if (d < 64) {   // first wave: splits d and d + 64
        const float m0 = d < n_splits ? p[d * (HD + 2) + HD] : -INFINITY;
        const float m1 = d + 64 < n_splits ? p[(d + 64) * (HD + 2) + HD] : -INFINITY;
        const float m = wmax(fmaxf(m0, m1));
        const float c0 = d < n_splits ? __expf(m0 - m) : 0.f, c1 = d + 64 < n_splits ? __expf(m1 - m) : 0.f;
        float den = (d < n_splits ? p[d * (HD + 2) + HD + 1] * c0 : 0.f) + (d + 64 < n_splits ? p[(d + 64) * (HD + 2) + HD + 1] * c1 : 0.f);
        den = wsum(den);
        coef[d] = c0;
        coef[d + 64] = c1;
        if (d == 0) den_s = den;
    }
    __syncthreads();
    float num = 0.f;
#pragma unroll 8
    for (int s = 0; s < n_splits; ++s) num += p[s * (HD + 2) + d] * coef[s];
    out[size_t(h) * HD + d] = num / den_s;
}

int decode_attention_splits(int n_keys, int n_kv) {
    const int n_tiles = (n_keys + 63) / 64;
    int want = std::max(1, 1024 / std::max(1, n_kv));            // about four workgroups per CU in total
    int splits = std::min({want, (n_tiles + 3) / 4, DEC_MAX_SPLITS});
    return std::max(1, splits);
}

size_t decode_attention_workspace_bytes(int n_q, int head_dim) {
    return size_t(n_q) * DEC_MAX_SPLITS * (head_dim + 2) * sizeof(float);
}

template <typename T, int HD>
static hipError_t decode_launch_r(int r, dim3 grid, hipStream_t st, const float* q, float* part, int n_keys, int tps,
                                  const KvView& kv) {
    switch (r) {
        case 1: hipLaunchKernelGGL((decode_attention_kernel<T, HD, 1>), grid, dim3(256), 0, st, q, part, n_keys, tps, kv); break;
        case 2: hipLaunchKernelGGL((decode_attention_kernel<T, HD, 2>), grid, dim3(256), 0, st, q, part, n_keys, tps, kv); break;
        case 4: hipLaunchKernelGGL((decode_attention_kernel<T, HD, 4>), grid, dim3(256), 0, st, q, part, n_keys, tps, kv); break;
        case 8: hipLaunchKernelGGL((decode_attention_kernel<T, HD, 8>), grid, dim3(256), 0, st, q, part, n_keys, tps, kv); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

// q[n_q][hd] (float32, rotated) against keys [0, n_keys) of the layer; out[n_q][hd] float32.
// `part` must hold decode_attention_workspace_bytes().  bf16 pages with head_dim 128 go to the
// MFMA kernel (one workgroup per CU, each wave streaming its own tiles); everything else to the
// vector-ALU kernel above.
hipError_t launch_decode_attention(int dtype, const float* q, float* out, float* part, int n_q, int n_keys,
                                   const KvView& kv, hipStream_t st, bool generic_only) {
    if (n_keys <= 0 || n_q % kv.n_kv) return hipErrorInvalidValue;
    const int r = n_q / kv.n_kv;
    const int n_tiles = (n_keys + 63) / 64;
    const bool mfma = !generic_only && decode_attention_mfma_supported(dtype, kv.head_dim, kv.page_tokens, r);
    int splits = mfma ? std::max(1, std::min({256 / std::max(1, kv.n_kv), (n_tiles + 3) / 4, DEC_MAX_SPLITS}))
                      : decode_attention_splits(n_keys, kv.n_kv);
    const int tps = (n_tiles + splits - 1) / splits;
    const int used = (n_tiles + tps - 1) / tps;   // every launched split owns at least one tile
    dim3 grid(kv.n_kv, used);
    hipError_t e;
    if (mfma) e = launch_decode_attention_mfma(q, part, n_q, n_keys, tps, used, kv, st);
    else if (dtype == 0 && kv.head_dim == 64) e = decode_launch_r<float, 64>(r, grid, st, q, part, n_keys, tps, kv);
    else if (dtype == 0 && kv.head_dim == 128) e = decode_launch_r<float, 128>(r, grid, st, q, part, n_keys, tps, kv);
    else if (dtype == 1 && kv.head_dim == 64) e = decode_launch_r<bf16_t, 64>(r, grid, st, q, part, n_keys, tps, kv);
    else if (dtype == 1 && kv.head_dim == 128) e = decode_launch_r<bf16_t, 128>(r, grid, st, q, part, n_keys, tps, kv);
    else return hipErrorInvalidValue;
    if (e != hipSuccess) return e;
    if (kv.head_dim == 64) hipLaunchKernelGGL(decode_combine_kernel<64>, dim3(n_q), dim3(64), 0, st, part, out, used);
    else hipLaunchKernelGGL(decode_combine_kernel<128>, dim3(n_q), dim3(128), 0, st, part, out, used);
    return hipGetLastError();
}

// ------------------------------------------------------------------ argmax over the logits
// result[0] = index of the largest value (the lowest index among equal values).
__global__ void __launch_bounds__(1024) argmax_kernel(const float* __restrict__ v, int n, int32_t* __restrict__ result) {
    __shared__ float bv[16];
    __shared__ int bi[16];
    float best = -INFINITY;
    int idx = 0x7fffffff;
    for (int i = threadIdx.x; i < n; i += 1024) {
        const float x = v[i];
        if (x > best || (x == best && i < idx)) { best = x; idx = i; }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const float ob = __shfl_xor(best, o, 64);
        const int oi = __shfl_xor(idx, o, 64);
        if (ob > best || (ob == best && oi < idx)) { best = ob; idx = oi; }
    }
    if ((threadIdx.x & 63) == 0) { bv[threadIdx.x >> 6] = best; bi[threadIdx.x >> 6] = idx; }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < 16; ++w)
            if (bv[w] > best || (bv[w] == best && bi[w] < idx)) { best = bv[w]; idx = bi[w]; }
        result[0] = idx;
    }
}

hipError_t launch_argmax(const float* v, int n, int32_t* result, hipStream_t st) {
    if (n <= 0) return hipErrorInvalidValue;
    hipLaunchKernelGGL(argmax_kernel, dim3(1), dim3(1024), 0, st, v, n, result);
    return hipGetLastError();
}

}  // namespace cake
