// Quantised stored KV on the load path (Sec. 5.5 combines KV compression with the method: a smaller
// stored KV loads faster, so the meet point moves towards the front).
//
// Store format per page, per layer, per K|V: codes [kv_head][token][hd] followed by float32
// scales [kv_head][token]; value = code * scale (one scale per token and KV head, symmetric,
// absmax / QMAX).  8-bit: one int8 code per element, QMAX 127.  4-bit: two codes per byte (element
// 2i in the low nibble, 2i+1 in the high nibble, two's complement), QMAX 7.  V is not transposed
// in the store; the pages hold V^T, so both kernels transpose V tiles through LDS.  Both kernels
// are plain streaming kernels bound by HBM.
#include "kernels.hpp"

namespace cake {

namespace {
template <typename T> __device__ __forceinline__ T qfrom_f(float v);
template <> __device__ __forceinline__ float qfrom_f<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16_t qfrom_f<bf16_t>(float v) { return bf16_t(v); }
template <typename T> __device__ __forceinline__ float qto_f(T v);
template <> __device__ __forceinline__ float qto_f<float>(float v) { return v; }
template <> __device__ __forceinline__ float qto_f<bf16_t>(bf16_t v) { return float(v); }
// sign-extended nibble n (0 or 1) of a byte
__device__ __forceinline__ int nibble(unsigned b, int n) { return (int(b << (28 - 4 * n))) >> 28; }
}  // namespace

// One page image -> layer pages.  grid.x: (layer, K|V, kv_head); grid.y: 64-token tiles of the page.
template <typename T, int HD, int BITS>
__global__ void __launch_bounds__(256)
dequant_page_kernel(const unsigned char* __restrict__ image, KvView kv, int phys_page, int n_layers) {
    __shared__ float tile[64][HD + 1];
    constexpr int ROWB = HD * BITS / 8;          // code bytes per token row
    const int pt = kv.page_tokens, n_kv = kv.n_kv;
    const int g = blockIdx.x % n_kv, which = (blockIdx.x / n_kv) & 1, layer = blockIdx.x / (2 * n_kv);
    const int t0 = blockIdx.y * 64;
    const size_t slab = size_t(n_kv) * pt * (ROWB + 4);
    const unsigned char* base = image + (size_t(layer) * 2 + which) * slab;
    const unsigned char* codes = base + (size_t(g) * pt + t0) * ROWB;
    const float* scales = (const float*)(base + size_t(n_kv) * pt * ROWB) + size_t(g) * pt + t0;
    T* page = (T*)kv.pool + (size_t(layer) * kv.n_physical_pages + phys_page) * kv.page_elems();
    // 64 tokens x HD elements, 4 per thread per pass (coalesced 4- or 2-byte reads)
    for (int idx = threadIdx.x * 4; idx < 64 * HD; idx += 256 * 4) {
        const int t = idx / HD, e = idx % HD;
        const float sc = scales[t];
        float v0, v1, v2, v3;
        if constexpr (BITS == 8) {
            const char4 c = *(const char4*)(codes + idx);
            v0 = float(c.x) * sc; v1 = float(c.y) * sc; v2 = float(c.z) * sc; v3 = float(c.w) * sc;
        } else {
            const unsigned c = *(const unsigned short*)(codes + idx / 2);
            v0 = float(nibble(c, 0)) * sc; v1 = float(nibble(c, 1)) * sc;
            v2 = float(nibble(c, 2)) * sc; v3 = float(nibble(c, 3)) * sc;
        }
        if (which == 0) {
            T* dst = page + (size_t(g) * pt + t0 + t) * HD + e;
            if constexpr (sizeof(T) == 2) {
                typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4_t;
                *(bf16x4_t*)dst = bf16x4_t{bf16_t(v0), bf16_t(v1), bf16_t(v2), bf16_t(v3)};
            } else {
                *(float4*)dst = make_float4(v0, v1, v2, v3);
            }
        } else {
            tile[t][e] = v0; tile[t][e + 1] = v1; tile[t][e + 2] = v2; tile[t][e + 3] = v3;
        }
    }
    if (which == 1) {
        __syncthreads();
        T* vpage = page + size_t(n_kv) * pt * HD + size_t(g) * HD * pt;
        for (int idx = threadIdx.x; idx < 64 * HD; idx += 256) {
            const int e = idx / 64, t = idx % 64;
            vpage[size_t(e) * pt + t0 + t] = qfrom_f<T>(tile[t][e]);
        }
    }
}

template <int BITS>
static hipError_t launch_dequant_bits(int dtype, const unsigned char* img, const KvView& kv, int phys_page, int n_layers,
                                      hipStream_t st) {
    dim3 grid(n_layers * 2 * kv.n_kv, kv.page_tokens / 64), block(256);
    if (dtype == 0 && kv.head_dim == 64) hipLaunchKernelGGL((dequant_page_kernel<float, 64, BITS>), grid, block, 0, st, img, kv, phys_page, n_layers);
    else if (dtype == 0 && kv.head_dim == 128) hipLaunchKernelGGL((dequant_page_kernel<float, 128, BITS>), grid, block, 0, st, img, kv, phys_page, n_layers);
    else if (dtype == 1 && kv.head_dim == 64) hipLaunchKernelGGL((dequant_page_kernel<bf16_t, 64, BITS>), grid, block, 0, st, img, kv, phys_page, n_layers);
    else if (dtype == 1 && kv.head_dim == 128) hipLaunchKernelGGL((dequant_page_kernel<bf16_t, 128, BITS>), grid, block, 0, st, img, kv, phys_page, n_layers);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

hipError_t launch_dequant_page(int dtype, const void* image, const KvView& kv, int phys_page, int n_layers, int bits,
                               hipStream_t st) {
    if (kv.page_tokens % 64) return hipErrorInvalidValue;
    const unsigned char* img = (const unsigned char*)image;
    if (bits == 8) return launch_dequant_bits<8>(dtype, img, kv, phys_page, n_layers, st);
    if (bits == 4) return launch_dequant_bits<4>(dtype, img, kv, phys_page, n_layers, st);
    return hipErrorInvalidValue;
}

// Layer pages -> one page image (the tool that writes a store from a cache that is in HBM).
// Same grid.  Four threads share a token row: absmax over the row, scale = absmax / QMAX,
// code = round-half-even(x / scale) clipped to +-QMAX; a row of zeros gets scale 0 and codes 0.
template <typename T, int HD, int BITS>
__global__ void __launch_bounds__(256)
quant_page_kernel(unsigned char* __restrict__ image, KvView kv, int phys_page, int n_layers) {
    __shared__ float tile[64][HD + 1];
    constexpr int ROWB = HD * BITS / 8;
    constexpr float QMAX = BITS == 8 ? 127.0f : 7.0f;
    const int pt = kv.page_tokens, n_kv = kv.n_kv;
    const int g = blockIdx.x % n_kv, which = (blockIdx.x / n_kv) & 1, layer = blockIdx.x / (2 * n_kv);
    const int t0 = blockIdx.y * 64;
    const size_t slab = size_t(n_kv) * pt * (ROWB + 4);
    unsigned char* base = image + (size_t(layer) * 2 + which) * slab;
    unsigned char* codes = base + (size_t(g) * pt + t0) * ROWB;
    float* scales = (float*)(base + size_t(n_kv) * pt * ROWB) + size_t(g) * pt + t0;
    const T* page = (const T*)kv.pool + (size_t(layer) * kv.n_physical_pages + phys_page) * kv.page_elems();
    if (which == 0) {
        const T* src = page + (size_t(g) * pt + t0) * HD;
        for (int idx = threadIdx.x; idx < 64 * HD; idx += 256) tile[idx / HD][idx % HD] = qto_f<T>(src[idx]);
    } else {
        const T* vpage = page + size_t(n_kv) * pt * HD + size_t(g) * HD * pt;
        for (int idx = threadIdx.x; idx < 64 * HD; idx += 256) {
            const int e = idx / 64, t = idx % 64;
            tile[t][e] = qto_f<T>(vpage[size_t(e) * pt + t0 + t]);
        }
    }
    __syncthreads();
    const int t = threadIdx.x >> 2, part = threadIdx.x & 3;   // 4 threads per token row
    float amax = 0.f;
    for (int e = part; e < HD; e += 4) amax = fmaxf(amax, fabsf(tile[t][e]));
    amax = fmaxf(amax, __shfl_xor(amax, 1, 64));
    amax = fmaxf(amax, __shfl_xor(amax, 2, 64));
    const float scale = amax / QMAX;
    const float safe = scale > 0.f ? scale : 1.0f;
    auto code = [&](int e) -> int {
        float q = rintf(tile[t][e] / safe);
        q = fminf(fmaxf(q, -QMAX), QMAX);
        return scale > 0.f ? int(q) : 0;
    };
    if constexpr (BITS == 8) {
        for (int e = part; e < HD; e += 4) codes[size_t(t) * ROWB + e] = (unsigned char)(signed char)code(e);
    } else {
        // a thread packs the element pairs (2b, 2b+1) of bytes b = part, part + 4, ...
        for (int b = part; b < HD / 2; b += 4)
            codes[size_t(t) * ROWB + b] = (unsigned char)((code(2 * b) & 0xF) | ((code(2 * b + 1) & 0xF) << 4));
    }
    if (part == 0) scales[t] = scale;
}

template <int BITS>
static hipError_t launch_quant_bits(int dtype, unsigned char* img, const KvView& kv, int phys_page, int n_layers, hipStream_t st) {
    dim3 grid(n_layers * 2 * kv.n_kv, kv.page_tokens / 64), block(256);
    if (dtype == 0 && kv.head_dim == 64) hipLaunchKernelGGL((quant_page_kernel<float, 64, BITS>), grid, block, 0, st, img, kv, phys_page, n_layers);
    else if (dtype == 0 && kv.head_dim == 128) hipLaunchKernelGGL((quant_page_kernel<float, 128, BITS>), grid, block, 0, st, img, kv, phys_page, n_layers);
    else if (dtype == 1 && kv.head_dim == 64) hipLaunchKernelGGL((quant_page_kernel<bf16_t, 64, BITS>), grid, block, 0, st, img, kv, phys_page, n_layers);
    else if (dtype == 1 && kv.head_dim == 128) hipLaunchKernelGGL((quant_page_kernel<bf16_t, 128, BITS>), grid, block, 0, st, img, kv, phys_page, n_layers);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

hipError_t launch_quant_page(int dtype, void* image, const KvView& kv, int phys_page, int n_layers, int bits, hipStream_t st) {
    if (kv.page_tokens % 64) return hipErrorInvalidValue;
    unsigned char* img = (unsigned char*)image;
    if (bits == 8) return launch_quant_bits<8>(dtype, img, kv, phys_page, n_layers, st);
    if (bits == 4) return launch_quant_bits<4>(dtype, img, kv, phys_page, n_layers, st);
    return hipErrorInvalidValue;
}

}  // namespace cake
