// bf16 MFMA kernels for gfx950: the four projection GEMMs of the decoder block and the
// chunk-vs-prefix causal attention over paged KV (Sec. 3 "Attention and KV cache",
// "Chunk Prefill": a chunk's queries attend to every cached key before and inside it).
//
// MFMA shape used throughout: v_mfma_f32_32x32x16_bf16.  For D[32x32] += A[32x16] * B[16x32]
// lane l supplies A[l%32][8*(l/32) .. +7] and B[8*(l/32) .. +7][l%32], and holds
// D[8*(v/4) + 4*(l/32) + v%4][l%32] in accumulator register v (0..15).
#include "kernels.hpp"

namespace cake {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// =====================================================================================
// GEMM: out[M][N] = a[M][K] * w[N][K]^T, bf16 in, float32 accumulate.
// 128x128 tile per 256-thread workgroup, 64-deep K slices staged through LDS (double
// buffered, 16-byte chunks XOR-swizzled by row so the 16-byte operand reads of the 32
// rows a half-wave touches fall in different banks).  Wave (wm, wn) owns a 64x64
// quadrant = 2x2 MFMA tiles.
//
// Epilogues: store float32; add into a float32 residual stream; SwiGLU, where the B tile is
// built from 32 gate rows + 32 up rows per wave column so that silu(gate) * up of one output
// column is formed in registers (the tile then yields 64 output columns).
// =====================================================================================
constexpr int GBM = 128, GBN = 128, GBK = 64;

template <int EPI>
__global__ void __launch_bounds__(256)
gemm_mfma_kernel(const bf16_t* __restrict__ A, const bf16_t* __restrict__ W, const bf16_t* __restrict__ W2,
                 void* __restrict__ outv, int M, int N, int K) {
    __shared__ __attribute__((aligned(16))) unsigned char lds[2][(GBM + GBN) * GBK * 2];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int m0 = blockIdx.y * GBM;
    const int n0 = blockIdx.x * (EPI == EPI_SWIGLU ? GBN / 2 : GBN);

    // global -> register staging: thread loads 16-byte chunk `c` of rows r, r+32, r+64, r+96
    const int c = tid & 7, r = tid >> 3;
    const bf16_t* ap[4];
    const bf16_t* bp[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        int row = r + 32 * i;
        int am = min(m0 + row, M - 1);
        ap[i] = A + size_t(am) * K + c * 8;
        if (EPI == EPI_SWIGLU) {
            // tile row -> (wave column, gate|up, column): rows [64*wn + 32*t + j], t = 0 gate, 1 up
            int wcol = row >> 6, t = (row >> 5) & 1, j = row & 31;
            const bf16_t* src = t ? W2 : W;
            bp[i] = src + size_t(n0 + wcol * 32 + j) * K + c * 8;
        } else {
            bp[i] = W + size_t(n0 + row) * K + c * 8;
        }
    }
    uint4 ra[4], rb[4];
    auto gload = [&](int k0) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            ra[i] = *(const uint4*)(ap[i] + k0);
            rb[i] = *(const uint4*)(bp[i] + k0);
        }
    };
    auto lstore = [&](int buf) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            int row = r + 32 * i;
            int off = row * (GBK * 2) + ((c ^ (row & 7)) << 4);
            *(uint4*)(&lds[buf][off]) = ra[i];
            *(uint4*)(&lds[buf][GBM * GBK * 2 + off]) = rb[i];
        }
    };

    f32x16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    const int nk = K / GBK;
    gload(0);
    lstore(0);
    __syncthreads();
    const int lrow = lane & 31, lhalf = lane >> 5;
    for (int kt = 0; kt < nk; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < nk) gload((kt + 1) * GBK);
        const unsigned char* la = &lds[buf][0];
        const unsigned char* lb = &lds[buf][GBM * GBK * 2];
#pragma unroll
        for (int ks = 0; ks < GBK / 16; ++ks) {
            bf16x8 a[2], b[2];
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                int arow = wm * 64 + t * 32 + lrow;
                int brow = wn * 64 + t * 32 + lrow;
                int chunk = 2 * ks + lhalf;
                a[t] = *(const bf16x8*)(la + arow * (GBK * 2) + ((chunk ^ (arow & 7)) << 4));
                b[t] = *(const bf16x8*)(lb + brow * (GBK * 2) + ((chunk ^ (brow & 7)) << 4));
            }
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j) acc[i][j] = mfma32(a[i], b[j], acc[i][j]);
        }
        if (kt + 1 < nk) lstore(buf ^ 1);
        __syncthreads();
    }

    // epilogue
#pragma unroll
    for (int i = 0; i < 2; ++i) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            int row = m0 + wm * 64 + i * 32 + 8 * (v >> 2) + 4 * lhalf + (v & 3);
            if (row >= M) continue;
            if (EPI == EPI_SWIGLU) {
                int col = n0 + wn * 32 + lrow;
                float g = acc[i][0][v], u = acc[i][1][v];
                ((bf16_t*)outv)[size_t(row) * N + col] = bf16_t(g / (1.0f + __expf(-g)) * u);
            } else {
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    int col = n0 + wn * 64 + j * 32 + lrow;
                    float* o = (float*)outv + size_t(row) * N + col;
                    if (EPI == EPI_RESIDUAL_F32) *o += acc[i][j][v];
                    else *o = acc[i][j][v];
                }
            }
        }
    }
}

bool gemm_mfma_supported(int epi, int M, int N, int K) {
    const int ncols = epi == EPI_SWIGLU ? GBN / 2 : GBN;
    return M > 0 && N > 0 && K > 0 && (K % GBK) == 0 && (N % ncols) == 0;
}

hipError_t launch_gemm_mfma(int epi, const void* a, const void* w, const void* w2, void* out, int M, int N, int K,
                            hipStream_t st) {
    // N is the number of output columns; the SwiGLU tile yields GBN/2 of them
    const bf16_t *A = (const bf16_t*)a, *W = (const bf16_t*)w, *W2 = (const bf16_t*)w2;
    dim3 block(256);
    if (epi == EPI_SWIGLU) {
        if (N % (GBN / 2)) return hipErrorInvalidValue;
        dim3 grid(N / (GBN / 2), (M + GBM - 1) / GBM);
        hipLaunchKernelGGL((gemm_mfma_kernel<EPI_SWIGLU>), grid, block, 0, st, A, W, W2, out, M, N, K);
    } else {
        dim3 grid(N / GBN, (M + GBM - 1) / GBM);
        if (epi == EPI_STORE_F32) hipLaunchKernelGGL((gemm_mfma_kernel<EPI_STORE_F32>), grid, block, 0, st, A, W, W2, out, M, N, K);
        else if (epi == EPI_RESIDUAL_F32) hipLaunchKernelGGL((gemm_mfma_kernel<EPI_RESIDUAL_F32>), grid, block, 0, st, A, W, W2, out, M, N, K);
        else return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

// =====================================================================================
// Attention: out[row][h*128 + :] = softmax_s(q_row . k_s / sqrt(128)) v_s over keys s <= tok_begin+row.
//
// Workgroup = 4 waves x 32 queries of one query head; keys are visited in tiles of 64.  The
// score tile is formed transposed, S^T[key][query] = K[key][:] . Q[query][:], so that in the
// accumulator a lane holds 32 keys of ONE query: the online-softmax row statistics are per-lane
// scalars (one exchange with lane^32 for the max), and the probabilities are already in the
// layout the next MFMA wants for its B operand, P^T[key][query].  The second product is
// O^T[hd][query] += V^T[hd][key] * P^T[key][query], whose A operand reads the transposed V pages
// directly (8 consecutive keys = 16 bytes).  The accumulator puts keys {0-3, 8-11} of each
// 16-key step in the low half-wave and {4-7, 12-15} in the high one; the V^T operand is read
// with the same permutation, which is legal because the contraction sums over keys.
// =====================================================================================
constexpr int AQ = 128;   // queries per workgroup
constexpr int AK = 64;    // keys per tile
constexpr int AHD = 128;  // head dim
constexpr int KROW = AHD * 2;      // bytes per K row in LDS (swizzled 16-byte chunks)
constexpr int VROW = AK * 2 + 8;   // bytes per V^T row in LDS (+8 pad: rows shift by two banks)

__global__ void __launch_bounds__(256)
attention_mfma_kernel(const bf16_t* __restrict__ q, bf16_t* __restrict__ out, int n_q, int tok_begin, int rows,
                      KvView kv) {
    __shared__ __attribute__((aligned(16))) unsigned char ldsK[AK * KROW];
    __shared__ __attribute__((aligned(16))) unsigned char ldsV[AHD * VROW];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int lrow = lane & 31, lhalf = lane >> 5;
    const int h = blockIdx.y;
    const int g = h / (n_q / kv.n_kv);
    const int q0 = blockIdx.x * AQ;                 // first query row of the workgroup
    const int my_row = min(q0 + wave * 32 + lrow, rows - 1);
    const int my_pos = tok_begin + my_row;          // this lane's query position
    const int wg_last_pos = tok_begin + min(q0 + AQ, rows) - 1;
    const int wave_first_pos = tok_begin + min(q0 + wave * 32, rows - 1);
    const int pt = kv.page_tokens;

    // Q^T operand: lane supplies q[my_row][16*ks + 8*lhalf .. +7]
    bf16x8 qreg[AHD / 16];
    {
        const bf16_t* qp = q + (size_t(h) * rows + my_row) * AHD + 8 * lhalf;
#pragma unroll
        for (int ks = 0; ks < AHD / 16; ++ks) qreg[ks] = *(const bf16x8*)(qp + 16 * ks);
    }

    f32x16 o[4];
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) o[t][v] = 0.f;
    float m_run = -INFINITY, l_part = 0.f;
    const float sl2 = 0.08838834764831845f * 1.4426950408889634f;  // 1/sqrt(128) * log2(e)

    const int n_tiles = wg_last_pos / AK + 1;
    for (int kt = 0; kt < n_tiles; ++kt) {
        const int key0 = kt * AK;
        const int lpage = key0 / pt;
        const int in_page0 = key0 - lpage * pt;
        const bf16_t* page = (const bf16_t*)kv.pool +
                             (size_t(kv.layer) * kv.n_physical_pages + kv.block_table[lpage]) * kv.page_elems();
        const bf16_t* kp = page + (size_t(g) * pt + in_page0) * AHD;                       // [64][128]
        const bf16_t* vp = page + size_t(kv.n_kv) * pt * AHD + size_t(g) * AHD * pt + in_page0;  // [128][pt]
        __syncthreads();  // previous tile fully consumed
        // K tile: 64 rows x 16 chunks of 16 B = 1024 chunks, 4 per thread
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            int idx = tid + 256 * i, row = idx >> 4, ch = idx & 15;
            uint4 v = *(const uint4*)(kp + size_t(row) * AHD + ch * 8);
            *(uint4*)(ldsK + row * KROW + ((ch ^ (row & 7)) << 4)) = v;
        }
        // V^T tile: 128 rows x 8 chunks of 16 B (8 keys) = 1024 chunks, 4 per thread
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            int idx = tid + 256 * i, row = idx >> 3, ch = idx & 7;
            uint4 v = *(const uint4*)(vp + size_t(row) * pt + ch * 8);
            uint2* dst = (uint2*)(ldsV + row * VROW + ch * 16);
            dst[0] = make_uint2(v.x, v.y);
            dst[1] = make_uint2(v.z, v.w);
        }
        __syncthreads();
        if (key0 > tok_begin + min(q0 + wave * 32 + 31, rows - 1)) continue;  // tile entirely in this wave's future

        // S^T = K Q^T : two 32-key tiles x 32 queries
        f32x16 s[2];
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int v = 0; v < 16; ++v) s[t][v] = 0.f;
#pragma unroll
        for (int ks = 0; ks < AHD / 16; ++ks) {
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                int row = t * 32 + lrow, ch = 2 * ks + lhalf;
                bf16x8 a = *(const bf16x8*)(ldsK + row * KROW + ((ch ^ (row & 7)) << 4));
                s[t] = mfma32(a, qreg[ks], s[t]);
            }
        }
        // causal mask (only tiles that reach past the wave's first query need it)
        if (key0 + AK - 1 > wave_first_pos) {
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    int key = key0 + t * 32 + 8 * (v >> 2) + 4 * lhalf + (v & 3);
                    if (key > my_pos) s[t][v] = -INFINITY;
                }
        }
        float mx = m_run;
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int v = 0; v < 16; ++v) mx = fmaxf(mx, s[t][v] * sl2);
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        // every query sees key 0 in tile 0, so mx is finite from the first visited tile on
        const float corr = exp2f(m_run - mx);
        m_run = mx;
        l_part *= corr;
        bf16x8 p[4];
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                float e = exp2f(s[t][v] * sl2 - mx);
                l_part += e;
                p[2 * t + (v >> 3)][v & 7] = bf16_t(e);
            }
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int v = 0; v < 16; ++v) o[t][v] *= corr;
        // O^T += V^T P^T : 4 tiles of 32 head dims, 4 steps of 16 keys
#pragma unroll
        for (int j = 0; j < 4; ++j) {
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const unsigned char* vr = ldsV + (t * 32 + lrow) * VROW + j * 32 + 8 * lhalf;
                uint2 lo = *(const uint2*)(vr);        // keys 16j + 4*lhalf + 0..3
                uint2 hi = *(const uint2*)(vr + 16);   // keys 16j + 8 + 4*lhalf + 0..3
                uint4 both = make_uint4(lo.x, lo.y, hi.x, hi.y);
                bf16x8 a = *(bf16x8*)&both;
                o[t] = mfma32(a, p[j], o[t]);
            }
        }
    }
    // finish: total row sum = this lane's partial + the partner half-wave's
    float l_tot = l_part + __shfl_xor(l_part, 32, 64);
    float inv = 1.0f / l_tot;
    const int row = q0 + wave * 32 + lrow;
    if (row < rows) {
        bf16_t* op = out + size_t(row) * n_q * AHD + h * AHD;
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int v4 = 0; v4 < 4; ++v4) {
                bf16x4 w;
#pragma unroll
                for (int e = 0; e < 4; ++e) w[e] = bf16_t(o[t][4 * v4 + e] * inv);
                *(bf16x4*)(op + t * 32 + 8 * v4 + 4 * lhalf) = w;
            }
    }
}

bool attention_mfma_supported(int head_dim, int page_tokens) {
    return head_dim == AHD && page_tokens % AK == 0;
}

hipError_t launch_attention_mfma(const void* q, void* out, int n_q, int tok_begin, int rows, const KvView& kv,
                                 hipStream_t st) {
    if (rows <= 0) return hipSuccess;
    dim3 grid((rows + AQ - 1) / AQ, n_q), block(256);
    hipLaunchKernelGGL(attention_mfma_kernel, grid, block, 0, st, (const bf16_t*)q, (bf16_t*)out, n_q, tok_begin, rows, kv);
    return hipGetLastError();
}

}  // namespace cake
