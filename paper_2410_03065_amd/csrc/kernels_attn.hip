// bf16 MFMA attention for gfx950: chunk-vs-prefix causal attention over paged KV
// (Sec. 3 "Attention and KV cache", "Chunk Prefill": a chunk's queries attend to every cached
// key before and inside it).  Built with MFMA results kept in ordinary VGPRs, because the
// softmax reads every score on the vector ALUs.
//
// MFMA shape used throughout: v_mfma_f32_32x32x16_bf16.  For D[32x32] += A[32x16] * B[16x32]
// lane l supplies A[l%32][8*(l/32) .. +7] and B[8*(l/32) .. +7][l%32], and holds
// D[8*(v/4) + 4*(l/32) + v%4][l%32] in accumulator register v (0..15).
#include <type_traits>

#include "kernels.hpp"

namespace cake {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

#define CAKE_GLOBAL_AS __attribute__((address_space(1)))
#define CAKE_LDS_AS __attribute__((address_space(3)))

// =====================================================================================
// Attention: out[row][h*128 + :] = softmax_s(q_row . k_s / sqrt(128)) v_s over keys s <= tok_begin+row.
//
// Workgroup = 4 waves x 32 queries of one query head; keys are visited in tiles of 64 held in a
// ring of LDS stages filled by direct global->LDS loads from the K pages ([key][hd]) and the
// transposed V pages ([hd][key]).
//
// The score tile is formed transposed, S^T[key][query] = K[key][:] . Q[query][:], so a lane
// holds 32 keys of ONE query: the online-softmax statistics are per-lane scalars (one exchange
// with lane^32 for the max) and the probabilities are already laid out as the B operand
// P^T[key][query] of the second product O^T[hd][query] += V^T[hd][key] P^T[key][query].
// The K rows fed to the first MFMA are permuted within each group of 16 (rows 4-7 and 8-11
// swapped).  With that, accumulator registers v = 8*(j&1) .. +7 of key tile j>>1 hold, in the
// low / high half-wave, keys 16j + 0..7 / 16j + 8..15 -- exactly the 8 consecutive k-slots each
// half-wave must supply for 16-key step j, so P needs no shuffle and the V^T operand is one
// aligned 16-byte read.
//
// Pipeline per key tile: wait for the next tile's loads, barrier, refill the stage freed one
// tile ago, then issue the NEXT tile's score MFMAs and, in their shadow, run this tile's
// softmax on the vector ALUs, then this tile's P V MFMAs.  The output accumulators are rescaled
// only when some lane's running maximum moved (wave-uniform test).
// =====================================================================================
constexpr int AQ = 128;   // queries per workgroup
constexpr int AK = 64;    // keys per tile
constexpr int AHD = 128;  // head dim
constexpr int A_STAGES = 4;
constexpr int A_KBYTES = AK * AHD * 2, A_STAGE = 2 * A_KBYTES;
constexpr int A_PER_TILE = 8;  // wave-loads per wave per tile (4 K + 4 V)

__device__ __forceinline__ int sigma16(int x) { return (x & 3) | ((x & 4) << 1) | ((x & 8) >> 1); }

__global__ void __launch_bounds__(256)
attention_mfma_kernel(const bf16_t* __restrict__ q, bf16_t* __restrict__ out, int n_q, int tok_begin, int rows,
                      KvView kv, int q_tiles) {
    extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lrow = lane & 31, lhalf = lane >> 5;
    const int G = kv.n_kv, r = n_q / G;
    // Workgroups that share a KV head go to the same XCD (block b runs on XCD b % 8).
    int g, rest;
    if ((G & 7) == 0) {
        const int xcd = blockIdx.x & 7, idx = blockIdx.x >> 3, gpx = G >> 3;
        g = xcd + 8 * (idx % gpx);
        rest = idx / gpx;
    } else {
        g = blockIdx.x % G;
        rest = blockIdx.x / G;
    }
    const int h = g * r + rest % r;
    const int q0 = (rest / r) * AQ;
    const int pt = kv.page_tokens;

    const int my_row = min(q0 + wave * 32 + lrow, rows - 1);
    const int my_pos = tok_begin + my_row;
    const int wave_first_pos = tok_begin + min(q0 + wave * 32, rows - 1);
    const int wg_last_pos = tok_begin + min(q0 + AQ, rows) - 1;
    const int n_tiles = wg_last_pos / AK + 1;

    // Q^T operand: lane supplies q[my_row][16*ks + 8*lhalf .. +7]
    bf16x8 qreg[AHD / 16];
    {
        const bf16_t* qp = q + (size_t(h) * rows + my_row) * AHD + 8 * lhalf;
#pragma unroll
        for (int ks = 0; ks < AHD / 16; ++ks) qreg[ks] = *(const bf16x8*)(qp + 16 * ks);
    }

    // global->LDS sources.  K wave-load j covers rows 4j..4j+3 (256 B each, chunk c stored at c ^ (row & 15));
    // V^T wave-load j covers rows 8j..8j+7 (128 B each, chunk c stored at c ^ ((row >> 1) & 7)).
    unsigned koffg[4], voffg[4];   // byte offsets from the tile's K / V^T base
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        int j = wave + 4 * i;
        int krow = 4 * j + (lane >> 4), kpos = lane & 15;
        koffg[i] = unsigned(krow * AHD + ((kpos ^ (krow & 15)) << 3)) * 2u;
        int vrow = 8 * j + (lane >> 3), vpos = lane & 7;
        voffg[i] = unsigned(vrow * pt + ((vpos ^ ((vrow >> 1) & 7)) << 3)) * 2u;
    }
    // Byte offset of every logical page this workgroup needs (this layer, this KV head's K block)
    // is put into LDS once: a global load in the issue path would share the vmcnt counter with
    // the tile loads and drain the whole ring.  The entry for the tile issued next is read one
    // tile ahead, so its LDS latency is off the issue path too.
    const int last_page = wg_last_pos / pt;
    unsigned long long* pg_lds = (unsigned long long*)(lds + A_STAGES * A_STAGE);
    {
        const size_t layer_base = size_t(kv.layer) * kv.n_physical_pages;
        const size_t page_bytes = kv.page_elems() * 2, k_head = size_t(g) * pt * AHD * 2;
        for (int i = tid; i <= last_page; i += 256) pg_lds[i] = (layer_base + kv.block_table[i]) * page_bytes + k_head;
    }
    __syncthreads();
    // from a page's K block of head g to its V^T block of head g
    const unsigned long long k_to_v = (size_t(G - g) * pt * AHD + size_t(g) * AHD * pt) * 2;
    unsigned long long pg_next = pg_lds[0];
    auto issue = [&](int stage, int kt) {
        const int key0 = kt * AK;
        const int lpage = key0 / pt;
        const unsigned in_page0 = unsigned(key0 - lpage * pt);
        // readfirstlane returns a signed int: go through unsigned, or offsets with bit 31 set sign-extend
        const unsigned long long lo = (unsigned)__builtin_amdgcn_readfirstlane((int)unsigned(pg_next));
        const unsigned long long hi = (unsigned)__builtin_amdgcn_readfirstlane((int)unsigned(pg_next >> 32));
        const char* kp = (const char*)kv.pool + ((hi << 32) | lo) + size_t(in_page0) * (AHD * 2);
        const char* vp = (const char*)kv.pool + ((hi << 32) | lo) + k_to_v + size_t(in_page0) * 2;
        pg_next = pg_lds[min((key0 + AK) / pt, last_page)];
        unsigned char* sa = lds + stage * A_STAGE;
#pragma unroll
        for (int i = 0; i < 4; ++i)
            __builtin_amdgcn_global_load_lds((const CAKE_GLOBAL_AS void*)(kp + size_t(koffg[i])),
                                             (CAKE_LDS_AS void*)(sa + (wave + 4 * i) * 1024), 16, 0, 0);
#pragma unroll
        for (int i = 0; i < 4; ++i)
            __builtin_amdgcn_global_load_lds((const CAKE_GLOBAL_AS void*)(vp + size_t(voffg[i])),
                                             (CAKE_LDS_AS void*)(sa + A_KBYTES + (wave + 4 * i) * 1024), 16, 0, 0);
    };

    // operand read offsets (per lane, in bytes from the start of a stage)
    const int sk = sigma16(lrow & 15);
    const int krow_base = (16 * (lrow >> 4) + sk) * (AHD * 2);   // + 32*t rows
    int kaddr[AHD / 16];
#pragma unroll
    for (int ks = 0; ks < AHD / 16; ++ks) kaddr[ks] = krow_base + (((2 * ks + lhalf) ^ sk) << 4);
    const int sv = (lrow >> 1) & 7;
    int vaddr[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) vaddr[j] = A_KBYTES + lrow * (AK * 2) + (((2 * j + lhalf) ^ sv) << 4);

    f32x16 o[4];
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) o[t][v] = 0.f;
    float m_run = -INFINITY, l_part = 0.f;
    const float sl2 = 0.08838834764831845f * 1.4426950408889634f;  // 1/sqrt(128) * log2(e)
    const f32x16 zero16 = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};

    // Running maximum of a score tile, in pieces so that it can be spread over MFMA groups:
    // (masking of the diagonal tiles), max over the lane's 32 scores, exchange with the partner
    // half-wave, correction factor for the old accumulators.
    float mx_cur = 0.f, corr_cur = 0.f;
    bool moved_cur = false;
    auto mask_tile = [&](f32x16* s, int kt) {
        const int key0 = kt * AK;
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                int key = key0 + 32 * t + (v & 7) + 8 * lhalf + 16 * (v >> 3);
                if (key > my_pos) s[t][v] = -INFINITY;
            }
    };
    auto part_max = [&](const f32x16* s, int part, float acc) {   // elements [8*part, 8*part+8) of the 32
#pragma unroll
        for (int i = 0; i < 8; ++i) acc = fmaxf(acc, s[part >> 1][8 * (part & 1) + i]);
        return acc;
    };
    // The exponentials use a reference value m_run per query that follows the running maximum
    // lazily: it is moved (and O, l rescaled) only when some lane's maximum has outgrown it by more
    // than 2^RESCALE_LOG2, so probabilities may reach 2^RESCALE_LOG2 instead of 1 -- harmless in
    // bf16 / fp32, and softmax is invariant to the reference.  Without this the rescale of the 64
    // accumulator registers would run on roughly every other tile.
    constexpr float RESCALE_LOG2 = 6.0f;
    auto finish_max = [&](float raw) {
        float mx = raw * sl2;
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));   // key 0 is visible to every query, so mx is finite
        moved_cur = mx > m_run + RESCALE_LOG2;    // -inf + 6 = -inf: the first tile always moves
        if (__builtin_amdgcn_ballot_w64(moved_cur) != 0) {
            mx = fmaxf(mx, m_run);
            corr_cur = __builtin_amdgcn_exp2f(m_run - mx);
            m_run = mx;
            moved_cur = true;
        } else {
            corr_cur = 1.0f;
        }
        mx_cur = m_run;
    };

    // One key tile = two MFMA phases of four groups each (4 LDS reads feeding 4 MFMAs per group);
    // a group's operands are read while the previous group's MFMAs run, and the vector-ALU work
    // is dealt out group by group so that it executes in the MFMAs' shadow:
    //   phase 1: S^T of tile kt+1  ||  exponentials + bf16 packing of tile kt (8 per group)
    //   phase 2: O^T += V^T P^T of tile kt  ||  (mask and) running max of tile kt+1
    // then the (rare) rescale of O by the correction of tile kt+1.
    auto step = [&](int kt, f32x16* s_cur, f32x16* s_nxt, auto masked_tag) {
        constexpr bool masked_next = decltype(masked_tag)::value;
        if (kt + A_STAGES - 2 < n_tiles) asm volatile("s_waitcnt vmcnt(%0)" ::"n"((A_STAGES - 3) * A_PER_TILE));
        else asm volatile("s_waitcnt vmcnt(0)");
        __builtin_amdgcn_s_barrier();
        if (kt + A_STAGES - 1 < n_tiles) issue((kt + A_STAGES - 1) % A_STAGES, kt + A_STAGES - 1);

        const float mx = mx_cur;
        // past the last tile the score MFMAs read a stale stage; that result is never used
        const unsigned char* stk = lds + ((kt + 1) % A_STAGES) * A_STAGE;
        const unsigned char* stv = lds + (kt % A_STAGES) * A_STAGE;
        bf16x8 opa[4], opb[4], p[4];
        auto read_k = [&](bf16x8* dst, int grp) {   // ks = 2*grp, 2*grp+1 ; t = 0, 1
#pragma unroll
            for (int i = 0; i < 4; ++i)
                dst[i] = *(const bf16x8*)(stk + (i & 1) * 32 * (AHD * 2) + kaddr[2 * grp + (i >> 1)]);
        };
        auto read_v = [&](bf16x8* dst, int j) {      // t = 0..3
#pragma unroll
            for (int i = 0; i < 4; ++i) dst[i] = *(const bf16x8*)(stv + i * 32 * (AK * 2) + vaddr[j]);
        };
        auto mma_k = [&](const bf16x8* src, int grp) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int ks = 2 * grp + (i >> 1), t = i & 1;
                s_nxt[t] = mfma32(src[i], qreg[ks], ks == 0 ? zero16 : s_nxt[t]);
            }
        };
        auto expo = [&](int grp) {                   // p[grp]: 8 probabilities of tile kt
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                float e = __builtin_amdgcn_exp2f(__builtin_fmaf(s_cur[grp >> 1][8 * (grp & 1) + i], sl2, -mx));
                l_part += e;
                p[grp][i] = bf16_t(e);
            }
        };
        // ---- phase 1
        read_k(opa, 0);
        __builtin_amdgcn_sched_barrier(0);
        read_k(opb, 1); mma_k(opa, 0); expo(0);
        __builtin_amdgcn_sched_barrier(0);
        read_k(opa, 2); mma_k(opb, 1); expo(1);
        __builtin_amdgcn_sched_barrier(0);
        read_k(opb, 3); mma_k(opa, 2); expo(2);
        __builtin_amdgcn_sched_barrier(0);
        read_v(opa, 0); mma_k(opb, 3); expo(3);
        __builtin_amdgcn_sched_barrier(0);
        // ---- phase 2
        float raw;
        if (masked_next) mask_tile(s_nxt, kt + 1);
        read_v(opb, 1);
#pragma unroll
        for (int t = 0; t < 4; ++t) o[t] = mfma32(opa[t], p[0], o[t]);
        raw = part_max(s_nxt, 0, s_nxt[0][0]);
        raw = part_max(s_nxt, 1, raw);
        __builtin_amdgcn_sched_barrier(0);
        read_v(opa, 2);
#pragma unroll
        for (int t = 0; t < 4; ++t) o[t] = mfma32(opb[t], p[1], o[t]);
        raw = part_max(s_nxt, 2, raw);
        raw = part_max(s_nxt, 3, raw);
        __builtin_amdgcn_sched_barrier(0);
        read_v(opb, 3);
#pragma unroll
        for (int t = 0; t < 4; ++t) o[t] = mfma32(opa[t], p[2], o[t]);
        finish_max(raw);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int t = 0; t < 4; ++t) o[t] = mfma32(opb[t], p[3], o[t]);
        __builtin_amdgcn_sched_barrier(0);
        if (__builtin_amdgcn_ballot_w64(moved_cur) != 0) {
            l_part *= corr_cur;
#pragma unroll
            for (int t = 0; t < 4; ++t)
#pragma unroll
                for (int v = 0; v < 16; ++v) o[t][v] *= corr_cur;
        }
    };

    // prologue
#pragma unroll
    for (int st = 0; st < A_STAGES - 1; ++st)
        if (st < n_tiles) issue(st, st);
    if (n_tiles >= A_STAGES - 1) asm volatile("s_waitcnt vmcnt(%0)" ::"n"((A_STAGES - 2) * A_PER_TILE));
    else asm volatile("s_waitcnt vmcnt(0)");
    __builtin_amdgcn_s_barrier();
    f32x16 s_a[2], s_b[2];
    {
        const unsigned char* stk = lds;
#pragma unroll
        for (int ks = 0; ks < AHD / 16; ++ks)
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                bf16x8 a = *(const bf16x8*)(stk + t * 32 * (AHD * 2) + kaddr[ks]);
                s_a[t] = mfma32(a, qreg[ks], ks == 0 ? zero16 : s_a[t]);
            }
    }
    // tiles below first_masked hold only keys every query of this wave may see
    const int first_masked = (wave_first_pos + 1) / AK;   // first tile with key0 + AK - 1 > wave_first_pos
    if (first_masked <= 0) mask_tile(s_a, 0);
    {
        float raw = s_a[0][0];
#pragma unroll
        for (int part = 0; part < 4; ++part) raw = part_max(s_a, part, raw);
        finish_max(raw);
    }
    // two tiles per trip so the score buffers alternate without copies
    int kt = 0;
    for (; kt + 2 < first_masked && kt + 1 < n_tiles; kt += 2) {
        step(kt, s_a, s_b, std::false_type{});
        step(kt + 1, s_b, s_a, std::false_type{});
    }
    for (; kt < n_tiles; kt += 2) {   // the few tiles on and past the diagonal
        step(kt, s_a, s_b, std::true_type{});
        if (kt + 1 < n_tiles) step(kt + 1, s_b, s_a, std::true_type{});
    }
    // finish: total row sum = this lane's partial + the partner half-wave's
    const float l_tot = l_part + __shfl_xor(l_part, 32, 64);
    const float inv = 1.0f / l_tot;
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

// =====================================================================================
// Eight-wave variant: two waves per SIMD, so that one wave's softmax (vector ALU) runs while the
// other's MFMAs occupy the matrix pipe -- a single wave cannot overlap the two (an MFMA holds its
// own wave's issue for most of its duration).  A chunk of 1024 queries x 32 heads only offers
// 4 waves of 32 queries per CU, so the second wave group takes the other half of the KEYS: waves
// 0-3 visit key tiles 0, 2, 4, ..., waves 4-7 tiles 1, 3, 5, ... with private softmax state, and
// the two partial results are merged through LDS at the end (softmax over a union of key sets:
// rescale both to the common reference and add).
//
// LDS: K ring of 2 x (two 16 KB tiles) and V^T ring of 2 x (two 16 KB tiles).  K of a tile pair
// is consumed one iteration before its V^T, so per iteration the V^T of pair i+1 and the K of
// pair i+2 are fetched, each into the buffer its group finished with in the previous iteration.
// Masked scores are -inf, the initial reference is a large FINITE negative: a row whose keys in
// one half are all above the diagonal then keeps exp2(-inf - finite) = 0 everywhere (no inf - inf),
// ends with O = 0, l = 0 and the initial reference, and the merge weighs that half by exactly 0.
// =====================================================================================
constexpr float A8_NEG = -1.0e30f;
constexpr int A8_RING = 2 * A_KBYTES;        // one ring slot: group A's tile then group B's tile
constexpr int A8_VBASE = 2 * A8_RING;        // V^T ring after the K ring
constexpr int A8_TABLE = 4 * A8_RING;        // page offsets after both rings

// QW = query waves per half (4: 128 queries per workgroup; 2: 64 queries, for launches whose
// 128-query grid would leave CUs idle, e.g. 512-token chunks of a 32-head model).
template <int QW>
__global__ void __launch_bounds__(128 * QW)
attention_mfma8_kernel(const bf16_t* __restrict__ q, bf16_t* __restrict__ out, int n_q, int tok_begin, int rows,
                       KvView kv, int q_tiles) {
    constexpr int AQW = 32 * QW;        // queries per workgroup
    constexpr int PER = 16 / QW;        // wave-loads per wave per K (or V^T) tile
    constexpr int KP = QW >= 4 ? 1 : 4 / QW;   // period after which the K swizzle term of a wave's loads repeats
    extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave8 = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wave = wave8 % QW, grp = wave8 / QW;
    const int lrow = lane & 31, lhalf = lane >> 5;
    const int G = kv.n_kv, r = n_q / G;
    int g, rest;
    if ((G & 7) == 0) {
        const int xcd = blockIdx.x & 7, idx = blockIdx.x >> 3, gpx = G >> 3;
        g = xcd + 8 * (idx % gpx);
        rest = idx / gpx;
    } else {
        g = blockIdx.x % G;
        rest = blockIdx.x / G;
    }
    const int h = g * r + rest % r;
    const int q0 = (rest / r) * AQW;
    const int pt = kv.page_tokens;

    const int my_row = min(q0 + wave * 32 + lrow, rows - 1);
    const int my_pos = tok_begin + my_row;
    const int wave_first_pos = tok_begin + min(q0 + wave * 32, rows - 1);
    const int wg_last_pos = tok_begin + min(q0 + AQW, rows) - 1;
    const int n_tiles = wg_last_pos / AK + 1;
    const int n_pairs = (n_tiles + 1) >> 1;
    const int first_masked = (wave_first_pos + 1) / AK;   // first tile with a key some query of this wave must not see

    bf16x8 qreg[AHD / 16];
    {
        const bf16_t* qp = q + (size_t(h) * rows + my_row) * AHD + 8 * lhalf;
#pragma unroll
        for (int ks = 0; ks < AHD / 16; ++ks) qreg[ks] = *(const bf16x8*)(qp + 16 * ks);
        // softmax scale and log2(e) go into Q once, so a score leaves the MFMA in the exponent's units
        const float sl2q = 0.08838834764831845f * 1.4426950408889634f;
#pragma unroll
        for (int ks = 0; ks < AHD / 16; ++ks)
#pragma unroll
            for (int e = 0; e < 8; ++e) qreg[ks][e] = bf16_t(float(qreg[ks][e]) * sl2q);
    }
    // lane offsets of this wave's K / V^T wave-loads of a tile: load i covers 1 KB = key rows
    // 4j .. 4j+3 (V^T: head-dim rows 8j .. 8j+7) with j = wave + QW*i.  The swizzle term of the K
    // rows repeats every KP loads, that of the V^T rows with every load, so the other loads are a
    // wave-uniform distance from these.
    unsigned koffp[KP], voff0;
#pragma unroll
    for (int i = 0; i < KP; ++i) {
        int krow = 4 * (wave + QW * i) + (lane >> 4), kpos = lane & 15;
        koffp[i] = unsigned(krow * AHD + ((kpos ^ (krow & 15)) << 3)) * 2u;
    }
    {
        int vrow = 8 * wave + (lane >> 3), vpos = lane & 7;
        voff0 = unsigned(vrow * pt + ((vpos ^ ((vrow >> 1) & 7)) << 3)) * 2u;
    }
    const int last_page = wg_last_pos / pt;
    unsigned long long* pg_lds = (unsigned long long*)(lds + A8_TABLE);
    {
        const size_t layer_base = size_t(kv.layer) * kv.n_physical_pages;
        const size_t page_bytes = kv.page_elems() * 2, k_head = size_t(g) * pt * AHD * 2;
        for (int i = tid; i <= last_page; i += 128 * QW) pg_lds[i] = (layer_base + kv.block_table[i]) * page_bytes + k_head;
    }
    __syncthreads();
    const unsigned long long k_to_v = (size_t(G - g) * pt * AHD + size_t(g) * AHD * pt) * 2;
    // this wave group's tile of a pair; a tile past the end re-reads the last real one (it is fully masked)
    auto tile_of = [&](int pair) { return min(2 * pair + grp, n_tiles - 1); };
    auto page_base = [&](int tile, unsigned* in_page0) {
        const int key0 = tile * AK, lpage = key0 / pt;
        *in_page0 = unsigned(key0 - lpage * pt);
        const unsigned long long off = pg_lds[lpage];
        const unsigned long long lo = (unsigned)__builtin_amdgcn_readfirstlane((int)unsigned(off));
        const unsigned long long hi = (unsigned)__builtin_amdgcn_readfirstlane((int)unsigned(off >> 32));
        return (const char*)kv.pool + ((hi << 32) | lo);
    };
    auto issue_k = [&](int pair) {
        unsigned in_page0;
        const char* kp = page_base(tile_of(pair), &in_page0) + size_t(in_page0) * (AHD * 2);
        unsigned char* sa = lds + (pair & 1) * A8_RING + grp * A_KBYTES;
#pragma unroll
        for (int i = 0; i < PER; ++i)
            __builtin_amdgcn_global_load_lds((const CAKE_GLOBAL_AS void*)(kp + size_t(i / KP) * (4 * QW * KP * AHD * 2) + koffp[i % KP]),
                                             (CAKE_LDS_AS void*)(sa + (wave + QW * i) * 1024), 16, 0, 0);
    };
    auto issue_v = [&](int pair) {
        unsigned in_page0;
        const char* vp = page_base(tile_of(pair), &in_page0) + k_to_v + size_t(in_page0) * 2;
        unsigned char* sa = lds + A8_VBASE + (pair & 1) * A8_RING + grp * A_KBYTES;
#pragma unroll
        for (int i = 0; i < PER; ++i)
            __builtin_amdgcn_global_load_lds((const CAKE_GLOBAL_AS void*)(vp + size_t(i) * (8 * QW) * pt * 2 + voff0),
                                             (CAKE_LDS_AS void*)(sa + (wave + QW * i) * 1024), 16, 0, 0);
    };

    const int sk = sigma16(lrow & 15);
    const int krow_base = (16 * (lrow >> 4) + sk) * (AHD * 2);
    int kaddr[AHD / 16];
#pragma unroll
    for (int ks = 0; ks < AHD / 16; ++ks) kaddr[ks] = grp * A_KBYTES + krow_base + (((2 * ks + lhalf) ^ sk) << 4);
    const int sv = (lrow >> 1) & 7;
    int vaddr[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) vaddr[j] = A8_VBASE + grp * A_KBYTES + lrow * (AK * 2) + (((2 * j + lhalf) ^ sv) << 4);

    f32x16 o[4];
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) o[t][v] = 0.f;
    // The running reference m_run of a query (log2 units) is SUBTRACTED INSIDE THE MFMA: the score
    // accumulators start from negm = -m_run instead of zero, so a finished score is already
    // s - m_run and the exponential needs no multiply-add of its own.  When the reference moves
    // (rarely, see RESCALE_LOG2) the scores formed against the old one are shifted by hand.
    float m_run = 0.f, l_part = 0.f;
    const f32x16 zero16 = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
    f32x16 negm = zero16;
    float corr_cur = 1.f, delta_cur = 0.f;
    bool moved_cur = false;
    constexpr float RESCALE_LOG2 = 6.0f;
    auto mask_tile = [&](f32x16* s, int tile) {
        const int key0 = tile * AK;
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                int key = key0 + 32 * t + (v & 7) + 8 * lhalf + 16 * (v >> 3);
                if (key > my_pos) s[t][v] = -INFINITY;
            }
    };
    auto part_max = [&](const f32x16* s, int part, float acc) {
#pragma unroll
        for (int i = 0; i < 8; ++i) acc = fmaxf(acc, s[part >> 1][8 * (part & 1) + i]);
        return acc;
    };
    // raw: this lane's largest score of the next tile, already relative to m_run
    auto finish_max = [&](float raw) {
        raw = fmaxf(raw, __shfl_xor(raw, 32, 64));
        moved_cur = raw > RESCALE_LOG2;
        if (__builtin_amdgcn_ballot_w64(moved_cur) != 0) {
            delta_cur = fmaxf(raw, 0.f);            // the reference only ever rises; -inf (all masked) leaves it
            corr_cur = __builtin_amdgcn_exp2f(-delta_cur);
            m_run += delta_cur;
            moved_cur = true;
        } else {
            delta_cur = 0.f;
            corr_cur = 1.0f;
        }
    };

    // iteration i: this group's tile 2i+grp is in K slot i&1 (scores already formed) and V slot i&1
    auto step = [&](int i, f32x16* s_cur, f32x16* s_nxt) {
        asm volatile("s_waitcnt vmcnt(0)");
        __builtin_amdgcn_s_barrier();
        if (i + 1 < n_pairs) issue_v(i + 1);
        if (i + 2 < n_pairs) issue_k(i + 2);
        const unsigned char* stk = lds + ((i + 1) & 1) * A8_RING;   // past the last pair: stale, result unused
        const unsigned char* stv = lds + (i & 1) * A8_RING;
        bf16x8 opa[4], opb[4], p[4];
        auto read_k = [&](bf16x8* dst, int grpk) {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                dst[e] = *(const bf16x8*)(stk + (e & 1) * 32 * (AHD * 2) + kaddr[2 * grpk + (e >> 1)]);
        };
        auto read_v = [&](bf16x8* dst, int j) {
#pragma unroll
            for (int e = 0; e < 4; ++e) dst[e] = *(const bf16x8*)(stv + e * 32 * (AK * 2) + vaddr[j]);
        };
        auto mma_k = [&](const bf16x8* src, int grpk) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int ks = 2 * grpk + (e >> 1), t = e & 1;
                s_nxt[t] = mfma32(src[e], qreg[ks], ks == 0 ? negm : s_nxt[t]);
            }
        };
        auto expo = [&](int grpe) {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                float x = __builtin_amdgcn_exp2f(s_cur[grpe >> 1][8 * (grpe & 1) + e]);
                l_part += x;
                p[grpe][e] = bf16_t(x);
            }
        };
        read_k(opa, 0);
        __builtin_amdgcn_sched_barrier(0);
        read_k(opb, 1); mma_k(opa, 0); expo(0);
        __builtin_amdgcn_sched_barrier(0);
        read_k(opa, 2); mma_k(opb, 1); expo(1);
        __builtin_amdgcn_sched_barrier(0);
        read_k(opb, 3); mma_k(opa, 2); expo(2);
        __builtin_amdgcn_sched_barrier(0);
        read_v(opa, 0); mma_k(opb, 3); expo(3);
        // the probabilities are only consumed after the branch below; pin them here, or the compiler
        // sinks the exponentials out of the block whose MFMAs they are meant to overlap with
#pragma unroll
        for (int e = 0; e < 4; ++e) asm volatile("" ::"v"(p[e]));
        asm volatile("" ::"v"(l_part));
        __builtin_amdgcn_sched_barrier(0);
        const int next_tile = 2 * (i + 1) + grp;
        if (next_tile >= first_masked) mask_tile(s_nxt, next_tile);   // also blanks tiles past the end
        float raw;
        read_v(opb, 1);
#pragma unroll
        for (int t = 0; t < 4; ++t) o[t] = mfma32(opa[t], p[0], o[t]);
        raw = part_max(s_nxt, 0, s_nxt[0][0]);
        raw = part_max(s_nxt, 1, raw);
        __builtin_amdgcn_sched_barrier(0);
        read_v(opa, 2);
#pragma unroll
        for (int t = 0; t < 4; ++t) o[t] = mfma32(opb[t], p[1], o[t]);
        raw = part_max(s_nxt, 2, raw);
        raw = part_max(s_nxt, 3, raw);
        __builtin_amdgcn_sched_barrier(0);
        read_v(opb, 3);
#pragma unroll
        for (int t = 0; t < 4; ++t) o[t] = mfma32(opa[t], p[2], o[t]);
        finish_max(raw);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int t = 0; t < 4; ++t) o[t] = mfma32(opb[t], p[3], o[t]);
        __builtin_amdgcn_sched_barrier(0);
        if (__builtin_amdgcn_ballot_w64(moved_cur) != 0) {
            l_part *= corr_cur;
#pragma unroll
            for (int t = 0; t < 4; ++t)
#pragma unroll
                for (int v = 0; v < 16; ++v) o[t][v] *= corr_cur;
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int v = 0; v < 16; ++v) s_nxt[t][v] -= delta_cur;   // formed against the old reference
#pragma unroll
            for (int v = 0; v < 16; ++v) negm[v] = -m_run;
        }
    };

    // prologue: K(0), V(0), K(1) in flight; K(0) landed; scores and reference of the first tile
    issue_k(0);
    issue_v(0);
    if (n_pairs > 1) {
        issue_k(1);
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * PER));
    } else {
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"(PER));
    }
    __builtin_amdgcn_s_barrier();
    f32x16 s_a[2], s_b[2];
    {
        const unsigned char* stk = lds;
#pragma unroll
        for (int ks = 0; ks < AHD / 16; ++ks)
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                bf16x8 a = *(const bf16x8*)(stk + t * 32 * (AHD * 2) + kaddr[ks]);
                s_a[t] = mfma32(a, qreg[ks], ks == 0 ? zero16 : s_a[t]);
            }
    }
    if (grp >= first_masked) mask_tile(s_a, grp);
    {
        // the first tile fixes the reference exactly; a row that sees none of its keys (possible for
        // the second wave half only) keeps reference 0 and contributes nothing
        float raw = s_a[0][0];
#pragma unroll
        for (int part = 0; part < 4; ++part) raw = part_max(s_a, part, raw);
        raw = fmaxf(raw, __shfl_xor(raw, 32, 64));
        m_run = raw > -INFINITY ? raw : 0.f;
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int v = 0; v < 16; ++v) s_a[t][v] -= m_run;
#pragma unroll
        for (int v = 0; v < 16; ++v) negm[v] = -m_run;
    }
    for (int i = 0; i < n_pairs; i += 2) {
        step(i, s_a, s_b);
        if (i + 1 < n_pairs) step(i + 1, s_b, s_a);
    }

    // merge the two key halves: group B parks (O, l, reference) in LDS, group A combines and stores
    __syncthreads();
    float* park = (float*)lds + size_t(wave) * 66 * 64 + lane;
    if (grp == 1) {
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int v = 0; v < 16; ++v) park[(16 * t + v) * 64] = o[t][v];
        park[64 * 64] = l_part;
        park[65 * 64] = m_run;
    }
    __syncthreads();
    if (grp == 0) {
        const float l_b = park[64 * 64];
        const float l_b_row = l_b + park[64 * 64 + ((lane ^ 32) - lane)];   // both half-waves of the row
        const float m_b = l_b_row > 0.f ? park[65 * 64] : -1.0e30f;         // a half that saw no key has no reference
        const float m = fmaxf(m_run, m_b);
        const float ca = __builtin_amdgcn_exp2f(m_run - m), cb = __builtin_amdgcn_exp2f(m_b - m);
        float l_mine = l_part * ca + l_b * cb;
        const float l_tot = l_mine + __shfl_xor(l_mine, 32, 64);
        const float inv = 1.0f / l_tot;
        const int row = q0 + wave * 32 + lrow;
        if (row < rows) {
            bf16_t* op = out + size_t(row) * n_q * AHD + h * AHD;
#pragma unroll
            for (int t = 0; t < 4; ++t)
#pragma unroll
                for (int v4 = 0; v4 < 4; ++v4) {
                    bf16x4 w;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int v = 4 * v4 + e;
                        w[e] = bf16_t((o[t][v] * ca + park[(16 * t + v) * 64] * cb) * inv);
                    }
                    *(bf16x4*)(op + t * 32 + 8 * v4 + 4 * lhalf) = w;
                }
        }
    }
}

// =====================================================================================
// One-token attention on the matrix cores (first-token step; bf16 pages, head_dim 128).
//
// The "queries" of a workgroup are the r query heads that share KV head g, all at the same
// position; they fill r of the 32 columns of the same transposed products as above
// (S^T = K Q^T, O^T = V^T P^T), the other columns stay zero.  That wastes most of the MFMA
// columns, which is free here: the kernel is bound by streaming the layer's K and V once, and
// one 32-wide MFMA step consumes 1 KB of them.  There is no reuse between waves, so nothing is
// staged in LDS: every lane loads its MFMA operand slices straight from the pages (K row
// sigma16-permuted as above, V^T row = head-dim index), a wave has the V^T tile of this step
// and the K tile of the next in flight while it works, and the four waves of a workgroup take
// the key tiles of the workgroup's range in turn.  Partial (max, sum, O) per wave are merged
// through LDS and written per key range for the combine kernel.
// =====================================================================================
__global__ void __launch_bounds__(256)
decode_attention_mfma_kernel(const float* __restrict__ q, float* __restrict__ part, int n_q, int n_keys,
                             int tiles_per_split, KvView kv) {
    extern __shared__ float dlds[];   // [4][r][AHD + 2]: O, then max (natural-log units), then sum
    const int g = blockIdx.x, split = blockIdx.y, n_splits = gridDim.y;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int lrow = lane & 31, lhalf = lane >> 5;
    const int r = n_q / kv.n_kv;
    const int pt = kv.page_tokens;
    const int n_tiles = (n_keys + AK - 1) / AK;
    const int tile_lo = split * tiles_per_split, tile_hi = min(tile_lo + tiles_per_split, n_tiles);
    const float sl2 = 0.08838834764831845f * 1.4426950408889634f;

    bf16x8 qB[AHD / 16];
#pragma unroll
    for (int ks = 0; ks < AHD / 16; ++ks)
#pragma unroll
        for (int e = 0; e < 8; ++e)
            qB[ks][e] = lrow < r ? bf16_t(q[size_t(g * r + lrow) * AHD + 16 * ks + 8 * lhalf + e] * sl2) : bf16_t(0.f);

    const int krow = 16 * (lrow >> 4) + sigma16(lrow & 15);
    const size_t layer_base = size_t(kv.layer) * kv.n_physical_pages;
    bf16x8 kA[2][AHD / 16], vA[4][4];
    auto tile_page = [&](int tile, int* in_page0) {
        const int key0 = tile * AK, lpage = key0 / pt;
        *in_page0 = key0 - lpage * pt;
        return (const bf16_t*)kv.pool + (layer_base + kv.block_table[lpage]) * kv.page_elems();
    };
    auto load_k = [&](int tile) {
        int in_page0;
        const bf16_t* kp = tile_page(tile, &in_page0) + (size_t(g) * pt + in_page0) * AHD + 8 * lhalf;
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int ks = 0; ks < AHD / 16; ++ks) kA[t][ks] = *(const bf16x8*)(kp + size_t(32 * t + krow) * AHD + 16 * ks);
    };
    auto load_v = [&](int tile) {
        int in_page0;
        const bf16_t* vp = tile_page(tile, &in_page0) + size_t(kv.n_kv) * pt * AHD + size_t(g) * AHD * pt + in_page0 + 8 * lhalf;
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
#pragma unroll
            for (int c = 0; c < 4; ++c) vA[dt][c] = *(const bf16x8*)(vp + size_t(32 * dt + lrow) * pt + 16 * c);
    };

    f32x16 o[4];
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) o[t][v] = 0.f;
    float m_run = -1.0e30f, l_part = 0.f;   // finite start: exp2(-inf - m) of a masked key is 0, never NaN
    const f32x16 zero16 = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};

    int tile = tile_lo + wave;
    if (tile < tile_hi) load_k(tile);
    for (; tile < tile_hi; tile += 4) {
        load_v(tile);
        f32x16 s[2];
#pragma unroll
        for (int ks = 0; ks < AHD / 16; ++ks)
#pragma unroll
            for (int t = 0; t < 2; ++t) s[t] = mfma32(kA[t][ks], qB[ks], ks == 0 ? zero16 : s[t]);
        if (tile + 4 < tile_hi) load_k(tile + 4);
        if ((tile + 1) * AK > n_keys) {   // ragged last tile: keys past the prompt
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int v = 0; v < 16; ++v)
                    if (tile * AK + 32 * t + 16 * (v >> 3) + 8 * lhalf + (v & 7) >= n_keys) s[t][v] = -INFINITY;
        }
        float mx = s[0][0];
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int v = 0; v < 16; ++v) mx = fmaxf(mx, s[t][v]);
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        const float m_new = fmaxf(m_run, mx);
        const float corr = __builtin_amdgcn_exp2f(m_run - m_new);
        m_run = m_new;
        if (__builtin_amdgcn_ballot_w64(corr != 1.0f) != 0) {   // what was summed so far moves to the new reference
            l_part *= corr;
#pragma unroll
            for (int t = 0; t < 4; ++t)
#pragma unroll
                for (int v = 0; v < 16; ++v) o[t][v] *= corr;
        }
        bf16x8 pB[4];
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const float x = __builtin_amdgcn_exp2f(s[t][v] - m_new);
                l_part += x;
                pB[2 * t + (v >> 3)][v & 7] = bf16_t(x);
            }
#pragma unroll
        for (int c = 0; c < 4; ++c)
#pragma unroll
            for (int dt = 0; dt < 4; ++dt) o[dt] = mfma32(vA[dt][c], pB[c], o[dt]);
    }

    // merge the four waves; column n of a wave belongs to query head g*r + n
    const float l_tot = l_part + __shfl_xor(l_part, 32, 64);
    if (lrow < r) {
        float* w = dlds + size_t(wave * r + lrow) * (AHD + 2);
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
#pragma unroll
            for (int v = 0; v < 16; ++v) w[32 * dt + 8 * (v >> 2) + 4 * lhalf + (v & 3)] = o[dt][v];
        if (lhalf == 0) { w[AHD] = m_run * 0.6931471805599453f; w[AHD + 1] = l_tot; }
    }
    __syncthreads();
    for (int idx = tid; idx < r * AHD; idx += 256) {
        const int j = idx / AHD, d = idx % AHD;
        float m = -INFINITY;
#pragma unroll
        for (int w = 0; w < 4; ++w) m = fmaxf(m, dlds[size_t(w * r + j) * (AHD + 2) + AHD]);
        float num = 0.f, den = 0.f;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const float* src = dlds + size_t(w * r + j) * (AHD + 2);
            const float c = __expf(src[AHD] - m);
            num += src[d] * c;
            den += src[AHD + 1] * c;
        }
        float* dst = part + (size_t(g * r + j) * n_splits + split) * (AHD + 2);
        dst[d] = num;
        if (d == 0) { dst[AHD] = m; dst[AHD + 1] = den; }
    }
}

bool decode_attention_mfma_supported(int dtype, int head_dim, int page_tokens, int r) {
    return dtype == 1 && head_dim == AHD && page_tokens % AK == 0 && r >= 1 && r <= 32;
}

// Writes n_splits partial results per query head into `part` ([n_q][n_splits][head_dim + 2]).
hipError_t launch_decode_attention_mfma(const float* q, float* part, int n_q, int n_keys, int tiles_per_split,
                                        int n_splits, const KvView& kv, hipStream_t st) {
    const int r = n_q / kv.n_kv;
    const size_t lds = size_t(4) * r * (AHD + 2) * sizeof(float);
    hipLaunchKernelGGL(decode_attention_mfma_kernel, dim3(kv.n_kv, n_splits), dim3(256), lds, st, q, part, n_q, n_keys,
                       tiles_per_split, kv);
    return hipGetLastError();
}

bool attention_mfma_supported(int head_dim, int page_tokens) {
    return head_dim == AHD && page_tokens % AK == 0;
}

hipError_t launch_attention_mfma(const void* q, void* out, int n_q, int tok_begin, int rows, const KvView& kv,
                                 hipStream_t st, int variant) {
    if (rows <= 0) return hipSuccess;
    static bool attr_set = false;
    constexpr int LDS_MAX = 160 * 1024;
    const int table = 8 * ((tok_begin + rows - 1) / kv.page_tokens + 1);   // one 8-byte page offset per logical page
    const int q_tiles = (rows + AQ - 1) / AQ;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void*)attention_mfma_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, LDS_MAX);
        if (e == hipSuccess) e = hipFuncSetAttribute((const void*)attention_mfma8_kernel<4>, hipFuncAttributeMaxDynamicSharedMemorySize, LDS_MAX);
        if (e == hipSuccess) e = hipFuncSetAttribute((const void*)attention_mfma8_kernel<2>, hipFuncAttributeMaxDynamicSharedMemorySize, LDS_MAX);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    if (variant == 1) {
        const int LDS = A_STAGES * A_STAGE + table;
        if (LDS > LDS_MAX) return hipErrorInvalidValue;
        hipLaunchKernelGGL(attention_mfma_kernel, dim3(q_tiles * n_q), dim3(256), LDS, st, (const bf16_t*)q, (bf16_t*)out, n_q,
                           tok_begin, rows, kv, q_tiles);
    } else {
        const int LDS = A8_TABLE + table;
        if (LDS > LDS_MAX) return hipErrorInvalidValue;
        // 64-query workgroups (four waves, one per SIMD: about 0.85 of the eight-wave kernel's rate per CU) when
        // they shorten the busiest CU's work: rounds of workgroups over 256 CUs times queries per workgroup
        const int q_tiles64 = (rows + 63) / 64;
        const long rounds128 = (long(q_tiles) * n_q + 255) / 256, rounds64 = (long(q_tiles64) * n_q + 255) / 256;
        const bool small_wins = q_tiles64 > q_tiles && double(rounds64) * 64 / 0.85 < double(rounds128) * 128;
        if (variant == 3 || (variant == 0 && small_wins))
            hipLaunchKernelGGL(attention_mfma8_kernel<2>, dim3(q_tiles64 * n_q), dim3(256), LDS, st, (const bf16_t*)q, (bf16_t*)out,
                               n_q, tok_begin, rows, kv, q_tiles64);
        else
            hipLaunchKernelGGL(attention_mfma8_kernel<4>, dim3(q_tiles * n_q), dim3(512), LDS, st, (const bf16_t*)q, (bf16_t*)out,
                               n_q, tok_begin, rows, kv, q_tiles);
    }
    return hipGetLastError();
}

}  // namespace cake
