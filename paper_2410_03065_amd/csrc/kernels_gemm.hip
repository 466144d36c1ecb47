// bf16 MFMA GEMMs for gfx950: the four projections of the decoder block
// (Sec. 3: Q = X W_Q, K = X W_K, V = X W_V, and the block's output and feed-forward products).
//
// MFMA shape used throughout: v_mfma_f32_32x32x16_bf16.  For D[32x32] += A[32x16] * B[16x32]
// lane l supplies A[l%32][8*(l/32) .. +7] and B[8*(l/32) .. +7][l%32], and holds
// D[8*(v/4) + 4*(l/32) + v%4][l%32] in accumulator register v (0..15).
#include <mutex>
#include <type_traits>
#include <vector>

#include "kernels.hpp"

namespace cake {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// =====================================================================================
// GEMM: out[M][N] = a[M][K] * w[N][K]^T, bf16 in, float32 accumulate.
//
// Workgroup tile BM x BN = (WAVES_M*WTM*32) x (WAVES_N*WTN*32); each wave owns WTM x WTN MFMA
// tiles.  K is consumed in BK-deep slices (32 or 64) held in a ring of STAGES LDS buffers that are filled
// by direct global->LDS loads (global_load_lds_dwordx4: 64 lanes x 16 B land contiguously, so
// the bank swizzle is applied by choosing which global chunk each lane fetches).  A slice row
// is 64 B or 128 B of 16-byte chunks; chunk c of row r is stored at c ^ ((r >> 2) & 3) resp.
// c ^ ((r >> 1) & 7), so the 16 rows that one quarter-wave reads with ds_read_b128 cover all
// 64 LDS banks once.  64-deep slices ask L2 for whole 128-byte lines (half as many requests).
//
// Software pipeline per slice (BK/16 MFMA steps of depth 16): while a step's MFMAs issue, the
// next step's operands are read; before the last step the wave waits for the NEXT slice's loads
// (vmcnt), meets the other waves at a bare s_barrier (no fence: a fence would drain every load in
// flight), refills the buffer freed one slice ago, and runs the last step's MFMAs while reading
// the next slice's first operands.  sched_group_barrier pins the 2-MFMA / 1-ds_read interleave.
//
// The block index is remapped so that workgroups that share a weight panel (the tiles_m tiles
// of one n-panel) sit on the same XCD and run at the same time: the panel is then fetched from
// HBM once and hit in that XCD's L2 by the others.
//
// Epilogues: store float32; add into a float32 residual stream; SwiGLU, where each wave's
// n-tiles alternate gate / up rows of the two weight matrices, so silu(gate) * up of one
// output column is formed in registers and the tile yields BN/2 output columns.
//
// Split K (ksplit > 1, not for SwiGLU): when a GEMM has too few large tiles to fill the chip, each
// tile is computed by ksplit workgroups, one per K range.  A workgroup writes its accumulators to
// its slot of a float32 workspace (in accumulator order, so the stores are contiguous), makes them
// visible device-wide and takes a ticket from the tile's counter; the one that draws the last
// ticket reads all parts back and adds them IN K-RANGE ORDER, so the result does not depend on
// which workgroup came last, runs the ordinary epilogue and puts the counter back to zero.  Nobody
// waits for anybody.  Launches that share a workspace must not overlap (one stream).
//
// Waves dividing K (KW = 2, 64-deep slices): every spatial part of the tile belongs to two waves,
// one taking the first two 16-deep steps of each slice, the other the last two.  The LDS traffic
// per MFMA is unchanged; what it buys is two waves per SIMD for a small tile (one CU's 128 x 128),
// so that one wave's waits (LDS, barrier) hide behind the other's MFMAs.  After the last slice the
// pair exchanges, through the idle ring, the 32-row bands each does not finish, and each runs the
// epilogue for its own bands.
// =====================================================================================
#define CAKE_GLOBAL_AS __attribute__((address_space(1)))
#define CAKE_LDS_AS __attribute__((address_space(3)))

// 16 consecutive rows must fall into 16 different 16-byte slots of a 256-byte bank window
template <int BK> __device__ __forceinline__ int gemm_swz(int row) { return BK == 64 ? ((row >> 1) & 7) : ((row >> 2) & 3); }

template <int WTM, int WTN, int WAVES_M, int WAVES_N, int BK, int STAGES, int EPI, int KW>
__global__ void __launch_bounds__(64 * WAVES_M * WAVES_N * KW)
gemm_mfma_kernel(const bf16_t* __restrict__ A, const bf16_t* __restrict__ W, const bf16_t* __restrict__ W2,
                 void* __restrict__ outv, int M, int N, int K, int tiles_m, int tiles_n,
                 float* __restrict__ part, unsigned* __restrict__ counters, int ksplit) {
    constexpr int NWS = WAVES_M * WAVES_N;   // waves that divide the tile in space
    constexpr int NW = NWS * KW;             // times the waves that divide each slice along K
    constexpr int KS = BK / 16 / KW;         // 16-deep MFMA steps per slice and wave
    static_assert(KW == 1 || (KW == 2 && BK == 64), "K is divided between two waves at most, two steps each");
    static_assert(KW == 1 || STAGES * (WAVES_M * WTM + WAVES_N * WTN) * 32 * BK * 2 >= NWS * WTM * WTN * 4096, "the ring holds the exchange");
    constexpr int BM = WAVES_M * WTM * 32, BN = WAVES_N * WTN * 32;
    constexpr int ROWB = BK * 2, CPR = BK / 8, RPL = 64 / CPR;
    constexpr int A_BYTES = BM * ROWB, B_BYTES = BN * ROWB, STAGE = A_BYTES + B_BYTES;
    constexpr int A_PER = A_BYTES / 1024 / NW, B_PER = B_BYTES / 1024 / NW, PER_TILE = A_PER + B_PER;
    static_assert((A_BYTES / 1024) % NW == 0 && (B_BYTES / 1024) % NW == 0, "slice loads must divide among the waves");
    static_assert(STAGES >= 3 && (STAGES - 2) * PER_TILE < 64, "vmcnt range");
    static_assert(EPI != EPI_SWIGLU || WTN % 2 == 0, "gate/up pairs");
    extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int kw = wave / NWS, wsp = wave % NWS;
    const int wm = wsp / WAVES_N, wn = wsp % WAVES_N;
    const int lrow = lane & 31, lhalf = lane >> 5;

    const int nb = tiles_m * tiles_n;
    const int bid = blockIdx.x;
    int t, kpart = 0;
    if (EPI == EPI_SWIGLU || ksplit == 1) {
        t = (nb % 8 == 0) ? (bid % 8) * (nb / 8) + bid / 8 : bid;
    } else if (8 % ksplit == 0 && nb % (8 / ksplit) == 0) {
        // block b runs on XCD b % 8: an XCD takes one K range of a group of whole weight panels
        const int xcd = bid & 7, per_group = nb / (8 / ksplit);
        kpart = xcd % ksplit;
        t = (xcd / ksplit) * per_group + (bid >> 3);
    } else {
        kpart = bid % ksplit;
        t = bid / ksplit;
    }
    const int tm = t % tiles_m, tn = t / tiles_m;
    const int k_begin = kpart * (K / ksplit);
    const int m0 = tm * BM;
    const int n0 = tn * (EPI == EPI_SWIGLU ? BN / 2 : BN);   // first output column of the tile

    // first row of weight-tile row `row` (for SwiGLU the tile's rows alternate between the two matrices)
    auto w_row = [&](int row) -> const bf16_t* {
        if (EPI == EPI_SWIGLU) {
            int wcol = row / (WTN * 32), j = (row / 32) % WTN, c = row % 32;
            return ((j & 1) ? W2 : W) + size_t(n0 + wcol * (WTN / 2) * 32 + (j >> 1) * 32 + c) * K + k_begin;
        }
        return W + size_t(n0 + row) * K + k_begin;
    };
    // global source of this lane for each 1 KB wave-load (16 rows x 64 B)
    const int lr = lane / CPR, lpos = lane % CPR;
    const bf16_t* ag[A_PER];
    const bf16_t* bg[B_PER];
#pragma unroll
    for (int i = 0; i < A_PER; ++i) {
        int row = (wave + i * NW) * RPL + lr;
        ag[i] = A + size_t(min(m0 + row, M - 1)) * K + k_begin + (lpos ^ gemm_swz<BK>(row)) * 8;
    }
#pragma unroll
    for (int i = 0; i < B_PER; ++i) {
        int row = (wave + i * NW) * RPL + lr;
        bg[i] = w_row(row) + (lpos ^ gemm_swz<BK>(row)) * 8;
    }
    // Wave-load idx of a slice (0 .. PER_TILE-1: the A loads, then the W loads) belongs to part idx % KS.  A slice
    // is not requested in one burst: the texture addresser takes 16 cycles per wave-load and a full address
    // FIFO blocks the issuing wave, MFMAs included.  Part 0 goes out after the barrier that frees the buffer,
    // part p in step p-1 of the following slice, each load between two operand reads.
    auto issue_one = [&](unsigned char* sa, int k0, int idx) {
        if (idx < A_PER)
            __builtin_amdgcn_global_load_lds((const CAKE_GLOBAL_AS void*)(ag[idx] + k0),
                                             (CAKE_LDS_AS void*)(sa + (wave + idx * NW) * 1024), 16, 0, 0);
        else
            __builtin_amdgcn_global_load_lds((const CAKE_GLOBAL_AS void*)(bg[idx - A_PER] + k0),
                                             (CAKE_LDS_AS void*)(sa + A_BYTES + (wave + (idx - A_PER) * NW) * 1024), 16, 0, 0);
    };
    auto issue = [&](int stage, int k0) {   // a whole slice at once (prologue)
        unsigned char* sa = lds + stage * STAGE;
#pragma unroll
        for (int idx = 0; idx < PER_TILE; ++idx) issue_one(sa, k0, idx);
    };
    constexpr int PART_MAX = (PER_TILE + KS - 1) / KS;

    f32x16 acc[WTM][WTN];
#pragma unroll
    for (int i = 0; i < WTM; ++i)
#pragma unroll
        for (int j = 0; j < WTN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    const int sw = gemm_swz<BK>(lrow);  // tile rows start at multiples of 32, so the swizzle depends on lrow only
    int koff[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) koff[ks] = ((2 * (kw * KS + ks) + lhalf) ^ sw) << 4;
    const int a_row_off = (wm * WTM * 32 + lrow) * ROWB;
    const int b_row_off = A_BYTES + (wn * WTN * 32 + lrow) * ROWB;
    auto rd = [&](bf16x8* a, bf16x8* bb, int stage, int koffv) {
        const unsigned char* st = lds + stage * STAGE;
#pragma unroll
        for (int i = 0; i < WTM; ++i) a[i] = *(const bf16x8*)(st + a_row_off + i * 32 * ROWB + koffv);
#pragma unroll
        for (int j = 0; j < WTN; ++j) bb[j] = *(const bf16x8*)(st + b_row_off + j * 32 * ROWB + koffv);
    };
    // the same reads with part `part` of the slice bound for `stage_ld` dealt between them (a load to LDS and an
    // LDS read may not pass each other, so this source order is the issue order)
    auto rd_ld = [&](bf16x8* a, bf16x8* bb, int stage, int koffv, int stage_ld, int k0, auto part_tag) {
        constexpr int PART = decltype(part_tag)::value;
        const unsigned char* st = lds + stage * STAGE;
        unsigned char* sa = lds + stage_ld * STAGE;
#pragma unroll
        for (int r = 0; r < WTM + WTN; ++r) {
            if (r < WTM) a[r] = *(const bf16x8*)(st + a_row_off + r * 32 * ROWB + koffv);
            else bb[r - WTM] = *(const bf16x8*)(st + b_row_off + (r - WTM) * 32 * ROWB + koffv);
            if (r < PART_MAX && PART + r * KS < PER_TILE) issue_one(sa, k0, PART + r * KS);
        }
    };
    auto mm = [&](const bf16x8* a, const bf16x8* bb) {
#pragma unroll
        for (int i = 0; i < WTM; ++i)
#pragma unroll
            for (int j = 0; j < WTN; ++j) acc[i][j] = mfma32(a[i], bb[j], acc[i][j]);
    };
    auto interleave = [&]() {
#pragma unroll
        for (int i = 0; i < WTM + WTN; ++i) {
            if constexpr ((WTM * WTN) / (WTM + WTN) > 0)
                __builtin_amdgcn_sched_group_barrier(0x008, (WTM * WTN) / (WTM + WTN), 0);  // MFMA
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);                          // DS read
        }
    };

    auto interleave_ld = [&](auto part_tag) {
        constexpr int PART = decltype(part_tag)::value;
#pragma unroll
        for (int i = 0; i < WTM + WTN; ++i) {
            if constexpr ((WTM * WTN) / (WTM + WTN) > 0)
                __builtin_amdgcn_sched_group_barrier(0x008, (WTM * WTN) / (WTM + WTN), 0);  // MFMA
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);                          // DS read
            if (i < PART_MAX && PART + i * KS < PER_TILE) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);   // load
        }
    };
    static_assert(PART_MAX <= WTM + WTN, "one load per operand read at most");

    const int nk = K / ksplit / BK;
    // Slices 0 .. n_steady-1 each request the slice STAGES-1 ahead (part 0 in their last step, the other parts in
    // the first steps of the slice after them); the slices after that request nothing.
    const int n_steady = nk > STAGES - 1 ? nk - (STAGES - 1) : 0;
    // prologue: STAGES-1 slices in flight (of the last of them only part 0 if slice 0 will deal out the rest);
    // slice 0 landed; its step-0 operands in registers
#pragma unroll
    for (int st = 0; st < STAGES - 2; ++st)
        if (st < nk) issue(st, st * BK);
    if (STAGES - 2 < nk) {
        if (n_steady > 0) {
            unsigned char* sa = lds + (STAGES - 2) * STAGE;
#pragma unroll
            for (int r = 0; r < PART_MAX; ++r)
                if (r * KS < PER_TILE) issue_one(sa, (STAGES - 2) * BK, r * KS);
        } else {
            issue(STAGES - 2, (STAGES - 2) * BK);
        }
    }
    constexpr int PART0 = (PER_TILE + KS - 1) / KS;   // loads in part 0
    if (n_steady > 0) asm volatile("s_waitcnt vmcnt(%0)" ::"n"((STAGES - 3) * PER_TILE + PART0));
    else if (nk >= STAGES - 1) asm volatile("s_waitcnt vmcnt(%0)" ::"n"((STAGES - 2) * PER_TILE));
    else asm volatile("s_waitcnt vmcnt(0)");
    __builtin_amdgcn_s_barrier();
    bf16x8 opa[2][WTM], opb[2][WTN];   // operands of the current and the next step
    rd(opa[0], opb[0], 0, koff[0]);
    // One slice.  NEW: this slice requests part 0 of slice kt+STAGES-1 after its barrier.  DEFER: its first
    // steps request the remaining parts of slice kt+STAGES-2 (whose part 0 the slice before requested).
    auto slice = [&](int kt, auto new_tag, auto defer_tag) {
        constexpr bool NEW = decltype(new_tag)::value, DEFER = decltype(defer_tag)::value;
        const int cur = kt % STAGES;
        const int st_prev = (kt + STAGES - 2) % STAGES, k_prev = (kt + STAGES - 2) * BK;
        // steps 0 .. KS-2: this step's MFMAs, next step's operands from the same slice
        [&]<int... PS>(std::integer_sequence<int, PS...>) {
            ([&] {
                constexpr int ks = PS;
                if constexpr (DEFER) {
                    rd_ld(opa[(ks + 1) & 1], opb[(ks + 1) & 1], cur, koff[ks + 1], st_prev, k_prev, std::integral_constant<int, ks + 1>{});
                    mm(opa[ks & 1], opb[ks & 1]);
                    interleave_ld(std::integral_constant<int, ks + 1>{});
                } else {
                    rd(opa[(ks + 1) & 1], opb[(ks + 1) & 1], cur, koff[ks + 1]);
                    mm(opa[ks & 1], opb[ks & 1]);
                    interleave();
                }
            }(), ...);
        }(std::make_integer_sequence<int, KS - 1>{});
        // slice kt+1 must have landed before the last step reads its first operands: in the steady state everything
        // but the STAGES-3 slices after it may still be out
        if constexpr (NEW || DEFER) asm volatile("s_waitcnt vmcnt(%0)" ::"n"((STAGES - 3) * PER_TILE));
        else asm volatile("s_waitcnt vmcnt(0)");
        __builtin_amdgcn_s_barrier();
        // every wave has finished reading slice kt-1: its buffer is refilled, starting now
        if constexpr (NEW) {
            rd_ld(opa[0], opb[0], (kt + 1) % STAGES, koff[0], (kt + STAGES - 1) % STAGES, (kt + STAGES - 1) * BK, std::integral_constant<int, 0>{});
            mm(opa[(KS - 1) & 1], opb[(KS - 1) & 1]);
            interleave_ld(std::integral_constant<int, 0>{});
        } else {
            // past the last slice this reads stale LDS that is never used
            rd(opa[0], opb[0], (kt + 1) % STAGES, koff[0]);
            mm(opa[(KS - 1) & 1], opb[(KS - 1) & 1]);
            interleave();
        }
    };
    {
        int kt = 0;
        for (; kt < n_steady; ++kt) slice(kt, std::true_type{}, std::true_type{});
        if (n_steady > 0) { slice(kt, std::false_type{}, std::true_type{}); ++kt; }
        for (; kt < nk; ++kt) slice(kt, std::false_type{}, std::false_type{});
    }

    // With K divided between two waves, wave kw finishes the 32-row bands i with (i & 1) == kw.
    auto band_is_mine = [&](int i) { return KW == 1 || (i & 1) == kw; };
    if constexpr (KW > 1) {
        // The two waves that shared a tile along K add up: each hands the other, through the ring (idle
        // by now), the bands it does not finish, and adds what it is handed (a + b = b + a exactly, so
        // the sum does not depend on which of the two holds it).
        static_assert(WTM % 2 == 0, "bands are dealt alternately");
        __syncthreads();
        float4* spot = (float4*)(lds + wsp * (WTM * WTN * 4096));
#pragma unroll
        for (int i = 0; i < WTM; ++i)
            if (!band_is_mine(i)) {
#pragma unroll
                for (int j = 0; j < WTN; ++j)
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        spot[((i * WTN + j) * 4 + q) * 64 + lane] =
                            make_float4(acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]);
            }
        __syncthreads();
#pragma unroll
        for (int i = 0; i < WTM; ++i)
            if (band_is_mine(i)) {
#pragma unroll
                for (int j = 0; j < WTN; ++j)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const float4 p = spot[((i * WTN + j) * 4 + q) * 64 + lane];
                        acc[i][j][4 * q] += p.x; acc[i][j][4 * q + 1] += p.y; acc[i][j][4 * q + 2] += p.z; acc[i][j][4 * q + 3] += p.w;
                    }
            }
    }
    const int tid_s = wsp * 64 + lane;   // thread index among the waves that hold a result

    if constexpr (EPI != EPI_SWIGLU) {
        if (ksplit > 1) {
            // Parts go through the workspace with device-scope accesses (the sc1 bit: written through to,
            // and read from, the level every XCD shares), so no cache-wide write-back or invalidate is
            // needed: a wave waits until its stores are acknowledged, the barrier collects all waves, then
            // one thread draws the ticket; the loads of the last workgroup are issued after its ticket.
            constexpr int TILE_B = BM * BN * 4, NT = NWS * 64;
            const __amdgpu_buffer_rsrc_t ws = __builtin_amdgcn_make_buffer_rsrc(part, 0, tiles_m * tiles_n * ksplit * TILE_B, 0x00020000);
            const unsigned slots = unsigned(t) * ksplit * TILE_B;
            const unsigned mine = slots + unsigned(kpart) * TILE_B;
            constexpr int DEVICE_SCOPE = 16;   // sc1
#pragma unroll
            for (int i = 0; i < WTM; ++i)
#pragma unroll
                for (int j = 0; j < WTN; ++j)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        if (!band_is_mine(i)) continue;
                        u32x4 v = {__float_as_uint(acc[i][j][4 * q]), __float_as_uint(acc[i][j][4 * q + 1]),
                                   __float_as_uint(acc[i][j][4 * q + 2]), __float_as_uint(acc[i][j][4 * q + 3])};
                        __builtin_amdgcn_raw_buffer_store_b128(v, ws, mine + (((i * WTN + j) * 4 + q) * NT + tid_s) * 16, 0, DEVICE_SCOPE);
                    }
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __syncthreads();
            if (tid == 0) *(volatile unsigned*)lds = __hip_atomic_fetch_add(&counters[t], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __syncthreads();
            if (*(volatile unsigned*)lds != unsigned(ksplit - 1)) return;
            // every part, this workgroup's too, comes from the workspace, in K-range order
            auto sum_parts = [&](auto nparts) {
                constexpr int NP = decltype(nparts)::value;
#pragma unroll
                for (int i = 0; i < WTM; ++i)
#pragma unroll
                    for (int j = 0; j < WTN; ++j) {
                        if (!band_is_mine(i)) continue;
                        u32x4 p[NP][4];
#pragma unroll
                        for (int sp = 0; sp < NP; ++sp)
#pragma unroll
                            for (int q = 0; q < 4; ++q)
                                p[sp][q] = __builtin_amdgcn_raw_buffer_load_b128(ws, slots + sp * TILE_B + (((i * WTN + j) * 4 + q) * NT + tid_s) * 16, 0, DEVICE_SCOPE);
#pragma unroll
                        for (int q = 0; q < 4; ++q)
#pragma unroll
                            for (int e = 0; e < 4; ++e) {
                                float tot = __uint_as_float(p[0][q][e]);
#pragma unroll
                                for (int sp = 1; sp < NP; ++sp) tot += __uint_as_float(p[sp][q][e]);
                                acc[i][j][4 * q + e] = tot;
                            }
                    }
            };
            if (ksplit == 2) sum_parts(std::integral_constant<int, 2>{});
            else if (ksplit == 4) sum_parts(std::integral_constant<int, 4>{});
            else sum_parts(std::integral_constant<int, 8>{});
            if (tid == 0) counters[t] = 0;   // every ticket of this tile is drawn: ready for the next launch
        }
    }

    // epilogue
#pragma unroll
    for (int i = 0; i < WTM; ++i) {
        if (!band_is_mine(i)) continue;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            int row = m0 + (wm * WTM + i) * 32 + 8 * (v >> 2) + 4 * lhalf + (v & 3);
            if (row >= M) continue;
            if (EPI == EPI_SWIGLU) {
#pragma unroll
                for (int j = 0; j < WTN; j += 2) {
                    int col = n0 + wn * (WTN / 2) * 32 + (j >> 1) * 32 + lrow;
                    float g = acc[i][j][v], u = acc[i][j + 1][v];
                    // silu(g) * u; the hardware reciprocal (1 ulp) instead of an IEEE division: the result is rounded to bf16
                    ((bf16_t*)outv)[size_t(row) * N + col] = bf16_t(g * __builtin_amdgcn_rcpf(1.0f + __expf(-g)) * u);
                }
            } else {
#pragma unroll
                for (int j = 0; j < WTN; ++j) {
                    int col = n0 + (wn * WTN + j) * 32 + lrow;
                    float* o = (float*)outv + size_t(row) * N + col;
                    if (EPI == EPI_RESIDUAL_F32) *o += acc[i][j][v];
                    else *o = acc[i][j][v];
                }
            }
        }
    }
}

// =====================================================================================
// Persistent GEMM for shapes with many 256 x 256 tiles (the gate/up product): out = a * w^T as above.
//
// What bounds a 256 x 256 tile on this chip is the LDS port, then the texture addresser: with eight
// waves of 128 x 64 the operand reads plus the incoming tile data keep the LDS busy for as long as the
// MFMAs take, and a burst of loads after the slice barrier fills the addresser's FIFO, which blocks the
// issuing wave (and its MFMAs) until it drains.  So here:
//  * four waves of 128 x 128 (8 x 8 tiles of v_mfma_f32_16x16x32_bf16, 256 accumulator registers each):
//    16 operand reads per 64 MFMAs instead of 24, two thirds of the LDS read traffic;
//  * K in 64-deep slices (whole 128-byte lines from L2, half the requests of 32-deep slices), each slice
//    two 32 KB items (the A rows, the W rows) in a ring of five LDS slots filled by buffer loads to LDS;
//    row r of an item stores its 16-byte chunk c at c ^ ((r >> 1) & 7), so the sixteen rows a
//    quarter-wave reads hit all 64 banks once (the rows of an item are permuted in LDS, see tile_off);
//  * a slice is two phases of 64 MFMAs: phase A computes k-step 0 while the operands of k-step 1 are read
//    and the W item of slice g+2 is loaded; then one barrier (this slice's slots are free, the next slice
//    has landed); phase B computes k-step 1 while the first operands of slice g+1 are read and the A item
//    of slice g+2 is loaded into a slot just freed.  Inside a phase the source interleaves two operand
//    reads with one load, eight times, and sched_group_barrier pins 2 MFMAs between any two of them: no
//    burst anywhere (a load to LDS and an LDS read may not pass each other, so source order is issue
//    order);
//  * workgroups are persistent: each takes its tiles one after another, the loads of the next tile's first
//    slices are already in flight during the epilogue, and the grid is a whole number of rounds
//    (448 tiles -> 224 workgroups of two tiles).  Past the end of its tiles a workgroup's loads use an
//    empty buffer descriptor: they return zeros into slots nobody reads again, which keeps the load count
//    per phase, and with it the s_waitcnt arithmetic, the same in every iteration.
// Rows past M are read as zeros and their stores dropped by the buffer bounds checks.
// SwiGLU: the 256 W rows of a tile alternate between the two matrices in groups of sixteen (even MFMA
// tiles of a wave hold gate columns, odd ones the same columns of up), so the tile yields 128 output
// columns and silu(gate) * up is formed in registers.
// =====================================================================================
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
constexpr int P_ITEM = 256 * 128, P_SLOTS = 5, P_LDS = P_ITEM * P_SLOTS;
// Operand fragments are held as four 32-bit words (eight bf16 values along K).
typedef __attribute__((__vector_size__(4 * sizeof(int)))) int p256_frag_t;

// An MFMA as an asm statement with the accumulator tied to an AGPR tuple: the 64 accumulators of a wave then
// fill the AGPR file exactly and stay where they are (left to itself the allocator rotates them through
// misaligned tuples with a hundred register copies per slice, each waiting for the MFMA that wrote its source),
// and, being volatile, the statements pin the order of the LDS reads and loads written between them: source
// order is issue order.  The compiler's hazard handling does not see them: the kernel puts the wait states
// between the last MFMA of an item and the first read of an accumulator itself.
__device__ __forceinline__ void p256_mfma(f32x4& c, const p256_frag_t& a, const p256_frag_t& b) {
    asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(c) : "v"(a), "v"(b));
}

// Column panels.  The N dimension is cut into panels of 8, 6 or 4 MFMA tiles per wave (256, 192 or 128 rows of
// W; the widest first), so that the number of work items can be made a whole number of rounds over the CUs where
// 256-wide panels alone leave some idle (448 items on 256 CUs: 224 workgroups of two; with 64 panels of 256 and
// 64 of 192 every CU gets one item of each width, 7/8 of the time).  A work item is one panel x one band of 256
// rows of A (x one K range when K is split, 256-wide panels only).
struct P256Plan { int n8, n6, n4; };

// SPLIT: the instantiation that runs one K range per item and leaves its accumulators in the workspace (256-wide
// panels only); kept apart so that each instantiation has a single epilogue path.
template <int EPI, bool SPLIT>
__global__ void __launch_bounds__(256)
gemm_p256_kernel(const bf16_t* __restrict__ A, const bf16_t* __restrict__ W, const bf16_t* __restrict__ W2,
                 void* __restrict__ outv, int M, int N, int K, int tiles_m, P256Plan plan, int tiles_per_wg,
                 float* __restrict__ part, int ksplit) {
    extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];
    constexpr int UNIT = EPI == EPI_SWIGLU ? 16 : 32;   // output columns per MFMA tile pair of a wave pair: panel of class c = c * UNIT columns
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;
    const int l16 = lane & 15, lq = lane >> 4;
    // Items are numbered class-major (all 256-wide panels, then the 192-wide, then the 128-wide), within a class
    // panel-major, and over the K ranges range-major (item = range * tiles + tile).
    const int t8 = tiles_m * plan.n8, t6 = tiles_m * plan.n6, n_tiles = t8 + t6 + tiles_m * plan.n4;
    const int nb = n_tiles * ksplit, G = gridDim.x;
    // item u of this workgroup: one per round of G items.  Workgroup b runs on XCD b % 8: where the grid divides,
    // an XCD takes G / 8 consecutive items of a round (whole weight panels, shared through its L2).
    const bool by_xcd = (G & 7) == 0;
    const int in_round = by_xcd ? (blockIdx.x & 7) * (G >> 3) + (blockIdx.x >> 3) : int(blockIdx.x);
    auto item_of = [&](int u) { return u * G + in_round; };
    int n_mine = 0;
    for (int u = 0; u < tiles_per_wg; ++u)
        if (item_of(u) < nb) ++n_mine;
    if (n_mine == 0) return;
    const int nk = K / ksplit / 64;   // slices per item
    // geometry of tile t: MFMA tiles per wave along N, first row of A, first column (in units of UNIT)
    auto tile_geom = [&](int t, int* nj, int* m0, int* col_units) {
        int c, p;
        if (t < t8) { c = 8; p = t; *col_units = 0; }
        else if (t < t8 + t6) { c = 6; p = t - t8; *col_units = 8 * plan.n8; }
        else { c = 4; p = t - t8 - t6; *col_units = 8 * plan.n8 + 6 * plan.n6; }
        *nj = c;
        *m0 = (p % tiles_m) * 256;
        *col_units += c * (p / tiles_m);
    };

    // ---- loads.  Wave-load wl = wave + 4 i of an item covers its rows 8 wl .. 8 wl + 7 (128 B each).
    const int lr = lane >> 3, lpos = lane & 7;
    const unsigned chunk = unsigned((lpos ^ (((wave & 1) << 2) + (lr >> 1))) << 4);
    const unsigned voff_a = unsigned((8 * wave + lr) * K * 2) + chunk, step_a = unsigned(32 * K * 2);
    // W rows: plain, item row = panel row; SwiGLU, waves 0 and 1 fetch gate rows, waves 2 and 3 up rows.  The
    // item always has 256 rows: those past the panel lie outside the descriptor and arrive as zeros.
    const unsigned voff_w = EPI == EPI_SWIGLU ? unsigned((8 * (wave & 1) + lr) * K * 2) + chunk : voff_a;
    const unsigned step_w = EPI == EPI_SWIGLU ? unsigned(16 * K * 2) : step_a;
    __amdgpu_buffer_rsrc_t ra, rw;
    int ka = 0, ua = 0, kw = 0, uw = 0, slot_a = 1, slot_w = 0;
    // descriptors start at the item's first row and first K element
    auto set_a = [&]() {
        const int q = item_of(ua), kbeg = (q / n_tiles) * nk * 64;
        int nj, m0, cu;
        tile_geom(q % n_tiles, &nj, &m0, &cu);
        ra = __builtin_amdgcn_make_buffer_rsrc((void*)(A + size_t(m0) * K + kbeg), 0, min(256, M - m0) * K * 2 - kbeg * 2, 0x00020000);
    };
    auto set_w = [&]() {
        const int q = item_of(uw), kbeg = (q / n_tiles) * nk * 64;
        int nj, m0, cu;
        tile_geom(q % n_tiles, &nj, &m0, &cu);
        const bf16_t* base = (EPI == EPI_SWIGLU && (wave >> 1) ? W2 : W) + size_t(cu) * UNIT * K;
        rw = __builtin_amdgcn_make_buffer_rsrc((void*)(base + kbeg), 0, nj * UNIT * K * 2 - kbeg * 2, 0x00020000);
    };
    auto next_a = [&]() {
        slot_a = slot_a >= P_SLOTS - 2 ? slot_a + 2 - P_SLOTS : slot_a + 2;
        if (++ka == nk) {
            ka = 0; ++ua;
            if (ua < n_mine) set_a();
            else ra = __builtin_amdgcn_make_buffer_rsrc((void*)A, 0, 0, 0x00020000);
        }
    };
    auto next_w = [&]() {
        slot_w = slot_w >= P_SLOTS - 2 ? slot_w + 2 - P_SLOTS : slot_w + 2;
        if (++kw == nk) {
            kw = 0; ++uw;
            if (uw < n_mine) set_w();
            else rw = __builtin_amdgcn_make_buffer_rsrc((void*)W, 0, 0, 0x00020000);
        }
    };
    // wave-load l of an item: LDS base of its half of the wave's eight, the immediate offset picks one of four (the
    // builtin wants it as a literal)
    auto load_one = [&](__amdgpu_buffer_rsrc_t rs, unsigned char* dst, unsigned voff, int kk, unsigned step, int l)
                        __attribute__((always_inline)) {
        CAKE_LDS_AS void* d = (CAKE_LDS_AS void*)(dst + (l >> 2) * 4096);
        const unsigned so = kk * 128 + l * step - (l & 3) * 1024;
        switch (l & 3) {
            case 0: __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, d, 16, voff, so, 0, 0); break;
            case 1: __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, d, 16, voff, so, 1024, 0); break;
            case 2: __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, d, 16, voff, so, 2048, 0); break;
            default: __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, d, 16, voff, so, 3072, 0); break;
        }
    };
    auto load_item = [&](__amdgpu_buffer_rsrc_t rs, int slot, unsigned voff, int kk, unsigned step) {
        unsigned char* dst = lds + slot * P_ITEM + wave * 8192;
#pragma unroll
        for (int r = 0; r < 8; ++r)
            load_one(rs, dst, voff, kk, step, r);
    };

    // ---- operand reads: MFMA tile i of this wave = rows 16 i .. 16 i + 15 of its share of the item (A: 128 rows from
    // 128 wm; W: 16 nj rows from 16 nj wn); k-step ks = chunks 4 ks .. 4 ks + 3
    const int sw = (l16 >> 1) & 7;
    // Where item row R sits in LDS: a wave's eight wave-loads of an item lie next to each other, 1 KB apart, so that
    // four of them share one value of M0 and differ in the instruction's immediate offset (which the hardware adds
    // to the LDS address and to the memory address alike; the scalar offset takes it off the latter again).  Every
    // write of M0 costs the one wave of a SIMD issue time: with one M0 per load the kernel ran 7 % longer.  Row
    // R = 32 r + 8 w + lr (wave-load r of wave w, row lr of its eight) is at byte 8192 w + 1024 r + 128 lr; for the
    // rows 16 i + l16 of MFMA tile i above a base that is a multiple of 32 rows that is
    // 8192 (2 (i & 1) + (l16 >> 3)) + 1024 (base / 32 + (i >> 1)) + 128 (l16 & 7).
    auto tile_off = [](int i) { return (i & 1) * 16384 + (i >> 1) * 1024; };
    const int lane_off = (l16 >> 3) * 8192 + (l16 & 7) * 128;
    const int a_lane = wm * 4096 + lane_off, b_lane = lane_off;
    int kch[2];
    kch[0] = (lq ^ sw) << 4;
    kch[1] = ((4 + lq) ^ sw) << 4;
    f32x4 acc[8][8];
    p256_frag_t a0[8], b0[8], a1[8], b1[8];
    // One phase of an item of class nj (a constant where this is called): the 8 nj MFMAs of a k-step on (a, b), with
    // the 8 + nj operand reads of the next k-step (into an, bn: W fragments first, they are needed by the first
    // MFMAs) and the eight wave-loads of one item dealt between them in `slots` places, two reads then a load,
    // at even distances, the last MFMAs after the last read.  b_wave: byte offset of this wave's W rows in an item,
    // of the class the fragments READ here belong to (the next item's in the last phase of an item).
    auto phase = [&](const int nj, const p256_frag_t* a, const p256_frag_t* b, p256_frag_t* an, p256_frag_t* bn, int sa, int sb,
                     int ks, int b_wave, __amdgpu_buffer_rsrc_t rs, int slot, unsigned voff, int kk, unsigned step)
                     __attribute__((always_inline)) {
        const unsigned char* pa = lds + sa * P_ITEM + a_lane + kch[ks];
        const unsigned char* pb = lds + sb * P_ITEM + b_wave + b_lane + kch[ks];
        unsigned char* dst = lds + slot * P_ITEM + wave * 8192;
        const int n_mfma = 8 * nj, reads = 8 + nj, slots = reads + 8, spread = n_mfma - (nj == 8 ? 16 : nj == 6 ? 8 : 6);
#pragma unroll
        for (int n = 0; n <= 64; ++n) {
#pragma unroll
            for (int sl = 0; sl < 24; ++sl) {
                if (sl < slots && ((sl + 1) * spread) / slots == n) {
                    const int grp = sl / 3, pos = sl % 3;
                    if (sl < 3 * (reads / 2) && pos < 2) {
                        const int r = 2 * grp + pos;
                        if (r < nj) bn[r] = *(const p256_frag_t*)(pb + tile_off(r));
                        else an[r - nj] = *(const p256_frag_t*)(pa + tile_off(r - nj));
                    } else {
                        const int l = sl < 3 * (reads / 2) ? grp : reads / 2 + (sl - 3 * (reads / 2));
                        load_one(rs, dst, voff, kk, step, l);
                    }
                }
            }
            if (n < n_mfma) p256_mfma(acc[n / nj][n % nj], a[n / nj], b[n % nj]);
        }
    };

    // prologue: items W0 A0 W1 A1 in flight (dummies past the end of the streams)
    set_a(); set_w();
    load_item(rw, slot_w, voff_w, kw, step_w); next_w();
    load_item(ra, slot_a, voff_a, ka, step_a); next_a();
    load_item(rw, slot_w, voff_w, kw, step_w); next_w();
    load_item(ra, slot_a, voff_a, ka, step_a); next_a();
    asm volatile("s_waitcnt vmcnt(16)");
    __builtin_amdgcn_s_barrier();
    int sa = 1, sb = 0;   // slots of the slice being consumed
    int nj_cur, m0_cur, cu_cur;
    tile_geom(item_of(0) % n_tiles, &nj_cur, &m0_cur, &cu_cur);
    {   // first operands of the first item
        const unsigned char* pa = lds + sa * P_ITEM + a_lane + kch[0];
        const unsigned char* pb = lds + sb * P_ITEM + wn * nj_cur * 512 + b_lane + kch[0];
#pragma unroll
        for (int j = 0; j < 8; ++j) b0[j] = *(const p256_frag_t*)(pb + tile_off(j));
#pragma unroll
        for (int i = 0; i < 8; ++i) a0[i] = *(const p256_frag_t*)(pa + tile_off(i));
    }
    constexpr int OUT_ELT = EPI == EPI_SWIGLU ? 2 : 4;
    const __amdgpu_buffer_rsrc_t obuf = __builtin_amdgcn_make_buffer_rsrc(outv, 0, int(size_t(M) * N * OUT_ELT), 0x00020000);
    // The K loop of an item of class nj (a constant at each of the three call sites)
    auto k_loop = [&](const int nj, int b_wave, int b_wave_next) __attribute__((always_inline)) {
        for (int kt = 0; kt < nk; ++kt) {
            // phase A: k-step 0; operands of k-step 1; the W item of the slice after next (the weights come from HBM
            // and get the longer run-up: a slice and a half; the activations are L2 hits)
            phase(nj, a0, b0, a1, b1, sa, sb, 1, b_wave, rw, slot_w, voff_w, kw, step_w);
            next_w();
            // this wave has read all of this slice; the next slice must have landed: only the item just issued may be out
            asm volatile("s_waitcnt vmcnt(8)");
            __builtin_amdgcn_s_barrier();
            sa = sa >= P_SLOTS - 2 ? sa + 2 - P_SLOTS : sa + 2;
            sb = sb >= P_SLOTS - 2 ? sb + 2 - P_SLOTS : sb + 2;
            // phase B: k-step 1; first operands of the next slice; the A item of the slice after next into a freed slot
            phase(nj, a1, b1, a0, b0, sa, sb, 0, kt + 1 == nk ? b_wave_next : b_wave, ra, slot_a, voff_a, ka, step_a);
            next_a();
        }
    };
    // Epilogue of an item of class nj; accumulator (i, j)[v] is row 16 i + 4 lq + v, column 16 j + l16 of the wave's share
    auto epilogue = [&](const int nj, int q, int m0, int col_units) __attribute__((always_inline)) {
        const int row0 = m0 + wm * 128 + 4 * lq;
        if constexpr (EPI == EPI_SWIGLU) {
            // silu(gate) * up from accumulator pairs (even j: gate, odd j: the same columns of up).  The row offsets go
            // through the scalar offset of the store.
            const int pitch = N * 2;
            const unsigned base = unsigned(row0 * N + col_units * UNIT + wn * nj * 8 + l16) * 2u;
#pragma unroll
            for (int i = 0; i < 8; ++i)
#pragma unroll
                for (int j = 0; j < 8; j += 2)
#pragma unroll
                    for (int v = 0; v < 4; ++v)
                        if (j < nj) {
                            const float g = acc[i][j][v], up = acc[i][j + 1][v];
                            // the hardware reciprocal (1 ulp) instead of an IEEE division: the result is rounded to bf16
                            const bf16_t o = bf16_t(g * __builtin_amdgcn_rcpf(1.0f + __expf(-g)) * up);
                            unsigned short bits;
                            __builtin_memcpy(&bits, &o, 2);
                            __builtin_amdgcn_raw_buffer_store_b16(bits, obuf, base, (i * 16 + v) * pitch + (j >> 1) * 32, 0);
                        }
        } else if constexpr (SPLIT) {
            // This K range's accumulators go to the item's slot of the workspace, in accumulator order (each store
            // is 4 KB contiguous over the workgroup); a second kernel adds the ranges up and runs the epilogue:
            // a single workgroup reading a tile's parts back would take longer than the whole K loop.
            constexpr int TILE_B = 256 * 256 * 4;
            const __amdgpu_buffer_rsrc_t ws = __builtin_amdgcn_make_buffer_rsrc(part, 0, n_tiles * ksplit * TILE_B, 0x00020000);
            const unsigned mine = (unsigned(q % n_tiles) * ksplit + unsigned(q / n_tiles)) * TILE_B + unsigned(tid) * 16;
#pragma unroll
            for (int i = 0; i < 8; ++i)
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    u32x4 v = {__float_as_uint(acc[i][j][0]), __float_as_uint(acc[i][j][1]), __float_as_uint(acc[i][j][2]),
                               __float_as_uint(acc[i][j][3])};
                    __builtin_amdgcn_raw_buffer_store_b128(v, ws, mine + (i * 8 + j) * 4096, 0, 0);
                }
        } else {
            const unsigned base = unsigned(row0 * N + col_units * UNIT + wn * nj * 16 + l16) * 4u;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                float old[8][4];
                if constexpr (EPI == EPI_RESIDUAL_F32) {   // all loads of a band of 16 rows in flight before the first add
#pragma unroll
                    for (int j = 0; j < 8; ++j)
#pragma unroll
                        for (int v = 0; v < 4; ++v)
                            if (j < nj)
                                old[j][v] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(obuf, base + unsigned((i * 16 + v) * N + j * 16) * 4u, 0, 0));
                }
#pragma unroll
                for (int j = 0; j < 8; ++j)
#pragma unroll
                    for (int v = 0; v < 4; ++v)
                        if (j < nj) {
                            float x = acc[i][j][v];
                            if constexpr (EPI == EPI_RESIDUAL_F32) x += old[j][v];
                            __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(x), obuf, base + unsigned((i * 16 + v) * N + j * 16) * 4u, 0, 0);
                        }
            }
        }
    };
    for (int u = 0; u < n_mine; ++u) {
        // cleared here and nowhere else, so that no accumulator value lives from one item to the next
#pragma unroll
        for (int i = 0; i < 8; ++i)
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};
        __builtin_amdgcn_sched_barrier(0);
        asm volatile("s_nop 7");
        __builtin_amdgcn_sched_barrier(0);
        const int q = item_of(u);
        int nj_next = nj_cur, m0_next = 0, cu_next = 0;
        if (u + 1 < n_mine) tile_geom(item_of(u + 1) % n_tiles, &nj_next, &m0_next, &cu_next);
        const int b_wave = wn * nj_cur * 512, b_wave_next = wn * nj_next * 512;   // 16 nj rows = nj / 2 KB steps
        if (nj_cur == 8) k_loop(8, b_wave, b_wave_next);
        else if (nj_cur == 6) k_loop(6, b_wave, b_wave_next);
        else k_loop(4, b_wave, b_wave_next);
        // The asm MFMAs are opaque to the compiler's hazard handling: let the last of them (four passes) retire
        // before the accumulators are read.
        __builtin_amdgcn_sched_barrier(0);
        asm volatile("s_nop 15\n\ts_nop 15");
        __builtin_amdgcn_sched_barrier(0);
        // (the next item's first slices are in flight during the epilogue)
        if (nj_cur == 8) epilogue(8, q, m0_cur, cu_cur);
        else if (nj_cur == 6) epilogue(6, q, m0_cur, cu_cur);
        else epilogue(4, q, m0_cur, cu_cur);
        nj_cur = nj_next; m0_cur = m0_next; cu_cur = cu_next;
        // loads and stores complete out of order with respect to each other: nothing is counted across them
        asm volatile("s_waitcnt vmcnt(0)");
    }
}

// Second pass of the persistent kernel with K split: workgroup (tile t, band i) adds up, in range order, the
// `ksplit` parts of the tile's i-th bands of sixteen rows per wave (so the result is the same bits on every
// launch) and stores them or adds them into the float32 residual stream.  Thread and accumulator layout are
// the producing kernel's: thread tid = wave (wm, wn) x lane (lq, l16), accumulator (i, j)[e] = row
// 128 wm + 16 i + 4 lq + e, column 128 wn + 16 j + l16 of the tile.
template <int EPI>
__global__ void __launch_bounds__(256)
gemm_p256_finish_kernel(const float* __restrict__ part, float* __restrict__ out, int M, int N, int tiles_m, int ksplit) {
    const int t = blockIdx.x >> 3, i = blockIdx.x & 7, tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63, wm = wave >> 1, wn = wave & 1, l16 = lane & 15, lq = lane >> 4;
    const int m0 = (t % tiles_m) * 256, c0 = (t / tiles_m) * 256;
    const float4* src = (const float4*)part + (size_t(t) * ksplit * 64 + i * 8) * 256 + tid;
    float4 tot[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) tot[j] = src[j * 256];
    for (int sp = 1; sp < ksplit; ++sp) {
        float4 p[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) p[j] = src[(size_t(sp) * 64 + j) * 256];
#pragma unroll
        for (int j = 0; j < 8; ++j) { tot[j].x += p[j].x; tot[j].y += p[j].y; tot[j].z += p[j].z; tot[j].w += p[j].w; }
    }
    const int row = m0 + wm * 128 + 16 * i + 4 * lq, col = c0 + wn * 128 + l16;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        if (row + e >= M) break;
        float* o = out + size_t(row + e) * N + col;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const float x = e == 0 ? tot[j].x : e == 1 ? tot[j].y : e == 2 ? tot[j].z : tot[j].w;
            if (EPI == EPI_RESIDUAL_F32) o[16 * j] += x;
            else o[16 * j] = x;
        }
    }
}

// =====================================================================================
// Yardstick: what the matrix pipes deliver with nothing else going on.  Every wave runs `iters`
// rounds of eight independent 32x32x16 bf16 MFMAs on operands it keeps in registers (no memory
// traffic, no LDS, no barriers); one value per wave is written so that the work is not dead.
// `acc[lane & 15]` at the end indexes a vector dynamically; the loop above keeps it in registers.
// =====================================================================================
__global__ void __launch_bounds__(512)
mfma_rate_kernel(float* __restrict__ out, int iters, unsigned seed) {
    const int lane = threadIdx.x & 63;
    // operands with the statistics of real data (what the pipes draw depends on how many bits toggle):
    // hashed values spread over [-2, 2), a different register set for every MFMA of a round, laid out
    // like one wave's 128x64 tile of the GEMM above (four A fragments, two B fragments)
    auto rnd = [&](unsigned k) {
        unsigned h = (k + seed) * 2654435761u; h ^= h >> 15; h *= 2246822519u; h ^= h >> 13;
        return bf16_t(float(int(h & 0xffff) - 32768) * (1.0f / 16384.0f));
    };
    bf16x8 a[4], b[2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int e = 0; e < 8; ++e) a[i][e] = rnd(unsigned((threadIdx.x * 4 + i) * 8 + e));
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int e = 0; e < 8; ++e) b[j][e] = rnd(0x9e3779b9u + unsigned((threadIdx.x * 2 + j) * 8 + e));
    f32x16 acc[4][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j) acc[i][j] = mfma32(a[i], b[j], acc[i][j]);
    }
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) sum += acc[i][j][lane & 15];
    if (lane == 0) out[(size_t(blockIdx.x) * blockDim.x + threadIdx.x) >> 6] = sum;
}

// grid: `workgroups` workgroups of eight waves.  FLOPs = workgroups * 8 * iters * 8 * 32768.
hipError_t launch_mfma_rate(float* out, int workgroups, int iters, hipStream_t st) {
    hipLaunchKernelGGL(mfma_rate_kernel, dim3(workgroups), dim3(512), 0, st, out, iters, 12345u);
    return hipGetLastError();
}

// Tile configurations.  Chosen per GEMM by gemm_pick() from how well the grid fills 256 CUs.
struct GemmCfg { int bm, bn; };
// GCFG_128x128K: the 128x128 tile as two 128x64 halves, each shared by two waves that divide K (KW = 2)
// GCFG_P256: the persistent four-wave kernel (256x256 tiles, several per workgroup)
enum { GCFG_256x256 = 0, GCFG_256x128 = 1, GCFG_128x128 = 2, GCFG_128x192 = 3, GCFG_128x64 = 4, GCFG_128x128K = 5, GCFG_P256 = 6,
       GCFG_COUNT = 7 };
static const GemmCfg kGemmCfg[GCFG_COUNT] = {{256, 256}, {256, 128}, {128, 128}, {128, 192}, {128, 64}, {128, 128}, {256, 256}};

struct P256Plan;
static P256Plan p256_plan(int epi, int tiles_m, int N);
static double p256_plan_cost(int tiles_m, int n8, int n6, int n4);

static int out_cols_per_tile(int cfg, int epi) { return epi == EPI_SWIGLU ? kGemmCfg[cfg].bn / 2 : kGemmCfg[cfg].bn; }

static bool gemm_cfg_ok(int cfg, int epi, int M, int N, int K) {
    if ((cfg == GCFG_128x192 || cfg == GCFG_128x64) && epi == EPI_SWIGLU) return false;   // odd n-tiles per wave: no gate/up pairs
    if (cfg == GCFG_128x128K && (epi == EPI_SWIGLU || (K % 64) != 0)) return false;
    // the persistent kernel addresses everything through 32-bit buffer offsets
    // (its column panels are 256, 192 or 128 rows of W wide: N in units of 64, of 32 for SwiGLU)
    if (cfg == GCFG_P256)
        return M > 0 && N > 0 && K >= 64 && (K % 64) == 0 && double(M) * N * 4 < 2147483648.0 && double(K) * 512 < 2147483648.0 &&
               (N % (epi == EPI_SWIGLU ? 32 : 64)) == 0;
    return M > 0 && N > 0 && K >= 32 && (K % 32) == 0 && (N % out_cols_per_tile(cfg, epi)) == 0;
}

bool gemm_mfma_supported(int epi, int M, int N, int K) { return gemm_cfg_ok(GCFG_128x128, epi, M, N, K); }

// Cost model: the busiest CU runs ceil(workgroups / 256) of them one after another, each costing its
// tile area times its share of K divided by a per-shape efficiency (measured: larger tiles feed the
// MFMAs better because they pull fewer bytes per flop through L2), plus a fixed part (pipeline fill,
// epilogue).  With K split `ks` ways every workgroup writes its part and the one that finishes a tile
// reads ks parts back; that pays only where the unsplit choice is a small tile over a long K (the
// down projections of the 512-token-chunk and the 8192-wide shapes).  Unit: one 256x256 tile over
// K = 4096 costs 100 (about a microsecond each).
struct GemmChoice { int cfg, ksplit; };
static bool ksplit_ok(int cfg, int ks, int epi, int M, int N, int K, const GemmSplitWs* ws) {
    if (ks == 1) return true;
    if (!ws || !ws->part || !ws->counters || epi == EPI_SWIGLU) return false;
    if (K % ks || (K / ks) % 64 || K / ks < 512) return false;
    const GemmCfg& c = kGemmCfg[cfg];
    if (N % c.bn) return false;
    const long tiles = long((M + c.bm - 1) / c.bm) * (N / c.bn);
    return tiles <= ws->n_counters && size_t(tiles) * ks * c.bm * c.bn * sizeof(float) <= ws->part_bytes;
}
static GemmChoice gemm_pick(int epi, int M, int N, int K, const GemmSplitWs* ws) {
    static const double eff[GCFG_COUNT] = {1.0, 0.60, 0.62, 0.80, 0.40, 0.65, 1.11};   // measured TFLOP/s per busy CU, relative to 256x256
    GemmChoice best{GCFG_128x128, 1};
    double best_cost = 1e30;
    for (int cfg = GCFG_COUNT - 1; cfg >= 0; --cfg) {
        if (!gemm_cfg_ok(cfg, epi, M, N, K)) continue;
        const GemmCfg& c = kGemmCfg[cfg];
        if (cfg == GCFG_P256) {
            // The persistent kernel needs a grid that fills the chip.  With K split, its parts (256 KB per workgroup)
            // go through memory to a second kernel, about 45 us for 256 of them: measured 487 us against 443 for the
            // eight-wave 256 x 256 kernel on 1024 x 8192 x 28672 in two ranges, 155 against 140 for 128 x 128 tiles
            // on 1024 x 4096 x 14336 in four.  So it is chosen unsplit only (the split path stays for forced use).
            const int tiles_m = (M + 255) / 256;
            const P256Plan plan = p256_plan(epi, tiles_m, N);
            const long items = long(tiles_m) * (plan.n8 + plan.n6 + plan.n4);
            if (items < 160) continue;
            // p256_plan_cost: the busiest workgroup's work in units of an eighth of a 256 x 256 tile
            const double cost = p256_plan_cost(tiles_m, plan.n8, plan.n6, plan.n4) * 12.5 * (double(K) / 4096.0) / eff[cfg] +
                                6.0 * double((items + 255) / 256);
            if (cost < best_cost) { best_cost = cost; best = GemmChoice{cfg, 1}; }
            continue;
        }
        const long tiles = long((M + c.bm - 1) / c.bm) * (N / out_cols_per_tile(cfg, epi));
        const double area = double(c.bm) * c.bn / 65536.0;
        for (int ks = 1; ks <= 8; ks *= 2) {
            if (!ksplit_ok(cfg, ks, epi, M, N, K, ws)) continue;
            const double rounds = double((tiles * ks + 255) / 256);
            double cost = rounds * (100.0 * area * (double(K) / ks / 4096.0) / eff[cfg] + 6.0);
            // measured: the parts cross the chip twice, at device scope; and a split must promise 8 % to be taken
            if (ks > 1) cost = (cost + 10.0 + 20.0 * area * ks) * 1.08;
            if (cost < best_cost) { best_cost = cost; best = GemmChoice{cfg, ks}; }
        }
    }
    return best;
}

template <int WTM, int WTN, int WAVES_M, int WAVES_N, int BK, int STAGES, int EPI, int KW = 1>
static hipError_t gemm_launch_t(const bf16_t* A, const bf16_t* W, const bf16_t* W2, void* out, int M, int N, int K,
                                hipStream_t st, int ksplit, const GemmSplitWs* ws) {
    constexpr int BM = WAVES_M * WTM * 32, BN = WAVES_N * WTN * 32;
    constexpr int LDS = (BM + BN) * BK * 2 * STAGES;
    auto kern = gemm_mfma_kernel<WTM, WTN, WAVES_M, WAVES_N, BK, STAGES, EPI, KW>;
    static bool attr_set = false;   // one flag per instantiation
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, LDS);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const int tiles_m = (M + BM - 1) / BM, tiles_n = N / (EPI == EPI_SWIGLU ? BN / 2 : BN);
    if (ksplit > 1 && (K / ksplit) % BK) return hipErrorInvalidValue;
    hipLaunchKernelGGL(kern, dim3(tiles_m * tiles_n * ksplit), dim3(64 * WAVES_M * WAVES_N * KW), LDS, st, A, W, W2, out, M, N, K,
                       tiles_m, tiles_n, ksplit > 1 ? ws->part : nullptr, ksplit > 1 ? ws->counters : nullptr, ksplit);
    return hipGetLastError();
}

// Panel widths of the persistent kernel for N columns and `tiles_m` row bands: counts of 8-, 6- and 4-tile panels
// with 8 n8 + 6 n6 + 4 n4 = N / unit that minimise the time of the busiest workgroup: items go out widest first,
// one per workgroup and round, so workgroup 0 takes the widest item of every round.  A narrow item is not
// faster in proportion (measured, 256 items over K = 4096: 108 us at 256 wide, 86 to 100 at 192, 70 to 74 at 128,
// and 1.2 us per slice at 128 wide over a long K against 1.46 at 256: the loads, reads and barriers of a slice
// stay the same), and every item costs an epilogue.
static double p256_plan_cost(int tiles_m, int n8, int n6, int n4) {
    const int c8 = tiles_m * n8, c6 = tiles_m * n6, nb = c8 + c6 + tiles_m * n4;
    const int rounds = (nb + 255) / 256, wgs = (nb + rounds - 1) / rounds;
    double cost = 0.0;
    for (int u = 0; u < rounds; ++u) {
        const int first = u * wgs;
        cost += (first < c8 ? 8.0 : first < c8 + c6 ? 7.0 : 6.2) + 0.4;
    }
    return cost;
}
static P256Plan p256_plan(int epi, int tiles_m, int N) {
    const int unit = epi == EPI_SWIGLU ? 16 : 32;
    if (N % (2 * unit)) return P256Plan{0, 0, 0};
    const int U = N / unit;
    struct Entry { int epi, tiles_m, N; P256Plan plan; };
    static std::mutex mu;
    static std::vector<Entry> cache;
    std::lock_guard<std::mutex> lock(mu);
    for (const Entry& e : cache)
        if (e.epi == epi && e.tiles_m == tiles_m && e.N == N) return e.plan;
    P256Plan best{0, 0, 0};
    double best_cost = 1e30;
    for (int n8 = 0; 8 * n8 <= U; ++n8)
        for (int n6 = 0; 8 * n8 + 6 * n6 <= U; ++n6) {
            const int rem = U - 8 * n8 - 6 * n6;
            if (rem % 4) continue;
            const double c = p256_plan_cost(tiles_m, n8, n6, rem / 4);
            if (c < best_cost - 1e-9) { best_cost = c; best = P256Plan{n8, n6, rem / 4}; }
        }
    cache.push_back(Entry{epi, tiles_m, N, best});
    return best;
}

template <int EPI>
static hipError_t gemm_launch_cfg(int cfg, int ks, const GemmSplitWs* ws, const bf16_t* A, const bf16_t* W, const bf16_t* W2,
                                  void* out, int M, int N, int K, hipStream_t st) {
    const long tiles128 = long((M + 127) / 128) * (N / (EPI == EPI_SWIGLU ? 64 : 128)) * ks;
    if (cfg == GCFG_P256) {
        const int tiles_m = (M + 255) / 256;
        const P256Plan plan = ks > 1 ? P256Plan{N / 256, 0, 0} : p256_plan(EPI, tiles_m, N);
        const int panels = plan.n8 + plan.n6 + plan.n4, nb = tiles_m * panels * ks;
        if (panels == 0) return hipErrorInvalidValue;
        // a whole number of rounds: every workgroup takes `rounds` items (the last may take one less)
        const int rounds = (nb + 255) / 256, wgs = (nb + rounds - 1) / rounds;
        auto kern = gemm_p256_kernel<EPI, false>;
        if constexpr (EPI != EPI_SWIGLU) {
            if (ks > 1) kern = gemm_p256_kernel<EPI, true>;
        }
        static bool attr_set[2] = {false, false};
        if (!attr_set[ks > 1]) {
            hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, P_LDS);
            if (e != hipSuccess) return e;
            attr_set[ks > 1] = true;
        }
        hipLaunchKernelGGL(kern, dim3(wgs), dim3(256), P_LDS, st, A, W, W2, out, M, N, K, tiles_m, plan, rounds,
                           ks > 1 ? ws->part : nullptr, ks);
        if (ks > 1) {
            if constexpr (EPI != EPI_SWIGLU)
                hipLaunchKernelGGL(gemm_p256_finish_kernel<EPI>, dim3(tiles_m * plan.n8 * 8), dim3(256), 0, st, ws->part, (float*)out,
                                   M, N, tiles_m, ks);
        }
        return hipGetLastError();
    }
    switch (cfg) {
        case GCFG_256x256: return gemm_launch_t<4, 2, 2, 4, 32, 5, EPI>(A, W, W2, out, M, N, K, st, ks, ws);
        case GCFG_256x128:
            if ((K / ks % 64) == 0) return gemm_launch_t<4, 2, 2, 2, 64, 3, EPI>(A, W, W2, out, M, N, K, st, ks, ws);
            return gemm_launch_t<4, 2, 2, 2, 32, 4, EPI>(A, W, W2, out, M, N, K, st, ks, ws);
        case GCFG_128x192:
            if constexpr (EPI != EPI_SWIGLU) {
                // at most one workgroup per CU: the whole 160 KB of LDS as a ring of 64-deep slices (120 KB in
                // flight hide the latency of weights that come from HBM: 64 against 75 us for N = 6144)
                if (long((M + 127) / 128) * (N / 192) * ks <= 256 && (K / ks % 64) == 0)
                    return gemm_launch_t<2, 3, 2, 2, 64, 4, EPI, 2>(A, W, W2, out, M, N, K, st, ks, ws);
                return gemm_launch_t<2, 3, 2, 2, 32, 4, EPI>(A, W, W2, out, M, N, K, st, ks, ws);
            } else {
                return hipErrorInvalidValue;
            }
        case GCFG_128x128K:
            if constexpr (EPI != EPI_SWIGLU) return gemm_launch_t<2, 2, 2, 2, 64, 5, EPI, 2>(A, W, W2, out, M, N, K, st, ks, ws);
            else return hipErrorInvalidValue;
        case GCFG_128x64:   // half-size chunks (M = 512): the only unsplit shape that still gives N = 4096 GEMMs 256 tiles
            if constexpr (EPI != EPI_SWIGLU) {
                if ((K / ks % 64) == 0) return gemm_launch_t<2, 1, 2, 2, 64, 4, EPI>(A, W, W2, out, M, N, K, st, ks, ws);
                return gemm_launch_t<2, 1, 2, 2, 32, 4, EPI>(A, W, W2, out, M, N, K, st, ks, ws);
            } else {
                return hipErrorInvalidValue;
            }
        default:
            // one workgroup per CU at most: spend the whole LDS on a deep ring of 64-deep slices
            // (96 KB in flight per CU); more tiles than CUs: 64 KB rings so two workgroups share a CU
            if (tiles128 <= 256 && (K / ks % 64) == 0) return gemm_launch_t<2, 2, 2, 2, 64, 4, EPI>(A, W, W2, out, M, N, K, st, ks, ws);
            return gemm_launch_t<2, 2, 2, 2, 32, 4, EPI>(A, W, W2, out, M, N, K, st, ks, ws);
    }
}

static GemmChoice gemm_choose(int epi, int M, int N, int K, int cfg_override, const GemmSplitWs* ws, int ksplit_override) {
    GemmChoice ch = gemm_pick(epi, M, N, K, ksplit_override == 1 ? nullptr : ws);
    if (cfg_override >= 0 && cfg_override < GCFG_COUNT && gemm_cfg_ok(cfg_override, epi, M, N, K)) ch = GemmChoice{cfg_override, 1};
    if (ksplit_override > 1 && gemm_cfg_ok(ch.cfg, epi, M, N, K) && ksplit_ok(ch.cfg, ksplit_override, epi, M, N, K, ws))
        ch.ksplit = ksplit_override;
    return ch;
}

void gemm_mfma_plan(int epi, int M, int N, int K, int cfg_override, const GemmSplitWs* ws, int ksplit_override,
                    int* bm, int* bn, int* ksplit) {
    const GemmChoice ch = gemm_choose(epi, M, N, K, cfg_override, ws, ksplit_override);
    *bm = kGemmCfg[ch.cfg].bm; *bn = kGemmCfg[ch.cfg].bn; *ksplit = ch.ksplit;
}

hipError_t launch_gemm_mfma(int epi, const void* a, const void* w, const void* w2, void* out, int M, int N, int K,
                            hipStream_t st, int cfg_override, const GemmSplitWs* ws, int ksplit_override) {
    const bf16_t *A = (const bf16_t*)a, *W = (const bf16_t*)w, *W2 = (const bf16_t*)w2;
    const GemmChoice ch = gemm_choose(epi, M, N, K, cfg_override, ws, ksplit_override);
    if (!gemm_cfg_ok(ch.cfg, epi, M, N, K)) return hipErrorInvalidValue;
    if (epi == EPI_SWIGLU) return gemm_launch_cfg<EPI_SWIGLU>(ch.cfg, 1, ws, A, W, W2, out, M, N, K, st);
    if (epi == EPI_RESIDUAL_F32) return gemm_launch_cfg<EPI_RESIDUAL_F32>(ch.cfg, ch.ksplit, ws, A, W, W2, out, M, N, K, st);
    if (epi == EPI_STORE_F32) return gemm_launch_cfg<EPI_STORE_F32>(ch.cfg, ch.ksplit, ws, A, W, W2, out, M, N, K, st);
    return hipErrorInvalidValue;
}

}  // namespace cake
