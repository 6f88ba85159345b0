// bf16 MFMA GEMM for the prefill-size projections and the grouped expert
// GEMMs:  C[M, N] = X[M, K] W[N, K]^T, fp32 accumulation, both operands
// contiguous along K.
//
// Shape of the kernel (gfx950):
//  * one workgroup = BM x BN output tile, K walked in tiles of 32;
//  * X and W k-tiles are staged in a ring of five LDS stages (5 x 32 KB, the
//    whole LDS of a CU), filled by 16-byte direct-to-LDS global loads (no
//    register hop).  A k-tile row is 64 bytes, half a cache line, so the
//    loads go out for two k-tiles at a time, the two halves of a line in
//    adjacent instructions, 2 to 2.5 k-tiles ahead of their use: a load's
//    round trip is about as long as the MFMAs of two k-tiles, so anything
//    shallower leaves the matrix pipe waiting;
//  * a tile row is 32 bf16 = 4 chunks of 16 bytes, chunk index XOR-ed with
//    (row / 4) % 4: the LDS has 64 banks of 4 bytes, four 64-byte rows fill
//    them once, and 16 lanes reading 16 consecutive rows at one k-offset (an
//    MFMA fragment read, ds_read_b128) touch 16 different 16-byte bank groups;
//  * v_mfma_f32_32x32x16_bf16 with the WEIGHT rows as the 32 MFMA rows and
//    the ACTIVATION rows as the 32 MFMA columns, so each lane ends up holding
//    4 consecutive output columns of one output row: the epilogue stages
//    32-row slabs in LDS as fp32 and writes 16-byte row-contiguous stores;
//  * epilogues: 0 = plain / + residual (fp32 add before the bf16 round), 1 =
//    SwiGLU on a stacked gate/up weight (each wave holds the gate and the up
//    tile of the same columns), 2 = fp32 output (router logits); per-row
//    scaling for the routed experts;
//  * workgroup ids are remapped so that each XCD (own L2) gets a contiguous
//    range of tiles, walked in groups of 8 row tiles per column tile.
#include <type_traits>

#include "common.h"

#define GEMM_BK 32       // k-tile
#define GEMM_STAGES 5   // LDS ring (5 x 32 KB = the whole LDS of a CU)

struct GemmParams {
    const bf16* X;
    const bf16* W;
    const bf16* R;
    bf16* C;
    int64_t M;
    int N;  // output columns (F for the SwiGLU epilogue, whose W has 2N rows)
    int K;
    int n_mtiles, n_ntiles;
    int r_f32;  // the residual R is fp32 rather than bf16
    GroupedArgs g;
};

// Workgroup barrier for the LDS ring: waits until at most `n` of this wave's
// global loads are still in flight (the older ones, whose data the others are
// about to read, have landed in LDS) and all of its LDS reads have returned (the
// stage they read is about to be refilled), then joins the barrier.  Unlike
// __syncthreads() it does not drain the newer loads.
template <int N_IN_FLIGHT>
__device__ __forceinline__ void ring_barrier() {
#if defined(__HIP_DEVICE_COMPILE__)
    static_assert(N_IN_FLIGHT >= 0 && N_IN_FLIGHT < 64, "vector-memory counter is 6 bits");
    __builtin_amdgcn_sched_barrier(0);
    // simm16: vmcnt[3:0] | expcnt (7 = no wait) << 4 | lgkmcnt (0) << 8 | vmcnt[5:4] << 14
    __builtin_amdgcn_s_waitcnt((N_IN_FLIGHT & 15) | (7 << 4) | (0 << 8) | ((N_IN_FLIGHT >> 4) << 14));
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
#endif
}

template <int BM, int BN, int WM, int WN, int EPI, bool GROUPED>
__global__ __launch_bounds__(WM* WN * 64) void gemm_bf16_kernel(const GemmParams p) {
    constexpr int NT = WM * WN * 64, BK = GEMM_BK, NSTAGE = GEMM_STAGES;
    constexpr int WTM = BM / WM, WTN = BN / WN, TM = WTM / 32, TN = WTN / 32;
    constexpr int STAGE = (BM + BN) * BK;  // elements
    constexpr int OUTN = EPI == 1 ? BN / 2 : BN;
    constexpr int WOUT = EPI == 1 ? WTN / 2 : WTN;  // output columns per wave
    static_assert(EPI != 1 || TN % 2 == 0, "SwiGLU epilogue needs an even number of column tiles per wave");
    extern __shared__ __attribute__((aligned(16))) char smem[];
    bf16* lds = reinterpret_cast<bf16*>(smem);

    // ---- which tile -------------------------------------------------------
    const int total = gridDim.x;
    const int per = total / 8, rem = total % 8;
    const int xcd = blockIdx.x % 8, loc = blockIdx.x / 8;
    const int pid = xcd * per + min(xcd, rem) + loc;
    constexpr int GM = 8;
    const int per_group = GM * p.n_ntiles;
    const int first_m = (pid / per_group) * GM;
    const int gsize = min(GM, p.n_mtiles - first_m);
    const int tm = first_m + (pid % per_group) % gsize;
    const int tn = (pid % per_group) / gsize;

    int64_t m0;
    int rows_valid;
    const bf16* Wb = p.W;
    if (GROUPED) {
        const int e = p.g.tile_expert[tm];
        if (e < 0) return;
        m0 = p.g.tile_row0[tm];
        rows_valid = p.g.tile_rows[tm];
        Wb += (int64_t)e * p.g.b_expert_stride;
    } else {
        m0 = (int64_t)tm * BM;
        rows_valid = (int)min((int64_t)BM, p.M - m0);
    }
    const int n0 = tn * OUTN;

    const int t = threadIdx.x;
    const int lane = t & 63, wave = t >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int r = lane & 31, h = lane >> 5;

    // ---- global -> LDS staging (direct-to-LDS 16-byte loads) ---------------------
    // One wave instruction fills 1 KB of LDS = 16 tile rows of 4 chunks, lane l at
    // (row l / 4, chunk position l % 4); the position is the XOR-swizzled one, so
    // the lane fetches global chunk (l % 4) ^ ((row / 4) % 4) of its row.  The
    // tile's BM + BN rows are dealt to the waves in units of 16 rows.
    constexpr int XU = BM / 16 / (WM * WN), WU = BN / 16 / (WM * WN);   // units per wave
    static_assert(BM % (16 * WM * WN) == 0 && BN % (16 * WM * WN) == 0, "tile rows must split into 16-row units per wave");
    const bf16* xptr[XU];
    const bf16* wptr[WU];
    const int lrow = lane >> 2, lpos = lane & 3;
#pragma unroll
    for (int i = 0; i < XU; ++i) {
        const int row = (wave * XU + i) * 16 + lrow;
        const int c = lpos ^ ((row >> 2) & 3);
        const int rr = min(row, rows_valid - 1);
        int64_t src = m0 + rr;
        if (GROUPED && p.g.a_gather) src = p.g.a_gather[src];
        xptr[i] = p.X + src * p.K + c * 8;
    }
#pragma unroll
    for (int i = 0; i < WU; ++i) {
        const int row = (wave * WU + i) * 16 + lrow;
        const int c = lpos ^ ((row >> 2) & 3);
        int n;
        if (EPI == 1)
            n = row < BN / 2 ? min(n0 + row, p.N - 1) : p.N + min(n0 + row - BN / 2, p.N - 1);
        else
            n = min(n0 + row, p.N - 1);
        wptr[i] = Wb + (int64_t)n * p.K + c * 8;
    }

    floatx16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    // fragment row offsets inside a stage (elements), swizzle term (r / 4) % 4
    int xrow[TM], wrow[TN];
#pragma unroll
    for (int i = 0; i < TM; ++i) xrow[i] = (wm * WTM + i * 32 + r) * BK;
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        int row;
        if (EPI == 1)
            row = j < TN / 2 ? wn * (WTN / 2) + j * 32 + r : BN / 2 + wn * (WTN / 2) + (j - TN / 2) * 32 + r;
        else
            row = wn * WTN + j * 32 + r;
        wrow[j] = BM * BK + row * BK;
    }
    const int sw = (r >> 2) & 3;
    const int nk = p.K / BK;

    // Software pipeline over k-tiles of 32 (two MFMA k-steps), five LDS stages.  A k-tile row is 64
    // bytes, half a cache line, so the loads go out for TWO k-tiles at a time, the two halves of every
    // line in adjacent instructions (the second request meets the first one's line in the vector cache
    // instead of fetching it from L2 again; issued one k-tile apart, every line crossed the L2-to-CU path
    // twice and that path, not the matrix pipe, set the pace).  Pairs (T, T+1), T even, go out during k-tile
    // T-3, half of the wave's 16-row units in each of its two k-steps; the barrier in the middle of a
    // k-tile follows a wait for this wave's loads of the NEXT k-tile only (the newer ones stay in
    // flight).  MFMA fragments are double-buffered in registers, so the LDS reads of one k-step run
    // under the MFMAs of the one before.  Past the end of K the last k-tile is loaded again (into
    // stages nobody reads) rather than branching.
    constexpr int NLD = XU + WU;
    static_assert(XU % 2 == 0 && WU % 2 == 0, "the units of a tile are dealt to the two k-steps of an iteration");
    const int swave = __builtin_amdgcn_readfirstlane(wave);   // wave-uniform: LDS bases stay scalar
    // units [half * XU/2, ..) and [half * WU/2, ..) of k-tiles t0 (stage s0) and t0 + 1 (stage s1)
    auto gload_pair = [&](int t0, bf16* s0, bf16* s1, int half) {
        const int k0 = min(t0, nk - 1) * BK, k1 = min(t0 + 1, nk - 1) * BK;
#pragma unroll
        for (int i = half * (XU / 2); i < (half + 1) * (XU / 2); ++i) {
            load16_to_lds(xptr[i] + k0, s0 + (swave * XU + i) * 16 * BK);
            load16_to_lds(xptr[i] + k1, s1 + (swave * XU + i) * 16 * BK);
        }
#pragma unroll
        for (int i = half * (WU / 2); i < (half + 1) * (WU / 2); ++i) {
            load16_to_lds(wptr[i] + k0, s0 + BM * BK + (swave * WU + i) * 16 * BK);
            load16_to_lds(wptr[i] + k1, s1 + BM * BK + (swave * WU + i) * 16 * BK);
        }
    };
    auto frags = [&](const bf16* stage, int kk, bf16x8 (&xf)[TM], bf16x8 (&wf)[TN]) {
        const int ch = ((2 * kk + h) ^ sw) << 3;
#pragma unroll
        for (int i = 0; i < TM; ++i) xf[i] = *reinterpret_cast<const bf16x8*>(stage + xrow[i] + ch);
#pragma unroll
        for (int j = 0; j < TN; ++j) wf[j] = *reinterpret_cast<const bf16x8*>(stage + wrow[j] + ch);
    };
    auto mfmas = [&](const bf16x8 (&xf)[TM], const bf16x8 (&wf)[TN]) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[j], xf[i], acc[i][j], 0, 0, 0);
    };
    // Pins the instruction order of one k-step: one MFMA first, then the LDS reads of
    // the next k-step's fragments two per MFMA (the last of them still has most of
    // the group to land), then the global loads one per MFMA.  The MFMA goes first
    // because its wait for this k-step's fragments comes out as "all LDS reads done"
    // (while loads that write LDS are in flight the compiler cannot wait for fewer):
    // placed behind the first reads of the next fragments it would wait for those too.
    constexpr int NRD = TM + TN, NMF = TM * TN;
    static_assert(NRD % 2 == 0 && NMF >= NRD / 2 + NLD + 1, "k-step shape not covered by the pinned order");
    auto pin_order = [&](auto n_loads_tag) {
        constexpr int n_loads = decltype(n_loads_tag)::value;
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
#pragma unroll
        for (int i = 0; i < NRD / 2; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);   // two LDS reads
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // one MFMA
        }
#pragma unroll
        for (int i = 0; i < n_loads; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);   // one global load
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        }
        __builtin_amdgcn_sched_group_barrier(0x008, NMF - 1 - NRD / 2 - n_loads, 0);
        __builtin_amdgcn_sched_barrier(0);
    };

    // prologue: pairs (0, 1) and (2, 3); k-tile 0 has landed when all but the last load of the first pair have
    gload_pair(0, lds, lds + STAGE, 0);
    gload_pair(0, lds, lds + STAGE, 1);
    gload_pair(2, lds + 2 * STAGE, lds + 3 * STAGE, 0);
    gload_pair(2, lds + 2 * STAGE, lds + 3 * STAGE, 1);
    ring_barrier<2 * NLD + 1>();
    bf16x8 xfA[TM], wfA[TN], xfB[TM], wfB[TN];
    frags(lds, 0, xfA, wfA);
    __builtin_amdgcn_sched_barrier(0);

    auto stage_of = [&](int st) { return lds + st * STAGE; };
    auto wrap = [](int st) { return st >= NSTAGE ? st - NSTAGE : st; };
    int sc = 0;   // stage of k-tile kt
    int kt = 0;
    for (; kt + 1 < nk; kt += 2) {
        // ---- even k-tile kt: no loads ------------------------------------------------------------
        frags(stage_of(sc), 1, xfB, wfB);
        mfmas(xfA, wfA);
        pin_order(std::integral_constant<int, 0>{});
        ring_barrier<2 * NLD>();   // k-tile kt + 1 (second half of its pair) has landed; pair (kt+2, kt+3) may fly
        frags(stage_of(wrap(sc + 1)), 0, xfA, wfA);
        mfmas(xfB, wfB);
        pin_order(std::integral_constant<int, 0>{});
        // ---- odd k-tile kt + 1: the loads of pair (kt + 4, kt + 5), into the stages of k-tiles kt - 1 and kt ----
        bf16* f0 = stage_of(wrap(sc + 4));
        bf16* f1 = stage_of(sc);
        frags(stage_of(wrap(sc + 1)), 1, xfB, wfB);
        gload_pair(kt + 4, f0, f1, 0);
        mfmas(xfA, wfA);
        pin_order(std::integral_constant<int, NLD>{});
        // k-tile kt + 2 = first halves of pair (kt+2, kt+3): all but that pair's last load, and not the NLD just issued
        ring_barrier<NLD + 1>();
        frags(stage_of(wrap(sc + 2)), 0, xfA, wfA);
        gload_pair(kt + 4, f0, f1, 1);
        mfmas(xfB, wfB);
        pin_order(std::integral_constant<int, NLD>{});
        sc = wrap(sc + 2);
    }
    if (kt < nk) {   // odd number of k-tiles: the last one on its own
        frags(stage_of(sc), 1, xfB, wfB);
        mfmas(xfA, wfA);
        mfmas(xfB, wfB);
    }
    wait_all_memory();   // the repeated loads of the last k-tile must not land in the epilogue's slabs
    __syncthreads();

    // ---- epilogue: 32 output rows per pass through a wave-private fp32 slab ----
    // acc[i][j][e]: output row m = wm*WTM + i*32 + r, column n = j*32 + (e/4)*8 + h*4 + (e%4)
    constexpr int SLD = WOUT + 4;
    float* slab = reinterpret_cast<float*>(smem) + wave * 32 * SLD;
    constexpr int NCH = WOUT / 8;  // 8-column chunks per row
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        __syncthreads();
        constexpr int TJ = EPI == 1 ? TN / 2 : TN;
#pragma unroll
        for (int j = 0; j < TJ; ++j)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                floatx4 v;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    float a = acc[i][j][g * 4 + e];
                    if (EPI == 1) {
                        const float u = acc[i][j + TN / 2][g * 4 + e];
                        a = a / (1.0f + __expf(-a)) * u;
                    }
                    v[e] = a;
                }
                *reinterpret_cast<floatx4*>(slab + r * SLD + j * 32 + g * 8 + h * 4) = v;
            }
        __syncthreads();
        for (int q = lane; q < 32 * NCH; q += 64) {
            const int row = q / NCH, c = q % NCH;
            const int lm = wm * WTM + i * 32 + row;  // row inside the tile
            const int n = n0 + wn * WOUT + c * 8;
            if (lm >= rows_valid || n >= p.N) continue;
            const int64_t gm = m0 + lm;
            float v[8];
            const floatx4 a = *reinterpret_cast<const floatx4*>(slab + row * SLD + c * 8);
            const floatx4 b = *reinterpret_cast<const floatx4*>(slab + row * SLD + c * 8 + 4);
            v[0] = a[0]; v[1] = a[1]; v[2] = a[2]; v[3] = a[3];
            v[4] = b[0]; v[5] = b[1]; v[6] = b[2]; v[7] = b[3];
            if (GROUPED && p.g.row_scale) {
                const float sc = p.g.row_scale[gm];
#pragma unroll
                for (int e = 0; e < 8; ++e) v[e] *= sc;
            }
            if (p.R && p.r_f32) {
                const float* rf = reinterpret_cast<const float*>(p.R) + gm * p.N + n;
                const floatx4 r0 = *reinterpret_cast<const floatx4*>(rf);
                const floatx4 r1 = *reinterpret_cast<const floatx4*>(rf + 4);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    v[e] += r0[e];
                    v[4 + e] += r1[e];
                }
            } else if (p.R) {
                const bf16x8 rv = *reinterpret_cast<const bf16x8*>(p.R + gm * p.N + n);
#pragma unroll
                for (int e = 0; e < 8; ++e) v[e] += (float)rv[e];
            }
            if (EPI == 2) {   // fp32 output (router logits)
                float* cf = reinterpret_cast<float*>(p.C) + gm * p.N + n;
                *reinterpret_cast<floatx4*>(cf) = floatx4{v[0], v[1], v[2], v[3]};
                *reinterpret_cast<floatx4*>(cf + 4) = floatx4{v[4], v[5], v[6], v[7]};
            } else {
                bf16x8 o;
#pragma unroll
                for (int e = 0; e < 8; ++e) o[e] = (bf16)v[e];
                *reinterpret_cast<bf16x8*>(p.C + gm * p.N + n) = o;
            }
        }
    }
}

template <int BM, int BN, int WM, int WN, int EPI, bool GROUPED>
static int launch_cfg(compact_ctx* ctx, GemmParams& p, hipStream_t s) {
    constexpr int OUTN = EPI == 1 ? BN / 2 : BN;
    constexpr int WOUT = (EPI == 1 ? BN / 2 : BN) / WN;
    if (!GROUPED) p.n_mtiles = (int)((p.M + BM - 1) / BM);
    p.n_ntiles = (p.N + OUTN - 1) / OUTN;
    const size_t stage_bytes = (size_t)GEMM_STAGES * (BM + BN) * GEMM_BK * sizeof(bf16);
    const size_t slab_bytes = (size_t)WM * WN * 32 * (WOUT + 4) * sizeof(float);
    const size_t smem = std::max(stage_bytes, slab_bytes);
    auto kern = gemm_bf16_kernel<BM, BN, WM, WN, EPI, GROUPED>;
    static bool attr_set = false;
    if (!attr_set) {
        HIP_TRY(ctx, hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
        attr_set = true;
    }
    const int64_t tiles = (int64_t)p.n_mtiles * p.n_ntiles;
    if (tiles == 0) return COMPACT_OK;
    kern<<<dim3((unsigned)tiles), WM * WN * 64, smem, s>>>(p);
    LAUNCH_CHECK(ctx);
    return COMPACT_OK;
}

// Row-tile height used for the grouped expert GEMMs.
int gemm_bf16_mtile() { return 256; }

int launch_gemm_bf16(compact_ctx* ctx, const bf16* A, const bf16* B, const void* R, bool r_f32, bf16* C, int64_t M, int N,
                     int K, int epilogue, const GroupedArgs* grouped, hipStream_t s) {
    if (M == 0) return COMPACT_OK;
    if (K % GEMM_BK != 0 || N % 8 != 0) return set_err(ctx, COMPACT_ESHAPE, "bf16 GEMM needs K % 32 == 0 and N % 8 == 0");
    GemmParams p{};
    p.X = A;
    p.W = B;
    p.R = reinterpret_cast<const bf16*>(R);
    p.r_f32 = r_f32 ? 1 : 0;
    p.C = C;
    p.M = M;
    p.N = N;
    p.K = K;
    if (grouped) {
        p.g = *grouped;
        p.n_mtiles = grouped->n_mtiles;
        if (epilogue == 1) return launch_cfg<256, 256, 2, 4, 1, true>(ctx, p, s);
        return launch_cfg<256, 256, 2, 4, 0, true>(ctx, p, s);
    }
    if (epilogue == 1) return launch_cfg<256, 256, 2, 4, 1, false>(ctx, p, s);
    if (epilogue == 2) return launch_cfg<256, 256, 2, 4, 2, false>(ctx, p, s);
    return launch_cfg<256, 256, 2, 4, 0, false>(ctx, p, s);
}
