// Weight-streaming GEMM for the decode step: a handful of activation rows
// (one per block, M <= 64) against a weight matrix that must be read once from
// HBM.  partials[slice][M][N] = X[M, kslice] W[N, kslice]^T in fp32; the
// caller's next row kernel sums the slices in slice order.
//
//  * each wavefront owns 16 weight rows and one K-slice; its 16-byte loads go
//    straight from global memory into the MFMA operand layout (lane (r, c)
//    holds 8 consecutive k of weight row r), all loads of the slice issued
//    before the first MFMA so that a wave keeps 16 KB in flight;
//  * v_mfma_f32_16x16x32_bf16 with the weight rows as MFMA rows and the
//    (zero-padded) activation rows as MFMA columns; the activation slice is
//    staged once per workgroup in LDS;
//  * the K-split depends on K alone, never on the number of activation rows,
//    so a block's result does not depend on the batch it is decoded in.
#include "common.h"

#define SKINNY_KSLICE 512
#define SKINNY_STEPS (SKINNY_KSLICE / 32)

int skinny_ksplit(int M, int N, int K) {
    (void)M;
    (void)N;
    return (K + SKINNY_KSLICE - 1) / SKINNY_KSLICE;
}

// GROUPED: blockIdx.z is an expert; its rows are rows offsets[e] .. offsets[e+1]-1
// of the expert-sorted order (at most MT*16 of them), read from X through
// a_gather (null: X is already in sorted order), multiplied with that expert's
// weight matrix, and the partials keep the sorted order: P[slice][sorted row][N].
// Experts nobody was routed to leave at once.  With a tile map (expert_list =
// the map's experts, tile_row0 / tile_rows its row ranges, tiles of at most MT*16
// rows) blockIdx.z is a tile: an expert with more rows than a tile holds is
// streamed once per tile.
struct SkinnyGroup {
    const int32_t* expert_list;  // [gridDim.z] experts to run, -1 = none (null: expert = blockIdx.z)
    const int32_t* tile_row0;    // [gridDim.z] first sorted row of the tile (null: the expert's first row)
    const int32_t* tile_rows;    // [gridDim.z] rows of the tile (null: all of the expert's rows)
    const int32_t* offsets;   // [E + 1]
    const int32_t* a_gather;  // [total_rows] or null
    int64_t w_expert_stride;  // elements
    int total_rows;
};

// Front half of an RMSNorm folded into the activation staging (null g: off): the
// staged operand is bf16(x * g) and the workgroups of the first column tile leave
// ssq_parts[slice][row] = sum of x^2 over the slice; the consumer of the partials
// multiplies by 1 / rms.
struct SkinnyNormIn {
    const bf16* g = nullptr;
    float* ssq_parts = nullptr;
};

// RING < SKINNY_STEPS: only the first RING loads of the slice go out at once, the rest one per k-step as the
// registers come free (half the registers per wavefront, twice the wavefronts per CU for the same bytes in flight).
template <int MT, bool GROUPED, int WAVES, int RING = SKINNY_STEPS>
__global__ __launch_bounds__(WAVES * 64, RING < SKINNY_STEPS ? 2 : 1) void gemm_skinny_kernel(const bf16* __restrict__ X, const bf16* __restrict__ W,
                                                          float* __restrict__ P, int M, int N, int K, const SkinnyGroup grp,
                                                          const SkinnyNormIn nin) {
    constexpr int LDX = SKINNY_KSLICE + 8;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    bf16* xs = reinterpret_cast<bf16*>(smem);  // [MT*16][LDX]
    const int t = threadIdx.x;
    const int lane = t & 63, wave = t >> 6;
    int row_base = 0, p_rows = M;
    if (GROUPED) {
        const int e = grp.expert_list ? grp.expert_list[blockIdx.z] : (int)blockIdx.z;
        if (e < 0) return;
        row_base = grp.tile_row0 ? grp.tile_row0[blockIdx.z] : grp.offsets[e];
        M = min(grp.tile_rows ? grp.tile_rows[blockIdx.z] : grp.offsets[e + 1] - row_base, MT * 16);
        if (M <= 0) return;
        W += (size_t)e * grp.w_expert_stride;
        p_rows = grp.total_rows;
    }
    // the K-slice is the fastest grid index: workgroups that run together read
    // neighbouring slices of the same weight rows (whole DRAM pages), not the same
    // slice of far-apart rows
    const int slice = blockIdx.x;
    const int k0 = slice * SKINNY_KSLICE;
    const int klen = min(SKINNY_KSLICE, K - k0);
    const int nsteps = klen / 32;
    const int r = lane & 15, c = lane >> 4;
    const int n0 = (blockIdx.y * WAVES + wave) * 16;
    const bool active = n0 < N;

    // the weight stream goes first: everything below overlaps with it
    bf16x8 a[RING];
    const bf16* wp = W + (size_t)(min(n0, N - 16) + r) * K + k0 + c * 8;
    if (active) {
#pragma unroll
        for (int s = 0; s < RING; ++s)
            if (s < nsteps) a[s] = *reinterpret_cast<const bf16x8*>(wp + s * 32);
    }

    const int cpr = klen / 8;  // 16-byte chunks per row (at most 64)
    if (!GROUPED && nin.g) {
        // RMSNorm front half: a wavefront stages whole rows, so that the row's sum of
        // squares over this slice is one butterfly (fixed order)
        for (int row = wave; row < MT * 16; row += WAVES) {
            bf16x8 v;
#pragma unroll
            for (int j = 0; j < 8; ++j) v[j] = (bf16)0.f;
            float ss = 0.f;
            if (row < M && lane < cpr) {
                v = *reinterpret_cast<const bf16x8*>(X + (size_t)row * K + k0 + lane * 8);
                const bf16x8 gv = *reinterpret_cast<const bf16x8*>(nin.g + k0 + lane * 8);
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const float f = (float)v[j];
                    ss += f * f;
                    v[j] = (bf16)(f * (float)gv[j]);
                }
            }
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) ss += __shfl_xor(ss, o, 64);
            if (lane == 0 && blockIdx.y == 0 && row < M) nin.ssq_parts[(size_t)slice * M + row] = ss;
            if (lane < cpr) *reinterpret_cast<bf16x8*>(xs + row * LDX + lane * 8) = v;
        }
    } else {
        for (int q = t; q < MT * 16 * cpr; q += WAVES * 64) {
            const int row = q / cpr, cc = q - row * cpr;
            bf16x8 v;
#pragma unroll
            for (int j = 0; j < 8; ++j) v[j] = (bf16)0.f;
            if (row < M) {
                size_t src = row_base + row;
                if (GROUPED && grp.a_gather) src = grp.a_gather[src];
                v = *reinterpret_cast<const bf16x8*>(X + src * K + k0 + cc * 8);
            }
            *reinterpret_cast<bf16x8*>(xs + row * LDX + cc * 8) = v;
        }
    }
    __syncthreads();
    if (!active) return;

    floatx4 acc[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) acc[mt] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s = 0; s < SKINNY_STEPS; ++s) {
        if (s < nsteps) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                const bf16x8 b = *reinterpret_cast<const bf16x8*>(xs + (mt * 16 + r) * LDX + s * 32 + c * 8);
                acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[s % RING], b, acc[mt], 0, 0, 0);
            }
            if (RING < SKINNY_STEPS && s + RING < SKINNY_STEPS && s + RING < nsteps)
                a[s % RING] = *reinterpret_cast<const bf16x8*>(wp + (s + RING) * 32);
        }
    }
    // acc[mt][e]: activation row m = mt*16 + r, weight row n = n0 + 4c + e
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const int m = mt * 16 + r;
        if (m < M) *reinterpret_cast<floatx4*>(P + ((size_t)slice * p_rows + row_base + m) * N + n0 + 4 * c) = acc[mt];
    }
}

// ---------------------------------------------------------------------------
// Gate/up projection of the decode step with the SwiGLU fused in:
// act[M, F] = silu(X Wg^T) * (X Wu^T) for M <= MROWS activation rows.
// A workgroup (16 wavefronts) owns 32 act columns = SG_TILES = four MFMA tiles of 8 gate +
// 8 up weight rows, over the whole K.  Wavefront (rt, kw) streams tile rt's
// k-steps kw, kw+4, kw+8, ... so that the four wavefronts of a tile read
// neighbouring 64-byte pieces of the same weight rows at the same time; each
// keeps a ring of 8 loads in flight.  The partial tiles are added in kw order
// through LDS (over the staged activations, dead by then), then gate and up
// values (32 lanes apart in the accumulator layout) are paired by shuffle.  No
// split-K partials leave the kernel.  SPW = k-steps of 32 per wavefront = K / 128.
// Four tiles per workgroup with 64 registers per lane: two workgroups per CU hold
// all 448 workgroups of the 8B-shaped layer at once (two tiles, 8 wavefronts, a
// ring of 16: 896 workgroups in 1.75 rounds and twice the activation staging,
// 52.2 us against 49.6 us).
// ---------------------------------------------------------------------------
#define SG_TILES 4
#define SG_RING 8
template <int MROWS, int SPW>
__global__ __launch_bounds__(SG_TILES * 256, 2) void gemm_skinny_swiglu_kernel(const bf16* __restrict__ X, const bf16* __restrict__ W,
                                                                 bf16* __restrict__ act, int M, int F, const RowNorm norm) {
    constexpr int K = SPW * 128;
    constexpr int LDX = K + 8;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    bf16* xs = reinterpret_cast<bf16*>(smem);                                          // [MROWS][LDX]
    float* red = reinterpret_cast<float*>(smem);  // [4 SG_TILES][64][4], over the activations once every wavefront is done with them
    __shared__ float rinv[16];
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int rt = wave >> 2, kw = wave & 3;
    const int r = lane & 15, c = lane >> 4;
    const int j0 = blockIdx.x * (SG_TILES * 8);

    // weight row of MFMA row r: 8 gate rows then the 8 matching up rows
    const int col = min(j0 + rt * 8 + (r & 7), F - 1);
    const bf16* wrow = W + (size_t)(r < 8 ? col : F + col) * K + kw * 32 + c * 8;
    bf16x8 ring[SG_RING];
#pragma unroll
    for (int i = 0; i < SG_RING && i < SPW; ++i) ring[i] = *reinterpret_cast<const bf16x8*>(wrow + i * 128);

    // activations: all of K for the M rows
    constexpr int CPR = K / 8;
    for (int q = t; q < MROWS * CPR; q += SG_TILES * 256) {
        const int row = q / CPR, cc = q - row * CPR;
        bf16x8 v;
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = (bf16)0.f;
        if (row < M) v = *reinterpret_cast<const bf16x8*>(X + (size_t)row * K + cc * 8);
        *reinterpret_cast<bf16x8*>(xs + row * LDX + cc * 8) = v;
    }
    // Column-group sums of squares of the rows this wavefront finishes (rows w and
    // w + 8): only loaded here (behind the weight ring and the activations),
    // lane-strided; they are added up after the main loop, so nothing waits for them.
    constexpr int NRW = MROWS / 8, PMAX = 8;   // rows per wavefront; parts per lane (nparts <= 512)
    float pv[NRW][PMAX];
#pragma unroll
    for (int j = 0; j < NRW; ++j)
#pragma unroll
        for (int u = 0; u < PMAX; ++u) {
            const int row = wave + 8 * j, pidx = lane + 64 * u;
            pv[j][u] = (norm.ssq_parts && wave < 8 && row < M && pidx < norm.nparts) ? norm.ssq_parts[(size_t)pidx * M + row] : 0.f;
        }
    __syncthreads();

    floatx4 acc = floatx4{0.f, 0.f, 0.f, 0.f};
    const bool xvalid = r < MROWS;
    const bf16* xrow = xs + (xvalid ? r : 0) * LDX + kw * 32 + c * 8;
#pragma unroll
    for (int i = 0; i < SPW; ++i) {
        bf16x8 b = *reinterpret_cast<const bf16x8*>(xrow + i * 128);
        if (MROWS < 16 && !xvalid) {
#pragma unroll
            for (int j = 0; j < 8; ++j) b[j] = (bf16)0.f;
        }
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ring[i % SG_RING], b, acc, 0, 0, 0);
        if (i + SG_RING < SPW) ring[i % SG_RING] = *reinterpret_cast<const bf16x8*>(wrow + (i + SG_RING) * 128);
    }

    // 1/rms of the rows: a fixed summation order (per lane, then a butterfly)
#pragma unroll
    for (int j = 0; j < NRW; ++j) {
        float ss = 0.f;
#pragma unroll
        for (int u = 0; u < PMAX; ++u) ss += pv[j][u];
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) ss += __shfl_xor(ss, o, 64);
        if (lane == 0 && wave < 8) rinv[wave + 8 * j] = norm.ssq_parts ? 1.0f / sqrtf(ss * norm.inv_d + norm.eps) : 1.0f;
    }
    // add the four k-interleaves of each tile in kw order
    __syncthreads();   // the activations are dead: the partial tiles take their place
    *reinterpret_cast<floatx4*>(red + (wave * 64 + lane) * 4) = acc;
    __syncthreads();
    if (kw != 0) return;
    floatx4 v = acc;
#pragma unroll
    for (int w = 1; w < 4; ++w) {
        const floatx4 o = *reinterpret_cast<const floatx4*>(red + ((rt * 4 + w) * 64 + lane) * 4);
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] += o[e];
    }
    // v[e]: activation row r, MFMA row 4c + e: c < 2 gate of column 4c + e, c >= 2 up of column 4(c-2) + e
    const float rs = rinv[xvalid ? r : 0];
    bf16x4 out;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const float up = __shfl_xor(v[e], 32, 64) * rs;
        const float g = v[e] * rs;
        out[e] = (bf16)(g / (1.0f + __expf(-g)) * up);
    }
    if (c < 2 && r < M && j0 + rt * 8 + 4 * c < F) *reinterpret_cast<bf16x4*>(act + (size_t)r * F + j0 + rt * 8 + 4 * c) = out;
}

static size_t swiglu_smem(int mrows, int K) { return std::max((size_t)mrows * (K + 8) * sizeof(bf16), (size_t)SG_TILES * 4 * 64 * 4 * sizeof(float)); }

// whether the fused SwiGLU kernel covers this shape (K in {2048, 4096, 8192}, the LDS holds the activations)
bool skinny_swiglu_supported(int M, int F, int K) {
    if (M < 1 || M > 16 || F % 16 != 0) return false;
    if (K != 2048 && K != 4096 && K != 8192) return false;
    return swiglu_smem(M <= 8 ? 8 : 16, K) <= 160 * 1024;
}

template <int MROWS, int SPT>
static int launch_swiglu_cfg(compact_ctx* ctx, const bf16* X, const bf16* W, bf16* act, int M, int F, const RowNorm& norm,
                             hipStream_t s) {
    const size_t smem = swiglu_smem(MROWS, SPT * 128);
    static bool attr = false;
    if (!attr) {
        HIP_TRY(ctx, hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_skinny_swiglu_kernel<MROWS, SPT>),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
        attr = true;
    }
    gemm_skinny_swiglu_kernel<MROWS, SPT><<<(F + SG_TILES * 8 - 1) / (SG_TILES * 8), SG_TILES * 256, smem, s>>>(X, W, act, M, F, norm);
    LAUNCH_CHECK(ctx);
    return COMPACT_OK;
}

int launch_gemm_skinny_swiglu(compact_ctx* ctx, const bf16* X, const bf16* W, bf16* act, int M, int F, int K,
                              const RowNorm* norm, hipStream_t s) {
    if (!skinny_swiglu_supported(M, F, K)) return set_err(ctx, COMPACT_ESHAPE, "fused gate/up decode kernel does not cover this shape");
    const RowNorm rn = norm ? *norm : RowNorm{};
    const bool small = M <= 8;
    switch (K) {
        case 2048: return small ? launch_swiglu_cfg<8, 16>(ctx, X, W, act, M, F, rn, s) : launch_swiglu_cfg<16, 16>(ctx, X, W, act, M, F, rn, s);
        case 4096: return small ? launch_swiglu_cfg<8, 32>(ctx, X, W, act, M, F, rn, s) : launch_swiglu_cfg<16, 32>(ctx, X, W, act, M, F, rn, s);
        default: return launch_swiglu_cfg<8, 64>(ctx, X, W, act, M, F, rn, s);   // K = 8192 fits 8 rows only
    }
}

template <int MT, int WAVES, int RING = SKINNY_STEPS>
static int launch_skinny_cfg(compact_ctx* ctx, const bf16* A, const bf16* B, float* partials, int M, int N, int K, int ks,
                             const SkinnyNormIn& nin, hipStream_t s) {
    const size_t smem = (size_t)MT * 16 * (SKINNY_KSLICE + 8) * sizeof(bf16);
    static bool attr = false;
    if (!attr && smem > 48 * 1024) {
        HIP_TRY(ctx, hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_skinny_kernel<MT, false, WAVES, RING>),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
        attr = true;
    }
    dim3 grid(ks, (N + 16 * WAVES - 1) / (16 * WAVES));
    gemm_skinny_kernel<MT, false, WAVES, RING><<<grid, WAVES * 64, smem, s>>>(A, B, partials, M, N, K, SkinnyGroup{}, nin);
    LAUNCH_CHECK(ctx);
    return COMPACT_OK;
}

// One workgroup = 4 wavefronts (64 weight rows) for up to 16 activation rows; with
// more rows the staged activation slice grows, so 8 wavefronts (128 weight rows)
// share it: half the activation traffic per weight byte, the same number of
// wavefronts per compute unit.
bool skinny_norm_in_supported(int M, int N, int K) { return M >= 1 && M <= 64 && N % 16 == 0 && K % 64 == 0; }

int launch_gemm_skinny(compact_ctx* ctx, const bf16* A, const bf16* B, float* partials, int M, int N, int K, int ks,
                       hipStream_t s, const bf16* norm_g, float* norm_ssq_parts) {
    if (M < 1 || M > 64) return set_err(ctx, COMPACT_ESHAPE, "weight-streaming GEMM takes 1..64 activation rows");
    if (N % 16 != 0 || K % 64 != 0) return set_err(ctx, COMPACT_ESHAPE, "weight-streaming GEMM needs N % 16 == 0 and K % 64 == 0");
    if (ks != skinny_ksplit(M, N, K)) return set_err(ctx, COMPACT_EINVAL, "unexpected K split");
    SkinnyNormIn nin;
    if (norm_g) {
        if (!skinny_norm_in_supported(M, N, K) || !norm_ssq_parts)
            return set_err(ctx, COMPACT_ESHAPE, "folding the RMSNorm into the weight-streaming GEMM needs K % 64 == 0");
        nin.g = norm_g;
        nin.ssq_parts = norm_ssq_parts;
    }
    // 49 .. 64 rows: two workgroups of 8 wavefronts fit a CU (the staged slice is 66 KB); a grid beyond what the
    // chip holds at once (the down projection of the 8B-shaped layer: 28 slices x 32 column groups) goes to
    // workgroups of 16 wavefronts with 6 of the 16 loads up front instead: again two per CU, all resident in one
    // round, half the activation staging (39.9 -> 34.9 us; at 32 rows the same change cost 2 us and is not made)
    int n_cus = 0;
    if (int rc = device_cu_count(ctx, &n_cus)) return rc;
    const bool fat = (int64_t)ks * ((N + 127) / 128) > 2 * (int64_t)n_cus;
    switch ((M + 15) / 16) {
        case 1: return launch_skinny_cfg<1, 4>(ctx, A, B, partials, M, N, K, ks, nin, s);
        case 2: return launch_skinny_cfg<2, 8>(ctx, A, B, partials, M, N, K, ks, nin, s);
        case 3: return launch_skinny_cfg<3, 8>(ctx, A, B, partials, M, N, K, ks, nin, s);
        default: return fat ? launch_skinny_cfg<4, 16, 6>(ctx, A, B, partials, M, N, K, ks, nin, s)
                            : launch_skinny_cfg<4, 8>(ctx, A, B, partials, M, N, K, ks, nin, s);
    }
}

// Per-expert weight streaming for routed decode rows (at most 16 rows per expert):
// partials[ks][total_rows][N], rows in expert-sorted order.
int launch_gemm_skinny_grouped(compact_ctx* ctx, const bf16* X, const int32_t* a_gather, const bf16* W, int64_t w_expert_stride,
                               const int32_t* offsets, int n_experts, int total_rows, float* partials, int N, int K, int ks,
                               hipStream_t s, const int32_t* expert_list, int n_listed, const int32_t* tile_row0,
                               const int32_t* tile_rows) {
    if (N % 16 != 0 || K % 64 != 0) return set_err(ctx, COMPACT_ESHAPE, "weight-streaming GEMM needs N % 16 == 0 and K % 64 == 0");
    if (ks != skinny_ksplit(1, N, K)) return set_err(ctx, COMPACT_EINVAL, "unexpected K split");
    SkinnyGroup g{expert_list, tile_row0, tile_rows, offsets, a_gather, w_expert_stride, total_rows};
    dim3 grid(ks, (N + 63) / 64, expert_list ? n_listed : n_experts);
    const size_t smem = (size_t)16 * (SKINNY_KSLICE + 8) * sizeof(bf16);
    gemm_skinny_kernel<1, true, 4><<<grid, 256, smem, s>>>(X, W, partials, 0, N, K, g, SkinnyNormIn{});
    LAUNCH_CHECK(ctx);
    return COMPACT_OK;
}

// C = sum_s partials[s] (+R), rounded to bf16
__global__ __launch_bounds__(256) void skinny_finish_kernel(const float* __restrict__ P, int ks, const bf16* __restrict__ R,
                                                            bf16* __restrict__ C, int M, int N) {
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    const size_t total = (size_t)M * N;
    if (i >= total) return;
    float v = R ? (float)R[i] : 0.f;
    for (int s = 0; s < ks; ++s) v += P[s * total + i];
    C[i] = (bf16)v;
}

int launch_skinny_finish(compact_ctx* ctx, const float* partials, int ks, const bf16* R, bf16* C, int M, int N,
                         hipStream_t s) {
    const size_t total = (size_t)M * N;
    skinny_finish_kernel<<<(unsigned)((total + 255) / 256), 256, 0, s>>>(partials, ks, R, C, M, N);
    LAUNCH_CHECK(ctx);
    return COMPACT_OK;
}
