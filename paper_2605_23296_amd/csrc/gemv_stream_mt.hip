// Whole-K weight-streaming projections of the decode step for 17 .. 64 activation
// rows (bf16 storage): the kernels of gemv_stream.hip / gemm_skinny.hip's fused
// gate/up kernel with MT = 2 .. 4 groups of 16 activation rows sharing every
// weight fragment (one MFMA per group and k-step).  As there, a workgroup owns
// complete output columns, so nothing but the finished result leaves the kernel:
// no split-K partials, no reduce launches.
//
//  * the activation rows do not fit in LDS beside the stream (64 rows x K), so they
//    pass through it slice by slice: all wavefronts of the workgroup copy the next
//    slice of K (all rows, whole 128-byte lines, from L2) while the current one
//    feeds the MFMAs, two LDS buffers, one barrier per slice that leaves global
//    loads in flight.  (Loading the MFMA operand fragments of the activations
//    straight from global memory, 16 rows x 64 bytes per instruction, as the
//    kernels for at most 16 rows do, moved 5 x the weight bytes through the vector
//    cache at a fifth of its line rate: 216 us for the gate/up projection.)
//  * the weight fragments travel through a ring of loads per wavefront, every load
//    unconditional (past the end the last k-step is read again), so that the ring
//    stays in flight across the barriers;
//  * the split over K between the wavefronts of a workgroup and the order in which
//    their partial tiles are added are those of the kernels for at most 16 rows:
//    a row's result does not depend on how many rows share the step.
#include <algorithm>

#include "common.h"

#define MTS_WAVES 16

// Workgroup barrier that waits for this wavefront's LDS operations only (global loads stay in flight).
__device__ __forceinline__ void mts_barrier() {
#if defined(__HIP_DEVICE_COMPILE__)
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_waitcnt(15 | (7 << 4) | (0 << 8) | (3 << 14));
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
#endif
}

// A slice of SLICE consecutive k of all MT*16 activation rows, copied by NT threads: chunk q (16 bytes) of the
// slice = row q / (SLICE/8), piece q % (SLICE/8); rows past M are zero.
template <int MT, int SLICE, int NT>
struct SliceStager {
    static constexpr int CPR = SLICE / 8;                 // 16-byte pieces per row
    static constexpr int TOTAL = MT * 16 * CPR;           // pieces of a slice
    static constexpr int PER = (TOTAL + NT - 1) / NT;     // pieces per thread (the last round may be partial)
    static constexpr int LDX = SLICE + 8;                 // LDS row stride (elements), padded against bank conflicts
    bf16x8 v[PER];
    __device__ __forceinline__ void load(const bf16* __restrict__ X, int M, int K, int k0, int t) {
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int q = min(t + i * NT, TOTAL - 1), row = q / CPR, cc = q % CPR;   // past the end: the last piece again
            v[i] = *reinterpret_cast<const bf16x8*>(X + (size_t)min(row, M - 1) * K + k0 + cc * 8);   // unconditional
        }
    }
    __device__ __forceinline__ void store(bf16* xs, int M, int t) const {
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int q = t + i * NT, row = q / CPR, cc = q % CPR;
            if (TOTAL % NT != 0 && q >= TOTAL) continue;
            bf16x8 w = v[i];
            if (row >= M) {
#pragma unroll
                for (int j = 0; j < 8; ++j) w[j] = (bf16)0.f;
            }
            *reinterpret_cast<bf16x8*>(xs + row * LDX + cc * 8) = w;
        }
    }
};

// ---------------------------------------------------------------------------
// One 16-column tile per workgroup of 16 wavefronts, wavefront kw takes the k-steps kw, kw + 16, ...: k-step j of
// every wavefront lies in the j-th slice of 512 k.
// h = resid + X W^T (fp32), hg = bf16(h * g), ssq_parts[tile][m] = sum over the tile's columns of h^2: the output
// projection with the residual add and the front half of the next RMSNorm.  (The down projection stays on the
// split-K kernels beyond 16 rows: its K is 3.5 x longer, and every workgroup of a whole-K kernel has to pull all
// M x K activations through L2: four times the weight bytes at 64 rows, 49 us against 31 us.)
// ---------------------------------------------------------------------------
#define MTS_RING 8
template <int MT>
__global__ __launch_bounds__(MTS_WAVES * 64) void stream_tile_mt_kernel(const bf16* __restrict__ X, const bf16* __restrict__ W,
                                                                        const bf16* __restrict__ resid, const bf16* __restrict__ g,
                                                                        float* __restrict__ h_out, bf16* __restrict__ out16,
                                                                        float* __restrict__ ssq_parts, int M, int N, int K) {
    typedef SliceStager<MT, 512, MTS_WAVES * 64> Stager;
    constexpr int LDX = Stager::LDX;
    extern __shared__ __attribute__((aligned(16))) char smem_mt[];
    bf16* xs0 = reinterpret_cast<bf16*>(smem_mt);                 // two slices [MT*16][LDX] ...
    bf16* xs1 = xs0 + MT * 16 * LDX;
    floatx4(*red)[MTS_WAVES * 64] = reinterpret_cast<floatx4(*)[MTS_WAVES * 64]>(smem_mt);   // ... reused for the partial tiles
    const int t = threadIdx.x, lane = t & 63;
    const int kw = __builtin_amdgcn_readfirstlane(t >> 6);
    const int r = lane & 15, c = lane >> 4;
    const int tile = blockIdx.x;
    const int S = K / 512;   // slices = k-steps per wavefront
    const bf16* w0 = W + (size_t)(tile * 16 + r) * K + kw * 32 + c * 8;
    bf16x8 wf[MTS_RING];
#pragma unroll
    for (int i = 0; i < MTS_RING; ++i) wf[i] = *reinterpret_cast<const bf16x8*>(w0 + (size_t)min(i, S - 1) * 512);
    Stager st;
    st.load(X, M, K, 0, t);
    st.store(xs0, M, t);
    st.load(X, M, K, min(1, S - 1) * 512, t);
    mts_barrier();
    floatx4 acc[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) acc[mt] = floatx4{0.f, 0.f, 0.f, 0.f};
    for (int j0 = 0; j0 < S; j0 += MTS_RING) {
#pragma unroll
        for (int i = 0; i < MTS_RING; ++i) {
            const int j = j0 + i;
            if (j < S) {   // uniform
                const bf16* xs = (i & 1) ? xs1 : xs0;   // MTS_RING is even: slice j sits in buffer j & 1 = i & 1
                bf16* xn = (i & 1) ? xs0 : xs1;
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) {
                    const bf16x8 b = *reinterpret_cast<const bf16x8*>(xs + (mt * 16 + r) * LDX + kw * 32 + c * 8);
                    acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[i], b, acc[mt], 0, 0, 0);
                }
                wf[i] = *reinterpret_cast<const bf16x8*>(w0 + (size_t)min(j + MTS_RING, S - 1) * 512);
                // slice j + 1 (loaded one round ago) goes into the buffer round j - 1 has finished with
                st.store(xn, M, t);
                st.load(X, M, K, min(j + 2, S - 1) * 512, t);
                mts_barrier();
            }
        }
    }
    // (the last round's barrier has passed: nobody reads the slices any more)
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) red[mt][kw * 64 + lane] = acc[mt];
    __syncthreads();
    if (kw >= MT) return;
    // wavefront kw finishes group kw: the 16 partial tiles in wavefront order
    const int mt = kw;
    floatx4 v = red[mt][lane];
#pragma unroll
    for (int w = 1; w < MTS_WAVES; ++w) {
        const floatx4 o = red[mt][w * 64 + lane];
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] += o[e];
    }
    // v[e]: activation row m = mt*16 + r, output column n = tile*16 + 4c + e
    const int m = mt * 16 + r;
    float ss = 0.f;
    if (m < M) {
        const size_t o = (size_t)m * N + tile * 16 + 4 * c;
        const bf16x4 rv = *reinterpret_cast<const bf16x4*>(resid + o);
        const bf16x4 gv = *reinterpret_cast<const bf16x4*>(g + tile * 16 + 4 * c);
        bf16x4 hg;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            v[e] += (float)rv[e];
            hg[e] = (bf16)(v[e] * (float)gv[e]);
            ss += v[e] * v[e];
        }
        *reinterpret_cast<floatx4*>(h_out + o) = v;
        *reinterpret_cast<bf16x4*>(out16 + o) = hg;
    }
    ss += __shfl_xor(ss, 16, 64);
    ss += __shfl_xor(ss, 32, 64);
    if (c == 0 && m < M) ssq_parts[(size_t)tile * M + m] = ss;
}

// ---------------------------------------------------------------------------
// Gate/up projection with the SwiGLU fused in, act[M, F] = silu(r X Wg^T) * (r X Wu^T), r = 1/rms of the row
// from the column-group sums of squares in `norm` (null parts: r = 1).
// A workgroup of 16 wavefronts owns 64 act columns = eight MFMA tiles of 8 gate + 8 up weight rows: every
// workgroup has to read all M x K activations, so few, fat workgroups keep that traffic (224 x 512 KB for the
// 8B-shaped layer at 64 rows) below the weight bytes.  The k-steps of a tile are dealt to four interleaves kw
// (k-step i of interleave kw starts at k = kw * 32 + i * 128) whose partial tiles are added in kw order, exactly as
// in the kernel for at most 16 rows; here wavefront (tile, kh) runs the interleaves 2 kh and 2 kh + 1 with separate
// accumulators, and wavefront (tile, 0) adds (p0 + p1) + p2 + p3.  Slices of 256 k = two k-steps per interleave.
// ---------------------------------------------------------------------------
#define SGM_RING 8
template <int MT>
__global__ __launch_bounds__(MTS_WAVES * 64) void swiglu_mt_kernel(const bf16* __restrict__ X, const bf16* __restrict__ W,
                                                                   bf16* __restrict__ act, int M, int F, int K,
                                                                   const RowNorm norm) {
    typedef SliceStager<MT, 256, MTS_WAVES * 64> Stager;
    constexpr int LDX = Stager::LDX;
    extern __shared__ __attribute__((aligned(16))) char smem_mt[];
    bf16* xs0 = reinterpret_cast<bf16*>(smem_mt);                 // two slices [MT*16][LDX] ...
    bf16* xs1 = xs0 + MT * 16 * LDX;
    floatx4* red = reinterpret_cast<floatx4*>(smem_mt);           // ... reused for the partial tiles [tile][2][MT][64 lanes]
    __shared__ float rinv[MT * 16];
    const int t = threadIdx.x, lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int rt = wave >> 1, kh = wave & 1;
    const int r = lane & 15, c = lane >> 4;
    const int j0 = blockIdx.x * 64;
    const int NS = K / 256;    // slices
    const int SPI = K / 128;   // k-steps per interleave
    // weight row of MFMA row r: 8 gate rows then the 8 matching up rows (columns past F: the last column again, not stored)
    const int col = min(j0 + rt * 8 + (r & 7), F - 1);
    const bf16* w0 = W + (size_t)(r < 8 ? col : F + col) * K + (2 * kh) * 32 + c * 8;
    // ring slot 4 (sl & 1) + 2 v + u: k-step 2 sl + u of interleave 2 kh + v
    auto wptr = [&](int step, int v) { return w0 + (size_t)min(step, SPI - 1) * 128 + v * 32; };
    bf16x8 wf[SGM_RING];
#pragma unroll
    for (int i = 0; i < SGM_RING; ++i) wf[i] = *reinterpret_cast<const bf16x8*>(wptr(2 * (i >> 2) + (i & 1), (i >> 1) & 1));
    Stager st;
    st.load(X, M, K, 0, t);
    st.store(xs0, M, t);
    st.load(X, M, K, min(1, NS - 1) * 256, t);
    mts_barrier();
    floatx4 acc[2][MT];
#pragma unroll
    for (int v = 0; v < 2; ++v)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) acc[v][mt] = floatx4{0.f, 0.f, 0.f, 0.f};
    for (int s0 = 0; s0 < NS; s0 += 2) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int sl = s0 + i;
            if (sl < NS) {   // uniform
                const bf16* xs = i ? xs1 : xs0;   // slice sl sits in buffer sl & 1 = i
                bf16* xn = i ? xs0 : xs1;
#pragma unroll
                for (int v = 0; v < 2; ++v)
#pragma unroll
                    for (int u = 0; u < 2; ++u) {
#pragma unroll
                        for (int mt = 0; mt < MT; ++mt) {
                            const bf16x8 b = *reinterpret_cast<const bf16x8*>(xs + (mt * 16 + r) * LDX + u * 128 + (2 * kh + v) * 32 + c * 8);
                            acc[v][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[4 * i + 2 * v + u], b, acc[v][mt], 0, 0, 0);
                        }
                        wf[4 * i + 2 * v + u] = *reinterpret_cast<const bf16x8*>(wptr(2 * (sl + 2) + u, v));
                    }
                st.store(xn, M, t);
                st.load(X, M, K, min(sl + 2, NS - 1) * 256, t);
                mts_barrier();
            }
        }
    }

    // 1/rms of the rows, MT rows per wavefront: a fixed summation order (per lane over the parts lane, lane + 64,
    // ..., then a butterfly), the loads of all rows issued together
    constexpr int PMAX = 8;   // parts per lane (nparts <= 512)
    float pv[MT][PMAX];
#pragma unroll
    for (int j = 0; j < MT; ++j)
#pragma unroll
        for (int u = 0; u < PMAX; ++u) {
            const int row = wave * MT + j, pidx = lane + 64 * u;
            pv[j][u] = (norm.ssq_parts && row < M && pidx < norm.nparts) ? norm.ssq_parts[(size_t)pidx * M + row] : 0.f;
        }
#pragma unroll
    for (int j = 0; j < MT; ++j) {
        float ss = 0.f;
#pragma unroll
        for (int u = 0; u < PMAX; ++u) ss += pv[j][u];
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) ss += __shfl_xor(ss, o, 64);
        if (lane == 0) rinv[wave * MT + j] = norm.ssq_parts ? 1.0f / sqrtf(ss * norm.inv_d + norm.eps) : 1.0f;
    }
    if (kh == 1) {
#pragma unroll
        for (int v = 0; v < 2; ++v)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) red[((rt * 2 + v) * MT + mt) * 64 + lane] = acc[v][mt];
    }
    __syncthreads();
    if (kh == 1) return;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        floatx4 v = acc[0][mt];
        const floatx4 p1 = acc[1][mt], p2 = red[((rt * 2 + 0) * MT + mt) * 64 + lane], p3 = red[((rt * 2 + 1) * MT + mt) * 64 + lane];
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = ((v[e] + p1[e]) + p2[e]) + p3[e];
        // v[e]: activation row m = mt*16 + r, MFMA row 4c + e: c < 2 gate of column 4c + e, c >= 2 up of column 4(c-2) + e
        const int m = mt * 16 + r;
        const float rs = rinv[m];
        bf16x4 out;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float up = __shfl_xor(v[e], 32, 64) * rs;
            const float gt = v[e] * rs;
            out[e] = (bf16)(gt / (1.0f + __expf(-gt)) * up);
        }
        const int cc = j0 + rt * 8 + 4 * c;
        if (c < 2 && m < M && cc < F) *reinterpret_cast<bf16x4*>(act + (size_t)m * F + cc) = out;
    }
}

bool stream_mt_supported(int M, int N, int K) { return M > 16 && M <= 64 && N % 16 == 0 && K >= 512 && K % 512 == 0; }

template <int MT>
static int launch_tile_cfg(compact_ctx* ctx, const bf16* X, const bf16* W, const bf16* resid, const bf16* g, float* h_out,
                           bf16* out16, float* ssq_parts, int M, int N, int K, hipStream_t s) {
    // two activation slices, reused for the MT x 16 KB of partial tiles at the end
    const size_t smem = std::max((size_t)2 * MT * 16 * (512 + 8) * sizeof(bf16), (size_t)MT * MTS_WAVES * 64 * sizeof(floatx4));
    static bool attr = false;
    if (!attr) {
        HIP_TRY(ctx, hipFuncSetAttribute(reinterpret_cast<const void*>(stream_tile_mt_kernel<MT>),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
        attr = true;
    }
    stream_tile_mt_kernel<MT><<<N / 16, MTS_WAVES * 64, smem, s>>>(X, W, resid, g, h_out, out16, ssq_parts, M, N, K);
    LAUNCH_CHECK(ctx);
    return COMPACT_OK;
}

int launch_resid_norm_stream_mt(compact_ctx* ctx, const bf16* X, const bf16* W, const bf16* resid, const bf16* g, float* h_out,
                                bf16* hg_out, float* ssq_parts, int M, int N, int K, hipStream_t s) {
    if (!stream_mt_supported(M, N, K)) return set_err(ctx, COMPACT_ESHAPE, "whole-K streaming kernel for 17..64 rows does not cover this shape");
    switch ((M + 15) / 16) {
        case 2: return launch_tile_cfg<2>(ctx, X, W, resid, g, h_out, hg_out, ssq_parts, M, N, K, s);
        case 3: return launch_tile_cfg<3>(ctx, X, W, resid, g, h_out, hg_out, ssq_parts, M, N, K, s);
        default: return launch_tile_cfg<4>(ctx, X, W, resid, g, h_out, hg_out, ssq_parts, M, N, K, s);
    }
}

// (the row norms come as at most 512 column-group sums per row: d_model <= 8192)
bool swiglu_mt_supported(int M, int F, int K) { return M > 16 && M <= 64 && F % 16 == 0 && K >= 256 && K % 256 == 0 && K <= 8192; }

template <int MT>
static int launch_swiglu_cfg_mt(compact_ctx* ctx, const bf16* X, const bf16* W, bf16* act, int M, int F, int K, const RowNorm& rn,
                                hipStream_t s) {
    const size_t smem = std::max((size_t)2 * MT * 16 * (256 + 8) * sizeof(bf16), (size_t)8 * 2 * MT * 64 * sizeof(floatx4));
    static bool attr = false;
    if (!attr) {
        HIP_TRY(ctx, hipFuncSetAttribute(reinterpret_cast<const void*>(swiglu_mt_kernel<MT>),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
        attr = true;
    }
    swiglu_mt_kernel<MT><<<(F + 63) / 64, MTS_WAVES * 64, smem, s>>>(X, W, act, M, F, K, rn);
    LAUNCH_CHECK(ctx);
    return COMPACT_OK;
}

int launch_swiglu_mt(compact_ctx* ctx, const bf16* X, const bf16* W, bf16* act, int M, int F, int K, const RowNorm* norm,
                     hipStream_t s) {
    if (!swiglu_mt_supported(M, F, K)) return set_err(ctx, COMPACT_ESHAPE, "fused gate/up kernel for 17..64 rows does not cover this shape");
    const RowNorm rn = norm ? *norm : RowNorm{};
    switch ((M + 15) / 16) {
        case 2: return launch_swiglu_cfg_mt<2>(ctx, X, W, act, M, F, K, rn, s);
        case 3: return launch_swiglu_cfg_mt<3>(ctx, X, W, act, M, F, K, rn, s);
        default: return launch_swiglu_cfg_mt<4>(ctx, X, W, act, M, F, K, rn, s);
    }
}
