// Whole-K weight-streaming projection of the decode step (bf16 storage, at most
// 16 activation rows): a workgroup of 16 wavefronts owns 16 complete output
// columns, so the sum over K is finished inside the kernel and the step that
// follows the projection (residual add + the pieces of the next RMSNorm) is
// applied before anything is written.  No split-K partials, no second launch.
//
//  * a 16 x 16 MFMA tile = 16 weight rows; the 16 wavefronts of the workgroup
//    interleave over K in 64-byte pieces (wavefront kw takes k-steps kw, kw + 16,
//    ...), so that together they read whole contiguous runs of every weight row;
//  * every weight load goes straight from global memory into the MFMA operand
//    layout, all S = K / 512 loads of a wavefront issued before any arithmetic;
//  * each wavefront loads the activation fragments of its own k-steps straight
//    from global memory (L2): no LDS staging, no barrier before the MFMAs;
//  * the 16 partial tiles are added in wavefront order through LDS (one barrier),
//    so the result does not depend on timing or on the batch a row is decoded in.
#include "common.h"

#define GS_WAVES 16

__device__ __forceinline__ float gs_wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// ---------------------------------------------------------------------------
// Projection with the residual add and the front half of the next RMSNorm:
// h[M, N] = resid + X W^T (fp32, kept as the residual stream), hg = bf16(h * g),
// and ssq_parts[tile][m] = sum over the tile's 16 columns of h^2.  One tile per
// workgroup; the consumer turns the parts into 1 / rms.
// ---------------------------------------------------------------------------
template <int S>
__global__ __launch_bounds__(GS_WAVES * 64) void resid_norm_stream_kernel(const bf16* __restrict__ X, const bf16* __restrict__ W,
                                                                           const bf16* __restrict__ resid,
                                                                           const bf16* __restrict__ g, float* __restrict__ h_out,
                                                                           bf16* __restrict__ hg_out, float* __restrict__ ssq_parts,
                                                                           int M, int N) {
    constexpr int K = S * GS_WAVES * 32;
    __shared__ floatx4 red[GS_WAVES * 64];
    const int t = threadIdx.x, lane = t & 63, kw = t >> 6;
    const int r = lane & 15, c = lane >> 4;
    const int tile = blockIdx.x;
    const bf16* w0 = W + (size_t)(tile * 16 + r) * K + kw * 32 + c * 8;
    bf16x8 wf[S], xf[S];
#pragma unroll
    for (int s = 0; s < S; ++s) wf[s] = *reinterpret_cast<const bf16x8*>(w0 + (size_t)s * GS_WAVES * 32);
#pragma unroll
    for (int s = 0; s < S; ++s) {
#pragma unroll
        for (int j = 0; j < 8; ++j) xf[s][j] = (bf16)0.f;
        if (r < M) xf[s] = *reinterpret_cast<const bf16x8*>(X + (size_t)r * K + kw * 32 + c * 8 + (size_t)s * GS_WAVES * 32);
    }
    floatx4 acc = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s = 0; s < S; ++s) acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[s], xf[s], acc, 0, 0, 0);
    red[kw * 64 + lane] = acc;
    __syncthreads();
    if (kw != 0) return;
    floatx4 v = red[lane];
#pragma unroll
    for (int w = 1; w < GS_WAVES; ++w) {
        const floatx4 o = red[w * 64 + lane];
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] += o[e];
    }
    // v[e]: activation row r, output column n = tile*16 + 4c + e
    float ss = 0.f;
    if (r < M) {
        const size_t o = (size_t)r * N + tile * 16 + 4 * c;
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
        *reinterpret_cast<bf16x4*>(hg_out + o) = hg;
    }
    ss += __shfl_xor(ss, 16, 64);
    ss += __shfl_xor(ss, 32, 64);
    if (c == 0 && r < M) ssq_parts[(size_t)tile * M + r] = ss;
}

bool resid_norm_stream_supported(int M, int N, int K) { return M >= 1 && M <= 16 && N % 16 == 0 && (K == 2048 || K == 4096); }

int launch_resid_norm_stream(compact_ctx* ctx, const bf16* X, const bf16* W, const bf16* resid, const bf16* g, float* h_out,
                             bf16* hg_out, float* ssq_parts, int M, int N, int K, hipStream_t s) {
    if (!resid_norm_stream_supported(M, N, K)) return set_err(ctx, COMPACT_ESHAPE, "residual/norm streaming kernel does not cover this shape");
    if (K == 2048)
        resid_norm_stream_kernel<4><<<N / 16, GS_WAVES * 64, 0, s>>>(X, W, resid, g, h_out, hg_out, ssq_parts, M, N);
    else
        resid_norm_stream_kernel<8><<<N / 16, GS_WAVES * 64, 0, s>>>(X, W, resid, g, h_out, hg_out, ssq_parts, M, N);
    LAUNCH_CHECK(ctx);
    return COMPACT_OK;
}

// ---------------------------------------------------------------------------
// Projection with the closing residual add: y[M, N] = bf16(resid_f32 + X W^T).
// One tile per workgroup, any K that is a multiple of 512: weight and
// activation fragments travel through a ring of GS_RING loads per wavefront.
// ---------------------------------------------------------------------------
#define GS_RING 14
__global__ __launch_bounds__(GS_WAVES * 64) void resid_out_stream_kernel(const bf16* __restrict__ X, const bf16* __restrict__ W,
                                                                          const float* __restrict__ resid, bf16* __restrict__ y,
                                                                          int M, int N, int K) {
    __shared__ floatx4 red[GS_WAVES * 64];
    const int t = threadIdx.x, lane = t & 63, kw = t >> 6;
    const int r = lane & 15, c = lane >> 4;
    const int tile = blockIdx.x;
    const int S = K / (GS_WAVES * 32);   // k-steps per wavefront
    const bf16* w0 = W + (size_t)(tile * 16 + r) * K + kw * 32 + c * 8;
    const bf16* x0 = X + (size_t)(r < M ? r : 0) * K + kw * 32 + c * 8;
    const bool xv = r < M;
    bf16x8 wf[GS_RING], xf[GS_RING];
#pragma unroll
    for (int i = 0; i < GS_RING; ++i) {
#pragma unroll
        for (int j = 0; j < 8; ++j) xf[i][j] = (bf16)0.f;
        if (i < S) {
            wf[i] = *reinterpret_cast<const bf16x8*>(w0 + (size_t)i * GS_WAVES * 32);
            if (xv) xf[i] = *reinterpret_cast<const bf16x8*>(x0 + (size_t)i * GS_WAVES * 32);
        }
    }
    floatx4 acc = floatx4{0.f, 0.f, 0.f, 0.f};
    for (int s0 = 0; s0 < S; s0 += GS_RING) {
#pragma unroll
        for (int i = 0; i < GS_RING; ++i) {
            const int s = s0 + i;
            if (s < S) {
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[i], xf[i], acc, 0, 0, 0);
                if (s + GS_RING < S) {
                    wf[i] = *reinterpret_cast<const bf16x8*>(w0 + (size_t)(s + GS_RING) * GS_WAVES * 32);
                    if (xv) xf[i] = *reinterpret_cast<const bf16x8*>(x0 + (size_t)(s + GS_RING) * GS_WAVES * 32);
                }
            }
        }
    }
    red[kw * 64 + lane] = acc;
    __syncthreads();
    if (kw != 0) return;
    floatx4 v = red[lane];
#pragma unroll
    for (int w = 1; w < GS_WAVES; ++w) {
        const floatx4 o = red[w * 64 + lane];
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] += o[e];
    }
    // v[e]: activation row r, output column n = tile*16 + 4c + e
    if (r < M) {
        const size_t o = (size_t)r * N + tile * 16 + 4 * c;
        const floatx4 h = *reinterpret_cast<const floatx4*>(resid + o);
        bf16x4 out;
#pragma unroll
        for (int e = 0; e < 4; ++e) out[e] = (bf16)(h[e] + v[e]);
        *reinterpret_cast<bf16x4*>(y + o) = out;
    }
}

bool resid_out_stream_supported(int M, int N, int K) { return M >= 1 && M <= 16 && N % 16 == 0 && K >= 512 && K % 512 == 0; }

int launch_resid_out_stream(compact_ctx* ctx, const bf16* X, const bf16* W, const float* resid, bf16* y, int M, int N, int K,
                            hipStream_t s) {
    if (!resid_out_stream_supported(M, N, K)) return set_err(ctx, COMPACT_ESHAPE, "residual streaming kernel does not cover this shape");
    resid_out_stream_kernel<<<N / 16, GS_WAVES * 64, 0, s>>>(X, W, resid, y, M, N, K);
    LAUNCH_CHECK(ctx);
    return COMPACT_OK;
}

// m[r][c] = bf16(hg[r][c] / rms_r), 1 / rms from the column sums of squares
__global__ __launch_bounds__(256) void rownorm_apply_kernel(const bf16* __restrict__ hg, const RowNorm norm, bf16* __restrict__ m,
                                                            int rows, int d) {
    __shared__ float s_rinv;
    const int row = blockIdx.x;
    if (threadIdx.x < 64) {
        float ss = 0.f;
        for (int p = threadIdx.x; p < norm.nparts; p += 64) ss += norm.ssq_parts[(size_t)p * rows + row];
        ss = gs_wave_sum(ss);
        if (threadIdx.x == 0) s_rinv = 1.0f / sqrtf(ss * norm.inv_d + norm.eps);
    }
    __syncthreads();
    const float rs = s_rinv;
    for (int c0 = threadIdx.x * 8; c0 < d; c0 += 256 * 8) {
        const bf16x8 v = *reinterpret_cast<const bf16x8*>(hg + (size_t)row * d + c0);
        bf16x8 o;
#pragma unroll
        for (int j = 0; j < 8; ++j) o[j] = (bf16)((float)v[j] * rs);
        *reinterpret_cast<bf16x8*>(m + (size_t)row * d + c0) = o;
    }
}

int launch_rownorm_apply(compact_ctx* ctx, const bf16* hg, const RowNorm& norm, bf16* m, int rows, int d, hipStream_t s) {
    rownorm_apply_kernel<<<rows, 256, 0, s>>>(hg, norm, m, rows, d);
    LAUNCH_CHECK(ctx);
    return COMPACT_OK;
}
