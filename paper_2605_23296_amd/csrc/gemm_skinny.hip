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

template <int MT>
__global__ __launch_bounds__(256) void gemm_skinny_kernel(const bf16* __restrict__ X, const bf16* __restrict__ W,
                                                          float* __restrict__ P, int M, int N, int K) {
    constexpr int LDX = SKINNY_KSLICE + 8;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    bf16* xs = reinterpret_cast<bf16*>(smem);  // [MT*16][LDX]
    const int t = threadIdx.x;
    const int slice = blockIdx.y;
    const int k0 = slice * SKINNY_KSLICE;
    const int klen = min(SKINNY_KSLICE, K - k0);
    const int cpr = klen / 8;  // 16-byte chunks per row
    for (int q = t; q < MT * 16 * cpr; q += 256) {
        const int row = q / cpr, c = q - row * cpr;
        bf16x8 v;
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = (bf16)0.f;
        if (row < M) v = *reinterpret_cast<const bf16x8*>(X + (size_t)row * K + k0 + c * 8);
        *reinterpret_cast<bf16x8*>(xs + row * LDX + c * 8) = v;
    }
    __syncthreads();

    const int lane = t & 63, wave = t >> 6;
    const int n0 = (blockIdx.x * 4 + wave) * 16;
    if (n0 >= N) return;
    const int r = lane & 15, c = lane >> 4;
    const bf16* wp = W + (size_t)(n0 + r) * K + k0 + c * 8;
    const int nsteps = klen / 32;

    bf16x8 a[SKINNY_STEPS];
#pragma unroll
    for (int s = 0; s < SKINNY_STEPS; ++s)
        if (s < nsteps) a[s] = *reinterpret_cast<const bf16x8*>(wp + s * 32);

    floatx4 acc[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) acc[mt] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s = 0; s < SKINNY_STEPS; ++s) {
        if (s < nsteps) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                const bf16x8 b = *reinterpret_cast<const bf16x8*>(xs + (mt * 16 + r) * LDX + s * 32 + c * 8);
                acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[s], b, acc[mt], 0, 0, 0);
            }
        }
    }
    // acc[mt][e]: activation row m = mt*16 + r, weight row n = n0 + 4c + e
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const int m = mt * 16 + r;
        if (m < M) *reinterpret_cast<floatx4*>(P + ((size_t)slice * M + m) * N + n0 + 4 * c) = acc[mt];
    }
}

int launch_gemm_skinny(compact_ctx* ctx, const bf16* A, const bf16* B, float* partials, int M, int N, int K, int ks,
                       hipStream_t s) {
    if (M < 1 || M > 64) return set_err(ctx, COMPACT_ESHAPE, "weight-streaming GEMM takes 1..64 activation rows");
    if (N % 16 != 0 || K % 64 != 0) return set_err(ctx, COMPACT_ESHAPE, "weight-streaming GEMM needs N % 16 == 0 and K % 64 == 0");
    if (ks != skinny_ksplit(M, N, K)) return set_err(ctx, COMPACT_EINVAL, "unexpected K split");
    dim3 grid((N + 63) / 64, ks);
    const int mt = (M + 15) / 16;
    const size_t smem = (size_t)mt * 16 * (SKINNY_KSLICE + 8) * sizeof(bf16);
    switch (mt) {
        case 1: gemm_skinny_kernel<1><<<grid, 256, smem, s>>>(A, B, partials, M, N, K); break;
        case 2: gemm_skinny_kernel<2><<<grid, 256, smem, s>>>(A, B, partials, M, N, K); break;
        case 3: {
            static bool set3 = false;
            if (!set3) {
                HIP_TRY(ctx, hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_skinny_kernel<3>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
                set3 = true;
            }
            gemm_skinny_kernel<3><<<grid, 256, smem, s>>>(A, B, partials, M, N, K);
            break;
        }
        default: {
            static bool set4 = false;
            if (!set4) {
                HIP_TRY(ctx, hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_skinny_kernel<4>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
                set4 = true;
            }
            gemm_skinny_kernel<4><<<grid, 256, smem, s>>>(A, B, partials, M, N, K);
            break;
        }
    }
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
