// fp32 GEMM for the fp32 storage mode: C[M,N] = A[M,K] B[N,K]^T (+ R).
// LDS-tiled FMA kernel, 64x64 tile, 4x4 outputs per thread.  The fp32 mode is
// the tight-tolerance checking mode of the library, not a throughput mode, so
// this kernel favours plain sequential-in-K fp32 accumulation over speed.
#include "common.h"

#define TM 64
#define TN 64
#define TK 16

// EPI 0: C = acc (+R).  EPI 1: B is [2N, K] (gate rows then up rows); C = silu(A Bg^T) * (A Bu^T)
template <int EPI>
__global__ __launch_bounds__(256) void gemm_f32_kernel(const float* __restrict__ A, const float* __restrict__ B,
                                                       const float* __restrict__ R, float* __restrict__ C, int64_t M,
                                                       int N, int K) {
    __shared__ float As[TK][TM + 4];
    __shared__ float Bs[EPI == 1 ? 2 : 1][TK][TN + 4];
    const int tx = threadIdx.x % 16, ty = threadIdx.x / 16;
    const int64_t m0 = (int64_t)blockIdx.y * TM;
    const int n0 = blockIdx.x * TN;
    float acc[4][4] = {};
    float acc2[4][4] = {};

    for (int k0 = 0; k0 < K; k0 += TK) {
        // 64 rows x 16 k per operand, 256 threads: 4 elements each
        for (int i = threadIdx.x; i < TM * TK; i += 256) {
            const int r = i / TK, kk = i % TK;
            const int64_t gm = m0 + r;
            As[kk][r] = (gm < M && k0 + kk < K) ? A[gm * K + k0 + kk] : 0.f;
            const int gn = n0 + r;
            const bool ok = gn < N && k0 + kk < K;
            Bs[0][kk][r] = ok ? B[(int64_t)gn * K + k0 + kk] : 0.f;
            if (EPI == 1) Bs[1][kk][r] = ok ? B[(int64_t)(N + gn) * K + k0 + kk] : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < TK; ++kk) {
            float a[4], b[4], b2[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = As[kk][ty * 4 + i];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                b[j] = Bs[0][kk][tx * 4 + j];
                if (EPI == 1) b2[j] = Bs[1][kk][tx * 4 + j];
            }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
                    if (EPI == 1) acc2[i][j] = fmaf(a[i], b2[j], acc2[i][j]);
                }
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int64_t gm = m0 + ty * 4 + i;
        if (gm >= M) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int gn = n0 + tx * 4 + j;
            if (gn >= N) continue;
            float v = acc[i][j];
            if (EPI == 1) {
                v = v / (1.0f + expf(-v)) * acc2[i][j];
            } else if (R != nullptr) {
                v += R[gm * N + gn];
            }
            C[gm * N + gn] = v;
        }
    }
}

int launch_gemm_f32(compact_ctx* ctx, const float* A, const float* B, const float* R, float* C, int64_t M, int N,
                    int K, int epilogue, hipStream_t s) {
    if (M == 0) return COMPACT_OK;
    dim3 grid((N + TN - 1) / TN, (unsigned)((M + TM - 1) / TM));
    if (epilogue == 1)
        gemm_f32_kernel<1><<<grid, 256, 0, s>>>(A, B, nullptr, C, M, N, K);
    else
        gemm_f32_kernel<0><<<grid, 256, 0, s>>>(A, B, R, C, M, N, K);
    LAUNCH_CHECK(ctx);
    return COMPACT_OK;
}
