// fp32 GEMM for the fp32 storage mode: C[M,N] = A[M,K] B[N,K]^T (+ R).
// LDS-tiled FMA kernel, 64x64 tile, 4x4 outputs per thread.  The fp32 mode is
// the tight-tolerance checking mode of the library, not a throughput mode, so
// this kernel favours plain sequential-in-K fp32 accumulation over speed.
#include "common.h"

#define TM 64
#define TN 64
#define TK 16

// EPI 0: C = acc (+R).  EPI 1: B is [2N, K] (gate rows then up rows); C = silu(A Bg^T) * (A Bu^T)
// With a GroupedArgs map, row tile blockIdx.y covers rows tile_row0 .. +tile_rows of
// the expert-sorted order, reads A rows through a_gather and uses expert
// tile_expert's slice of B.
template <int EPI>
__global__ __launch_bounds__(256) void gemm_f32_kernel(const float* __restrict__ A, const float* __restrict__ B,
                                                       const float* __restrict__ R, float* __restrict__ C, int64_t M,
                                                       int N, int K, const GroupedArgs g) {
    __shared__ float As[TK][TM + 4];
    __shared__ float Bs[EPI == 1 ? 2 : 1][TK][TN + 4];
    const int tx = threadIdx.x % 16, ty = threadIdx.x / 16;
    int64_t m0 = (int64_t)blockIdx.y * TM;
    if (g.tile_expert) {
        const int e = g.tile_expert[blockIdx.y];
        if (e < 0) return;
        m0 = g.tile_row0[blockIdx.y];
        M = m0 + g.tile_rows[blockIdx.y];
        B += (int64_t)e * g.b_expert_stride;
    }
    const int n0 = blockIdx.x * TN;
    float acc[4][4] = {};
    float acc2[4][4] = {};

    for (int k0 = 0; k0 < K; k0 += TK) {
        // 64 rows x 16 k per operand, 256 threads: 4 elements each
        for (int i = threadIdx.x; i < TM * TK; i += 256) {
            const int r = i / TK, kk = i % TK;
            const int64_t gm = m0 + r;
            float av = 0.f;
            if (gm < M && k0 + kk < K) av = A[(g.a_gather ? (int64_t)g.a_gather[gm] : gm) * K + k0 + kk];
            As[kk][r] = av;
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
            if (g.row_scale) v *= g.row_scale[gm];
            C[gm * N + gn] = v;
        }
    }
}

int gemm_f32_mtile() { return TM; }

int launch_gemm_f32(compact_ctx* ctx, const float* A, const float* B, const float* R, float* C, int64_t M, int N,
                    int K, int epilogue, const GroupedArgs* grouped, hipStream_t s) {
    if (M == 0) return COMPACT_OK;
    GroupedArgs g{};
    if (grouped) g = *grouped;
    dim3 grid((N + TN - 1) / TN, grouped ? (unsigned)grouped->n_mtiles : (unsigned)((M + TM - 1) / TM));
    if (epilogue == 1)
        gemm_f32_kernel<1><<<grid, 256, 0, s>>>(A, B, nullptr, C, M, N, K, g);
    else
        gemm_f32_kernel<0><<<grid, 256, 0, s>>>(A, B, R, C, M, N, K, g);
    LAUNCH_CHECK(ctx);
    return COMPACT_OK;
}
