// Block-scaled 4-bit expert weights (the format the paper's largest model is
// served in, Sec. IV-B "mxfp4 weights"; OCP Microscaling Formats v1.0): FP4
// E2M1 elements, two per byte (even index in the low nibble), one E8M0 scale
// 2^(e-127) per block of 32 consecutive elements along the contraction index.
//
// Routed decode rows are bound by the bytes of the expert weights they stream,
// so reading 4.25 bits per weight instead of 16 is worth 3.76x.  Every product
// of an element and a scale is exact in bf16, so the weights are expanded in
// registers and fed to the same bf16 MFMA as the 16-bit path:
//
//  * a lane loads 16 bytes = one whole block of 32 elements of one weight row
//    plus its scale byte; the four lane groups of an MFMA row take four
//    consecutive blocks, so a wave-instruction still reads 64 contiguous bytes
//    of each of 16 rows;
//  * expansion is the hardware's scaled conversion (v_cvt_scalef32_pk_bf16_fp4:
//    one byte = two elements -> two bf16, times a float scale), so a block of
//    32 costs 16 conversions and the elements come out in their natural order.
#include "common.h"

#define MX_BLOCK 32
#define MX_KSLICE 1024                       // k per workgroup: 8 blocks per lane in flight
#define MX_GROUPS (MX_KSLICE / (4 * MX_BLOCK))

int mxfp4_ksplit(int K) { return (K + MX_KSLICE - 1) / MX_KSLICE; }

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));

// 2^(e-127) as a float (e in 1..254)
__device__ __forceinline__ float e8m0_to_float(uint32_t scale_byte) { return __uint_as_float(scale_byte << 23); }

// Eight codes (one dword, element i in nibble i) -> eight bf16, each times `scale`.
__device__ __forceinline__ bf16x8 fp4_expand8(uint32_t w, float scale) {
    union {
        bf16x2_t p[4];
        bf16x8 v;
    } out;
#if defined(__HIP_DEVICE_COMPILE__)
    out.p[0] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(w, scale, 0);
    out.p[1] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(w, scale, 1);
    out.p[2] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(w, scale, 2);
    out.p[3] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(w, scale, 3);
#else
    (void)w;
    (void)scale;
#endif
    return out.v;
}

// ---------------------------------------------------------------------------
// Expansion to bf16 [rows, K] (the 16-bit copy the prefill GEMMs read).
// One thread per block of 32 elements.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void mxfp4_dequant_kernel(const uint8_t* __restrict__ codes, const uint8_t* __restrict__ scales,
                                                            bf16* __restrict__ out, int64_t n_blocks) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n_blocks) return;
    const uint4 cw = *reinterpret_cast<const uint4*>(codes + i * 16);
    const float sc = e8m0_to_float(scales[i]);
    const uint32_t w[4] = {cw.x, cw.y, cw.z, cw.w};
#pragma unroll
    for (int d = 0; d < 4; ++d) *reinterpret_cast<bf16x8*>(out + i * MX_BLOCK + d * 8) = fp4_expand8(w[d], sc);
}

int launch_mxfp4_dequant(compact_ctx* ctx, const uint8_t* codes, const uint8_t* scales, bf16* out, int64_t rows, int K,
                         hipStream_t s) {
    if (rows < 0 || K < MX_BLOCK || K % MX_BLOCK != 0) return set_err(ctx, COMPACT_ESHAPE, "4-bit weights need K % 32 == 0");
    const int64_t nb = rows * (K / MX_BLOCK);
    if (nb == 0) return COMPACT_OK;
    mxfp4_dequant_kernel<<<(unsigned)((nb + 255) / 256), 256, 0, s>>>(codes, scales, out, nb);
    LAUNCH_CHECK(ctx);
    return COMPACT_OK;
}

// ---------------------------------------------------------------------------
// Per-expert weight streaming for routed decode rows, 4-bit weights:
// partials[slice][sorted row][N] = X[rows of expert e, kslice] W_e[N, kslice]^T.
// grid (k-slices, N / 64, experts); 4 wavefronts of 16 weight rows each.
// ---------------------------------------------------------------------------
struct MxGroup {
    const int32_t* expert_list;  // [gridDim.z] experts to run, -1 = none (null: expert = blockIdx.z)
    const int32_t* tile_row0;    // [gridDim.z] first sorted row of the grid slice's tile (null: the expert's first row)
    const int32_t* tile_rows;    // [gridDim.z] its rows, at most 16 (null: all of the expert's rows)
    const int32_t* offsets;    // [E + 1] rows of every expert in the expert-sorted order
    const int32_t* a_gather;   // [total_rows] source row of X, or null (X already sorted)
    int64_t q_expert_stride;   // bytes between consecutive experts' codes
    int64_t s_expert_stride;   // bytes between consecutive experts' scales
    int total_rows;
};

__global__ __launch_bounds__(256) void gemm_skinny_mxfp4_kernel(const bf16* __restrict__ X, const uint8_t* __restrict__ Wq,
                                                                const uint8_t* __restrict__ Ws, float* __restrict__ P, int N,
                                                                int K, const MxGroup grp) {
    constexpr int LDX = MX_KSLICE + 8;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    bf16* xs = reinterpret_cast<bf16*>(smem);  // [16][LDX]
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int r = lane & 15, c = lane >> 4;
    const int e = grp.expert_list ? grp.expert_list[blockIdx.z] : (int)blockIdx.z;
    if (e < 0) return;
    const int row_base = grp.tile_row0 ? grp.tile_row0[blockIdx.z] : grp.offsets[e];
    const int M = min(grp.tile_rows ? grp.tile_rows[blockIdx.z] : grp.offsets[e + 1] - row_base, 16);
    if (M <= 0) return;   // nobody was routed to this expert
    Wq += (size_t)e * grp.q_expert_stride;
    Ws += (size_t)e * grp.s_expert_stride;
    const int slice = blockIdx.x;
    const int k0 = slice * MX_KSLICE;
    const int klen = min(MX_KSLICE, K - k0);
    const int nblk = klen / MX_BLOCK;            // blocks of this slice
    const int ngrp = (nblk + 3) / 4;             // MFMA groups of four blocks (the last may be partial)
    const int n0 = (blockIdx.y * 4 + wave) * 16;
    const bool active = n0 < N;

    // the weight stream goes first: everything below overlaps with it
    uint4 cw[MX_GROUPS];
    uint32_t sc[MX_GROUPS];
    if (active) {
        const uint8_t* wp = Wq + (size_t)(n0 + r) * (K / 2) + k0 / 2;
        const uint8_t* sp = Ws + (size_t)(n0 + r) * (K / MX_BLOCK) + k0 / MX_BLOCK;
#pragma unroll
        for (int g = 0; g < MX_GROUPS; ++g) {
            const int blk = 4 * g + c;
            cw[g] = make_uint4(0u, 0u, 0u, 0u);   // a block past the row's end contributes nothing
            sc[g] = 127u;
            if (blk < nblk) {
                cw[g] = *reinterpret_cast<const uint4*>(wp + (size_t)blk * 16);
                sc[g] = sp[blk];
            }
        }
    }

    // activations of this expert's rows, zero rows up to 16 and zero columns up to the last group's end
    const int cpr = ngrp * 16;   // 16-byte chunks per staged row
    for (int q = t; q < 16 * cpr; q += 256) {
        const int row = q / cpr, cc = q - row * cpr;
        bf16x8 v;
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = (bf16)0.f;
        if (row < M && cc * 8 < klen) {
            size_t src = row_base + row;
            if (grp.a_gather) src = grp.a_gather[src];
            v = *reinterpret_cast<const bf16x8*>(X + src * K + k0 + cc * 8);
        }
        *reinterpret_cast<bf16x8*>(xs + row * LDX + cc * 8) = v;
    }
    __syncthreads();
    if (!active) return;

    floatx4 acc = floatx4{0.f, 0.f, 0.f, 0.f};
    const bf16* xrow = xs + r * LDX + c * MX_BLOCK;
#pragma unroll
    for (int g = 0; g < MX_GROUPS; ++g) {
        if (g < ngrp) {
            const float scale = e8m0_to_float(sc[g]);
            const uint32_t w[4] = {cw[g].x, cw[g].y, cw[g].z, cw[g].w};
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                const bf16x8 a = fp4_expand8(w[d], scale);
                const bf16x8 b = *reinterpret_cast<const bf16x8*>(xrow + g * 4 * MX_BLOCK + d * 8);
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, acc, 0, 0, 0);
            }
        }
    }
    // acc[e]: activation row r, weight row n0 + 4c + e
    if (r < M) *reinterpret_cast<floatx4*>(P + ((size_t)slice * grp.total_rows + row_base + r) * N + n0 + 4 * c) = acc;
}

int launch_gemm_skinny_grouped_mxfp4(compact_ctx* ctx, const bf16* X, const int32_t* a_gather, const uint8_t* Wq,
                                     const uint8_t* Ws, const int32_t* offsets, int n_experts, int total_rows,
                                     float* partials, int N, int K, int ks, hipStream_t s, const int32_t* expert_list,
                                     int n_listed, const int32_t* tile_row0, const int32_t* tile_rows) {
    if (N % 16 != 0 || K % MX_BLOCK != 0) return set_err(ctx, COMPACT_ESHAPE, "4-bit weight streaming needs N % 16 == 0 and K % 32 == 0");
    if (ks != mxfp4_ksplit(K)) return set_err(ctx, COMPACT_EINVAL, "unexpected K split");
    MxGroup g{expert_list, tile_row0, tile_rows, offsets, a_gather, (int64_t)N * (K / 2), (int64_t)N * (K / MX_BLOCK), total_rows};
    dim3 grid(ks, (N + 63) / 64, expert_list ? n_listed : n_experts);
    const size_t smem = (size_t)16 * (MX_KSLICE + 8) * sizeof(bf16);
    gemm_skinny_mxfp4_kernel<<<grid, 256, smem, s>>>(X, Wq, Ws, partials, N, K, g);
    LAUNCH_CHECK(ctx);
    return COMPACT_OK;
}
