// Split-KV decode attention (bf16 storage): one query token per block against
// that block's own KV cache.  HBM-bound: every cached K and V byte is read
// exactly once per step, with 16-byte loads that land directly in the MFMA
// operand layout (no LDS staging of K/V).
//
//  * grid = (chunk, kv head, block); a workgroup owns DECODE_CHUNK cached
//    tokens of one (block, kv head) and all query heads of that KV head's
//    group (the cache is read once for the whole group).  Chunks are fixed
//    size, so the split of a block depends on its own length only.
//  * per 32-token window a wavefront computes S^T = K Q^T with
//    v_mfma_f32_16x16x32_bf16 (K rows as MFMA rows, the group's query heads,
//    padded to 16, as MFMA columns) and O^T += V^T P^T with the V slab's
//    transposed layout [hd][token] supplying the MFMA rows.  The MFMA rows of
//    the two S^T tiles are assigned to tokens so that the accumulator layout
//    of S^T is exactly the operand layout of P^T: no shuffle, no LDS.
//  * softmax statistics are per lane-column; the max/sum across the four lane
//    groups uses wavefront shuffles.  The four wavefronts of a workgroup are
//    merged through LDS; chunks are merged by a second small kernel with a
//    log-sum-exp combine in fixed chunk order.
#include "common.h"

#define LOG2E 1.4426950408889634f

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

template <int HD>
__global__ __launch_bounds__(256) void attn_decode_bf16_kernel(const BlockMeta* __restrict__ meta, int step, int max_chunks,
                                                               const bf16* __restrict__ q, const bf16* __restrict__ kbase,
                                                               const bf16* __restrict__ vbase, float* __restrict__ partials,
                                                               int Hq, int Hkv, float scale_log2) {
    constexpr int KS = HD / 32;  // k-steps of the QK product
    constexpr int DT = HD / 16;  // 16-row tiles of O^T
    constexpr int PLD = HD + 2;  // partial record: HD values, max, sum
    __shared__ float so[4][16][PLD];

    const int b = blockIdx.z, kvh = blockIdx.y, ch = blockIdx.x;
    const BlockMeta bm = meta[b];
    const int n_keys = bm.len + step + 1;
    const int c0 = ch * DECODE_CHUNK;
    if (c0 >= n_keys) return;
    const int G = Hq / Hkv;
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int r = lane & 15, c = lane >> 4;

    const bf16* kslab = kbase + bm.slab + (size_t)kvh * bm.capacity * HD;
    const bf16* vslab = vbase + bm.slab + (size_t)kvh * HD * bm.capacity;

    // query operand: lane (g = r, c) holds q[g][s*32 + c*8 .. +7]
    bf16x8 qf[KS];
#pragma unroll
    for (int s = 0; s < KS; ++s) {
#pragma unroll
        for (int j = 0; j < 8; ++j) qf[s][j] = (bf16)0.f;
        if (r < G) qf[s] = *reinterpret_cast<const bf16x8*>(q + ((size_t)b * Hq + kvh * G + r) * HD + s * 32 + c * 8);
    }

    floatx4 oacc[DT];
#pragma unroll
    for (int d = 0; d < DT; ++d) oacc[d] = floatx4{0.f, 0.f, 0.f, 0.f};
    float m_run = -INFINITY, l_run = 0.f;

    const int w0 = c0 + wave * (DECODE_CHUNK / 4);
    constexpr int NWIN = DECODE_CHUNK / 4 / 32;
    // ---- all loads of the wavefront's windows are issued before any arithmetic ----
    // S^T tile tt, MFMA row m  <->  token t0 + 8*(m/4) + 4*tt + (m%4)
    // V^T tile d: lane (row dd = d*16 + r, c) holds tokens t0 + 8c .. +7
    bf16x8 kf[NWIN][2][KS];
    bf16x8 vf[NWIN][DT];
#pragma unroll
    for (int win = 0; win < NWIN; ++win) {
        const int t0 = w0 + win * 32;
        if (t0 < n_keys) {
#pragma unroll
            for (int tt = 0; tt < 2; ++tt) {
                const int tok = min(t0 + 8 * (r >> 2) + 4 * tt + (r & 3), n_keys - 1);
                const bf16* kp = kslab + (size_t)tok * HD + c * 8;
#pragma unroll
                for (int s = 0; s < KS; ++s) kf[win][tt][s] = *reinterpret_cast<const bf16x8*>(kp + s * 32);
            }
            const int voff = min(t0 + 8 * c, bm.capacity - 8);
#pragma unroll
            for (int d = 0; d < DT; ++d)
                vf[win][d] = *reinterpret_cast<const bf16x8*>(vslab + (size_t)(d * 16 + r) * bm.capacity + voff);
        }
    }
#pragma unroll
    for (int win = 0; win < NWIN; ++win) {
        const int t0 = w0 + win * 32;
        if (t0 < n_keys) {
            if (t0 + 32 > n_keys) {  // ragged tail: rows past the cache end must not reach the MFMA
#pragma unroll
                for (int d = 0; d < DT; ++d)
#pragma unroll
                    for (int j = 0; j < 8; ++j)
                        if (t0 + 8 * c + j >= n_keys) vf[win][d][j] = (bf16)0.f;
            }
            // ---- S^T = K Q^T --------------------------------------------------
            floatx4 sacc[2];
#pragma unroll
            for (int tt = 0; tt < 2; ++tt) {
                sacc[tt] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int s = 0; s < KS; ++s)
                    sacc[tt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[win][tt][s], qf[s], sacc[tt], 0, 0, 0);
            }
            // sacc[tt][e]: column g = r, token t0 + 8c + 4tt + e
            float sv[8];
            float mx = -INFINITY;
#pragma unroll
            for (int tt = 0; tt < 2; ++tt)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int tok = t0 + 8 * c + 4 * tt + e;
                    const float sc = tok < n_keys ? sacc[tt][e] * scale_log2 : -INFINITY;
                    sv[tt * 4 + e] = sc;
                    mx = fmaxf(mx, sc);
                }
            mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
            mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
            const float m_new = fmaxf(m_run, mx);  // finite: the window holds at least one valid token
            const float corr = fast_exp2(m_run - m_new);
            bf16x8 pf;
            float ps = 0.f;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const float p = fast_exp2(sv[j] - m_new);
                ps += p;
                pf[j] = (bf16)p;
            }
            l_run = l_run * corr + ps;
            m_run = m_new;
            // ---- O^T = O^T * corr + V^T P^T -------------------------------------
#pragma unroll
            for (int d = 0; d < DT; ++d) {
#pragma unroll
                for (int e = 0; e < 4; ++e) oacc[d][e] *= corr;
                oacc[d] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf[win][d], pf, oacc[d], 0, 0, 0);
            }
        }
    }
    // sum of p over the four lane groups of the column
    l_run += __shfl_xor(l_run, 16, 64);
    l_run += __shfl_xor(l_run, 32, 64);

    // ---- merge the four wavefronts ----------------------------------------------
    // oacc[d][e]: column g = r, output element dd = d*16 + 4c + e
    if (r < G) {
#pragma unroll
        for (int d = 0; d < DT; ++d)
#pragma unroll
            for (int e = 0; e < 4; ++e) so[wave][r][d * 16 + 4 * c + e] = oacc[d][e];
        if (c == 0) {
            so[wave][r][HD] = m_run;
            so[wave][r][HD + 1] = l_run;
        }
    }
    __syncthreads();
    for (int idx = t; idx < G * HD; idx += 256) {
        const int g = idx / HD, dd = idx - g * HD;
        float mm = -INFINITY;
#pragma unroll
        for (int w = 0; w < 4; ++w) mm = fmaxf(mm, so[w][g][HD]);
        float o = 0.f, l = 0.f;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const float lw = so[w][g][HD + 1];
            const float f = lw > 0.f ? fast_exp2(so[w][g][HD] - mm) : 0.f;
            o += f * so[w][g][dd];
            l += f * lw;
        }
        float* rec = partials + (((size_t)b * Hq + kvh * G + g) * max_chunks + ch) * PLD;
        rec[dd] = o;
        if (dd == 0) {
            rec[HD] = mm;
            rec[HD + 1] = l;
        }
    }
}

// merges the chunks of one (block, head) in chunk order and normalises
template <int HD>
__global__ __launch_bounds__(HD) void attn_decode_combine_kernel(const BlockMeta* __restrict__ meta, int step, int max_chunks,
                                                                 const float* __restrict__ partials, bf16* __restrict__ o,
                                                                 int Hq) {
    constexpr int PLD = HD + 2;
    const int b = blockIdx.y, head = blockIdx.x, dd = threadIdx.x;
    const int n_keys = meta[b].len + step + 1;
    const int nch = (n_keys + DECODE_CHUNK - 1) / DECODE_CHUNK;
    const float* rec = partials + ((size_t)b * Hq + head) * max_chunks * PLD;
    float mm = -INFINITY;
    for (int ch = 0; ch < nch; ++ch) mm = fmaxf(mm, rec[ch * PLD + HD]);
    float acc = 0.f, l = 0.f;
    for (int ch = 0; ch < nch; ++ch) {
        const float f = fast_exp2(rec[ch * PLD + HD] - mm);
        acc += f * rec[ch * PLD + dd];
        l += f * rec[ch * PLD + HD + 1];
    }
    o[((size_t)b * Hq + head) * HD + dd] = (bf16)(acc / l);
}

size_t attn_decode_partial_floats(const compact_layer_cfg& cfg, int n_blocks, int max_chunks) {
    return (size_t)n_blocks * cfg.n_q_heads * max_chunks * (cfg.head_dim + 2);
}

int launch_attn_decode_bf16(compact_ctx* ctx, const BlockMeta* d_meta, int n_blocks, int step, int max_chunks,
                            const bf16* q, const bf16* d_k, const bf16* d_v, float* partials, bf16* o, hipStream_t s) {
    const compact_layer_cfg& c = ctx->cfg;
    const float scale_log2 = LOG2E / sqrtf((float)c.head_dim);
    dim3 grid(max_chunks, c.n_kv_heads, n_blocks);
    dim3 cgrid(c.n_q_heads, n_blocks);
    if (c.head_dim == 128) {
        {
            ProfileScope ps(ctx, COMPACT_K_ATTN_DECODE, s);
            attn_decode_bf16_kernel<128><<<grid, 256, 0, s>>>(d_meta, step, max_chunks, q, d_k, d_v, partials, c.n_q_heads,
                                                             c.n_kv_heads, scale_log2);
        }
        LAUNCH_CHECK(ctx);
        attn_decode_combine_kernel<128><<<cgrid, 128, 0, s>>>(d_meta, step, max_chunks, partials, o, c.n_q_heads);
    } else {
        {
            ProfileScope ps(ctx, COMPACT_K_ATTN_DECODE, s);
            attn_decode_bf16_kernel<64><<<grid, 256, 0, s>>>(d_meta, step, max_chunks, q, d_k, d_v, partials, c.n_q_heads,
                                                            c.n_kv_heads, scale_log2);
        }
        LAUNCH_CHECK(ctx);
        attn_decode_combine_kernel<64><<<cgrid, 64, 0, s>>>(d_meta, step, max_chunks, partials, o, c.n_q_heads);
    }
    LAUNCH_CHECK(ctx);
    return COMPACT_OK;
}
