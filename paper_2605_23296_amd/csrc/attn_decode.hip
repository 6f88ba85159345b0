// Split-KV decode attention (bf16 storage): one query token per block against
// that block's own KV cache.  HBM-bound: every cached K and V byte is read
// exactly once per step, with 16-byte loads that land directly in the MFMA
// operand layout (no LDS staging of K/V).
//
//  * grid = (chunk item, kv head), the items being the (block, chunk) pairs
//    of the ragged batch listed by the host; a workgroup owns DECODE_CHUNK cached
//    tokens of one (block, kv head) and all query heads of that KV head's
//    group (the cache is read once for the whole group).  Chunks are fixed
//    size, so the split of a block depends on its own length only.
//  * scores: per 32-token window a wavefront computes S^T = K Q^T with
//    v_mfma_f32_16x16x32_bf16 (K rows as MFMA rows, the group's query heads,
//    padded to 16, as MFMA columns).  The MFMA rows of the two S^T tiles are
//    assigned to tokens so that a lane ends up with 8 consecutive tokens of
//    one column.  A workgroup is 8 wavefronts, one window each (many short
//    wavefronts keep the memory system busier than few long ones).
//  * the windows exchange their column maxima through LDS, so that all of them
//    exponentiate against the chunk's maximum; the probabilities P^T go to LDS
//    as bf16 ([column][token], 8 KB).
//  * output: wavefront w owns rows 16w .. 16w+15 of O^T = V^T P^T over ALL tokens
//    of the chunk: its V^T operand rows are 512-byte contiguous runs of the
//    transposed V slab [hd][token], and nothing has to be merged across
//    wavefronts.  Chunks are merged by a second small kernel with a log-sum-exp
//    combine in fixed chunk order.
#include "common.h"

#define LOG2E 1.4426950408889634f

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

#define DEC_WAVES (DECODE_CHUNK / 32)   // one 32-token window per wavefront

#define DEC_PLD (DECODE_CHUNK + 8)   // bf16 per column of the probability tile (padded against bank conflicts)

template <int HD>
__global__ __launch_bounds__(DEC_WAVES * 64, 4) void attn_decode_bf16_kernel(const BlockMeta* __restrict__ meta,
                                                                            const TileItem* __restrict__ chunks, int step,
                                                                            int max_chunks, const bf16* __restrict__ q,
                                                                            const bf16* __restrict__ kbase,
                                                                            const bf16* __restrict__ vbase,
                                                                            float* __restrict__ partials, int Hq, int Hkv,
                                                                            float scale_log2, const int32_t* __restrict__ qrow,
                                                                            int q_stride) {
    constexpr int KS = HD / 32;            // k-steps of the QK product
    constexpr int DT = HD / 16;            // 16-row tiles of O^T, one per wavefront (the first DT wavefronts)
    constexpr int PLD = HD + 2;            // partial record: HD values, max, sum
    constexpr int VS = DECODE_CHUNK / 32;  // k-steps of the PV product
    __shared__ __attribute__((aligned(16))) bf16 qs[16 * HD];        // [G][HD] query rows of the group
    __shared__ __attribute__((aligned(16))) bf16 ps[16 * DEC_PLD];   // P^T: [column][token of the chunk]
    __shared__ float s_max[DEC_WAVES][16], s_sum[DEC_WAVES][16];     // per-window maximum and sum of every column

    const TileItem it = chunks[blockIdx.x];
    const int b = it.block, kvh = blockIdx.y, c0 = it.row0, ch = c0 / DECODE_CHUNK;
    const BlockMeta bm = meta[b];
    const int n_keys = bm.len + step + 1;
    if (c0 >= n_keys) return;   // a chunk this step does not reach yet
    const int n_rows = min(n_keys - c0, DECODE_CHUNK);
    const int G = Hq / Hkv;
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int r = lane & 15, c = lane >> 4;
    const int w_lo = wave * 32;
    const int t0 = c0 + w_lo;
    const bool live = w_lo < n_rows;

    const bf16* kslab = kbase + bm.slab + (size_t)kvh * bm.capacity * HD;
    const bf16* vslab = vbase + bm.slab + (size_t)kvh * HD * bm.capacity;

    // ---- all loads are issued before any arithmetic ----------------------------
    // scores: S^T tile tt, MFMA row m  <->  token t0 + 8*(m/4) + 4*tt + (m%4)
    // output: lane (r, c) of k-step j holds V^T[16*wave + r][c0 + 32j + 8c .. +7]
    bf16x8 kf[2][KS];
    bf16x8 vf[VS];
    if (live) {
#pragma unroll
        for (int tt = 0; tt < 2; ++tt) {
            const int tok = min(t0 + 8 * (r >> 2) + 4 * tt + (r & 3), n_keys - 1);
            const bf16* kp = kslab + (size_t)tok * HD + c * 8;
#pragma unroll
            for (int s = 0; s < KS; ++s) kf[tt][s] = *reinterpret_cast<const bf16x8*>(kp + s * 32);
        }
    }
    if (wave < DT) {
        const bf16* vp = vslab + (size_t)(wave * 16 + r) * bm.capacity;
#pragma unroll
        for (int j = 0; j < VS; ++j) {
            // tokens past the cache end are never used: keep the load inside the slab row
            const int voff = min(c0 + 32 * j + 8 * c, bm.capacity - 8);
            vf[j] = *reinterpret_cast<const bf16x8*>(vp + voff);
        }
    }
    // the group's query rows go through LDS: they are needed only once the K rows
    // have arrived, and parking them in registers until then would cost occupancy
    for (int i = t; i < G * (HD / 8); i += DEC_WAVES * 64)
        *reinterpret_cast<bf16x8*>(qs + i * 8) =
            *reinterpret_cast<const bf16x8*>(q + (size_t)(qrow ? qrow[b] : b) * q_stride + (size_t)kvh * G * HD + i * 8);
    __syncthreads();

    // ---- S^T = K Q^T over the wavefront's window; the window's column maxima ------
    float sv[8];
    float mx = -INFINITY;
    if (live) {
        // query operand: lane (g = r, c) holds q[g][s*32 + c*8 .. +7], read k-step by k-step
        floatx4 sacc[2] = {floatx4{0.f, 0.f, 0.f, 0.f}, floatx4{0.f, 0.f, 0.f, 0.f}};
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            bf16x8 qf = *reinterpret_cast<const bf16x8*>(qs + (r < G ? r : 0) * HD + s * 32 + c * 8);
            if (r >= G) {
#pragma unroll
                for (int j = 0; j < 8; ++j) qf[j] = (bf16)0.f;
            }
            sacc[0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[0][s], qf, sacc[0], 0, 0, 0);
            sacc[1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[1][s], qf, sacc[1], 0, 0, 0);
        }
        // sacc[tt][e]: column g = r, token t0 + 8c + 4tt + e
#pragma unroll
        for (int tt = 0; tt < 2; ++tt)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int row = w_lo + 8 * c + 4 * tt + e;
                const float sc = row < n_rows ? sacc[tt][e] * scale_log2 : -INFINITY;
                sv[tt * 4 + e] = sc;
                mx = fmaxf(mx, sc);
            }
        mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    }
    if (c == 0) s_max[wave][r] = mx;
    if (wave < DT && n_rows < DECODE_CHUNK) {  // ragged tail: bits past the cache end must not reach the MFMA
#pragma unroll
        for (int j = 0; j < VS; ++j)
#pragma unroll
            for (int i = 0; i < 8; ++i)
                if (32 * j + 8 * c + i >= n_rows) vf[j][i] = (bf16)0.f;
    }
    __syncthreads();

    // ---- one maximum per column for the whole chunk: P = exp2(S - max) ------------
    float m_all = s_max[0][r];   // finite: the chunk holds at least one valid token
#pragma unroll
    for (int w = 1; w < DEC_WAVES; ++w) m_all = fmaxf(m_all, s_max[w][r]);
    bf16x8 pf;
    float l_run = 0.f;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const float p = live ? fast_exp2(sv[j] - m_all) : 0.f;
        l_run += p;
        pf[j] = (bf16)p;
    }
    l_run += __shfl_xor(l_run, 16, 64);
    l_run += __shfl_xor(l_run, 32, 64);
    if (c == 0) s_sum[wave][r] = l_run;
    *reinterpret_cast<bf16x8*>(ps + r * DEC_PLD + w_lo + 8 * c) = pf;
    __syncthreads();

    // ---- O^T rows 16*wave .. +15 = V^T P^T over all tokens of the chunk --------------
    if (wave < DT) {
        floatx4 oacc = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int j = 0; j < VS; ++j) {
            const bf16x8 pb = *reinterpret_cast<const bf16x8*>(ps + r * DEC_PLD + 32 * j + 8 * c);
            oacc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf[j], pb, oacc, 0, 0, 0);
        }
        // oacc[e]: column g = r, output element 16*wave + 4c + e
        if (r < G) {
            float* out = partials + (((size_t)b * Hq + kvh * G + r) * max_chunks + ch) * PLD;
            *reinterpret_cast<float2*>(out + wave * 16 + 4 * c) = float2{oacc[0], oacc[1]};
            *reinterpret_cast<float2*>(out + wave * 16 + 4 * c + 2) = float2{oacc[2], oacc[3]};
            if (wave == 0 && c == 0) {
                float l = s_sum[0][r];
#pragma unroll
                for (int w = 1; w < DEC_WAVES; ++w) l += s_sum[w][r];
                out[HD] = m_all;
                out[HD + 1] = l;
            }
        }
    }
}

// merges the chunks of one (block, head) in chunk order and normalises.
// The chunk weights exp2(m_ch - M) / L are formed once in LDS; every thread
// then owns one output element and reads its chunk values 8 loads at a time.
#define COMBINE_MAX_CHUNKS 1024
template <int HD>
__global__ __launch_bounds__(HD) void attn_decode_combine_kernel(const BlockMeta* __restrict__ meta, int step, int max_chunks,
                                                                 const float* __restrict__ partials, bf16* __restrict__ o,
                                                                 int Hq, const int32_t* __restrict__ qrow) {
    constexpr int PLD = HD + 2;
    __shared__ float wgt[COMBINE_MAX_CHUNKS];
    __shared__ float red_m[HD / 64], red_l[HD / 64];
    const int b = blockIdx.y, head = blockIdx.x, dd = threadIdx.x;
    const int n_keys = meta[b].len + step + 1;
    const int nch = (n_keys + DECODE_CHUNK - 1) / DECODE_CHUNK;
    const float* rec = partials + ((size_t)b * Hq + head) * max_chunks * PLD;
    // global max of the chunk maxima
    float mm = -INFINITY;
    for (int ch = dd; ch < nch; ch += HD) mm = fmaxf(mm, rec[ch * PLD + HD]);
#pragma unroll
    for (int ofs = 32; ofs > 0; ofs >>= 1) mm = fmaxf(mm, __shfl_xor(mm, ofs, 64));
    if ((dd & 63) == 0) red_m[dd >> 6] = mm;
    __syncthreads();
    mm = red_m[0];
#pragma unroll
    for (int i = 1; i < HD / 64; ++i) mm = fmaxf(mm, red_m[i]);
    // chunk weights; the normaliser is summed in chunk order by thread 0 afterwards
    for (int ch = dd; ch < nch; ch += HD) wgt[ch] = fast_exp2(rec[ch * PLD + HD] - mm);
    __syncthreads();
    if (dd == 0) {
        float l = 0.f;
        for (int ch = 0; ch < nch; ++ch) l += wgt[ch] * rec[ch * PLD + HD + 1];
        red_l[0] = l;
    }
    float acc = 0.f;
    int ch = 0;
    for (; ch + 8 <= nch; ch += 8) {
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = rec[(ch + u) * PLD + dd];
#pragma unroll
        for (int u = 0; u < 8; ++u) acc += wgt[ch + u] * v[u];
    }
    for (; ch < nch; ++ch) acc += wgt[ch] * rec[ch * PLD + dd];
    __syncthreads();
    o[((size_t)(qrow ? qrow[b] : b) * Hq + head) * HD + dd] = (bf16)(acc / red_l[0]);
}

size_t attn_decode_partial_floats(const compact_layer_cfg& cfg, int n_blocks, int max_chunks) {
    return (size_t)n_blocks * cfg.n_q_heads * max_chunks * (cfg.head_dim + 2);
}

int launch_attn_decode_bf16(compact_ctx* ctx, const BlockMeta* d_meta, const TileItem* d_chunks, int n_chunks, int n_blocks,
                            int step, int max_chunks, const bf16* q, const bf16* d_k, const bf16* d_v, float* partials, bf16* o,
                            hipStream_t s, const int32_t* d_qrow, int q_stride) {
    const compact_layer_cfg& c = ctx->cfg;
    const float scale_log2 = LOG2E / sqrtf((float)c.head_dim);
    if (n_chunks == 0) return COMPACT_OK;
    if (!d_qrow) q_stride = c.n_q_heads * c.head_dim;   // q [n_blocks, Hq * hd], row b for block b
    dim3 grid(n_chunks, c.n_kv_heads);
    dim3 cgrid(c.n_q_heads, n_blocks);
    if (max_chunks > COMBINE_MAX_CHUNKS) return set_err(ctx, COMPACT_ECAPACITY, "KV cache longer than the decode combine supports");
    if (c.head_dim == 128) {
        {
            ProfileScope ps(ctx, COMPACT_K_ATTN_DECODE, s);
            attn_decode_bf16_kernel<128><<<grid, DEC_WAVES * 64, 0, s>>>(d_meta, d_chunks, step, max_chunks, q, d_k, d_v, partials,
                                                                           c.n_q_heads, c.n_kv_heads, scale_log2, d_qrow, q_stride);
        }
        LAUNCH_CHECK(ctx);
        attn_decode_combine_kernel<128><<<cgrid, 128, 0, s>>>(d_meta, step, max_chunks, partials, o, c.n_q_heads, d_qrow);
    } else {
        {
            ProfileScope ps(ctx, COMPACT_K_ATTN_DECODE, s);
            attn_decode_bf16_kernel<64><<<grid, DEC_WAVES * 64, 0, s>>>(d_meta, d_chunks, step, max_chunks, q, d_k, d_v, partials,
                                                                          c.n_q_heads, c.n_kv_heads, scale_log2, d_qrow, q_stride);
        }
        LAUNCH_CHECK(ctx);
        attn_decode_combine_kernel<64><<<cgrid, 64, 0, s>>>(d_meta, step, max_chunks, partials, o, c.n_q_heads, d_qrow);
    }
    LAUNCH_CHECK(ctx);
    return COMPACT_OK;
}
