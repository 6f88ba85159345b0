// Decode attention of the prefix-aware layout (paper Sec. IV, Dispatch: worker
// k's prompt is blocks 1..k, so every worker's cache prefix is a prefix of the
// one shared cache of the whole history): worker b attends rows
// 0 .. prefix_len[b]-1 of the SHARED slab plus its own private tail.
//
// Cascade over the shared rows: a work item is a 256-row chunk of the shared
// slab together with ALL workers whose prefix reaches into it (a suffix of the
// workers, prefixes being nested).  The chunk's K rows and V^T rows are loaded
// from HBM once, straight into MFMA operand layout, and then multiplied with
// the query heads of those workers 16 MFMA columns (workers x heads of the KV
// group) at a time: the bytes read per step are those of the history once,
// not once per worker.  A worker's private tail is a one-worker item of the
// same kernel.  Every item leaves one record (un-normalised output, max, sum)
// per (worker, head); a second kernel merges a worker's records.
#include "common.h"

#define LOG2E 1.4426950408889634f
#define PFX_WAVES (DECODE_CHUNK / 32)

__device__ __forceinline__ float pfx_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

template <int HD>
__global__ __launch_bounds__(PFX_WAVES * 64) void attn_decode_prefix_kernel(const BlockMeta* __restrict__ tail_meta,
                                                                           const BlockMeta shared, const PrefixItem* __restrict__ items,
                                                                           int step, const bf16* __restrict__ q,
                                                                           const bf16* __restrict__ kshared,
                                                                           const bf16* __restrict__ vshared,
                                                                           const bf16* __restrict__ ktail,
                                                                           const bf16* __restrict__ vtail,
                                                                           float* __restrict__ records, int64_t total_recs, int Hq,
                                                                           int Hkv, float scale_log2) {
    constexpr int KS = HD / 32;  // k-steps of the QK product
    constexpr int DT = HD / 16;  // 16-row tiles of O^T
    constexpr int PLD = HD + 2;  // record: HD values, max, sum
    extern __shared__ float so[];                                // [PFX_WAVES][16][PLD]
    __shared__ __attribute__((aligned(16))) bf16 qs[16 * HD];    // the 16 query rows of the current column group
    __shared__ int s_valid[16];                                  // rows of the item each column may see

    const PrefixItem it = items[blockIdx.x];
    const int kvh = blockIdx.y;
    const int G = Hq / Hkv;
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int r = lane & 15, c = lane >> 4;

    const bf16 *kslab, *vslab;
    int cap, n_rows;   // rows of the item that exist at all
    if (it.tail) {
        const BlockMeta bm = tail_meta[it.w0];
        n_rows = min(bm.len + step + 1 - it.row0, DECODE_CHUNK);
        if (n_rows <= 0) return;   // a tail chunk this step does not reach yet
        cap = bm.capacity;
        kslab = ktail + bm.slab + (size_t)kvh * cap * HD;
        vslab = vtail + bm.slab + (size_t)kvh * HD * cap;
    } else {
        n_rows = it.n_rows;
        cap = shared.capacity;
        kslab = kshared + shared.slab + (size_t)kvh * cap * HD;
        vslab = vshared + shared.slab + (size_t)kvh * HD * cap;
    }
    const int w_lo = wave * 32;                 // first item row of this wavefront's window
    const bool live = w_lo < n_rows;
    const int t0 = it.row0 + w_lo;              // slab row of the window
    const int last_row = it.row0 + n_rows - 1;

    // ---- the window's K rows and V^T rows: loaded once, used by every column group ----
    // S^T tile tt, MFMA row m  <->  row t0 + 8*(m/4) + 4*tt + (m%4);  V^T tile d: lane (row d*16 + r, c) holds rows t0 + 8c .. +7
    bf16x8 kf[2][KS];
    bf16x8 vf[DT];
    if (live) {
#pragma unroll
        for (int tt = 0; tt < 2; ++tt) {
            const int row = min(t0 + 8 * (r >> 2) + 4 * tt + (r & 3), last_row);
            const bf16* kp = kslab + (size_t)row * HD + c * 8;
#pragma unroll
            for (int s = 0; s < KS; ++s) kf[tt][s] = *reinterpret_cast<const bf16x8*>(kp + s * 32);
        }
        const int voff = min(t0 + 8 * c, cap - 8);
#pragma unroll
        for (int d = 0; d < DT; ++d)
            vf[d] = *reinterpret_cast<const bf16x8*>(vslab + (size_t)(d * 16 + r) * cap + voff);
    }
    bool v_fixed = false;

    const int ncols = it.nw * G;
    for (int col0 = 0; col0 < ncols; col0 += 16) {
        // ---- stage the group's query rows and their row limits -----------------------
        __syncthreads();   // the previous group's merge has read so[] and qs[]
        for (int i = t; i < 16 * (HD / 8); i += PFX_WAVES * 64) {
            const int col = col0 + i / (HD / 8), ch8 = i % (HD / 8);
            bf16x8 v;
#pragma unroll
            for (int j = 0; j < 8; ++j) v[j] = (bf16)0.f;
            if (col < ncols) {
                const int w = it.w0 + col / G, head = kvh * G + col % G;
                v = *reinterpret_cast<const bf16x8*>(q + ((size_t)w * Hq + head) * HD + ch8 * 8);
            }
            *reinterpret_cast<bf16x8*>(qs + (size_t)(i / (HD / 8)) * HD + ch8 * 8) = v;
        }
        if (t < 16) {
            const int col = col0 + t;
            int lim = 0;
            if (col < ncols) lim = it.tail ? n_rows : min(n_rows, tail_meta[it.w0 + col / G].pos_offset - it.row0);
            s_valid[t] = lim;
        }
        __syncthreads();

        floatx4 oacc[DT];
#pragma unroll
        for (int d = 0; d < DT; ++d) oacc[d] = floatx4{0.f, 0.f, 0.f, 0.f};
        float m_run = -INFINITY, l_run = 0.f;
        if (live) {
            if (!v_fixed && w_lo + 32 > n_rows) {   // rows past the item's end must not reach the MFMA
#pragma unroll
                for (int d = 0; d < DT; ++d)
#pragma unroll
                    for (int j = 0; j < 8; ++j)
                        if (w_lo + 8 * c + j >= n_rows) vf[d][j] = (bf16)0.f;
            }
            v_fixed = true;
            const int lim = s_valid[r];   // rows of the item column r may see
            // ---- S^T = K Q^T ------------------------------------------------------
            floatx4 sacc[2] = {floatx4{0.f, 0.f, 0.f, 0.f}, floatx4{0.f, 0.f, 0.f, 0.f}};
#pragma unroll
            for (int s = 0; s < KS; ++s) {
                const bf16x8 qf = *reinterpret_cast<const bf16x8*>(qs + r * HD + s * 32 + c * 8);
                sacc[0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[0][s], qf, sacc[0], 0, 0, 0);
                sacc[1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[1][s], qf, sacc[1], 0, 0, 0);
            }
            // sacc[tt][e]: column r, item row w_lo + 8c + 4tt + e
            float sv[8];
            float mx = -INFINITY;
#pragma unroll
            for (int tt = 0; tt < 2; ++tt)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int row = w_lo + 8 * c + 4 * tt + e;
                    const float sc = row < lim ? sacc[tt][e] * scale_log2 : -INFINITY;
                    sv[tt * 4 + e] = sc;
                    mx = fmaxf(mx, sc);
                }
            mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
            mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
            m_run = mx;                                   // -inf when the column sees none of the window
            const float m_use = mx == -INFINITY ? 0.f : mx;
            bf16x8 pf;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const float p = pfx_exp2(sv[j] - m_use);
                l_run += p;
                pf[j] = (bf16)p;
            }
            // ---- O^T = V^T P^T ----------------------------------------------------
#pragma unroll
            for (int d = 0; d < DT; ++d) oacc[d] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf[d], pf, oacc[d], 0, 0, 0);
            l_run += __shfl_xor(l_run, 16, 64);
            l_run += __shfl_xor(l_run, 32, 64);
        }

        // ---- merge the wavefronts in window order ------------------------------------
        // oacc[d][e]: column r, output element d*16 + 4c + e
        {
            float* rec = so + ((size_t)wave * 16 + r) * PLD;
#pragma unroll
            for (int d = 0; d < DT; ++d)
#pragma unroll
                for (int e = 0; e < 4; ++e) rec[d * 16 + 4 * c + e] = oacc[d][e];
            if (c == 0) {
                rec[HD] = m_run;
                rec[HD + 1] = l_run;
            }
        }
        __syncthreads();
        const int gcols = min(16, ncols - col0);
        for (int idx = t; idx < gcols * HD; idx += PFX_WAVES * 64) {
            const int g = idx / HD, dd = idx - g * HD;
            float mm = -INFINITY;
#pragma unroll
            for (int w = 0; w < PFX_WAVES; ++w) mm = fmaxf(mm, so[((size_t)w * 16 + g) * PLD + HD]);
            float ov = 0.f, l = 0.f;
#pragma unroll
            for (int w = 0; w < PFX_WAVES; ++w) {
                const float* rec = so + ((size_t)w * 16 + g) * PLD;
                const float lw = rec[HD + 1];
                const float f = lw > 0.f ? pfx_exp2(rec[HD] - mm) : 0.f;
                ov += f * rec[dd];
                l += f * lw;
            }
            float* out = records + ((size_t)kvh * total_recs + it.rec0 + col0 + g) * PLD;
            out[dd] = ov;
            if (dd == 0) {
                out[HD] = mm;
                out[HD + 1] = l;
            }
        }
    }
}

// Merges the records of one (worker, head): the items on the worker's list, in list
// order.  Tail chunks the step has not reached yet are skipped (nobody wrote them).
#define PFX_MAX_ITEMS 1024
template <int HD>
__global__ __launch_bounds__(HD) void attn_decode_prefix_combine_kernel(const BlockMeta* __restrict__ tail_meta,
                                                                        const PrefixItem* __restrict__ items,
                                                                        const int32_t* __restrict__ wl_off,
                                                                        const int32_t* __restrict__ wl, int step,
                                                                        const float* __restrict__ records, int64_t total_recs,
                                                                        bf16* __restrict__ o, int Hq, int Hkv) {
    constexpr int PLD = HD + 2;
    __shared__ float wgt[PFX_MAX_ITEMS];
    __shared__ int32_t roff[PFX_MAX_ITEMS];   // record index of every live item of this (worker, head)
    __shared__ float red_m[HD / 64], red_l[HD / 64];
    __shared__ int s_n;
    const int b = blockIdx.y, head = blockIdx.x, dd = threadIdx.x;
    const int G = Hq / Hkv, kvh = head / G, g = head % G;
    const int tail_rows = tail_meta[b].len + step + 1;
    if (dd == 0) {   // the list is short; one thread keeps its order
        int n = 0;
        for (int i = wl_off[b]; i < wl_off[b + 1]; ++i) {
            const PrefixItem it = items[wl[i]];
            if (it.tail && it.row0 >= tail_rows) continue;
            roff[n++] = it.rec0 + (b - it.w0) * G + g;
        }
        s_n = n;
    }
    __syncthreads();
    const int n = s_n;
    const float* base = records + (size_t)kvh * total_recs * PLD;
    float mm = -INFINITY;
    for (int i = dd; i < n; i += HD) mm = fmaxf(mm, base[(size_t)roff[i] * PLD + HD]);
#pragma unroll
    for (int ofs = 32; ofs > 0; ofs >>= 1) mm = fmaxf(mm, __shfl_xor(mm, ofs, 64));
    if ((dd & 63) == 0) red_m[dd >> 6] = mm;
    __syncthreads();
    mm = red_m[0];
#pragma unroll
    for (int i = 1; i < HD / 64; ++i) mm = fmaxf(mm, red_m[i]);
    for (int i = dd; i < n; i += HD) {
        const float* rec = base + (size_t)roff[i] * PLD;
        wgt[i] = rec[HD + 1] > 0.f ? pfx_exp2(rec[HD] - mm) : 0.f;
    }
    __syncthreads();
    if (dd == 0) {
        float l = 0.f;
        for (int i = 0; i < n; ++i) l += wgt[i] * base[(size_t)roff[i] * PLD + HD + 1];
        red_l[0] = l;
    }
    float acc = 0.f;
    for (int i = 0; i < n; ++i) acc += wgt[i] * base[(size_t)roff[i] * PLD + dd];
    __syncthreads();
    o[((size_t)b * Hq + head) * HD + dd] = (bf16)(acc / red_l[0]);
}

int launch_attn_decode_prefix_bf16(compact_ctx* ctx, const BlockMeta* d_tail_meta, const BlockMeta& shared,
                                   const PrefixItem* d_items, int n_items, const int32_t* d_wl_off, const int32_t* d_wl,
                                   int max_list, int n_workers, int step, const bf16* q, const bf16* kshared,
                                   const bf16* vshared, const bf16* ktail, const bf16* vtail, float* records,
                                   int64_t total_recs, bf16* o, hipStream_t s) {
    const compact_layer_cfg& c = ctx->cfg;
    if (n_items == 0) return COMPACT_OK;
    if (max_list > PFX_MAX_ITEMS) return set_err(ctx, COMPACT_ECAPACITY, "prefix longer than the prefix-aware combine supports");
    const float scale_log2 = LOG2E / sqrtf((float)c.head_dim);
    dim3 grid(n_items, c.n_kv_heads);
    dim3 cgrid(c.n_q_heads, n_workers);
    const size_t smem = (size_t)PFX_WAVES * 16 * (c.head_dim + 2) * sizeof(float);
    static bool attr_set = false;
    if (!attr_set) {
        const int big = PFX_WAVES * 16 * (128 + 2) * (int)sizeof(float);
        HIP_TRY(ctx, hipFuncSetAttribute(reinterpret_cast<const void*>(attn_decode_prefix_kernel<128>), hipFuncAttributeMaxDynamicSharedMemorySize, big));
        HIP_TRY(ctx, hipFuncSetAttribute(reinterpret_cast<const void*>(attn_decode_prefix_kernel<64>), hipFuncAttributeMaxDynamicSharedMemorySize, big));
        attr_set = true;
    }
    if (c.head_dim == 128) {
        {
            ProfileScope ps(ctx, COMPACT_K_ATTN_DECODE, s);
            attn_decode_prefix_kernel<128><<<grid, PFX_WAVES * 64, smem, s>>>(d_tail_meta, shared, d_items, step, q, kshared, vshared,
                                                                             ktail, vtail, records, total_recs, c.n_q_heads,
                                                                             c.n_kv_heads, scale_log2);
        }
        LAUNCH_CHECK(ctx);
        attn_decode_prefix_combine_kernel<128><<<cgrid, 128, 0, s>>>(d_tail_meta, d_items, d_wl_off, d_wl, step, records,
                                                                     total_recs, o, c.n_q_heads, c.n_kv_heads);
    } else {
        {
            ProfileScope ps(ctx, COMPACT_K_ATTN_DECODE, s);
            attn_decode_prefix_kernel<64><<<grid, PFX_WAVES * 64, smem, s>>>(d_tail_meta, shared, d_items, step, q, kshared, vshared,
                                                                            ktail, vtail, records, total_recs, c.n_q_heads,
                                                                            c.n_kv_heads, scale_log2);
        }
        LAUNCH_CHECK(ctx);
        attn_decode_prefix_combine_kernel<64><<<cgrid, 64, 0, s>>>(d_tail_meta, d_items, d_wl_off, d_wl, step, records, total_recs, o,
                                                                   c.n_q_heads, c.n_kv_heads);
    }
    LAUNCH_CHECK(ctx);
    return COMPACT_OK;
}
