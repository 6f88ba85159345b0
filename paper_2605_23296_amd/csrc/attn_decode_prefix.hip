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
#define PFX_WAVES (PREFIX_CHUNK / 32)
#define PFX_QCOLS 32   // query columns staged at a time (two MFMA column groups)

__device__ __forceinline__ float pfx_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

#define PFX_PLD (PREFIX_CHUNK + 8)   // bf16 per column of the shared probability tile (padded against bank conflicts)

template <int HD>
__global__ __launch_bounds__(PFX_WAVES * 64, 4) void attn_decode_prefix_kernel(const BlockMeta* __restrict__ tail_meta,
                                                                              const BlockMeta shared, const PrefixItem* __restrict__ items,
                                                                              int step, const bf16* __restrict__ q,
                                                                              const bf16* __restrict__ kshared,
                                                                              const bf16* __restrict__ vshared,
                                                                              const bf16* __restrict__ ktail,
                                                                              const bf16* __restrict__ vtail,
                                                                              float* __restrict__ records, int64_t total_recs, int Hq,
                                                                              int Hkv, float scale_log2) {
    constexpr int KS = HD / 32;            // k-steps of the QK product
    constexpr int DT = HD / 16;            // 16-row tiles of O^T, one per wavefront (the first DT wavefronts)
    constexpr int PLD = HD + 2;            // record: HD values, max, sum
    constexpr int VS = PREFIX_CHUNK / 32;  // k-steps of the PV product
    __shared__ __attribute__((aligned(16))) bf16 qs[PFX_QCOLS * HD];    // query rows of the staged columns
    __shared__ __attribute__((aligned(16))) bf16 ps[16 * PFX_PLD];      // P^T of the current column group: [column][item row]
    __shared__ float s_max[PFX_WAVES][16], s_sum[PFX_WAVES][16];        // per-window maximum and sum of every column
    __shared__ int s_valid[PFX_QCOLS];                                  // rows of the item each column may see

    const PrefixItem it = items[blockIdx.x];
    const int kvh = blockIdx.y;
    const int G = Hq / Hkv;
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int r = lane & 15, c = lane >> 4;

    const bf16 *kslab, *vslab;
    int cap, n_rows;   // rows of the item that exist at all
    if (it.tail) {
        const BlockMeta bm = tail_meta[it.w0];
        n_rows = min(bm.len + step + 1 - it.row0, PREFIX_CHUNK);
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
    const int w_lo = wave * 32;                 // first item row of this wavefront's score window
    const bool live = w_lo < n_rows;
    const int t0 = it.row0 + w_lo;              // slab row of the window
    const int last_row = it.row0 + n_rows - 1;

    // ---- loaded once, used by every column group ------------------------------------
    // scores: this wavefront's 32-row window of K.  S^T tile tt, MFMA row m <-> row t0 + 8*(m/4) + 4*tt + (m%4)
    // output: rows wave*16 .. +15 of V^T over all rows of the item; lane (r, c) of k-step j holds item rows 32j + 8c .. +7
    bf16x8 kf[2][KS];
    bf16x8 vf[VS];
    if (live) {
#pragma unroll
        for (int tt = 0; tt < 2; ++tt) {
            const int row = min(t0 + 8 * (r >> 2) + 4 * tt + (r & 3), last_row);
            const bf16* kp = kslab + (size_t)row * HD + c * 8;
#pragma unroll
            for (int s = 0; s < KS; ++s) kf[tt][s] = *reinterpret_cast<const bf16x8*>(kp + s * 32);
        }
    }
    if (wave < DT) {
        const bf16* vp = vslab + (size_t)(wave * 16 + r) * cap;
#pragma unroll
        for (int j = 0; j < VS; ++j) {
            const int ro = 32 * j + 8 * c;                       // item row of the lane's first element
            const int voff = min(it.row0 + ro, cap - 8);        // rows past the item are never used: keep the load in bounds
            vf[j] = *reinterpret_cast<const bf16x8*>(vp + voff);
        }
        // rows past the item's end must not reach the MFMA (their probabilities are zero, their bits are anything)
        if (n_rows < PREFIX_CHUNK) {
#pragma unroll
            for (int j = 0; j < VS; ++j)
#pragma unroll
                for (int i = 0; i < 8; ++i)
                    if (32 * j + 8 * c + i >= n_rows) vf[j][i] = (bf16)0.f;
        }
    }

    const int ncols = it.nw * G;
    for (int col0 = 0; col0 < ncols; col0 += 16) {
        // ---- every PFX_QCOLS columns: stage their query rows and row limits ---------
        __syncthreads();   // the previous group has read ps[], s_max[], s_sum[], qs[] and s_valid[]
        if (col0 % PFX_QCOLS == 0) {
            for (int i = t; i < PFX_QCOLS * (HD / 8); i += PFX_WAVES * 64) {
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
            if (t < PFX_QCOLS) {
                const int col = col0 + t;
                int lim = 0;
                if (col < ncols) lim = it.tail ? n_rows : min(n_rows, tail_meta[it.w0 + col / G].pos_offset - it.row0);
                s_valid[t] = lim;
            }
            __syncthreads();
        }
        const int qc = col0 % PFX_QCOLS;   // first staged column of this group

        // ---- S^T = K Q^T over the wavefront's window; the window's column maxima ----
        float sv[8];
        float mx = -INFINITY;
        if (live) {
            const int lim = s_valid[qc + r];   // rows of the item column r may see
            floatx4 sacc[2] = {floatx4{0.f, 0.f, 0.f, 0.f}, floatx4{0.f, 0.f, 0.f, 0.f}};
#pragma unroll
            for (int s = 0; s < KS; ++s) {
                const bf16x8 qf = *reinterpret_cast<const bf16x8*>(qs + (qc + r) * HD + s * 32 + c * 8);
                sacc[0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[0][s], qf, sacc[0], 0, 0, 0);
                sacc[1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[1][s], qf, sacc[1], 0, 0, 0);
            }
            // sacc[tt][e]: column r, item row w_lo + 8c + 4tt + e
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
        }
        if (c == 0) s_max[wave][r] = mx;
        __syncthreads();

        // ---- one maximum per column for the whole item: P = exp2(S - max) -----------
        float m_all = s_max[0][r];
#pragma unroll
        for (int w = 1; w < PFX_WAVES; ++w) m_all = fmaxf(m_all, s_max[w][r]);
        const float m_use = m_all == -INFINITY ? 0.f : m_all;   // a column that sees none of the item
        bf16x8 pf;
        float l_run = 0.f;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const float p = live ? pfx_exp2(sv[j] - m_use) : 0.f;
            l_run += p;
            pf[j] = (bf16)p;
        }
        l_run += __shfl_xor(l_run, 16, 64);
        l_run += __shfl_xor(l_run, 32, 64);
        if (c == 0) s_sum[wave][r] = l_run;
        *reinterpret_cast<bf16x8*>(ps + r * PFX_PLD + w_lo + 8 * c) = pf;
        __syncthreads();

        // ---- O^T rows wave*16 .. +15 = V^T P^T over all rows of the item --------------
        if (wave < DT) {
            floatx4 oacc = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int j = 0; j < VS; ++j) {
                const bf16x8 pb = *reinterpret_cast<const bf16x8*>(ps + r * PFX_PLD + 32 * j + 8 * c);
                oacc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf[j], pb, oacc, 0, 0, 0);
            }
            // oacc[e]: column r, output element wave*16 + 4c + e
            if (col0 + r < ncols) {
                float* out = records + ((size_t)kvh * total_recs + it.rec0 + col0 + r) * PLD;
                *reinterpret_cast<float2*>(out + wave * 16 + 4 * c) = float2{oacc[0], oacc[1]};
                *reinterpret_cast<float2*>(out + wave * 16 + 4 * c + 2) = float2{oacc[2], oacc[3]};
                if (wave == 0 && c == 0) {
                    float l = s_sum[0][r];
#pragma unroll
                    for (int w = 1; w < PFX_WAVES; ++w) l += s_sum[w][r];
                    out[HD] = m_all;
                    out[HD + 1] = l;
                }
            }
        }
    }
}

// Merges the records of one (worker, head): the items on the worker's list.  Tail
// chunks the step has not reached yet carry weight zero and are never read (nobody
// wrote them).  256 threads: HD / 2 threads span a record, 512 / HD records are read
// side by side, 16 loads in flight per thread (4: 30.6 us at 24 workers, 16: 24.5 us); all sums run in a fixed order.
#define PFX_MAX_ITEMS 1024
#define PFX_CT 256
#define PFX_FLIGHT 16
template <int HD>
__global__ __launch_bounds__(PFX_CT) void attn_decode_prefix_combine_kernel(const BlockMeta* __restrict__ tail_meta,
                                                                            const PrefixItem* __restrict__ items,
                                                                            const int32_t* __restrict__ wl_off,
                                                                            const int32_t* __restrict__ wl, int step,
                                                                            const float* __restrict__ records, int64_t total_recs,
                                                                            bf16* __restrict__ o, int Hq, int Hkv) {
    constexpr int PLD = HD + 2;
    constexpr int TPR = HD / 2;          // threads per record (two floats each)
    constexpr int NS = PFX_CT / TPR;     // records read side by side
    __shared__ float wgt[PFX_MAX_ITEMS];
    __shared__ int32_t roff[PFX_MAX_ITEMS];
    __shared__ float red[PFX_CT / 64];
    __shared__ float2 part[NS][TPR];
    const int b = blockIdx.y, head = blockIdx.x, t = threadIdx.x;
    const int G = Hq / Hkv, kvh = head / G, g = head % G;
    const int tail_rows = tail_meta[b].len + step + 1;
    const int l0 = wl_off[b], n = wl_off[b + 1] - l0;
    const float* base = records + (size_t)kvh * total_recs * PLD;
    // record index of every item on the list, -1 for a tail chunk not reached yet; running maximum
    float mm = -INFINITY;
    for (int i = t; i < n; i += PFX_CT) {
        const PrefixItem it = items[wl[l0 + i]];
        const bool dead = it.tail && it.row0 >= tail_rows;
        const int ro = dead ? -1 : it.rec0 + (b - it.w0) * G + g;
        roff[i] = ro;
        if (!dead) mm = fmaxf(mm, base[(size_t)ro * PLD + HD]);
    }
#pragma unroll
    for (int ofs = 32; ofs > 0; ofs >>= 1) mm = fmaxf(mm, __shfl_xor(mm, ofs, 64));
    if ((t & 63) == 0) red[t >> 6] = mm;
    __syncthreads();
    mm = red[0];
#pragma unroll
    for (int i = 1; i < PFX_CT / 64; ++i) mm = fmaxf(mm, red[i]);
    __syncthreads();   // red[] is reused below
    float l = 0.f;
    for (int i = t; i < n; i += PFX_CT) {
        float wi = 0.f;
        if (roff[i] >= 0) {
            const float* rec = base + (size_t)roff[i] * PLD;
            const float li = rec[HD + 1];
            wi = li > 0.f ? pfx_exp2(rec[HD] - mm) : 0.f;
            l += wi * li;
        }
        wgt[i] = wi;
    }
#pragma unroll
    for (int ofs = 32; ofs > 0; ofs >>= 1) l += __shfl_xor(l, ofs, 64);
    if ((t & 63) == 0) red[t >> 6] = l;
    __syncthreads();   // wgt[] complete as well
    l = red[0];
#pragma unroll
    for (int i = 1; i < PFX_CT / 64; ++i) l += red[i];
    const int sl = t / TPR, e = t % TPR;
    // PFX_FLIGHT records in flight per thread; a record that carries no weight (a tail chunk nobody wrote)
    // is read from a valid address and dropped
    float2 acc = float2{0.f, 0.f};
    for (int i0 = sl; i0 < n; i0 += PFX_FLIGHT * NS) {
        float2 v[PFX_FLIGHT];
        float wi[PFX_FLIGHT];
#pragma unroll
        for (int u = 0; u < PFX_FLIGHT; ++u) {
            const int i = i0 + u * NS;
            wi[u] = i < n ? wgt[i] : 0.f;
            const int ro = i < n ? max(roff[i], 0) : 0;
            v[u] = *reinterpret_cast<const float2*>(base + (size_t)ro * PLD + 2 * e);
        }
#pragma unroll
        for (int u = 0; u < PFX_FLIGHT; ++u)
            if (wi[u] != 0.f) {
                acc.x += wi[u] * v[u].x;
                acc.y += wi[u] * v[u].y;
            }
    }
    part[sl][e] = acc;
    __syncthreads();
    if (sl == 0) {
#pragma unroll
        for (int j = 1; j < NS; ++j) {
            acc.x += part[j][e].x;
            acc.y += part[j][e].y;
        }
        bf16x2 out;
        out[0] = (bf16)(acc.x / l);
        out[1] = (bf16)(acc.y / l);
        *reinterpret_cast<bf16x2*>(o + ((size_t)b * Hq + head) * HD + 2 * e) = out;
    }
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
    if (c.head_dim == 128) {
        {
            ProfileScope ps(ctx, COMPACT_K_ATTN_DECODE, s);
            attn_decode_prefix_kernel<128><<<grid, PFX_WAVES * 64, 0, s>>>(d_tail_meta, shared, d_items, step, q, kshared, vshared,
                                                                             ktail, vtail, records, total_recs, c.n_q_heads,
                                                                             c.n_kv_heads, scale_log2);
        }
        LAUNCH_CHECK(ctx);
        attn_decode_prefix_combine_kernel<128><<<cgrid, PFX_CT, 0, s>>>(d_tail_meta, d_items, d_wl_off, d_wl, step, records,
                                                                     total_recs, o, c.n_q_heads, c.n_kv_heads);
    } else {
        {
            ProfileScope ps(ctx, COMPACT_K_ATTN_DECODE, s);
            attn_decode_prefix_kernel<64><<<grid, PFX_WAVES * 64, 0, s>>>(d_tail_meta, shared, d_items, step, q, kshared, vshared,
                                                                            ktail, vtail, records, total_recs, c.n_q_heads,
                                                                            c.n_kv_heads, scale_log2);
        }
        LAUNCH_CHECK(ctx);
        attn_decode_prefix_combine_kernel<64><<<cgrid, PFX_CT, 0, s>>>(d_tail_meta, d_items, d_wl_off, d_wl, step, records, total_recs, o,
                                                                   c.n_q_heads, c.n_kv_heads);
    }
    LAUNCH_CHECK(ctx);
    return COMPACT_OK;
}
