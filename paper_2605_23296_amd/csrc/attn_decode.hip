// Split-KV decode attention (bf16 storage): one query token per block against
// that block's own KV cache.  HBM-bound: every cached K and V byte is read
// exactly once per step, with 16-byte loads that land directly in the MFMA
// operand layout (no LDS staging of K/V).
//
//  * work item = (DECODE_CHUNK cached tokens of one block, one kv head): all query
//    heads of that KV head's group are served from one read of the cache, and the
//    item yields one split-KV record (un-normalised output, maximum, sum) per query
//    head.  Chunks are fixed size, so the split of a block (and hence every record)
//    depends on its own length only.  Items are numbered kv-head-major over the
//    host-built (block, chunk) list.
//  * the kernel is persistent: a workgroup of 4 wavefronts takes a contiguous
//    share of the items and walks it in steps of DEC_SUB = 128 tokens, merging the
//    steps of an item in registers (running maximum, rescaled accumulators: the
//    online softmax), with its loads software-pipelined across steps and items.
//    The K operand registers of a step are free once its score MFMAs have issued,
//    the V^T operand registers once its output MFMAs have: the next step's K
//    loads go out right behind the former, its V^T loads right behind the latter,
//    so between half and all of a wavefront's load registers are in flight at
//    any time.
//  * records are stored once per item, as rarely as the fixed split allows: a
//    store in the middle of the load stream stalls it out of all proportion to
//    its bytes (measured: 2 KB of record stores per 64 KB of loads cost 25 %).
//  * scores: per 32-token window a wavefront computes S^T = K Q^T with
//    v_mfma_f32_16x16x32_bf16 (K rows as MFMA rows, the group's query heads,
//    padded to 16, as MFMA columns).  The MFMA rows of the two S^T tiles are
//    assigned to tokens so that a lane ends up with 8 consecutive tokens of
//    one column.
//  * the windows exchange their column maxima through LDS, so that all of them
//    exponentiate against the same maximum; the probabilities P^T go to LDS
//    as bf16 ([column][token]).
//  * output: wavefront w owns rows (HD/4) w .. of O^T = V^T P^T over ALL tokens
//    of the step: its V^T operand rows are contiguous runs of the transposed V
//    slab [hd][token], and nothing has to be merged across wavefronts.  Chunks
//    are merged by a second small kernel with a log-sum-exp combine in fixed
//    chunk order.
#include <algorithm>

#include "common.h"

#define LOG2E 1.4426950408889634f

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Workgroup barrier that leaves global loads in flight: only this wavefront's LDS operations are
// waited for.  (__syncthreads() would also wait for every outstanding global load, i.e. for the
// next step's K and V^T rows that the loop keeps in flight across its barriers.)
__device__ __forceinline__ void lds_barrier() {
#if defined(__HIP_DEVICE_COMPILE__)
    __builtin_amdgcn_sched_barrier(0);
    // simm16: vmcnt[3:0] = 15 | expcnt 7 << 4 | lgkmcnt 0 << 8 | vmcnt[5:4] = 3 << 14: wait for LDS only
    __builtin_amdgcn_s_waitcnt(15 | (7 << 4) | (0 << 8) | (3 << 14));
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
#endif
}

#define DEC_SUB 128                     // tokens per step of the walk through an item
#define DEC_WAVES (DEC_SUB / 32)        // one 32-token window per wavefront
#define DEC_PLD (DEC_SUB + 8)           // bf16 per column of the probability tile (padded against bank conflicts)
#define DEC_MAX_GROUPS(HD) ((HD) == 128 ? 3 : 4)   // workgroups per CU the grid is sized for (= the launch bounds)
#define DEC_REC_SLOTS 8                 // finished records (one per item, all columns) a workgroup can hold back
static_assert(DECODE_CHUNK % DEC_SUB == 0, "an item is a whole number of steps");

// Every vector-memory load of the loop is issued unconditionally (with a harmless in-bounds address
// where there is nothing to fetch) and the only conditional vector-memory instructions, the record
// stores, sit right before the V^T loads: the compiler counts outstanding operations per register
// to place its waits, and a load it cannot prove to have been issued makes it wait for newer loads
// than the one it needs, which would serialise the pipeline.  The work list and block table are
// read through the scalar cache (constant address space), outside the vector-memory counter.
template <int HD>
__global__ __launch_bounds__(DEC_WAVES * 64, HD == 128 ? 3 : 4) void attn_decode_bf16_kernel(
    const BlockMeta* __restrict__ meta_, const TileItem* __restrict__ chunks_, int n_chunks, int step, int max_chunks,
    const bf16* __restrict__ q, const bf16* __restrict__ kbase, const bf16* __restrict__ vbase, float* __restrict__ partials,
    int Hq, int Hkv, float scale_log2, const int32_t* __restrict__ qrow_, int q_stride, int64_t n_rec, int rec_slots) {
    constexpr int KS = HD / 32;                 // k-steps of the QK product
    constexpr int RT = HD / 16 / DEC_WAVES;     // 16-row tiles of O^T per wavefront
    constexpr int VS = DEC_SUB / 32;            // k-steps of the PV product
    static_assert(RT >= 1, "every wavefront owns at least one row tile of O^T");
    __shared__ __attribute__((aligned(16))) bf16 qs[16 * HD];        // [G][HD] query rows of the group
    __shared__ __attribute__((aligned(16))) bf16 ps[16 * DEC_PLD];   // P^T: [column][token of the step]
    __shared__ float s_max[DEC_WAVES][16], s_sum[DEC_WAVES][16];     // per-window maximum and sum of every column
    // finished records wait here ([slot][column][HD values, max, sum, 2 pad]) and leave for memory together, when the
    // share is done or the buffer is full: see the note on stores in the load stream above
    extern __shared__ __attribute__((aligned(16))) float recbuf[];
    __shared__ int rec_index[DEC_REC_SLOTS];
    typedef const __attribute__((address_space(4))) BlockMeta* MetaPtr;
    typedef const __attribute__((address_space(4))) TileItem* ItemPtr;
    typedef const __attribute__((address_space(4))) int32_t* IntPtr;
    const MetaPtr meta = (MetaPtr)meta_;
    const ItemPtr chunks = (ItemPtr)chunks_;
    const IntPtr qrow = (IntPtr)qrow_;

    const int G = Hq / Hkv;
    const int t = threadIdx.x, lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int r = lane & 15, c = lane >> 4;
    const int w_lo = wave * 32;

    // this workgroup's contiguous share of the items (item w: kv head w / n_chunks, list entry w % n_chunks)
    const int n_work = n_chunks * Hkv;
    int w = (int)((int64_t)blockIdx.x * n_work / gridDim.x);
    const int w_end = (int)((int64_t)(blockIdx.x + 1) * n_work / gridDim.x);

    // one step of the walk: DEC_SUB tokens from row c0 of (block b, kv head kvh); first / last step of its item
    struct Step {
        int b, kvh, c0, n_keys, n_rows, capacity, qr, chunk, first, last;
        const bf16 *kslab, *vslab;
    };
    // the step after `it` (the next DEC_SUB tokens of the item, or the first ones of the share's next item that
    // this call reaches: a list may hold chunks only later decode steps open); false when the share is exhausted
    auto next_step = [&](Step& it) -> bool {
        if (!it.last) {
            it.c0 += DEC_SUB;
            const int end = min(it.n_keys, (it.chunk + 1) * DECODE_CHUNK);
            it.n_rows = min(end - it.c0, DEC_SUB);
            it.first = 0;
            it.last = it.c0 + DEC_SUB >= end;
            return true;
        }
        while (w < w_end) {
            const int kvh = w / n_chunks;
            const int ci = w - kvh * n_chunks;
            const int b = chunks[ci].block, row0 = chunks[ci].row0;
            ++w;
            const int n_keys = meta[b].len + step + 1;
            if (row0 >= n_keys) continue;
            const int capacity = meta[b].capacity;
            const int64_t slab = meta[b].slab;
            it.b = b;
            it.kvh = kvh;
            it.c0 = row0;
            it.chunk = row0 / DECODE_CHUNK;
            it.n_keys = n_keys;
            const int end = min(n_keys, row0 + DECODE_CHUNK);
            it.n_rows = min(end - row0, DEC_SUB);
            it.first = 1;
            it.last = row0 + DEC_SUB >= end;
            it.capacity = capacity;
            it.qr = qrow_ ? qrow[b] : b;
            it.kslab = kbase + slab + (size_t)kvh * capacity * HD;
            it.vslab = vbase + slab + (size_t)kvh * HD * capacity;
            return true;
        }
        return false;
    };

    // scores: S^T tile tt, MFMA row m  <->  token c0 + w_lo + 8*(m/4) + 4*tt + (m%4)
    // output: lane (r, c) of row tile i, k-step j holds V^T[(wave*RT + i)*16 + r][c0 + 32j + 8c .. +7]
    bf16x8 kf[2][KS];
    bf16x8 vf[RT][VS];
    bf16x8 qreg;
    // real = 0: nothing to fetch (the share is exhausted): the same load instructions go out with every
    // offset masked to the first rows of the slab (masking, not a branch: both cases must be one instruction
    // stream for the compiler's load counting)
    auto load_k = [&](const Step& it, int real) {
        const int keep = -real;   // all ones or zero
#pragma unroll
        for (int tt = 0; tt < 2; ++tt) {
            // windows past the step's rows read the cache's last row (never used)
            const int tok = min(it.c0 + w_lo + 8 * (r >> 2) + 4 * tt + (r & 3), it.n_keys - 1) & keep;
            const bf16* kp = it.kslab + (size_t)tok * HD + c * 8;
#pragma unroll
            for (int s = 0; s < KS; ++s) kf[tt][s] = *reinterpret_cast<const bf16x8*>(kp + s * 32);
        }
    };
    auto load_v = [&](const Step& it, int real) {
        const int keep = -real;
#pragma unroll
        for (int i = 0; i < RT; ++i) {
            const bf16* vp = it.vslab + (size_t)((wave * RT + i) * 16 + r) * it.capacity;
#pragma unroll
            for (int j = 0; j < VS; ++j) {
                // tokens past the cache end are never used: keep the load inside the slab row
                const int voff = min((it.c0 & keep) + 32 * j + 8 * c, it.capacity - 8);
                vf[i][j] = *reinterpret_cast<const bf16x8*>(vp + voff);
            }
        }
    };
    // the group's query rows [G][HD] of a step's item, 16 bytes per thread (threads past the end re-read the last piece)
    const int q_piece = min(t, G * (HD / 8) - 1);
    auto load_q = [&](const Step& it) {
        qreg = *reinterpret_cast<const bf16x8*>(q + (size_t)it.qr * q_stride + (size_t)it.kvh * G * HD + q_piece * 8);
    };

    Step cur, nxt;
    cur.last = 1;
    if (!next_step(cur)) return;
    load_q(cur);
    load_k(cur, 1);
    load_v(cur, 1);
    int q_b = -1, q_kvh = -1;
    // running state of the item, per lane: maximum of column r (in the exp2 domain), this lane's share of the
    // column's sum, and the un-normalised output rows of this wavefront
    float m_run = -INFINITY, l_part = 0.f;
    int n_held = 0;   // records in the buffer
    floatx4 oacc[RT];
#pragma unroll
    for (int i = 0; i < RT; ++i) oacc[i] = floatx4{0.f, 0.f, 0.f, 0.f};
    for (;;) {
        nxt = cur;
        const int has_next = next_step(nxt) ? 1 : 0;
        const bool live = w_lo < cur.n_rows;
        // the group's query rows go through LDS; restaged only when (block, kv head) changes
        if (cur.b != q_b || cur.kvh != q_kvh) {
            q_b = cur.b;
            q_kvh = cur.kvh;
            if (t < G * (HD / 8)) *reinterpret_cast<bf16x8*>(qs + t * 8) = qreg;
            lds_barrier();
        }
        load_q(nxt);

        // ---- S^T = K Q^T over the wavefront's window; the window's column maxima ------
        float sv[8];
        float mx = -INFINITY;
        {
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
            // sacc[tt][e]: column g = r, token c0 + w_lo + 8c + 4tt + e
#pragma unroll
            for (int tt = 0; tt < 2; ++tt)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int row = w_lo + 8 * c + 4 * tt + e;
                    const float sc = row < cur.n_rows ? sacc[tt][e] * scale_log2 : -INFINITY;
                    sv[tt * 4 + e] = sc;
                    mx = fmaxf(mx, sc);
                }
            mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
            mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        }
        // the K operand registers are free: the next step's K rows go out now
        load_k(nxt, has_next);
        if (c == 0) s_max[wave][r] = mx;
        lds_barrier();

        // ---- running maximum of the item's columns; P = exp2(S - max); rescale what was accumulated ----
        float m_new = m_run;   // finite after this: the step holds at least one valid token
#pragma unroll
        for (int wv = 0; wv < DEC_WAVES; ++wv) m_new = fmaxf(m_new, s_max[wv][r]);
        const float alpha = fast_exp2(m_run - m_new);   // 0 on an item's first step (m_run = -inf)
        m_run = m_new;
        bf16x8 pf;
        float l_step = 0.f;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const float p = live ? fast_exp2(sv[j] - m_new) : 0.f;
            l_step += p;
            pf[j] = (bf16)p;
        }
        l_part = l_part * alpha + l_step;
#pragma unroll
        for (int i = 0; i < RT; ++i)
#pragma unroll
            for (int e = 0; e < 4; ++e) oacc[i][e] *= alpha;
        *reinterpret_cast<bf16x8*>(ps + r * DEC_PLD + w_lo + 8 * c) = pf;
        if (cur.n_rows < DEC_SUB) {  // ragged tail: bits past the cache end must not reach the MFMA
#pragma unroll
            for (int i = 0; i < RT; ++i)
#pragma unroll
                for (int j = 0; j < VS; ++j)
#pragma unroll
                    for (int e = 0; e < 8; ++e)
                        if (32 * j + 8 * c + e >= cur.n_rows) vf[i][j][e] = (bf16)0.f;
        }
        lds_barrier();

        // ---- O^T rows of this wavefront += V^T P^T over all tokens of the step ---------------
#pragma unroll
        for (int j = 0; j < VS; ++j) {
            const bf16x8 pb = *reinterpret_cast<const bf16x8*>(ps + r * DEC_PLD + 32 * j + 8 * c);
#pragma unroll
            for (int i = 0; i < RT; ++i) oacc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf[i][j], pb, oacc[i], 0, 0, 0);
        }
        if (cur.last) {
            // ---- the item is complete: its record goes to the buffer -------------------------------
            float l = l_part;
            l += __shfl_xor(l, 16, 64);
            l += __shfl_xor(l, 32, 64);
            if (c == 0) s_sum[wave][r] = l;
            lds_barrier();
            // oacc[i][e]: column g = r, output element (wave*RT + i)*16 + 4c + e
            float* slot = recbuf + (size_t)n_held * G * (HD + 4);
            if (r < G) {
#pragma unroll
                for (int i = 0; i < RT; ++i) *reinterpret_cast<floatx4*>(slot + r * (HD + 4) + (wave * RT + i) * 16 + 4 * c) = oacc[i];
                if (wave == 0 && c == 0) {
                    float lt = s_sum[0][r];
#pragma unroll
                    for (int wv = 1; wv < DEC_WAVES; ++wv) lt += s_sum[wv][r];
                    slot[r * (HD + 4) + HD] = m_run;
                    slot[r * (HD + 4) + HD + 1] = lt;
                }
            }
            if (t == 0) rec_index[n_held] = (int)(((size_t)cur.b * Hq + cur.kvh * G) * max_chunks + cur.chunk);   // column 0's record
            ++n_held;
            m_run = -INFINITY;
            l_part = 0.f;
#pragma unroll
            for (int i = 0; i < RT; ++i) oacc[i] = floatx4{0.f, 0.f, 0.f, 0.f};
        }
        if (n_held == rec_slots || (!has_next && n_held > 0)) {
            // ---- the held records leave: per record HD values (whole 128-byte lines) + (max, sum) in an
            // array of their own behind all the values
            lds_barrier();
            for (int k = 0; k < n_held; ++k) {
                const float* slot = recbuf + (size_t)k * G * (HD + 4);
                const int64_t rec0 = rec_index[k];
                for (int i = t; i < G * (HD / 4); i += DEC_WAVES * 64) {
                    const int g = i / (HD / 4), e = i % (HD / 4);
                    *reinterpret_cast<floatx4*>(partials + (rec0 + (int64_t)g * max_chunks) * HD + 4 * e) =
                        *reinterpret_cast<const floatx4*>(slot + g * (HD + 4) + 4 * e);
                }
                if (t < G)
                    *reinterpret_cast<float2*>(partials + (size_t)n_rec * HD + (rec0 + (int64_t)t * max_chunks) * 2) =
                        *reinterpret_cast<const float2*>(slot + t * (HD + 4) + HD);
            }
            n_held = 0;
            lds_barrier();
        }
        // the V^T operand registers are free: the next step's V^T rows go out now (behind the record stores)
        load_v(nxt, has_next);
        if (!has_next) break;
        cur = nxt;
    }
}

// merges the chunks of one (block, head) in chunk order and normalises.
// The chunk weights exp2(m_ch - M) / L are formed once in LDS; every thread
// then owns one output element and reads its chunk values 8 loads at a time.
#define COMBINE_MAX_CHUNKS 2048
template <int HD>
__global__ __launch_bounds__(HD) void attn_decode_combine_kernel(const BlockMeta* __restrict__ meta, int step, int max_chunks,
                                                                 const float* __restrict__ partials, bf16* __restrict__ o,
                                                                 int Hq, const int32_t* __restrict__ qrow, int64_t n_rec) {
    __shared__ float wgt[COMBINE_MAX_CHUNKS];
    __shared__ float red_m[HD / 64], red_l[HD / 64];
    const int b = blockIdx.y, head = blockIdx.x, dd = threadIdx.x;
    const int n_keys = meta[b].len + step + 1;
    const int nch = (n_keys + DECODE_CHUNK - 1) / DECODE_CHUNK;
    const size_t rec0 = ((size_t)b * Hq + head) * max_chunks;
    const float* val = partials + rec0 * HD;                         // [chunk][HD]
    const float* ml = partials + (size_t)n_rec * HD + rec0 * 2;      // [chunk](max, sum)
    // global max of the chunk maxima
    float mm = -INFINITY;
    for (int ch = dd; ch < nch; ch += HD) mm = fmaxf(mm, ml[ch * 2]);
#pragma unroll
    for (int ofs = 32; ofs > 0; ofs >>= 1) mm = fmaxf(mm, __shfl_xor(mm, ofs, 64));
    if ((dd & 63) == 0) red_m[dd >> 6] = mm;
    __syncthreads();
    mm = red_m[0];
#pragma unroll
    for (int i = 1; i < HD / 64; ++i) mm = fmaxf(mm, red_m[i]);
    // chunk weights; the normaliser is summed in chunk order by thread 0 afterwards
    for (int ch = dd; ch < nch; ch += HD) wgt[ch] = fast_exp2(ml[ch * 2] - mm);
    __syncthreads();
    if (dd == 0) {
        float l = 0.f;
        for (int ch = 0; ch < nch; ++ch) l += wgt[ch] * ml[ch * 2 + 1];
        red_l[0] = l;
    }
    float acc = 0.f;
    int ch = 0;
    for (; ch + 8 <= nch; ch += 8) {
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = val[(size_t)(ch + u) * HD + dd];
#pragma unroll
        for (int u = 0; u < 8; ++u) acc += wgt[ch + u] * v[u];
    }
    for (; ch < nch; ++ch) acc += wgt[ch] * val[(size_t)ch * HD + dd];
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
    // persistent workgroups: as many as stay resident (DEC_MAX_GROUPS per CU), each with a contiguous share
    int n_cus = 0;
    if (int rc = device_cu_count(ctx, &n_cus)) return rc;
    const int64_t n_work = (int64_t)n_chunks * c.n_kv_heads;
    // as many workgroups as stay resident (measured: fewer, evenly loaded ones -- 544 x 2 items instead of 768 x 1-2 --
    // and more than stay resident are both slower)
    dim3 grid((unsigned)std::min<int64_t>(n_work, (int64_t)n_cus * DEC_MAX_GROUPS(c.head_dim)));
    dim3 cgrid(c.n_q_heads, n_blocks);
    const int64_t n_rec = (int64_t)n_blocks * c.n_q_heads * max_chunks;   // records the partial buffer is laid out for
    const int G = c.n_q_heads / c.n_kv_heads;
    const size_t slot_bytes = (size_t)G * (c.head_dim + 4) * sizeof(float);
    const int rec_slots = (int)std::max<size_t>(1, std::min<size_t>(DEC_REC_SLOTS, (16 << 10) / slot_bytes));
    const size_t smem = rec_slots * slot_bytes;
    if (n_rec * (int64_t)1 > INT32_MAX) return set_err(ctx, COMPACT_ECAPACITY, "more split-KV records than the decode attention indexes");
    if (max_chunks > COMBINE_MAX_CHUNKS) return set_err(ctx, COMPACT_ECAPACITY, "KV cache longer than the decode combine supports");
    if (c.head_dim == 128) {
        {
            ProfileScope ps(ctx, COMPACT_K_ATTN_DECODE, s);
            attn_decode_bf16_kernel<128><<<grid, DEC_WAVES * 64, smem, s>>>(d_meta, d_chunks, n_chunks, step, max_chunks, q, d_k, d_v, partials,
                                                                           c.n_q_heads, c.n_kv_heads, scale_log2, d_qrow, q_stride, n_rec, rec_slots);
        }
        LAUNCH_CHECK(ctx);
        attn_decode_combine_kernel<128><<<cgrid, 128, 0, s>>>(d_meta, step, max_chunks, partials, o, c.n_q_heads, d_qrow, n_rec);
    } else {
        {
            ProfileScope ps(ctx, COMPACT_K_ATTN_DECODE, s);
            attn_decode_bf16_kernel<64><<<grid, DEC_WAVES * 64, smem, s>>>(d_meta, d_chunks, n_chunks, step, max_chunks, q, d_k, d_v, partials,
                                                                          c.n_q_heads, c.n_kv_heads, scale_log2, d_qrow, q_stride, n_rec, rec_slots);
        }
        LAUNCH_CHECK(ctx);
        attn_decode_combine_kernel<64><<<cgrid, 64, 0, s>>>(d_meta, step, max_chunks, partials, o, c.n_q_heads, d_qrow, n_rec);
    }
    LAUNCH_CHECK(ctx);
    return COMPACT_OK;
}
