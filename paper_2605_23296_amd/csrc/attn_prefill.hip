// Varlen causal flash-style prefill attention (bf16 storage, MFMA).
// Every block attends only its own tokens; the packed batch is walked through
// a list of (block, 128-row query tile) items sorted heaviest-first.
//
//  * workgroup = 4 wavefronts = one query tile x one query head; wave w owns
//    32 query rows and keeps Q^T in registers as the MFMA column operand;
//  * K tiles [64 tok][hd] and V^T tiles [hd][64 tok] (the V slab is stored
//    transposed, so no transposition happens here) are staged in LDS, double
//    buffered, register-prefetched, with XOR-swizzled 16-byte chunks;
//  * S^T = K Q^T and O^T += V^T P^T with v_mfma_f32_32x32x16_bf16.  Working
//    on the transposed problem puts one query row in one lane column, so the
//    online-softmax max/sum are in-lane reductions plus one cross-half
//    shuffle, and P^T feeds the second MFMA straight from the accumulator
//    registers: the MFMA rows of S^T are assigned to tokens such that each
//    lane's 8 accumulator values of a k-step are 8 consecutive tokens, which
//    is one 16-byte read of the V^T tile;
//  * causal tiles above the diagonal are skipped per wavefront; rows of the
//    V^T tile past the block's length are zeroed when staged.
#include "common.h"

#define KV_TILE 64
#define LOG2E 1.4426950408889634f

typedef float floatx2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

// Chunk swizzles.  The LDS has 64 banks of 4 bytes (256 bytes per cycle) and a
// 16-byte read is served 16 lanes at a time, so the 16 lanes must land in 16
// different 16-byte bank groups.  K-tile rows of 256 bytes (16 chunks) cover all
// groups by themselves: the 16 lanes read 16 different rows (a permutation of
// 0..15, +16), so the chunk index is XOR-ed with row % 16.  Rows of 128 bytes (8
// chunks: K at head_dim 64, every V^T tile) fill the banks two rows at a time:
// the chunk index is XOR-ed with (row / 2) % 8.
template <int CHUNKS>
__device__ __forceinline__ int swz(int row) { return CHUNKS == 16 ? (row & 15) : ((row >> 1) & 7); }

// eight floats to eight bf16 with four packed conversions
__device__ __forceinline__ bf16x8 pack_bf16x8(const float (&v)[8]) {
    union {
        bf16x8 v8;
        bf16x2 v2[4];
    } u;
#pragma unroll
    for (int j = 0; j < 4; ++j) u.v2[j] = __builtin_convertvector(floatx2{v[2 * j], v[2 * j + 1]}, bf16x2);
    return u.v8;
}

template <int HD>
__global__ __launch_bounds__(256, 2) void attn_prefill_bf16_kernel(const BlockMeta* __restrict__ meta,
                                                                const TileItem* __restrict__ qtiles,
                                                                const bf16* __restrict__ qkv, const bf16* __restrict__ kbase,
                                                                const bf16* __restrict__ vbase, bf16* __restrict__ o, int Hq,
                                                                int Hkv, float scale_log2) {
    constexpr int KK = HD / 16;        // k16 steps of S^T
    constexpr int DT = HD / 32;        // 32-row tiles of O^T
    constexpr int KCH = HD / 8;        // 16-byte chunks per K row
    constexpr int KTILE = KV_TILE * HD;   // elements of a K tile == elements of a V^T tile
    constexpr int NLD = KTILE / 8 / 256;  // chunks per thread per tile
    extern __shared__ __attribute__((aligned(16))) char smem[];
    bf16* lds = reinterpret_cast<bf16*>(smem);  // [2 stages][K tile | V^T tile]

    const TileItem it = qtiles[blockIdx.x];
    const BlockMeta bm = meta[it.block];
    const int head = blockIdx.y, kvh = head / (Hq / Hkv);
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int r = lane & 31, h = lane >> 5;
    const int ld = (Hq + 2 * Hkv) * HD;
    const int len = bm.prior + bm.len;   // cache rows once this call's rows are in
    const int prior = bm.prior;          // query row i of the call is cache row prior + i

    const bf16* kslab = kbase + bm.slab + (size_t)kvh * bm.capacity * HD;
    const bf16* vslab = vbase + bm.slab + (size_t)kvh * HD * bm.capacity;

    // ---- Q^T operand: lane (q = r, h) holds Q[q][kk*16 + h*8 .. +7] -----------
    const int qrow = prior + it.row0 + wave * 32 + r;   // as a cache row
    const int qrow_c = min(qrow, len - 1);
    const bf16* qp = qkv + (size_t)(bm.row0 + qrow_c - prior) * ld + head * HD + h * 8;
    bf16x8 qf[KK];
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) qf[kk] = *reinterpret_cast<const bf16x8*>(qp + kk * 16);

    floatx16 oacc[DT];
#pragma unroll
    for (int d = 0; d < DT; ++d)
#pragma unroll
        for (int e = 0; e < 16; ++e) oacc[d][e] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;

    const int q_hi_wg = min(prior + it.row0 + PREFILL_QTILE, len) - 1;   // last query row of the workgroup
    const int q_hi_wave = prior + it.row0 + wave * 32 + 31;              // last query row of this wave
    const int n_tiles = q_hi_wg / KV_TILE + 1;

    // ---- staging: 16-byte global loads that land in LDS directly ---------------------
    // A wave-instruction fills 64 consecutive 16-byte chunks of a tile; chunk L of the K tile is
    // (row L / KCH, position L % KCH) and holds the row's chunk (L % KCH) ^ swz(row), chunk L of the
    // V^T tile likewise with 8 chunks per row: each lane picks the global address that belongs in
    // its slot.  Wavefront w issues instructions w, w + 4, ...; nothing passes through registers.
    unsigned koff[NLD], voff[NLD];   // element offsets inside a tile's source rows, fixed per lane
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
        const int L = (i * 4 + wave) * 64 + lane;
        const int krow = L / KCH, kc = (L % KCH) ^ swz<KCH>(krow);
        koff[i] = (unsigned)(krow * HD + kc * 8);
        const int vrow = L >> 3, vc = (L & 7) ^ swz<8>(vrow);
        voff[i] = (unsigned)(vrow * bm.capacity + vc * 8);
    }
    auto issue_tile = [&](int kt, int stage) {
        const int kv0 = kt * KV_TILE;
        bf16* ks = lds + stage * 2 * KTILE;
        bf16* vs = ks + KTILE;
        if (kv0 + KV_TILE <= len) {   // the whole tile lies inside the cache: no clamps
            const bf16* kt0 = kslab + (size_t)kv0 * HD;
            const bf16* vt0 = vslab + kv0;
#pragma unroll
            for (int i = 0; i < NLD; ++i) {
                load16_to_lds(kt0 + koff[i], ks + (i * 4 + wave) * 64 * 8);
                load16_to_lds(vt0 + voff[i], vs + (i * 4 + wave) * 64 * 8);
            }
        } else {   // last tile of the block: rows past the end are clamped (their scores are masked)
#pragma unroll
            for (int i = 0; i < NLD; ++i) {
                const int L = (i * 4 + wave) * 64 + lane;
                const int krow = L / KCH, kc = (L % KCH) ^ swz<KCH>(krow);
                const int tok = min(kv0 + krow, len - 1);
                load16_to_lds(kslab + (size_t)tok * HD + kc * 8, ks + (i * 4 + wave) * 64 * 8);
                const int vrow = L >> 3, vc = (L & 7) ^ swz<8>(vrow);
                const int vt = min(kv0 + vc * 8, bm.capacity - 8);
                load16_to_lds(vslab + (size_t)vrow * bm.capacity + vt, vs + (i * 4 + wave) * 64 * 8);
            }
        }
    };
    // After a wavefront's own loads of a LAST tile have landed: zero the V^T entries of tokens past
    // the block's end (whatever the slab holds there must not reach the MFMA; their probabilities are 0).
    auto fix_tail = [&](int kt, int stage) {
        const int kv0 = kt * KV_TILE;
        if (kv0 + KV_TILE <= len) return;
        bf16* vs = lds + stage * 2 * KTILE + KTILE;
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            const int L = (i * 4 + wave) * 64 + lane;
            const int vrow = L >> 3, vc = (L & 7) ^ swz<8>(vrow);
            if (kv0 + vc * 8 + 8 > len) {
                bf16x8 v = *reinterpret_cast<bf16x8*>(vs + (size_t)L * 8);
#pragma unroll
                for (int j = 0; j < 8; ++j)
                    if (kv0 + vc * 8 + j >= len) v[j] = (bf16)0.f;
                *reinterpret_cast<bf16x8*>(vs + (size_t)L * 8) = v;
            }
        }
    };

    issue_tile(0, 0);
    wait_all_memory();
    fix_tail(0, 0);
    __syncthreads();

    // token of MFMA row i of S^T tile tt: tt*32 + pi(i); pi keeps each lane's
    // accumulator values of one k-step on 8 consecutive tokens
    const int pi_r = (r >> 4) * 16 + ((r >> 2) & 1) * 8 + ((r >> 3) & 1) * 4 + (r & 3);

    // One KV tile for this wavefront.  `diag` (wavefront-uniform) is set only for
    // tiles that straddle the wavefront's diagonal, so the tiles below it carry no
    // compare/select.
    auto tile_step = [&](bool diag, int kv0, const bf16* ks, const bf16* vs) {
        // ---- S^T = K Q^T ----------------------------------------------------
        floatx16 sacc[2];
#pragma unroll
        for (int tt = 0; tt < 2; ++tt) {
#pragma unroll
            for (int e = 0; e < 16; ++e) sacc[tt][e] = 0.f;
            const int row = tt * 32 + pi_r;
            const bf16* kr = ks + row * HD;
#pragma unroll
            for (int kk = 0; kk < KK; ++kk) {
                const bf16x8 kf = *reinterpret_cast<const bf16x8*>(kr + (((kk * 2 + h) ^ swz<KCH>(row)) << 3));
                sacc[tt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[kk], sacc[tt], 0, 0, 0);
            }
        }
        // sacc[tt][e]: query column r, token kv0 + tt*32 + (e/8)*16 + h*8 + (e%8)
        if (__builtin_amdgcn_readfirstlane((int)diag)) {
#pragma unroll
            for (int tt = 0; tt < 2; ++tt)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int tok = kv0 + tt * 32 + (e >> 3) * 16 + h * 8 + (e & 7);
                    if (tok > qrow) sacc[tt][e] = -INFINITY;
                }
        }
        float mx = -INFINITY;
#pragma unroll
        for (int tt = 0; tt < 2; ++tt)
#pragma unroll
            for (int e = 0; e < 16; ++e) mx = fmaxf(mx, sacc[tt][e]);
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64)) * scale_log2;
        // The running maximum is only a scaling reference: it is moved (and the
        // accumulators rescaled) when some row's scores outgrow it by more than 2^8;
        // until then exp2 stays within a factor 256 of 1, which fp32 sums and bf16
        // probabilities carry without loss.  The first tile always takes this path.
        if (__any(mx > m_run + 8.0f)) {
            const float m_new = fmaxf(m_run, mx);   // finite: tile 0 holds token 0 <= every query row
            const float corr = __builtin_amdgcn_exp2f(m_run - m_new);
            l_run *= corr;
            m_run = m_new;
#pragma unroll
            for (int d = 0; d < DT; ++d)
#pragma unroll
                for (int e = 0; e < 16; ++e) oacc[d][e] *= corr;
        }
        const float neg_m = -m_run;
        float ps = 0.f;
        bf16x8 pf[4];
#pragma unroll
        for (int tt = 0; tt < 2; ++tt)
#pragma unroll
            for (int g8 = 0; g8 < 2; ++g8) {
                float pv[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    pv[j] = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[tt][g8 * 8 + j], scale_log2, neg_m));
                    ps += pv[j];
                }
                pf[tt * 2 + g8] = pack_bf16x8(pv);
            }
        l_run += ps;
        // ---- O^T += V^T P^T ---------------------------------------------------
#pragma unroll
        for (int d = 0; d < DT; ++d) {
            const int row = d * 32 + r;
            const bf16* vr = vs + row * KV_TILE;
#pragma unroll
            for (int u = 0; u < 4; ++u) {   // k-step u covers tokens u*16 .. u*16+15 of the tile
                const bf16x8 vf = *reinterpret_cast<const bf16x8*>(vr + (((u * 2 + h) ^ swz<8>(row)) << 3));
                oacc[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[u], oacc[d], 0, 0, 0);
            }
        }
    };

    const int q_lo_wave = prior + it.row0 + wave * 32;   // first query row of this wave
    for (int kt = 0; kt < n_tiles; ++kt) {
        const int kv0 = kt * KV_TILE;
        const bf16* ks = lds + (kt & 1) * 2 * KTILE;
        const bf16* vs = ks + KTILE;
        const bool more = kt + 1 < n_tiles;
        // the other stage was last read in the previous iteration, which every wavefront has left
        if (more) issue_tile(kt + 1, (kt + 1) & 1);

        if (kv0 <= q_hi_wave) {   // otherwise the whole tile is above this wave's diagonal
            tile_step(kv0 + KV_TILE - 1 > q_lo_wave, kv0, ks, vs);   // diag: some entry may be masked
        }
        if (more) {
            wait_all_memory();
            fix_tail(kt + 1, (kt + 1) & 1);
        }
        __syncthreads();
    }

    // ---- normalise and store: lane (q = r) holds elements d*32 + (e/4)*8 + h*4 + (e%4) ----
    l_run += __shfl_xor(l_run, 32, 64);
    if (qrow < len) {
        const float inv = 1.0f / l_run;
        bf16* op = o + (size_t)(bm.row0 + qrow - prior) * Hq * HD + head * HD;
#pragma unroll
        for (int d = 0; d < DT; ++d)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                bf16x4 v;
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = (bf16)(oacc[d][g * 4 + e] * inv);
                *reinterpret_cast<bf16x4*>(op + d * 32 + g * 8 + h * 4) = v;
            }
    }
}

int launch_attn_prefill_bf16(compact_ctx* ctx, const BlockMeta* d_meta, const TileItem* d_qtiles, int n_qtiles,
                             const bf16* qkv, const bf16* d_k, const bf16* d_v, bf16* o, hipStream_t s) {
    if (n_qtiles == 0) return COMPACT_OK;
    const compact_layer_cfg& c = ctx->cfg;
    const float scale_log2 = LOG2E / sqrtf((float)c.head_dim);
    dim3 grid(n_qtiles, c.n_q_heads);
    const size_t smem = (size_t)2 * 2 * KV_TILE * c.head_dim * sizeof(bf16);
    if (c.head_dim == 128)
        attn_prefill_bf16_kernel<128><<<grid, 256, smem, s>>>(d_meta, d_qtiles, qkv, d_k, d_v, o, c.n_q_heads, c.n_kv_heads, scale_log2);
    else
        attn_prefill_bf16_kernel<64><<<grid, 256, smem, s>>>(d_meta, d_qtiles, qkv, d_k, d_v, o, c.n_q_heads, c.n_kv_heads, scale_log2);
    LAUNCH_CHECK(ctx);
    return COMPACT_OK;
}
