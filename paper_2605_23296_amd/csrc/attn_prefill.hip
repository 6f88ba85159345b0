// Varlen causal flash-style prefill attention (bf16 storage, MFMA).
// Every block attends only its own tokens; the packed batch is walked through
// a list of (block, 128-row query tile) items sorted heaviest-first.
//
//  * two kernels.  Head_dim 128 with an even GQA group: a workgroup of 8
//    wavefronts takes one query tile x TWO query heads of one KV head; the
//    wavefronts w and w + 4 share a SIMD and run the same loop one phase apart
//    ("ping-pong": one in its matrix phase while the other does its softmax),
//    separated by workgroup barriers.  Otherwise (head_dim 64, odd group): a
//    workgroup of 4 wavefronts = one query tile x one query head.  In both, a
//    wavefront owns 32 query rows and keeps Q^T in registers as the MFMA
//    column operand;
//  * K tiles [64 tok][hd] and V^T tiles [hd][64 tok] (the V slab is stored
//    transposed, so no transposition happens here) are staged by 16-byte
//    global loads that land in LDS directly (no register hop, no LDS stores),
//    in XOR-swizzled 16-byte chunks: a ring of four stages shared by the two
//    heads in the ping-pong kernel, of two stages in the other;
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

// 16-byte buffer load whose result goes straight into LDS: lane l deposits its 16 bytes at
// lds_base + 16 * l (lds_base is wave-uniform) from byte base + voff + soff of the buffer.  The range
// check (voff + 16 <= size, soff is not part of it) makes an out-of-range lane read zeros.  Offsets are
// 32-bit and the descriptor sits in scalar registers, so staging needs no 64-bit address arithmetic.
__device__ __forceinline__ void buf_load16_to_lds(__amdgpu_buffer_rsrc_t rsrc, void* lds_base, unsigned voff, unsigned soff) {
#if defined(__HIP_DEVICE_COMPILE__)
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (__attribute__((address_space(3))) void*)lds_base, 16, voff, soff, 0, 0);
#else
    (void)rsrc, (void)lds_base, (void)voff, (void)soff;
#endif
}
// raw buffer descriptor over [p, p + bytes): stride 0, 32-bit data format
__device__ __forceinline__ __amdgpu_buffer_rsrc_t raw_buffer(const void* p, unsigned bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, (int)bytes, 0x00020000);
}

// Waits until at most N of this wavefront's vector-memory operations are still in flight
// (they complete in order, so everything older has landed); LDS traffic is not waited for.
template <int N>
__device__ __forceinline__ void wait_vm() {
#if defined(__HIP_DEVICE_COMPILE__)
    static_assert(N >= 0 && N < 64, "vector-memory counter is 6 bits");
    __builtin_amdgcn_sched_barrier(0);
    // simm16: vmcnt[3:0] | expcnt (7 = no wait) << 4 | lgkmcnt (15 = no wait) << 8 | vmcnt[5:4] << 14
    __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | (15 << 8) | ((N >> 4) << 14));
    __builtin_amdgcn_sched_barrier(0);
#endif
}

// Workgroup barrier that leaves global loads in flight: only this wavefront's LDS
// operations are waited for (its reads of a stage about to be refilled, its writes
// into a stage about to be read).
__device__ __forceinline__ void phase_barrier() {
#if defined(__HIP_DEVICE_COMPILE__)
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_waitcnt(15 | (7 << 4) | (0 << 8) | (3 << 14));
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
#endif
}

// PP = false: workgroup = 4 wavefronts = 128 query rows x one query head, two workgroups per
// CU, two-stage K/V ring, every wavefront runs QK^T -> softmax -> PV per tile.
// PP = true ("ping-pong"): workgroup = 8 wavefronts = the same 128 query rows x TWO query heads
// of one KV head.  Wavefronts w and w + 4 share a SIMD; group 0 (waves 0-3, first head) and
// group 1 (waves 4-7, second head) run the same loop one phase apart, with a workgroup barrier
// at every phase boundary: while one group's wavefront is in its matrix phase (PV of the previous
// tile, QK^T of this one: 32 MFMAs) the other wavefront on the same SIMD is in its softmax phase
// (VALU only), so the matrix pipe and the vector ALU work at the same time instead of both
// wavefronts asking for the same one.  Both groups read the same K/V tiles (one staging for two
// heads); a tile stays live for four phases, hence a four-stage ring.
template <int HD, bool PP>
__global__ __launch_bounds__(PP ? 512 : 256, 2) void attn_prefill_bf16_kernel(const BlockMeta* __restrict__ meta,
                                                                           const TileItem* __restrict__ qtiles,
                                                                           const bf16* __restrict__ qkv,
                                                                           const bf16* __restrict__ kbase,
                                                                           const bf16* __restrict__ vbase, bf16* __restrict__ o,
                                                                           int Hq, int Hkv, float scale_log2) {
    constexpr int KK = HD / 16;        // k16 steps of S^T
    constexpr int DT = HD / 32;        // 32-row tiles of O^T
    constexpr int KCH = HD / 8;        // 16-byte chunks per K row
    constexpr int KTILE = KV_TILE * HD;   // elements of a K tile == elements of a V^T tile
    constexpr int NW = PP ? 8 : 4;        // wavefronts that stage a tile
    constexpr int NLD = KTILE / 8 / (NW * 64);  // chunks per thread per tile
    extern __shared__ __attribute__((aligned(16))) char smem[];
    bf16* lds = reinterpret_cast<bf16*>(smem);  // [stages][K tile | V^T tile]

    const TileItem it = qtiles[blockIdx.x];
    const BlockMeta bm = meta[it.block];
    const int t = threadIdx.x, lane = t & 63;
    const int wave = t >> 6;
    const int grp = PP ? wave >> 2 : 0, wq = wave & 3;   // head of the pair, 32-row slice of the query tile
    const int head = PP ? blockIdx.y * 2 + grp : blockIdx.y;
    const int kvh = (PP ? blockIdx.y * 2 : blockIdx.y) / (Hq / Hkv);   // the pair shares it (even GQA group)
    const int r = lane & 31, h = lane >> 5;
    const int ld = (Hq + 2 * Hkv) * HD;
    const int len = bm.prior + bm.len;   // cache rows once this call's rows are in
    const int prior = bm.prior;          // query row i of the call is cache row prior + i

    const bf16* kslab = kbase + bm.slab + (size_t)kvh * bm.capacity * HD;
    const bf16* vslab = vbase + bm.slab + (size_t)kvh * HD * bm.capacity;

    // ---- Q^T operand: lane (q = r, h) holds Q[q][kk*16 + h*8 .. +7] -----------
    const int qrow = prior + it.row0 + wq * 32 + r;   // as a cache row
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
    const int q_hi_wave = prior + it.row0 + wq * 32 + 31;                // last query row of this wave
    const int q_lo_wave = prior + it.row0 + wq * 32;                     // first query row of this wave
    const int n_tiles = q_hi_wg / KV_TILE + 1;

    // ---- staging: 16-byte global loads that land in LDS directly ---------------------
    // A wave-instruction fills 64 consecutive 16-byte chunks of a tile; chunk L of the K tile is
    // (row L / KCH, position L % KCH) and holds the row's chunk (L % KCH) ^ swz(row), chunk L of the
    // V^T tile likewise with 8 chunks per row: each lane picks the global address that belongs in
    // its slot.  Wavefront w issues instructions w, w + NW, ...; nothing passes through registers.
    // Two flavours, chosen by what measured faster: the four-wavefront kernel addresses the slabs through
    // buffer descriptors (32-bit offsets, no 64-bit per-lane pointers: 60 registers fewer, which at head_dim 64
    // buys a third workgroup per CU); the ping-pong kernel has the registers anyway and ran 5 % slower with them,
    // so it keeps per-lane global pointers.
    constexpr bool BUF = !PP;
    unsigned koff[NLD], voff[NLD];   // element offsets inside a tile's source rows, fixed per lane
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
        const int L = (i * NW + wave) * 64 + lane;
        const int krow = L / KCH, kc = (L % KCH) ^ swz<KCH>(krow);
        koff[i] = (unsigned)(krow * HD + kc * 8);
        const int vrow = L >> 3, vc = (L & 7) ^ swz<8>(vrow);
        voff[i] = (unsigned)(vrow * bm.capacity + vc * 8);
    }
    const unsigned slab_bytes = (unsigned)bm.capacity * HD * 2u;   // one KV head's K slab, and its V^T slab
    const __amdgpu_buffer_rsrc_t krsrc = raw_buffer(kslab, slab_bytes), vrsrc = raw_buffer(vslab, slab_bytes);
    auto issue_tile = [&](int kt, int stage) {
        const int kv0 = kt * KV_TILE;
        bf16* ks = lds + stage * 2 * KTILE;
        bf16* vs = ks + KTILE;
        if constexpr (BUF) {
            const unsigned kt_off = (unsigned)kv0 * HD * 2u, vt_off = (unsigned)kv0 * 2u;
            if (kv0 + KV_TILE <= len) {   // the whole tile lies inside the cache: tile offset as scalar offset
#pragma unroll
                for (int i = 0; i < NLD; ++i) {
                    buf_load16_to_lds(krsrc, ks + (i * NW + wave) * 64 * 8, koff[i] * 2u, kt_off);
                    buf_load16_to_lds(vrsrc, vs + (i * NW + wave) * 64 * 8, voff[i] * 2u, vt_off);
                }
            } else {
                // last tile of the block: the tile offset goes through the range check, so K rows and V^T
                // columns past the slab read zeros; rows past the block's end inside the slab read whatever
                // is there (their scores are masked, their V^T columns are zeroed by fix_tail)
#pragma unroll
                for (int i = 0; i < NLD; ++i) {
                    buf_load16_to_lds(krsrc, ks + (i * NW + wave) * 64 * 8, koff[i] * 2u + kt_off, 0);
                    buf_load16_to_lds(vrsrc, vs + (i * NW + wave) * 64 * 8, voff[i] * 2u + vt_off, 0);
                }
            }
        } else if (kv0 + KV_TILE <= len) {   // the whole tile lies inside the cache: no clamps
            const bf16* kt0 = kslab + (size_t)kv0 * HD;
            const bf16* vt0 = vslab + kv0;
#pragma unroll
            for (int i = 0; i < NLD; ++i) {
                load16_to_lds(kt0 + koff[i], ks + (i * NW + wave) * 64 * 8);
                load16_to_lds(vt0 + voff[i], vs + (i * NW + wave) * 64 * 8);
            }
        } else {   // last tile of the block: rows past the end are clamped (their scores are masked)
#pragma unroll
            for (int i = 0; i < NLD; ++i) {
                const int L = (i * NW + wave) * 64 + lane;
                const int krow = L / KCH, kc = (L % KCH) ^ swz<KCH>(krow);
                const int tok = min(kv0 + krow, len - 1);
                load16_to_lds(kslab + (size_t)tok * HD + kc * 8, ks + (i * NW + wave) * 64 * 8);
                const int vrow = L >> 3, vc = (L & 7) ^ swz<8>(vrow);
                const int vt = min(kv0 + vc * 8, bm.capacity - 8);
                load16_to_lds(vslab + (size_t)vrow * bm.capacity + vt, vs + (i * NW + wave) * 64 * 8);
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
            const int L = (i * NW + wave) * 64 + lane;
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

    // token of MFMA row i of S^T tile tt: tt*32 + pi(i); pi keeps each lane's
    // accumulator values of one k-step on 8 consecutive tokens
    const int pi_r = (r >> 4) * 16 + ((r >> 2) & 1) * 8 + ((r >> 3) & 1) * 4 + (r & 3);

    floatx16 sacc[2];   // S^T of the current tile: query column r, token kv0 + tt*32 + (e/8)*16 + h*8 + (e%8)
    bf16x8 pf[4];       // P^T of the current tile as the column operand of the second MFMA

    // ---- S^T = K Q^T ----------------------------------------------------
    auto qk = [&](const bf16* ks) {
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
    };
    // ---- online softmax of the tile: sacc -> pf.  `diag` (wavefront-uniform) is set only for tiles
    // that straddle the wavefront's diagonal, so the tiles below it carry no compare/select.
    auto softmax = [&](bool diag, int kv0) {
        if (__builtin_amdgcn_readfirstlane((int)diag)) {
#pragma unroll
            for (int tt = 0; tt < 2; ++tt)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int tok = kv0 + tt * 32 + (e >> 3) * 16 + h * 8 + (e & 7);
                    if (tok > qrow) sacc[tt][e] = -INFINITY;
                }
        }
        // The running maximum is only a scaling reference.  The common case takes the probabilities
        // against the reference as it stands and looks at nothing but their sum: while every lane's
        // sum of its 32 values stays below 2^12, fp32 sums and bf16 probabilities carry them without
        // loss and the tile's maximum is never formed.  Otherwise (always on the first tile, whose
        // reference is -inf: the sum comes out inf or NaN) the exact maximum is taken, the reference
        // moves there, the accumulators are rescaled and the probabilities are formed again.
        auto probs = [&]() {
            const float neg_m = -m_run;
            float ps = 0.f;
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
            return ps;
        };
        float ps = probs();
        // (query columns past the block's end see unmasked cache rows past it -- whatever the slab holds --
        // and must not take part in the decision: a row's bits may depend on its own block only)
        if (__any(!(ps < 4096.0f) && qrow < len)) {
            float mx = -INFINITY;
#pragma unroll
            for (int tt = 0; tt < 2; ++tt)
#pragma unroll
                for (int e = 0; e < 16; ++e) mx = fmaxf(mx, sacc[tt][e]);
            mx = fmaxf(mx, __shfl_xor(mx, 32, 64)) * scale_log2;
            const float m_new = fmaxf(m_run, mx);   // finite: tile 0 holds token 0 <= every query row
            const float corr = __builtin_amdgcn_exp2f(m_run - m_new);
            l_run *= corr;
            m_run = m_new;
#pragma unroll
            for (int d = 0; d < DT; ++d)
#pragma unroll
                for (int e = 0; e < 16; ++e) oacc[d][e] *= corr;
            ps = probs();
        }
        l_run += ps;
    };
    // ---- O^T += V^T P^T ---------------------------------------------------
    auto pv_mm = [&](const bf16* vs) {
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
    // Matrix phase of the ping-pong loop: PV of the previous tile, then QK^T of this one, as ONE stream of
    // 4 DT + 2 KK operand reads and as many MFMAs.  The other wavefront on this SIMD issues no MFMA in the
    // meantime, so nothing hides an LDS round trip: the reads run AHEAD fragments ahead of the MFMAs (pinned).
    auto pv_qk = [&](const bf16* vs, const bf16* ks) {
        constexpr int NV = 4 * DT, NK = 2 * KK, AHEAD = 6;
        bf16x8 fr[NV + NK];
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int d = 0; d < DT; ++d) {
                const int row = d * 32 + r;
                fr[u * DT + d] = *reinterpret_cast<const bf16x8*>(vs + row * KV_TILE + (((u * 2 + h) ^ swz<8>(row)) << 3));
            }
#pragma unroll
        for (int kk = 0; kk < KK; ++kk)
#pragma unroll
            for (int tt = 0; tt < 2; ++tt) {
                const int row = tt * 32 + pi_r;
                fr[NV + kk * 2 + tt] = *reinterpret_cast<const bf16x8*>(ks + row * HD + (((kk * 2 + h) ^ swz<KCH>(row)) << 3));
            }
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int d = 0; d < DT; ++d) oacc[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[u * DT + d], pf[u], oacc[d], 0, 0, 0);
#pragma unroll
        for (int tt = 0; tt < 2; ++tt)
#pragma unroll
            for (int e = 0; e < 16; ++e) sacc[tt][e] = 0.f;
#pragma unroll
        for (int kk = 0; kk < KK; ++kk)
#pragma unroll
            for (int tt = 0; tt < 2; ++tt)
                sacc[tt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[NV + kk * 2 + tt], qf[kk], sacc[tt], 0, 0, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, AHEAD, 0);   // LDS reads
#pragma unroll
        for (int i = 0; i < NV + NK - AHEAD; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // one MFMA
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // one LDS read
        }
        __builtin_amdgcn_sched_group_barrier(0x008, AHEAD, 0);
    };
    // a tile wholly above this wavefront's diagonal is skipped; `diag`: some entry of it may be masked
    auto active = [&](int kt) { return kt * KV_TILE <= q_hi_wave; };
    auto diag = [&](int kt) { return kt * KV_TILE + KV_TILE - 1 > q_lo_wave; };

    if constexpr (!PP) {
        issue_tile(0, 0);
        wait_all_memory();
        fix_tail(0, 0);
        __syncthreads();
        for (int kt = 0; kt < n_tiles; ++kt) {
            const bf16* ks = lds + (kt & 1) * 2 * KTILE;
            const bool more = kt + 1 < n_tiles;
            // the other stage was last read in the previous iteration, which every wavefront has left
            if (more) issue_tile(kt + 1, (kt + 1) & 1);
            if (active(kt)) {
                // head_dim 64: three wavefronts per SIMD compete; the one inside a run of MFMAs goes first
                // (measured +2 %; at head_dim 128, two wavefronts per SIMD, -2 %)
                constexpr int MM_PRIO = HD == 64 ? 3 : 0;
                __builtin_amdgcn_s_setprio(MM_PRIO);
                qk(ks);
                __builtin_amdgcn_s_setprio(0);
                softmax(diag(kt), kt * KV_TILE);
                __builtin_amdgcn_s_setprio(MM_PRIO);
                pv_mm(ks + KTILE);
                __builtin_amdgcn_s_setprio(0);
            }
            if (more) {
                wait_all_memory();
                fix_tail(kt + 1, (kt + 1) & 1);
            }
            __syncthreads();
        }
    } else {
        // Phase 2j of a group: PV of tile j-1 and QK^T of tile j ("matrix phase"); phase 2j+1: softmax
        // of tile j.  Group 0 runs phase s in time slot s, group 1 in slot s + 1; slots are separated by
        // workgroup barriers, and every wavefront passes the same number of them (2 n_tiles + 3).
        // Tile T is read in slots 2T .. 2T+3 (K by both groups, then V^T by both) and its stage is free
        // again from slot 2T+4 on.  The staging rides in the softmax phases, which are the shorter ones
        // and read no LDS (while a load that writes LDS is pending, the compiler turns every wait for
        // an LDS read into a wait for all of them): in its softmax phase j, group g first waits for its
        // part of tile j+1+g, issued one softmax phase earlier, then issues its part of tile j+2+g.
        // Group 0 thus confirms tile T in slot 2T-1 and group 1 in slot 2T-2, before the barrier that
        // precedes the first read; the stage of tile j+2+g was last read in slot 2j-1+2g.
        issue_tile(0, 0);
        if (n_tiles > 1) issue_tile(1, 1);
        if (grp == 1) {   // group 1 runs one tile ahead with its loads
            if (n_tiles > 2) {
                issue_tile(2, 2);
                wait_vm<2 * NLD>();
            } else {
                wait_vm<0>();
            }
            fix_tail(0, 0);
            if (n_tiles > 1) fix_tail(1, 1);
        } else {
            if (n_tiles > 1)
                wait_vm<2 * NLD>();
            else
                wait_vm<0>();
            fix_tail(0, 0);
        }
        phase_barrier();
        if (grp == 1) phase_barrier();
        for (int kt = 0; kt <= n_tiles; ++kt) {
            const bool do_pv = kt > 0 && active(kt - 1), do_qk = kt < n_tiles && active(kt);
            __builtin_amdgcn_s_setprio(3);   // the matrix phase is the one the slot waits for
            if (do_pv && do_qk) {
                pv_qk(lds + ((kt - 1) & 3) * 2 * KTILE + KTILE, lds + (kt & 3) * 2 * KTILE);
            } else {
                if (do_pv) pv_mm(lds + ((kt - 1) & 3) * 2 * KTILE + KTILE);
                if (do_qk) qk(lds + (kt & 3) * 2 * KTILE);
            }
            __builtin_amdgcn_s_setprio(0);
            phase_barrier();
            if (kt == n_tiles) break;
            if (active(kt)) softmax(diag(kt), kt * KV_TILE);
            const int t_wait = kt + 1 + grp, t_issue = kt + 2 + grp;
            if (t_wait < n_tiles) {
                wait_vm<0>();
                fix_tail(t_wait, t_wait & 3);
            }
            if (t_issue < n_tiles) issue_tile(t_issue, t_issue & 3);
            phase_barrier();
        }
        if (grp == 0) phase_barrier();
        wait_vm<0>();
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

template <int HD, bool PP>
static int launch_prefill_variant(compact_ctx* ctx, const BlockMeta* d_meta, const TileItem* d_qtiles, int n_qtiles,
                                  const bf16* qkv, const bf16* d_k, const bf16* d_v, bf16* o, float scale_log2, hipStream_t s) {
    const compact_layer_cfg& c = ctx->cfg;
    auto kern = attn_prefill_bf16_kernel<HD, PP>;
    const size_t smem = (size_t)(PP ? 4 : 2) * 2 * KV_TILE * HD * sizeof(bf16);
    static bool attr_set = false;
    if (!attr_set) {
        HIP_TRY(ctx, hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
        attr_set = true;
    }
    dim3 grid(n_qtiles, PP ? c.n_q_heads / 2 : c.n_q_heads);
    kern<<<grid, PP ? 512 : 256, smem, s>>>(d_meta, d_qtiles, qkv, d_k, d_v, o, c.n_q_heads, c.n_kv_heads, scale_log2);
    LAUNCH_CHECK(ctx);
    return COMPACT_OK;
}

int launch_attn_prefill_bf16(compact_ctx* ctx, const BlockMeta* d_meta, const TileItem* d_qtiles, int n_qtiles,
                             const bf16* qkv, const bf16* d_k, const bf16* d_v, bf16* o, hipStream_t s) {
    if (n_qtiles == 0) return COMPACT_OK;
    const compact_layer_cfg& c = ctx->cfg;
    const float scale_log2 = LOG2E / sqrtf((float)c.head_dim);
    // two query heads of one KV head per workgroup whenever the GQA group is even
    const bool pair = (c.n_q_heads / c.n_kv_heads) % 2 == 0;
    if (c.head_dim == 128)
        return pair ? launch_prefill_variant<128, true>(ctx, d_meta, d_qtiles, n_qtiles, qkv, d_k, d_v, o, scale_log2, s)
                    : launch_prefill_variant<128, false>(ctx, d_meta, d_qtiles, n_qtiles, qkv, d_k, d_v, o, scale_log2, s);
    // head_dim 64 halves the matrix phase but not the softmax: the phases no longer balance (measured 31 % against
    // 38 % of peak), so it stays with the four-wavefront kernel
    return launch_prefill_variant<64, false>(ctx, d_meta, d_qtiles, n_qtiles, qkv, d_k, d_v, o, scale_log2, s);
}
