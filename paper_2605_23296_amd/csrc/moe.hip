// Mixture-of-experts plumbing: top-k routing from fp32 logits, the
// token -> expert permutation (histogram, scan, scatter, row-tile map for the
// grouped GEMM) and the weighted un-permute + residual.
#include "common.h"
#include "vecio.h"

// ---------------------------------------------------------------------------
// top-k of E fp32 logits per row (descending, equal logits -> lower index),
// gate = softmax over the selected logits.  One wavefront per row; lane l owns
// experts l, l+64, l+128, l+192.
// ---------------------------------------------------------------------------
// ks > 0: the logits arrive as ks split-K partials [ks][rows][E]; they are summed in
// slice order here and the sums are written to `logits`.
__global__ __launch_bounds__(256) void topk_route_kernel(float* __restrict__ logits, const float* __restrict__ partials, int ks,
                                                         int64_t rows, int E, int k, int32_t* __restrict__ idx,
                                                         float* __restrict__ gate) {
    const int64_t row = (int64_t)blockIdx.x * 4 + threadIdx.x / WAVE;
    if (row >= rows) return;
    const int lane = threadIdx.x & (WAVE - 1);
    float v[4];
    if (ks > 0) {
        // all partials of the lane's experts are requested before the first is used (slices in groups of
        // 8), then added in slice order: the kernel is a few memory round trips long, not ks * 4
        float a[4] = {0.f, 0.f, 0.f, 0.f};
        for (int s0 = 0; s0 < ks; s0 += 8) {
            float pv[4][8];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int e = lane + i * 64;
                    pv[i][u] = (e < E && s0 + u < ks) ? partials[((size_t)(s0 + u) * rows + row) * E + e] : 0.f;
                }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int u = 0; u < 8; ++u)
                    if (s0 + u < ks) a[i] += pv[i][u];
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int e = lane + i * 64;
            v[i] = -INFINITY;
            if (e < E) {
                logits[row * E + e] = a[i];
                v[i] = a[i];
            }
        }
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int e = lane + i * 64;
            v[i] = e < E ? logits[row * E + e] : -INFINITY;
        }
    }
    float sel_v[8];
    int sel_i[8];
    for (int j = 0; j < k; ++j) {
        // lane-local best (lower index wins ties: scan in increasing index order with strict >)
        float bv = v[0];
        int bi = lane;
#pragma unroll
        for (int i = 1; i < 4; ++i)
            if (v[i] > bv) {
                bv = v[i];
                bi = lane + i * 64;
            }
        // wavefront arg-max on (value desc, index asc)
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            const float ov = __shfl_xor(bv, o, 64);
            const int oi = __shfl_xor(bi, o, 64);
            if (ov > bv || (ov == bv && oi < bi)) {
                bv = ov;
                bi = oi;
            }
        }
        sel_v[j] = bv;
        sel_i[j] = bi;
        if ((bi & 63) == lane) v[bi >> 6] = -INFINITY;  // remove the winner
    }
    if (lane == 0) {
        float den = 0.f;
        float p[8];
        for (int j = 0; j < k; ++j) {
            p[j] = expf(sel_v[j] - sel_v[0]);
            den += p[j];
        }
        for (int j = 0; j < k; ++j) {
            idx[row * k + j] = sel_i[j];
            gate[row * k + j] = p[j] / den;
        }
    }
}

int launch_moe_route(compact_ctx* ctx, const void* m, const void* w_router, int64_t rows, int32_t* idx, float* gate,
                     float* logits, hipStream_t s, float* partials_ws) {
    if (rows == 0) return COMPACT_OK;
    const compact_layer_cfg& c = ctx->cfg;
    int rc;
    if (c.dtype == COMPACT_BF16 && partials_ws && rows <= 64 && c.n_experts % 16 == 0 && c.d_model % 64 == 0) {
        // a few decode rows: the router matrix is streamed once by the weight-streaming kernel
        const int ks = skinny_ksplit((int)rows, c.n_experts, c.d_model);
        rc = launch_gemm_skinny(ctx, (const bf16*)m, (const bf16*)w_router, partials_ws, (int)rows, c.n_experts, c.d_model, ks, s);
        if (rc != COMPACT_OK) return rc;
        topk_route_kernel<<<(unsigned)((rows + 3) / 4), 256, 0, s>>>(logits, partials_ws, ks, rows, c.n_experts, c.top_k, idx, gate);
        LAUNCH_CHECK(ctx);
        return COMPACT_OK;
    }
    if (c.dtype == COMPACT_BF16)
        rc = launch_gemm_bf16(ctx, (const bf16*)m, (const bf16*)w_router, nullptr, false, (bf16*)logits, rows,
                              c.n_experts, c.d_model, 2, nullptr, s);
    else
        rc = launch_gemm_f32(ctx, (const float*)m, (const float*)w_router, nullptr, logits, rows, c.n_experts,
                             c.d_model, 0, nullptr, s);
    if (rc != COMPACT_OK) return rc;
    topk_route_kernel<<<(unsigned)((rows + 3) / 4), 256, 0, s>>>(logits, nullptr, 0, rows, c.n_experts, c.top_k, idx, gate);
    LAUNCH_CHECK(ctx);
    return COMPACT_OK;
}

// ---------------------------------------------------------------------------
// permutation plan
// ---------------------------------------------------------------------------
__global__ void zero_i32_kernel(int32_t* p, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0;
}

// rank[i] = position of entry i among the entries routed to the same expert
// (any order: the order of rows inside an expert's group does not enter the
// arithmetic).  Workgroup-local ranks from an LDS histogram, one global
// reservation per (workgroup, expert).
__global__ __launch_bounds__(256) void expert_rank_kernel(const int32_t* __restrict__ idx, int64_t n, int E,
                                                          int32_t* __restrict__ counts, int32_t* __restrict__ rank) {
    __shared__ int32_t lc[256], base[256];
    const int t = threadIdx.x;
    lc[t] = 0;
    __syncthreads();
    constexpr int PER = 4;
    int e[PER], lr[PER];
    const int64_t i0 = ((int64_t)blockIdx.x * 256 + t) * PER;
#pragma unroll
    for (int j = 0; j < PER; ++j) {
        e[j] = -1;
        if (i0 + j < n) {
            e[j] = idx[i0 + j];
            lr[j] = atomicAdd(&lc[e[j]], 1);
        }
    }
    __syncthreads();
    if (t < E && lc[t] > 0) base[t] = atomicAdd(&counts[t], lc[t]);
    __syncthreads();
#pragma unroll
    for (int j = 0; j < PER; ++j)
        if (e[j] >= 0) rank[i0 + j] = base[e[j]] + lr[j];
}

// offsets = exclusive scan of counts; row-tile map for the grouped GEMM
__global__ __launch_bounds__(256) void expert_scan_kernel(const int32_t* __restrict__ counts, int E, int mtile,
                                                          int32_t* __restrict__ offsets, int32_t* __restrict__ tile_expert,
                                                          int32_t* __restrict__ tile_row0, int32_t* __restrict__ tile_rows,
                                                          int max_mtiles) {
    __shared__ int32_t off[257], toff[257];
    if (threadIdx.x == 0) {
        int a = 0, b = 0;
        for (int e = 0; e < E; ++e) {
            off[e] = a;
            toff[e] = b;
            a += counts[e];
            b += (counts[e] + mtile - 1) / mtile;
        }
        off[E] = a;
        toff[E] = b;
    }
    __syncthreads();
    for (int e = threadIdx.x; e <= E; e += 256) offsets[e] = off[e];
    for (int e = threadIdx.x; e < E; e += 256) {
        const int cnt = off[e + 1] - off[e];
        for (int i = 0; toff[e] + i < toff[e + 1]; ++i) {
            const int ti = toff[e] + i;
            tile_expert[ti] = e;
            tile_row0[ti] = off[e] + i * mtile;
            tile_rows[ti] = min(mtile, cnt - i * mtile);
        }
    }
    for (int ti = toff[E] + threadIdx.x; ti < max_mtiles; ti += 256) {
        tile_expert[ti] = -1;
        tile_row0[ti] = 0;
        tile_rows[ti] = 0;
    }
}

__global__ __launch_bounds__(256) void expert_scatter_kernel(const int32_t* __restrict__ idx, const float* __restrict__ gate,
                                                             const int32_t* rank,
                                                             const int32_t* __restrict__ offsets, int64_t n, int k,
                                                             int32_t* __restrict__ sorted_token,
                                                             float* __restrict__ sorted_gate, int32_t* slot_of) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    const int pos = offsets[idx[i]] + rank[i];
    sorted_token[pos] = (int32_t)(i / k);
    sorted_gate[pos] = gate[i];
    slot_of[i] = pos;
}

// The whole plan in one workgroup, for at most 256 routed entries (a decode step) and
// at most 256 experts: rank = number of earlier entries with the same expert (so the
// order inside an expert's group is the token order), counts, scan, tile map, scatter.
__global__ __launch_bounds__(256) void moe_plan_small_kernel(const int32_t* __restrict__ idx, const float* __restrict__ gate,
                                                             int n, int k, int E, int mtile, int32_t* __restrict__ counts,
                                                             int32_t* __restrict__ offsets, int32_t* __restrict__ tile_expert,
                                                             int32_t* __restrict__ tile_row0, int32_t* __restrict__ tile_rows,
                                                             int max_mtiles, int32_t* __restrict__ sorted_token,
                                                             float* __restrict__ sorted_gate, int32_t* __restrict__ slot_of) {
    __shared__ int32_t se[256], off[257], toff[257];
    const int t = threadIdx.x;
    const int my = t < n ? idx[t] : -1;
    se[t] = my;
    __syncthreads();
    int rank = 0;
    for (int j = 0; j < t; ++j) rank += (se[j] == my) ? 1 : 0;
    int cnt = 0;
    if (t < E) {
        for (int j = 0; j < n; ++j) cnt += (se[j] == t) ? 1 : 0;
        counts[t] = cnt;
    }
    __syncthreads();
    // exclusive scans of the counts and of the tiles per expert over the 256 threads
    // (thread e = expert e; Hillis-Steele in LDS, integer sums: any order gives the same result)
    const int tiles = (cnt + mtile - 1) / mtile;
    off[t + 1] = cnt;
    toff[t + 1] = tiles;
    if (t == 0) off[0] = toff[0] = 0;
    __syncthreads();
    for (int st = 1; st < 256; st <<= 1) {
        const int a = t + 1 > st ? off[t + 1 - st] : 0;
        const int b = t + 1 > st ? toff[t + 1 - st] : 0;
        __syncthreads();
        off[t + 1] += a;
        toff[t + 1] += b;
        __syncthreads();
    }
    for (int e = t; e <= E; e += 256) offsets[e] = off[e];
    if (t < E) {
        for (int i = 0; toff[t] + i < toff[t + 1]; ++i) {
            const int ti = toff[t] + i;
            tile_expert[ti] = t;
            tile_row0[ti] = off[t] + i * mtile;
            tile_rows[ti] = min(mtile, cnt - i * mtile);
        }
    }
    for (int ti = toff[E] + t; ti < max_mtiles; ti += 256) {
        tile_expert[ti] = -1;
        tile_row0[ti] = 0;
        tile_rows[ti] = 0;
    }
    if (my >= 0) {
        const int pos = off[my] + rank;
        sorted_token[pos] = t / k;
        sorted_gate[pos] = gate[t];
        slot_of[t] = pos;
    }
}

int launch_moe_plan(compact_ctx* ctx, const int32_t* idx, const float* gate, int64_t rows, int mtile,
                    const MoePlan& plan, hipStream_t s) {
    const compact_layer_cfg& c = ctx->cfg;
    const int64_t n = rows * c.top_k;
    if (n == 0) return COMPACT_OK;
    if (n <= 256 && c.n_experts <= 256) {
        moe_plan_small_kernel<<<1, 256, 0, s>>>(idx, gate, (int)n, c.top_k, c.n_experts, mtile, plan.counts, plan.offsets,
                                                plan.tile_expert, plan.tile_row0, plan.tile_rows, plan.max_mtiles,
                                                plan.sorted_token, plan.sorted_gate, plan.slot_of);
        LAUNCH_CHECK(ctx);
        return COMPACT_OK;
    }
    zero_i32_kernel<<<1, 256, 0, s>>>(plan.counts, c.n_experts);
    // slot_of doubles as the rank buffer until the scatter overwrites it entry by entry
    expert_rank_kernel<<<(unsigned)((n + 1023) / 1024), 256, 0, s>>>(idx, n, c.n_experts, plan.counts, plan.slot_of);
    expert_scan_kernel<<<1, 256, 0, s>>>(plan.counts, c.n_experts, mtile, plan.offsets, plan.tile_expert, plan.tile_row0,
                                         plan.tile_rows, plan.max_mtiles);
    expert_scatter_kernel<<<(unsigned)((n + 255) / 256), 256, 0, s>>>(idx, gate, plan.slot_of, plan.offsets, n, c.top_k,
                                                                      plan.sorted_token, plan.sorted_gate, plan.slot_of);
    LAUNCH_CHECK(ctx);
    return COMPACT_OK;
}

// ---------------------------------------------------------------------------
// y[t] = h[t] + sum_j expert_out[slot_of[t*k + j]]   (rows already gate-scaled)
// ---------------------------------------------------------------------------
template <typename T, typename HT>
__global__ __launch_bounds__(256) void moe_combine_kernel(const T* __restrict__ expert_out, const HT* __restrict__ hres,
                                                          const int32_t* __restrict__ slot_of, int k, int d,
                                                          T* __restrict__ y) {
    const int64_t row = blockIdx.x;
    for (int c = threadIdx.x * 8; c < d; c += 256 * 8) {
        float acc[8];
        load8(hres + row * d + c, acc);
        for (int j = 0; j < k; ++j) {
            float v[8];
            load8(expert_out + (int64_t)slot_of[row * k + j] * d + c, v);
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[e] += v[e];
        }
        store8(y + row * d + c, acc);
    }
}

int launch_moe_combine(compact_ctx* ctx, const void* expert_out, const void* h, bool h_is_f32, const int32_t* slot_of,
                       int64_t rows, void* y, hipStream_t s) {
    if (rows == 0) return COMPACT_OK;
    const compact_layer_cfg& c = ctx->cfg;
    const unsigned g = (unsigned)rows;
    if (c.dtype == COMPACT_BF16 && h_is_f32)
        moe_combine_kernel<bf16, float><<<g, 256, 0, s>>>((const bf16*)expert_out, (const float*)h, slot_of, c.top_k, c.d_model, (bf16*)y);
    else if (c.dtype == COMPACT_BF16)
        moe_combine_kernel<bf16, bf16><<<g, 256, 0, s>>>((const bf16*)expert_out, (const bf16*)h, slot_of, c.top_k, c.d_model, (bf16*)y);
    else
        moe_combine_kernel<float, float><<<g, 256, 0, s>>>((const float*)expert_out, (const float*)h, slot_of, c.top_k, c.d_model, (float*)y);
    LAUNCH_CHECK(ctx);
    return COMPACT_OK;
}

// ---------------------------------------------------------------------------
// Decode: y[t] = h[t] + sum_j gate_j * (sum_s P[s][slot_of[t*k + j]]), with the
// split-K partials of the routed down projection still in fp32: one rounding.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void moe_combine_partials_kernel(const float* __restrict__ P, int ks, int64_t total_rows,
                                                                   const float* __restrict__ hres,
                                                                   const int32_t* __restrict__ slot_of,
                                                                   const float* __restrict__ sorted_gate, int k, int d,
                                                                   bf16* __restrict__ y) {
    const int64_t row = blockIdx.y;
    const int c = (blockIdx.x * 256 + threadIdx.x) * 4;
    if (c >= d) return;
    // the loads go out in three waves (all slots, then all gate weights, then per expert all its slices, 8 at a
    // time) instead of one after the other; the sums keep their order: slices in slice order, experts in j order
    constexpr int KMAX = 8;   // top_k <= 8
    int64_t slot[KMAX];
    float gw[KMAX];
#pragma unroll
    for (int j = 0; j < KMAX; ++j) slot[j] = slot_of[row * k + min(j, k - 1)];
#pragma unroll
    for (int j = 0; j < KMAX; ++j) gw[j] = sorted_gate[slot[j]];
    float4 acc = *reinterpret_cast<const float4*>(hres + row * d + c);
#pragma unroll
    for (int j = 0; j < KMAX; ++j) {
        if (j >= k) break;
        float4 e = make_float4(0.f, 0.f, 0.f, 0.f);
        for (int s0 = 0; s0 < ks; s0 += 8) {
            float4 v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u)
                v[u] = *reinterpret_cast<const float4*>(P + ((int64_t)min(s0 + u, ks - 1) * total_rows + slot[j]) * d + c);
#pragma unroll
            for (int u = 0; u < 8; ++u)
                if (s0 + u < ks) { e.x += v[u].x; e.y += v[u].y; e.z += v[u].z; e.w += v[u].w; }
        }
        acc.x += gw[j] * e.x; acc.y += gw[j] * e.y; acc.z += gw[j] * e.z; acc.w += gw[j] * e.w;
    }
    bf16x4 o;
    o[0] = (bf16)acc.x; o[1] = (bf16)acc.y; o[2] = (bf16)acc.z; o[3] = (bf16)acc.w;
    *reinterpret_cast<bf16x4*>(y + row * d + c) = o;
}

int launch_moe_combine_partials(compact_ctx* ctx, const float* partials, int ks, int64_t total_rows, const float* h,
                                const int32_t* slot_of, const float* sorted_gate, int64_t rows, void* y, hipStream_t s) {
    if (rows == 0) return COMPACT_OK;
    const compact_layer_cfg& c = ctx->cfg;
    dim3 grid((c.d_model / 4 + 255) / 256, (unsigned)rows);
    moe_combine_partials_kernel<<<grid, 256, 0, s>>>(partials, ks, total_rows, h, slot_of, sorted_gate, c.top_k, c.d_model,
                                                     (bf16*)y);
    LAUNCH_CHECK(ctx);
    return COMPACT_OK;
}
