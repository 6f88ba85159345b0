// RMSNorm, rotary embedding + KV-cache write, and the row epilogues of the
// decode step.  All of these are bandwidth-bound row kernels: 16-byte loads,
// fp32 arithmetic, one workgroup per row (or per 64-token tile).
#include "common.h"
#include "vecio.h"

#define NT 256

// sum over the workgroup; every thread gets the result
__device__ __forceinline__ float block_sum(float v, float* red) {
    v = wave_sum(v);
    const int w = threadIdx.x / WAVE;
    __syncthreads();
    if ((threadIdx.x & (WAVE - 1)) == 0) red[w] = v;
    __syncthreads();
    float t = 0.f;
#pragma unroll
    for (int i = 0; i < NT / WAVE; ++i) t += red[i];
    return t;
}

// ---------------------------------------------------------------------------
// y = x / sqrt(mean(x^2) + eps) * g
// ---------------------------------------------------------------------------
template <typename TI, typename T>
__global__ __launch_bounds__(NT) void rmsnorm_kernel(const TI* __restrict__ x, const T* __restrict__ g,
                                                     T* __restrict__ y, int d, float eps) {
    __shared__ float red[NT / WAVE];
    const TI* xr = x + (size_t)blockIdx.x * d;
    T* yr = y + (size_t)blockIdx.x * d;
    float ss = 0.f;
    for (int c = threadIdx.x * 8; c < d; c += NT * 8) {
        float v[8];
        load8(xr + c, v);
#pragma unroll
        for (int j = 0; j < 8; ++j) ss += v[j] * v[j];
    }
    ss = block_sum(ss, red);
    const float inv = 1.0f / sqrtf(ss / (float)d + eps);
    for (int c = threadIdx.x * 8; c < d; c += NT * 8) {
        float v[8], gv[8];
        load8(xr + c, v);
        load8(g + c, gv);
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = v[j] * inv * gv[j];
        store8(yr + c, v);
    }
}

int launch_rmsnorm(compact_ctx* ctx, const void* x, bool x_is_f32, const void* g, void* y, int64_t rows, hipStream_t s) {
    if (rows == 0) return COMPACT_OK;
    const int d = ctx->cfg.d_model;
    const dim3 grid((unsigned)rows);
    if (ctx->cfg.dtype == COMPACT_BF16 && x_is_f32)
        rmsnorm_kernel<float, bf16><<<grid, NT, 0, s>>>((const float*)x, (const bf16*)g, (bf16*)y, d, ctx->cfg.rms_eps);
    else if (ctx->cfg.dtype == COMPACT_BF16)
        rmsnorm_kernel<bf16, bf16><<<grid, NT, 0, s>>>((const bf16*)x, (const bf16*)g, (bf16*)y, d, ctx->cfg.rms_eps);
    else
        rmsnorm_kernel<float, float><<<grid, NT, 0, s>>>((const float*)x, (const float*)g, (float*)y, d, ctx->cfg.rms_eps);
    LAUNCH_CHECK(ctx);
    return COMPACT_OK;
}

// ---------------------------------------------------------------------------
// Rotary embedding of q and k for a 64-token tile of one block, K rows to the
// K slab, V rows transposed to the V slab.  The rotation angle is formed in
// fp64 (position * theta^(-2i/hd)) so that positions in the thousands do not
// cost fp32 angle precision; cos/sin are then used as fp32.
// ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(NT) void rope_kvwrite_kernel(const BlockMeta* __restrict__ meta,
                                                          const TileItem* __restrict__ tiles, T* __restrict__ qkv,
                                                          T* __restrict__ kbase, T* __restrict__ vbase, int Hq, int Hkv,
                                                          int hd, double log2_theta) {
    extern __shared__ char smem[];
    const int half = hd / 2;
    float2* cs = reinterpret_cast<float2*>(smem);                       // [ROPE_TILE][half]
    T* vt = reinterpret_cast<T*>(smem + (size_t)ROPE_TILE * half * 8);  // [ROPE_TILE][hd + 8]
    const int vld = hd + 8;

    const TileItem it = tiles[blockIdx.x];
    const BlockMeta bm = meta[it.block];
    const int p0 = it.row0;
    const int ntok = min(ROPE_TILE, bm.len - p0);
    const int ld = (Hq + 2 * Hkv) * hd;
    T* rows = qkv + (size_t)(bm.row0 + p0) * ld;

    for (int idx = threadIdx.x; idx < ntok * half; idx += NT) {
        const int tok = idx / half, i = idx - tok * half;
        const double inv_freq = exp2(-2.0 * (double)i / (double)hd * log2_theta);
        const double ang = (double)(bm.pos_offset + bm.prior + p0 + tok) * inv_freq;
        double sn, cn;
        sincos(ang, &sn, &cn);
        cs[idx] = make_float2((float)cn, (float)sn);
    }
    __syncthreads();

    // q heads (in place) and k heads (to the slab)
    const int chunks = half / 8;
    const int per_tok = (Hq + Hkv) * chunks;
    T* kslab = kbase + bm.slab;
    for (int idx = threadIdx.x; idx < ntok * per_tok; idx += NT) {
        const int tok = idx / per_tok;
        const int r = idx - tok * per_tok;
        const int head = r / chunks, c = r - head * chunks;
        T* src = rows + (size_t)tok * ld + head * hd + c * 8;
        float lo[8], hi[8], olo[8], ohi[8];
        load8(src, lo);
        load8(src + half, hi);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const float2 t = cs[tok * half + c * 8 + j];
            olo[j] = lo[j] * t.x - hi[j] * t.y;
            ohi[j] = hi[j] * t.x + lo[j] * t.y;
        }
        T* dst = src;
        if (head >= Hq) dst = kslab + ((size_t)(head - Hq) * bm.capacity + bm.prior + p0 + tok) * hd + c * 8;
        store8(dst, olo);
        store8(dst + half, ohi);
    }

    // v heads: stage [tok][hd] in LDS, write [hd][tok]
    T* vslab = vbase + bm.slab;
    for (int kvh = 0; kvh < Hkv; ++kvh) {
        __syncthreads();
        for (int idx = threadIdx.x; idx < ntok * (hd / 8); idx += NT) {
            const int tok = idx / (hd / 8), c = idx - tok * (hd / 8);
            const T* src = rows + (size_t)tok * ld + (Hq + Hkv + kvh) * hd + c * 8;
            float v[8];
            load8(src, v);
#pragma unroll
            for (int j = 0; j < 8; ++j) vt[tok * vld + c * 8 + j] = from_f32<T>(v[j]);
        }
        __syncthreads();
        for (int idx = threadIdx.x; idx < hd * (ROPE_TILE / 8); idx += NT) {
            const int dd = idx / (ROPE_TILE / 8), c = idx - dd * (ROPE_TILE / 8);
            const int t0 = c * 8;
            if (t0 >= ntok) continue;
            T* dst = vslab + ((size_t)kvh * hd + dd) * bm.capacity + bm.prior + p0 + t0;
            if (t0 + 8 <= ntok && (bm.prior & 7) == 0) {   // 16-byte stores need an aligned cache row
                float v[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) v[j] = to_f32(vt[(t0 + j) * vld + dd]);
                store8(dst, v);
            } else {
                for (int j = 0; t0 + j < ntok; ++j) dst[j] = vt[(t0 + j) * vld + dd];
            }
        }
    }
}

int launch_rope_kvwrite(compact_ctx* ctx, const BlockMeta* d_meta, const TileItem* d_tiles, int n_tiles, void* qkv,
                        void* d_k, void* d_v, hipStream_t s) {
    if (n_tiles == 0) return COMPACT_OK;
    const compact_layer_cfg& c = ctx->cfg;
    const double l2t = log2((double)c.rope_theta);
    const size_t es = dtype_size(c.dtype);
    const size_t smem = (size_t)ROPE_TILE * (c.head_dim / 2) * 8 + (size_t)ROPE_TILE * (c.head_dim + 8) * es;
    if (c.dtype == COMPACT_BF16)
        rope_kvwrite_kernel<bf16><<<n_tiles, NT, smem, s>>>(d_meta, d_tiles, (bf16*)qkv, (bf16*)d_k, (bf16*)d_v,
                                                           c.n_q_heads, c.n_kv_heads, c.head_dim, l2t);
    else
        rope_kvwrite_kernel<float><<<n_tiles, NT, smem, s>>>(d_meta, d_tiles, (float*)qkv, (float*)d_k, (float*)d_v,
                                                            c.n_q_heads, c.n_kv_heads, c.head_dim, l2t);
    LAUNCH_CHECK(ctx);
    return COMPACT_OK;
}

// ---------------------------------------------------------------------------
// Decode row epilogues.  The weight-streaming GEMM leaves ks split-K partials
// [ks][rows][cols] in fp32; these kernels sum them in slice order (all slice
// loads of a thread are issued together) and apply the step that follows.
// ---------------------------------------------------------------------------

// One workgroup (one wavefront) per (head, block token): q heads and k heads are
// rotated at position pos_offset + len + step, q goes to q_out, the K row and
// the V column are appended at cache row len + step.
template <typename T, int KS_UNROLL>
__global__ __launch_bounds__(64) void decode_qkv_epilogue_kernel(const BlockMeta* __restrict__ meta, int n_rows, int step,
                                                                const float* __restrict__ partials, int ks,
                                                                T* __restrict__ q_out, T* __restrict__ kbase,
                                                                T* __restrict__ vbase, int Hq, int Hkv, int hd,
                                                                double log2_theta, const RowNorm norm) {
    const int head = blockIdx.x, b = blockIdx.y;
    const int i = threadIdx.x;
    const int half = hd / 2;
    if (i >= half) return;
    const BlockMeta bm = meta[b];
    const int p = bm.len + step;
    const int ld = (Hq + 2 * Hkv) * hd;
    const size_t ps = (size_t)n_rows * ld;  // stride between split partials
    const float* row = partials + (size_t)b * ld + head * hd;
    float lo = 0.f, hi = 0.f;
    int s = 0;
    for (; s + KS_UNROLL <= ks; s += KS_UNROLL) {
        float a[KS_UNROLL], c[KS_UNROLL];
#pragma unroll
        for (int u = 0; u < KS_UNROLL; ++u) {
            a[u] = row[(s + u) * ps + i];
            c[u] = row[(s + u) * ps + half + i];
        }
#pragma unroll
        for (int u = 0; u < KS_UNROLL; ++u) {
            lo += a[u];
            hi += c[u];
        }
    }
    for (; s < ks; ++s) {
        lo += row[s * ps + i];
        hi += row[s * ps + half + i];
    }
    if (norm.ssq_parts) {
        float ss = 0.f;
        for (int pi = 0; pi < norm.nparts; ++pi) ss += norm.ssq_parts[(size_t)pi * n_rows + b];
        const float rinv = 1.0f / sqrtf(ss * norm.inv_d + norm.eps);
        lo *= rinv;
        hi *= rinv;
    }
    if (head < Hq + Hkv) {
        const double inv_freq = exp2(-2.0 * (double)i / (double)hd * log2_theta);
        double sn, cn;
        sincos((double)(bm.pos_offset + p) * inv_freq, &sn, &cn);
        const float cf = (float)cn, sf = (float)sn;
        const float olo = lo * cf - hi * sf;
        const float ohi = hi * cf + lo * sf;
        T* dst = head < Hq ? q_out + ((size_t)b * Hq + head) * hd + i
                           : kbase + bm.slab + ((size_t)(head - Hq) * bm.capacity + p) * hd + i;
        dst[0] = from_f32<T>(olo);
        dst[half] = from_f32<T>(ohi);
    } else {
        T* vcol = vbase + bm.slab + (size_t)(head - Hq - Hkv) * hd * bm.capacity + p;
        vcol[(size_t)i * bm.capacity] = from_f32<T>(lo);
        vcol[(size_t)(i + half) * bm.capacity] = from_f32<T>(hi);
    }
}

int launch_decode_qkv_epilogue(compact_ctx* ctx, const BlockMeta* d_meta, int n_blocks, int step, const float* partials,
                               int ks, void* q_out, void* d_k, void* d_v, hipStream_t s, const RowNorm* norm) {
    const compact_layer_cfg& c = ctx->cfg;
    const RowNorm rn = norm ? *norm : RowNorm{};
    const double l2t = log2((double)c.rope_theta);
    dim3 grid(c.n_q_heads + 2 * c.n_kv_heads, n_blocks);
    if (c.dtype == COMPACT_BF16)
        decode_qkv_epilogue_kernel<bf16, 8><<<grid, 64, 0, s>>>(d_meta, n_blocks, step, partials, ks, (bf16*)q_out,
                                                               (bf16*)d_k, (bf16*)d_v, c.n_q_heads, c.n_kv_heads,
                                                               c.head_dim, l2t, rn);
    else
        decode_qkv_epilogue_kernel<float, 1><<<grid, 64, 0, s>>>(d_meta, n_blocks, step, partials, ks, (float*)q_out,
                                                                (float*)d_k, (float*)d_v, c.n_q_heads, c.n_kv_heads,
                                                                c.head_dim, l2t, rn);
    LAUNCH_CHECK(ctx);
    return COMPACT_OK;
}

// sum of ks partial float4s at p, p + ps, ... in slice order, loads issued in groups of 8
__device__ __forceinline__ float4 sum_slices4(const float* __restrict__ p, size_t ps, int ks, float4 acc) {
    int s = 0;
    for (; s + 8 <= ks; s += 8) {
        float4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = *reinterpret_cast<const float4*>(p + (s + u) * ps);
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            acc.x += v[u].x; acc.y += v[u].y; acc.z += v[u].z; acc.w += v[u].w;
        }
    }
    for (; s < ks; ++s) {
        const float4 v = *reinterpret_cast<const float4*>(p + s * ps);
        acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
    }
    return acc;
}

// ---------------------------------------------------------------------------
// Decode: h = resid + sum_s partial_s (kept in fp32), m = RMSNorm(h; g).
// One workgroup per row, 4 columns per thread and trip (d <= RN_TRIPS * NT * 4 = 8192).
// ---------------------------------------------------------------------------
#define RN_TRIPS 8
template <typename T>
__global__ __launch_bounds__(NT) void residual_norm_kernel(const float* __restrict__ partials, int ks, int rows,
                                                           const T* __restrict__ resid, const T* __restrict__ g,
                                                           float* __restrict__ h_out, T* __restrict__ m_out, int d,
                                                           float eps) {
    __shared__ float red[NT / WAVE];
    const int r = blockIdx.x;
    const size_t ps = (size_t)rows * d;
    float4 hv[RN_TRIPS];
    float ss = 0.f;
#pragma unroll
    for (int it = 0; it < RN_TRIPS; ++it) {
        const int c = (it * NT + threadIdx.x) * 4;
        if (c < d) {
            const T* rp = resid + (size_t)r * d + c;
            float4 a = make_float4(to_f32(rp[0]), to_f32(rp[1]), to_f32(rp[2]), to_f32(rp[3]));
            a = sum_slices4(partials + (size_t)r * d + c, ps, ks, a);
            hv[it] = a;
            *reinterpret_cast<float4*>(h_out + (size_t)r * d + c) = a;
            ss += a.x * a.x + a.y * a.y + a.z * a.z + a.w * a.w;
        }
    }
    ss = block_sum(ss, red);
    const float inv = 1.0f / sqrtf(ss / (float)d + eps);
#pragma unroll
    for (int it = 0; it < RN_TRIPS; ++it) {
        const int c = (it * NT + threadIdx.x) * 4;
        if (c < d) {
            T* mp = m_out + (size_t)r * d + c;
            mp[0] = from_f32<T>(hv[it].x * inv * to_f32(g[c]));
            mp[1] = from_f32<T>(hv[it].y * inv * to_f32(g[c + 1]));
            mp[2] = from_f32<T>(hv[it].z * inv * to_f32(g[c + 2]));
            mp[3] = from_f32<T>(hv[it].w * inv * to_f32(g[c + 3]));
        }
    }
}

int launch_residual_norm(compact_ctx* ctx, const float* partials, int ks, const void* resid, const void* g,
                         void* h_out, void* m_out, int rows, hipStream_t s) {
    const compact_layer_cfg& c = ctx->cfg;
    if (c.d_model > RN_TRIPS * NT * 4) return set_err(ctx, COMPACT_ESHAPE, "d_model above 8192 is not supported by the decode row kernels");
    if (c.dtype == COMPACT_BF16)
        residual_norm_kernel<bf16><<<rows, NT, 0, s>>>(partials, ks, rows, (const bf16*)resid, (const bf16*)g,
                                                      (float*)h_out, (bf16*)m_out, c.d_model, c.rms_eps);
    else
        residual_norm_kernel<float><<<rows, NT, 0, s>>>(partials, ks, rows, (const float*)resid, (const float*)g,
                                                       (float*)h_out, (float*)m_out, c.d_model, c.rms_eps);
    LAUNCH_CHECK(ctx);
    return COMPACT_OK;
}

// ---------------------------------------------------------------------------
// Decode: act = silu(gate) * up, gate/up = sum of partials of the stacked
// projection [rows, 2F]
// ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(NT) void swiglu_reduce_kernel(const float* __restrict__ partials, int ks, int rows,
                                                           T* __restrict__ act, int F) {
    const int r = blockIdx.y;
    const int c = blockIdx.x * NT + threadIdx.x;
    if (c >= F) return;
    const size_t ps = (size_t)rows * 2 * F;
    float gt = 0.f, up = 0.f;
    for (int s = 0; s < ks; ++s) {
        gt += partials[s * ps + (size_t)r * 2 * F + c];
        up += partials[s * ps + (size_t)r * 2 * F + F + c];
    }
    const float sg = gt / (1.0f + expf(-gt));
    act[(size_t)r * F + c] = from_f32<T>(sg * up);
}

int launch_swiglu_reduce(compact_ctx* ctx, const float* partials, int ks, void* act, int rows, int F, hipStream_t s) {
    dim3 grid((F + NT - 1) / NT, rows);
    if (ctx->cfg.dtype == COMPACT_BF16)
        swiglu_reduce_kernel<bf16><<<grid, NT, 0, s>>>(partials, ks, rows, (bf16*)act, F);
    else
        swiglu_reduce_kernel<float><<<grid, NT, 0, s>>>(partials, ks, rows, (float*)act, F);
    LAUNCH_CHECK(ctx);
    return COMPACT_OK;
}

// ---------------------------------------------------------------------------
// Decode: y = resid (fp32) + sum_s partial_s ; 4 columns per thread
// ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(NT) void residual_reduce_kernel(const float* __restrict__ partials, int ks, int rows,
                                                             const float* __restrict__ resid, T* __restrict__ y,
                                                             int cols) {
    const size_t i = ((size_t)blockIdx.x * NT + threadIdx.x) * 4;
    const size_t total = (size_t)rows * cols;
    if (i >= total) return;
    float4 a = *reinterpret_cast<const float4*>(resid + i);
    a = sum_slices4(partials + i, total, ks, a);
    y[i] = from_f32<T>(a.x);
    y[i + 1] = from_f32<T>(a.y);
    y[i + 2] = from_f32<T>(a.z);
    y[i + 3] = from_f32<T>(a.w);
}

int launch_residual_reduce(compact_ctx* ctx, const float* partials, int ks, const void* resid, void* y, int rows,
                           int cols, hipStream_t s) {
    const size_t total = (size_t)rows * cols;  // cols is a multiple of 64
    const unsigned grid = (unsigned)((total / 4 + NT - 1) / NT);
    if (ctx->cfg.dtype == COMPACT_BF16)
        residual_reduce_kernel<bf16><<<grid, NT, 0, s>>>(partials, ks, rows, (const float*)resid, (bf16*)y, cols);
    else
        residual_reduce_kernel<float><<<grid, NT, 0, s>>>(partials, ks, rows, (const float*)resid, (float*)y, cols);
    LAUNCH_CHECK(ctx);
    return COMPACT_OK;
}

// ---------------------------------------------------------------------------
// y_last[b] = y[last row of block b]
// ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(NT) void gather_last_rows_kernel(const BlockMeta* __restrict__ meta,
                                                              const T* __restrict__ y, T* __restrict__ y_last, int d) {
    const BlockMeta bm = meta[blockIdx.x];
    const T* src = y + (size_t)(bm.row0 + bm.len - 1) * d;
    T* dst = y_last + (size_t)blockIdx.x * d;
    for (int c = threadIdx.x; c < d; c += NT) dst[c] = src[c];
}

int launch_gather_last_rows(compact_ctx* ctx, const BlockMeta* d_meta, int n_blocks, const void* y, void* y_last,
                            hipStream_t s) {
    if (ctx->cfg.dtype == COMPACT_BF16)
        gather_last_rows_kernel<bf16><<<n_blocks, NT, 0, s>>>(d_meta, (const bf16*)y, (bf16*)y_last, ctx->cfg.d_model);
    else
        gather_last_rows_kernel<float><<<n_blocks, NT, 0, s>>>(d_meta, (const float*)y, (float*)y_last, ctx->cfg.d_model);
    LAUNCH_CHECK(ctx);
    return COMPACT_OK;
}

// ---------------------------------------------------------------------------
// Row mover of the mixed-batch scheduler: packed row i is read from / written to
// the row a table names.  Table value v >= 0: row v of base 0; v <= -2: row
// (-v - 2) of base 1; v == -1: no row (skip).  A null table means row i of base 0.
// ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(NT) void move_rows_kernel(const T* __restrict__ src0, const T* __restrict__ src1,
                                                       const int32_t* __restrict__ src_tab, T* __restrict__ dst0,
                                                       T* __restrict__ dst1, const int32_t* __restrict__ dst_tab, int d) {
    const int i = blockIdx.x;
    const int sv = src_tab ? src_tab[i] : i;
    const int dv = dst_tab ? dst_tab[i] : i;
    if (sv == -1 || dv == -1) return;
    const T* src = sv >= 0 ? src0 + (size_t)sv * d : src1 + (size_t)(-sv - 2) * d;
    T* dst = dv >= 0 ? dst0 + (size_t)dv * d : dst1 + (size_t)(-dv - 2) * d;
    for (int c = threadIdx.x; c < d; c += NT) dst[c] = src[c];
}

int launch_move_rows(compact_ctx* ctx, const void* src0, const void* src1, const int32_t* src_tab, void* dst0, void* dst1,
                     const int32_t* dst_tab, int rows, hipStream_t s) {
    if (rows == 0) return COMPACT_OK;
    const int d = ctx->cfg.d_model;
    if (ctx->cfg.dtype == COMPACT_BF16)
        move_rows_kernel<bf16><<<rows, NT, 0, s>>>((const bf16*)src0, (const bf16*)src1, src_tab, (bf16*)dst0, (bf16*)dst1, dst_tab, d);
    else
        move_rows_kernel<float><<<rows, NT, 0, s>>>((const float*)src0, (const float*)src1, src_tab, (float*)dst0, (float*)dst1, dst_tab, d);
    LAUNCH_CHECK(ctx);
    return COMPACT_OK;
}
