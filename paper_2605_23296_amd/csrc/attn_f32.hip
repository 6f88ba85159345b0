// fp32 attention for the fp32 storage mode: one wavefront per query row,
// lanes over head_dim, keys visited in order with a running (max, sum, acc).
// Checking-mode kernels: plain and sequential, not tuned.
#include "common.h"
#include "vecio.h"

// running softmax state of one query row held across a wavefront:
// lane l owns output elements l and l + 64 (the second only when hd = 128)
struct RowState {
    float m, l, acc0, acc1;
};

template <int HD>
__device__ __forceinline__ void visit_key(RowState& st, float q0, float q1, const float* __restrict__ krow,
                                          const float* __restrict__ vcol, int64_t vstride, float scale) {
    const int lane = threadIdx.x & (WAVE - 1);
    float part = q0 * krow[lane];
    if (HD == 128) part += q1 * krow[lane + 64];
    const float sc = wave_sum(part) * scale;
    const float mn = fmaxf(st.m, sc);
    const float corr = expf(st.m - mn);  // exp(-inf) = 0 on the first key
    const float p = expf(sc - mn);
    st.l = st.l * corr + p;
    st.acc0 = st.acc0 * corr + p * vcol[(int64_t)lane * vstride];
    if (HD == 128) st.acc1 = st.acc1 * corr + p * vcol[(int64_t)(lane + 64) * vstride];
    st.m = mn;
}

template <int HD>
__global__ __launch_bounds__(256) void attn_prefill_f32_kernel(const BlockMeta* __restrict__ meta,
                                                               const float* __restrict__ qkv,
                                                               const float* __restrict__ kbase,
                                                               const float* __restrict__ vbase, float* __restrict__ o,
                                                               int Hq, int Hkv, float scale) {
    const BlockMeta bm = meta[blockIdx.z];
    const int i = blockIdx.x * 4 + threadIdx.x / WAVE;
    if (i >= bm.len) return;
    const int h = blockIdx.y, kvh = h / (Hq / Hkv);
    const int lane = threadIdx.x & (WAVE - 1);
    const int ld = (Hq + 2 * Hkv) * HD;
    const float* qrow = qkv + (size_t)(bm.row0 + i) * ld + h * HD;
    const float q0 = qrow[lane];
    const float q1 = HD == 128 ? qrow[lane + 64] : 0.f;
    const float* kslab = kbase + bm.slab + (size_t)kvh * bm.capacity * HD;
    const float* vslab = vbase + bm.slab + (size_t)kvh * HD * bm.capacity;
    RowState st = {-INFINITY, 0.f, 0.f, 0.f};
    for (int j = 0; j <= bm.prior + i; ++j) visit_key<HD>(st, q0, q1, kslab + (size_t)j * HD, vslab + j, bm.capacity, scale);
    float* orow = o + (size_t)(bm.row0 + i) * Hq * HD + h * HD;
    orow[lane] = st.acc0 / st.l;
    if (HD == 128) orow[lane + 64] = st.acc1 / st.l;
}

int launch_attn_prefill_f32(compact_ctx* ctx, const BlockMeta* d_meta, int n_blocks, int max_len, const float* qkv,
                            const float* d_k, const float* d_v, float* o, hipStream_t s) {
    const compact_layer_cfg& c = ctx->cfg;
    dim3 grid((max_len + 3) / 4, c.n_q_heads, n_blocks);
    const float scale = 1.0f / sqrtf((float)c.head_dim);
    if (c.head_dim == 128)
        attn_prefill_f32_kernel<128><<<grid, 256, 0, s>>>(d_meta, qkv, d_k, d_v, o, c.n_q_heads, c.n_kv_heads, scale);
    else
        attn_prefill_f32_kernel<64><<<grid, 256, 0, s>>>(d_meta, qkv, d_k, d_v, o, c.n_q_heads, c.n_kv_heads, scale);
    LAUNCH_CHECK(ctx);
    return COMPACT_OK;
}

// one workgroup per (head, block); its 4 wavefronts take keys w, w+4, ... and
// their states are merged in wavefront order
template <int HD>
__global__ __launch_bounds__(256) void attn_decode_f32_kernel(const BlockMeta* __restrict__ meta, int step,
                                                              const float* __restrict__ q,
                                                              const float* __restrict__ kbase,
                                                              const float* __restrict__ vbase, float* __restrict__ o,
                                                              int Hq, int Hkv, float scale) {
    __shared__ float sm[4], sl[4], sacc[4][HD];
    const BlockMeta bm = meta[blockIdx.y];
    const int n_keys = bm.len + step + 1;  // the appended row is included
    const int h = blockIdx.x, kvh = h / (Hq / Hkv);
    const int lane = threadIdx.x & (WAVE - 1), w = threadIdx.x / WAVE;
    const float* qrow = q + (size_t)blockIdx.y * Hq * HD + h * HD;
    const float q0 = qrow[lane];
    const float q1 = HD == 128 ? qrow[lane + 64] : 0.f;
    const float* kslab = kbase + bm.slab + (size_t)kvh * bm.capacity * HD;
    const float* vslab = vbase + bm.slab + (size_t)kvh * HD * bm.capacity;
    RowState st = {-INFINITY, 0.f, 0.f, 0.f};
    for (int j = w; j < n_keys; j += 4) visit_key<HD>(st, q0, q1, kslab + (size_t)j * HD, vslab + j, bm.capacity, scale);
    if (lane == 0) {
        sm[w] = st.m;
        sl[w] = st.l;
    }
    sacc[w][lane] = st.acc0;
    if (HD == 128) sacc[w][lane + 64] = st.acc1;
    __syncthreads();
    if (w == 0) {
        float m = -INFINITY;
        for (int i = 0; i < 4; ++i) m = fmaxf(m, sm[i]);
        float l = 0.f, a0 = 0.f, a1 = 0.f;
        for (int i = 0; i < 4; ++i) {
            const float f = sl[i] > 0.f ? expf(sm[i] - m) : 0.f;  // a wavefront may have seen no key
            l += sl[i] * f;
            a0 += sacc[i][lane] * f;
            if (HD == 128) a1 += sacc[i][lane + 64] * f;
        }
        float* orow = o + (size_t)blockIdx.y * Hq * HD + h * HD;
        orow[lane] = a0 / l;
        if (HD == 128) orow[lane + 64] = a1 / l;
    }
}

int launch_attn_decode_f32(compact_ctx* ctx, const BlockMeta* d_meta, int n_blocks, int step, const float* q,
                           const float* d_k, const float* d_v, float* o, hipStream_t s) {
    const compact_layer_cfg& c = ctx->cfg;
    dim3 grid(c.n_q_heads, n_blocks);
    const float scale = 1.0f / sqrtf((float)c.head_dim);
    if (c.head_dim == 128)
        attn_decode_f32_kernel<128><<<grid, 256, 0, s>>>(d_meta, step, q, d_k, d_v, o, c.n_q_heads, c.n_kv_heads, scale);
    else
        attn_decode_f32_kernel<64><<<grid, 256, 0, s>>>(d_meta, step, q, d_k, d_v, o, c.n_q_heads, c.n_kv_heads, scale);
    LAUNCH_CHECK(ctx);
    return COMPACT_OK;
}
