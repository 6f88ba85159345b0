// C ABI of libcompact: argument validation, host-side planning (ragged tile
// lists, workspace carving, metadata upload) and the launch sequences of the
// prefill pass and the decode step.  All arithmetic is in the kernels.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <mutex>

#include "common.h"

static std::string g_create_err;

int set_err(compact_ctx* ctx, int code, const std::string& msg) {
    if (ctx)
        ctx->err = msg;
    else
        g_create_err = msg;
    return code;
}

int device_cu_count(compact_ctx* ctx, int* n_cus) {
    if (ctx->n_cus <= 0) {
        int dev = 0, n = 0;
        HIP_TRY(ctx, hipGetDevice(&dev));
        HIP_TRY(ctx, hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev));
        if (n <= 0) return set_err(ctx, COMPACT_EHIP, "device reports no compute units");
        ctx->n_cus = n;
    }
    *n_cus = ctx->n_cus;
    return COMPACT_OK;
}

// ---------------------------------------------------------------------------
// profiling
// ---------------------------------------------------------------------------
ProfileScope::ProfileScope(compact_ctx* c, int klass, hipStream_t s) : ctx(c), stream(s), on(false) {
    if (c->profile_class != klass || klass == COMPACT_K_NONE) return;
    if (c->prof_used == c->prof_events.size()) {
        ProfileSlot ns;
        if (hipEventCreate(&ns.start) != hipSuccess || hipEventCreate(&ns.stop) != hipSuccess) return;
        c->prof_events.push_back(ns);
    }
    slot = c->prof_events[c->prof_used++];
    on = hipEventRecord(slot.start, stream) == hipSuccess;
}
ProfileScope::~ProfileScope() {
    if (on) (void)hipEventRecord(slot.stop, stream);
}

extern "C" int compact_profile_select(compact_ctx* ctx, int32_t klass) {
    if (!ctx) return COMPACT_EINVAL;
    if (klass < 0 || klass >= COMPACT_K_COUNT) return set_err(ctx, COMPACT_EINVAL, "unknown kernel class");
    ctx->profile_class = klass;
    ctx->prof_used = 0;
    ctx->prof_launches = 0;
    ctx->prof_ms = 0.0;
    return COMPACT_OK;
}

extern "C" int compact_profile_read(compact_ctx* ctx, int64_t* n_launches, double* total_ms) {
    if (!ctx || !n_launches || !total_ms) return COMPACT_EINVAL;
    for (size_t i = 0; i < ctx->prof_used; ++i) {
        HIP_TRY(ctx, hipEventSynchronize(ctx->prof_events[i].stop));
        float ms = 0.f;
        HIP_TRY(ctx, hipEventElapsedTime(&ms, ctx->prof_events[i].start, ctx->prof_events[i].stop));
        ctx->prof_ms += ms;
        ctx->prof_launches += 1;
    }
    ctx->prof_used = 0;
    *n_launches = ctx->prof_launches;
    *total_ms = ctx->prof_ms;
    return COMPACT_OK;
}

// ---------------------------------------------------------------------------
// context
// ---------------------------------------------------------------------------
static int validate_cfg(const compact_layer_cfg* c, std::string& why) {
    if (c->d_model <= 0 || c->n_q_heads <= 0 || c->n_kv_heads <= 0 || c->head_dim <= 0 || c->ffn_dim <= 0) {
        why = "non-positive layer dimension";
        return COMPACT_EINVAL;
    }
    if (c->dtype != COMPACT_FP32 && c->dtype != COMPACT_BF16) {
        why = "dtype must be COMPACT_FP32 or COMPACT_BF16";
        return COMPACT_EUNSUPPORTED;
    }
    if (c->head_dim != 64 && c->head_dim != 128) {
        why = "head_dim must be 64 or 128";
        return COMPACT_ESHAPE;
    }
    if (c->n_q_heads % c->n_kv_heads != 0 || c->n_q_heads / c->n_kv_heads > 16) {
        why = "n_q_heads must be a multiple of n_kv_heads with a group of at most 16";
        return COMPACT_ESHAPE;
    }
    if (c->d_model % 64 != 0 || c->ffn_dim % 64 != 0 || c->d_model > 8192) {
        why = "d_model and ffn_dim must be multiples of 64, d_model at most 8192";
        return COMPACT_ESHAPE;
    }
    if (c->n_experts < 0 || c->n_experts > 256) {
        why = "n_experts must be in 0..256";
        return COMPACT_ESHAPE;
    }
    if (c->n_experts > 0 && (c->top_k < 1 || c->top_k > 8 || c->top_k > c->n_experts)) {
        why = "top_k must be in 1..min(8, n_experts)";
        return COMPACT_ESHAPE;
    }
    if (c->n_experts % 8 != 0 && c->dtype == COMPACT_BF16) {
        why = "bf16 storage needs n_experts to be a multiple of 8 (the router logits come out of the MFMA GEMM in 8-column pieces)";
        return COMPACT_ESHAPE;
    }
    if (!(c->rms_eps >= 0.f) || !(c->rope_theta > 0.f)) {
        why = "rms_eps must be >= 0 and rope_theta > 0";
        return COMPACT_EINVAL;
    }
    return COMPACT_OK;
}

extern "C" int compact_create(const compact_layer_cfg* cfg, compact_ctx** out) {
    if (!cfg || !out) return set_err(nullptr, COMPACT_EINVAL, "null cfg or out");
    std::string why;
    const int rc = validate_cfg(cfg, why);
    if (rc != COMPACT_OK) return set_err(nullptr, rc, why);
    compact_ctx* ctx = new compact_ctx();
    ctx->cfg = *cfg;
    *out = ctx;
    return COMPACT_OK;
}

static void drop_step_cache(compact_ctx* ctx);

extern "C" void compact_destroy(compact_ctx* ctx) {
    if (!ctx) return;
    if (ctx->d_meta) (void)hipFree(ctx->d_meta);
    if (ctx->h_stage) (void)hipHostFree(ctx->h_stage);
    if (ctx->stage_event) (void)hipEventDestroy(ctx->stage_event);
    drop_step_cache(ctx);
    for (auto& e : ctx->prof_events) {
        (void)hipEventDestroy(e.start);
        (void)hipEventDestroy(e.stop);
    }
    delete ctx;
}

extern "C" const char* compact_last_error(const compact_ctx* ctx) { return ctx ? ctx->err.c_str() : g_create_err.c_str(); }

// ---------------------------------------------------------------------------
// workspace carving: the same routine sizes the workspace (base == nullptr)
// and hands out its pieces
// ---------------------------------------------------------------------------
struct Carver {
    char* base;
    size_t off = 0;
    explicit Carver(void* b) : base((char*)b) {}
    void* take(size_t bytes) {
        off = align_up(off, 256);
        void* p = base ? base + off : nullptr;
        off += bytes;
        return p;
    }
};

struct PrefillBufs {
    void *n, *qkv, *o, *h, *act;
    // MoE
    float* logits;
    int32_t* idx;
    float* gate;
    MoePlan plan;
    void* expert_out;
};

struct DecodeBufs {
    void *n, *q, *o, *m, *act;
    void* hg;          // bf16(h * g_ffn): the FFN input before its 1/rms factor
    float* ssq_parts;  // [d_model / 16][N] column-group sums of squares of h
    float *h, *partials, *attn_partials;
    float* logits;
    int32_t* idx;
    float* gate;
    MoePlan plan;
    void* expert_out;
};

static size_t max_partial_cols(const compact_layer_cfg& c) {
    size_t cols = (size_t)(c.n_q_heads + 2 * c.n_kv_heads) * c.head_dim;
    cols = std::max(cols, (size_t)c.d_model);
    cols = std::max(cols, (size_t)2 * c.ffn_dim);
    return cols;
}

static int moe_mtile(const compact_layer_cfg& c) { return c.dtype == COMPACT_BF16 ? gemm_bf16_mtile() : gemm_f32_mtile(); }

// mt = rows per tile of the plan's tile map: the row tile of the prefill-size expert GEMMs, or 16 for the decode
// steps' per-expert streaming
static void carve_moe_plan(Carver& cv, const compact_layer_cfg& c, int64_t rows, MoePlan& plan, int mt) {
    const int64_t rk = rows * c.top_k;
    plan.max_mtiles = (int32_t)(rk / mt + c.n_experts + 1);
    plan.counts = (int32_t*)cv.take(sizeof(int32_t) * c.n_experts);
    plan.offsets = (int32_t*)cv.take(sizeof(int32_t) * (c.n_experts + 1));
    plan.sorted_token = (int32_t*)cv.take(sizeof(int32_t) * rk);
    plan.sorted_gate = (float*)cv.take(sizeof(float) * rk);
    plan.slot_of = (int32_t*)cv.take(sizeof(int32_t) * rk);
    plan.tile_expert = (int32_t*)cv.take(sizeof(int32_t) * plan.max_mtiles);
    plan.tile_row0 = (int32_t*)cv.take(sizeof(int32_t) * plan.max_mtiles);
    plan.tile_rows = (int32_t*)cv.take(sizeof(int32_t) * plan.max_mtiles);
}

static void carve_prefill(Carver& cv, const compact_layer_cfg& c, int64_t T, PrefillBufs& b) {
    const size_t es = dtype_size(c.dtype);
    const size_t ld = (size_t)(c.n_q_heads + 2 * c.n_kv_heads) * c.head_dim;
    b.n = cv.take((size_t)T * c.d_model * es);  // reused for m
    // at least d_model columns per row: a forward pass whose caller wants no prefill output
    // writes the [T, d_model] result of the feed-forward half over this scratch, dead by then
    b.qkv = cv.take((size_t)T * std::max(ld, (size_t)c.d_model) * es);
    b.o = cv.take((size_t)T * c.n_q_heads * c.head_dim * es);
    b.h = cv.take((size_t)T * c.d_model * 4);  // the residual stream between the two halves stays fp32
    if (c.n_experts == 0) {
        b.act = cv.take((size_t)T * c.ffn_dim * es);
    } else {
        b.act = cv.take((size_t)T * c.top_k * c.ffn_dim * es);
        b.logits = (float*)cv.take((size_t)T * c.n_experts * 4);
        b.idx = (int32_t*)cv.take((size_t)T * c.top_k * 4);
        b.gate = (float*)cv.take((size_t)T * c.top_k * 4);
        carve_moe_plan(cv, c, T, b.plan, moe_mtile(c));
        b.expert_out = cv.take((size_t)T * c.top_k * c.d_model * es);
    }
}

static int decode_max_ksplit(const compact_layer_cfg& c, int N);

static void carve_decode(Carver& cv, const compact_layer_cfg& c, int N, int max_chunks, DecodeBufs& b) {
    const size_t es = dtype_size(c.dtype);
    b.n = cv.take((size_t)N * c.d_model * es);
    b.q = cv.take((size_t)N * c.n_q_heads * c.head_dim * es);
    b.o = cv.take((size_t)N * c.n_q_heads * c.head_dim * es);
    b.m = cv.take((size_t)N * c.d_model * es);
    b.hg = cv.take((size_t)N * c.d_model * es);
    b.ssq_parts = (float*)cv.take((size_t)((c.d_model + 15) / 16) * N * 4);
    b.h = (float*)cv.take((size_t)N * c.d_model * 4);
    const int rows = c.n_experts == 0 ? N : N * c.top_k;
    b.act = cv.take((size_t)rows * c.ffn_dim * es);
    b.partials = (float*)cv.take((size_t)decode_max_ksplit(c, N) * rows * max_partial_cols(c) * 4);
    b.attn_partials = (float*)cv.take(attn_decode_partial_floats(c, N, max_chunks) * 4);
    if (c.n_experts > 0) {
        b.logits = (float*)cv.take((size_t)N * c.n_experts * 4);
        b.idx = (int32_t*)cv.take((size_t)N * c.top_k * 4);
        b.gate = (float*)cv.take((size_t)N * c.top_k * 4);
        carve_moe_plan(cv, c, N, b.plan, 16);
        b.expert_out = cv.take((size_t)N * c.top_k * c.d_model * es);
    }
}

static int decode_max_ksplit(const compact_layer_cfg& c, int N) {
    if (c.dtype != COMPACT_BF16) return 1;
    const int Dtot = (c.n_q_heads + 2 * c.n_kv_heads) * c.head_dim;
    int ks = skinny_ksplit(N, Dtot, c.d_model);
    ks = std::max(ks, skinny_ksplit(N, c.d_model, c.n_q_heads * c.head_dim));
    ks = std::max(ks, skinny_ksplit(N, 2 * c.ffn_dim, c.d_model));
    ks = std::max(ks, skinny_ksplit(N, c.d_model, c.ffn_dim));
    return ks;
}

static int chunks_for(int len) { return (len + DECODE_CHUNK - 1) / DECODE_CHUNK; }
static int prefix_chunks_for(int len) { return (len + PREFIX_CHUNK - 1) / PREFIX_CHUNK; }

extern "C" int compact_workspace_bytes(const compact_ctx* ctx, int64_t max_tokens, int32_t max_blocks,
                                       int32_t max_kv_len, size_t* bytes) {
    if (!ctx || !bytes) return COMPACT_EINVAL;
    compact_ctx* c = const_cast<compact_ctx*>(ctx);
    if (max_tokens < 0 || max_blocks < 1 || max_kv_len < 1)
        return set_err(c, COMPACT_EINVAL, "max_tokens >= 0, max_blocks >= 1, max_kv_len >= 1 required");
    Carver cp(nullptr), cd(nullptr);
    PrefillBufs pb;
    DecodeBufs db;
    carve_prefill(cp, ctx->cfg, max_tokens, pb);
    carve_decode(cd, ctx->cfg, max_blocks, chunks_for(max_kv_len), db);
    // the decode region follows the prefill region, so a forward pass can keep
    // the prefill outputs alive while it decodes
    *bytes = align_up(cp.off, 256) + align_up(cd.off, 256) + 256;
    return COMPACT_OK;
}

// ---------------------------------------------------------------------------
// metadata upload
// ---------------------------------------------------------------------------
struct Plan {
    std::vector<BlockMeta> meta;
    std::vector<TileItem> rope_tiles, q_tiles;
    std::vector<TileItem> kv_chunks;   // decode attention work list: (block, first cached row of a chunk)
    int max_len = 0;
    // device views
    const BlockMeta* d_meta = nullptr;
    const TileItem* d_rope_tiles = nullptr;
    const TileItem* d_q_tiles = nullptr;
    const TileItem* d_kv_chunks = nullptr;
    std::vector<char> extra;           // further host-built tables, uploaded behind the lists
    const char* d_extra = nullptr;
};

static int upload_plan(compact_ctx* ctx, Plan& p, hipStream_t s) {
    ++ctx->upload_serial;   // the device views of every earlier plan are gone
    const size_t b0 = align_up(p.meta.size() * sizeof(BlockMeta), 256);
    const size_t b1 = align_up(p.rope_tiles.size() * sizeof(TileItem), 256);
    const size_t b2 = align_up(p.q_tiles.size() * sizeof(TileItem), 256);
    const size_t b3 = align_up(p.kv_chunks.size() * sizeof(TileItem), 256);
    const size_t b4 = align_up(p.extra.size(), 256);
    const size_t total = b0 + b1 + b2 + b3 + b4;
    if (total > ctx->meta_bytes) {
        // growing the metadata buffer: wait for work that may still read the old one
        HIP_TRY(ctx, hipDeviceSynchronize());
        if (ctx->d_meta) HIP_TRY(ctx, hipFree(ctx->d_meta));
        if (ctx->h_stage) HIP_TRY(ctx, hipHostFree(ctx->h_stage));
        ctx->d_meta = nullptr;
        ctx->h_stage = nullptr;
        ctx->meta_bytes = 0;
        // 1 MiB holds the lists of every named workload several times over, so that in practice only the
        // first call through a context allocates (and synchronises)
        const size_t cap = std::max(total * 2, (size_t)1 << 20);
        HIP_TRY(ctx, hipMalloc(&ctx->d_meta, cap));
        HIP_TRY(ctx, hipHostMalloc(&ctx->h_stage, cap, hipHostMallocDefault));
        ctx->meta_bytes = cap;
    }
    if (!ctx->stage_event) HIP_TRY(ctx, hipEventCreateWithFlags(&ctx->stage_event, hipEventDisableTiming));
    if (ctx->stage_pending) {  // the previous upload must have left the staging buffer
        HIP_TRY(ctx, hipEventSynchronize(ctx->stage_event));
        ctx->stage_pending = false;
    }
    char* hs = (char*)ctx->h_stage;
    memcpy(hs, p.meta.data(), p.meta.size() * sizeof(BlockMeta));
    if (!p.rope_tiles.empty()) memcpy(hs + b0, p.rope_tiles.data(), p.rope_tiles.size() * sizeof(TileItem));
    if (!p.q_tiles.empty()) memcpy(hs + b0 + b1, p.q_tiles.data(), p.q_tiles.size() * sizeof(TileItem));
    if (!p.kv_chunks.empty()) memcpy(hs + b0 + b1 + b2, p.kv_chunks.data(), p.kv_chunks.size() * sizeof(TileItem));
    if (!p.extra.empty()) memcpy(hs + b0 + b1 + b2 + b3, p.extra.data(), p.extra.size());
    HIP_TRY(ctx, hipMemcpyAsync(ctx->d_meta, hs, total, hipMemcpyHostToDevice, s));
    HIP_TRY(ctx, hipEventRecord(ctx->stage_event, s));
    ctx->stage_pending = true;
    char* dm = (char*)ctx->d_meta;
    p.d_meta = (const BlockMeta*)dm;
    p.d_rope_tiles = (const TileItem*)(dm + b0);
    p.d_q_tiles = (const TileItem*)(dm + b0 + b1);
    p.d_kv_chunks = (const TileItem*)(dm + b0 + b1 + b2);
    p.d_extra = dm + b0 + b1 + b2 + b3;
    return COMPACT_OK;
}

// ---------------------------------------------------------------------------
// validation shared by the entry points
// ---------------------------------------------------------------------------
static int check_kv(compact_ctx* ctx, const compact_kv* kv, int n_blocks) {
    if (!kv || !kv->d_k || !kv->d_v || !kv->h_slab_offset || !kv->h_capacity || !kv->h_len)
        return set_err(ctx, COMPACT_EINVAL, "kv and its d_k, d_v, h_slab_offset, h_capacity, h_len must be non-null");
    for (int b = 0; b < n_blocks; ++b) {
        if (kv->h_capacity[b] < 8 || kv->h_capacity[b] % 8 != 0)
            return set_err(ctx, COMPACT_EINVAL, "h_capacity[b] must be a positive multiple of 8");
        if (kv->h_slab_offset[b] < 0 || kv->h_slab_offset[b] % 8 != 0)
            return set_err(ctx, COMPACT_EINVAL, "h_slab_offset[b] must be a non-negative multiple of 8");
    }
    return COMPACT_OK;
}

static int check_weights(compact_ctx* ctx, const compact_weights* w) {
    if (!w) return set_err(ctx, COMPACT_EINVAL, "null weights");
    if (!w->g_attn || !w->w_qkv || !w->w_o || !w->g_ffn) return set_err(ctx, COMPACT_EINVAL, "null attention weights");
    if (ctx->cfg.n_experts == 0) {
        if (!w->w_gate_up || !w->w_down) return set_err(ctx, COMPACT_EINVAL, "null dense FFN weights");
    } else {
        if (!w->w_router || !w->w_exp_gate_up || !w->w_exp_down) return set_err(ctx, COMPACT_EINVAL, "null MoE weights");
        const int nq = (w->w_exp_gate_up_q != nullptr) + (w->w_exp_gate_up_s != nullptr) + (w->w_exp_down_q != nullptr) +
                       (w->w_exp_down_s != nullptr);
        if (nq != 0 && nq != 4) return set_err(ctx, COMPACT_EINVAL, "4-bit expert weights: give all four arrays or none");
        if (nq == 4 && ctx->cfg.dtype != COMPACT_BF16)
            return set_err(ctx, COMPACT_EUNSUPPORTED, "4-bit expert weights need bf16 storage");
        if (nq == 4 && (ctx->cfg.d_model % 32 != 0 || ctx->cfg.ffn_dim % 32 != 0))
            return set_err(ctx, COMPACT_ESHAPE, "4-bit expert weights need d_model % 32 == 0 and ffn_dim % 32 == 0");
    }
    return COMPACT_OK;
}

static int check_blocks(compact_ctx* ctx, int n_blocks, const int32_t* cu) {
    if (n_blocks < 1) return set_err(ctx, COMPACT_EINVAL, "n_blocks must be >= 1");
    if (!cu) return set_err(ctx, COMPACT_EINVAL, "null h_cu_seqlens");
    if (cu[0] != 0) return set_err(ctx, COMPACT_EINVAL, "h_cu_seqlens[0] must be 0");
    for (int b = 0; b < n_blocks; ++b)
        if (cu[b + 1] <= cu[b]) return set_err(ctx, COMPACT_EINVAL, "h_cu_seqlens must be strictly increasing (empty blocks are not allowed)");
    return COMPACT_OK;
}

// extend: the rows of the call are appended behind the h_len[b] rows the cache holds
static void build_prefill_plan(const compact_kv* kv, int n_blocks, const int32_t* cu, Plan& p, bool extend = false) {
    p.meta.resize(n_blocks);
    for (int b = 0; b < n_blocks; ++b) {
        BlockMeta& m = p.meta[b];
        m.row0 = cu[b];
        m.len = cu[b + 1] - cu[b];
        m.prior = extend ? kv->h_len[b] : 0;
        m.capacity = kv->h_capacity[b];
        m.pos_offset = kv->h_pos_offset ? kv->h_pos_offset[b] : 0;
        m.slab = kv->h_slab_offset[b];
        p.max_len = std::max(p.max_len, m.len);
        for (int r = 0; r < m.len; r += ROPE_TILE) p.rope_tiles.push_back({b, r});
        for (int r = 0; r < m.len; r += PREFILL_QTILE) p.q_tiles.push_back({b, r});
    }
    // causal work of a query tile grows with its cache row: heaviest first
    const std::vector<BlockMeta>& mt = p.meta;
    std::stable_sort(p.q_tiles.begin(), p.q_tiles.end(), [&mt](const TileItem& a, const TileItem& b) {
        return mt[a.block].prior + a.row0 > mt[b.block].prior + b.row0;
    });
}

// Work list of the split-KV decode attention: every DECODE_CHUNK-row chunk that some
// step of the call touches, block by block (`extra` = rows the call appends to each
// cache).  Chunks a given step does not reach yet leave at once.
static void add_kv_chunks(Plan& p, int extra) {
    p.kv_chunks.clear();
    for (int b = 0; b < (int)p.meta.size(); ++b)
        for (int r = 0; r < p.meta[b].len + extra; r += DECODE_CHUNK) p.kv_chunks.push_back({b, r});
}

static void build_decode_plan(const compact_kv* kv, int n_blocks, Plan& p) {
    p.meta.resize(n_blocks);
    for (int b = 0; b < n_blocks; ++b) {
        BlockMeta& m = p.meta[b];
        m.row0 = b;
        m.len = kv->h_len[b];
        m.capacity = kv->h_capacity[b];
        m.pos_offset = kv->h_pos_offset ? kv->h_pos_offset[b] : 0;
        m.slab = kv->h_slab_offset[b];
        p.max_len = std::max(p.max_len, m.len);
    }
}

// ---------------------------------------------------------------------------
// GEMM dispatch by storage type
// ---------------------------------------------------------------------------
// prefill-size: C = A B^T (+R) or SwiGLU epilogue.  epi 2 = fp32 output; r_f32 = fp32 residual
// (both only matter for bf16 storage: in fp32 storage everything is fp32 anyway).
static int gemm_full(compact_ctx* ctx, const void* A, const void* B, const void* R, bool r_f32, void* C, int64_t M,
                     int N, int K, int epi, hipStream_t s) {
    if (ctx->cfg.dtype == COMPACT_BF16) {
        ProfileScope ps(ctx, COMPACT_K_GEMM, s);
        return launch_gemm_bf16(ctx, (const bf16*)A, (const bf16*)B, R, r_f32, (bf16*)C, M, N, K, epi, nullptr, s);
    }
    return launch_gemm_f32(ctx, (const float*)A, (const float*)B, (const float*)R, (float*)C, M, N, K, epi == 2 ? 0 : epi,
                           nullptr, s);
}

// decode-size: fp32 split-K partials [ks][M][N]
static int gemm_partials(compact_ctx* ctx, const void* A, const void* B, float* partials, int M, int N, int K, int* ks,
                         hipStream_t s) {
    if (ctx->cfg.dtype == COMPACT_BF16) {
        *ks = skinny_ksplit(M, N, K);
        ProfileScope ps(ctx, COMPACT_K_GEMM_SKINNY, s);
        return launch_gemm_skinny(ctx, (const bf16*)A, (const bf16*)B, partials, M, N, K, *ks, s);
    }
    *ks = 1;
    return launch_gemm_f32(ctx, (const float*)A, (const float*)B, nullptr, partials, M, N, K, 0, nullptr, s);
}

#define TRY(expr)                      \
    do {                               \
        const int _rc = (expr);        \
        if (_rc != COMPACT_OK) return _rc; \
    } while (0)

// ---------------------------------------------------------------------------
// prefill
// ---------------------------------------------------------------------------
static int run_attn_prefill(compact_ctx* ctx, const Plan& p, int n_blocks, const void* qkv, const compact_kv* kv, void* o,
                            hipStream_t s) {
    ProfileScope ps(ctx, COMPACT_K_ATTN_PREFILL, s);
    if (ctx->cfg.dtype == COMPACT_BF16)
        return launch_attn_prefill_bf16(ctx, p.d_meta, p.d_q_tiles, (int)p.q_tiles.size(), (const bf16*)qkv,
                                        (const bf16*)kv->d_k, (const bf16*)kv->d_v, (bf16*)o, s);
    return launch_attn_prefill_f32(ctx, p.d_meta, n_blocks, p.max_len, (const float*)qkv, (const float*)kv->d_k,
                                   (const float*)kv->d_v, (float*)o, s);
}

static int moe_ffn_rows(compact_ctx* ctx, const compact_weights* w, const void* m, const void* h, bool h_is_f32,
                        const int32_t* idx, const float* gate, int64_t rows, void* act, const MoePlan& plan,
                        void* expert_out, void* y, hipStream_t s);

static int prefill_impl(compact_ctx* ctx, const compact_weights* w, int n_blocks, const int32_t* cu, const void* x,
                        compact_kv* kv, void* y, void* y_last, const compact_route_out* route, void* ws, size_t ws_bytes,
                        Plan& plan, hipStream_t s) {
    const compact_layer_cfg& c = ctx->cfg;
    const int64_t T = cu[n_blocks];
    Carver cv(ws);
    PrefillBufs b;
    carve_prefill(cv, c, T, b);
    if (cv.off > ws_bytes) return set_err(ctx, COMPACT_EWORKSPACE, "workspace too small for this prefill");
    const int Dq = c.n_q_heads * c.head_dim, Dtot = (c.n_q_heads + 2 * c.n_kv_heads) * c.head_dim;

    if (!plan.d_meta) TRY(upload_plan(ctx, plan, s));   // a depth of layers shares one plan
    TRY(launch_rmsnorm(ctx, x, false, w->g_attn, b.n, T, s));
    TRY(gemm_full(ctx, b.n, w->w_qkv, nullptr, false, b.qkv, T, Dtot, c.d_model, 0, s));
    TRY(launch_rope_kvwrite(ctx, plan.d_meta, plan.d_rope_tiles, (int)plan.rope_tiles.size(), b.qkv, kv->d_k, kv->d_v, s));
    TRY(run_attn_prefill(ctx, plan, n_blocks, b.qkv, kv, b.o, s));
    TRY(gemm_full(ctx, b.o, w->w_o, x, false, b.h, T, c.d_model, Dq, 2, s));   // h = x + o Wo^T, kept in fp32
    TRY(launch_rmsnorm(ctx, b.h, true, w->g_ffn, b.n, T, s));
    if (c.n_experts == 0) {
        TRY(gemm_full(ctx, b.n, w->w_gate_up, nullptr, false, b.act, T, c.ffn_dim, c.d_model, 1, s));
        TRY(gemm_full(ctx, b.act, w->w_down, b.h, true, y, T, c.d_model, c.ffn_dim, 0, s));
    } else {
        int32_t* idx = route && route->d_expert_idx ? route->d_expert_idx : b.idx;
        float* gate = route && route->d_gate ? route->d_gate : b.gate;
        TRY(launch_moe_route(ctx, b.n, w->w_router, T, idx, gate, b.logits, s));
        TRY(moe_ffn_rows(ctx, w, b.n, b.h, true, idx, gate, T, b.act, b.plan, b.expert_out, y, s));
    }
    if (y_last) TRY(launch_gather_last_rows(ctx, plan.d_meta, n_blocks, y, y_last, s));
    return COMPACT_OK;
}

static int validate_prefill(compact_ctx* ctx, const compact_weights* w, int n_blocks, const int32_t* cu, const void* x,
                            compact_kv* kv, void* ws, int extra_rows) {
    TRY(check_blocks(ctx, n_blocks, cu));
    TRY(check_weights(ctx, w));
    if (!x) return set_err(ctx, COMPACT_EINVAL, "null input");
    if (!ws) return set_err(ctx, COMPACT_EWORKSPACE, "null workspace");
    TRY(check_kv(ctx, kv, n_blocks));
    for (int b = 0; b < n_blocks; ++b)
        if ((int64_t)(cu[b + 1] - cu[b]) + extra_rows > kv->h_capacity[b])
            return set_err(ctx, COMPACT_ECAPACITY, "block " + std::to_string(b) + " does not fit its KV slab");
    return COMPACT_OK;
}

extern "C" int compact_prefill(compact_ctx* ctx, const compact_weights* w, int32_t n_blocks, const int32_t* h_cu_seqlens,
                               const void* d_x, compact_kv* kv, void* d_y, const compact_route_out* route,
                               void* d_workspace, size_t ws_bytes, void* hip_stream) {
    if (!ctx) return COMPACT_EINVAL;
    TRY(validate_prefill(ctx, w, n_blocks, h_cu_seqlens, d_x, kv, d_workspace, 0));
    if (!d_y) return set_err(ctx, COMPACT_EINVAL, "null output");
    Plan plan;
    build_prefill_plan(kv, n_blocks, h_cu_seqlens, plan);
    TRY(prefill_impl(ctx, w, n_blocks, h_cu_seqlens, d_x, kv, d_y, nullptr, route, d_workspace, ws_bytes, plan,
                     (hipStream_t)hip_stream));
    for (int b = 0; b < n_blocks; ++b) kv->h_len[b] = h_cu_seqlens[b + 1] - h_cu_seqlens[b];
    return COMPACT_OK;
}

extern "C" int compact_prefill_extend(compact_ctx* ctx, const compact_weights* w, int32_t n_blocks,
                                      const int32_t* h_cu_seqlens, const void* d_x, compact_kv* kv, void* d_y,
                                      const compact_route_out* route, void* d_workspace, size_t ws_bytes, void* hip_stream) {
    if (!ctx) return COMPACT_EINVAL;
    TRY(validate_prefill(ctx, w, n_blocks, h_cu_seqlens, d_x, kv, d_workspace, 0));
    if (!d_y) return set_err(ctx, COMPACT_EINVAL, "null output");
    for (int b = 0; b < n_blocks; ++b) {
        if (kv->h_len[b] < 0) return set_err(ctx, COMPACT_EINVAL, "negative h_len");
        if ((int64_t)kv->h_len[b] + (h_cu_seqlens[b + 1] - h_cu_seqlens[b]) > kv->h_capacity[b])
            return set_err(ctx, COMPACT_ECAPACITY, "block " + std::to_string(b) + ": cached rows + chunk exceed its KV slab");
    }
    Plan plan;
    build_prefill_plan(kv, n_blocks, h_cu_seqlens, plan, true);
    TRY(prefill_impl(ctx, w, n_blocks, h_cu_seqlens, d_x, kv, d_y, nullptr, route, d_workspace, ws_bytes, plan,
                     (hipStream_t)hip_stream));
    for (int b = 0; b < n_blocks; ++b) kv->h_len[b] += h_cu_seqlens[b + 1] - h_cu_seqlens[b];
    return COMPACT_OK;
}

// ---------------------------------------------------------------------------
// decode
// ---------------------------------------------------------------------------
static int run_attn_decode(compact_ctx* ctx, const Plan& p, int n_blocks, int step, const void* q, const compact_kv* kv,
                           float* attn_partials, void* o, hipStream_t s) {
    if (ctx->cfg.dtype == COMPACT_BF16) {
        const int max_chunks = chunks_for(p.max_len + step + 1);
        return launch_attn_decode_bf16(ctx, p.d_meta, p.d_kv_chunks, (int)p.kv_chunks.size(), n_blocks, step, max_chunks,
                                       (const bf16*)q, (const bf16*)kv->d_k, (const bf16*)kv->d_v, attn_partials, (bf16*)o, s);
    }
    return launch_attn_decode_f32(ctx, p.d_meta, n_blocks, step, (const float*)q, (const float*)kv->d_k,
                                  (const float*)kv->d_v, (float*)o, s);
}

// Prefix-aware layout: what the decode step needs besides the per-worker tails.
struct PrefixArgs {
    BlockMeta shared{};           // the one shared block (the whole history)
    const void *d_k, *d_v;        // its slabs
    std::vector<PrefixItem> items;
    std::vector<int32_t> wl_off, wl;
    int64_t total_recs = 0;
    int max_list = 0;
    size_t off_items = 0, off_wl_off = 0, off_wl = 0;   // byte offsets inside Plan::extra
    float* records = nullptr;
};

// Step-by-step callers (compact_decode_step, compact_prefix_decode_step) come back with the same
// caches one token longer each time.  The plan of the first call is built to cover `headroom`
// steps and stays on the device; later calls reuse it with step = k instead of building and
// uploading a new one, as long as nothing else has uploaded metadata in between, the stream and
// the cache geometry are the same and every block has grown by the same k.
struct StepCache {
    bool valid = false;
    uint64_t serial = 0;             // ctx->upload_serial right after this plan went up
    std::vector<int64_t> geom;       // everything the plan depends on except the lengths
    std::vector<int32_t> base_len;   // lengths the plan was built for
    int headroom = 0;                // steps the uploaded lists cover
    Plan plan;
    PrefixArgs pa;
};

static void drop_step_cache(compact_ctx* ctx) {
    delete ctx->step_cache;
    ctx->step_cache = nullptr;
}

// Steps taken since the cached plan was built, or -1 when it does not cover this call.
static int step_cache_lookup(const compact_ctx* ctx, const std::vector<int64_t>& geom, const int32_t* h_len, int n) {
    const StepCache* sc = ctx->step_cache;
    if (!sc || !sc->valid || sc->serial != ctx->upload_serial || sc->geom != geom) return -1;
    const int k = h_len[0] - sc->base_len[0];
    if (k < 0 || k >= sc->headroom) return -1;
    for (int b = 1; b < n; ++b)
        if (h_len[b] - sc->base_len[b] != k) return -1;
    return k;
}

static StepCache& step_cache_begin(compact_ctx* ctx) {
    if (!ctx->step_cache) ctx->step_cache = new StepCache;
    *ctx->step_cache = StepCache();
    return *ctx->step_cache;
}

static void step_cache_commit(compact_ctx* ctx, StepCache& sc, std::vector<int64_t>& geom, const int32_t* h_len, int n,
                              int headroom) {
    sc.geom.swap(geom);
    sc.base_len.assign(h_len, h_len + n);
    sc.headroom = headroom;
    sc.serial = ctx->upload_serial;
    sc.valid = true;
}

// Parts of one decode step: the projections before the attention (rows r0 .. r0 + n_rows - 1 of the step), the
// attention (always all n_total blocks), the projections and the feed-forward half after it (rows again).
enum { DECODE_FRONT = 1, DECODE_ATTN = 2, DECODE_BACK = 4, DECODE_ALL = 7 };
// most rows the decode-step projection kernels take at once (bf16 storage)
constexpr int DECODE_MAX_ROWS = 64;

// plan.meta.len = cached tokens before step 0.  Only the query and attention-output rows travel between the parts; every
// other buffer of `b_all` is scratch that a later group of rows may overwrite (the launches are ordered on the stream).
static int decode_part(compact_ctx* ctx, const compact_weights* w, int n_total, int r0, int n_rows, int part, int step,
                       const void* x_all, compact_kv* kv, void* y_all, const compact_route_out* route_all,
                       const DecodeBufs& b_all, const Plan& plan, hipStream_t s, const PrefixArgs* pfx) {
    const compact_layer_cfg& c = ctx->cfg;
    const int N = n_rows;
    const int Dq = c.n_q_heads * c.head_dim, Dtot = (c.n_q_heads + 2 * c.n_kv_heads) * c.head_dim;
    const size_t es = c.dtype == COMPACT_BF16 ? 2 : 4;
    const void* x = (const char*)x_all + (size_t)r0 * c.d_model * es;
    void* y = (char*)y_all + (size_t)r0 * c.d_model * es;
    DecodeBufs b = b_all;
    b.q = (char*)b_all.q + (size_t)r0 * Dq * es;
    b.o = (char*)b_all.o + (size_t)r0 * Dq * es;
    const BlockMeta* meta = plan.d_meta + r0;
    compact_route_out route_rows{};
    const compact_route_out* route = nullptr;
    if (route_all) {
        route_rows = *route_all;
        if (route_rows.d_expert_idx) route_rows.d_expert_idx += (size_t)r0 * c.top_k;
        if (route_rows.d_gate) route_rows.d_gate += (size_t)r0 * c.top_k;
        route = &route_rows;
    }
    int ks = 1;
    if (part & DECODE_FRONT) {
    // RMSNorm + QKV projection.  bf16 storage: the projection stages bf16(x * g) itself and leaves the row sums of squares, the
    // epilogue multiplies by 1 / rms before the rotation.
    if (c.dtype == COMPACT_BF16 && skinny_norm_in_supported(N, Dtot, c.d_model)) {
        ks = skinny_ksplit(N, Dtot, c.d_model);
        {
            ProfileScope ps(ctx, COMPACT_K_GEMM_SKINNY, s);
            TRY(launch_gemm_skinny(ctx, (const bf16*)x, (const bf16*)w->w_qkv, b.partials, N, Dtot, c.d_model, ks, s,
                                   (const bf16*)w->g_attn, b.ssq_parts));
        }
        RowNorm rq;
        rq.ssq_parts = b.ssq_parts;
        rq.nparts = ks;
        rq.inv_d = 1.0f / (float)c.d_model;
        rq.eps = c.rms_eps;
        TRY(launch_decode_qkv_epilogue(ctx, meta, N, step, b.partials, ks, b.q, kv->d_k, kv->d_v, s, &rq));
    } else {
        TRY(launch_rmsnorm(ctx, x, false, w->g_attn, b.n, N, s));
        TRY(gemm_partials(ctx, b.n, w->w_qkv, b.partials, N, Dtot, c.d_model, &ks, s));
        TRY(launch_decode_qkv_epilogue(ctx, meta, N, step, b.partials, ks, b.q, kv->d_k, kv->d_v, s));
    }
    }
    if ((part & DECODE_ATTN) && pfx) {
        TRY(launch_attn_decode_prefix_bf16(ctx, plan.d_meta, pfx->shared, (const PrefixItem*)(plan.d_extra + pfx->off_items),
                                           (int)pfx->items.size(), (const int32_t*)(plan.d_extra + pfx->off_wl_off),
                                           (const int32_t*)(plan.d_extra + pfx->off_wl), pfx->max_list, n_total, step,
                                           (const bf16*)b_all.q, (const bf16*)pfx->d_k, (const bf16*)pfx->d_v, (const bf16*)kv->d_k,
                                           (const bf16*)kv->d_v, pfx->records, pfx->total_recs, (bf16*)b_all.o, s));
    } else if (part & DECODE_ATTN) {
        TRY(run_attn_decode(ctx, plan, n_total, step, b_all.q, kv, b_all.attn_partials, b_all.o, s));
    }
    if (!(part & DECODE_BACK)) return COMPACT_OK;
    // O projection + residual, and the RMSNorm that feeds the FFN.  bf16 storage with
    // few rows: one whole-K kernel leaves h, the un-normalised FFN input h * g and the
    // row sums of squares; whoever consumes the input applies 1/rms.
    const bool bf = c.dtype == COMPACT_BF16;
    const void* ffn_in = b.m;
    RowNorm rn{};
    bool pending_norm = false;
    // (17 .. 64 rows: the same kernels with several groups of 16 rows per weight fragment, used where the kernel for
    // at most 16 rows covers the shape too, so that both split K alike and a row's bits do not depend on the batch)
    const bool o_few = bf && resid_norm_stream_supported(N, c.d_model, Dq);
    const bool o_many = bf && !o_few && stream_mt_supported(N, c.d_model, Dq) && resid_norm_stream_supported(16, c.d_model, Dq);
    if (o_few || o_many) {
        ProfileScope ps(ctx, COMPACT_K_GEMM_SKINNY, s);
        if (o_few)
            TRY(launch_resid_norm_stream(ctx, (const bf16*)b.o, (const bf16*)w->w_o, (const bf16*)x, (const bf16*)w->g_ffn, b.h,
                                         (bf16*)b.hg, b.ssq_parts, N, c.d_model, Dq, s));
        else
            TRY(launch_resid_norm_stream_mt(ctx, (const bf16*)b.o, (const bf16*)w->w_o, (const bf16*)x, (const bf16*)w->g_ffn,
                                            b.h, (bf16*)b.hg, b.ssq_parts, N, c.d_model, Dq, s));
        rn.ssq_parts = b.ssq_parts;
        rn.nparts = c.d_model / 16;
        rn.inv_d = 1.0f / (float)c.d_model;
        rn.eps = c.rms_eps;
        pending_norm = true;
        ffn_in = b.hg;
    } else {
        TRY(gemm_partials(ctx, b.o, w->w_o, b.partials, N, c.d_model, Dq, &ks, s));
        TRY(launch_residual_norm(ctx, b.partials, ks, x, w->g_ffn, b.h, b.m, N, s));
    }
    if (c.n_experts == 0) {
        if (bf && skinny_swiglu_supported(N, c.ffn_dim, c.d_model)) {
            ProfileScope ps(ctx, COMPACT_K_GEMM_SKINNY, s);
            TRY(launch_gemm_skinny_swiglu(ctx, (const bf16*)ffn_in, (const bf16*)w->w_gate_up, (bf16*)b.act, N, c.ffn_dim,
                                          c.d_model, pending_norm ? &rn : nullptr, s));
        } else if (bf && swiglu_mt_supported(N, c.ffn_dim, c.d_model) && skinny_swiglu_supported(16, c.ffn_dim, c.d_model)) {
            ProfileScope ps(ctx, COMPACT_K_GEMM_SKINNY, s);
            TRY(launch_swiglu_mt(ctx, (const bf16*)ffn_in, (const bf16*)w->w_gate_up, (bf16*)b.act, N, c.ffn_dim, c.d_model,
                                 pending_norm ? &rn : nullptr, s));
        } else {
            if (pending_norm) {
                TRY(launch_rownorm_apply(ctx, (const bf16*)b.hg, rn, (bf16*)b.m, N, c.d_model, s));
                ffn_in = b.m;
            }
            TRY(gemm_partials(ctx, ffn_in, w->w_gate_up, b.partials, N, 2 * c.ffn_dim, c.d_model, &ks, s));
            TRY(launch_swiglu_reduce(ctx, b.partials, ks, b.act, N, c.ffn_dim, s));
        }
        if (bf && resid_out_stream_supported(N, c.d_model, c.ffn_dim)) {
            ProfileScope ps(ctx, COMPACT_K_GEMM_SKINNY, s);
            TRY(launch_resid_out_stream(ctx, (const bf16*)b.act, (const bf16*)w->w_down, b.h, (bf16*)y, N, c.d_model,
                                        c.ffn_dim, s));
        } else {
            // (more than 16 rows: a whole-K workgroup would have to pull all M x F activations through L2 for its 16 columns,
            // four times the weight bytes at 64 rows; measured 49 us against 31 us for split-K + reduce on the 8B-shaped layer)
            TRY(gemm_partials(ctx, b.act, w->w_down, b.partials, N, c.d_model, c.ffn_dim, &ks, s));
            TRY(launch_residual_reduce(ctx, b.partials, ks, b.h, y, N, c.d_model, s));
        }
    } else {
        if (pending_norm) TRY(launch_rownorm_apply(ctx, (const bf16*)b.hg, rn, (bf16*)b.m, N, c.d_model, s));
        int32_t* idx = route && route->d_expert_idx ? route->d_expert_idx : b.idx;
        float* gate = route && route->d_gate ? route->d_gate : b.gate;
        TRY(launch_moe_route(ctx, b.m, w->w_router, N, idx, gate, b.logits, s, b.partials));
        if (bf && N * c.top_k <= 256) {
            // few rows per expert: stream every routed expert's weights once (split-K
            // partials in the expert-sorted row order), SwiGLU, down projection, and a
            // combine that applies the gate weights to the fp32 sums.  The routing plan (one
            // workgroup, at most 256 routed rows = 64 blocks at top-4) cuts every expert's rows
            // into tiles of 16, one grid slice each: an expert with more than 16 rows (possible
            // beyond 16 blocks) is streamed once per tile.
            const int rk = N * c.top_k;
            TRY(launch_moe_plan(ctx, idx, gate, N, 16, b.plan, s));
            const bool q4 = w->w_exp_gate_up_q != nullptr;   // block-scaled 4-bit copy of the experts
            // the tile map lists the tiles (then -1): at most one per routed row, and no more than experts + rows / 16
            const int n_listed = std::min(rk, c.n_experts + rk / 16);
            const int ks1 = q4 ? mxfp4_ksplit(c.d_model) : skinny_ksplit(1, 2 * c.ffn_dim, c.d_model);
            {
                ProfileScope ps(ctx, COMPACT_K_GEMM_SKINNY, s);
                if (q4)
                    TRY(launch_gemm_skinny_grouped_mxfp4(ctx, (const bf16*)b.m, b.plan.sorted_token,
                                                         (const uint8_t*)w->w_exp_gate_up_q, (const uint8_t*)w->w_exp_gate_up_s,
                                                         b.plan.offsets, c.n_experts, rk, b.partials, 2 * c.ffn_dim, c.d_model,
                                                         ks1, s, b.plan.tile_expert, n_listed, b.plan.tile_row0, b.plan.tile_rows));
                else
                    TRY(launch_gemm_skinny_grouped(ctx, (const bf16*)b.m, b.plan.sorted_token, (const bf16*)w->w_exp_gate_up,
                                                   (int64_t)2 * c.ffn_dim * c.d_model, b.plan.offsets, c.n_experts, rk,
                                                   b.partials, 2 * c.ffn_dim, c.d_model, ks1, s, b.plan.tile_expert, n_listed,
                                                   b.plan.tile_row0, b.plan.tile_rows));
            }
            TRY(launch_swiglu_reduce(ctx, b.partials, ks1, b.act, rk, c.ffn_dim, s));
            const int ks2 = q4 ? mxfp4_ksplit(c.ffn_dim) : skinny_ksplit(1, c.d_model, c.ffn_dim);
            {
                ProfileScope ps(ctx, COMPACT_K_GEMM_SKINNY, s);
                if (q4)
                    TRY(launch_gemm_skinny_grouped_mxfp4(ctx, (const bf16*)b.act, nullptr, (const uint8_t*)w->w_exp_down_q,
                                                         (const uint8_t*)w->w_exp_down_s, b.plan.offsets, c.n_experts, rk,
                                                         b.partials, c.d_model, c.ffn_dim, ks2, s, b.plan.tile_expert, n_listed,
                                                         b.plan.tile_row0, b.plan.tile_rows));
                else
                    TRY(launch_gemm_skinny_grouped(ctx, (const bf16*)b.act, nullptr, (const bf16*)w->w_exp_down,
                                                   (int64_t)c.d_model * c.ffn_dim, b.plan.offsets, c.n_experts, rk, b.partials,
                                                   c.d_model, c.ffn_dim, ks2, s, b.plan.tile_expert, n_listed, b.plan.tile_row0,
                                                   b.plan.tile_rows));
            }
            TRY(launch_moe_combine_partials(ctx, b.partials, ks2, rk, b.h, b.plan.slot_of, b.plan.sorted_gate, N, y, s));
        } else {
            TRY(moe_ffn_rows(ctx, w, b.m, b.h, true, idx, gate, N, b.act, b.plan, b.expert_out, y, s));
        }
    }
    return COMPACT_OK;
}

// one decode step for all blocks.  bf16 storage with more than DECODE_MAX_ROWS blocks: the projections run group of
// rows after group of rows (each group streams the weights once more), the attention once for all blocks; a block's
// bits are those of the kernels for 17 .. 64 rows whatever its group.
static int decode_impl(compact_ctx* ctx, const compact_weights* w, int n_blocks, int step, const void* x,
                       compact_kv* kv, void* y, const compact_route_out* route, const DecodeBufs& b,
                       const Plan& plan, hipStream_t s, const PrefixArgs* pfx = nullptr) {
    if (ctx->cfg.dtype != COMPACT_BF16 || n_blocks <= DECODE_MAX_ROWS)
        return decode_part(ctx, w, n_blocks, 0, n_blocks, DECODE_ALL, step, x, kv, y, route, b, plan, s, pfx);
    // as few groups as possible, of (nearly) equal size: at least 33 rows each, so that every row goes through the
    // kernel family for 17 .. 64 rows
    const int n_groups = (n_blocks + DECODE_MAX_ROWS - 1) / DECODE_MAX_ROWS;
    const int per = (n_blocks + n_groups - 1) / n_groups;
    for (int r0 = 0; r0 < n_blocks; r0 += per)
        TRY(decode_part(ctx, w, n_blocks, r0, std::min(per, n_blocks - r0), DECODE_FRONT, step, x, kv, y, route, b, plan, s, pfx));
    TRY(decode_part(ctx, w, n_blocks, 0, n_blocks, DECODE_ATTN, step, x, kv, y, route, b, plan, s, pfx));
    for (int r0 = 0; r0 < n_blocks; r0 += per)
        TRY(decode_part(ctx, w, n_blocks, r0, std::min(per, n_blocks - r0), DECODE_BACK, step, x, kv, y, route, b, plan, s, pfx));
    return COMPACT_OK;
}

static int validate_decode(compact_ctx* ctx, const compact_weights* w, int n_blocks, const void* x, compact_kv* kv,
                           void* y, void* ws, int n_steps) {
    if (n_blocks < 1) return set_err(ctx, COMPACT_EINVAL, "n_blocks must be >= 1");
    TRY(check_weights(ctx, w));
    if (!x || !y) return set_err(ctx, COMPACT_EINVAL, "null input or output");
    if (!ws) return set_err(ctx, COMPACT_EWORKSPACE, "null workspace");
    TRY(check_kv(ctx, kv, n_blocks));
    for (int b = 0; b < n_blocks; ++b) {
        if (kv->h_len[b] < 0) return set_err(ctx, COMPACT_EINVAL, "negative h_len");
        if ((int64_t)kv->h_len[b] + n_steps > kv->h_capacity[b])
            return set_err(ctx, COMPACT_ECAPACITY, "block " + std::to_string(b) + ": len + steps exceeds its KV slab");
    }
    return COMPACT_OK;
}

// Steps one uploaded decode plan is built to cover (bounded by the room left in the slabs).
constexpr int STEP_PLAN_HEADROOM = 1024;

extern "C" int compact_decode_step(compact_ctx* ctx, const compact_weights* w, int32_t n_blocks, const void* d_x,
                                   compact_kv* kv, void* d_y, const compact_route_out* route, void* d_workspace,
                                   size_t ws_bytes, void* hip_stream) {
    if (!ctx) return COMPACT_EINVAL;
    TRY(validate_decode(ctx, w, n_blocks, d_x, kv, d_y, d_workspace, 1));
    hipStream_t s = (hipStream_t)hip_stream;
    int max_len = 0, room = STEP_PLAN_HEADROOM;
    std::vector<int64_t> geom = {0, (int64_t)(intptr_t)s, n_blocks};
    for (int b = 0; b < n_blocks; ++b) {
        max_len = std::max(max_len, kv->h_len[b]);
        room = std::min(room, kv->h_capacity[b] - kv->h_len[b]);
        geom.push_back(kv->h_capacity[b]);
        geom.push_back(kv->h_pos_offset ? kv->h_pos_offset[b] : 0);
        geom.push_back(kv->h_slab_offset[b]);
    }
    Carver cv(d_workspace);
    DecodeBufs b;
    carve_decode(cv, ctx->cfg, n_blocks, chunks_for(max_len + 1), b);
    if (cv.off > ws_bytes) return set_err(ctx, COMPACT_EWORKSPACE, "workspace too small for this decode step");
    int k = step_cache_lookup(ctx, geom, kv->h_len, n_blocks);
    if (k < 0) {
        StepCache& sc = step_cache_begin(ctx);
        build_decode_plan(kv, n_blocks, sc.plan);
        add_kv_chunks(sc.plan, room);
        TRY(upload_plan(ctx, sc.plan, s));
        step_cache_commit(ctx, sc, geom, kv->h_len, n_blocks, room);
        k = 0;
    }
    TRY(decode_impl(ctx, w, n_blocks, k, d_x, kv, d_y, route, b, ctx->step_cache->plan, s));
    for (int b2 = 0; b2 < n_blocks; ++b2) kv->h_len[b2] += 1;
    return COMPACT_OK;
}

extern "C" int compact_layer_forward(compact_ctx* ctx, const compact_weights* w, int32_t n_blocks,
                                     const int32_t* h_cu_seqlens, const void* d_x_prefill, int32_t n_steps,
                                     const void* d_x_decode, compact_kv* kv, void* d_y_prefill, void* d_y_last,
                                     void* d_y_decode, void* d_workspace, size_t ws_bytes, void* hip_stream) {
    if (!ctx) return COMPACT_EINVAL;
    if (n_steps < 0) return set_err(ctx, COMPACT_EINVAL, "n_steps must be >= 0");
    TRY(validate_prefill(ctx, w, n_blocks, h_cu_seqlens, d_x_prefill, kv, d_workspace, n_steps));
    if (n_steps > 0 && (!d_x_decode || !d_y_decode)) return set_err(ctx, COMPACT_EINVAL, "null decode input or output");
    const compact_layer_cfg& c = ctx->cfg;
    hipStream_t s = (hipStream_t)hip_stream;
    Plan plan;
    build_prefill_plan(kv, n_blocks, h_cu_seqlens, plan);
    if (n_steps > 0) add_kv_chunks(plan, n_steps);
    const int64_t T = h_cu_seqlens[n_blocks];

    // workspace: [prefill region][prefill y if the caller wants none][decode region]
    Carver cp(d_workspace);
    PrefillBufs pb;
    carve_prefill(cp, c, T, pb);
    size_t off = align_up(cp.off, 256);
    void* y_pre = d_y_prefill;
    if (!y_pre) {
        // the FFN output may overwrite the attention scratch that is dead by then (carve_prefill
        // gives it max(Dq + 2 Dkv, d_model) columns per row, so [T, d_model] fits)
        y_pre = pb.qkv;
    }
    Carver cd(d_workspace ? (char*)d_workspace + off : nullptr);
    DecodeBufs db;
    carve_decode(cd, c, n_blocks, chunks_for(plan.max_len + n_steps), db);
    if (off + cd.off > ws_bytes) return set_err(ctx, COMPACT_EWORKSPACE, "workspace too small for this forward pass");

    TRY(prefill_impl(ctx, w, n_blocks, h_cu_seqlens, d_x_prefill, kv, y_pre, d_y_last, nullptr, d_workspace, off, plan, s));
    const size_t row_bytes = (size_t)n_blocks * c.d_model * dtype_size(c.dtype);
    // every step is self-contained (as in autoregressive use, where a step's input exists
    // only once the previous step has finished): nothing is hoisted across steps
    for (int st = 0; st < n_steps; ++st) {
        TRY(decode_impl(ctx, w, n_blocks, st, (const char*)d_x_decode + st * row_bytes, kv,
                        (char*)d_y_decode + st * row_bytes, nullptr, db, plan, s));
    }
    for (int b = 0; b < n_blocks; ++b) kv->h_len[b] = h_cu_seqlens[b + 1] - h_cu_seqlens[b] + n_steps;
    return COMPACT_OK;
}

// ---------------------------------------------------------------------------
// mixed batches: prefill chunks of some blocks together with decode tokens of others
// ---------------------------------------------------------------------------
extern "C" int compact_mixed_workspace_bytes(const compact_ctx* ctx, int32_t max_batched_tokens, int32_t max_blocks,
                                             int32_t max_kv_len, size_t* bytes) {
    size_t one = 0;
    const int rc = compact_workspace_bytes(ctx, max_batched_tokens, max_blocks, max_kv_len, &one);
    if (rc != COMPACT_OK) return rc;
    const size_t es = dtype_size(ctx->cfg.dtype);
    // packed input and output rows of a mixed step, and of a decode-only step
    *bytes = one + 2 * align_up((size_t)max_batched_tokens * ctx->cfg.d_model * es, 256) +
             2 * align_up((size_t)max_blocks * ctx->cfg.d_model * es, 256) + 256;
    return COMPACT_OK;
}

namespace {
struct MixExtra {   // byte offsets inside Plan::extra of one mixed step
    size_t dec_meta = 0, qrow = 0, src_tab = 0, dst_tab = 0;
};
template <typename T>
size_t put(std::vector<char>& buf, const std::vector<T>& v) {
    const size_t off = align_up(buf.size(), 256);
    buf.resize(off + v.size() * sizeof(T));
    if (!v.empty()) memcpy(buf.data() + off, v.data(), v.size() * sizeof(T));
    return off;
}
}  // namespace

extern "C" int compact_mixed_forward(compact_ctx* ctx, const compact_weights* w, int32_t n_blocks,
                                     const int32_t* h_cu_seqlens, const void* d_x_prefill, int32_t n_steps,
                                     const void* d_x_decode, compact_kv* kv, int32_t max_batched_tokens, void* d_y_last,
                                     void* d_y_decode, void* d_workspace, size_t ws_bytes, void* hip_stream) {
    if (!ctx) return COMPACT_EINVAL;
    if (n_steps < 0) return set_err(ctx, COMPACT_EINVAL, "n_steps must be >= 0");
    TRY(validate_prefill(ctx, w, n_blocks, h_cu_seqlens, d_x_prefill, kv, d_workspace, n_steps));
    if (n_steps > 0 && (!d_x_decode || !d_y_decode)) return set_err(ctx, COMPACT_EINVAL, "null decode input or output");
    if (max_batched_tokens <= n_blocks)
        return set_err(ctx, COMPACT_EINVAL, "max_batched_tokens must exceed n_blocks (every decoding block takes one row)");
    const compact_layer_cfg& c = ctx->cfg;
    hipStream_t s = (hipStream_t)hip_stream;
    const int N = n_blocks, S = n_steps, TM = max_batched_tokens;
    const size_t es = dtype_size(c.dtype);
    const bool bf = c.dtype == COMPACT_BF16;
    const int Dq = c.n_q_heads * c.head_dim, Dtot = (c.n_q_heads + 2 * c.n_kv_heads) * c.head_dim;
    int max_len = 0;
    for (int b = 0; b < N; ++b) max_len = std::max(max_len, h_cu_seqlens[b + 1] - h_cu_seqlens[b]);

    // workspace: [prefill region for TM rows][decode region for N blocks][xp, yp: TM rows][xs, ys: N rows]
    Carver cp(d_workspace);
    PrefillBufs pb;
    carve_prefill(cp, c, TM, pb);
    const size_t off = align_up(cp.off, 256);
    Carver cd((char*)d_workspace + off);
    DecodeBufs db;
    const int max_chunks = chunks_for(max_len + S);
    carve_decode(cd, c, N, max_chunks, db);
    size_t end = off + align_up(cd.off, 256);
    char* base = (char*)d_workspace;
    void* xp = base + end;
    end += align_up((size_t)TM * c.d_model * es, 256);
    void* yp = base + end;
    end += align_up((size_t)TM * c.d_model * es, 256);
    void* xs = base + end;
    end += align_up((size_t)N * c.d_model * es, 256);
    void* ys = base + end;
    end += align_up((size_t)N * c.d_model * es, 256);
    if (end > ws_bytes) return set_err(ctx, COMPACT_EWORKSPACE, "workspace too small for this mixed pass");

    std::vector<int> done(N, 0), sdone(N, 0);   // prefilled rows / finished decode steps per block
    for (int b = 0; b < N; ++b) kv->h_len[b] = 0;
    for (;;) {
        std::vector<int> dec, pre;
        for (int b = 0; b < N; ++b) {
            const int L = h_cu_seqlens[b + 1] - h_cu_seqlens[b];
            if (done[b] < L)
                pre.push_back(b);
            else if (sdone[b] < S)
                dec.push_back(b);
        }
        if (pre.empty() && dec.empty()) break;

        if (pre.empty()) {
            // ---- decode-only step over the blocks that still have steps left ----------
            const int n = (int)dec.size();
            Plan plan;
            plan.meta.resize(n);
            std::vector<int32_t> src_tab(n), dst_tab(n);
            for (int i = 0; i < n; ++i) {
                const int b = dec[i];
                BlockMeta& m = plan.meta[i];
                m.row0 = i;
                m.len = kv->h_len[b];
                m.capacity = kv->h_capacity[b];
                m.pos_offset = kv->h_pos_offset ? kv->h_pos_offset[b] : 0;
                m.slab = kv->h_slab_offset[b];
                plan.max_len = std::max(plan.max_len, m.len);
                src_tab[i] = -(sdone[b] * N + b) - 2;    // row of x_decode [S * N, d] (base 1)
                dst_tab[i] = sdone[b] * N + b;           // row of y_decode (base 0)
            }
            add_kv_chunks(plan, 1);
            MixExtra mx;
            mx.src_tab = put(plan.extra, src_tab);
            mx.dst_tab = put(plan.extra, dst_tab);
            TRY(upload_plan(ctx, plan, s));
            TRY(launch_move_rows(ctx, nullptr, d_x_decode, (const int32_t*)(plan.d_extra + mx.src_tab), xs, nullptr, nullptr, n, s));
            TRY(decode_impl(ctx, w, n, 0, xs, kv, ys, nullptr, db, plan, s));
            TRY(launch_move_rows(ctx, ys, nullptr, nullptr, d_y_decode, nullptr, (const int32_t*)(plan.d_extra + mx.dst_tab), n, s));
            for (int b : dec) {
                sdone[b] += 1;
                kv->h_len[b] += 1;
            }
            continue;
        }

        // ---- mixed step: chunks of the blocks still in prefill (block order, within the
        // token budget), one token of every block that is decoding -------------------
        int budget = TM - (int)dec.size();
        Plan plan;
        std::vector<int> part, rows_of;   // participating blocks and their rows in this step
        for (int b : pre) {
            if (budget == 0) break;
            const int L = h_cu_seqlens[b + 1] - h_cu_seqlens[b];
            const int cnt = std::min(L - done[b], budget);
            part.push_back(b);
            rows_of.push_back(cnt);
            budget -= cnt;
        }
        const int n_chunk = (int)part.size(), n_dec = (int)dec.size();
        for (int b : dec) {
            part.push_back(b);
            rows_of.push_back(1);
        }
        const int n_part = (int)part.size();
        plan.meta.resize(n_part);
        std::vector<BlockMeta> dec_meta(n_dec);
        std::vector<int32_t> qrow(n_dec), src_tab, dst_tab;
        int Tm = 0;
        for (int i = 0; i < n_part; ++i) {
            const int b = part[i], cnt = rows_of[i];
            BlockMeta& m = plan.meta[i];
            m.row0 = Tm;
            m.len = cnt;
            m.prior = kv->h_len[b];
            m.capacity = kv->h_capacity[b];
            m.pos_offset = kv->h_pos_offset ? kv->h_pos_offset[b] : 0;
            m.slab = kv->h_slab_offset[b];
            plan.max_len = std::max(plan.max_len, cnt);
            for (int r = 0; r < cnt; r += ROPE_TILE) plan.rope_tiles.push_back({i, r});
            if (i < n_chunk) {
                const int L = h_cu_seqlens[b + 1] - h_cu_seqlens[b];
                if (bf)
                    for (int r = 0; r < cnt; r += PREFILL_QTILE) plan.q_tiles.push_back({i, r});
                for (int r = 0; r < cnt; ++r) {
                    src_tab.push_back(h_cu_seqlens[b] + done[b] + r);                       // row of x_prefill (base 0)
                    dst_tab.push_back(d_y_last && done[b] + r == L - 1 ? -b - 2 : -1);      // the block's last row -> y_last[b]
                }
            } else {
                const int j = i - n_chunk;
                dec_meta[j] = m;
                dec_meta[j].row0 = j;
                dec_meta[j].len = m.prior;   // cached rows before this token; the token's own row is written first
                dec_meta[j].prior = 0;
                qrow[j] = Tm;
                for (int r = 0; r < m.prior + 1; r += DECODE_CHUNK) plan.kv_chunks.push_back({j, r});
                src_tab.push_back(-(sdone[b] * N + b) - 2);
                dst_tab.push_back(sdone[b] * N + b);
            }
            Tm += cnt;
        }
        {
            const std::vector<BlockMeta>& mt = plan.meta;
            std::stable_sort(plan.q_tiles.begin(), plan.q_tiles.end(), [&mt](const TileItem& a, const TileItem& b2) {
                return mt[a.block].prior + a.row0 > mt[b2.block].prior + b2.row0;
            });
        }
        MixExtra mx;
        mx.dec_meta = put(plan.extra, dec_meta);
        mx.qrow = put(plan.extra, qrow);
        mx.src_tab = put(plan.extra, src_tab);
        mx.dst_tab = put(plan.extra, dst_tab);
        TRY(upload_plan(ctx, plan, s));
        const int32_t* d_src = (const int32_t*)(plan.d_extra + mx.src_tab);
        const int32_t* d_dst = (const int32_t*)(plan.d_extra + mx.dst_tab);

        TRY(launch_move_rows(ctx, d_x_prefill, d_x_decode, d_src, xp, nullptr, nullptr, Tm, s));
        TRY(launch_rmsnorm(ctx, xp, false, w->g_attn, pb.n, Tm, s));
        TRY(gemm_full(ctx, pb.n, w->w_qkv, nullptr, false, pb.qkv, Tm, Dtot, c.d_model, 0, s));
        TRY(launch_rope_kvwrite(ctx, plan.d_meta, plan.d_rope_tiles, (int)plan.rope_tiles.size(), pb.qkv, kv->d_k, kv->d_v, s));
        if (bf) {
            {
                ProfileScope ps(ctx, COMPACT_K_ATTN_PREFILL, s);
                TRY(launch_attn_prefill_bf16(ctx, plan.d_meta, plan.d_q_tiles, (int)plan.q_tiles.size(), (const bf16*)pb.qkv,
                                             (const bf16*)kv->d_k, (const bf16*)kv->d_v, (bf16*)pb.o, s));
            }
            if (n_dec > 0)   // one query row per decoding block, read in place from the packed QKV rows
                TRY(launch_attn_decode_bf16(ctx, (const BlockMeta*)(plan.d_extra + mx.dec_meta), plan.d_kv_chunks,
                                            (int)plan.kv_chunks.size(), n_dec, 0, max_chunks, (const bf16*)pb.qkv,
                                            (const bf16*)kv->d_k, (const bf16*)kv->d_v, db.attn_partials, (bf16*)pb.o, s,
                                            (const int32_t*)(plan.d_extra + mx.qrow), Dtot));
        } else {
            // fp32 storage: a decoding block is a chunk of one row to the plain kernel
            TRY(launch_attn_prefill_f32(ctx, plan.d_meta, n_part, plan.max_len, (const float*)pb.qkv, (const float*)kv->d_k,
                                        (const float*)kv->d_v, (float*)pb.o, s));
        }
        TRY(gemm_full(ctx, pb.o, w->w_o, xp, false, pb.h, Tm, c.d_model, Dq, 2, s));
        TRY(launch_rmsnorm(ctx, pb.h, true, w->g_ffn, pb.n, Tm, s));
        if (c.n_experts == 0) {
            TRY(gemm_full(ctx, pb.n, w->w_gate_up, nullptr, false, pb.act, Tm, c.ffn_dim, c.d_model, 1, s));
            TRY(gemm_full(ctx, pb.act, w->w_down, pb.h, true, yp, Tm, c.d_model, c.ffn_dim, 0, s));
        } else {
            TRY(launch_moe_route(ctx, pb.n, w->w_router, Tm, pb.idx, pb.gate, pb.logits, s));
            TRY(moe_ffn_rows(ctx, w, pb.n, pb.h, true, pb.idx, pb.gate, Tm, pb.act, pb.plan, pb.expert_out, yp, s));
        }
        TRY(launch_move_rows(ctx, yp, nullptr, nullptr, d_y_decode, d_y_last, d_dst, Tm, s));

        for (int i = 0; i < n_part; ++i) {
            const int b = part[i];
            kv->h_len[b] += rows_of[i];
            if (i < n_chunk)
                done[b] += rows_of[i];
            else
                sdone[b] += 1;
        }
    }
    return COMPACT_OK;
}

// ---------------------------------------------------------------------------
// a depth of layers
// ---------------------------------------------------------------------------
extern "C" int compact_stack_workspace_bytes(const compact_ctx* ctx, int64_t max_tokens, int32_t max_blocks,
                                             int32_t max_kv_len, size_t* bytes) {
    size_t one = 0;
    const int rc = compact_workspace_bytes(ctx, max_tokens, max_blocks, max_kv_len, &one);
    if (rc != COMPACT_OK) return rc;
    const size_t es = dtype_size(ctx->cfg.dtype);
    // two [T, d] and two [N, d] hand-over buffers behind one layer's workspace
    *bytes = one + 2 * align_up((size_t)max_tokens * ctx->cfg.d_model * es, 256) +
             2 * align_up((size_t)max_blocks * ctx->cfg.d_model * es, 256) + 256;
    return COMPACT_OK;
}

extern "C" int compact_stack_forward(compact_ctx* ctx, int32_t n_layers, const compact_weights* w, int32_t n_blocks,
                                     const int32_t* h_cu_seqlens, const void* d_x_prefill, int32_t n_steps,
                                     const void* d_x_decode, compact_kv* kv, void* d_y_last, void* d_y_decode,
                                     void* d_workspace, size_t ws_bytes, void* hip_stream) {
    if (!ctx) return COMPACT_EINVAL;
    if (n_layers < 1) return set_err(ctx, COMPACT_EINVAL, "n_layers must be >= 1");
    if (n_steps < 0) return set_err(ctx, COMPACT_EINVAL, "n_steps must be >= 0");
    if (!w || !kv) return set_err(ctx, COMPACT_EINVAL, "null per-layer weights or caches");
    for (int l = 0; l < n_layers; ++l) {
        TRY(validate_prefill(ctx, &w[l], n_blocks, h_cu_seqlens, d_x_prefill, &kv[l], d_workspace, n_steps));
        for (int b = 0; l > 0 && b < n_blocks; ++b) {
            const bool same = kv[l].h_capacity[b] == kv[0].h_capacity[b] && kv[l].h_slab_offset[b] == kv[0].h_slab_offset[b] &&
                              (kv[l].h_pos_offset ? kv[l].h_pos_offset[b] : 0) == (kv[0].h_pos_offset ? kv[0].h_pos_offset[b] : 0);
            if (!same) return set_err(ctx, COMPACT_EINVAL, "the caches of all layers must share one geometry");
        }
    }
    if (n_steps > 0 && (!d_x_decode || !d_y_decode)) return set_err(ctx, COMPACT_EINVAL, "null decode input or output");
    const compact_layer_cfg& c = ctx->cfg;
    hipStream_t s = (hipStream_t)hip_stream;
    Plan plan;
    build_prefill_plan(&kv[0], n_blocks, h_cu_seqlens, plan);
    if (n_steps > 0) add_kv_chunks(plan, n_steps);
    const int64_t T = h_cu_seqlens[n_blocks];
    const size_t es = dtype_size(c.dtype);

    // workspace: [one layer's prefill region][decode region][two [T, d]][two [N, d]]
    Carver cp(d_workspace);
    PrefillBufs pb;
    carve_prefill(cp, c, T, pb);
    const size_t off = align_up(cp.off, 256);
    Carver cd(d_workspace ? (char*)d_workspace + off : nullptr);
    DecodeBufs db;
    carve_decode(cd, c, n_blocks, chunks_for(plan.max_len + n_steps), db);
    size_t end = off + align_up(cd.off, 256);
    char* base = (char*)d_workspace;
    void* big[2];
    void* small[2];
    for (int i = 0; i < 2; ++i) {
        big[i] = base + end;
        end += align_up((size_t)T * c.d_model * es, 256);
    }
    for (int i = 0; i < 2; ++i) {
        small[i] = base + end;
        end += align_up((size_t)n_blocks * c.d_model * es, 256);
    }
    if (end > ws_bytes) return set_err(ctx, COMPACT_EWORKSPACE, "workspace too small for this stack");

    const void* x = d_x_prefill;
    for (int l = 0; l < n_layers; ++l) {
        void* y = big[l & 1];
        TRY(prefill_impl(ctx, &w[l], n_blocks, h_cu_seqlens, x, &kv[l], y, l == n_layers - 1 ? d_y_last : nullptr, nullptr,
                         d_workspace, off, plan, s));
        x = y;
    }
    const size_t row_bytes = (size_t)n_blocks * c.d_model * es;
    for (int st = 0; st < n_steps; ++st) {
        const void* xs = (const char*)d_x_decode + st * row_bytes;
        for (int l = 0; l < n_layers; ++l) {
            void* ys = l == n_layers - 1 ? (void*)((char*)d_y_decode + st * row_bytes) : small[l & 1];
            TRY(decode_impl(ctx, &w[l], n_blocks, st, xs, &kv[l], ys, nullptr, db, plan, s));
            xs = ys;
        }
    }
    for (int l = 0; l < n_layers; ++l)
        for (int b = 0; b < n_blocks; ++b) kv[l].h_len[b] = h_cu_seqlens[b + 1] - h_cu_seqlens[b] + n_steps;
    return COMPACT_OK;
}

// ---------------------------------------------------------------------------
// prefix-aware layout: shared prefix + private tails
// ---------------------------------------------------------------------------
static int64_t prefix_max_recs(const compact_layer_cfg& c, int n_workers, int max_prefix_len, int max_tail_len) {
    const int G = c.n_q_heads / c.n_kv_heads;
    return ((int64_t)prefix_chunks_for(max_prefix_len) * n_workers + (int64_t)n_workers * prefix_chunks_for(max_tail_len + 1)) * G;
}

extern "C" int compact_prefix_workspace_bytes(const compact_ctx* ctx, int32_t n_workers, int32_t max_prefix_len,
                                              int32_t max_tail_len, size_t* bytes) {
    if (!ctx || !bytes) return COMPACT_EINVAL;
    compact_ctx* c = const_cast<compact_ctx*>(ctx);
    if (n_workers < 1 || max_prefix_len < 0 || max_tail_len < 1)
        return set_err(c, COMPACT_EINVAL, "n_workers >= 1, max_prefix_len >= 0, max_tail_len >= 1 required");
    Carver cd(nullptr);
    DecodeBufs db;
    carve_decode(cd, ctx->cfg, n_workers, 1, db);
    const size_t recs = (size_t)prefix_max_recs(ctx->cfg, n_workers, max_prefix_len, max_tail_len) * ctx->cfg.n_kv_heads *
                        (ctx->cfg.head_dim + 2) * 4;
    *bytes = align_up(cd.off, 256) + align_up(recs, 256) + 256;
    return COMPACT_OK;
}

// Validates the prefix-aware arguments and builds the tail metadata, the work items and the
// per-worker item lists.  `steps` = tokens this call appends to every tail.
static int build_prefix_plan(compact_ctx* ctx, int n_workers, const compact_kv* shared, const int32_t* h_prefix_len,
                             const compact_kv* tails, int steps, Plan& plan, PrefixArgs& pa) {
    const compact_layer_cfg& c = ctx->cfg;
    if (c.dtype != COMPACT_BF16) return set_err(ctx, COMPACT_EUNSUPPORTED, "the prefix-aware decode path exists for bf16 storage only");
    if (n_workers < 1 || n_workers > 64) return set_err(ctx, COMPACT_EINVAL, "n_workers must be in 1..64");
    if (!h_prefix_len) return set_err(ctx, COMPACT_EINVAL, "null h_prefix_len");
    TRY(check_kv(ctx, shared, 1));
    TRY(check_kv(ctx, tails, n_workers));
    const int shared_len = shared->h_len[0];
    if (shared_len < 0 || shared_len > shared->h_capacity[0]) return set_err(ctx, COMPACT_ECAPACITY, "shared h_len must be in 0..capacity");
    for (int b = 0; b < n_workers; ++b) {
        if (h_prefix_len[b] < 0 || h_prefix_len[b] > shared_len)
            return set_err(ctx, COMPACT_EINVAL, "h_prefix_len[b] must be in 0..shared h_len");
        if (b > 0 && h_prefix_len[b] < h_prefix_len[b - 1])
            return set_err(ctx, COMPACT_EINVAL, "h_prefix_len must not decrease (every worker's prefix extends the previous one's)");
        if (tails->h_len[b] < 0 || (int64_t)tails->h_len[b] + steps > tails->h_capacity[b])
            return set_err(ctx, COMPACT_ECAPACITY, "worker " + std::to_string(b) + ": tail len + steps exceeds its slab");
    }
    plan.meta.resize(n_workers);
    for (int b = 0; b < n_workers; ++b) {
        BlockMeta& m = plan.meta[b];
        m.row0 = b;
        m.len = tails->h_len[b];
        m.capacity = tails->h_capacity[b];
        m.pos_offset = h_prefix_len[b];   // the new token's rotary position is prefix_len + tail len
        m.slab = tails->h_slab_offset[b];
        plan.max_len = std::max(plan.max_len, m.len);
    }
    pa.shared.row0 = 0;
    pa.shared.len = shared_len;
    pa.shared.capacity = shared->h_capacity[0];
    pa.shared.pos_offset = 0;
    pa.shared.slab = shared->h_slab_offset[0];
    pa.d_k = shared->d_k;
    pa.d_v = shared->d_v;
    const int G = c.n_q_heads / c.n_kv_heads;
    const int max_prefix = h_prefix_len[n_workers - 1];
    std::vector<std::vector<int32_t>> lists(n_workers);
    int32_t rec = 0;
    int w0 = 0;
    for (int r0 = 0; r0 < max_prefix; r0 += PREFIX_CHUNK) {
        while (h_prefix_len[w0] <= r0) ++w0;   // first worker whose prefix reaches into the chunk
        PrefixItem it{r0, std::min(PREFIX_CHUNK, max_prefix - r0), w0, n_workers - w0, 0, rec};
        for (int b = w0; b < n_workers; ++b) lists[b].push_back((int32_t)pa.items.size());
        pa.items.push_back(it);
        rec += it.nw * G;
    }
    for (int b = 0; b < n_workers; ++b)
        for (int r0 = 0; r0 < tails->h_len[b] + steps; r0 += PREFIX_CHUNK) {
            PrefixItem it{r0, PREFIX_CHUNK, b, 1, 1, rec};
            lists[b].push_back((int32_t)pa.items.size());
            pa.items.push_back(it);
            rec += G;
        }
    pa.total_recs = rec;
    pa.wl_off.assign(1, 0);
    for (int b = 0; b < n_workers; ++b) {
        pa.max_list = std::max(pa.max_list, (int)lists[b].size());
        pa.wl.insert(pa.wl.end(), lists[b].begin(), lists[b].end());
        pa.wl_off.push_back((int32_t)pa.wl.size());
    }
    // pack the tables behind the plan's lists
    pa.off_items = 0;
    pa.off_wl_off = align_up(pa.items.size() * sizeof(PrefixItem), 16);
    pa.off_wl = pa.off_wl_off + align_up(pa.wl_off.size() * 4, 16);
    plan.extra.assign(pa.off_wl + pa.wl.size() * 4 + 16, 0);
    memcpy(plan.extra.data() + pa.off_items, pa.items.data(), pa.items.size() * sizeof(PrefixItem));
    memcpy(plan.extra.data() + pa.off_wl_off, pa.wl_off.data(), pa.wl_off.size() * 4);
    if (!pa.wl.empty()) memcpy(plan.extra.data() + pa.off_wl, pa.wl.data(), pa.wl.size() * 4);
    return COMPACT_OK;
}

extern "C" int compact_prefix_decode_step(compact_ctx* ctx, const compact_weights* w, int32_t n_workers, const void* d_x,
                                          const compact_kv* shared, const int32_t* h_prefix_len, compact_kv* tails,
                                          void* d_y, const compact_route_out* route, void* d_workspace, size_t ws_bytes,
                                          void* hip_stream) {
    if (!ctx) return COMPACT_EINVAL;
    TRY(check_weights(ctx, w));
    if (!d_x || !d_y) return set_err(ctx, COMPACT_EINVAL, "null input or output");
    if (!d_workspace) return set_err(ctx, COMPACT_EWORKSPACE, "null workspace");
    if (!shared || !tails) return set_err(ctx, COMPACT_EINVAL, "null shared or tails");
    hipStream_t s = (hipStream_t)hip_stream;
    // a plan built for one step covers every further step that opens no new chunk in any tail
    // (the record slots, hence the workspace, stay the same) and still fits the slabs
    int k = -1, room = PREFIX_CHUNK;
    std::vector<int64_t> geom;
    if (ctx->step_cache && ctx->step_cache->valid && h_prefix_len && n_workers >= 1 && n_workers <= 64 &&
        shared->d_k && shared->d_v && shared->h_len && shared->h_capacity && shared->h_slab_offset && tails->d_k &&
        tails->d_v && tails->h_len && tails->h_capacity && tails->h_slab_offset) {
        geom = {1, (int64_t)(intptr_t)s, n_workers, shared->h_len[0], shared->h_capacity[0], shared->h_slab_offset[0]};
        for (int b = 0; b < n_workers; ++b) {
            geom.push_back(h_prefix_len[b]);
            geom.push_back(tails->h_capacity[b]);
            geom.push_back(tails->h_slab_offset[b]);
        }
        k = step_cache_lookup(ctx, geom, tails->h_len, n_workers);
    }
    if (k < 0) {
        Plan plan;
        PrefixArgs pa;
        TRY(build_prefix_plan(ctx, n_workers, shared, h_prefix_len, tails, 1, plan, pa));   // validates everything
        geom = {1, (int64_t)(intptr_t)s, n_workers, shared->h_len[0], shared->h_capacity[0], shared->h_slab_offset[0]};
        for (int b = 0; b < n_workers; ++b) {
            geom.push_back(h_prefix_len[b]);
            geom.push_back(tails->h_capacity[b]);
            geom.push_back(tails->h_slab_offset[b]);
            const int len = tails->h_len[b];
            room = std::min(room, std::min(tails->h_capacity[b] - len, prefix_chunks_for(len + 1) * PREFIX_CHUNK - len));
        }
        Carver cv(d_workspace);
        DecodeBufs b;
        carve_decode(cv, ctx->cfg, n_workers, 1, b);
        (void)cv.take((size_t)pa.total_recs * ctx->cfg.n_kv_heads * (ctx->cfg.head_dim + 2) * 4);
        if (cv.off > ws_bytes) return set_err(ctx, COMPACT_EWORKSPACE, "workspace too small for this prefix-aware decode step");
        StepCache& sc = step_cache_begin(ctx);
        sc.plan = std::move(plan);
        sc.pa = std::move(pa);
        TRY(upload_plan(ctx, sc.plan, s));
        step_cache_commit(ctx, sc, geom, tails->h_len, n_workers, room);
        k = 0;
    }
    StepCache& sc = *ctx->step_cache;
    Carver cv(d_workspace);
    DecodeBufs b;
    carve_decode(cv, ctx->cfg, n_workers, 1, b);
    sc.pa.records = (float*)cv.take((size_t)sc.pa.total_recs * ctx->cfg.n_kv_heads * (ctx->cfg.head_dim + 2) * 4);
    if (cv.off > ws_bytes) return set_err(ctx, COMPACT_EWORKSPACE, "workspace too small for this prefix-aware decode step");
    sc.pa.d_k = shared->d_k;
    sc.pa.d_v = shared->d_v;
    TRY(decode_impl(ctx, w, n_workers, k, d_x, tails, d_y, route, b, sc.plan, s, &sc.pa));
    for (int b2 = 0; b2 < n_workers; ++b2) tails->h_len[b2] += 1;
    return COMPACT_OK;
}

extern "C" int compact_prefix_stack_workspace_bytes(const compact_ctx* ctx, int64_t history_tokens, int32_t n_workers,
                                                    int32_t max_tail_len, size_t* bytes) {
    size_t pre = 0, dec = 0;
    int rc = compact_workspace_bytes(ctx, history_tokens, 1, 1, &pre);
    if (rc != COMPACT_OK) return rc;
    if (history_tokens > INT32_MAX) return set_err(const_cast<compact_ctx*>(ctx), COMPACT_EINVAL, "history too long");
    rc = compact_prefix_workspace_bytes(ctx, n_workers, (int32_t)history_tokens, max_tail_len, &dec);
    if (rc != COMPACT_OK) return rc;
    const size_t es = dtype_size(ctx->cfg.dtype);
    *bytes = pre + dec + 2 * align_up((size_t)history_tokens * ctx->cfg.d_model * es, 256) +
             2 * align_up((size_t)n_workers * ctx->cfg.d_model * es, 256) + 256;
    return COMPACT_OK;
}

extern "C" int compact_prefix_stack_forward(compact_ctx* ctx, int32_t n_layers, const compact_weights* w, int32_t n_workers,
                                            const int32_t* h_prefix_len, int64_t history_tokens, const void* d_x_history,
                                            int32_t n_steps, const void* d_x_decode, compact_kv* shared, compact_kv* tails,
                                            void* d_y_decode, void* d_workspace, size_t ws_bytes, void* hip_stream) {
    if (!ctx) return COMPACT_EINVAL;
    if (n_layers < 1) return set_err(ctx, COMPACT_EINVAL, "n_layers must be >= 1");
    if (n_steps < 0) return set_err(ctx, COMPACT_EINVAL, "n_steps must be >= 0");
    if (!w || !shared || !tails) return set_err(ctx, COMPACT_EINVAL, "null per-layer weights or caches");
    if (history_tokens < 1 || history_tokens > INT32_MAX) return set_err(ctx, COMPACT_EINVAL, "history_tokens must be >= 1");
    if (n_steps > 0 && (!d_x_decode || !d_y_decode)) return set_err(ctx, COMPACT_EINVAL, "null decode input or output");
    const compact_layer_cfg& c = ctx->cfg;
    hipStream_t s = (hipStream_t)hip_stream;
    const int N = n_workers;
    const int32_t T = (int32_t)history_tokens;
    const int32_t cu[2] = {0, T};
    for (int l = 0; l < n_layers; ++l) TRY(validate_prefill(ctx, &w[l], 1, cu, d_x_history, &shared[l], d_workspace, 0));
    // the decode plan doubles as the argument check of the prefix-aware part (layer 0's caches, with the
    // shared length the prefill below will leave); the other layers must share that geometry
    Plan dplan;
    PrefixArgs pa;
    {
        const int32_t before = shared[0].h_len[0];
        shared[0].h_len[0] = T;
        const int rc = build_prefix_plan(ctx, N, &shared[0], h_prefix_len, &tails[0], n_steps, dplan, pa);
        shared[0].h_len[0] = before;   // nothing is changed until every check has passed
        if (rc != COMPACT_OK) return rc;
    }
    for (int l = 1; l < n_layers; ++l) {
        TRY(check_kv(ctx, &tails[l], N));
        bool same = shared[l].h_capacity[0] == shared[0].h_capacity[0] && shared[l].h_slab_offset[0] == shared[0].h_slab_offset[0];
        for (int b = 0; same && b < N; ++b)
            same = tails[l].h_capacity[b] == tails[0].h_capacity[b] && tails[l].h_slab_offset[b] == tails[0].h_slab_offset[b] &&
                   tails[l].h_len[b] == tails[0].h_len[b];
        if (!same) return set_err(ctx, COMPACT_EINVAL, "the caches of all layers must share one geometry");
    }
    const size_t es = dtype_size(c.dtype);

    // workspace: [prefill region for the history][decode region][records][two [T, d]][two [N, d]]
    Carver cp(d_workspace);
    PrefillBufs pb;
    carve_prefill(cp, c, T, pb);
    const size_t off = align_up(cp.off, 256);
    Carver cd((char*)d_workspace + off);
    DecodeBufs db;
    carve_decode(cd, c, N, 1, db);
    pa.records = (float*)cd.take((size_t)pa.total_recs * c.n_kv_heads * (c.head_dim + 2) * 4);
    size_t end = off + align_up(cd.off, 256);
    char* base = (char*)d_workspace;
    void *big[2], *small[2];
    for (int i = 0; i < 2; ++i) {
        big[i] = base + end;
        end += align_up((size_t)T * c.d_model * es, 256);
    }
    for (int i = 0; i < 2; ++i) {
        small[i] = base + end;
        end += align_up((size_t)N * c.d_model * es, 256);
    }
    if (end > ws_bytes) return set_err(ctx, COMPACT_EWORKSPACE, "workspace too small for this prefix-aware stack");
    for (int l = 0; l < n_layers; ++l) shared[l].h_len[0] = T;

    // every layer prefills the whole history as one causal block: its cache serves all workers
    Plan pplan;
    build_prefill_plan(&shared[0], 1, cu, pplan);
    const void* x = d_x_history;
    for (int l = 0; l < n_layers; ++l) {
        void* y = big[l & 1];
        TRY(prefill_impl(ctx, &w[l], 1, cu, x, &shared[l], y, nullptr, nullptr, d_workspace, off, pplan, s));
        x = y;
    }
    if (n_steps > 0) TRY(upload_plan(ctx, dplan, s));   // behind the prefill kernels on the stream
    const size_t row_bytes = (size_t)N * c.d_model * es;
    for (int st = 0; st < n_steps; ++st) {
        const void* xs = (const char*)d_x_decode + st * row_bytes;
        for (int l = 0; l < n_layers; ++l) {
            void* ys = l == n_layers - 1 ? (void*)((char*)d_y_decode + st * row_bytes) : small[l & 1];
            pa.d_k = shared[l].d_k;
            pa.d_v = shared[l].d_v;
            TRY(decode_impl(ctx, &w[l], N, st, xs, &tails[l], ys, nullptr, db, dplan, s, &pa));
            xs = ys;
        }
    }
    for (int l = 0; l < n_layers; ++l)
        for (int b = 0; b < N; ++b) tails[l].h_len[b] += n_steps;
    return COMPACT_OK;
}

extern "C" int compact_attn_decode_prefix(compact_ctx* ctx, int32_t n_workers, const void* d_q, const compact_kv* shared,
                                          const int32_t* h_prefix_len, const compact_kv* tails, void* d_o,
                                          void* d_workspace, size_t ws_bytes, void* hip_stream) {
    if (!ctx) return COMPACT_EINVAL;
    if (!d_q || !d_o) return set_err(ctx, COMPACT_EINVAL, "null q or o");
    if (!shared || !tails) return set_err(ctx, COMPACT_EINVAL, "null shared or tails");
    hipStream_t s = (hipStream_t)hip_stream;
    Plan plan;
    PrefixArgs pa;
    // the hook attends tail rows 0 .. h_len-1: plan it as the step that appended the last of them
    for (int b = 0; b < n_workers && tails->h_len; ++b)
        if (tails->h_len[b] < 1) return set_err(ctx, COMPACT_EINVAL, "every tail must hold at least the current token");
    TRY(build_prefix_plan(ctx, n_workers, shared, h_prefix_len, tails, 0, plan, pa));
    for (auto& m : plan.meta) m.len -= 1;
    const size_t need = (size_t)pa.total_recs * ctx->cfg.n_kv_heads * (ctx->cfg.head_dim + 2) * 4;
    if (!d_workspace || ws_bytes < need) return set_err(ctx, COMPACT_EWORKSPACE, "workspace too small for the prefix-aware records");
    TRY(upload_plan(ctx, plan, s));
    return launch_attn_decode_prefix_bf16(ctx, plan.d_meta, pa.shared, (const PrefixItem*)(plan.d_extra + pa.off_items),
                                          (int)pa.items.size(), (const int32_t*)(plan.d_extra + pa.off_wl_off),
                                          (const int32_t*)(plan.d_extra + pa.off_wl), pa.max_list, n_workers, 0, (const bf16*)d_q,
                                          (const bf16*)shared->d_k, (const bf16*)shared->d_v, (const bf16*)tails->d_k,
                                          (const bf16*)tails->d_v, (float*)d_workspace, pa.total_recs, (bf16*)d_o, s);
}

// ---------------------------------------------------------------------------
// MoE feed-forward over rows with given routing (shared by prefill and hooks)
// ---------------------------------------------------------------------------
static int moe_ffn_rows(compact_ctx* ctx, const compact_weights* w, const void* m, const void* h, bool h_is_f32,
                        const int32_t* idx, const float* gate, int64_t rows, void* act, const MoePlan& plan,
                        void* expert_out, void* y, hipStream_t s) {
    const compact_layer_cfg& c = ctx->cfg;
    const int64_t rk = rows * c.top_k;
    TRY(launch_moe_plan(ctx, idx, gate, rows, moe_mtile(c), plan, s));
    GroupedArgs g{};
    g.tile_expert = plan.tile_expert;
    g.tile_row0 = plan.tile_row0;
    g.tile_rows = plan.tile_rows;
    g.n_mtiles = plan.max_mtiles;
    // gate/up + SwiGLU on the rows gathered per expert
    g.a_gather = plan.sorted_token;
    g.row_scale = nullptr;
    g.b_expert_stride = (int64_t)2 * c.ffn_dim * c.d_model;
    if (c.dtype == COMPACT_BF16) {
        ProfileScope ps(ctx, COMPACT_K_GEMM, s);
        TRY(launch_gemm_bf16(ctx, (const bf16*)m, (const bf16*)w->w_exp_gate_up, nullptr, false, (bf16*)act, rk,
                             c.ffn_dim, c.d_model, 1, &g, s));
    } else {
        TRY(launch_gemm_f32(ctx, (const float*)m, (const float*)w->w_exp_gate_up, nullptr, (float*)act, rk, c.ffn_dim,
                            c.d_model, 1, &g, s));
    }
    // down projection, each row scaled by its gate weight
    g.a_gather = nullptr;
    g.row_scale = plan.sorted_gate;
    g.b_expert_stride = (int64_t)c.d_model * c.ffn_dim;
    if (c.dtype == COMPACT_BF16) {
        ProfileScope ps(ctx, COMPACT_K_GEMM, s);
        TRY(launch_gemm_bf16(ctx, (const bf16*)act, (const bf16*)w->w_exp_down, nullptr, false, (bf16*)expert_out, rk,
                             c.d_model, c.ffn_dim, 0, &g, s));
    } else {
        TRY(launch_gemm_f32(ctx, (const float*)act, (const float*)w->w_exp_down, nullptr, (float*)expert_out, rk,
                            c.d_model, c.ffn_dim, 0, &g, s));
    }
    return launch_moe_combine(ctx, expert_out, h, h_is_f32, plan.slot_of, rows, y, s);
}

// ---------------------------------------------------------------------------
// per-kernel entry points
// ---------------------------------------------------------------------------
extern "C" int compact_rmsnorm(compact_ctx* ctx, const void* d_x, const void* d_g, void* d_y, int64_t rows,
                               void* hip_stream) {
    if (!ctx) return COMPACT_EINVAL;
    if (!d_x || !d_g || !d_y || rows < 0) return set_err(ctx, COMPACT_EINVAL, "null pointer or negative rows");
    return launch_rmsnorm(ctx, d_x, false, d_g, d_y, rows, (hipStream_t)hip_stream);
}

extern "C" int compact_rope_kvwrite(compact_ctx* ctx, int32_t n_blocks, const int32_t* h_cu_seqlens, void* d_qkv,
                                    compact_kv* kv, void* hip_stream) {
    if (!ctx) return COMPACT_EINVAL;
    TRY(check_blocks(ctx, n_blocks, h_cu_seqlens));
    if (!d_qkv) return set_err(ctx, COMPACT_EINVAL, "null qkv");
    TRY(check_kv(ctx, kv, n_blocks));
    for (int b = 0; b < n_blocks; ++b)
        if (h_cu_seqlens[b + 1] - h_cu_seqlens[b] > kv->h_capacity[b])
            return set_err(ctx, COMPACT_ECAPACITY, "block does not fit its KV slab");
    hipStream_t s = (hipStream_t)hip_stream;
    Plan plan;
    build_prefill_plan(kv, n_blocks, h_cu_seqlens, plan);
    TRY(upload_plan(ctx, plan, s));
    TRY(launch_rope_kvwrite(ctx, plan.d_meta, plan.d_rope_tiles, (int)plan.rope_tiles.size(), d_qkv, kv->d_k, kv->d_v, s));
    for (int b = 0; b < n_blocks; ++b) kv->h_len[b] = h_cu_seqlens[b + 1] - h_cu_seqlens[b];
    return COMPACT_OK;
}

extern "C" int compact_gemm(compact_ctx* ctx, const void* d_a, const void* d_b, const void* d_r, void* d_c, int64_t M,
                            int32_t N, int32_t K, int32_t epilogue, void* d_workspace, size_t ws_bytes,
                            void* hip_stream) {
    if (!ctx) return COMPACT_EINVAL;
    if (!d_a || !d_b || !d_c) return set_err(ctx, COMPACT_EINVAL, "null operand");
    if (M < 0 || N < 1 || K < 1) return set_err(ctx, COMPACT_EINVAL, "bad GEMM shape");
    if (epilogue != 0 && epilogue != 1) return set_err(ctx, COMPACT_EINVAL, "epilogue must be 0 or 1");
    if (ctx->cfg.dtype == COMPACT_BF16 && (K % 64 != 0 || N % 8 != 0))
        return set_err(ctx, COMPACT_ESHAPE, "bf16 GEMM needs K % 64 == 0 and N % 8 == 0");
    hipStream_t s = (hipStream_t)hip_stream;
    // rows at or below the decode batch limit take the weight-streaming kernel
    if (ctx->cfg.dtype == COMPACT_BF16 && M <= 64 && M > 0 && epilogue == 0 && d_workspace) {
        const int ks = skinny_ksplit((int)M, N, K);
        if ((size_t)ks * M * N * 4 > ws_bytes) return set_err(ctx, COMPACT_EWORKSPACE, "workspace too small for split-K partials");
        {
            ProfileScope ps(ctx, COMPACT_K_GEMM_SKINNY, s);
            TRY(launch_gemm_skinny(ctx, (const bf16*)d_a, (const bf16*)d_b, (float*)d_workspace, (int)M, N, K, ks, s));
        }
        return launch_skinny_finish(ctx, (const float*)d_workspace, ks, (const bf16*)d_r, (bf16*)d_c, (int)M, N, s);
    }
    return gemm_full(ctx, d_a, d_b, d_r, false, d_c, M, N, K, epilogue, s);
}

extern "C" int compact_attn_prefill(compact_ctx* ctx, int32_t n_blocks, const int32_t* h_cu_seqlens, const void* d_qkv,
                                    const compact_kv* kv, void* d_o, void* hip_stream) {
    if (!ctx) return COMPACT_EINVAL;
    TRY(check_blocks(ctx, n_blocks, h_cu_seqlens));
    if (!d_qkv || !d_o) return set_err(ctx, COMPACT_EINVAL, "null qkv or o");
    TRY(check_kv(ctx, kv, n_blocks));
    for (int b = 0; b < n_blocks; ++b)
        if (h_cu_seqlens[b + 1] - h_cu_seqlens[b] > kv->h_capacity[b])
            return set_err(ctx, COMPACT_ECAPACITY, "block does not fit its KV slab");
    hipStream_t s = (hipStream_t)hip_stream;
    Plan plan;
    build_prefill_plan(kv, n_blocks, h_cu_seqlens, plan);
    TRY(upload_plan(ctx, plan, s));
    return run_attn_prefill(ctx, plan, n_blocks, d_qkv, kv, d_o, s);
}

extern "C" int compact_attn_decode(compact_ctx* ctx, int32_t n_blocks, const void* d_q, const compact_kv* kv, void* d_o,
                                   void* d_workspace, size_t ws_bytes, void* hip_stream) {
    if (!ctx) return COMPACT_EINVAL;
    if (n_blocks < 1) return set_err(ctx, COMPACT_EINVAL, "n_blocks must be >= 1");
    if (!d_q || !d_o) return set_err(ctx, COMPACT_EINVAL, "null q or o");
    TRY(check_kv(ctx, kv, n_blocks));
    for (int b = 0; b < n_blocks; ++b)
        if (kv->h_len[b] < 1 || kv->h_len[b] > kv->h_capacity[b])
            return set_err(ctx, COMPACT_ECAPACITY, "h_len must be in 1..capacity");
    hipStream_t s = (hipStream_t)hip_stream;
    Plan plan;
    build_decode_plan(kv, n_blocks, plan);
    for (auto& m : plan.meta) m.len -= 1;  // the kernels attend rows 0..len inclusive
    plan.max_len -= 1;
    add_kv_chunks(plan, 1);
    const size_t need = attn_decode_partial_floats(ctx->cfg, n_blocks, chunks_for(plan.max_len + 1)) * 4;
    if (ctx->cfg.dtype == COMPACT_BF16 && (!d_workspace || ws_bytes < need))
        return set_err(ctx, COMPACT_EWORKSPACE, "workspace too small for the split-KV partials");
    TRY(upload_plan(ctx, plan, s));
    return run_attn_decode(ctx, plan, n_blocks, 0, d_q, kv, (float*)d_workspace, d_o, s);
}

// ---------------------------------------------------------------------------
// decode attention for callers that cannot allocate
// ---------------------------------------------------------------------------
// The split-KV partial records and the work list live in one file-scope device array
// instead of the caller's workspace and the context's metadata buffer.  Every GPU the
// library runs on holds its own copy of the array, at its own address, until the
// process ends; host code reaches it only through the address hipGetSymbolAddress
// returns for the current device (the array's name is a host-side stand-in, never a
// device address).  The work list is written by a small kernel from values passed as
// kernel arguments, so nothing is copied from host memory either.
#define NOALLOC_MAX_BLOCKS 64
#define NOALLOC_MAX_CHUNKS 4096
#define NOALLOC_META_BYTES ((size_t)64 << 10)      // BlockMeta[64] (2 KB) + TileItem[4096] (32 KB)
#define NOALLOC_PARTIAL_BYTES ((size_t)32 << 20)
static __device__ __align__(256) unsigned char scratch[NOALLOC_META_BYTES + NOALLOC_PARTIAL_BYTES];

#define NOALLOC_MAX_DEVICES 64
static std::mutex g_scratch_mu;
static unsigned char* g_scratch_ptr[NOALLOC_MAX_DEVICES] = {};

// device address of the current device's copy of `scratch` (looked up once per device)
static int scratch_of_current_device(compact_ctx* ctx, unsigned char** out) {
    int dev = -1;
    HIP_TRY(ctx, hipGetDevice(&dev));
    if (dev < 0 || dev >= NOALLOC_MAX_DEVICES) return set_err(ctx, COMPACT_EHIP, "device ordinal out of range");
    std::lock_guard<std::mutex> lk(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        HIP_TRY(ctx, hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return set_err(ctx, COMPACT_EHIP, "hipGetSymbolAddress returned a null address");
        g_scratch_ptr[dev] = (unsigned char*)p;
    }
    *out = g_scratch_ptr[dev];
    return COMPACT_OK;
}

struct NoallocPlanArgs {          // passed by value as a kernel argument (1.3 KB)
    int32_t n_blocks;
    int32_t len[NOALLOC_MAX_BLOCKS];
    int32_t capacity[NOALLOC_MAX_BLOCKS];
    int64_t slab[NOALLOC_MAX_BLOCKS];
};

// One wavefront: lane b writes block b's record and, after a prefix sum of the chunk
// counts over the wavefront, that block's (block, first row) chunk items in block order
// (the order the host-built lists of the other entry points have).
__global__ __launch_bounds__(64) void noalloc_plan_kernel(NoallocPlanArgs a, BlockMeta* meta, TileItem* chunks) {
    const int b = threadIdx.x;
    int nch = 0;
    if (b < a.n_blocks) {
        BlockMeta m;
        m.row0 = b;
        m.len = a.len[b] - 1;        // the attention kernels attend rows 0 .. len inclusive
        m.capacity = a.capacity[b];
        m.pos_offset = 0;
        m.slab = a.slab[b];
        m.prior = 0;
        m.pad_ = 0;
        meta[b] = m;
        nch = (a.len[b] + DECODE_CHUNK - 1) / DECODE_CHUNK;
    }
    int incl = nch;
#pragma unroll
    for (int ofs = 1; ofs < 64; ofs <<= 1) {
        const int v = __shfl_up(incl, ofs, 64);
        if (b >= ofs) incl += v;
    }
    const int first = incl - nch;
    for (int i = 0; i < nch; ++i) chunks[first + i] = TileItem{b, i * DECODE_CHUNK};
}

extern "C" int compact_attn_decode_noalloc(compact_ctx* ctx, int32_t n_blocks, const void* d_q, const compact_kv* kv,
                                           void* d_o, void* hip_stream) {
    if (!ctx) return COMPACT_EINVAL;
    if (ctx->cfg.dtype != COMPACT_BF16) return set_err(ctx, COMPACT_EUNSUPPORTED, "the allocation-free decode attention is built for bf16 storage");
    if (n_blocks < 1) return set_err(ctx, COMPACT_EINVAL, "n_blocks must be >= 1");
    if (!d_q || !d_o) return set_err(ctx, COMPACT_EINVAL, "null q or o");
    TRY(check_kv(ctx, kv, n_blocks));
    if (n_blocks > NOALLOC_MAX_BLOCKS)
        return set_err(ctx, COMPACT_ECAPACITY, "more than 64 blocks: beyond the fixed scratch of the allocation-free entry point");
    NoallocPlanArgs a;
    memset(&a, 0, sizeof(a));
    a.n_blocks = n_blocks;
    int max_len = 0;
    int64_t n_chunks = 0;
    for (int b = 0; b < n_blocks; ++b) {
        if (kv->h_len[b] < 1 || kv->h_len[b] > kv->h_capacity[b])
            return set_err(ctx, COMPACT_ECAPACITY, "h_len must be in 1..capacity");
        a.len[b] = kv->h_len[b];
        a.capacity[b] = kv->h_capacity[b];
        a.slab[b] = kv->h_slab_offset[b];
        max_len = std::max(max_len, kv->h_len[b]);
        n_chunks += chunks_for(kv->h_len[b]);
    }
    const int max_chunks = chunks_for(max_len);
    if (n_chunks > NOALLOC_MAX_CHUNKS)
        return set_err(ctx, COMPACT_ECAPACITY, "more than 4096 chunks of 256 cached rows in total: beyond the fixed scratch of the allocation-free entry point");
    if (attn_decode_partial_floats(ctx->cfg, n_blocks, max_chunks) * 4 > NOALLOC_PARTIAL_BYTES)
        return set_err(ctx, COMPACT_ECAPACITY, "split-KV records (n_blocks * n_q_heads * chunks of the longest cache * (head_dim + 2) floats) exceed the 32 MiB scratch of the allocation-free entry point");
    hipStream_t s = (hipStream_t)hip_stream;
    unsigned char* base = nullptr;
    TRY(scratch_of_current_device(ctx, &base));
    BlockMeta* meta = (BlockMeta*)base;
    TileItem* chunks = (TileItem*)(base + align_up(sizeof(BlockMeta) * NOALLOC_MAX_BLOCKS, 256));
    float* partials = (float*)(base + NOALLOC_META_BYTES);
    // Nothing in the scratch has to start at zero: the plan kernel writes every record and item the
    // attention kernels read, and the combine reads only partial records the same call has written.
    noalloc_plan_kernel<<<1, 64, 0, s>>>(a, meta, chunks);
    LAUNCH_CHECK(ctx);
    const int keep = ctx->profile_class;   // the per-kernel timer creates events on demand: not through this entry point
    ctx->profile_class = COMPACT_K_NONE;
    const int rc = launch_attn_decode_bf16(ctx, meta, chunks, (int)n_chunks, n_blocks, 0, max_chunks, (const bf16*)d_q,
                                           (const bf16*)kv->d_k, (const bf16*)kv->d_v, partials, (bf16*)d_o, s);
    ctx->profile_class = keep;
    return rc;
}

extern "C" int compact_mxfp4_dequant(compact_ctx* ctx, const void* d_codes, const void* d_scales, int64_t rows, int32_t K,
                                     void* d_out, void* hip_stream) {
    if (!ctx) return COMPACT_EINVAL;
    if (!d_codes || !d_scales || !d_out) return set_err(ctx, COMPACT_EINVAL, "null codes, scales or output");
    if (rows < 0) return set_err(ctx, COMPACT_EINVAL, "rows must be >= 0");
    return launch_mxfp4_dequant(ctx, (const uint8_t*)d_codes, (const uint8_t*)d_scales, (bf16*)d_out, rows, K,
                                (hipStream_t)hip_stream);
}

extern "C" int compact_moe_route(compact_ctx* ctx, const void* d_m, const void* d_w_router, int64_t rows,
                                 int32_t* d_expert_idx, float* d_gate, float* d_logits, void* d_workspace,
                                 size_t ws_bytes, void* hip_stream) {
    if (!ctx) return COMPACT_EINVAL;
    if (ctx->cfg.n_experts == 0) return set_err(ctx, COMPACT_EINVAL, "layer has no experts");
    if (!d_m || !d_w_router || !d_expert_idx || !d_gate || rows < 0) return set_err(ctx, COMPACT_EINVAL, "null pointer or negative rows");
    float* logits = d_logits;
    if (!logits) {
        if (!d_workspace || ws_bytes < (size_t)rows * ctx->cfg.n_experts * 4)
            return set_err(ctx, COMPACT_EWORKSPACE, "workspace too small for the router logits");
        logits = (float*)d_workspace;
    }
    return launch_moe_route(ctx, d_m, d_w_router, rows, d_expert_idx, d_gate, logits, (hipStream_t)hip_stream);
}

extern "C" int compact_moe_ffn(compact_ctx* ctx, const compact_weights* w, const void* d_m, const void* d_h,
                               const int32_t* d_expert_idx, const float* d_gate, int64_t rows, void* d_y,
                               void* d_workspace, size_t ws_bytes, void* hip_stream) {
    if (!ctx) return COMPACT_EINVAL;
    if (ctx->cfg.n_experts == 0) return set_err(ctx, COMPACT_EINVAL, "layer has no experts");
    TRY(check_weights(ctx, w));
    if (!d_m || !d_h || !d_expert_idx || !d_gate || !d_y || rows < 0) return set_err(ctx, COMPACT_EINVAL, "null pointer or negative rows");
    const compact_layer_cfg& c = ctx->cfg;
    const size_t es = dtype_size(c.dtype);
    Carver cv(d_workspace);
    void* act = cv.take((size_t)rows * c.top_k * c.ffn_dim * es);
    MoePlan plan;
    carve_moe_plan(cv, c, rows, plan, moe_mtile(c));
    void* expert_out = cv.take((size_t)rows * c.top_k * c.d_model * es);
    if (!d_workspace || cv.off > ws_bytes) return set_err(ctx, COMPACT_EWORKSPACE, "workspace too small for the expert feed-forward");
    return moe_ffn_rows(ctx, w, d_m, d_h, false, d_expert_idx, d_gate, rows, act, plan, expert_out, d_y, (hipStream_t)hip_stream);
}
