// Internal declarations shared by the translation units of libcompact.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include <string>
#include <vector>

#include "../../include/compact.h"

typedef __bf16 bf16;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

#define WAVE 64

// Chunk of cached tokens that gives one split-KV record of the decode attention
// (one work item of its kernel).  Fixed, so that the split of a block's cache
// depends on that block's length only.
#define DECODE_CHUNK 256
// The same for the prefix-aware (cascade) decode attention.
#define PREFIX_CHUNK 256
// Query rows per prefill-attention tile and token rows per rotary/KV-write tile.
#define PREFILL_QTILE 128
#define ROPE_TILE 64

// Per-block metadata as the kernels see it (device copy lives in the context).
struct BlockMeta {
    int32_t row0;        // first packed row of the block (prefill) / unused in decode
    int32_t len;         // prefill: L_b; decode: cached tokens before this call
    int32_t capacity;    // slab rows
    int32_t pos_offset;  // added to the block-local index to get the rotary position
    int64_t slab;        // element offset of the block's slabs in d_k / d_v
    int32_t prior;       // prefill of a further chunk: rows the cache already holds (row i of the call is cache row prior + i)
    int32_t pad_;
};

// Per-row 1/rms handed from one kernel to the next as per-column-group sums of
// squares [nparts][rows] (null ssq_parts: the rows are already normalised).
struct RowNorm {
    const float* ssq_parts = nullptr;
    int nparts = 0;
    float inv_d = 0.f, eps = 0.f;
};

struct TileItem {  // (block, first block-local row) of a row tile
    int32_t block;
    int32_t row0;
};

// Work item of the prefix-aware decode attention: rows row0 .. row0 + n_rows - 1 of
// the shared slab (tail = 0) for workers w0 .. w0 + nw - 1, or a chunk of worker w0's
// private tail slab (tail = 1, nw = 1; its live rows follow from the tail length).
// rec0 = index of the item's first (worker, head-in-group) record.
struct PrefixItem {
    int32_t row0, n_rows, w0, nw, tail, rec0;
};

struct ProfileSlot {
    hipEvent_t start, stop;
};

struct compact_ctx {
    compact_layer_cfg cfg;
    std::string err;
    // device metadata (allocated on first use)
    void* d_meta = nullptr;
    void* h_stage = nullptr;      // pinned staging copy of the metadata
    hipEvent_t stage_event = nullptr;
    bool stage_pending = false;
    size_t meta_bytes = 0;
    uint64_t upload_serial = 0;          // counts metadata uploads: whoever cached device views checks it
    struct StepCache* step_cache = nullptr;   // plan kept between step-by-step decode calls (owned; see api.hip)
    // profiling
    int profile_class = COMPACT_K_NONE;
    std::vector<ProfileSlot> prof_events;
    size_t prof_used = 0;
    int64_t prof_launches = 0;
    double prof_ms = 0.0;
    int n_cus = 0;                       // compute units of the device, 0 = not looked up yet
};

// RAII-free helper used by launchers: brackets a launch with events when its
// class is the one being profiled.
struct ProfileScope {
    compact_ctx* ctx;
    hipStream_t stream;
    bool on;
    ProfileSlot slot;
    ProfileScope(compact_ctx* c, int klass, hipStream_t s);
    ~ProfileScope();
};

int set_err(compact_ctx* ctx, int code, const std::string& msg);
// compute units of the current device (looked up once per context); COMPACT_OK or an error code
int device_cu_count(compact_ctx* ctx, int* n_cus);
#define HIP_TRY(ctx, expr)                                                             \
    do {                                                                               \
        hipError_t _e = (expr);                                                        \
        if (_e != hipSuccess)                                                          \
            return set_err(ctx, COMPACT_EHIP, std::string(#expr) + ": " + hipGetErrorString(_e)); \
    } while (0)
#define LAUNCH_CHECK(ctx) HIP_TRY(ctx, hipGetLastError())

// 16-byte global load whose result goes straight into LDS: lane l of the wave
// deposits its 16 bytes at lds_base + 16 * l (lds_base is wave-uniform); the
// global address is per lane.  Completion is tracked by the vector-memory counter.
__device__ __forceinline__ void load16_to_lds(const void* gptr, void* lds_base) {
#if defined(__HIP_DEVICE_COMPILE__)
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)gptr,
                                     (__attribute__((address_space(3))) void*)lds_base, 16, 0, 0);
#else
    (void)gptr;
    (void)lds_base;
#endif
}
__device__ __forceinline__ void wait_all_memory() {
#if defined(__HIP_DEVICE_COMPILE__)
    __builtin_amdgcn_s_waitcnt(0);
#endif
}

static inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
static inline size_t dtype_size(int dtype) { return dtype == COMPACT_BF16 ? 2 : 4; }

// ---------------------------------------------------------------------------
// kernel launchers (one translation unit each)
// ---------------------------------------------------------------------------

// norm_rope.hip
// x_is_f32: the input rows are fp32 (the prefill residual stream) instead of the storage type
int launch_rmsnorm(compact_ctx* ctx, const void* x, bool x_is_f32, const void* g, void* y, int64_t rows, hipStream_t s);
int launch_rope_kvwrite(compact_ctx* ctx, const BlockMeta* d_meta, const TileItem* d_tiles, int n_tiles,
                        void* qkv, void* d_k, void* d_v, hipStream_t s);
// decode: reduce ks split partials of the QKV projection, rotate, append K/V, emit q
// norm (nullable): the partials were formed from un-normalised rows; every row is
// multiplied by its 1 / rms first
int launch_decode_qkv_epilogue(compact_ctx* ctx, const BlockMeta* d_meta, int n_blocks, int step,
                               const float* partials, int ks, void* q_out, void* d_k, void* d_v,
                               hipStream_t s, const RowNorm* norm = nullptr);
// decode: h = resid + sum partials; writes h and m = RMSNorm(h; g)
int launch_residual_norm(compact_ctx* ctx, const float* partials, int ks, const void* resid,
                         const void* g, void* h_out, void* m_out, int rows, hipStream_t s);
// decode: act = silu(gate) * up from ks partials of the stacked gate/up projection
int launch_swiglu_reduce(compact_ctx* ctx, const float* partials, int ks, void* act, int rows, int F,
                         hipStream_t s);
// decode: y = resid + sum partials
int launch_residual_reduce(compact_ctx* ctx, const float* partials, int ks, const void* resid, void* y,
                           int rows, int cols, hipStream_t s);
// copies the last row of every block of y [T, d] to y_last [N, d]
// rows between packed buffers and the caller's (table value v >= 0: row v of base 0, v <= -2: row -v-2 of base 1,
// -1: skip; null table: row i of base 0)
int launch_move_rows(compact_ctx* ctx, const void* src0, const void* src1, const int32_t* src_tab, void* dst0, void* dst1,
                     const int32_t* dst_tab, int rows, hipStream_t s);
int launch_gather_last_rows(compact_ctx* ctx, const BlockMeta* d_meta, int n_blocks, const void* y,
                            void* y_last, hipStream_t s);

// row-tile map of a grouped (per-expert) GEMM
struct GroupedArgs {          // all device pointers; null tile_expert => plain GEMM
    const int32_t* tile_expert;   // [n_mtiles] expert of every row tile (-1 = no work)
    const int32_t* tile_row0;     // [n_mtiles] first row (in expert-sorted order)
    const int32_t* tile_rows;     // [n_mtiles] valid rows in the tile
    const int32_t* a_gather;      // [rows] source row of A for every sorted row (null = identity)
    const float* row_scale;       // [rows] multiplies the output row (null = 1)
    int64_t b_expert_stride;      // elements between consecutive experts' B
    int32_t n_mtiles;
};
// gemm_f32.hip : C = A B^T (+R) ; epilogue 1 = SwiGLU on stacked gate/up
int launch_gemm_f32(compact_ctx* ctx, const float* A, const float* B, const float* R, float* C,
                    int64_t M, int N, int K, int epilogue, const GroupedArgs* grouped, hipStream_t s);
int gemm_f32_mtile();

// gemm_bf16.hip
// epilogue 0: bf16 C = acc (+R); 1: SwiGLU on stacked gate/up; 2: fp32 C = acc (+R).  R is bf16, or fp32 if r_f32.
int launch_gemm_bf16(compact_ctx* ctx, const bf16* A, const bf16* B, const void* R, bool r_f32, bf16* C,
                     int64_t M, int N, int K, int epilogue, const GroupedArgs* grouped, hipStream_t s);
int gemm_bf16_mtile();

// mxfp4.hip : block-scaled 4-bit expert weights
int mxfp4_ksplit(int K);
int launch_mxfp4_dequant(compact_ctx* ctx, const uint8_t* codes, const uint8_t* scales, bf16* out, int64_t rows, int K,
                         hipStream_t s);
int launch_gemm_skinny_grouped_mxfp4(compact_ctx* ctx, const bf16* X, const int32_t* a_gather, const uint8_t* Wq,
                                     const uint8_t* Ws, const int32_t* offsets, int n_experts, int total_rows,
                                     float* partials, int N, int K, int ks, hipStream_t s,
                                     const int32_t* expert_list = nullptr, int n_listed = 0,
                                     const int32_t* tile_row0 = nullptr, const int32_t* tile_rows = nullptr);

// gemm_skinny.hip : partials[ks][M][N] (fp32) = A[M,K] B[N,K]^T split over K
int skinny_ksplit(int M, int N, int K);
// norm_g (nullable): A holds un-normalised rows x; the operand becomes bf16(x * norm_g) and
// norm_ssq_parts[ks][M] receives the per-slice sums of x^2 (the consumer applies 1 / rms)
int launch_gemm_skinny(compact_ctx* ctx, const bf16* A, const bf16* B, float* partials, int M, int N, int K,
                       int ks, hipStream_t s, const bf16* norm_g = nullptr, float* norm_ssq_parts = nullptr);
bool skinny_norm_in_supported(int M, int N, int K);
// the same per expert, for routed decode rows: expert e multiplies the rows offsets[e] ..
// offsets[e+1]-1 of the expert-sorted order (at most 16; X is read through a_gather when
// given); partials[ks][total_rows][N] keep the sorted order
int launch_gemm_skinny_grouped(compact_ctx* ctx, const bf16* X, const int32_t* a_gather, const bf16* W, int64_t w_expert_stride,
                               const int32_t* offsets, int n_experts, int total_rows, float* partials, int N, int K, int ks,
                               hipStream_t s, const int32_t* expert_list = nullptr, int n_listed = 0,
                               const int32_t* tile_row0 = nullptr, const int32_t* tile_rows = nullptr);
// expert_list (nullable): the experts to run, one per grid slice, -1 = none; spares launching a slice per idle
// expert.  With tile_row0 / tile_rows (the routing plan's tile map, tiles of at most 16 rows) a grid slice is a
// tile: an expert with more than 16 rows is streamed once per tile of 16
// decode gate/up projection with the SwiGLU fused in (no partials): act[M, F] =
// silu(r X Wg^T) * (r X Wu^T); X may hold un-normalised rows (x * g) whose 1/rms r
// comes from `norm` (null: r = 1)
bool skinny_swiglu_supported(int M, int F, int K);
int launch_gemm_skinny_swiglu(compact_ctx* ctx, const bf16* X, const bf16* W, bf16* act, int M, int F, int K,
                              const RowNorm* norm, hipStream_t s);
// C = sum of partials (+R), rounded to bf16
int launch_skinny_finish(compact_ctx* ctx, const float* partials, int ks, const bf16* R, bf16* C, int M, int N,
                         hipStream_t s);

// gemv_stream.hip : whole-K decode projections with the following step fused in (bf16, <= 16 rows)
// h = resid + X W^T (fp32), hg = bf16(h * g), ssq_parts[N / 16][M] = column-group sums of h^2
bool resid_norm_stream_supported(int M, int N, int K);
int launch_resid_norm_stream(compact_ctx* ctx, const bf16* X, const bf16* W, const bf16* resid, const bf16* g, float* h_out,
                             bf16* hg_out, float* ssq_parts, int M, int N, int K, hipStream_t s);
// y = bf16(resid_f32 + X W^T), K a multiple of 512
bool resid_out_stream_supported(int M, int N, int K);
int launch_resid_out_stream(compact_ctx* ctx, const bf16* X, const bf16* W, const float* resid, bf16* y, int M, int N, int K,
                            hipStream_t s);
// gemv_stream_mt.hip : the output projection (+ residual, RMSNorm statistics) and the fused gate/up projection for
// 17 .. 64 rows, whole K (same split over K and summation order as the kernels for at most 16 rows, so a row's result
// does not depend on how many rows share the step)
bool stream_mt_supported(int M, int N, int K);
int launch_resid_norm_stream_mt(compact_ctx* ctx, const bf16* X, const bf16* W, const bf16* resid, const bf16* g, float* h_out,
                                bf16* hg_out, float* ssq_parts, int M, int N, int K, hipStream_t s);
bool swiglu_mt_supported(int M, int F, int K);
int launch_swiglu_mt(compact_ctx* ctx, const bf16* X, const bf16* W, bf16* act, int M, int F, int K, const RowNorm* norm,
                     hipStream_t s);
// m = bf16(hg / rms): finishes the RMSNorm whose sums of squares are in `norm`
int launch_rownorm_apply(compact_ctx* ctx, const bf16* hg, const RowNorm& norm, bf16* m, int rows, int d, hipStream_t s);

// attn_f32.hip
int launch_attn_prefill_f32(compact_ctx* ctx, const BlockMeta* d_meta, int n_blocks, int max_len,
                            const float* qkv, const float* d_k, const float* d_v, float* o, hipStream_t s);
int launch_attn_decode_f32(compact_ctx* ctx, const BlockMeta* d_meta, int n_blocks, int step, const float* q,
                           const float* d_k, const float* d_v, float* o, hipStream_t s);

// attn_prefill.hip (bf16 MFMA)
int launch_attn_prefill_bf16(compact_ctx* ctx, const BlockMeta* d_meta, const TileItem* d_qtiles, int n_qtiles,
                             const bf16* qkv, const bf16* d_k, const bf16* d_v, bf16* o, hipStream_t s);

// attn_decode.hip (bf16 MFMA, split-KV)
size_t attn_decode_partial_floats(const compact_layer_cfg& cfg, int n_blocks, int max_chunks);
// d_chunks: the (block, first row) list of the DECODE_CHUNK-row pieces the call's steps touch
int launch_attn_decode_bf16(compact_ctx* ctx, const BlockMeta* d_meta, const TileItem* d_chunks, int n_chunks, int n_blocks,
                            int step, int max_chunks,
                            const bf16* q, const bf16* d_k, const bf16* d_v, float* partials, bf16* o,
                            hipStream_t s, const int32_t* d_qrow = nullptr, int q_stride = 0);
// d_qrow (nullable): block b's query is row d_qrow[b] of q, rows q_stride elements apart (its output goes to the same
// row of o [rows, Hq * hd]); null: q and o are [n_blocks, Hq * hd]

// attn_decode_prefix.hip (bf16): cascade over the shared prefix + private tails
int launch_attn_decode_prefix_bf16(compact_ctx* ctx, const BlockMeta* d_tail_meta, const BlockMeta& shared,
                                   const PrefixItem* d_items, int n_items, const int32_t* d_wl_off, const int32_t* d_wl,
                                   int max_list, int n_workers, int step, const bf16* q, const bf16* kshared,
                                   const bf16* vshared, const bf16* ktail, const bf16* vtail, float* records,
                                   int64_t total_recs, bf16* o, hipStream_t s);

// moe.hip
struct MoePlan {              // device buffers carved from the workspace
    int32_t* counts;          // [E]
    int32_t* offsets;         // [E+1]
    int32_t* sorted_token;    // [rows*k] source token of every sorted row
    float* sorted_gate;       // [rows*k]
    int32_t* slot_of;         // [rows*k] sorted position of (token, j)
    int32_t* tile_expert;     // [max_mtiles]
    int32_t* tile_row0;
    int32_t* tile_rows;
    int32_t max_mtiles;
};
int launch_moe_route(compact_ctx* ctx, const void* m, const void* w_router, int64_t rows, int32_t* idx,
                     float* gate, float* logits, hipStream_t s,
                     float* partials_ws = nullptr);   // partials_ws: [ks][rows][E] scratch; enables the few-rows path
int launch_moe_plan(compact_ctx* ctx, const int32_t* idx, const float* gate, int64_t rows, int mtile,
                    const MoePlan& plan, hipStream_t s);
// decode: y[t] = h[t] + sum_j gate * (sum over K-slices of partials[slot_of[t*k + j]]), one rounding
int launch_moe_combine_partials(compact_ctx* ctx, const float* partials, int ks, int64_t total_rows, const float* h,
                                const int32_t* slot_of, const float* sorted_gate, int64_t rows, void* y, hipStream_t s);
// h_is_f32: the residual h is fp32 (decode) instead of the storage type
int launch_moe_combine(compact_ctx* ctx, const void* expert_out, const void* h, bool h_is_f32,
                       const int32_t* slot_of, int64_t rows, void* y, hipStream_t s);
