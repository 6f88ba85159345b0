/*
 * compact.h -- C ABI of libcompact: one transformer layer's forward over a
 * batch of independent token blocks, for parallel context compaction.
 *
 * The method (paper Sec. IV, "Parallel Compaction"): when a conversation
 * exceeds the compaction threshold it is snapshotted, cut into
 * N = ceil(|X| / B) contiguous blocks, every block is summarised by its own
 * worker concurrently, and the N per-block results are concatenated in block
 * order.  On the device the N concurrent workers are one ragged batch: a
 * varlen causal prefill in which no token attends outside its own block,
 * followed by batched single-token decode steps, each block against its own
 * KV cache.  The calls below take "N blocks with token spans" in and give
 * "per-block hidden states and KV caches" out, in block order.
 *
 * Conventions
 *  - All d_* pointers are DEVICE pointers, all h_* pointers are HOST pointers.
 *    Every buffer is owned by the caller and only borrowed for the call; the
 *    library owns nothing but the context and a small device metadata buffer.
 *  - Host arrays are read (and h_len written) before the call returns.
 *  - Work is enqueued on `hip_stream` (a hipStream_t passed as void*; NULL =
 *    the default stream) and the call returns without synchronising.  One
 *    exception: the first call through a context that needs device metadata
 *    (block table, tile lists) allocates a 1 MiB device buffer and a pinned
 *    staging copy for it (hipMalloc + hipHostMalloc) after one
 *    hipDeviceSynchronize; a later call does so again only if its lists
 *    outgrow the buffer (then doubled).  Steady-state calls neither allocate
 *    nor synchronise the device; a call that uploads metadata waits on the
 *    host until the previous upload has left the staging buffer.
 *  - A context serves ONE stream at a time: its metadata buffer and staging
 *    copy are shared by all its calls, so calls through one context on
 *    different streams must be ordered by the caller.  Use one context per
 *    stream for concurrent work.
 *  - Activations and weights are row-major, dtype per cfg.dtype (fp32 or
 *    bf16).  Weights are [out, in], so both GEMM operands are contiguous
 *    along the contraction.
 *  - Return value 0 = COMPACT_OK, otherwise one of the COMPACT_E* codes;
 *    compact_last_error() gives a readable detail.  All argument validation
 *    happens before the first HIP call.
 *  - Results are deterministic run to run, and a block's results do not
 *    depend on which other blocks share the call nor on its place among
 *    them: no work split is chosen from the batch, with one exception.  The
 *    decode projections come in one kernel family for at most 16 blocks and
 *    one for more (beyond 64 blocks the rows of a step go through the second
 *    family in groups of 33 .. 64, each group streaming the weights again): the
 *    caches and every output are bit-identical within a family; across the two,
 *    the caches still are, the outputs agree to rounding (the down projection
 *    adds over K in another order).
 */
#ifndef COMPACT_H
#define COMPACT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    COMPACT_OK = 0,
    COMPACT_EINVAL = 1,       /* null pointer, non-positive size, empty block, cu_seqlens not increasing */
    COMPACT_ESHAPE = 2,       /* layer shape violates a kernel constraint */
    COMPACT_ECAPACITY = 3,    /* a block (or len+1) exceeds its KV slab capacity */
    COMPACT_EWORKSPACE = 4,   /* workspace missing or too small */
    COMPACT_EUNSUPPORTED = 5, /* dtype / feature not built */
    COMPACT_EHIP = 6          /* HIP runtime failure (allocation, launch) */
};

enum { COMPACT_FP32 = 0, COMPACT_BF16 = 1 };

/* Layer shape.  Pre-norm, two residual branches, no biases:
 *   n = RMSNorm(x; g_attn); [q,k,v] = n W_qkv^T; rotary(q,k); o = causal GQA attention;
 *   h = x + o W_o^T; m = RMSNorm(h; g_ffn);
 *   dense: y = h + (silu(m W_g^T) * (m W_u^T)) W_d^T
 *   MoE:   l = m W_r^T (fp32); I = top_k(l) (descending, ties to the lower index);
 *          w = softmax(l_I); y = h + sum_{e in I} w_e FFN_e(m)   (no capacity limit)
 * Rotary pairing is rotate-half: (x_i, x_{i+hd/2}) turned by pos * theta^(-2i/hd).
 * Query head h reads KV head h / (n_q_heads / n_kv_heads).
 * Constraints: head_dim in {64, 128}; n_q_heads % n_kv_heads == 0 with a
 * group of at most 16; d_model, ffn_dim multiples of 64; d_model <= 8192; top_k <= 8;
 * n_experts <= 256, a multiple of 8 in bf16 storage.                      */
typedef struct compact_layer_cfg {
    int32_t d_model;
    int32_t n_q_heads;
    int32_t n_kv_heads;
    int32_t head_dim;
    int32_t ffn_dim;      /* F: width of the SwiGLU hidden layer (per expert for MoE) */
    int32_t n_experts;    /* 0 = dense */
    int32_t top_k;        /* experts per token (MoE only) */
    float   rms_eps;
    float   rope_theta;
    int32_t dtype;        /* COMPACT_FP32 or COMPACT_BF16: storage type of activations, weights, KV */
} compact_layer_cfg;

/* Device pointers to the layer's weights, dtype per cfg. Unused ones may be NULL. */
typedef struct compact_weights {
    const void* g_attn;         /* [d]                                   */
    const void* w_qkv;          /* [Dq + 2 Dkv, d]: q rows, then k, then v */
    const void* w_o;            /* [d, Dq]                               */
    const void* g_ffn;          /* [d]                                   */
    const void* w_gate_up;      /* dense: [2F, d], rows 0..F-1 gate, F..2F-1 up */
    const void* w_down;         /* dense: [d, F]                         */
    const void* w_router;       /* MoE: [E, d]                           */
    const void* w_exp_gate_up;  /* MoE: [E, 2F, d]                       */
    const void* w_exp_down;     /* MoE: [E, d, F]                        */
    /* Optional block-scaled 4-bit copy of the expert weights (the "mxfp4 weights" the
     * paper's largest model is served with, Sec. IV-B; OCP Microscaling Formats v1.0):
     * FP4 E2M1 elements, two per byte with the even-indexed element in the low nibble
     * (*_q: uint8 [E, rows, K/2]), and one E8M0 scale 2^(e-127) per 32 consecutive
     * elements along K (*_s: uint8 [E, rows, K/32]; e in 8..246, 255 = NaN is not
     * supported).  All four or none.  When given, decode steps with at most 256
     * routed rows (blocks x top_k: 64 blocks at top-4) stream these instead of the 16-bit copy, which must then hold exactly their
     * expanded values (compact_mxfp4_dequant writes them); bf16 storage only.      */
    const void* w_exp_gate_up_q;
    const void* w_exp_gate_up_s;
    const void* w_exp_down_q;
    const void* w_exp_down_s;
} compact_weights;

/* Per-block KV caches.  Block b owns one K slab and one V slab, both starting
 * h_slab_offset[b] ELEMENTS into d_k / d_v and holding Hkv*capacity*hd elements:
 *   K slab: [Hkv][capacity_b][hd]   (row = cached token, after rotary embedding)
 *   V slab: [Hkv][hd][capacity_b]   (transposed: cached tokens contiguous)
 * h_capacity[b] and h_slab_offset[b] must be multiples of 8.  h_len[b] is the
 * number of cached tokens: written by compact_prefill, read and incremented by
 * compact_decode_step.  h_pos_offset[b] (NULL => 0) is added to the block-local
 * index to get the rotary position.                                         */
typedef struct compact_kv {
    void*          d_k;
    void*          d_v;
    const int64_t* h_slab_offset;   /* [N] */
    const int32_t* h_capacity;      /* [N] */
    int32_t*       h_len;           /* [N] in/out */
    const int32_t* h_pos_offset;    /* [N] or NULL */
} compact_kv;

/* Optional MoE routing outputs (all nullable): the k expert ids per token in
 * selection order and their gate weights.                                   */
typedef struct compact_route_out {
    int32_t* d_expert_idx;   /* [rows, top_k] */
    float*   d_gate;         /* [rows, top_k] */
} compact_route_out;

typedef struct compact_ctx compact_ctx;

/* Validates cfg and creates a context.  No HIP call is made here. */
int compact_create(const compact_layer_cfg* cfg, compact_ctx** out);
/* Frees the context and the library's metadata buffer; never caller buffers. */
void compact_destroy(compact_ctx* ctx);
/* Detail of the last non-zero return on this context ("" if none). ctx may be
 * NULL, which gives the detail of the last failed compact_create.            */
const char* compact_last_error(const compact_ctx* ctx);

/* Bytes of device workspace needed by any call with at most max_tokens packed
 * prefill tokens, max_blocks blocks and max_kv_len cached tokens per block.
 * The caller allocates it once and passes it to every call.                 */
int compact_workspace_bytes(const compact_ctx* ctx, int64_t max_tokens, int32_t max_blocks,
                            int32_t max_kv_len, size_t* bytes);

/* Prefill: the layer's forward over N ragged blocks (paper Sec. IV phases 1-2:
 * the N blocks of the partitioned snapshot, dispatched together).  Block b is
 * rows h_cu_seqlens[b] .. h_cu_seqlens[b+1]-1 of d_x [T, d]; attention is
 * causal within a block and never crosses blocks.  Writes d_y [T, d], rows
 * 0..L_b-1 of block b's K and V slabs, and h_len[b] = L_b.  L_b >= 1.
 * route (nullable) receives [T, top_k] routing tables for MoE layers.       */
int compact_prefill(compact_ctx* ctx, const compact_weights* w, int32_t n_blocks,
                    const int32_t* h_cu_seqlens, const void* d_x, compact_kv* kv, void* d_y,
                    const compact_route_out* route, void* d_workspace, size_t ws_bytes,
                    void* hip_stream);

/* The next chunk of every block (a prefill cut into chunks as the paper's server
 * does, Sec. IV-B "chunked prefill"; also a worker's own block behind an
 * already cached prefix, Sec. IV Dispatch): as compact_prefill, but block b's
 * rows are appended behind the h_len[b] rows its cache already holds.  Row i
 * of the chunk sits at rotary position pos_offset[b] + h_len[b] + i, is
 * written to cache row h_len[b] + i and attends cache rows 0 .. h_len[b] + i.
 * h_len[b] grows by the chunk length; with h_len[b] = 0 this is
 * compact_prefill.  COMPACT_ECAPACITY when h_len[b] + L_b exceeds the slab.  */
int compact_prefill_extend(compact_ctx* ctx, const compact_weights* w, int32_t n_blocks,
                           const int32_t* h_cu_seqlens, const void* d_x, compact_kv* kv, void* d_y,
                           const compact_route_out* route, void* d_workspace, size_t ws_bytes,
                           void* hip_stream);

/* One batched decode step (the concurrent workers each emitting one summary
 * token): d_x [N, d] holds one new token per block, at rotary position
 * pos_offset[b] + len[b].  Its K/V row is appended at row len[b], it attends
 * rows 0..len[b] inclusive, and h_len[b] is incremented.  Writes d_y [N, d].
 * Calls that come back with the same cache geometry on the same stream, every
 * block one row longer, reuse the metadata the first of them uploaded (no
 * host-to-device copy per step); anything else rebuilds it.  The results do
 * not depend on which of the two happens. */
int compact_decode_step(compact_ctx* ctx, const compact_weights* w, int32_t n_blocks,
                        const void* d_x, compact_kv* kv, void* d_y,
                        const compact_route_out* route, void* d_workspace, size_t ws_bytes,
                        void* hip_stream);

/* The whole compaction pass for one layer (paper Sec. IV phases 2-3): prefill
 * of all blocks, then n_steps batched decode steps with caller-supplied step
 * inputs d_x_decode [S, N, d] (no LM head or sampling at layer level).
 * d_y_prefill [T, d] and d_y_last [N, d] (last prefill row of each block) are
 * nullable; d_y_decode [S, N, d] holds the per-block outputs of every step in
 * block order (the merge is the identity on this layout).  h_len ends at
 * L_b + n_steps.                                                            */
int compact_layer_forward(compact_ctx* ctx, const compact_weights* w, int32_t n_blocks,
                          const int32_t* h_cu_seqlens, const void* d_x_prefill, int32_t n_steps,
                          const void* d_x_decode, compact_kv* kv, void* d_y_prefill,
                          void* d_y_last, void* d_y_decode, void* d_workspace, size_t ws_bytes,
                          void* hip_stream);

/* ---- prefix-aware target-at-end layout (paper Sec. IV, Dispatch: worker k's
 * prompt is blocks 1..k in order; "Prefix-aware target-at-end layout": every
 * worker's prefix strictly extends the previous one's, so one cache of the
 * whole history serves all of them) -----------------------------------------
 * The history is prefilled ONCE as a single block (compact_prefill with
 * n_blocks = 1, rows 0..T-1 at positions 0..T-1): `shared` is that one-block
 * compact_kv and stays read-only.  Worker b sees its first h_prefix_len[b] rows
 * (the end of its block k: h_prefix_len must not decrease with b, each at most
 * shared->h_len[0]) followed by its own private tail: `tails` is a compact_kv
 * with one slab per worker holding the tokens that worker has generated
 * (h_len[b] of them; h_pos_offset is ignored).
 *
 * compact_prefix_decode_step advances all N <= 64 workers by one token: d_x
 * [N, d] holds worker b's new token at rotary position h_prefix_len[b] +
 * tails->h_len[b]; its K/V row is appended to tail b, it attends the shared rows
 * 0..h_prefix_len[b]-1 and tail rows 0..h_len[b] inclusive, tails->h_len[b] is
 * incremented, d_y [N, d] receives the layer outputs.  The shared rows are read
 * from memory once per step for all workers together (a 256-row chunk is
 * multiplied with the query heads of every worker whose prefix covers it).
 * bf16 storage only.  Errors as compact_decode_step; COMPACT_EINVAL for a
 * decreasing or out-of-range h_prefix_len.  The workspace must hold
 * compact_prefix_workspace_bytes(ctx, N, max h_prefix_len, max tail length). */
int compact_prefix_workspace_bytes(const compact_ctx* ctx, int32_t n_workers, int32_t max_prefix_len,
                                   int32_t max_tail_len, size_t* bytes);
int compact_prefix_decode_step(compact_ctx* ctx, const compact_weights* w, int32_t n_workers,
                               const void* d_x, const compact_kv* shared, const int32_t* h_prefix_len,
                               compact_kv* tails, void* d_y, const compact_route_out* route,
                               void* d_workspace, size_t ws_bytes, void* hip_stream);

/* The same pass as compact_layer_forward, scheduled the way the paper's server
 * runs it (Sec. IV-B: chunked prefill): no step handles more than
 * max_batched_tokens rows.  Each step takes one decode token of every block
 * whose prefill is complete and that still has steps left, and fills the rest
 * of the budget with the next prefill chunks of the other blocks, in block
 * order; chunks and decode tokens share one packed batch through the
 * projections (each weight is read once for both), chunk rows go through the
 * prefill attention against their block's cached rows, decode rows through the
 * split-KV decode attention.  Once every prefill is complete the remaining
 * decode steps run batched over the blocks that still have steps left.  Blocks
 * therefore advance at different rates; block b's step s still reads
 * d_x_decode[s, b] and writes d_y_decode[s, b], and the outputs equal those of
 * compact_layer_forward up to rounding.  Activation workspace is sized by
 * max_batched_tokens, not by the total prefill length.  d_y_last [N, d] is
 * nullable.  max_batched_tokens must exceed n_blocks.  The workspace must hold
 * compact_mixed_workspace_bytes(ctx, max_batched_tokens, n_blocks, max L_b + n_steps). */
int compact_mixed_workspace_bytes(const compact_ctx* ctx, int32_t max_batched_tokens, int32_t max_blocks,
                                  int32_t max_kv_len, size_t* bytes);
int compact_mixed_forward(compact_ctx* ctx, const compact_weights* w, int32_t n_blocks,
                          const int32_t* h_cu_seqlens, const void* d_x_prefill, int32_t n_steps,
                          const void* d_x_decode, compact_kv* kv, int32_t max_batched_tokens, void* d_y_last,
                          void* d_y_decode, void* d_workspace, size_t ws_bytes, void* hip_stream);

/* A depth of layers (the models of paper Sec. IV-A are 32- to 80-layer stacks
 * of the layer above; embedding and output head excluded): layer l's output
 * rows are layer l+1's input rows, in the prefill of all blocks and in each of
 * the n_steps batched decode steps; d_x_decode [S, N, d] are the step inputs of
 * layer 0.  w [n_layers] and kv [n_layers] are host arrays of per-layer
 * weights and per-layer caches; all caches must share one geometry
 * (h_slab_offset, h_capacity, h_pos_offset equal across layers; d_k / d_v
 * differ).  d_y_last [N, d] (nullable) receives the last layer's last prefill
 * row of each block, d_y_decode [S, N, d] the last layer's step outputs.
 * With n_blocks = 1 and one block spanning the whole history this is the
 * sequential baseline the paper compares against (Sec. V, Tables VII-IX).
 * Every kv[l].h_len ends at L_b + n_steps.  Errors as compact_layer_forward;
 * COMPACT_EINVAL for n_layers < 1 or caches of differing geometry.  The
 * workspace must hold compact_stack_workspace_bytes(...).                     */
int compact_stack_workspace_bytes(const compact_ctx* ctx, int64_t max_tokens, int32_t max_blocks,
                                  int32_t max_kv_len, size_t* bytes);
int compact_stack_forward(compact_ctx* ctx, int32_t n_layers, const compact_weights* w, int32_t n_blocks,
                          const int32_t* h_cu_seqlens, const void* d_x_prefill, int32_t n_steps,
                          const void* d_x_decode, compact_kv* kv, void* d_y_last, void* d_y_decode,
                          void* d_workspace, size_t ws_bytes, void* hip_stream);

/* The depth of layers in the prefix-aware target-at-end layout (the paper's own
 * configuration, Sec. IV Dispatch + Sec. IV-A models): every layer prefills the
 * whole history d_x_history [history_tokens, d] as ONE causal block into its
 * shared cache shared[l] (one block of capacity >= history_tokens), then every
 * one of n_steps batched decode steps runs worker b's token through all layers,
 * attending in layer l rows 0 .. h_prefix_len[b]-1 of shared[l] plus its own
 * tail in tails[l] (as compact_prefix_decode_step).  d_x_decode / d_y_decode
 * [S, N, d] are layer 0's step inputs and the last layer's step outputs.  w,
 * shared, tails are host arrays [n_layers]; all layers' caches share one
 * geometry.  With n_layers = 1 this is the prefix-aware pass of one layer with
 * a single work list for all steps.  bf16 storage only.  shared[l].h_len[0] ends
 * at history_tokens, tails[l].h_len[b] grows by n_steps.                      */
int compact_prefix_stack_workspace_bytes(const compact_ctx* ctx, int64_t history_tokens, int32_t n_workers,
                                         int32_t max_tail_len, size_t* bytes);
int compact_prefix_stack_forward(compact_ctx* ctx, int32_t n_layers, const compact_weights* w, int32_t n_workers,
                                 const int32_t* h_prefix_len, int64_t history_tokens, const void* d_x_history,
                                 int32_t n_steps, const void* d_x_decode, compact_kv* shared, compact_kv* tails,
                                 void* d_y_decode, void* d_workspace, size_t ws_bytes, void* hip_stream);

/* ---- per-kernel timing ----------------------------------------------------
 * When enabled, every launch of the selected kernel class is bracketed by HIP
 * events on the launch stream.  compact_profile_read synchronises those
 * events and returns the number of launches and their summed duration since
 * the last reset.  Classes: see COMPACT_K_*.                                */
enum {
    COMPACT_K_NONE = 0,
    COMPACT_K_GEMM = 1,          /* bf16 MFMA GEMM (prefill projections, expert GEMMs) */
    COMPACT_K_ATTN_PREFILL = 2,  /* varlen causal flash prefill attention */
    COMPACT_K_ATTN_DECODE = 3,   /* split-KV decode attention (streaming part) */
    COMPACT_K_GEMM_SKINNY = 4,   /* weight-streaming decode projections */
    COMPACT_K_COUNT = 5
};
int compact_profile_select(compact_ctx* ctx, int32_t kernel_class);
int compact_profile_read(compact_ctx* ctx, int64_t* n_launches, double* total_ms);

/* ---- per-kernel entry points (used by the parity tests; same kernels as the
 * layer calls launch).  All pointers are device pointers unless named h_*. -- */

/* y[r] = x[r] / sqrt(mean(x[r]^2) + eps) * g, rows x d. */
int compact_rmsnorm(compact_ctx* ctx, const void* d_x, const void* d_g, void* d_y, int64_t rows,
                    void* hip_stream);
/* Rotary embedding of q and k in a packed qkv [T, Dq+2Dkv] buffer (q rotated
 * in place) and scatter of k (rotated) and v into the block slabs.          */
int compact_rope_kvwrite(compact_ctx* ctx, int32_t n_blocks, const int32_t* h_cu_seqlens,
                         void* d_qkv, compact_kv* kv, void* hip_stream);
/* C[M, N] = A[M, K] B[N, K]^T (+ R[M, N] if d_r != NULL); epilogue 1 treats B
 * as [2N, K] stacked gate/up and stores silu(A Bg^T) * (A Bu^T).            */
int compact_gemm(compact_ctx* ctx, const void* d_a, const void* d_b, const void* d_r, void* d_c,
                 int64_t M, int32_t N, int32_t K, int32_t epilogue, void* d_workspace,
                 size_t ws_bytes, void* hip_stream);
/* Causal attention of every block over its own tokens.  q is read from the
 * packed qkv buffer (row stride Dq+2Dkv), K/V from the slabs (lens in h_len),
 * o [T, Dq].                                                                 */
int compact_attn_prefill(compact_ctx* ctx, int32_t n_blocks, const int32_t* h_cu_seqlens,
                         const void* d_qkv, const compact_kv* kv, void* d_o, void* hip_stream);
/* One query token per block against rows 0..h_len[b]-1 of its slabs.
 * q [N, Dq] -> o [N, Dq].                                                    */
int compact_attn_decode(compact_ctx* ctx, int32_t n_blocks, const void* d_q, const compact_kv* kv,
                        void* d_o, void* d_workspace, size_t ws_bytes, void* hip_stream);
/* compact_attn_decode for callers that cannot allocate device memory or have the library
 * do so on their behalf: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same inputs, same kernels and bit-identical output, but there is no
 * workspace argument: the split-KV partial records and the (block, chunk) work list live in
 * a fixed 32 MiB + 64 KiB device array inside the library (one copy per GPU, held until the
 * process ends), and the work list is written by a kernel from the call's arguments instead
 * of being copied from host memory.  The call makes no hipMalloc / hipFree / hipHostMalloc
 * and no host-to-device copy, and enqueues three kernels on hip_stream.  bf16 storage only.
 * Limits, checked before any HIP call (COMPACT_ECAPACITY beyond them): n_blocks <= 64; at
 * most 4096 chunks of 256 cached rows over all blocks; n_blocks * n_q_heads *
 * ceil(max h_len / 256) * (head_dim + 2) * 4 bytes of partial records <= 32 MiB.
 * All calls on one GPU share that array, through whatever context or stream: calls that
 * overlap in time on one GPU race; serialise them (one stream, or events).  Nothing in
 * the array has to be cleared between calls (every record a call reads it has written).
 * Launches through this entry point are not counted by compact_profile_read.          */
int compact_attn_decode_noalloc(compact_ctx* ctx, int32_t n_blocks, const void* d_q, const compact_kv* kv,
                                void* d_o, void* hip_stream);
/* Prefix-aware decode attention alone: worker b's query q [N, Dq] against rows
 * 0..h_prefix_len[b]-1 of the shared block and rows 0..tails->h_len[b]-1 of its
 * tail (h_len >= 1: the current token's row is already there).  o [N, Dq].
 * The workspace holds the per-item records.                                  */
int compact_attn_decode_prefix(compact_ctx* ctx, int32_t n_workers, const void* d_q,
                               const compact_kv* shared, const int32_t* h_prefix_len,
                               const compact_kv* tails, void* d_o, void* d_workspace, size_t ws_bytes,
                               void* hip_stream);
/* Expands block-scaled 4-bit weights (layout: see compact_weights) to bf16
 * d_out [rows, K]; exact.  K % 32 == 0.                                      */
int compact_mxfp4_dequant(compact_ctx* ctx, const void* d_codes, const void* d_scales, int64_t rows,
                          int32_t K, void* d_out, void* hip_stream);
/* Router: logits in fp32, top-k ids (descending, ties to the lower id) and
 * softmax gate over the selected logits, for rows of m [rows, d].           */
int compact_moe_route(compact_ctx* ctx, const void* d_m, const void* d_w_router, int64_t rows,
                      int32_t* d_expert_idx, float* d_gate, float* d_logits, void* d_workspace,
                      size_t ws_bytes, void* hip_stream);
/* y = h + sum_k gate_k FFN_{idx_k}(m) for rows of m/h [rows, d], routing given. */
int compact_moe_ffn(compact_ctx* ctx, const compact_weights* w, const void* d_m, const void* d_h,
                    const int32_t* d_expert_idx, const float* d_gate, int64_t rows, void* d_y,
                    void* d_workspace, size_t ws_bytes, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* COMPACT_H */
