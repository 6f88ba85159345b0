// temporary: launchers not written yet
#include "common.h"
int launch_gemm_bf16(compact_ctx* ctx, const bf16*, const bf16*, const bf16*, bf16*, int64_t, int, int, int, const GroupedArgs*, hipStream_t) { return set_err(ctx, COMPACT_EUNSUPPORTED, "bf16 GEMM not built"); }
int gemm_bf16_mtile() { return 128; }
int skinny_ksplit(int, int, int) { return 1; }
int launch_gemm_skinny(compact_ctx* ctx, const bf16*, const bf16*, float*, int, int, int, int, hipStream_t) { return set_err(ctx, COMPACT_EUNSUPPORTED, "skinny GEMM not built"); }
int launch_skinny_finish(compact_ctx* ctx, const float*, int, const bf16*, bf16*, int, int, hipStream_t) { return set_err(ctx, COMPACT_EUNSUPPORTED, "skinny GEMM not built"); }
int launch_attn_prefill_bf16(compact_ctx* ctx, const BlockMeta*, const TileItem*, int, const bf16*, const bf16*, const bf16*, bf16*, hipStream_t) { return set_err(ctx, COMPACT_EUNSUPPORTED, "bf16 prefill attention not built"); }
size_t attn_decode_partial_floats(const compact_layer_cfg&, int, int) { return 64; }
int launch_attn_decode_bf16(compact_ctx* ctx, const BlockMeta*, int, int, int, const bf16*, const bf16*, const bf16*, float*, bf16*, hipStream_t) { return set_err(ctx, COMPACT_EUNSUPPORTED, "bf16 decode attention not built"); }
int launch_moe_route(compact_ctx* ctx, const void*, const void*, int64_t, int32_t*, float*, float*, hipStream_t) { return set_err(ctx, COMPACT_EUNSUPPORTED, "MoE not built"); }
int launch_moe_plan(compact_ctx* ctx, const int32_t*, const float*, int64_t, int, const MoePlan&, hipStream_t) { return set_err(ctx, COMPACT_EUNSUPPORTED, "MoE not built"); }
int launch_moe_combine(compact_ctx* ctx, const void*, const void*, const int32_t*, int64_t, void*, hipStream_t) { return set_err(ctx, COMPACT_EUNSUPPORTED, "MoE not built"); }
