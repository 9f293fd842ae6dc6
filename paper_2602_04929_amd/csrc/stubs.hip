// Entry points not implemented yet fail loudly.
#include "internal.h"
#define NOT_YET(ctx, name) (ctx ? tboa_fail(ctx, TBOA_EINVAL, name ": not implemented") : TBOA_EINVAL)
extern "C" int tboa_gemm_bf16_nt(tboa_ctx* ctx, int, int, int, float, const void*, int64_t, const void*, int64_t, void*, int64_t, int, int, int, int, int64_t, int64_t, int64_t) { return NOT_YET(ctx, "tboa_gemm_bf16_nt"); }
extern "C" int tboa_build_hessians(tboa_ctx* ctx, const tboa_attn_desc*, const void*, const void*, const void*, const void*, const void*, const void*, float*, float*, float*, float*, float*, float*, float*) { return NOT_YET(ctx, "tboa_build_hessians"); }
extern "C" int tboa_build_hessian_out_proj(tboa_ctx* ctx, const tboa_attn_desc*, const void*, const void*, const float*, const float*, const float*, const void*, const void*, const void*, float*, float*) { return NOT_YET(ctx, "tboa_build_hessian_out_proj"); }
extern "C" int tboa_act_fakequant(tboa_ctx* ctx, int64_t, int, int, int, const void*, void*) { return NOT_YET(ctx, "tboa_act_fakequant"); }
