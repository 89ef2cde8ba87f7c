// smoe_route: cache-aware top-k routing for T tokens (paper Section 2.1), one work-group per token.
#include "route_device.hpp"

template <int ACT>
__global__ __launch_bounds__(256) void route_kernel(RouteArgs a) {
  __shared__ RouteShared sh;
  route_token<ACT>(a, blockIdx.x, sh);
}

extern "C" int smoe_route(smoe_ctx* ctx, int T, int E, int k, int d_model, const float* logits_dev,
                          const void* x_dev, int act_dtype, const float* w_router_dev, const float* bias_dev,
                          int norm_topk, float routed_scale, float* logits_out_dev, int32_t* idx_dev, float* w_dev) {
  if (!ctx || !idx_dev || !w_dev) return SMOE_EINVAL;
  if (!logits_dev && (!x_dev || !w_router_dev)) return SMOE_EINVAL;
  if (act_dtype != SMOE_F32 && act_dtype != SMOE_BF16) return SMOE_EINVAL;
  if (T < 0 || E <= 0 || E > SMOE_MAX_EXPERTS || k <= 0 || k > E || k > SMOE_MAX_TOPK) return SMOE_ESHAPE;
  if (!logits_dev && d_model <= 0) return SMOE_ESHAPE;
  if (!aligned16(logits_dev) || !aligned16(x_dev) || !aligned16(w_router_dev) || !aligned16(bias_dev) ||
      !aligned16(logits_out_dev) || !aligned16(idx_dev) || !aligned16(w_dev))
    return SMOE_EALIGN;
  if (T == 0) return SMOE_OK;
  HIPCHK(ctx, hipSetDevice(ctx->device));
  RouteArgs a{E, k, d_model, logits_dev, x_dev, w_router_dev, bias_dev, norm_topk, routed_scale,
              logits_out_dev, idx_dev, w_dev};
  if (act_dtype == SMOE_F32) route_kernel<SMOE_F32><<<T, 256, 0, ctx->stream>>>(a);
  else route_kernel<SMOE_BF16><<<T, 256, 0, ctx->stream>>>(a);
  HIPCHK(ctx, hipGetLastError());
  return SMOE_OK;
}
