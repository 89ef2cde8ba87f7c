// smoe_route: cache-aware top-k routing for T tokens (paper Section 2.1), and the router mat-vec
// alone for the one-token decode path.
#include "route_device.hpp"

template <int ACT, int NT>
__global__ __launch_bounds__(RT_THREADS) void route_batch_kernel(RouteArgs a, int T) {
  extern __shared__ __align__(16) uint8_t rdyn[];
  route_tokens_block<ACT, NT>(a, T, rdyn);
}

// z[e] = w_router[e, :] . x for one token: one wave per expert, so the mat-vec of a single token is
// spread over E/4 work-groups instead of one.
template <int ACT>
__global__ __launch_bounds__(256) void router_logits_kernel(const float* __restrict__ w_router, const void* __restrict__ x,
                                                            int E, int d, float* __restrict__ z) {
  const int lane = threadIdx.x & 63, e = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (e >= E) return;
  // Same sum as router_row_dots (lane l adds columns l, l+64, ... in that order by fused
  // multiply-add, then the wave sum), but 32 columns per lane are fetched before the first is used:
  // one memory round trip per 2048 columns instead of four.
  const uint32_t* wrow = (const uint32_t*)(w_router + (size_t)e * d);
  float p = 0.0f;
  for (int i0 = 0; i0 < d; i0 += 2048) {
    // raw load results only (a column past the end re-reads the last one and is masked below):
    // any arithmetic on a loaded value here would make the wave wait for that load at once
    uint32_t w[32], xv[32];
#pragma unroll
    for (int u = 0; u < 32; u++) {
      const int i = min(i0 + u * 64 + lane, d - 1);
      w[u] = wrow[i];
      xv[u] = ACT == SMOE_BF16 ? (uint32_t)((const uint16_t*)x)[i] : ((const uint32_t*)x)[i];
    }
#pragma unroll
    for (int u = 0; u < 32; u++) {
      const float xf = __uint_as_float(ACT == SMOE_BF16 ? xv[u] << 16 : xv[u]);
      const float q = fmaf(__uint_as_float(w[u]), xf, p);
      p = (i0 + u * 64 + lane) < d ? q : p;
    }
  }
  p = wave_sum(p);
  if (lane == 0) z[e] = p;
}

int smoe_launch_router_logits(smoe_ctx* ctx, int E, int d, const void* x, int act_dtype, const float* w_router, float* z) {
  const int n_wg = (E + 3) / 4;
  if (act_dtype == SMOE_F32) router_logits_kernel<SMOE_F32><<<n_wg, 256, 0, ctx->stream>>>(w_router, x, E, d, z);
  else router_logits_kernel<SMOE_BF16><<<n_wg, 256, 0, ctx->stream>>>(w_router, x, E, d, z);
  HIPCHK(ctx, hipGetLastError());
  return SMOE_OK;
}

// Dynamic LDS beyond the default 64 KB per work-group (wide activations) has to be granted to the
// kernel once per device.
template <typename K>
static int route_lds_grant(smoe_ctx* ctx, K kernel, size_t lds, size_t& granted) {
  if (lds > 160u * 1024u) return SMOE_ESIZE;
  if (lds > 64u * 1024u && lds > granted) {
    if (hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess) {
      (void)hipGetLastError();
      return SMOE_ESIZE;
    }
    granted = lds;
  }
  return SMOE_OK;
}

int smoe_launch_route(smoe_ctx* ctx, const RouteArgs& a, int T, int act_dtype) {
  const bool given = a.logits != nullptr;
  if (act_dtype == SMOE_BF16) {
    const size_t lds = RouteLds<SMOE_BF16, 8>::bytes(a.E, a.d_model, given);
    const int rc = route_lds_grant(ctx, route_batch_kernel<SMOE_BF16, 8>, lds, ctx->route_lds_granted[0]);
    if (rc != SMOE_OK) return rc;
    route_batch_kernel<SMOE_BF16, 8><<<(T + 7) / 8, RT_THREADS, lds, ctx->stream>>>(a, T);
  } else {
    const size_t lds = RouteLds<SMOE_F32, 4>::bytes(a.E, a.d_model, given);
    const int rc = route_lds_grant(ctx, route_batch_kernel<SMOE_F32, 4>, lds, ctx->route_lds_granted[1]);
    if (rc != SMOE_OK) return rc;
    route_batch_kernel<SMOE_F32, 4><<<(T + 3) / 4, RT_THREADS, lds, ctx->stream>>>(a, T);
  }
  HIPCHK(ctx, hipGetLastError());
  return SMOE_OK;
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
  return smoe_launch_route(ctx, a, T, act_dtype);
}
