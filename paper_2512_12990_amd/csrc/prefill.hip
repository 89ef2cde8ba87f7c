// Prefill: route all tokens, per-expert histogram, grouped high-bit expert GEMM (paper Section 4.3).
#include "route_device.hpp"

extern "C" int smoe_prefill_bytes(int T, int E, int k, int d_model, int d_ff, int shared_d_ff, size_t* scratch_bytes) {
  (void)T; (void)E; (void)k; (void)d_model; (void)d_ff; (void)shared_d_ff; (void)scratch_bytes;
  return SMOE_ENOTIMPL;
}

extern "C" int smoe_prefill_histogram(smoe_ctx* ctx, const smoe_bank* routed, const smoe_bank* shared, int T,
                                      const void* x_dev, int act_dtype, int k, const float* logits_dev,
                                      const float* w_router_dev, int norm_topk, float routed_scale,
                                      const void* shared_gate_w_dev, int add_residual, void* scratch_dev,
                                      size_t scratch_bytes, void* y_dev, int32_t* idx_dev, float* w_dev,
                                      uint32_t* hist_dev) {
  return SMOE_ENOTIMPL;
}
