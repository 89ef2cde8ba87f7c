// Decode-time expert FFN over bit-sliced weights (paper Section 4.1: full precision when both
// slices of an expert are resident, MSB-only otherwise; Section 4.2: the MSB nibble with the
// truncated zero-point IS the low-bit model).
//
// Three launches per token-layer:
//   setup   1 work-group : (route,) precision select, gamma, slot table
//   gateup  many waves   : h = silu(Wg x) * (Wu x) for every slot, one wave per row pair
//   down    d_model/8 WGs: y = sum_slots weight * Wd h  (+ x), each wave owns two output rows
// A lane always works on one 32-column chunk (16 bytes of a nibble plane, one 128-bit load); the
// group-wise affine terms are applied per lane before the cross-lane sum:
//   HIGH  s * (sum (16 m + l) x  -  zp * sum x)        LOW  16 s * (sum m x - (zp >> 4) * sum x)
#include "route_device.hpp"

// ---------------------------------------------------------------------------------- setup
struct SetupArgs {
  BankDev routed, shared;
  int has_routed, n_shared, k, do_route;
  RouteArgs r;
  const int32_t* idx_in; const float* w_in;
  const uint8_t* mask; float tau;
  const void* x; const void* shared_gate_w;
  SlotTable* tab;
  int32_t* idx_out; float* w_out; uint8_t* prec_out;
};

__device__ __forceinline__ void fill_slot(Slot& s, const BankDev& b, int e, int prec, float weight, int h_off) {
  const size_t ee = (size_t)e;
  s.gu_msb = b.gu.msb + ee * b.gu.plane_stride; s.gu_lsb = b.gu.lsb + ee * b.gu.plane_stride;
  s.gu_zp = b.gu.zp + ee * b.gu.zp_stride;      s.gu_sc = b.gu.sc + ee * b.gu.sc_stride;
  s.dn_msb = b.dn.msb + ee * b.dn.plane_stride; s.dn_lsb = b.dn.lsb + ee * b.dn.plane_stride;
  s.dn_zp = b.dn.zp + ee * b.dn.zp_stride;      s.dn_sc = b.dn.sc + ee * b.dn.sc_stride;
  s.f = b.d_ff; s.h_off = h_off; s.prec = prec; s.weight = weight;
  s.gu_ng = b.gu.ng; s.gu_cpg = b.gu.cpg; s.dn_ng = b.dn.ng; s.dn_cpg = b.dn.cpg; s.sc_bf16 = b.sc_bf16; s.pad = 0;
}

template <int ACT>
__global__ __launch_bounds__(256) void decode_setup_kernel(SetupArgs a) {
  __shared__ RouteShared sh;
  __shared__ float red[4];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (a.k > 0) {
    if (a.do_route) {
      route_token<ACT>(a.r, 0, sh);
    } else {
      if (tid < a.k) { sh.sel[tid] = a.idx_in[tid]; sh.wsel[tid] = a.w_in[tid]; }
      __syncthreads();
    }
  }
  float gamma = 1.0f;
  if (a.shared_gate_w) {
    const int d = a.n_shared ? a.shared.d_model : a.routed.d_model;
    float p = 0.0f;
    for (int i = tid; i < d; i += 256) p = fmaf(load_act<ACT>(a.shared_gate_w, i), load_act<ACT>(a.x, i), p);
    p = wave_sum(p);
    if (lane == 0) red[wave] = p;
    __syncthreads();
    const float dot = (red[0] + red[1]) + (red[2] + red[3]);
    gamma = 1.0f / (1.0f + expf(-dot));
  }
  const int k = a.has_routed ? a.k : 0;
  const int n_slots = k + a.n_shared;
  if (tid < k) {
    int e = sh.sel[tid];
    e = min(max(e, 0), a.routed.n_experts - 1);
    const float w = sh.wsel[tid];
    const int both = a.mask ? ((a.mask[e] & 3) == 3) : 1;
    const int prec = both && (a.tau <= 0.0f || w >= a.tau);
    fill_slot(a.tab->s[tid], a.routed, e, prec, w, tid * a.routed.d_ff);
    if (a.prec_out) a.prec_out[tid] = (uint8_t)prec;
    if (a.idx_out) a.idx_out[tid] = e;
    if (a.w_out) a.w_out[tid] = w;
  } else if (tid < n_slots) {
    const int i = tid - k;
    fill_slot(a.tab->s[tid], a.shared, i, 1, gamma, k * (a.has_routed ? a.routed.d_ff : 0) + i * a.shared.d_ff);
  }
  if (tid == 0) {
    a.tab->n_slots = n_slots;
    a.tab->total_f = k * (a.has_routed ? a.routed.d_ff : 0) + a.n_shared * (a.n_shared ? a.shared.d_ff : 0);
  }
}

// ---------------------------------------------------------------------------------- nibble dots
// 32 weights of one plane chunk against the lane's 32 activations (fp32).
__device__ __forceinline__ float dot_bytes(uint32_t e, uint32_t o, const float* x, float acc0, float& acc1) {
  acc0 = fmaf((float)(e & 0xFF), x[0], acc0);
  acc1 = fmaf((float)(o & 0xFF), x[1], acc1);
  acc0 = fmaf((float)((e >> 8) & 0xFF), x[2], acc0);
  acc1 = fmaf((float)((o >> 8) & 0xFF), x[3], acc1);
  acc0 = fmaf((float)((e >> 16) & 0xFF), x[4], acc0);
  acc1 = fmaf((float)((o >> 16) & 0xFF), x[5], acc1);
  acc0 = fmaf((float)(e >> 24), x[6], acc0);
  acc1 = fmaf((float)(o >> 24), x[7], acc1);
  return acc0;
}

__device__ __forceinline__ float dot_low(const uint4& m, const float* x) {
  const uint32_t w[4] = {m.x, m.y, m.z, m.w};
  float a0 = 0.0f, a1 = 0.0f;
#pragma unroll
  for (int j = 0; j < 4; j++)
    a0 = dot_bytes(w[j] & 0x0F0F0F0Fu, (w[j] >> 4) & 0x0F0F0F0Fu, x + 8 * j, a0, a1);
  return a0 + a1;
}

__device__ __forceinline__ float dot_high(const uint4& m, const uint4& l, const float* x) {
  const uint32_t wm[4] = {m.x, m.y, m.z, m.w}, wl[4] = {l.x, l.y, l.z, l.w};
  float a0 = 0.0f, a1 = 0.0f;
#pragma unroll
  for (int j = 0; j < 4; j++) {
    const uint32_t qe = ((wm[j] & 0x0F0F0F0Fu) << 4) | (wl[j] & 0x0F0F0F0Fu);      // codes of even columns
    const uint32_t qo = (wm[j] & 0xF0F0F0F0u) | ((wl[j] >> 4) & 0x0F0F0F0Fu);     // codes of odd columns
    a0 = dot_bytes(qe, qo, x + 8 * j, a0, a1);
  }
  return a0 + a1;
}

// One matrix row chunk -> the lane's share of the dequantised dot product.
__device__ __forceinline__ float row_chunk(const uint8_t* msb, const uint8_t* lsb, const uint8_t* zp, const uint8_t* sc,
                                           int sc_bf16, size_t plane_off, size_t meta_idx, int prec,
                                           const float* x, float xs) {
  const uint4 m = *(const uint4*)(msb + plane_off);
  const int z = zp[meta_idx];
  const float s = load_scale(sc, sc_bf16, meta_idx);
  if (prec) {
    const uint4 l = *(const uint4*)(lsb + plane_off);
    return s * fmaf(-(float)z, xs, dot_high(m, l, x));
  }
  return (16.0f * s) * fmaf(-(float)(z >> 4), xs, dot_low(m, x));
}

// ---------------------------------------------------------------------------------- gate/up
// Flat row-pair space over all slots: pair p belongs to the slot with h_off <= p < h_off + f.
// Wave gw handles pairs [gw*ppw, (gw+1)*ppw).  d_model <= 2048: one chunk per lane.
template <int ACT>
__global__ __launch_bounds__(256) void gateup_kernel(const SlotTable* __restrict__ tab, const void* __restrict__ x,
                                                     float* __restrict__ h, int d_model, int ppw) {
  const int lane = threadIdx.x & 63;
  const int gw = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int total = tab->total_f, n_slots = tab->n_slots;
  int p = gw * ppw;
  if (p >= total) return;
  const int pend = min(total, p + ppw);
  const int C = d_model >> 5;
  const bool act = lane < C;
  float xr[32];
  float xs = 0.0f;
#pragma unroll
  for (int i = 0; i < 32; i++) { xr[i] = act ? load_act<ACT>(x, (size_t)lane * 32 + i) : 0.0f; }
#pragma unroll
  for (int i = 0; i < 32; i++) xs += xr[i];
  int si = 0;
  const size_t rowb = (size_t)d_model >> 1;
  for (; p < pend; p++) {
    while (si + 1 < n_slots && p >= tab->s[si + 1].h_off) si++;
    const Slot& s = tab->s[si];
    const int r = p - s.h_off;
    float a = 0.0f, u = 0.0f;
    if (act) {
      const int g = lane / s.gu_cpg;
      a = row_chunk(s.gu_msb, s.gu_lsb, s.gu_zp, s.gu_sc, s.sc_bf16, (size_t)(2 * r) * rowb + lane * 16,
                    (size_t)(2 * r) * s.gu_ng + g, s.prec, xr, xs);
      u = row_chunk(s.gu_msb, s.gu_lsb, s.gu_zp, s.gu_sc, s.sc_bf16, (size_t)(2 * r + 1) * rowb + lane * 16,
                    (size_t)(2 * r + 1) * s.gu_ng + g, s.prec, xr, xs);
    }
    a = wave_sum(a);
    u = wave_sum(u);
    if (lane == 0) h[p] = a / (1.0f + __expf(-a)) * u;
  }
}

// ---------------------------------------------------------------------------------- down + combine
// Work-group of 4 waves owns 8 output rows (2 per wave) and walks every slot.  The weighted
// SwiGLU vectors of all slots are staged in LDS, chunk-interleaved inside each 64-chunk k-slice
// so that a lane's 8 x 16-byte reads are conflict free.
template <int ACT>
__global__ __launch_bounds__(256) void down_kernel(const SlotTable* __restrict__ tab, const float* __restrict__ h,
                                                   const void* __restrict__ x, void* __restrict__ y, int d_model,
                                                   int add_residual) {
  extern __shared__ float lds[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int total = tab->total_f, n_slots = tab->n_slots;
  float* hs = lds;                 // [total] staged, permuted
  float* cs = lds + total;         // [total/32] per-chunk sums
  for (int si = 0; si < n_slots; si++) {
    const Slot& s = tab->s[si];
    const int C = s.f >> 5;
    for (int i = tid; i < s.f; i += 256) {
      const int c = i >> 5, j = (i >> 2) & 7, e = i & 3;
      const int ks = c >> 6, cw = min(64, C - ks * 64), cl = c & 63;
      hs[s.h_off + ks * 2048 + (j * cw + cl) * 4 + e] = s.weight * h[s.h_off + i];
    }
  }
  __syncthreads();
  for (int si = 0; si < n_slots; si++) {
    const Slot& s = tab->s[si];
    const int C = s.f >> 5;
    for (int c = tid; c < C; c += 256) {
      const int ks = c >> 6, cw = min(64, C - ks * 64), cl = c & 63;
      float t = 0.0f;
      for (int j = 0; j < 8; j++)
        for (int e = 0; e < 4; e++) t += hs[s.h_off + ks * 2048 + (j * cw + cl) * 4 + e];
      cs[(s.h_off >> 5) + c] = t;
    }
  }
  __syncthreads();
  const int n0 = blockIdx.x * 8 + wave * 2;
  float acc0 = 0.0f, acc1 = 0.0f;
  for (int si = 0; si < n_slots; si++) {
    const Slot& s = tab->s[si];
    const int C = s.f >> 5;
    const size_t rowb = (size_t)s.f >> 1;
    for (int ks = 0; ks * 64 < C; ks++) {
      const int cw = min(64, C - ks * 64);
      if (lane < cw) {
        const int c = ks * 64 + lane;
        float xr[32];
        const float4* src = (const float4*)(hs + s.h_off + ks * 2048);
#pragma unroll
        for (int j = 0; j < 8; j++) {
          const float4 v = src[j * cw + lane];
          xr[4 * j] = v.x; xr[4 * j + 1] = v.y; xr[4 * j + 2] = v.z; xr[4 * j + 3] = v.w;
        }
        const float xs = cs[(s.h_off >> 5) + c];
        const int g = c / s.dn_cpg;
        acc0 += row_chunk(s.dn_msb, s.dn_lsb, s.dn_zp, s.dn_sc, s.sc_bf16, (size_t)n0 * rowb + c * 16,
                          (size_t)n0 * s.dn_ng + g, s.prec, xr, xs);
        acc1 += row_chunk(s.dn_msb, s.dn_lsb, s.dn_zp, s.dn_sc, s.sc_bf16, (size_t)(n0 + 1) * rowb + c * 16,
                          (size_t)(n0 + 1) * s.dn_ng + g, s.prec, xr, xs);
      }
    }
  }
  acc0 = wave_sum(acc0);
  acc1 = wave_sum(acc1);
  if (lane == 0) {
    if (add_residual) { acc0 += load_act<ACT>(x, n0); acc1 += load_act<ACT>(x, n0 + 1); }
    store_act<ACT>(y, n0, acc0);
    store_act<ACT>(y, n0 + 1, acc1);
  }
}

// ---------------------------------------------------------------------------------- host entry
static int check_bank_pair(const smoe_ctx* ctx, const smoe_bank* routed, const smoe_bank* shared, int k, int* d_model,
                           int* total_f) {
  if (!routed && !shared) return SMOE_EINVAL;
  if (routed && routed->device != ctx->device) return SMOE_EINVAL;
  if (shared && shared->device != ctx->device) return SMOE_EINVAL;
  if (routed && shared && routed->desc.d_model != shared->desc.d_model) return SMOE_ESHAPE;
  if (!routed && k != 0) return SMOE_ESHAPE;
  if (routed && (k <= 0 || k > routed->desc.n_experts || k > SMOE_MAX_TOPK)) return SMOE_ESHAPE;
  if (routed && routed->desc.n_experts > SMOE_MAX_EXPERTS) return SMOE_ESHAPE;
  const int ns = shared ? shared->desc.n_experts : 0;
  if (k + ns > SMOE_MAX_SLOTS) return SMOE_ESHAPE;
  *d_model = routed ? routed->desc.d_model : shared->desc.d_model;
  if (*d_model > 2048) return SMOE_ENOTIMPL;       // gate/up keeps one 32-column chunk per lane
  if (*d_model % 8) return SMOE_ESHAPE;
  *total_f = (routed ? k * routed->desc.d_ff : 0) + (shared ? ns * shared->desc.d_ff : 0);
  if ((size_t)*total_f * 4 + WS_H_OFF > SMOE_WORKSPACE_BYTES) return SMOE_ESIZE;
  if ((size_t)*total_f * 4 + (size_t)*total_f / 8 > 160u * 1024u) return SMOE_ESIZE;   // LDS staging of h
  return SMOE_OK;
}

static int launch_decode(smoe_ctx* ctx, const smoe_bank* routed, const smoe_bank* shared, const void* x, int act_dtype,
                         int k, SetupArgs& sa, int add_residual, void* y) {
  int d_model = 0, total_f = 0;
  int rc = check_bank_pair(ctx, routed, shared, k, &d_model, &total_f);
  if (rc) return rc;
  HIPCHK(ctx, hipSetDevice(ctx->device));
  SlotTable* tab = (SlotTable*)(ctx->ws + WS_TABLE_OFF);
  float* h = (float*)(ctx->ws + WS_H_OFF);
  if (routed) sa.routed = routed->dev;
  if (shared) sa.shared = shared->dev;
  sa.has_routed = routed != nullptr; sa.n_shared = shared ? shared->desc.n_experts : 0; sa.k = k;
  sa.x = x; sa.tab = tab;
  const int ppw = 2;
  const int n_wg = (total_f + 4 * ppw - 1) / (4 * ppw);
  const size_t lds = (size_t)total_f * 4 + (size_t)(total_f / 32) * 4;
  if (act_dtype == SMOE_F32) {
    static bool attr_done = false;
    if (!attr_done) { HIPCHK(ctx, hipFuncSetAttribute((const void*)down_kernel<SMOE_F32>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024)); attr_done = true; }
    decode_setup_kernel<SMOE_F32><<<1, 256, 0, ctx->stream>>>(sa);
    gateup_kernel<SMOE_F32><<<n_wg, 256, 0, ctx->stream>>>(tab, x, h, d_model, ppw);
    down_kernel<SMOE_F32><<<d_model / 8, 256, lds, ctx->stream>>>(tab, h, x, y, d_model, add_residual);
  } else {
    static bool attr_done = false;
    if (!attr_done) { HIPCHK(ctx, hipFuncSetAttribute((const void*)down_kernel<SMOE_BF16>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024)); attr_done = true; }
    decode_setup_kernel<SMOE_BF16><<<1, 256, 0, ctx->stream>>>(sa);
    gateup_kernel<SMOE_BF16><<<n_wg, 256, 0, ctx->stream>>>(tab, x, h, d_model, ppw);
    down_kernel<SMOE_BF16><<<d_model / 8, 256, lds, ctx->stream>>>(tab, h, x, y, d_model, add_residual);
  }
  HIPCHK(ctx, hipGetLastError());
  return SMOE_OK;
}

extern "C" int smoe_expert_ffn(smoe_ctx* ctx, const smoe_bank* routed, const smoe_bank* shared, const void* x_dev,
                               int act_dtype, int k, const int32_t* idx_dev, const float* w_dev,
                               const uint8_t* slice_mask_dev, float tau_head, const void* shared_gate_w_dev,
                               int add_residual, void* y_dev, uint8_t* prec_out_dev) {
  if (!ctx || !x_dev || !y_dev || x_dev == y_dev) return SMOE_EINVAL;
  if (act_dtype != SMOE_F32 && act_dtype != SMOE_BF16) return SMOE_EINVAL;
  if (routed && (!idx_dev || !w_dev)) return SMOE_EINVAL;
  if (!aligned16(x_dev) || !aligned16(y_dev) || !aligned16(idx_dev) || !aligned16(w_dev) || !aligned16(shared_gate_w_dev))
    return SMOE_EALIGN;
  SetupArgs sa{};
  sa.do_route = 0; sa.idx_in = idx_dev; sa.w_in = w_dev; sa.mask = slice_mask_dev; sa.tau = tau_head;
  sa.shared_gate_w = shared_gate_w_dev; sa.prec_out = prec_out_dev;
  return launch_decode(ctx, routed, shared, x_dev, act_dtype, k, sa, add_residual, y_dev);
}

extern "C" int smoe_decode_layer(smoe_ctx* ctx, const smoe_bank* routed, const smoe_bank* shared, const void* x_dev,
                                 int act_dtype, int k, const float* logits_dev, const float* w_router_dev,
                                 const float* bias_dev, int norm_topk, float routed_scale,
                                 const uint8_t* slice_mask_dev, float tau_head, const void* shared_gate_w_dev,
                                 int add_residual, void* y_dev, int32_t* idx_out_dev, float* w_out_dev,
                                 uint8_t* prec_out_dev) {
  if (!ctx || !x_dev || !y_dev || x_dev == y_dev || !routed) return SMOE_EINVAL;
  if (act_dtype != SMOE_F32 && act_dtype != SMOE_BF16) return SMOE_EINVAL;
  if (!logits_dev && !w_router_dev) return SMOE_EINVAL;
  if (!aligned16(x_dev) || !aligned16(y_dev) || !aligned16(logits_dev) || !aligned16(w_router_dev) ||
      !aligned16(bias_dev) || !aligned16(shared_gate_w_dev))
    return SMOE_EALIGN;
  SetupArgs sa{};
  sa.do_route = 1;
  int32_t* ws_idx = (int32_t*)(ctx->ws + WS_IDX_OFF);
  float* ws_w = (float*)(ctx->ws + WS_IDX_OFF + 256);
  sa.r = RouteArgs{routed->desc.n_experts, k, routed->desc.d_model, logits_dev, x_dev, w_router_dev, bias_dev,
                   norm_topk, routed_scale, nullptr, ws_idx, ws_w};
  sa.mask = slice_mask_dev; sa.tau = tau_head; sa.shared_gate_w = shared_gate_w_dev;
  sa.idx_out = idx_out_dev; sa.w_out = w_out_dev; sa.prec_out = prec_out_dev;
  return launch_decode(ctx, routed, shared, x_dev, act_dtype, k, sa, add_residual, y_dev);
}
