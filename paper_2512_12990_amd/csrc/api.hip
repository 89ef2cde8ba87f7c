// Context, bank construction and export: the host side of the C ABI.
#include "common.hpp"
#include <new>
#include <vector>
#include <string.h>

extern "C" const char* smoe_strerror(int status) {
  switch (status) {
    case SMOE_OK: return "ok";
    case SMOE_EINVAL: return "null or invalid argument";
    case SMOE_ESHAPE: return "inconsistent or unsupported dimensions";
    case SMOE_EALIGN: return "device pointer not 16-byte aligned";
    case SMOE_ESIZE: return "buffer or workspace too small";
    case SMOE_EHIP: return "a HIP call failed (see smoe_last_hip_error)";
    case SMOE_ENOTIMPL: return "not implemented in this build";
    default: return "unknown status";
  }
}

extern "C" int smoe_workspace_bytes(int tokens, int k, int d_ff, int n_shared, int shared_d_ff, size_t* bytes) {
  if (!bytes) return SMOE_EINVAL;
  if (tokens < 1 || tokens > SMOE_MAX_MULTI || k < 0 || k > SMOE_MAX_TOPK || n_shared < 0 || n_shared > SMOE_MAX_SLOTS - SMOE_MAX_TOPK ||
      d_ff < 0 || shared_d_ff < 0)
    return SMOE_ESHAPE;
  // one token: its k + n_shared SwiGLU vectors; several tokens: vectors a fixed stride apart (room for the largest top-k)
  const size_t nsf = (size_t)n_shared * (size_t)shared_d_ff;
  const size_t floats = tokens > 1 ? (size_t)tokens * (nsf + (size_t)SMOE_MAX_TOPK * (size_t)d_ff) : nsf + (size_t)k * (size_t)d_ff;
  *bytes = (size_t)WS_H_OFF + ((floats * 4 + 255) & ~(size_t)255);
  return SMOE_OK;
}

extern "C" int smoe_ctx_create(int device, void* hip_stream, void* workspace_dev, size_t workspace_bytes, smoe_ctx** out) {
  if (!out || device < 0) return SMOE_EINVAL;
  *out = nullptr;
  if (!workspace_dev && workspace_bytes) return SMOE_EINVAL;
  if (((uintptr_t)workspace_dev) & 255u) return SMOE_EALIGN;
  if (workspace_dev && workspace_bytes < (size_t)WS_H_OFF) return SMOE_ESIZE;
  smoe_ctx* c = new (std::nothrow) smoe_ctx();
  if (!c) return SMOE_EINVAL;
  c->device = device; c->stream = (hipStream_t)hip_stream; c->ws = (uint8_t*)workspace_dev; c->ws_bytes = workspace_bytes;
  c->last_hip = 0; c->n_cu = 256; c->timing = 0; c->timing_events = nullptr;
  for (size_t& g : c->down_lds_granted) g = 0;
  for (size_t& g : c->route_lds_granted) g = 0;
  c->one_launch = 0; c->one_spin_limit = 0; c->one_calls = 0;
  for (int& b : c->one_blocks_per_cu) b = 0;
  for (size_t& g : c->one_lds_seen) g = 0;
  hipError_t e = hipSetDevice(device);
  if (e == hipSuccess) {
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, device) == hipSuccess && prop.multiProcessorCount > 0)
      c->n_cu = prop.multiProcessorCount;
  }
  if (e != hipSuccess) { (void)hipGetLastError(); delete c; return SMOE_EHIP; }
  *out = c;
  return SMOE_OK;
}

extern "C" int smoe_ctx_destroy(smoe_ctx* ctx) {
  if (!ctx) return SMOE_EINVAL;
  if (ctx->timing_events) {
    std::vector<hipEvent_t>* ev = (std::vector<hipEvent_t>*)ctx->timing_events;
    for (hipEvent_t e : *ev) (void)hipEventDestroy(e);
    delete ev;
  }
  delete ctx;
  return SMOE_OK;
}

extern "C" int smoe_last_hip_error(const smoe_ctx* ctx) { return ctx ? ctx->last_hip : 0; }

extern "C" int smoe_ctx_timing(smoe_ctx* ctx, int enable) {
  if (!ctx) return SMOE_EINVAL;
  if (!ctx->timing_events) ctx->timing_events = new (std::nothrow) std::vector<hipEvent_t>();
  if (!ctx->timing_events) return SMOE_EINVAL;
  ctx->timing = enable ? 1 : 0;
  return SMOE_OK;
}

extern "C" int smoe_ctx_timing_read(smoe_ctx* ctx, double* gateup_us, double* down_us, int* n_calls) {
  if (!ctx || !gateup_us || !down_us || !n_calls) return SMOE_EINVAL;
  *gateup_us = *down_us = 0.0; *n_calls = 0;
  if (!ctx->timing_events) return SMOE_OK;
  std::vector<hipEvent_t>* ev = (std::vector<hipEvent_t>*)ctx->timing_events;
  HIPCHK(ctx, hipSetDevice(ctx->device));
  HIPCHK(ctx, hipStreamSynchronize(ctx->stream));
  for (size_t i = 0; i + 3 < ev->size(); i += 4) {
    float a = 0.0f, b = 0.0f;
    HIPCHK(ctx, hipEventElapsedTime(&a, (*ev)[i], (*ev)[i + 1]));
    HIPCHK(ctx, hipEventElapsedTime(&b, (*ev)[i + 2], (*ev)[i + 3]));
    *gateup_us += 1e3 * a; *down_us += 1e3 * b; ++*n_calls;
  }
  for (hipEvent_t e : *ev) (void)hipEventDestroy(e);
  ev->clear();
  return SMOE_OK;
}

// ---- bank layout ------------------------------------------------------------------------------
static inline size_t up256(size_t x) { return (x + 255) & ~(size_t)255; }
static inline size_t up16(size_t x) { return (x + 15) & ~(size_t)15; }

static int check_desc(const smoe_bank_desc* d) {
  if (!d) return SMOE_EINVAL;
  if (d->n_experts <= 0 || d->d_model <= 0 || d->d_ff <= 0 || d->group <= 0) return SMOE_ESHAPE;
  if (d->d_model % 32 || d->d_ff % 32 || d->group % 32) return SMOE_ESHAPE;
  if ((d->w_dtype != SMOE_F32 && d->w_dtype != SMOE_BF16) || (d->scale_dtype != SMOE_F32 && d->scale_dtype != SMOE_BF16))
    return SMOE_EINVAL;
  if (d->symmetric != 0 && d->symmetric != 1) return SMOE_EINVAL;
  if (d->b_high <= d->b_low || d->b_low < 1 || d->b_high > 8) return SMOE_ESHAPE;
  if (!((d->b_high == 8 && d->b_low == 4) || (d->b_high == 6 && d->b_low == 3) || (d->b_high == 4 && d->b_low == 2)))
    return SMOE_ENOTIMPL;
  return SMOE_OK;
}

struct MatOff { size_t msb, lsb, zp, sc; };

static size_t layout(const smoe_bank_desc* d, BankDev* b, MatOff* ogu, MatOff* odn) {
  const size_t E = (size_t)d->n_experts, ssz = d->scale_dtype == SMOE_BF16 ? 2 : 4;
  MatDev* m[2] = {&b->gu, &b->dn};
  MatOff* o[2] = {ogu, odn};
  m[0]->N = 2 * d->d_ff; m[0]->K = d->d_model;
  m[1]->N = d->d_model;  m[1]->K = d->d_ff;
  size_t off = 0;
  for (int i = 0; i < 2; i++) {
    m[i]->ng = (m[i]->K + d->group - 1) / d->group;
    m[i]->cpg = d->group / 32;
    m[i]->bits = d->b_low;
    m[i]->plane_stride = (size_t)m[i]->N * m[i]->K * d->b_low / 8;
    m[i]->zp_stride = up16((size_t)m[i]->N * m[i]->ng);
    m[i]->sng = (m[i]->ng + 1) & ~1;
    m[i]->sc_stride = up16((size_t)m[i]->N * m[i]->sng * ssz);
    m[i]->ps32 = (unsigned)m[i]->plane_stride; m[i]->zs32 = (unsigned)m[i]->zp_stride; m[i]->ss32 = (unsigned)m[i]->sc_stride;
    m[i]->fits32 = (E * m[i]->plane_stride < 0x7FFF0000ull) ? 1u : 0u;
  }
  // MSB planes of both families first, then zero-points, then scales, then the LSB planes: a
  // low-bit read never touches the LSB region.
  for (int i = 0; i < 2; i++) { o[i]->msb = off; off = up256(off + E * m[i]->plane_stride); }
  for (int i = 0; i < 2; i++) { o[i]->zp = off; off = up256(off + E * m[i]->zp_stride); }
  for (int i = 0; i < 2; i++) { o[i]->sc = off; off = up256(off + E * m[i]->sc_stride); }
  for (int i = 0; i < 2; i++) { o[i]->lsb = off; off = up256(off + E * m[i]->plane_stride); }
  b->n_experts = d->n_experts; b->d_model = d->d_model; b->d_ff = d->d_ff; b->group = d->group;
  b->sc_bf16 = d->scale_dtype == SMOE_BF16;
  b->bits = d->b_low;
  return off;
}

extern "C" int smoe_bank_bytes(const smoe_bank_desc* desc, size_t* store_bytes) {
  int rc = check_desc(desc);
  if (rc) return rc;
  if (!store_bytes) return SMOE_EINVAL;
  BankDev b; MatOff a, c;
  *store_bytes = layout(desc, &b, &a, &c);
  return SMOE_OK;
}

extern "C" int smoe_bank_create(smoe_ctx* ctx, const smoe_bank_desc* desc, void* store_dev, size_t store_bytes,
                                smoe_bank** out) {
  if (!ctx || !out || !store_dev) return SMOE_EINVAL;
  *out = nullptr;
  int rc = check_desc(desc);
  if (rc) return rc;
  if (((uintptr_t)store_dev) & 255u) return SMOE_EALIGN;
  smoe_bank* b = new (std::nothrow) smoe_bank();
  if (!b) return SMOE_EINVAL;
  MatOff ogu, odn;
  size_t need = layout(desc, &b->dev, &ogu, &odn);
  if (store_bytes < need) { delete b; return SMOE_ESIZE; }
  uint8_t* s = (uint8_t*)store_dev;
  b->dev.gu.msb = s + ogu.msb; b->dev.gu.lsb = s + ogu.lsb; b->dev.gu.zp = s + ogu.zp; b->dev.gu.sc = s + ogu.sc;
  b->dev.dn.msb = s + odn.msb; b->dev.dn.lsb = s + odn.lsb; b->dev.dn.zp = s + odn.zp; b->dev.dn.sc = s + odn.sc;
  b->desc = *desc; b->store = s; b->store_bytes = store_bytes; b->device = ctx->device;
  *out = b;
  return SMOE_OK;
}

extern "C" int smoe_bank_destroy(smoe_bank* bank) {
  if (!bank) return SMOE_EINVAL;
  delete bank;
  return SMOE_OK;
}

extern "C" int smoe_quantize_slice(smoe_ctx* ctx, smoe_bank* bank, int e0, int n, const void* w_gate_dev,
                                   const void* w_up_dev, const void* w_down_dev) {
  if (!ctx || !bank || !w_gate_dev || !w_up_dev || !w_down_dev) return SMOE_EINVAL;
  if (e0 < 0 || n <= 0 || e0 + n > bank->desc.n_experts) return SMOE_ESHAPE;
  if (!aligned16(w_gate_dev) || !aligned16(w_up_dev) || !aligned16(w_down_dev)) return SMOE_EALIGN;
  return smoe_launch_quantize(ctx, bank, e0, n, w_gate_dev, w_up_dev, w_down_dev);
}

// ---- export ---------------------------------------------------------------------------------
extern "C" int smoe_export_codes(smoe_ctx* ctx, const smoe_bank* bank, int expert, int matrix, uint8_t* q_host,
                                 uint8_t* msb_host, uint8_t* lsb_host, uint8_t* zp_host, float* scale_host) {
  if (!ctx || !bank) return SMOE_EINVAL;
  if (expert < 0 || expert >= bank->desc.n_experts || matrix < 0 || matrix > 2) return SMOE_ESHAPE;
  const MatDev& m = matrix == 2 ? bank->dev.dn : bank->dev.gu;
  const int N = matrix == 2 ? m.N : m.N / 2, K = m.K, ng = m.ng;
  const int bits = m.bits;
  const size_t row_b = (size_t)K * bits / 8, ssz = bank->dev.sc_bf16 ? 2 : 4;
  HIPCHK(ctx, hipStreamSynchronize(ctx->stream));
  std::vector<uint8_t> pm(m.plane_stride), pl(m.plane_stride), zp((size_t)m.N * ng), sc((size_t)m.N * m.sng * ssz);
  HIPCHK(ctx, hipMemcpy(pm.data(), m.msb + (size_t)expert * m.plane_stride, pm.size(), hipMemcpyDeviceToHost));
  HIPCHK(ctx, hipMemcpy(pl.data(), m.lsb + (size_t)expert * m.plane_stride, pl.size(), hipMemcpyDeviceToHost));
  HIPCHK(ctx, hipMemcpy(zp.data(), m.zp + (size_t)expert * m.zp_stride, zp.size(), hipMemcpyDeviceToHost));
  HIPCHK(ctx, hipMemcpy(sc.data(), m.sc + (size_t)expert * m.sc_stride, sc.size(), hipMemcpyDeviceToHost));
  for (int r = 0; r < N; r++) {
    // gate rows are the even rows of the interleaved family, up rows the odd ones
    const size_t sr = matrix == 2 ? (size_t)r : (size_t)2 * r + (matrix == 1);
    for (int kk = 0; kk < K; kk++) {
      uint8_t mv, lv;
      if (bits == 4) {
        const uint8_t bm = pm[sr * row_b + kk / 2] ^ 0x88, bl = pl[sr * row_b + kk / 2] ^ 0x88;   // stored as n ^ 8
        mv = (kk & 1) ? (bm >> 4) : (bm & 15); lv = (kk & 1) ? (bl >> 4) : (bl & 15);
      } else if (bits == 3) {                                   // 12-byte chunks of 32 columns (see quantize.hip)
        const int t = (kk & 31) >> 3, j = kk & 7;
        auto code3 = [&](const std::vector<uint8_t>& pl8) {
          uint32_t w[3];
          memcpy(w, &pl8[sr * row_b + (size_t)(kk >> 5) * 12], 12);
          return (uint8_t)(((w[t >> 1] >> (4 * j + 2 * (t & 1))) & 3u) | (((w[2] >> (4 * j + t)) & 1u) << 2));
        };
        mv = code3(pm); lv = code3(pl);
      } else {                                                  // four 2-bit codes per byte, column 4j in bits 0-1
        mv = (pm[sr * row_b + kk / 4] >> (2 * (kk & 3))) & 3; lv = (pl[sr * row_b + kk / 4] >> (2 * (kk & 3))) & 3;
      }
      const size_t o = (size_t)r * K + kk;
      if (msb_host) msb_host[o] = mv;
      if (lsb_host) lsb_host[o] = lv;
      if (q_host) q_host[o] = (uint8_t)((mv << bits) | lv);
    }
    for (int g = 0; g < ng; g++) {
      if (zp_host) zp_host[(size_t)r * ng + g] = zp[sr * ng + g];
      if (scale_host) {
        float f;
        if (bank->dev.sc_bf16) {
          uint32_t u = (uint32_t)((const uint16_t*)sc.data())[sr * m.sng + g] << 16;
          memcpy(&f, &u, 4);
        } else {
          f = ((const float*)sc.data())[sr * m.sng + g];
        }
        scale_host[(size_t)r * ng + g] = f;
      }
    }
  }
  return SMOE_OK;
}
