// Cache-aware top-k routing of one token by one 256-thread work-group (paper Section 2.1:
// experts whose slices are resident get their gating score boosted before selection).
#pragma once
#include "common.hpp"

struct RouteArgs {
  int E, k, d_model;
  const float* logits;     // [T, E] or null
  const void* x;           // [T, d_model] act dtype (used when logits is null)
  const float* w_router;   // [E, d_model]
  const float* bias;       // [E] or null
  int norm_topk;
  float routed_scale;
  float* logits_out;       // [T, E] or null
  int32_t* idx;            // [T, k]
  float* w;                // [T, k]
};

struct RouteShared {
  float z[SMOE_MAX_EXPERTS];
  unsigned long long key[SMOE_MAX_EXPERTS];
  int sel[SMOE_MAX_TOPK];
  float wsel[SMOE_MAX_TOPK];
};

// Monotone map float -> uint32 (a < b  <=>  map(a) < map(b)); -0 is first folded onto +0 so
// equal scores compare equal.
__device__ __forceinline__ uint32_t orderable(float f) {
  if (f == 0.0f) f = 0.0f;
  uint32_t u = __float_as_uint(f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ __forceinline__ unsigned long long wave_max_u64(unsigned long long v) {
  for (int m = 32; m >= 1; m >>= 1) {
    uint32_t lo = __shfl_xor((uint32_t)v, m), hi = __shfl_xor((uint32_t)(v >> 32), m);
    unsigned long long o = ((unsigned long long)hi << 32) | lo;
    v = o > v ? o : v;
  }
  return v;
}

// All 256 threads of the block call this.  On return sh.sel[0..k) and sh.wsel[0..k) hold the
// decision (also written to a.idx / a.w for token t) and the block is synchronised.
template <int ACT>
__device__ void route_token(const RouteArgs& a, int t, RouteShared& sh) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int E = a.E;
  if (a.logits) {
    if (tid < E) sh.z[tid] = a.logits[(size_t)t * E + tid];
  } else {
    for (int e = wave; e < E; e += 4) {
      float p = 0.0f;
      for (int i = lane; i < a.d_model; i += 64)
        p = fmaf(a.w_router[(size_t)e * a.d_model + i], load_act<ACT>(a.x, (size_t)t * a.d_model + i), p);
      p = wave_sum(p);
      if (lane == 0) sh.z[e] = p;
    }
  }
  __syncthreads();
  if (tid < E) {
    const float z = sh.z[tid];
    if (a.logits_out) a.logits_out[(size_t)t * E + tid] = z;
    const float score = z + (a.bias ? a.bias[tid] : 0.0f);          // one fp32 add
    // larger score first; equal scores -> lower expert index
    sh.key[tid] = ((unsigned long long)orderable(score) << 32) | (uint32_t)(0xFFFFFFFFu - (uint32_t)tid);
  }
  __syncthreads();
  if (wave == 0) {
    float m = -INFINITY;
    for (int e = lane; e < E; e += 64) m = fmaxf(m, sh.z[e]);
    for (int s = 32; s >= 1; s >>= 1) m = fmaxf(m, __shfl_xor(m, s));
    float den = 0.0f;
    for (int e = lane; e < E; e += 64) den += expf(sh.z[e] - m);
    den = wave_sum(den);
    float wsum = 0.0f;
    for (int j = 0; j < a.k; j++) {
      unsigned long long best = 0;
      for (int e = lane; e < E; e += 64) best = sh.key[e] > best ? sh.key[e] : best;
      best = wave_max_u64(best);
      const int e_star = (int)(0xFFFFFFFFu - (uint32_t)best);
      const float wj = expf(sh.z[e_star] - m) / den;
      wsum += wj;
      if (lane == 0) { sh.sel[j] = e_star; sh.wsel[j] = wj; sh.key[e_star] = 0; }
      // the key write must be visible to the whole wave before the next scan
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
      __builtin_amdgcn_wave_barrier();
    }
    const float mul = (a.norm_topk ? 1.0f / wsum : 1.0f) * a.routed_scale;
    if (lane < a.k) {
      const float wj = sh.wsel[lane] * mul;
      sh.wsel[lane] = wj;
      a.idx[(size_t)t * a.k + lane] = sh.sel[lane];
      a.w[(size_t)t * a.k + lane] = wj;
    }
  }
  __syncthreads();
}
