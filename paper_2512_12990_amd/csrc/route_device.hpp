// Cache-aware top-k routing (paper Section 2.1: experts whose slices are resident get their
// gating score boosted before selection): device routines shared by the routing entry points.
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

// Top-k selection of one token by ONE wave.  z[0..E) are the token's logits (LDS), key[0..E) is
// scratch (LDS).  Writes a.idx / a.w for token t and leaves the decision in sel[] / wsel[] (LDS).
// Rule: k largest z + bias from the highest down, equal scores to the lower expert index; weights
// = softmax of the unbiased logits at the selected experts (optionally renormalised), * scale.
__device__ __forceinline__ void select_topk_wave(const RouteArgs& a, int t, const float* z, unsigned long long* key,
                                                 int* sel, float* wsel, int lane) {
  const int E = a.E;
  for (int e = lane; e < E; e += 64) {
    const float score = z[e] + (a.bias ? a.bias[e] : 0.0f);          // one fp32 add
    key[e] = ((unsigned long long)orderable(score) << 32) | (uint32_t)(0xFFFFFFFFu - (uint32_t)e);
  }
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
  __builtin_amdgcn_wave_barrier();
  float m = -INFINITY;
  for (int e = lane; e < E; e += 64) m = fmaxf(m, z[e]);
  for (int s = 32; s >= 1; s >>= 1) m = fmaxf(m, __shfl_xor(m, s));
  float den = 0.0f;
  for (int e = lane; e < E; e += 64) den += expf(z[e] - m);
  den = wave_sum(den);
  float wsum = 0.0f;
  for (int j = 0; j < a.k; j++) {
    unsigned long long best = 0;
    for (int e = lane; e < E; e += 64) best = key[e] > best ? key[e] : best;
    best = wave_max_u64(best);
    const int e_star = (int)(0xFFFFFFFFu - (uint32_t)best);
    const float wj = expf(z[e_star] - m) / den;
    wsum += wj;
    if (lane == 0) { sel[j] = e_star; wsel[j] = wj; key[e_star] = 0; }
    // the key write must be visible to the whole wave before the next scan
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_wave_barrier();
  }
  const float mul = (a.norm_topk ? 1.0f / wsum : 1.0f) * a.routed_scale;
  if (lane < a.k) {
    const float wj = wsel[lane] * mul;
    wsel[lane] = wj;
    a.idx[(size_t)t * a.k + lane] = sel[lane];
    a.w[(size_t)t * a.k + lane] = wj;
  }
}

// Dot products of one router row with NT activation vectors by one wave.  Lane l sums columns
// l, l+64, l+128, ... in that order by fused multiply-add, then the wave sum: every kernel that
// produces router logits uses this routine, so logits are bit-identical between entry points.
// xget(q, i) returns activation i of vector q.  The results are valid in every lane.
template <int NT, class XF>
__device__ __forceinline__ void router_row_dots(const float* __restrict__ wrow, int d, int lane, XF xget, float* p) {
#pragma unroll
  for (int q = 0; q < NT; q++) p[q] = 0.0f;
  int i0 = 0;
  for (; i0 + 512 <= d; i0 += 512) {          // eight loads in flight per lane
    float w[8];
#pragma unroll
    for (int u = 0; u < 8; u++) w[u] = wrow[i0 + u * 64 + lane];
#pragma unroll
    for (int u = 0; u < 8; u++)
#pragma unroll
      for (int q = 0; q < NT; q++) p[q] = fmaf(w[u], xget(q, i0 + u * 64 + lane), p[q]);
  }
  for (int i = i0 + lane; i < d; i += 64) {
    const float w = wrow[i];
#pragma unroll
    for (int q = 0; q < NT; q++) p[q] = fmaf(w, xget(q, i), p[q]);
  }
#pragma unroll
  for (int q = 0; q < NT; q++) p[q] = wave_sum(p[q]);
}

// Dot products of RT_R consecutive router rows (first row e0; rows past E repeat row E-1 and are
// discarded by the caller) with the NT activation vectors of the work-group.  xs holds the vectors
// column by column ([d][NT] in storage dtype, 16 bytes per column), so one LDS read feeds NT*RT_R
// multiply-adds.  Every (row, vector) sum takes the columns in the order router_row_dots does.
#define RT_R 4
// Position (in 16-byte units) of column i of the staged activations: one unit of padding after every
// nt columns, so the nt-column blocks that the staging threads of a wave write start in different banks.
__device__ __forceinline__ int rt_col(int i, int nt) { return i + i / nt; }
template <int ACT, int NT>
__device__ __forceinline__ void router_rows_dots_lds(const float* __restrict__ w_router, int e0, int E, int d, int lane,
                                                     const uint4* xs, float (&p)[RT_R][NT]) {
  static_assert((ACT == SMOE_BF16 && NT == 8) || (ACT == SMOE_F32 && NT == 4), "one column of xs is 16 bytes");
  const float* wrow[RT_R];
#pragma unroll
  for (int r = 0; r < RT_R; r++) {
    wrow[r] = w_router + (size_t)min(e0 + r, E - 1) * d;
#pragma unroll
    for (int q = 0; q < NT; q++) p[r][q] = 0.0f;
  }
  auto column = [&](int i, float (&xf)[NT]) {
    const uint4 v = xs[rt_col(i, NT)];
    if (ACT == SMOE_BF16) {
      const uint32_t u[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
      for (int j = 0; j < 4; j++) {
        xf[(2 * j) % NT] = __uint_as_float(u[j] << 16);
        xf[(2 * j + 1) % NT] = __uint_as_float(u[j] & 0xFFFF0000u);
      }
    } else {
      xf[0] = __uint_as_float(v.x); xf[1] = __uint_as_float(v.y);
      xf[2 % NT] = __uint_as_float(v.z); xf[3 % NT] = __uint_as_float(v.w);
    }
  };
  int i0 = 0;
  for (; i0 + 512 <= d; i0 += 512) {
    float w[RT_R][8];
#pragma unroll
    for (int r = 0; r < RT_R; r++)
#pragma unroll
      for (int u = 0; u < 8; u++) w[r][u] = wrow[r][i0 + u * 64 + lane];
#pragma unroll
    for (int u = 0; u < 8; u++) {
      float xf[NT];
      column(i0 + u * 64 + lane, xf);
#pragma unroll
      for (int r = 0; r < RT_R; r++)
#pragma unroll
        for (int q = 0; q < NT; q++) p[r][q] = fmaf(w[r][u], xf[q], p[r][q]);
    }
  }
  for (int i = i0 + lane; i < d; i += 64) {
    float xf[NT];
    column(i, xf);
#pragma unroll
    for (int r = 0; r < RT_R; r++) {
      const float w = wrow[r][i];
#pragma unroll
      for (int q = 0; q < NT; q++) p[r][q] = fmaf(w, xf[q], p[r][q]);
    }
  }
#pragma unroll
  for (int r = 0; r < RT_R; r++)
#pragma unroll
    for (int q = 0; q < NT; q++) p[r][q] = wave_sum(p[r][q]);
}

// Routes NT tokens per work-group of RT_NW waves: every router row is read once per group, each wave
// then selects for its share of the tokens.
// Dynamic LDS: NT*E floats, RT_NW*E 64-bit keys, RT_NW*16 ints, RT_NW*16 floats, then (without given logits)
// the activations, 16 bytes per column plus padding.
#define RT_NW 16
#define RT_THREADS (RT_NW * 64)
template <int ACT, int NT>
__device__ __forceinline__ void route_tokens_block(const RouteArgs& a, int T, uint8_t* dyn) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int E = a.E, d = a.d_model;
  const int t0 = blockIdx.x * NT, nt = min(NT, T - t0);
  float* zt = (float*)dyn;                                            // [NT][E]
  unsigned long long* key = (unsigned long long*)(zt + NT * E);      // [RT_NW waves][E]
  int* sel = (int*)(key + RT_NW * E);                                 // [RT_NW][16]
  float* wsel = (float*)(sel + RT_NW * SMOE_MAX_TOPK);                // [RT_NW][16]
  if (a.logits) {
    for (int i = tid; i < nt * E; i += RT_THREADS) zt[i] = a.logits[(size_t)t0 * E + i];
  } else {
    uint8_t* xs = (uint8_t*)(wsel + RT_NW * SMOE_MAX_TOPK);           // 16 bytes per column, see rt_col()
    constexpr int ESZ = ACT == SMOE_BF16 ? 2 : 4;
    if (d % NT == 0) {
      // a thread moves NT consecutive columns of one vector: one 16-byte load, NT LDS stores
      const int q = tid % NT;
      for (int cb = tid / NT; cb * NT < d; cb += RT_THREADS / NT) {
        uint4 v = make_uint4(0, 0, 0, 0);
        if (q < nt) v = *(const uint4*)((const uint8_t*)a.x + ((size_t)(t0 + q) * d + (size_t)cb * NT) * ESZ);
        const uint32_t u[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int j = 0; j < NT; j++) {
          uint8_t* dst = xs + (size_t)rt_col(cb * NT + j, NT) * 16 + q * ESZ;
          if (ACT == SMOE_BF16) *(uint16_t*)dst = (uint16_t)(u[j / 2] >> ((j & 1) * 16));
          else *(uint32_t*)dst = u[j % 4];
        }
      }
    } else {
      for (int i = tid; i < NT * d; i += RT_THREADS) {
        const int q = i / d, c = i - q * d;
        uint8_t* dst = xs + (size_t)rt_col(c, NT) * 16 + q * ESZ;
        if (ACT == SMOE_BF16) *(uint16_t*)dst = q < nt ? ((const uint16_t*)a.x)[(size_t)t0 * d + i] : (uint16_t)0;
        else *(float*)dst = q < nt ? ((const float*)a.x)[(size_t)t0 * d + i] : 0.0f;
      }
    }
    __syncthreads();
    for (int e0 = wave * RT_R; e0 < E; e0 += RT_NW * RT_R) {
      float p[RT_R][NT];
      router_rows_dots_lds<ACT, NT>(a.w_router, e0, E, d, lane, (const uint4*)xs, p);
      if (lane == 0)
#pragma unroll
        for (int r = 0; r < RT_R; r++)
          if (e0 + r < E)
#pragma unroll
            for (int q = 0; q < NT; q++) zt[q * E + e0 + r] = p[r][q];
    }
  }
  __syncthreads();
  if (a.logits_out)
    for (int i = tid; i < nt * E; i += RT_THREADS) a.logits_out[(size_t)t0 * E + i] = zt[i];
  for (int q = wave; q < nt; q += RT_NW) {
    select_topk_wave(a, t0 + q, zt + q * E, key + wave * E, sel + wave * SMOE_MAX_TOPK, wsel + wave * SMOE_MAX_TOPK, lane);
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_wave_barrier();
  }
}

template <int ACT, int NT> struct RouteLds {
  static size_t bytes(int E, int d, bool given_logits) {
    return (size_t)NT * E * 4 + (size_t)RT_NW * E * 8 + RT_NW * SMOE_MAX_TOPK * 8 +
           (given_logits ? 0 : (size_t)(d + d / NT + 1) * 16);
  }
};
