// Prefill (paper Section 4.3: token-parallel, every expert high-bit, per-expert access counts):
//   route        eight tokens per work-group: router mat-vec, top-k (route.hip)
//   group        one work-group per expert: histogram, row offsets, list of (expert, row) tiles, stable
//                list of the expert's (token, slot) pairs
//   gemm<0>      grouped GEMM  H = silu(X Wg^T) * (X Wu^T)     (bf16 MFMA, fp32 accumulate)
//   gemm<1>      grouped GEMM  O = w * (H Wd^T)
//   combine      Y[t] = sum over slots (slot order) O[(t, slot)]  (+ x)
// Weights are read from the same nibble planes the decode path uses and expanded to
// bf16 s*(16 msb + lsb - zp) on the way into LDS.
#include "route_device.hpp"

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

#define PF_BM 192          // token rows per work-group tile
#define PF_BN 128          // weight rows per work-group tile
#define PF_BK 64
#define PF_LDK 72          // padded LDS row length in bf16 (144 bytes)

// ------------------------------------------------------------------------------- small kernels
#define GR_THREADS 1024
// One work-group per expert e, no global atomics and no ordering between work-groups: each counts
// every expert's selections in LDS, so it knows its own row offset and tile offset.  Writes
//   hist[e]    number of (token, slot) pairs routed to e (the per-expert access count of the layer)
//   offsets[e] first row of expert e in the grouped layout (offsets[E] = total)
//   tiles[0]   number of row tiles; tiles[1 + 2i], tiles[2 + 2i] = expert and first row (inside the
//              expert) of tile i, experts ascending
//   rows[p]    flat (token*k + slot) index of the p-th row of the grouped layout, ascending inside an
//              expert; pos = inverse of rows.
__global__ __launch_bounds__(GR_THREADS) void group_kernel(const int32_t* idx, int n, int E, uint32_t* hist,
                                                           int32_t* offsets, int32_t* tiles, int32_t* rows, int32_t* pos) {
  __shared__ int cnt[SMOE_MAX_EXPERTS];
  __shared__ int wtot[GR_THREADS / 64];
  const int e = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (tid < SMOE_MAX_EXPERTS) cnt[tid] = 0;
  __syncthreads();
  const int c = (n + GR_THREADS - 1) / GR_THREADS;          // every thread owns a contiguous run of c pairs
  const int i0 = min(n, tid * c), i1 = min(n, i0 + c);
  int mine = 0;
  for (int i = i0; i < i1; i++) {
    const int v = idx[i];
    if ((unsigned)v < (unsigned)E) atomicAdd(&cnt[v], 1);
    mine += v == e;
  }
  int incl = mine;
  for (int s = 1; s < 64; s <<= 1) { const int o = __shfl_up(incl, s); if (lane >= s) incl += o; }
  if (lane == 63) wtot[wave] = incl;
  __syncthreads();
  int p = incl - mine;
  for (int w = 0; w < wave; w++) p += wtot[w];
  int off = 0, nt = 0;
  for (int j = 0; j < e; j++) { off += cnt[j]; nt += (cnt[j] + PF_BM - 1) / PF_BM; }
  p += off;
  for (int i = i0; i < i1; i++)
    if (idx[i] == e) { rows[p] = i; pos[i] = p; p++; }
  if (tid == 0) {
    const int ne = cnt[e];
    hist[e] = (uint32_t)ne;
    offsets[e] = off;
    for (int m0 = 0; m0 < ne; m0 += PF_BM) { tiles[1 + 2 * nt] = e; tiles[2 + 2 * nt] = m0; nt++; }
    if (e == E - 1) { offsets[E] = off + ne; tiles[0] = nt; }
  }
}

// ------------------------------------------------------------------------------- grouped GEMM
struct GemmArgs {
  MatDev w;                 // gu (MODE 0) or dn (MODE 1) family of the bank
  int sc_bf16, group;
  const int32_t* offsets;   // [E+1]
  const int32_t* tiles;     // tile list written by group_kernel
  const int32_t* rows;      // [T*k]
  const uint16_t* x;        // MODE 0: X [T, d_model] bf16
  uint16_t* h;              // H [T*k, d_ff] bf16 (MODE 0 output, MODE 1 input)
  float* o;                 // MODE 1 output [T*k, d_model] fp32
  const float* wgt;         // [T*k] gate weights (flat token*k + slot)
  int k, d_model, d_ff;
};

__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
  f32x2 v = {a, b};
  bf16x2 r = __builtin_convertvector(v, bf16x2);
  return *(uint32_t*)&r;
}

// Work-group barrier that orders LDS traffic only: the global loads of the prefetch stay in flight
// across it (__syncthreads would wait for them and undo the prefetch).
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

template <int MODE>
__global__ __launch_bounds__(256) void grouped_gemm_kernel(GemmArgs a) {
  __shared__ __align__(16) uint16_t As[PF_BM * PF_LDK];
  __shared__ __align__(16) uint16_t Bs[PF_BN * PF_LDK];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int nt = blockIdx.x, ti = blockIdx.y;
  if (ti >= a.tiles[0]) return;
  const int e = a.tiles[1 + 2 * ti], m0 = a.tiles[2 + 2 * ti];
  const int row0 = a.offsets[e];
  const int m_cnt = min(PF_BM, a.offsets[e + 1] - row0 - m0);
  const int K = MODE == 0 ? a.d_model : a.d_ff;
  const int mh = wave >> 1, nh = wave & 1;

  // ---- loader roles
  // A: 192 rows x 8 sixteen-byte columns = 1536 vectors, 6 per thread
  const uint16_t* a_src[6];                 // an absent row reads the start of the matrix and is stored as zeros
  int a_dst[6];
  unsigned a_live = 0;
#pragma unroll
  for (int q = 0; q < 6; q++) {
    const int i = tid + 256 * q, r = i >> 3, c = i & 7;
    a_dst[q] = r * PF_LDK + c * 8;
    a_src[q] = MODE == 0 ? a.x : (const uint16_t*)a.h;
    if (r < m_cnt) {
      a_live |= 1u << q;
      if (MODE == 0) a_src[q] = a.x + (size_t)(a.rows[row0 + m0 + r] / a.k) * a.d_model + c * 8;
      else a_src[q] = a.h + (size_t)(row0 + m0 + r) * a.d_ff + c * 8;
    }
  }
  // B: 128 weight rows x 2 chunks of 32 columns; thread -> (row, chunk)
  const int wr = tid >> 1, wc = tid & 1;
  int grow;                                   // row inside the bank's matrix family
  if (MODE == 0) {
    const int half = wr >> 6, t = wr & 63;    // wave column block, then 32 gate rows + 32 up rows
    const int col = nt * 64 + half * 32 + (t & 31);
    grow = 2 * col + (t >> 5);
  } else {
    grow = nt * PF_BN + wr;
  }
  const uint8_t* pm = a.w.msb + (size_t)e * a.w.plane_stride + (size_t)grow * (K >> 1) + wc * 16;
  const uint8_t* pl = a.w.lsb + (size_t)e * a.w.plane_stride + (size_t)grow * (K >> 1) + wc * 16;
  const uint8_t* pz = a.w.zp + (size_t)e * a.w.zp_stride + (size_t)grow * a.w.ng;
  const uint8_t* ps = a.w.sc + (size_t)e * a.w.sc_stride;
  const size_t srow = (size_t)grow * a.w.sng;
  const int b_dst = wr * PF_LDK + wc * 32;

  f32x16 acc[3][2];
#pragma unroll
  for (int i = 0; i < 3; i++)
#pragma unroll
    for (int j = 0; j < 2; j++)
#pragma unroll
      for (int r = 0; r < 16; r++) acc[i][j][r] = 0.0f;

  // number of 32-row fragments this wave really has (fragments are mh, mh+2, mh+4)
  const int n_frag_total = (m_cnt + 31) >> 5;

  // two register sets of prefetched inputs: the loads of K step t+2 are issued while step t is
  // computed, which is what it takes to cover the memory latency of a loaded machine
  // (the registers hold what the loads return, untouched: any arithmetic on them at this point
  // would make it wait for the loads)
  struct Pre { uint4 ra[6], rm, rl; uint32_t rs, rz, rzs; };
  auto gload = [&](int k0, Pre& p) {
#pragma unroll
    for (int q = 0; q < 6; q++) p.ra[q] = *(const uint4*)(a_src[q] + k0);
    p.rm = *(const uint4*)(pm + (k0 >> 1));
    p.rl = *(const uint4*)(pl + (k0 >> 1));
    const unsigned g = (unsigned)(k0 + wc * 32) / (unsigned)a.group;
    if (a.sc_bf16) p.rs = ((const uint16_t*)ps)[srow + g];
    else p.rs = ((const uint32_t*)ps)[srow + g];
    const size_t zi = (size_t)(pz - a.w.zp) + g;                  // byte index inside the zero-point section
    p.rz = ((const uint32_t*)a.w.zp)[zi >> 2];                    // the aligned word that holds it
    p.rzs = (unsigned)(zi & 3) * 8u;
  };
  auto lstore = [&](const Pre& p) {
#pragma unroll
    for (int q = 0; q < 6; q++) *(uint4*)(As + a_dst[q]) = (a_live >> q) & 1 ? p.ra[q] : make_uint4(0, 0, 0, 0);
    const uint32_t wm[4] = {p.rm.x, p.rm.y, p.rm.z, p.rm.w}, wl[4] = {p.rl.x, p.rl.y, p.rl.z, p.rl.w};
    const float rs = __uint_as_float(a.sc_bf16 ? p.rs << 16 : p.rs);
    const float c0 = -(float)((p.rz >> p.rzs) & 0xFFu) * rs;
    uint32_t out[16];
#pragma unroll
    for (int j = 0; j < 4; j++) {
      // the planes hold n ^ 8 per nibble
      const uint32_t qe = (((wm[j] & 0x0F0F0F0Fu) << 4) | (wl[j] & 0x0F0F0F0Fu)) ^ 0x88888888u;      // even columns
      const uint32_t qo = ((wm[j] & 0xF0F0F0F0u) | ((wl[j] >> 4) & 0x0F0F0F0Fu)) ^ 0x88888888u;     // odd columns
#pragma unroll
      for (int b = 0; b < 4; b++) {
        const float we = fmaf((float)((qe >> (8 * b)) & 0xFF), rs, c0);
        const float wo = fmaf((float)((qo >> (8 * b)) & 0xFF), rs, c0);
        out[4 * j + b] = pack_bf16(we, wo);
      }
    }
#pragma unroll
    for (int v = 0; v < 4; v++)
      *(uint4*)(Bs + b_dst + 8 * v) = make_uint4(out[4 * v], out[4 * v + 1], out[4 * v + 2], out[4 * v + 3]);
  };
  auto compute = [&]() {
#pragma unroll
    for (int s = 0; s < PF_BK / 16; s++) {
      const int ko = s * 16 + (lane >> 5) * 8;
      bf16x8 bf[2];
#pragma unroll
      for (int j = 0; j < 2; j++) bf[j] = *(const bf16x8*)(Bs + (nh * 64 + j * 32 + (lane & 31)) * PF_LDK + ko);
#pragma unroll
      for (int i = 0; i < 3; i++) {
        const int frag = mh + 2 * i;
        if (frag < n_frag_total) {
          const bf16x8 af = *(const bf16x8*)(As + (frag * 32 + (lane & 31)) * PF_LDK + ko);
#pragma unroll
          for (int j = 0; j < 2; j++) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af, bf[j], acc[i][j], 0, 0, 0);
        }
      }
    }
  };

  const int nk = K / PF_BK;
  Pre p0, p1;
  gload(0, p0);
  if (nk > 1) gload(PF_BK, p1);
  for (int t = 0; t < nk; t += 2) {
    lds_barrier();                // previous tile fully consumed
    lstore(p0);
    lds_barrier();
    if (t + 2 < nk) gload((t + 2) * PF_BK, p0);
    compute();
    if (t + 1 < nk) {
      lds_barrier();
      lstore(p1);
      lds_barrier();
      if (t + 3 < nk) gload((t + 3) * PF_BK, p1);
      compute();
    }
  }

  // ---- epilogue.  D layout: register r of lane l is row 8*(r/4) + 4*(l/32) + r%4, column l%32.
#pragma unroll
  for (int i = 0; i < 3; i++) {
    const int frag = mh + 2 * i;
    if (frag >= n_frag_total) continue;
#pragma unroll
    for (int r = 0; r < 16; r++) {
      const int m = frag * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
      if (m >= m_cnt) continue;
      const size_t prow = (size_t)(row0 + m0 + m);
      if (MODE == 0) {
        const int col = nt * 64 + nh * 32 + (lane & 31);
        const float g = acc[i][0][r], u = acc[i][1][r];
        const float hv = g / (1.0f + __expf(-g)) * u;
        a.h[prow * a.d_ff + col] = (uint16_t)f32_to_bf16_bits(hv);
      } else {
        const float wt = a.wgt[a.rows[prow]];
#pragma unroll
        for (int j = 0; j < 2; j++) {
          const int col = nt * PF_BN + nh * 64 + j * 32 + (lane & 31);
          a.o[prow * a.d_model + col] = wt * acc[i][j][r];
        }
      }
    }
  }
}

// Y[t, c] = sum_j O[pos[t*k + j], c]  (+ x[t, c]); 4 columns per thread.
__global__ __launch_bounds__(256) void combine_kernel(const float* o, const int32_t* pos, const uint16_t* x, uint16_t* y,
                                                      int k, int d_model, int add_residual) {
  const int t = blockIdx.x;
  for (int c = threadIdx.x * 4; c < d_model; c += 256 * 4) {
    float4 s = make_float4(0, 0, 0, 0);
    for (int j = 0; j < k; j++) {
      const float4 v = *(const float4*)(o + (size_t)pos[t * k + j] * d_model + c);
      s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
    }
    if (add_residual) {
      const uint2 xv = *(const uint2*)(x + (size_t)t * d_model + c);
      s.x += bf16_bits_to_f32(xv.x & 0xFFFF); s.y += bf16_bits_to_f32(xv.x >> 16);
      s.z += bf16_bits_to_f32(xv.y & 0xFFFF); s.w += bf16_bits_to_f32(xv.y >> 16);
    }
    uint2 r;
    r.x = f32_to_bf16_bits(s.x) | (f32_to_bf16_bits(s.y) << 16);
    r.y = f32_to_bf16_bits(s.z) | (f32_to_bf16_bits(s.w) << 16);
    *(uint2*)(y + (size_t)t * d_model + c) = r;
  }
}

// ------------------------------------------------------------------------------- host entry
static inline size_t up256(size_t x) { return (x + 255) & ~(size_t)255; }

struct PrefillLayout { size_t rows, pos, offsets, tiles, h, o, total; };

static inline int max_tiles(int T, int E, int k) { return E + (T * k) / PF_BM; }

static PrefillLayout prefill_layout(int T, int E, int k, int d_model, int d_ff) {
  PrefillLayout L;
  size_t off = 0;
  L.rows = off;    off = up256(off + (size_t)T * k * 4);
  L.pos = off;     off = up256(off + (size_t)T * k * 4);
  L.offsets = off; off = up256(off + (size_t)(E + 1) * 4);
  L.tiles = off;   off = up256(off + (size_t)(1 + 2 * max_tiles(T, E, k)) * 4);
  L.h = off;       off = up256(off + (size_t)T * k * d_ff * 2);
  L.o = off;       off = up256(off + (size_t)T * k * d_model * 4);
  L.total = off;
  return L;
}

extern "C" int smoe_prefill_bytes(int T, int E, int k, int d_model, int d_ff, int shared_d_ff, size_t* scratch_bytes) {
  if (!scratch_bytes) return SMOE_EINVAL;
  if (T <= 0 || E <= 0 || k <= 0 || k > E || d_model <= 0 || d_ff <= 0 || shared_d_ff < 0) return SMOE_ESHAPE;
  *scratch_bytes = prefill_layout(T, E, k, d_model, d_ff).total;
  return SMOE_OK;
}

extern "C" int smoe_prefill_histogram(smoe_ctx* ctx, const smoe_bank* routed, const smoe_bank* shared, int T,
                                      const void* x_dev, int act_dtype, int k, const float* logits_dev,
                                      const float* w_router_dev, int norm_topk, float routed_scale,
                                      const void* shared_gate_w_dev, int add_residual, void* scratch_dev,
                                      size_t scratch_bytes, void* y_dev, int32_t* idx_dev, float* w_dev,
                                      uint32_t* hist_dev) {
  if (!ctx || !routed || !x_dev || !scratch_dev || !y_dev || !idx_dev || !w_dev || !hist_dev) return SMOE_EINVAL;
  if (!logits_dev && !w_router_dev) return SMOE_EINVAL;
  if (shared || shared_gate_w_dev) return SMOE_ENOTIMPL;          // shared-expert group: decode path only
  if (act_dtype != SMOE_BF16) return SMOE_ENOTIMPL;
  if (routed->device != ctx->device) return SMOE_EINVAL;
  const int E = routed->desc.n_experts, d = routed->desc.d_model, f = routed->desc.d_ff;
  if (T <= 0 || k <= 0 || k > E || k > SMOE_MAX_TOPK || E > SMOE_MAX_EXPERTS) return SMOE_ESHAPE;
  if (d % PF_BN || f % PF_BK || d % PF_BK || f % 64 || (routed->desc.group % 32)) return SMOE_ESHAPE;
  if (!aligned16(x_dev) || !aligned16(y_dev) || !aligned16(idx_dev) || !aligned16(w_dev) || !aligned16(hist_dev) ||
      !aligned16(logits_dev) || !aligned16(w_router_dev) || (((uintptr_t)scratch_dev) & 255u))
    return SMOE_EALIGN;
  const PrefillLayout L = prefill_layout(T, E, k, d, f);
  if (scratch_bytes < L.total) return SMOE_ESIZE;
  HIPCHK(ctx, hipSetDevice(ctx->device));
  uint8_t* s = (uint8_t*)scratch_dev;
  int32_t* rows = (int32_t*)(s + L.rows);
  int32_t* pos = (int32_t*)(s + L.pos);
  int32_t* offsets = (int32_t*)(s + L.offsets);
  int32_t* tiles = (int32_t*)(s + L.tiles);
  uint16_t* h = (uint16_t*)(s + L.h);
  float* o = (float*)(s + L.o);
  hipStream_t st = ctx->stream;

  RouteArgs ra{E, k, d, logits_dev, x_dev, w_router_dev, nullptr, norm_topk, routed_scale, nullptr, idx_dev, w_dev};
  { const int rc = smoe_launch_route(ctx, ra, T, SMOE_BF16); if (rc) return rc; }
  group_kernel<<<E, GR_THREADS, 0, st>>>(idx_dev, T * k, E, hist_dev, offsets, tiles, rows, pos);

  GemmArgs g{};
  g.sc_bf16 = routed->dev.sc_bf16; g.group = routed->dev.group; g.offsets = offsets; g.tiles = tiles; g.rows = rows;
  g.x = (const uint16_t*)x_dev; g.h = h; g.o = o; g.wgt = w_dev; g.k = k; g.d_model = d; g.d_ff = f;
  const int mt = max_tiles(T, E, k);             // upper bound of the tile count; surplus work-groups return at once
  g.w = routed->dev.gu;
  grouped_gemm_kernel<0><<<dim3(f / 64, mt), 256, 0, st>>>(g);
  g.w = routed->dev.dn;
  grouped_gemm_kernel<1><<<dim3(d / PF_BN, mt), 256, 0, st>>>(g);
  combine_kernel<<<T, 256, 0, st>>>(o, pos, (const uint16_t*)x_dev, (uint16_t*)y_dev, k, d, add_residual);
  HIPCHK(ctx, hipGetLastError());
  return SMOE_OK;
}
