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
#include <type_traits>

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x8 __attribute__((ext_vector_type(8)));
struct __attribute__((packed)) U32x2Unaligned { uint32_t x, y; };
struct __attribute__((packed, aligned(4))) U32x3Words { uint32_t x, y, z; };      // twelve bytes on a 4-byte boundary

#define PF_BM 192          // token rows per work-group tile
#define PF_BN 256          // weight rows per work-group tile
#define PF_BK 64
#define PF_NT 512          // threads per work-group
#define PF_LDK 72          // padded LDS row length in bf16 (144 bytes)

// ------------------------------------------------------------------------------- small kernels
#define GR_THREADS 1024
// One work-group per expert e, no global atomics and no ordering between work-groups: each counts
// every expert's selections in LDS, so it knows its own row offset and tile offset.  Writes
//   hist[e]    number of (token, slot) pairs routed to e (the per-expert access count of the layer)
//   offsets[e] first row of expert e in the grouped layout (offsets[E] = total)
//   tiles[0]   number of row tiles; tiles[4 + 4i ..] = {expert, first row inside the expert, first row
//              in the grouped layout, rows} of tile i, tiles with more rows first (equal sizes:
//              expert, then row, ascending), so that the work-groups that start last are the short ones
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
  // a run of up to GR_RUN pairs is fetched into registers before the first is used (all loads in
  // flight at once) and serves both passes; longer runs are read pair by pair
  constexpr int GR_RUN = 8;
  int v8[GR_RUN];
  const bool in_regs = c <= GR_RUN;
  if (in_regs) {
#pragma unroll
    for (int u = 0; u < GR_RUN; u++) v8[u] = i0 + u < i1 ? idx[i0 + u] : -1;
  }
  int mine = 0;
  if (in_regs) {
#pragma unroll
    for (int u = 0; u < GR_RUN; u++) {
      if ((unsigned)v8[u] < (unsigned)E) atomicAdd(&cnt[v8[u]], 1);
      mine += v8[u] == e;
    }
  } else {
    for (int i = i0; i < i1; i++) {
      const int v = idx[i];
      if ((unsigned)v < (unsigned)E) atomicAdd(&cnt[v], 1);
      mine += v == e;
    }
  }
  int incl = mine;
  for (int s = 1; s < 64; s <<= 1) { const int o = __shfl_up(incl, s); if (lane >= s) incl += o; }
  if (lane == 63) wtot[wave] = incl;
  __syncthreads();
  // Wave 0 turns the counts into what the work-group needs (lane x takes experts x, x + 64, ...): rows
  // and tiles of the experts before e, all full tiles, and the ragged tiles that precede e's ragged one
  // (more rows first; equal sizes by expert).
  __shared__ int summary[4];      // rows before e, full tiles before e, full tiles in all, ragged tiles before e's
  const int ne = cnt[e];
  const int rem = ne % PF_BM;
  if (wave == 0) {
    int s_off = 0, s_fb = 0, s_fa = 0, s_rb = 0, s_ra = 0;
    for (int x = lane; x < E; x += 64) {
      const int cx = cnt[x], fx = cx / PF_BM, rx = cx - fx * PF_BM;
      s_fa += fx;
      s_ra += rx > 0;
      if (x < e) { s_off += cx; s_fb += fx; }
      s_rb += rx > rem || (rx == rem && x < e);
    }
    for (int m = 32; m >= 1; m >>= 1) {
      s_off += __shfl_xor(s_off, m); s_fb += __shfl_xor(s_fb, m); s_fa += __shfl_xor(s_fa, m);
      s_rb += __shfl_xor(s_rb, m); s_ra += __shfl_xor(s_ra, m);
    }
    if (lane == 0) { summary[0] = s_off; summary[1] = s_fb; summary[2] = s_fa; summary[3] = s_rb; }
    if (lane == 0 && e == E - 1) { offsets[E] = s_off + ne; tiles[0] = s_fa + s_ra; }
  }
  __syncthreads();
  int p = incl - mine;
  for (int w = 0; w < wave; w++) p += wtot[w];
  const int off = summary[0];
  p += off;
  if (in_regs) {
#pragma unroll
    for (int u = 0; u < GR_RUN; u++)
      if (v8[u] == e) { rows[p] = i0 + u; pos[i0 + u] = p; p++; }
  } else {
    for (int i = i0; i < i1; i++)
      if (idx[i] == e) { rows[p] = i; pos[i] = p; p++; }
  }
  if (tid == 0) {
    hist[e] = (uint32_t)ne;
    offsets[e] = off;
  }
  // Position of each of this expert's tiles in the list = number of tiles that precede it: every
  // full tile precedes a ragged one; full tiles among themselves and ragged tiles of equal size go
  // by expert (an expert has at most one ragged tile, its last).
  const int n_full = ne / PF_BM;
  for (int j = tid; j < n_full + (rem > 0); j += GR_THREADS) {
    const int rank = j < n_full ? summary[1] + j : summary[2] + summary[3];
    int4 rec;
    rec.x = e; rec.y = j * PF_BM; rec.z = off + j * PF_BM; rec.w = min(PF_BM, ne - j * PF_BM);
    *(int4*)(tiles + 4 + 4 * rank) = rec;
  }
}

// ------------------------------------------------------------------------------- grouped GEMM
struct GemmArgs {
  MatDev w;                 // gu (MODE 0) or dn (MODE 1) family of the bank
  int sc_bf16, group_shift; // quantisation group = 1 << group_shift columns
  const int32_t* offsets;   // [E+1]
  const int32_t* tiles;     // tile list written by group_kernel
  const int32_t* rows;      // [T*k]
  const uint16_t* x;        // MODE 0: X [T, d_model] bf16
  uint16_t* h;              // H [T*k, d_ff] bf16 (MODE 0 output, MODE 1 input)
  float* o;                 // MODE 1 output [T*k, d_model] fp32
  const float* wgt;         // [T*k] gate weights (flat token*k + slot)
  int k, d_model, d_ff;
  int n_col_tiles;          // column tiles of this GEMM (grid = 8 * ceil(max row tiles / 8) * n_col_tiles)
  // dense_rows > 0: one expert (dense_expert) takes rows 0..dense_rows-1 = tokens in their own order
  // (a shared expert): no tile list, no row list, H and O rows are token rows; wgt[t] scales row t
  int dense_rows, dense_expert;
  int accumulate;           // MODE 1: add to O instead of overwriting it
};

__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
  f32x2 v = {a, b};
  bf16x2 r = __builtin_convertvector(v, bf16x2);
  return *(uint32_t*)&r;
}

// Work-group barrier that orders LDS traffic only: the global loads of the prefetch stay in flight
// across it (__syncthreads would wait for them and undo the prefetch).
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// One work-group of eight waves (two per SIMD) per CU: the tile is 192 token rows x 256 weight rows,
// a wave owns 96 x 64 of it (3 x 2 MFMA fragments), and LDS holds two copies of the K slice so that
// one barrier per K step is enough.
template <int MODE, int SCB, int FMT>      // FMT 0: 8/4 nest, nibble planes; 1: 4/2 nest, 2-bit planes; 2: 6/3 nest, 3-bit planes
__global__ __launch_bounds__(PF_NT) void grouped_gemm_kernel(GemmArgs a) {
  // (separate arrays, so that the compiler knows a write into one buffer cannot alias a read of the other)
  __shared__ __align__(16) uint16_t As0[PF_BM * PF_LDK], As1[PF_BM * PF_LDK];
  __shared__ __align__(16) uint16_t Bs0[PF_BN * PF_LDK], Bs1[PF_BN * PF_LDK];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  // Work-groups go to the eight XCDs round-robin by their linear index.  All column tiles of one row
  // tile are given to the same XCD, consecutively, so its rows of A are fetched into one L2 only and
  // stay there while they are re-read.
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int ti = (slot / a.n_col_tiles) * 8 + xcd, nt = slot % a.n_col_tiles;
  int e, m0, row0, m_cnt;
  if (a.dense_rows) {
    if (ti * PF_BM >= a.dense_rows) return;
    e = a.dense_expert; m0 = ti * PF_BM; row0 = 0;
    m_cnt = min(PF_BM, a.dense_rows - m0);
  } else {
    const int n_tiles = a.tiles[0];
    const int4 rec = *(const int4*)(a.tiles + 4 + 4 * ti);      // (read before the count is known: inside the list's allocation)
    if (ti >= n_tiles) return;
    e = rec.x; m0 = rec.y; row0 = rec.z - rec.y; m_cnt = rec.w;
  }
  const int K = MODE == 0 ? a.d_model : a.d_ff;
  const int N = MODE == 0 ? a.d_ff : a.d_model;         // output columns of this GEMM
  // MODE 1: the weight of every row of the tile, fetched now for the epilogue (the barriers of the
  // K loop order it)
  __shared__ float row_wt[PF_BM];
  if (MODE == 1 && tid < PF_BM)
    row_wt[tid] = tid < m_cnt ? a.wgt[a.dense_rows ? m0 + tid : a.rows[row0 + m0 + tid]] : 0.0f;
  const int mh = wave >> 2, nq = wave & 3;

  // ---- loader roles
  // A: 192 rows x 8 sixteen-byte columns = 1536 vectors, 3 per thread
  // (a row past the tile's last one repeats that row: rows of the product are independent and the
  // epilogue stores none of the surplus ones)
  const uint16_t* a_base = MODE == 0 ? a.x : (const uint16_t*)a.h;
  uint32_t a_src[3];                        // element offsets into a_base (the host checks they fit 32 bits)
  const int a_dst0 = (tid >> 3) * PF_LDK + (tid & 7) * 8;       // vector q goes 64 rows further down
#pragma unroll
  for (int q = 0; q < 3; q++) {
    const int i = tid + PF_NT * q, r = min(i >> 3, m_cnt - 1), c = i & 7;
    if (MODE == 0) a_src[q] = (uint32_t)(a.dense_rows ? m0 + r : a.rows[row0 + m0 + r] / a.k) * (uint32_t)a.d_model + c * 8;
    else a_src[q] = (uint32_t)(row0 + m0 + r) * (uint32_t)a.d_ff + c * 8;
  }
  // B: thread -> (weight row b of the tile, half hb of the 64 columns of the K slice).  MODE 0: the 64
  // rows of a wave's column block are [gate 32 | up 32] of 32 output columns, so that gate and up
  // of one output element land in the same lane of two accumulators.
  const int b = tid >> 1, hb = tid & 1;
  int grow;                                   // row inside the bank's matrix family (clamped)
  if (MODE == 0) {
    const int col = nt * (PF_BN / 2) + (b >> 6) * 32 + (b & 31);
    grow = 2 * min(col, N - 1) + ((b >> 5) & 1);
  } else {
    grow = min(nt * PF_BN + b, N - 1);
  }
  // uniform 64-bit section bases + 32-bit per-thread offsets (every section of a bank is below 2 GiB)
  const uint8_t* pm = a.w.msb + (size_t)e * a.w.plane_stride;
  const uint8_t* pl = a.w.lsb + (size_t)e * a.w.plane_stride;
  const uint8_t* ps = a.w.sc + (size_t)e * a.w.sc_stride;
  const uint8_t* pz = a.w.zp + (size_t)e * a.w.zp_stride;       // 4-byte aligned: zp_stride is a multiple of 4
  constexpr int PB32 = FMT == 0 ? 16 : FMT == 1 ? 8 : 12;      // plane bytes of 32 columns
  const uint32_t poff = (uint32_t)grow * (uint32_t)((K >> 5) * PB32) + hb * PB32;
  const uint32_t srow = (uint32_t)grow * (uint32_t)a.w.sng;
  const uint32_t zrow = (uint32_t)grow * (uint32_t)a.w.ng;
  const int b_dst = b * PF_LDK + hb * 32;

  // Two register sets of prefetched inputs: the loads of K step t+2 are issued while step t is
  // computed.  The registers hold what the loads return, untouched: arithmetic on them at this
  // point would make the wave wait for the loads.
  struct PreA { u32x4 ra[3]; };
  typedef typename std::conditional<FMT == 1, u32x2, u32x4>::type PlaneV;      // a thread's 32 codes of one plane (FMT 2: three words used)
  struct Pre { PlaneV rm, rl; };
  // Scales and zero-points of eight consecutive groups of the thread's row (the chunk that holds the
  // groups of a K step), kept in registers and reloaded only when a step enters a new chunk: loading
  // them step by step costs a cache line per thread and step.  Reads are clamped to the expert's
  // section (what is read past the row's end belongs to groups the row does not have).
  constexpr int NSD = SCB ? 4 : 8;
  struct Meta { typename std::conditional<SCB != 0, u32x4, u32x8>::type s; u32x2 z; };     // (vector registers: picking one element by a run-time index stays in registers)
  const uint32_t last_s = (uint32_t)(a.w.sc_stride >> 2) - 1u, last_z = (uint32_t)a.w.zp_stride - 8u;
  auto chunk_of = [&](int k0) __attribute__((always_inline)) { return ((uint32_t)k0 >> a.group_shift) >> 3; };
  auto mload = [&](int k0, Meta& m) __attribute__((always_inline)) {
    const uint32_t c0 = chunk_of(k0) << 3;
    const uint32_t sd = SCB ? (srow + c0) >> 1 : srow + c0;         // srow is even
    const U32x2Unaligned zz = *(const U32x2Unaligned*)(pz + min(zrow + c0, last_z));    // eight bytes at any alignment
    m.z = u32x2{zz.x, zz.y};
#pragma unroll
    for (int j = 0; j < NSD; j++) m.s[j] = ((const uint32_t*)ps)[min(sd + j, last_s)];
  };
  auto gload_a = [&](int k0, PreA& p) __attribute__((always_inline)) {
#pragma unroll
    for (int q = 0; q < 3; q++) p.ra[q] = *(const u32x4*)(a_base + (a_src[q] + (uint32_t)k0));
  };
  auto lstore_a = [&](const PreA& p, uint16_t* As) __attribute__((always_inline)) {
#pragma unroll
    for (int q = 0; q < 3; q++) *(u32x4*)(As + a_dst0 + q * 64 * PF_LDK) = p.ra[q];
  };
  auto gload = [&](int k0, Pre& p) __attribute__((always_inline)) {
    const uint32_t o = poff + (uint32_t)((k0 >> 5) * PB32);
    if constexpr (FMT == 2) {
      const U32x3Words vm = *(const U32x3Words*)(pm + o), vl = *(const U32x3Words*)(pl + o);
      p.rm = u32x4{vm.x, vm.y, vm.z, 0u};
      p.rl = u32x4{vl.x, vl.y, vl.z, 0u};
    } else {
      p.rm = *(const PlaneV*)(pm + o);
      p.rl = *(const PlaneV*)(pl + o);
    }
  };
  auto lstore = [&](int k0, const Pre& p, const Meta& m, uint16_t* Bs) __attribute__((always_inline)) {
    const uint32_t g = (uint32_t)(k0 + 32 * hb) >> a.group_shift, gi = g & 7u;
    float rs;
    if (SCB) {
      const uint32_t d = m.s[gi >> 1];
      rs = __uint_as_float((gi & 1u) ? d & 0xFFFF0000u : d << 16);
    } else {
      rs = __uint_as_float(m.s[gi]);
    }
    const uint32_t zb = zrow + (g & ~7u);
    const uint32_t zo = zb - min(zb, last_z) + gi;                 // byte of the zero-point inside m.z
    const uint32_t zw = m.z[(zo >> 2) & 1u];
    const float c0 = -(float)((zw >> ((zo & 3u) * 8u)) & 0xFFu) * rs;
    uint32_t out[16];
#pragma unroll
    for (int j = 0; j < 4; j++) {
      uint32_t qe, qo;                          // codes of the even / odd columns of columns 8j .. 8j+7, one per byte
      if constexpr (FMT == 0) {
        // the planes hold n ^ 8 per nibble
        const uint32_t wm = p.rm[j], wl = p.rl[j];
        qe = (((wm & 0x0F0F0F0Fu) << 4) | (wl & 0x0F0F0F0Fu)) ^ 0x88888888u;
        qo = ((wm & 0xF0F0F0F0u) | ((wl >> 4) & 0x0F0F0F0Fu)) ^ 0x88888888u;
      } else if constexpr (FMT == 2) {
        // column 8j + i: two low bits in word j >> 1 at bits 4i + 2(j & 1), third bit in word 2 at bit
        // 4i + j; one value per nibble first, then code = 8 msb + lsb, one per byte
        auto nib = [&](const PlaneV& w) {
          const uint32_t lo = (w[j >> 1] >> (2 * (j & 1))) & 0x33333333u;
          const uint32_t hi = w[2] & (0x11111111u << j);
          return lo | (j < 2 ? hi << (2 - j) : hi >> (j - 2));
        };
        const uint32_t nm = nib(p.rm), nl = nib(p.rl);
        qe = ((nm & 0x0F0F0F0Fu) << 3) | (nl & 0x0F0F0F0Fu);
        qo = (((nm >> 4) & 0x0F0F0F0Fu) << 3) | ((nl >> 4) & 0x0F0F0F0Fu);
      } else {
        // sixteen 2-bit codes per plane word, column c in bits 2c, 2c+1: spread half a word to one
        // code per nibble, then code = 4 msb + lsb
        auto spread = [](uint32_t h) {
          h = (h | (h << 8)) & 0x00FF00FFu;
          h = (h | (h << 4)) & 0x0F0F0F0Fu;
          return (h | (h << 2)) & 0x33333333u;
        };
        const uint32_t hm = (p.rm[j >> 1] >> (16 * (j & 1))) & 0xFFFFu, hl = (p.rl[j >> 1] >> (16 * (j & 1))) & 0xFFFFu;
        const uint32_t qn = (spread(hm) << 2) | spread(hl);
        qe = qn & 0x0F0F0F0Fu;
        qo = (qn >> 4) & 0x0F0F0F0Fu;
      }
#pragma unroll
      for (int bb = 0; bb < 4; bb++) {
        const float we = fmaf((float)((qe >> (8 * bb)) & 0xFF), rs, c0);
        const float wo = fmaf((float)((qo >> (8 * bb)) & 0xFF), rs, c0);
        out[4 * j + bb] = pack_bf16(we, wo);
      }
    }
#pragma unroll
    for (int v = 0; v < 4; v++)
      *(u32x4*)(Bs + b_dst + 8 * v) = u32x4{out[4 * v], out[4 * v + 1], out[4 * v + 2], out[4 * v + 3]};
  };

  f32x16 acc[3][2];
#pragma unroll
  for (int i = 0; i < 3; i++)
#pragma unroll
    for (int j = 0; j < 2; j++)
#pragma unroll
      for (int r = 0; r < 16; r++) acc[i][j][r] = 0.0f;

  // 32-row fragments of this wave are mh, mh+2, mh+4; the first nf of them hold rows of the tile
  const int n_frag_total = (m_cnt + 31) >> 5;
  const int nf = n_frag_total > mh ? (n_frag_total - mh + 1) >> 1 : 0;
  const int nk = K / PF_BK;

  // K loop for a wave with NF live fragments: step t multiplies out of LDS buffer t&1 while the
  // inputs of step t+1 are expanded into the other buffer; the expansion (VALU) and the products
  // (MFMA) are independent instruction streams of one basic block, which the compiler interleaves.  Loads run two steps ahead;
  // past the end they repeat the last step (their results are not used).
  auto kloop = [&](auto nf_c) __attribute__((always_inline)) {
    constexpr int NF = decltype(nf_c)::value;
    auto compute = [&](const uint16_t* As, const uint16_t* Bs) __attribute__((always_inline)) {
#pragma unroll
      for (int s = 0; s < PF_BK / 16; s++) {
        const int ko = s * 16 + (lane >> 5) * 8;
        bf16x8 bf[2];
#pragma unroll
        for (int j = 0; j < 2; j++) bf[j] = *(const bf16x8*)(Bs + (nq * 64 + j * 32 + (lane & 31)) * PF_LDK + ko);
#pragma unroll
        for (int i = 0; i < NF; i++) {
          const bf16x8 af = *(const bf16x8*)(As + ((mh + 2 * i) * 32 + (lane & 31)) * PF_LDK + ko);
#pragma unroll
          for (int j = 0; j < 2; j++) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af, bf[j], acc[i][j], 0, 0, 0);
        }
      }
    };
    // The weight planes are prefetched two steps ahead in two register sets; the rows of A go
    // through one set: they are written to LDS first thing in a step and reloaded at once.
    Pre p0, p1;
    Meta m0, m1;
    PreA pa;
    const int k1 = min(1, nk - 1) * PF_BK, k2 = min(2, nk - 1) * PF_BK;
    gload_a(0, pa);
    gload(0, p0);
    mload(0, m0);
    gload(k1, p1);
    mload(k1, m1);
    lstore_a(pa, As0);
    gload_a(k1, pa);
    lstore(0, p0, m0, Bs0);
    gload(k2, p0);
    if (chunk_of(k2) != chunk_of(0)) mload(k2, m0);
    for (int t = 0; t < nk; t += 2) {
      lds_barrier();
      lstore_a(pa, As1);
      gload_a(min(t + 2, nk - 1) * PF_BK, pa);
      lstore((t + 1) * PF_BK, p1, m1, Bs1);
      compute(As0, Bs0);
      const int ka = min(t + 3, nk - 1) * PF_BK;
      gload(ka, p1);
      if (chunk_of(ka) != chunk_of(min(t + 1, nk - 1) * PF_BK)) mload(ka, m1);
      if (t + 1 < nk) {
        lds_barrier();
        lstore_a(pa, As0);
        gload_a(min(t + 3, nk - 1) * PF_BK, pa);
        lstore((t + 2) * PF_BK, p0, m0, Bs0);
        compute(As1, Bs1);
        const int kb = min(t + 4, nk - 1) * PF_BK;
        gload(kb, p0);
          if (chunk_of(kb) != chunk_of(min(t + 2, nk - 1) * PF_BK)) mload(kb, m0);
      }
    }
  };
  if (nf == 3) kloop(std::integral_constant<int, 3>());
  else if (nf == 2) kloop(std::integral_constant<int, 2>());
  else if (nf == 1) kloop(std::integral_constant<int, 1>());
  else kloop(std::integral_constant<int, 0>());

  // ---- epilogue.  D layout: register r of lane l is row 8*(r/4) + 4*(l/32) + r%4, column l%32.
#pragma unroll
  for (int i = 0; i < 3; i++) {
    if (i >= nf) continue;
    const int frag = mh + 2 * i;
#pragma unroll
    for (int r = 0; r < 16; r++) {
      const int m = frag * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
      if (m >= m_cnt) continue;
      const size_t prow = (size_t)(row0 + m0 + m);
      if (MODE == 0) {
        const int col = nt * (PF_BN / 2) + nq * 32 + (lane & 31);
        const float g = acc[i][0][r], u = acc[i][1][r];
        const float hv = g / (1.0f + __expf(-g)) * u;
        if (col < N) a.h[prow * a.d_ff + col] = (uint16_t)f32_to_bf16_bits(hv);
      } else {
        const float wt = row_wt[m];
#pragma unroll
        for (int j = 0; j < 2; j++) {
          const int col = nt * PF_BN + nq * 64 + j * 32 + (lane & 31);
          if (col < N) {
            float* dst = a.o + prow * a.d_model + col;
            *dst = a.accumulate ? *dst + wt * acc[i][j][r] : wt * acc[i][j][r];
          }
        }
      }
    }
  }
}

// gamma[t] = sigmoid(w_sg . x[t]) (one wave per token), or 1 without a gate vector: the weight of
// the shared experts' output for token t.
__global__ __launch_bounds__(256) void shared_gate_kernel(const uint16_t* x, const uint16_t* w_sg, int T, int d, float* gamma) {
  const int lane = threadIdx.x & 63, t = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (t >= T) return;
  float g = 1.0f;
  if (w_sg) {
    // 32 columns per lane are fetched into raw registers before the first is used (arithmetic on a
    // loaded value at the load site would make the wave wait for every load in turn)
    const uint16_t* xr = x + (size_t)t * d;
    float s = 0.0f;
    for (int i0 = 0; i0 < d; i0 += 2048) {
      uint32_t wv[32], xv[32];
#pragma unroll
      for (int u = 0; u < 32; u++) {
        const int i = min(i0 + u * 64 + lane, d - 1);
        wv[u] = w_sg[i];
        xv[u] = xr[i];
      }
#pragma unroll
      for (int u = 0; u < 32; u++) {
        const float q = fmaf(__uint_as_float(wv[u] << 16), __uint_as_float(xv[u] << 16), s);
        s = (i0 + u * 64 + lane) < d ? q : s;
      }
    }
    s = wave_sum(s);
    g = 1.0f / (1.0f + __expf(-s));
  }
  if (lane == 0) gamma[t] = g;
}

// Y[t, c] = sum_j O[pos[t*k + j], c]  (+ OS[t, c], the shared experts' sum)  (+ x[t, c]); 4 columns per thread.
__global__ __launch_bounds__(256) void combine_kernel(const float* o, const int32_t* pos, const float* o_s, const uint16_t* x,
                                                      uint16_t* y, int k, int d_model, int add_residual) {
  const int t = blockIdx.x;
  for (int c = threadIdx.x * 4; c < d_model; c += 256 * 4) {
    float4 s = make_float4(0, 0, 0, 0);
    for (int j = 0; j < k; j++) {
      const float4 v = *(const float4*)(o + (size_t)pos[t * k + j] * d_model + c);
      s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
    }
    if (o_s) {
      const float4 v = *(const float4*)(o_s + (size_t)t * d_model + c);
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

// bits = plane bits per code of the bank (4: 8/4 nest, 3: 6/3 nest, 2: 4/2 nest)
template <int MODE>
static void launch_gemm(const GemmArgs& g, int bits, int grid, hipStream_t st) {
  if (bits == 2) {
    if (g.sc_bf16) grouped_gemm_kernel<MODE, 1, 1><<<grid, PF_NT, 0, st>>>(g);
    else grouped_gemm_kernel<MODE, 0, 1><<<grid, PF_NT, 0, st>>>(g);
  } else if (bits == 3) {
    if (g.sc_bf16) grouped_gemm_kernel<MODE, 1, 2><<<grid, PF_NT, 0, st>>>(g);
    else grouped_gemm_kernel<MODE, 0, 2><<<grid, PF_NT, 0, st>>>(g);
  } else {
    if (g.sc_bf16) grouped_gemm_kernel<MODE, 1, 0><<<grid, PF_NT, 0, st>>>(g);
    else grouped_gemm_kernel<MODE, 0, 0><<<grid, PF_NT, 0, st>>>(g);
  }
}

struct PrefillLayout { size_t rows, pos, offsets, tiles, h, o, gamma, h_s, o_s, total; };

static inline int max_tiles(int T, int E, int k) { return E + (T * k) / PF_BM; }

static PrefillLayout prefill_layout(int T, int E, int k, int d_model, int d_ff, int shared_d_ff) {
  PrefillLayout L;
  size_t off = 0;
  L.rows = off;    off = up256(off + (size_t)T * k * 4);
  L.pos = off;     off = up256(off + (size_t)T * k * 4);
  L.offsets = off; off = up256(off + (size_t)(E + 1) * 4);
  L.tiles = off;   off = up256(off + (size_t)(4 + 4 * (max_tiles(T, E, k) + 8)) * 4);   // the grid rounds the tile count up to 8
  L.h = off;       off = up256(off + (size_t)T * k * d_ff * 2);
  L.o = off;       off = up256(off + (size_t)T * k * d_model * 4);
  L.gamma = L.h_s = L.o_s = off;
  if (shared_d_ff > 0) {       // one shared expert at a time: its H rows, and the running sum of their outputs
    L.gamma = off; off = up256(off + (size_t)T * 4);
    L.h_s = off;   off = up256(off + (size_t)T * shared_d_ff * 2);
    L.o_s = off;   off = up256(off + (size_t)T * d_model * 4);
  }
  L.total = off;
  return L;
}

extern "C" int smoe_prefill_bytes(int T, int E, int k, int d_model, int d_ff, int shared_d_ff, size_t* scratch_bytes) {
  if (!scratch_bytes) return SMOE_EINVAL;
  if (T <= 0 || E <= 0 || k <= 0 || k > E || d_model <= 0 || d_ff <= 0 || shared_d_ff < 0) return SMOE_ESHAPE;
  *scratch_bytes = prefill_layout(T, E, k, d_model, d_ff, shared_d_ff).total;
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
  if (shared_gate_w_dev && !shared) return SMOE_EINVAL;
  if (act_dtype != SMOE_BF16) return SMOE_ENOTIMPL;
  if (routed->device != ctx->device || (shared && shared->device != ctx->device)) return SMOE_EINVAL;
  const int E = routed->desc.n_experts, d = routed->desc.d_model, f = routed->desc.d_ff;
  if (T <= 0 || k <= 0 || k > E || k > SMOE_MAX_TOPK || E > SMOE_MAX_EXPERTS) return SMOE_ESHAPE;
  if (f % PF_BK || d % PF_BK || routed->desc.group < 32 || (routed->desc.group & (routed->desc.group - 1))) return SMOE_ESHAPE;
  if ((size_t)T * d >= 0x7FFFFFFFu || (size_t)T * k * f >= 0x7FFFFFFFu) return SMOE_ESHAPE;   // 32-bit element offsets
  const int f_s = shared ? shared->desc.d_ff : 0;
  if (shared) {
    const int gs = shared->desc.group;
    if (shared->desc.d_model != d || f_s % PF_BK || gs < 32 || (gs & (gs - 1))) return SMOE_ESHAPE;
    if ((size_t)T * f_s >= 0x7FFFFFFFu) return SMOE_ESHAPE;
  }
  if (!aligned16(x_dev) || !aligned16(y_dev) || !aligned16(idx_dev) || !aligned16(w_dev) || !aligned16(hist_dev) ||
      !aligned16(logits_dev) || !aligned16(w_router_dev) || !aligned16(shared_gate_w_dev) || (((uintptr_t)scratch_dev) & 255u))
    return SMOE_EALIGN;
  const PrefillLayout L = prefill_layout(T, E, k, d, f, f_s);
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
  g.sc_bf16 = routed->dev.sc_bf16; g.group_shift = __builtin_ctz((unsigned)routed->dev.group); g.offsets = offsets; g.tiles = tiles; g.rows = rows;
  g.x = (const uint16_t*)x_dev; g.h = h; g.o = o; g.wgt = w_dev; g.k = k; g.d_model = d; g.d_ff = f;
  const int mt = max_tiles(T, E, k);             // upper bound of the tile count; surplus work-groups return at once
  const int mt8 = (mt + 7) / 8 * 8;
  g.w = routed->dev.gu; g.n_col_tiles = (2 * f + PF_BN - 1) / PF_BN;
  launch_gemm<0>(g, routed->dev.bits, mt8 * g.n_col_tiles, st);
  g.w = routed->dev.dn; g.n_col_tiles = (d + PF_BN - 1) / PF_BN;
  launch_gemm<1>(g, routed->dev.bits, mt8 * g.n_col_tiles, st);
  float* o_s = nullptr;
  if (shared) {
    // the shared experts see every token: dense GEMMs over the token rows in their own order, one
    // expert after the other into one H buffer, their gate-weighted outputs summed in O_s
    float* gamma = (float*)(s + L.gamma);
    o_s = (float*)(s + L.o_s);
    shared_gate_kernel<<<(T + 3) / 4, 256, 0, st>>>((const uint16_t*)x_dev, (const uint16_t*)shared_gate_w_dev, T, d, gamma);
    GemmArgs q{};
    q.sc_bf16 = shared->dev.sc_bf16; q.group_shift = __builtin_ctz((unsigned)shared->dev.group);
    q.x = (const uint16_t*)x_dev; q.h = (uint16_t*)(s + L.h_s); q.o = o_s; q.wgt = gamma; q.k = 1; q.d_model = d; q.d_ff = f_s;
    q.dense_rows = T;
    const int nt8 = ((T + PF_BM - 1) / PF_BM + 7) / 8 * 8;
    for (int e = 0; e < shared->desc.n_experts; e++) {
      q.dense_expert = e; q.accumulate = e > 0;
      q.w = shared->dev.gu; q.n_col_tiles = (2 * f_s + PF_BN - 1) / PF_BN;
      launch_gemm<0>(q, shared->dev.bits, nt8 * q.n_col_tiles, st);
      q.w = shared->dev.dn; q.n_col_tiles = (d + PF_BN - 1) / PF_BN;
      launch_gemm<1>(q, shared->dev.bits, nt8 * q.n_col_tiles, st);
    }
  }
  combine_kernel<<<T, 256, 0, st>>>(o, pos, o_s, (const uint16_t*)x_dev, (uint16_t*)y_dev, k, d, add_residual);
  HIPCHK(ctx, hipGetLastError());
  return SMOE_OK;
}
