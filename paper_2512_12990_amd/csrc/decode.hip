// Decode-time expert FFN over bit-sliced weights (paper Section 4.1: full precision when both
// slices of an expert are resident, MSB-only otherwise; Section 4.2: the MSB nibble with the
// truncated zero-point IS the low-bit model; Section 2.1: cache-aware top-k in the prologue).
//
// Two launches per token-layer, both HBM-streaming kernels of 512-thread (8-wave) work-groups, two of
// which share a CU:
//   gateup  h = silu(Wg x) * (Wu x) for every slot.  Work-group b takes the row pairs
//           r = b' + n_wg*q of EVERY slot (b' rotated per slot), so all work-groups move the same
//           bytes whatever the precision mix, and nothing about the split depends on routing:
//           loads of the shared experts are in flight while the last wave routes the token.
//   down    y = sum_slots weight * Wd h (+ x): a work-group owns 8 output rows, each wave takes the
//           rows of one (slot, k-slice) piece; partial sums meet in LDS in a fixed order.
// A wave issues at most one instruction every four cycles, so the instruction count of the
// longest wave bounds a kernel from below as surely as the bytes do: the code is flat, and what
// can be worked out once per piece or on the host is.
// A lane always handles one 32-column chunk = 16 bytes of a nibble plane (one 128-bit load) and
// a wave issues all loads of a batch before it touches the first result.  Loads go through buffer
// resources: wave-uniform row offsets in scalar registers, the per-lane part is lane*16, and a
// lane or load with nothing to read is sent out of range (returns 0, moves no bytes), so the
// issue code has no branches.
// The inner product is integer:
// with bf16 activations each 32-value chunk of x (or h) is rewritten once, in LDS, as integers
// |q| <= 1911 times a power-of-two chunk scale, in three balanced hex digits (q = 256 d2 + 16 d1
// + d0, d in [-8, 7]).  The planes store every nibble n as n - 8, so one signed 8 x 4-bit dot
// instruction per plane word and digit does the work, with nothing to unpack.  All sums are exact
// int32; with m' = m - 8, l' = l - 8, X = sum q, sx the chunk scale:
//   HIGH  (s sx) * (16 m'.q + l'.q + (136 - zp) X)      LOW  (16 s sx) * (m'.q + (8 - (zp >> 4)) X)
// fp32 activations take a plain fp32 path (byte -> float conversions and FMAs).
#include "route_device.hpp"
#include "fastdiv.hpp"
#include <hip/hip_ext.h>
#include <vector>
#include <mutex>

#define DEC_NT 512                  // threads per work-group
#define DEC_NW (DEC_NT / 64)
#define DEC_MAXP 3                  // row pairs per batch and wave (gate/up kernel)
#define DEC_RPW 8                   // output rows per work-group (down kernel)

// One expert matrix family as the kernels see it (56 bytes).
struct MatK {
  const uint8_t* msb; const uint8_t* lsb; const uint8_t* zp; const uint8_t* sc;
  unsigned ps32, zs32, ss32;       // bytes per expert in the plane / zero-point / scale sections
  int ng, sng;                     // quantisation groups per row; scales stored per row (ng rounded up to even)
  int pad0;
};

// Kernel arguments, kept compact and ordered by use: a dispatch's arguments are cold in every
// cache, each 64-byte line of them costs a memory round trip when first touched, and the kernels
// therefore fetch all their lines at once in their first instructions (KARGS_FETCH).
struct DecodeArgs {
  MatK rgu, sgu;                   // gate/up families of the routed / shared bank        [gate/up kernel]
  const int32_t* idx_in; const float* w_in;
  const void* shared_gate_w;
  int32_t* idx_out; float* w_out; uint8_t* prec_out;
  float routed_scale, tau;
  int norm_topk;
  int cap_r, cap_s;                // gate/up: row pairs per work-group and slot = ceil(f / n_wg)
  uint32_t inv_cap_r, inv_cap_s;   // fastdiv_magic(cap): slot of entry e = fastdiv(e, inv_cap)
  int rot;                         // gate/up: per-slot rotation of the work-group index
  int gu_L;                        // gate/up: entries per wave
  int gu_sh_r, gu_sh_s;            // log2(32-column chunks per quantisation group), gate/up families
  int n_shared;                    // experts in the shared bank                          [both kernels]
  const void* x;
  RouteRec* rec;                   // routing record (gate/up block 0 writes, down reads)
  float* h;                        // SwiGLU vectors: shared experts first, then the routed slots, fp32
  int E, k;                        // experts in the routed bank, routed slots (0 without a routed bank)
  int f_r, f_s;                    // d_ff of the routed / shared bank (0 if absent)
  void* y;                         //                                                     [down kernel]
  MatK rdn, sdn;                   // down families
  int ks_r, ks_s, inv_ks_r, inv_ks_s;   // down: 64-chunk k-slices per row, fastdiv_magic(ks)
  int dn_sh_r, dn_sh_s;
  int add_residual;
  int d_model;                     // host side only (the kernels get it as a leading parameter)
};

// The routing inputs and the few numbers a wave needs for its first loads are not in this struct:
// they are the kernels' leading scalar parameters (RouteIn; rec, h, unit shares), which the
// hardware hands to a wave in registers at launch (kernel-argument preload), so those loads are
// issued in the first instructions without waiting for a kernel-argument fetch.
struct RouteIn {
  const float* logits; const float* bias; const uint8_t* mask;   // [E] each; bias / mask may be null
  int E, k, do_route;              // do_route 0: idx_in / w_in of DecodeArgs hold the decision
};

// Kernel-argument fetch: KARGS_FETCH issues one scalar load per 64-byte line of the argument
// segment (eight lines) and waits for them; afterwards the compiler's own argument loads hit the
// scalar cache.  It stands behind the first vector loads of a kernel (which need only the leading
// parameters), so the argument lines and those loads are in flight together.  Issue and wait are one
// statement on purpose: the destination registers hold dead values, and between two statements the
// compiler is free to give them to live values, which a load still in flight then overwrites.
#define KARG_OFF(i, size) ((i) * 64 < (size) ? (i) * 64 : (size) - 4)      /* never past the last argument */
#define KARGS_FETCH(size)                                                                                                 \
  do {                                                                                                                    \
    unsigned kt0_, kt1_, kt2_, kt3_, kt4_, kt5_, kt6_;                                                                    \
    asm volatile("s_load_dword %0, %7, %8\n\ts_load_dword %1, %7, %9\n\ts_load_dword %2, %7, %10\n\t"                  \
                 "s_load_dword %3, %7, %11\n\ts_load_dword %4, %7, %12\n\ts_load_dword %5, %7, %13\n\t"                \
                 "s_load_dword %6, %7, %14\n\ts_waitcnt lgkmcnt(0)"                                                       \
                 : "=&s"(kt0_), "=&s"(kt1_), "=&s"(kt2_), "=&s"(kt3_), "=&s"(kt4_), "=&s"(kt5_), "=&s"(kt6_)              \
                 : "s"(__builtin_amdgcn_kernarg_segment_ptr()), "n"(KARG_OFF(1, size)), "n"(KARG_OFF(2, size)),           \
                   "n"(KARG_OFF(3, size)), "n"(KARG_OFF(4, size)), "n"(KARG_OFF(5, size)), "n"(KARG_OFF(6, size)),        \
                   "n"(KARG_OFF(7, size))                                                                                 \
                 : "memory");                                                                                             \
  } while (0)
/* floats between the h vectors of consecutive tokens of a multi-token launch (both kernels must
 * know it from their leading parameters: room for the largest top-k) */
#define DEC_H_STRIDE(nsf, f_r) ((nsf) + SMOE_MAX_TOPK * (f_r))
#define DEC_LEAD_BYTES 56      /* both kernels have 56 bytes of leading parameters before the struct */
static_assert(sizeof(DecodeArgs) + DEC_LEAD_BYTES <= 8 * 64, "KARGS_FETCH covers eight lines");

__device__ __forceinline__ void lds_barrier() {
  // orders LDS traffic only; outstanding global loads stay in flight across it
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

__device__ __forceinline__ int uni(int v) { return __builtin_amdgcn_readfirstlane(v); }

template <int CTRL, int ROWM, int BANKM> __device__ __forceinline__ float dpp_add(float v) {
  return v + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, ROWM, BANKM, true));
}
// Sum over the wave; the total is valid in lane 63 only.  Every lane must take part.
__device__ __forceinline__ float wave_sum_to63(float v) {
  v = dpp_add<0xB1, 0xF, 0xF>(v);      // quad_perm [1,0,3,2]
  v = dpp_add<0x4E, 0xF, 0xF>(v);      // quad_perm [2,3,0,1]: every lane holds its quad's sum
  // all lanes enabled from here on (the result is only read from the lanes named; with no lane
  // masked each step is a single add with a lane-shifted operand)
  v = dpp_add<0x114, 0xF, 0xF>(v);     // row_shr 4
  v = dpp_add<0x118, 0xF, 0xF>(v);     // row_shr 8: lanes 12..15 hold the row sum
  v = dpp_add<0x142, 0xF, 0xF>(v);     // row_bcast 15: lane 15 of a row into the next row; lanes 31 / 63: rows 0+1 / 2+3
  v = dpp_add<0x143, 0xF, 0xF>(v);     // row_bcast 31: lane 31 into rows 2 and 3
  return v;
}
template <int CTRL> __device__ __forceinline__ int quad_xchg(int v) {
  return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xF, 0xF, true);
}

// ---------------------------------------------------------------------------------- buffer addressing
// Every bank section is read through a buffer resource: address = section base + a wave-uniform
// byte offset (scalar register) + a small per-lane offset.  A lane (or a whole load) that has
// nothing to read gets the per-lane offset DEC_OOB, which the hardware range check turns into
// "return 0, touch no memory".  So every load below is unconditional, the issue code is straight
// line, and the compiler can count outstanding loads exactly (partial s_waitcnt instead of
// waiting for everything).  A zero scale makes a lane's contribution exactly 0.
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2_t __attribute__((ext_vector_type(2)));
#define DEC_OOB 0x80000000u

struct SecRsrc { __amdgpu_buffer_rsrc_t msb, lsb, zp, sc; };

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* base, unsigned bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)bytes, 0x00020000);
}
__device__ __forceinline__ SecRsrc make_sec(const MatK& m, int n_experts) {
  SecRsrc r;
  r.msb = make_rsrc(m.msb, (unsigned)n_experts * m.ps32);
  r.lsb = make_rsrc(m.lsb, (unsigned)n_experts * m.ps32);
  r.zp = make_rsrc(m.zp, (unsigned)n_experts * m.zs32);
  r.sc = make_rsrc(m.sc, (unsigned)n_experts * m.ss32);
  return r;
}
__device__ __forceinline__ uint4 bload128(__amdgpu_buffer_rsrc_t r, unsigned voff, unsigned soff) {
  const u32x4_t v = __builtin_amdgcn_raw_buffer_load_b128(r, (int)voff, (int)soff, 0);
  return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ uint2 bload64(__amdgpu_buffer_rsrc_t r, unsigned voff, unsigned soff) {
  const u32x2_t v = __builtin_amdgcn_raw_buffer_load_b64(r, (int)voff, (int)soff, 0);
  return make_uint2(v.x, v.y);
}
// A lane's 32 codes of one plane as loaded.  FMT 0: 8/4 nest, nibble planes (16 bytes, every nibble n
// stored as n ^ 8); FMT 1: 4/2 nest, 2-bit planes (8 bytes, column c of a word in bits 2c, 2c+1);
// FMT 2: 6/3 nest, 3-bit planes (12 bytes: two words of 2-bit fields and one word of third bits).
template <int FMT> struct PlaneT { typedef uint4 t; enum { BYTES = 16 }; };
template <> struct PlaneT<1> { typedef uint2 t; enum { BYTES = 8 }; };
template <> struct PlaneT<2> { typedef uint3 t; enum { BYTES = 12 }; };
template <int FMT> __device__ __forceinline__ typename PlaneT<FMT>::t pload(__amdgpu_buffer_rsrc_t r, unsigned voff, unsigned soff);
// The same load at device scope (sc1): it returns what other compute dies have written through, whatever
// this die's L2 holds.  Marked volatile for the compiler (bit 31 of the cache-policy operand): a poll
// loop must issue it anew every time round.
__device__ __forceinline__ uint4 bload128_dev(__amdgpu_buffer_rsrc_t r, unsigned voff, unsigned soff) {
  const u32x4_t v = __builtin_amdgcn_raw_buffer_load_b128(r, (int)voff, (int)soff, (int)(16u | 0x80000000u));
  return make_uint4(v.x, v.y, v.z, v.w);
}
template <> __device__ __forceinline__ uint4 pload<0>(__amdgpu_buffer_rsrc_t r, unsigned voff, unsigned soff) { return bload128(r, voff, soff); }
template <> __device__ __forceinline__ uint2 pload<1>(__amdgpu_buffer_rsrc_t r, unsigned voff, unsigned soff) { return bload64(r, voff, soff); }
template <> __device__ __forceinline__ uint3 pload<2>(__amdgpu_buffer_rsrc_t r, unsigned voff, unsigned soff) {
  typedef unsigned int u32x3_t __attribute__((ext_vector_type(3)));
  const u32x3_t v = __builtin_amdgcn_raw_buffer_load_b96(r, (int)voff, (int)soff, 0);
  return make_uint3(v.x, v.y, v.z);
}
__device__ __forceinline__ uint32_t bload32(__amdgpu_buffer_rsrc_t r, unsigned voff, unsigned soff) {
  return __builtin_amdgcn_raw_buffer_load_b32(r, (int)voff, (int)soff, 0);
}
__device__ __forceinline__ uint32_t bload8(__amdgpu_buffer_rsrc_t r, unsigned voff, unsigned soff) {
  return __builtin_amdgcn_raw_buffer_load_b8(r, (int)voff, (int)soff, 0);
}

// Value of a scale fetched as the aligned dword that contains it; `odd` tells which half holds a 16-bit scale.
template <int SCB> __device__ __forceinline__ float scale_val(uint32_t raw, int odd) {
  return SCB ? __uint_as_float(odd ? (raw & 0xFFFF0000u) : (raw << 16)) : __uint_as_float(raw);
}

// ---------------------------------------------------------------------------------- lane operands
// The lane's 32 activations.
//   BF16: the chunk as integers q = 256 d2 + 16 d1 + d0 with balanced digits d in [-8, 7] times a
//         power-of-two chunk scale sx; p[4 d + j] = digit d of columns 8j .. 8j+7, one 4-bit two's
//         complement value each, in the nibble order of a plane word; xs = sum of the chunk's q.
//   F32 : plain values and their sum.
template <int ACT> struct XR;
template <> struct XR<SMOE_BF16> { uint32_t p[12]; float sx; int xs; };
template <> struct XR<SMOE_F32> { float v[32]; float xs; };

// acc[t] += sum over the chunk of (plane nibble - 8) * digit t
__device__ __forceinline__ void dot_plane_i4(const uint4& m, const XR<SMOE_BF16>& x, int& a0, int& a1, int& a2) {
  const uint32_t w[4] = {m.x, m.y, m.z, m.w};
#pragma unroll
  for (int j = 0; j < 4; j++) {
    a0 = __builtin_amdgcn_sdot8((int)w[j], (int)x.p[j], a0, false);
    a1 = __builtin_amdgcn_sdot8((int)w[j], (int)x.p[4 + j], a1, false);
    a2 = __builtin_amdgcn_sdot8((int)w[j], (int)x.p[8 + j], a2, false);
  }
}

// With m' = m - 8 and l' = l - 8 the stored nibbles:
//   HIGH: s (16 m + l - zp) x = s sx (16 m'.q + l'.q + (136 - zp) sum q)
//   LOW : 16 s (m - (zp >> 4)) x = 16 s sx (m'.q + (8 - (zp >> 4)) sum q)
__device__ __forceinline__ float lane_value(const XR<SMOE_BF16>& x, const uint4& m, const uint4& l, int high, int zp,
                                            float s) {
  int p0 = 0, p1 = 0, p2 = 0;
  if (high) {
    int p3 = 0;
    dot_plane_i4(l, x, p0, p1, p2);      // powers 16^0..16^2
    dot_plane_i4(m, x, p1, p2, p3);      // powers 16^1..16^3
    const int t = ((((((p3 << 4) + p2) << 4) + p1) << 4) + p0) + __mul24(136 - zp, x.xs);      // |xs| < 2^17
    return (s * x.sx) * (float)t;
  }
  dot_plane_i4(m, x, p0, p1, p2);
  const int t = ((((p2 << 4) + p1) << 4) + p0) + __mul24(8 - (zp >> 4), x.xs);
  return (16.0f * s * x.sx) * (float)t;
}

// 2-bit planes: the sixteen 2-bit codes of half a plane word, one per nibble (values 0..3)
__device__ __forceinline__ uint32_t spread2(uint32_t h) {
  h = (h | (h << 8)) & 0x00FF00FFu;
  h = (h | (h << 4)) & 0x0F0F0F0Fu;
  return (h | (h << 2)) & 0x33333333u;
}
__device__ __forceinline__ uint4 nibbles_of(const uint2& p) {
  return make_uint4(spread2(p.x & 0xFFFFu), spread2(p.x >> 16), spread2(p.y & 0xFFFFu), spread2(p.y >> 16));
}
// 4/2 nest, codes as plain nibbles 0..3 (no offset):
//   HIGH: s (4 m + l - zp) x = s sx (4 m.q + l.q - zp sum q)
//   LOW : 4 s (m - (zp >> 2)) x = 4 s sx (m.q - (zp >> 2) sum q)
__device__ __forceinline__ float lane_value(const XR<SMOE_BF16>& x, const uint2& m2, const uint2& l2, int high, int zp,
                                            float s) {
  int m0 = 0, m1 = 0, mm2 = 0;
  dot_plane_i4(nibbles_of(m2), x, m0, m1, mm2);
  const int tm = (((mm2 << 4) + m1) << 4) + m0;
  if (high) {
    int l0 = 0, l1 = 0, ll2 = 0;
    dot_plane_i4(nibbles_of(l2), x, l0, l1, ll2);
    const int tl = (((ll2 << 4) + l1) << 4) + l0;
    return (s * x.sx) * (float)(4 * tm + tl - __mul24(zp, x.xs));
  }
  return (4.0f * s * x.sx) * (float)(tm - __mul24(zp >> 2, x.xs));
}
__device__ __forceinline__ float lane_value(const XR<SMOE_F32>& x, const uint2& m2, const uint2& l2, int high, int zp,
                                            float s) {
  const uint32_t wm[2] = {m2.x, m2.y}, wl[2] = {l2.x, l2.y};
  float a0 = 0.0f, a1 = 0.0f;
#pragma unroll
  for (int j = 0; j < 2; j++)
#pragma unroll
    for (int c = 0; c < 16; c += 2) {
      const uint32_t q0 = high ? (((wm[j] >> (2 * c)) & 3u) << 2) | ((wl[j] >> (2 * c)) & 3u) : (wm[j] >> (2 * c)) & 3u;
      const uint32_t q1 = high ? (((wm[j] >> (2 * c + 2)) & 3u) << 2) | ((wl[j] >> (2 * c + 2)) & 3u) : (wm[j] >> (2 * c + 2)) & 3u;
      a0 = fmaf((float)q0, x.v[16 * j + c], a0);
      a1 = fmaf((float)q1, x.v[16 * j + c + 1], a1);
    }
  if (high) return s * fmaf(-(float)zp, x.xs, a0 + a1);
  return (4.0f * s) * fmaf(-(float)(zp >> 2), x.xs, a0 + a1);
}

// 3-bit planes: word t of the result holds the values of columns 8t .. 8t+7, one per nibble (0..7).
// Column 8t + j keeps its two low bits in word t >> 1 of the plane at bits 4j + 2(t & 1) and its
// third bit in word 2 at bit 4j + t, so every nibble word is two shifts, two masks and an or.
__device__ __forceinline__ uint4 nibbles_of(const uint3& p) {
  return make_uint4((p.x & 0x33333333u) | ((p.z & 0x11111111u) << 2), ((p.x >> 2) & 0x33333333u) | ((p.z & 0x22222222u) << 1),
                    (p.y & 0x33333333u) | (p.z & 0x44444444u), ((p.y >> 2) & 0x33333333u) | ((p.z & 0x88888888u) >> 1));
}
// 6/3 nest, codes as plain nibbles 0..7 (no offset):
//   HIGH: s (8 m + l - zp) x = s sx (8 m.q + l.q - zp sum q)
//   LOW : 8 s (m - (zp >> 3)) x = 8 s sx (m.q - (zp >> 3) sum q)
__device__ __forceinline__ float lane_value(const XR<SMOE_BF16>& x, const uint3& m3, const uint3& l3, int high, int zp,
                                            float s) {
  int m0 = 0, m1 = 0, mm2 = 0;
  dot_plane_i4(nibbles_of(m3), x, m0, m1, mm2);
  const int tm = (((mm2 << 4) + m1) << 4) + m0;
  if (high) {
    int l0 = 0, l1 = 0, ll2 = 0;
    dot_plane_i4(nibbles_of(l3), x, l0, l1, ll2);
    const int tl = (((ll2 << 4) + l1) << 4) + l0;
    return (s * x.sx) * (float)(8 * tm + tl - __mul24(zp, x.xs));
  }
  return (8.0f * s * x.sx) * (float)(tm - __mul24(zp >> 3, x.xs));
}

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

__device__ __forceinline__ float lane_value(const XR<SMOE_F32>& x, const uint4& m, const uint4& l, int high, int zp,
                                            float s) {
  const uint32_t f = 0x88888888u;      // the planes hold n ^ 8 per nibble
  const uint32_t wm[4] = {m.x ^ f, m.y ^ f, m.z ^ f, m.w ^ f}, wl[4] = {l.x ^ f, l.y ^ f, l.z ^ f, l.w ^ f};
  float a0 = 0.0f, a1 = 0.0f;
  if (high) {
#pragma unroll
    for (int j = 0; j < 4; j++) {
      const uint32_t qe = ((wm[j] & 0x0F0F0F0Fu) << 4) | (wl[j] & 0x0F0F0F0Fu);     // codes of even columns
      const uint32_t qo = (wm[j] & 0xF0F0F0F0u) | ((wl[j] >> 4) & 0x0F0F0F0Fu);    // codes of odd columns
      a0 = dot_bytes(qe, qo, x.v + 8 * j, a0, a1);
    }
    return s * fmaf(-(float)zp, x.xs, a0 + a1);
  }
#pragma unroll
  for (int j = 0; j < 4; j++) a0 = dot_bytes(wm[j] & 0x0F0F0F0Fu, (wm[j] >> 4) & 0x0F0F0F0Fu, x.v + 8 * j, a0, a1);
  return (16.0f * s) * fmaf(-(float)(zp >> 4), x.xs, a0 + a1);
}

__device__ __forceinline__ float lane_value(const XR<SMOE_F32>& x, const uint3& m3, const uint3& l3, int high, int zp,
                                            float s) {
  const uint4 nm = nibbles_of(m3), nl = nibbles_of(l3);
  const uint32_t wm[4] = {nm.x, nm.y, nm.z, nm.w}, wl[4] = {nl.x, nl.y, nl.z, nl.w};
  float a0 = 0.0f, a1 = 0.0f;
  if (high) {
#pragma unroll
    for (int j = 0; j < 4; j++) {
      const uint32_t qe = ((wm[j] & 0x0F0F0F0Fu) << 3) | (wl[j] & 0x0F0F0F0Fu);              // codes of even columns
      const uint32_t qo = (((wm[j] >> 4) & 0x0F0F0F0Fu) << 3) | ((wl[j] >> 4) & 0x0F0F0F0Fu);   // codes of odd columns
      a0 = dot_bytes(qe, qo, x.v + 8 * j, a0, a1);
    }
    return s * fmaf(-(float)zp, x.xs, a0 + a1);
  }
#pragma unroll
  for (int j = 0; j < 4; j++) a0 = dot_bytes(wm[j] & 0x0F0F0F0Fu, (wm[j] >> 4) & 0x0F0F0F0Fu, x.v + 8 * j, a0, a1);
  return (8.0f * s) * fmaf(-(float)(zp >> 3), x.xs, a0 + a1);
}

// ---------------------------------------------------------------------------------- LDS staging
// A vector of n = 32*C values is kept in LDS per 64-chunk k-slice as [piece][chunk][16 bytes] so
// that the lanes of a wave read consecutive 16-byte pieces.  BF16: 3 pieces per chunk (the digit
// words of XR; 64 B per chunk are reserved), F32: 8 pieces of 4 floats (128 B).  cs[c] = (chunk scale, chunk sum).
template <int ACT> struct StageTraits;
template <> struct StageTraits<SMOE_BF16> { enum { BYTES_PER_VAL = 2, COMBO_BYTES = 64 * 48 }; };     // one 64-chunk k-slice
template <> struct StageTraits<SMOE_F32> { enum { BYTES_PER_VAL = 4, COMBO_BYTES = 64 * 128 }; };

// Eight consecutive values as loaded (no arithmetic on them, so nothing waits for the load).
struct Raw8 { uint4 a, b; };
template <int SRC> __device__ __forceinline__ void load8_raw(const void* src, size_t i0, Raw8& r) {
  if (SRC == SMOE_F32) {
    r.a = *(const uint4*)((const float*)src + i0);
    r.b = *(const uint4*)((const float*)src + i0 + 4);
  } else {
    r.a = *(const uint4*)((const uint16_t*)src + i0);
  }
}
template <int SRC> __device__ __forceinline__ void unpack8(const Raw8& r, float* v) {
  if (SRC == SMOE_F32) {
    v[0] = __uint_as_float(r.a.x); v[1] = __uint_as_float(r.a.y); v[2] = __uint_as_float(r.a.z); v[3] = __uint_as_float(r.a.w);
    v[4] = __uint_as_float(r.b.x); v[5] = __uint_as_float(r.b.y); v[6] = __uint_as_float(r.b.z); v[7] = __uint_as_float(r.b.w);
  } else {
    const uint32_t w[4] = {r.a.x, r.a.y, r.a.z, r.a.w};
#pragma unroll
    for (int i = 0; i < 4; i++) { v[2 * i] = bf16_bits_to_f32(w[i] & 0xFFFF); v[2 * i + 1] = bf16_bits_to_f32(w[i] >> 16); }
  }
}

// Stages the 8 values v[0..8) = word j of chunk c of a vector with C chunks into dst (byte
// address of that vector inside LDS) and its chunk figures into cs[c].  The four words of a chunk
// must be handled by the four lanes of one quad in the same call.
template <int ACT>
__device__ __forceinline__ void stage_regs(float* v, int C, int c, int j, uint8_t* dst, float2* cs) {
  const int ks = c >> 6, cw = min(64, C - ks * 64), cl = c & 63;
  if (ACT == SMOE_BF16) {
    float amax = 0.0f;
#pragma unroll
    for (int i = 0; i < 8; i++) amax = fmaxf(amax, fabsf(v[i]));
    amax = fmaxf(amax, __int_as_float(quad_xchg<0xB1>(__float_as_int(amax))));
    amax = fmaxf(amax, __int_as_float(quad_xchg<0x4E>(__float_as_int(amax))));
    // chunk scale 2^(e-10), e = exponent of the largest magnitude, or 2^(e-9) when that would exceed
    // 1911 = 7 * 273, the largest integer three balanced hex digits hold
    int be = (int)(__float_as_uint(amax) >> 23);
    const bool live = be >= 20 && be < 255;
    if (amax * __uint_as_float((uint32_t)(264 - (live ? be : 127)) << 23) >= 1911.5f) be += 1;
    const float inv = live ? __uint_as_float((uint32_t)(264 - be) << 23) : 0.0f;
    const float sx = live ? __uint_as_float((uint32_t)(be - 10) << 23) : 0.0f;
    // u = q + 0x888 with q = rne(v * inv): one fused multiply-add onto 1.5 * 2^23 + 0x888 leaves u in
    // the low 12 bits (and zeros in bits 12..21).  Nibble d of u ^ 0x888 is digit d in two's
    // complement.  The 8 x 3 nibbles are regrouped by digit with byte permutes: two values per
    // register, then the nibbles of neighbouring values merged into bytes.
    uint32_t t[8];
#pragma unroll
    for (int i = 0; i < 8; i++) t[i] = __float_as_uint(fmaf(v[i], inv, 12585096.0f));
    uint32_t r[2], y[2];
#pragma unroll
    for (int h = 0; h < 2; h++) {
      const uint32_t pa = __builtin_amdgcn_perm(t[4 * h + 2], t[4 * h], 0x05040100u);       // values 0 and 2 of this half
      const uint32_t pb = __builtin_amdgcn_perm(t[4 * h + 3], t[4 * h + 1], 0x05040100u);   // values 1 and 3
      r[h] = ((pb & 0x0F0F0F0Fu) << 4) | (pa & 0x0F0F0F0Fu);      // bytes: d0 of (0,1), d2 of (0,1), d0 of (2,3), d2 of (2,3)
      y[h] = ((pa >> 4) & 0x000F000Fu) | (pb & 0x00F000F0u);      // bytes: d1 of (0,1), 0, d1 of (2,3), 0
    }
    const uint32_t w0 = __builtin_amdgcn_perm(r[1], r[0], 0x06040200u) ^ 0x88888888u;
    const uint32_t w2 = __builtin_amdgcn_perm(r[1], r[0], 0x07050301u) ^ 0x88888888u;
    const uint32_t w1 = __builtin_amdgcn_perm(y[1], y[0], 0x06040200u) ^ 0x88888888u;
    // sum of the eight q from the digit sums
    int part = __builtin_amdgcn_sdot8((int)w0, 0x11111111, 0, false) + 16 * __builtin_amdgcn_sdot8((int)w1, 0x11111111, 0, false) +
               256 * __builtin_amdgcn_sdot8((int)w2, 0x11111111, 0, false);
    part += quad_xchg<0xB1>(part);
    part += quad_xchg<0x4E>(part);
    uint8_t* base = dst + (size_t)ks * 4096 + (size_t)j * 4;
    *(uint32_t*)(base + (size_t)cl * 16) = w0;
    *(uint32_t*)(base + (size_t)(cw + cl) * 16) = w1;
    *(uint32_t*)(base + (size_t)(2 * cw + cl) * 16) = w2;
    if (j == 0) cs[c] = make_float2(sx, __int_as_float(part));
  } else {
    float part = 0.0f;
#pragma unroll
    for (int i = 0; i < 8; i++) part += v[i];
    uint8_t* base = dst + (size_t)ks * 8192;
    *(float4*)(base + (size_t)((2 * j) * cw + cl) * 16) = make_float4(v[0], v[1], v[2], v[3]);
    *(float4*)(base + (size_t)((2 * j + 1) * cw + cl) * 16) = make_float4(v[4], v[5], v[6], v[7]);
    part += __int_as_float(quad_xchg<0xB1>(__float_as_int(part)));
    part += __int_as_float(quad_xchg<0x4E>(__float_as_int(part)));
    if (j == 0) cs[c] = make_float2(1.0f, part);
  }
}

template <int ACT>
__device__ __forceinline__ void load_xr(XR<ACT>& x, const uint8_t* vec, const float2* cs, int ks, int cw, int lane) {
  const float2 c = cs[ks * 64 + lane];
  if (ACT == SMOE_BF16) {
    const uint4* b = (const uint4*)(vec + (size_t)ks * 4096);
    XR<SMOE_BF16>& xb = *(XR<SMOE_BF16>*)&x;
#pragma unroll
    for (int j = 0; j < 3; j++) {
      const uint4 q = b[j * cw + lane];
      xb.p[4 * j] = q.x; xb.p[4 * j + 1] = q.y; xb.p[4 * j + 2] = q.z; xb.p[4 * j + 3] = q.w;
    }
    xb.sx = c.x; xb.xs = __float_as_int(c.y);
  } else {
    const float4* b = (const float4*)(vec + (size_t)ks * 8192);
    XR<SMOE_F32>& xf = *(XR<SMOE_F32>*)&x;
#pragma unroll
    for (int j = 0; j < 8; j++) {
      const float4 q = b[j * cw + lane];
      xf.v[4 * j] = q.x; xf.v[4 * j + 1] = q.y; xf.v[4 * j + 2] = q.z; xf.v[4 * j + 3] = q.w;
    }
    xf.xs = c.y;
  }
}

// ---------------------------------------------------------------------------------- routing by one wave
template <int CTRL, int ROWM, int BANKM> __device__ __forceinline__ uint32_t dpp_umax(uint32_t v) {
  const uint32_t t = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, ROWM, BANKM, true);
  return t > v ? t : v;
}
// Unsigned maximum over the wave, returned in every lane.
__device__ __forceinline__ uint32_t wave_umax(uint32_t v) {
  v = dpp_umax<0xB1, 0xF, 0xF>(v);
  v = dpp_umax<0x4E, 0xF, 0xF>(v);
  v = dpp_umax<0x114, 0xF, 0xE>(v);
  v = dpp_umax<0x118, 0xF, 0xC>(v);
  v = dpp_umax<0x142, 0xA, 0xF>(v);
  v = dpp_umax<0x143, 0xC, 0xF>(v);
  return (uint32_t)__builtin_amdgcn_readlane((int)v, 63);
}
__device__ __forceinline__ float wave_sum_all(float v) {
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(wave_sum_to63(v)), 63));
}
__device__ __forceinline__ float unorderable(uint32_t o) {
  return __uint_as_float((o & 0x80000000u) ? (o ^ 0x80000000u) : ~o);
}

// Same decision rule as select_topk_wave (route_device.hpp) -- k largest biased scores, ties to the
// lower expert index, weights from the softmax of the unbiased logits -- executed by a single
// wave with cross-lane DPP reductions only.  Lane e (+64j) holds logit, bias and slice mask of
// expert e; the loads are issued by route_load so that they overlap other work.
struct RouteRegs { float z[4]; float b[4]; int mk[4]; };

// Unconditional loads: an absent input is a buffer of zero records, which reads as 0, and a wave
// that does not route (`on` false) reads out of range.  No branch, so no value has to be complete
// where control flow merges: the byte -> int conversions wait where the values are first used.
__device__ __forceinline__ void route_load(const RouteIn& in, int lane, RouteRegs& r, bool on) {
  const unsigned E = (unsigned)in.E;
  const __amdgpu_buffer_rsrc_t rz = make_rsrc(in.logits, in.do_route ? E * 4u : 0u);
  const __amdgpu_buffer_rsrc_t rb = make_rsrc(in.bias, (in.do_route && in.bias) ? E * 4u : 0u);
  const __amdgpu_buffer_rsrc_t rm = make_rsrc(in.mask, in.mask ? E : 0u);      // (also read when the decision is given)
#pragma unroll
  for (int j = 0; j < 4; j++) {
    const unsigned e = (unsigned)(lane + 64 * j);
    r.z[j] = __uint_as_float(bload32(rz, on ? e * 4u : DEC_OOB, 0));
    r.b[j] = __uint_as_float(bload32(rb, on ? e * 4u : DEC_OOB, 0));
    r.mk[j] = (int)bload8(rm, on ? e : DEC_OOB, 0);
  }
}

// Lane r < k gets slot r: expert (mysel), slice-mask bits of that expert (mymask) and, with WEIGHTS,
// the gate weight (myw).  NJ = experts per lane.  The selection alone is what the row loads of the
// gate/up kernel wait for; the softmax is left out where nothing needs the weights.
template <int NJ, bool WEIGHTS>
__device__ __forceinline__ void route_topk(const RouteIn& in, const DecodeArgs& a, int lane, const RouteRegs& rr, int& mysel,
                                           int& mymask, float& myw) {
  const int E = in.E, k = in.k;
  uint32_t ord[NJ];              // orderable biased score; 0 = absent or already taken
  float p[NJ];
  uint32_t zmax_o = 0;
#pragma unroll
  for (int j = 0; j < NJ; j++) {
    const bool ok = lane + 64 * j < E;
    ord[j] = ok ? orderable(rr.z[j] + rr.b[j]) : 0u;
    const uint32_t zo = ok ? orderable(rr.z[j]) : 0u;
    zmax_o = zo > zmax_o ? zo : zmax_o;
  }
  float den = 1.0f;
  if (WEIGHTS) {
    const float m = unorderable(wave_umax(zmax_o));
    den = 0.0f;
#pragma unroll
    for (int j = 0; j < NJ; j++) { p[j] = (lane + 64 * j < E) ? __expf(rr.z[j] - m) : 0.0f; den += p[j]; }
    den = wave_sum_all(den);
  }
  float psum = 0.0f, myp = 0.0f;
  mysel = 0; mymask = 3;
  for (int r = 0; r < k; r++) {
    uint32_t best = ord[0];
    int jb = 0;
#pragma unroll
    for (int j = 1; j < NJ; j++) if (ord[j] > best) { best = ord[j]; jb = j; }
    const uint32_t top = wave_umax(best);
    int ls, js;
    if (NJ == 1) {                                            // lowest lane among equal scores
      ls = (int)__builtin_ctzll(__ballot(best == top)); js = 0;
    } else {
      const uint32_t cand = best == top ? (uint32_t)(lane + 64 * jb) : 0xFFFFFFFFu;
      const int e_star = (int)~wave_umax(~cand);              // lowest index among equal scores
      ls = e_star & 63; js = e_star >> 6;
    }
    float pw = 0.0f;
    int mk = 0;
#pragma unroll
    for (int j = 0; j < NJ; j++) {
      const int u = __builtin_amdgcn_readlane(rr.mk[j], ls);
      if (js == j) mk = u;
      if (WEIGHTS) {
        const float t = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(p[j]), ls));
        if (js == j) pw = t;
      }
      if (js == j && lane == ls) ord[j] = 0u;      // taken
    }
    psum += pw;
    // slot r belongs to lane r
    if (lane == r) { mysel = ls + 64 * js; mymask = in.mask ? mk : 3; myp = pw; }
  }
  myw = 0.0f;
  if (WEIGHTS) {
    myw = myp / den;
    if (a.norm_topk) myw = myw / (psum / den);
    myw *= a.routed_scale;
  }
}

// The decision was made elsewhere: slot r's expert and weight are read from idx_in / w_in.
// The slice mask of every expert is already in rr.mk (route_load), so the mask of the selected
// expert is a lane exchange and not a second, dependent load.
__device__ __forceinline__ void route_given(const RouteIn& in, const DecodeArgs& a, int lane, const RouteRegs& rr, int& mysel,
                                            int& mymask, float& myw) {
  const int k = in.k;
  const unsigned vo = lane < k ? (unsigned)lane * 4u : DEC_OOB;
  const int idx = (int)bload32(make_rsrc(a.idx_in, (unsigned)k * 4u), vo, 0);
  myw = __uint_as_float(bload32(make_rsrc(a.w_in, (unsigned)k * 4u), vo, 0));
  mysel = min(max(idx, 0), in.E - 1);
  int mk = 0;
#pragma unroll
  for (int j = 0; j < 4; j++) {
    const int t = __shfl(rr.mk[j], mysel & 63);
    if ((mysel >> 6) == j) mk = t;
  }
  mymask = in.mask ? mk : 3;
}

// Routing by one wave.  FULL: weights too (they are needed where the record is published, and
// where tau > 0 lets the weight decide the precision).
template <bool FULL>
__device__ __forceinline__ void route_wave(const RouteIn& in, const DecodeArgs& a, int lane, const RouteRegs& rr, int& mysel,
                                           int& myprec, float& myw) {
  int mymask;
  if (!in.do_route) route_given(in, a, lane, rr, mysel, mymask, myw);
  else if (in.E <= 64) route_topk<1, FULL>(in, a, lane, rr, mysel, mymask, myw);
  else route_topk<4, FULL>(in, a, lane, rr, mysel, mymask, myw);
  myprec = ((mymask & 3) == 3) && (a.tau <= 0.0f || myw >= a.tau);
}

// Gate weights for a selection made by route_topk<., false>: lane r < k holds slot r's expert in
// mysel.  Same arithmetic, in the same order, as route_topk<., true>.
template <int NJ>
__device__ __forceinline__ float route_weights(const RouteIn& in, const DecodeArgs& a, int lane, const RouteRegs& rr, int mysel) {
  const int E = in.E, k = in.k;
  uint32_t zmax_o = 0;
#pragma unroll
  for (int j = 0; j < NJ; j++) {
    const uint32_t zo = (lane + 64 * j < E) ? orderable(rr.z[j]) : 0u;
    zmax_o = zo > zmax_o ? zo : zmax_o;
  }
  const float m = unorderable(wave_umax(zmax_o));
  float den = 0.0f;
#pragma unroll
  for (int j = 0; j < NJ; j++) den += (lane + 64 * j < E) ? __expf(rr.z[j] - m) : 0.0f;
  den = wave_sum_all(den);
  float zsel = 0.0f;
#pragma unroll
  for (int j = 0; j < NJ; j++) {
    const float t = __shfl(rr.z[j], mysel & 63);
    if ((mysel >> 6) == j) zsel = t;
  }
  const float myp = lane < k ? __expf(zsel - m) : 0.0f;
  float psum = 0.0f;
  for (int r = 0; r < k; r++) psum += __int_as_float(__builtin_amdgcn_readlane(__float_as_int(myp), r));
  float myw = myp / den;
  if (a.norm_topk) myw = myw / (psum / den);
  return myw * a.routed_scale;
}

// ---------------------------------------------------------------------------------- gate/up kernel
// Work-group b < n_wg takes the row pairs r = b' + n_wg*q (q < cap) of every slot, b' = (b +
// slot*rot) mod n_wg, so all work-groups move the same bytes whatever the precision mix.  These
// (slot, q) entries, shared experts first, are dealt to the 8 waves in runs of L; a run is worked
// through as pieces = its entries of one slot, so expert, precision and base addresses are set up
// once per piece and the rows of a piece differ by constant offsets.  Entries of shared experts
// have their loads in flight before the routing decision exists; the last wave routes (selection
// only), the four waves before it put x into LDS in digit form.
// Work-group 0 also publishes the record for the down kernel and the caller (gate weights, weight of
// the shared experts), after the barrier, so that nothing but the selection is on the path of the
// row loads.
struct GuPiece {
  unsigned po, zo, so;      // byte offsets of the first row pair in the plane / zero-point / scale sections
  int r0, hb;               // its row, its index in h
  int prec;
};

// hand-over words of the single-launch kernel (see grid_wait)
#define ONE_MAX_WG 512                                 /* work-groups a single launch can hand over between */
#define ONE_PARITY 0                                   /* word: which flag array the running launch uses */
#define ONE_TIMEOUTS 1                                 /* word: work-groups that ever gave up waiting */
#define ONE_FLAGS(par) (64 + (par) * ONE_MAX_WG)       /* word offset of flag array 0 / 1: one word per work-group */
#define ONE_SYNC_WORDS (64 + 2 * ONE_MAX_WG)

// A value other work-groups read: within one launch (WT, the single-launch kernel) it is stored
// write-through at device scope, so that once the store is acknowledged (vmcnt) the value is where
// every other compute die's loads find it, without a write-back of the whole L2 afterwards; across a
// kernel boundary an ordinary store does.
template <bool WT, typename T> __device__ __forceinline__ void put_shared(T* p, T v) {
  if (WT) __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  else *p = v;
}

// The gate/up phase of one work-group (the body of gateup_kernel, and the first half of the
// single-launch kernel).  KARG_BYTES: size of the calling kernel's argument segment.  WT: h and the
// routing record are stored write-through at device scope (see put_shared).
template <int ACT, int SCB, int FMT, int KARG_BYTES, bool WT>
__device__ __forceinline__ void gateup_body(const float* logits, const float* bias, const uint8_t* mask, const void* x_in, int E, int k,
                                            int do_route, int d_model, int n_wg, int n_se, DecodeArgs& a, int* sel_lds, int* prec_lds,
                                            uint8_t* xvec, float2* xcs, unsigned* const* sync, unsigned* par) {
  const int tid = threadIdx.x, lane = tid & 63, wave = uni(tid >> 6);
  // Several tokens in one launch: grid (8, tokens, work-groups / 8), so that the work-groups that
  // read the same weight rows for different tokens are dispatched together on one XCD and share
  // its L2.  One token: grid (work-groups, 1, 1).  Token t uses row t of logits, x, y and of the
  // routing outputs, record t and its own h vector.
  const int tok = blockIdx.y, wg = (int)blockIdx.x + 8 * (int)blockIdx.z;
  if (tok) {
    logits += (size_t)tok * E;
    x_in = (const uint8_t*)x_in + (size_t)tok * d_model * (ACT == SMOE_BF16 ? 2 : 4);
  }
  const RouteIn in{logits, bias, mask, E, k, do_route};
  const int d = d_model, C = d >> 5;
  // ---- first instructions: the loads that need only the leading parameters -- x (stager waves)
  // and the routing inputs (router wave) -- then the fetch of all other arguments.  The explicit
  // wait closes these loads for every wave: a load still pending where control flow merges would
  // make all later code wait for every load.
  const int xt = tid - (k > 0 ? (DEC_NW - 5) * 64 : 0);
  const bool stager = xt >= 0 && xt < 4 * C;
  const bool router = k > 0 && wave == DEC_NW - 1;
  Raw8 xraw = {};
  RouteRegs rr = {};
  if (stager) load8_raw<ACT>(x_in, (size_t)xt * 8, xraw);
  route_load(in, lane, rr, router);
  KARGS_FETCH(KARG_BYTES);      // four pointers and six 4-byte leading parameters, then the struct(s)
  __builtin_amdgcn_s_waitcnt(0x0F70);      // vmcnt(0)
  // (single launch: the parity of the hand-over, needed when the work-group arrives -- see grid_wait)
  if (WT) *par = __hip_atomic_load(*sync + ONE_PARITY, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);      // (consumed at the end of the phase)
  if (tok) {
    a.h += (size_t)tok * DEC_H_STRIDE(a.n_shared * a.f_s, a.f_r);
    a.rec += tok;
    if (a.idx_in) a.idx_in += tok * k;
    if (a.w_in) a.w_in += tok * k;
    if (a.idx_out) a.idx_out += tok * k;
    if (a.w_out) a.w_out += tok * k;
    if (a.prec_out) a.prec_out += tok * k;
  }

  constexpr unsigned PB = PlaneT<FMT>::BYTES;          // plane bytes of one 32-column chunk
  const unsigned rowb32 = ((unsigned)d >> 5) * PB;
  const bool live_lane = lane < C;
  const unsigned voff = live_lane ? (unsigned)lane * PB : DEC_OOB;
  const int nsf = a.n_shared * a.f_s;
  const int N_e = n_se + k * a.cap_r;
  const int e_lo = wave * a.gu_L, e_hi = uni(min(e_lo + a.gu_L, N_e));

  typename PlaneT<FMT>::t gm[DEC_MAXP], um[DEC_MAXP], gl[DEC_MAXP], ul[DEC_MAXP];
  uint32_t zg[DEC_MAXP], zu[DEC_MAXP], sg[DEC_MAXP], su[DEC_MAXP];      // raw zero-points and scale bits

  // s = slot (shared experts first), q0 = first entry of the piece inside the slot
  auto setup = [&](bool is_sh, int s, int q0, int e, int prec, const MatK& md) {
    GuPiece pc;
    int bp = wg + s * a.rot;
    bp = bp >= n_wg ? bp - n_wg : bp;
    pc.r0 = bp + n_wg * q0;
    pc.po = (unsigned)e * md.ps32 + (unsigned)(2 * pc.r0) * rowb32;
    pc.zo = (unsigned)e * md.zs32 + (unsigned)(2 * pc.r0) * (unsigned)md.ng;
    pc.so = (unsigned)e * md.ss32 + (unsigned)(2 * pc.r0) * (unsigned)md.sng * (SCB ? 2u : 4u);
    pc.hb = (is_sh ? s * a.f_s : nsf + (s - a.n_shared) * a.f_r) + pc.r0;
    pc.prec = prec;
    return pc;
  };
  // eight unconditional loads per row pair (dead pairs / lanes / LSB planes read nothing): the small
  // metadata loads of a batch first, so that a pair's arithmetic waits for its own planes only.
  // Entry t of the batch is row pair r0 + n_wg*t.
  auto issue = [&](const GuPiece& pc, int nb, int f, const SecRsrc& R, const MatK& md, int sh) {
    const unsigned gi = (unsigned)(lane >> sh);
    const unsigned vz = live_lane ? gi : DEC_OOB;
    const unsigned vs = live_lane ? (SCB ? (gi >> 1) << 2 : gi << 2) : DEC_OOB;
    const unsigned ng = (unsigned)md.ng, sb = (unsigned)md.sng * (SCB ? 2u : 4u);
    const unsigned dz = 2u * (unsigned)n_wg * ng, ds = 2u * (unsigned)n_wg * sb, dp = 2u * (unsigned)n_wg * rowb32;
#pragma unroll
    for (int t = 0; t < DEC_MAXP; t++) {
      const bool valid = t < nb && pc.r0 + n_wg * t < f;
      zg[t] = bload8(R.zp, valid ? vz : DEC_OOB, pc.zo + (unsigned)t * dz);
      zu[t] = bload8(R.zp, valid ? vz : DEC_OOB, pc.zo + (unsigned)t * dz + ng);
      sg[t] = bload32(R.sc, valid ? vs : DEC_OOB, pc.so + (unsigned)t * ds);
      su[t] = bload32(R.sc, valid ? vs : DEC_OOB, pc.so + (unsigned)t * ds + sb);
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int t = 0; t < DEC_MAXP; t++) {
      const bool valid = t < nb && pc.r0 + n_wg * t < f;
      const unsigned vo = valid ? voff : DEC_OOB, vl = (valid && pc.prec) ? voff : DEC_OOB;
      gm[t] = pload<FMT>(R.msb, vo, pc.po + (unsigned)t * dp);
      gl[t] = pload<FMT>(R.lsb, vl, pc.po + (unsigned)t * dp);
      um[t] = pload<FMT>(R.msb, vo, pc.po + (unsigned)t * dp + rowb32);
      ul[t] = pload<FMT>(R.lsb, vl, pc.po + (unsigned)t * dp + rowb32);
    }
    __builtin_amdgcn_sched_barrier(0);
  };
  auto finish = [&](const GuPiece& pc, int nb, int f, int sh, const XR<ACT>& x) {
    const int odd = SCB ? ((lane >> sh) & 1) : 0;
#pragma unroll
    for (int t = 0; t < DEC_MAXP; t++) {
      if (t < nb && pc.r0 + n_wg * t < f) {                 // wave-uniform
        float av = lane_value(x, gm[t], gl[t], pc.prec, (int)zg[t], scale_val<SCB>(sg[t], odd));
        float uv = lane_value(x, um[t], ul[t], pc.prec, (int)zu[t], scale_val<SCB>(su[t], odd));
        av = wave_sum_to63(av);
        uv = wave_sum_to63(uv);
        if (lane == 63) put_shared<WT>(&a.h[pc.hb + n_wg * t], av * __builtin_amdgcn_rcpf(1.0f + __expf(-av)) * uv);
      }
    }
  };

  // ---- prologue: x into LDS, routing decision into LDS
  if (stager) {
    float xv[8];
    unpack8<ACT>(xraw, xv);
    stage_regs<ACT>(xv, C, xt >> 2, xt & 3, xvec, xcs);
  }
  int mysel = 0, myprec = 0;
  float myw = 0.0f;
  const bool have_w = a.tau > 0.0f || !do_route;      // the weight decides the precision, or was handed in
  if (router) {
    if (have_w) route_wave<true>(in, a, lane, rr, mysel, myprec, myw);
    else route_wave<false>(in, a, lane, rr, mysel, myprec, myw);
    if (lane < k) { sel_lds[lane] = mysel; prec_lds[lane] = myprec; }
  }

  // ---- a first batch of shared-expert entries: rows in flight before the routing decision exists
  int e_cur = uni(e_lo), nb0 = 0;
  GuPiece pc0 = {};
  const bool pre = e_lo < min(e_hi, n_se);
  if (pre) {
    const int s = fastdiv(e_cur, a.inv_cap_s), q0 = e_cur - s * a.cap_s;
    nb0 = uni(min(DEC_MAXP, min(min(e_hi, n_se) - e_cur, a.cap_s - q0)));
    pc0 = setup(true, s, q0, s, 1, a.sgu);
    issue(pc0, nb0, a.f_s, make_sec(a.sgu, a.n_shared), a.sgu, a.gu_sh_s);
  }
  lds_barrier();
  if (wg == 0) {
    if (router) {                                        // publish for the down kernel and the caller
      if (!have_w) myw = E <= 64 ? route_weights<1>(in, a, lane, rr, mysel) : route_weights<4>(in, a, lane, rr, mysel);
      if (lane < k) {
        put_shared<WT>(&a.rec->sel[lane], mysel); put_shared<WT>(&a.rec->prec[lane], myprec); put_shared<WT>(&a.rec->w[lane], myw);
        if (a.prec_out) a.prec_out[lane] = (uint8_t)myprec;
        if (a.idx_out) a.idx_out[lane] = mysel;
        if (a.w_out) a.w_out[lane] = myw;
      }
    }
    if (wave == DEC_NW - 3) {                            // weight of the shared experts
      float g = 1.0f;
      if (a.shared_gate_w) {
        // d <= 2048: at most four 8-element pieces per lane; all loads go out before the first use
        Raw8 wr[4], xr[4];
#pragma unroll
        for (int j = 0; j < 4; j++) {
          const int i0 = (lane + 64 * j) * 8;
          wr[j] = Raw8{}; xr[j] = Raw8{};
          if (i0 < d) { load8_raw<ACT>(a.shared_gate_w, (size_t)i0, wr[j]); load8_raw<ACT>(x_in, (size_t)i0, xr[j]); }
        }
        float p = 0.0f;
#pragma unroll
        for (int j = 0; j < 4; j++) {
          float wv[8], xv8[8];
          unpack8<ACT>(wr[j], wv);
          unpack8<ACT>(xr[j], xv8);
#pragma unroll
          for (int i = 0; i < 8; i++) p = fmaf(wv[i], xv8[i], p);
        }
        g = 1.0f / (1.0f + expf(-wave_sum(p)));
      }
      if (lane == 0) put_shared<WT>(&a.rec->gamma, g);
    }
  }
  XR<ACT> x = {};
  if (live_lane) load_xr<ACT>(x, xvec, xcs, 0, C, lane);
  if (pre) {
    finish(pc0, nb0, a.f_s, a.gu_sh_s, x);
    e_cur = uni(e_cur + nb0);
  }
  // ---- everything else, batch by batch
  while (e_cur < e_hi) {
    if (e_cur < n_se) {
      const int s = fastdiv(e_cur, a.inv_cap_s), q0 = e_cur - s * a.cap_s;
      const int nb = uni(min(DEC_MAXP, min(min(e_hi, n_se) - e_cur, a.cap_s - q0)));
      const GuPiece pc = setup(true, s, q0, s, 1, a.sgu);
      issue(pc, nb, a.f_s, make_sec(a.sgu, a.n_shared), a.sgu, a.gu_sh_s);
      finish(pc, nb, a.f_s, a.gu_sh_s, x);
      e_cur = uni(e_cur + nb);
    } else {
      const int er = e_cur - n_se;
      const int sr = fastdiv(er, a.inv_cap_r), q0 = er - sr * a.cap_r;
      const int nb = uni(min(DEC_MAXP, min(e_hi - e_cur, a.cap_r - q0)));
      const GuPiece pc = setup(false, a.n_shared + sr, q0, uni(sel_lds[sr]), uni(prec_lds[sr]), a.rgu);
      issue(pc, nb, a.f_r, make_sec(a.rgu, E), a.rgu, a.gu_sh_r);
      finish(pc, nb, a.f_r, a.gu_sh_r, x);
      e_cur = uni(e_cur + nb);
    }
  }
}

template <int ACT, int SCB, int FMT>
__global__ __launch_bounds__(DEC_NT) void gateup_kernel(const float* logits, const float* bias, const uint8_t* mask, const void* x_in,
                                                        int E, int k, int do_route, int d_model, int n_wg, int n_se,
                                                        DecodeArgs a) {
  __shared__ int sel_lds[SMOE_MAX_TOPK], prec_lds[SMOE_MAX_TOPK];
  __shared__ __align__(16) uint8_t xvec[StageTraits<ACT>::COMBO_BYTES];
  __shared__ float2 xcs[64];
  gateup_body<ACT, SCB, FMT, DEC_LEAD_BYTES + (int)sizeof(DecodeArgs), false>(logits, bias, mask, x_in, E, k, do_route, d_model, n_wg, n_se, a,
                                                                             sel_lds, prec_lds, xvec, xcs, nullptr, nullptr);
}

// ---------------------------------------------------------------------------------- gate/up kernel, wide rows
// d_model above 2048 (up to DEC_WIDE_MAX_D): a row has more 32-column chunks than a wave has lanes, so a
// lane takes one chunk of each of up to four 64-chunk k-slices and adds the partial values before the
// wave sum.  Same split of the row pairs over work-groups and waves, same routing wave and record as
// gateup_kernel; one row pair at a time per wave, all k-slices of the pair in flight together.
#define DEC_WIDE_KS 4
#define DEC_WIDE_MAX_D (DEC_WIDE_KS * 2048)
template <int ACT> struct WideTraits;
template <> struct WideTraits<SMOE_BF16> { enum { SLICE_BYTES = 4096 }; };      // the k-slice stride of stage_regs / load_xr
template <> struct WideTraits<SMOE_F32> { enum { SLICE_BYTES = 8192 }; };

template <int ACT, int SCB, int FMT, int NKS>      // NKS: k-slices a lane has registers for (2: d_model <= 4096, else 4)
__global__ __launch_bounds__(DEC_NT) void gateup_wide_kernel(const float* logits, const float* bias, const uint8_t* mask, const void* x_in,
                                                             int E, int k, int do_route, int d_model, int n_wg, int n_se,
                                                             DecodeArgs a) {
  __shared__ int sel_lds[SMOE_MAX_TOPK], prec_lds[SMOE_MAX_TOPK];
  __shared__ __align__(16) uint8_t xvec[DEC_WIDE_KS * WideTraits<ACT>::SLICE_BYTES];
  __shared__ float2 xcs[DEC_WIDE_KS * 64];
  const int tid = threadIdx.x, lane = tid & 63, wave = uni(tid >> 6);
  const int tok = blockIdx.y, wg = (int)blockIdx.x + 8 * (int)blockIdx.z;
  if (tok) {
    logits += (size_t)tok * E;
    x_in = (const uint8_t*)x_in + (size_t)tok * d_model * (ACT == SMOE_BF16 ? 2 : 4);
    a.h += (size_t)tok * DEC_H_STRIDE(a.n_shared * a.f_s, a.f_r);
    a.rec += tok;
    if (a.idx_in) a.idx_in += tok * k;
    if (a.w_in) a.w_in += tok * k;
    if (a.idx_out) a.idx_out += tok * k;
    if (a.w_out) a.w_out += tok * k;
    if (a.prec_out) a.prec_out += tok * k;
  }
  const RouteIn in{logits, bias, mask, E, k, do_route};
  const int d = d_model, C = d >> 5, KS = (C + 63) >> 6;
  const bool router = k > 0 && wave == DEC_NW - 1;
  RouteRegs rr = {};
  route_load(in, lane, rr, router);
  // ---- x into LDS in digit form: word i (8 values) of the vector belongs to chunk i / 4; a quad handles a chunk
  for (int i = tid; i < 4 * C; i += DEC_NT) {
    Raw8 xraw = {};
    load8_raw<ACT>(x_in, (size_t)i * 8, xraw);
    float xv[8];
    unpack8<ACT>(xraw, xv);
    stage_regs<ACT>(xv, C, i >> 2, i & 3, xvec, xcs);
  }
  int mysel = 0, myprec = 0;
  float myw = 0.0f;
  if (router) {
    route_wave<true>(in, a, lane, rr, mysel, myprec, myw);
    if (lane < k) { sel_lds[lane] = mysel; prec_lds[lane] = myprec; }
  }
  __syncthreads();
  if (wg == 0) {
    if (router && lane < k) {
      a.rec->sel[lane] = mysel; a.rec->prec[lane] = myprec; a.rec->w[lane] = myw;
      if (a.prec_out) a.prec_out[lane] = (uint8_t)myprec;
      if (a.idx_out) a.idx_out[lane] = mysel;
      if (a.w_out) a.w_out[lane] = myw;
    }
    if (wave == 0) {                                       // weight of the shared experts
      float g = 1.0f;
      if (a.shared_gate_w) {
        float p = 0.0f;
        for (int i0 = lane * 8; i0 < d; i0 += 512) {
          Raw8 wr = {}, xr = {};
          load8_raw<ACT>(a.shared_gate_w, (size_t)i0, wr);
          load8_raw<ACT>(x_in, (size_t)i0, xr);
          float wv[8], xv8[8];
          unpack8<ACT>(wr, wv);
          unpack8<ACT>(xr, xv8);
#pragma unroll
          for (int i = 0; i < 8; i++) p = fmaf(wv[i], xv8[i], p);
        }
        g = 1.0f / (1.0f + expf(-wave_sum(p)));
      }
      if (lane == 0) a.rec->gamma = g;
    }
  }

  constexpr unsigned PB = PlaneT<FMT>::BYTES;
  const unsigned rowb32 = (unsigned)C * PB;
  const int nsf = a.n_shared * a.f_s;
  const int N_e = n_se + k * a.cap_r;
  const int e_lo = wave * a.gu_L, e_hi = uni(min(e_lo + a.gu_L, N_e));
  for (int e_cur = e_lo; e_cur < e_hi; e_cur++) {
    const bool is_sh = e_cur < n_se;
    int s, q0, ex, prec, f, sh;
    if (is_sh) {
      s = fastdiv(e_cur, a.inv_cap_s); q0 = e_cur - s * a.cap_s; ex = s; prec = 1; f = a.f_s; sh = a.gu_sh_s;
    } else {
      const int er = e_cur - n_se, sr = fastdiv(er, a.inv_cap_r);
      s = a.n_shared + sr; q0 = er - sr * a.cap_r; ex = uni(sel_lds[sr]); prec = uni(prec_lds[sr]); f = a.f_r; sh = a.gu_sh_r;
    }
    const MatK& md = is_sh ? a.sgu : a.rgu;
    int bp = wg + s * a.rot;
    bp = bp >= n_wg ? bp - n_wg : bp;
    const int r0 = bp + n_wg * q0;
    if (r0 >= f) continue;                                  // wave-uniform
    const SecRsrc R = make_sec(md, is_sh ? a.n_shared : E);
    const unsigned po = (unsigned)ex * md.ps32 + (unsigned)(2 * r0) * rowb32;
    const unsigned zo = (unsigned)ex * md.zs32 + (unsigned)(2 * r0) * (unsigned)md.ng;
    const unsigned sb = (unsigned)md.sng * (SCB ? 2u : 4u);
    const unsigned so = (unsigned)ex * md.ss32 + (unsigned)(2 * r0) * sb;
    typename PlaneT<FMT>::t gm[NKS], um[NKS], gl[NKS], ul[NKS];
    uint32_t zg[NKS], zu[NKS], sg[NKS], su[NKS];
#pragma unroll
    for (int ks = 0; ks < NKS; ks++) {
      const unsigned c = (unsigned)(ks * 64 + lane), gi = c >> sh;
      const bool live = ks < KS && c < (unsigned)C;
      const unsigned vz = live ? gi : DEC_OOB, vs = live ? (SCB ? (gi >> 1) << 2 : gi << 2) : DEC_OOB;
      const unsigned vo = live ? c * PB : DEC_OOB, vl = (live && prec) ? c * PB : DEC_OOB;
      zg[ks] = bload8(R.zp, vz, zo);
      zu[ks] = bload8(R.zp, vz, zo + (unsigned)md.ng);
      sg[ks] = bload32(R.sc, vs, so);
      su[ks] = bload32(R.sc, vs, so + sb);
      gm[ks] = pload<FMT>(R.msb, vo, po);
      gl[ks] = pload<FMT>(R.lsb, vl, po);
      um[ks] = pload<FMT>(R.msb, vo, po + rowb32);
      ul[ks] = pload<FMT>(R.lsb, vl, po + rowb32);
    }
    float av = 0.0f, uv = 0.0f;
#pragma unroll
    for (int ks = 0; ks < NKS; ks++) {
      if (ks < KS) {                                        // wave-uniform
        const int cw = min(64, C - ks * 64);
        const int odd = SCB ? (((ks * 64 + lane) >> sh) & 1) : 0;
        XR<ACT> x = {};
        if (lane < cw) load_xr<ACT>(x, xvec, xcs, ks, cw, lane);
        av += lane_value(x, gm[ks], gl[ks], prec, (int)zg[ks], scale_val<SCB>(sg[ks], odd));
        uv += lane_value(x, um[ks], ul[ks], prec, (int)zu[ks], scale_val<SCB>(su[ks], odd));
      }
    }
    av = wave_sum_to63(av);
    uv = wave_sum_to63(uv);
    if (lane == 63) a.h[(is_sh ? s * a.f_s : nsf + (s - a.n_shared) * a.f_r) + r0] = av * __builtin_amdgcn_rcpf(1.0f + __expf(-av)) * uv;
  }
}

// ---------------------------------------------------------------------------------- down kernel
// A work-group owns DEC_RPW = 8 output rows.  Its work is cut into pieces = (combo, part): a combo
// is one (slot, 64-chunk k-slice) pair -- shared experts first, then the routed slots -- and a
// combo's 8 rows are split into P parts of 8/P rows (P = the largest power of two that gives the 8
// waves at most one piece each; the host picks it).  Wave w takes pieces w, w+8, ...  Everything a
// piece needs beyond its rows -- expert, precision, weight, the h chunk in digit form -- belongs to
// its combo, so a wave works it out once, and no wave depends on another before the final sum:
// every wave puts the h chunks of its own combo into a private LDS area (the digit transposition
// needs a trip through LDS, not a barrier).  The instruction count of the longest wave bounds the
// kernel from below (a wave issues at most one instruction every four cycles), hence the flat
// structure and the host-side arithmetic.

// Totals of v0..v3 over the wave, left in lanes 60..63 (lane 60 + i holds the total of v_i).
__device__ __forceinline__ float wave_sum4_to_last(float v0, float v1, float v2, float v3, int lane) {
  const bool o1 = lane & 1, o2 = lane & 2;
  const float t01 = (o1 ? v1 : v0) + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(o1 ? v0 : v1), 0xB1, 0xF, 0xF, true));
  const float t23 = (o1 ? v3 : v2) + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(o1 ? v2 : v3), 0xB1, 0xF, 0xF, true));
  float s = (o2 ? t23 : t01) + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(o2 ? t01 : t23), 0x4E, 0xF, 0xF, true));
  s = dpp_add<0x114, 0xF, 0xF>(s);     // lane % 4 = i now holds the quad sum of v_i: fold the quads of a row
  s = dpp_add<0x118, 0xF, 0xF>(s);     // lanes 12..15 of every row: the row's totals of v0..v3
  s += __shfl_xor(s, 16);              // fold the four rows (the row broadcasts of the single-value
  s += __shfl_xor(s, 32);              // reduction would mix the four interleaved sums)
  return s;
}

#define DEC_HQ 4      // h words of 8 values per lane that cover one combo (64 chunks)

// What the single-launch kernel adds to the arguments of the two kernels.
struct OneArgs {
  unsigned* sync;                  // hand-over words in the workspace, see below
  int n_combo_s, n_pieces, psh;    // the down split (the down kernel's leading parameters)
  int n_dn;                        // work-groups that go on to a down phase
  int spin_limit;                  // polls before a work-group gives up waiting
  int pad0;
};
static_assert(sizeof(DecodeArgs) + sizeof(OneArgs) + DEC_LEAD_BYTES <= 8 * 64, "KARGS_FETCH covers eight lines");

// The grid-wide hand-over of the single-launch kernel.  No read-modify-write: every work-group owns one
// word of a flag array and sets it (write-through) once all its waves' stores of h are acknowledged; a
// waiting wave reads the whole array with device-scope loads until every word is set.  Two arrays take
// turns: the launch uses the one the parity word names (every work-group reads the parity in its first
// instructions, long before it arrives), work-group 0 clears the other array for the next launch and,
// once its own wait is over -- so every work-group has arrived and has therefore read the parity --
// flips the parity.  Launches of one context are ordered by its stream, so the next launch finds its
// array cleared and the parity flipped.  The wait is bounded: after spin_limit polls the work-group
// goes on (its result is then wrong) and counts itself in the timeouts word, which the host reads
// back; work-group 0 flips the parity all the same, and the work-groups that arrive late only set
// words of an array that is cleared again before it is next used.  All work-groups of the launch
// must be resident together (the host checks the occupancy).
__device__ __forceinline__ void grid_set_flag(unsigned* sync, unsigned par, int wg) {
  __hip_atomic_store(sync + ONE_FLAGS(par) + wg, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// one wave; n_wg <= ONE_MAX_WG: lane l looks at words 8 l .. 8 l + 7
__device__ __forceinline__ void grid_wait(unsigned* sync, unsigned par, int n_wg, int wg, int spin_limit, int lane) {
  if (wg == 0) {      // the other array, all of it, for the next launch
    uint4* o = (uint4*)(sync + ONE_FLAGS(par ^ 1u) + 8 * lane);
    o[0] = make_uint4(0, 0, 0, 0);
    o[1] = make_uint4(0, 0, 0, 0);
  }
  const __amdgpu_buffer_rsrc_t RF = make_rsrc(sync + ONE_FLAGS(par), (unsigned)n_wg * 4u);      // words past n_wg read as 0
  const int mine = min(8, max(0, n_wg - 8 * lane));                                               // words this lane must see set
  int spins = 0;
  for (;;) {
    const uint4 f0 = bload128_dev(RF, (unsigned)lane * 32u, 0), f1 = bload128_dev(RF, (unsigned)lane * 32u, 16);
    const int set = (int)(f0.x + f0.y + f0.z + f0.w + f1.x + f1.y + f1.z + f1.w);
    if (__builtin_amdgcn_ballot_w64(set < mine) == 0) break;
    if (++spins >= spin_limit) {
      if (lane == 0) __hip_atomic_fetch_add(sync + ONE_TIMEOUTS, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      break;
    }
    __builtin_amdgcn_s_sleep(1);
  }
  if (wg == 0 && lane == 0) __hip_atomic_store(sync + ONE_PARITY, par ^ 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// The down phase of one work-group: the body of down_kernel, and the second half of the single-launch
// kernel (ONE).  There the expert and precision of a routed slot come from the work-group's own routing
// decision in LDS, a wave first puts the loads of its piece's first rows in flight and only then joins
// the hand-over (the last wave, which does the polling, issues no loads before it: a poll's answer would
// queue behind them), and h and the gate weights are read after it.
template <int ACT, int SCB, int FMT, int RPW, bool ONE>
__device__ __forceinline__ void down_body(const int* rec, const float* h, int n_combo_s, int n_pieces, int psh, int f_s, int f_r, int ks_s,
                                          int ks_r, int inv_ks_s, int inv_ks_r, int nsf, const DecodeArgs& a, uint8_t* dyn, int wg, int tok,
                                          const int* sel_lds, const int* prec_lds, const OneArgs* one, int n_wg, unsigned par) {
  const int tid = threadIdx.x, lane = tid & 63, wave = uni(tid >> 6);
  constexpr int XB = StageTraits<ACT>::COMBO_BYTES, WS = XB + 64 * 8;
  constexpr int DEC_RB = ACT == SMOE_BF16 ? 4 : 2;      // rows per batch (the fp32 path keeps 32 activations per lane in registers)
  uint8_t* xbuf = dyn + wave * WS;
  float2* xcs = (float2*)(xbuf + XB);
  float* part = (float*)(dyn + DEC_NW * WS);         // [combo][row]
  const int n0 = wg * RPW;
  bool kargs_here = ONE, handed_over = !ONE;
  const bool poller = ONE && wave == DEC_NW - 1;
  if (ONE && wave >= n_pieces) {                     // a wave without a piece still takes part in the hand-over
    if (poller) grid_wait(one->sync, par, n_wg, wg, one->spin_limit, lane);
    lds_barrier();
  }

  for (int p = wave; p < n_pieces; p += DEC_NW) {
    // ---- which piece (leading parameters only)
    const int combo = p >> psh, row0 = (p & ((1 << psh) - 1)) * (RPW >> psh), n_rows = RPW >> psh;
    const bool is_sh = combo < n_combo_s;
    const int c2 = is_sh ? combo : combo - n_combo_s;
    const int ksn = is_sh ? ks_s : ks_r, inv_ks = is_sh ? inv_ks_s : inv_ks_r, f = is_sh ? f_s : f_r;
    const int slot = fastdiv(c2, (uint32_t)inv_ks), ks = c2 - slot * ksn;
    const int cw = min(64, (f >> 5) - ks * 64);
    const int hoff = (is_sh ? 0 : nsf) + slot * f + ks * 2048;      // first h value of the combo
    // ---- first loads: the combo's h values (8 per lane and word, words past the combo read nothing)
    // and the routing record (sizeof(RouteRec) == 64 words: sel / prec / w of slot s in words s,
    // 16+s, 32+s, gamma in word 48)
    const __amdgpu_buffer_rsrc_t RH = make_rsrc(h + hoff, (unsigned)cw * 128u);
    uint4 hraw[DEC_HQ][2];
    int rec_word = 0;
    auto load_h = [&]() {
#pragma unroll
      for (int q = 0; q < DEC_HQ; q++) {
        // (single launch: h and the record were written in this very launch, by other compute dies too)
        hraw[q][0] = ONE ? bload128_dev(RH, (unsigned)(lane + 64 * q) * 32u, 0) : bload128(RH, (unsigned)(lane + 64 * q) * 32u, 0);
        hraw[q][1] = ONE ? bload128_dev(RH, (unsigned)(lane + 64 * q) * 32u, 16) : bload128(RH, (unsigned)(lane + 64 * q) * 32u, 16);
      }
      rec_word = ONE ? __hip_atomic_load(rec + lane, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : rec[lane];
    };
    int e, prec;
    if (ONE) {
      e = is_sh ? slot : uni(sel_lds[is_sh ? 0 : slot]);
      prec = is_sh ? 1 : uni(prec_lds[is_sh ? 0 : slot]);
      if (handed_over) load_h();
    } else {
      load_h();
      if (!kargs_here) {      // two pointers and ten 4-byte leading parameters, then the struct
        KARGS_FETCH(DEC_LEAD_BYTES + (int)sizeof(DecodeArgs));
        kargs_here = true;
      }
      __builtin_amdgcn_s_waitcnt(0x0F70);      // vmcnt(0)
      e = is_sh ? slot : __builtin_amdgcn_readlane(rec_word, slot);
      prec = is_sh ? 1 : __builtin_amdgcn_readlane(rec_word, SMOE_MAX_TOPK + slot);
    }

    // ---- the piece's rows: per batch of DEC_RB rows issue metadata, then planes; then h -> digits
    // while they stream in; then the dot products
    const MatK& md = is_sh ? a.sdn : a.rdn;
    const SecRsrc R = make_sec(md, is_sh ? a.n_shared : a.E);
    const int sh = is_sh ? a.dn_sh_s : a.dn_sh_r;
    const bool live = lane < cw;
    constexpr unsigned PB = PlaneT<FMT>::BYTES;
    const unsigned vo = live ? (unsigned)lane * PB : DEC_OOB, vl = (live && prec) ? vo : DEC_OOB;
    const int g0 = (ks * 64) >> sh;                                  // first group of the k-slice
    const int tg = (lane >> sh) + (g0 & 1);                          // scale position relative to an even element
    const unsigned vz = live ? (unsigned)(lane >> sh) : DEC_OOB;
    const unsigned vs = live ? (SCB ? (unsigned)(tg >> 1) << 2 : (unsigned)(lane >> sh) << 2) : DEC_OOB;
    const int odd = SCB ? (tg & 1) : 0;
    const unsigned rowb = ((unsigned)f >> 5) * PB, ng = (unsigned)md.ng, srow = (unsigned)md.sng * (SCB ? 2u : 4u);
    unsigned po = (unsigned)e * md.ps32 + (unsigned)(n0 + row0) * rowb + (unsigned)ks * (64u * PB);
    unsigned zo = (unsigned)e * md.zs32 + (unsigned)(n0 + row0) * ng + (unsigned)g0;
    unsigned so = (unsigned)e * md.ss32 + (unsigned)(n0 + row0) * srow + (SCB ? (unsigned)(g0 & ~1) * 2u : (unsigned)g0 * 4u);
    XR<ACT> x = {};
    float wt = 0.0f;
    for (int b0 = 0; b0 < n_rows; b0 += DEC_RB) {
      const int nr = min(DEC_RB, n_rows - b0);
      typename PlaneT<FMT>::t wm[DEC_RB], wl[DEC_RB];
      uint32_t zz[DEC_RB], ss[DEC_RB];
      if (ONE && !handed_over && poller) {           // (b0 == 0 of the wave's first piece)
        grid_wait(one->sync, par, n_wg, wg, one->spin_limit, lane);
        lds_barrier();
        load_h();
        handed_over = true;
      }
#pragma unroll
      for (int r = 0; r < DEC_RB; r++) {
        zz[r] = bload8(R.zp, r < nr ? vz : DEC_OOB, zo + (unsigned)r * ng);
        ss[r] = bload32(R.sc, r < nr ? vs : DEC_OOB, so + (unsigned)r * srow);
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int r = 0; r < DEC_RB; r++) {
        wm[r] = pload<FMT>(R.msb, r < nr ? vo : DEC_OOB, po + (unsigned)r * rowb);
        wl[r] = pload<FMT>(R.lsb, r < nr ? vl : DEC_OOB, po + (unsigned)r * rowb);
      }
      __builtin_amdgcn_sched_barrier(0);
      po += DEC_RB * rowb; zo += DEC_RB * ng; so += DEC_RB * srow;
      if (ONE && !handed_over) {                     // the rows are in flight: now wait for the other work-groups' h
        lds_barrier();
        load_h();
        handed_over = true;
      }
      if (b0 == 0) {
        wt = __int_as_float(__builtin_amdgcn_readlane(rec_word, is_sh ? 3 * SMOE_MAX_TOPK : 2 * SMOE_MAX_TOPK + slot));
        // h -> LDS in digit form (the four lanes of a quad hold one chunk), back as one chunk per lane
#pragma unroll
        for (int q = 0; q < DEC_HQ; q++) {
          if (64 * q < 4 * cw) {
            const int item = lane + 64 * q;
            if (item < 4 * cw) {
              Raw8 raw; raw.a = hraw[q][0]; raw.b = hraw[q][1];
              float hv[8];
              unpack8<SMOE_F32>(raw, hv);
              stage_regs<ACT>(hv, cw, item >> 2, item & 3, xbuf, xcs);
            }
          }
        }
        if (live) load_xr<ACT>(x, xbuf, xcs, 0, cw, lane);
      }
      float v[4] = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
      for (int r = 0; r < DEC_RB; r++) v[r] = lane_value(x, wm[r], wl[r], prec, (int)zz[r], scale_val<SCB>(ss[r], odd));
      const float tot = wave_sum4_to_last(v[0], v[1], v[2], v[3], lane);
      if (lane >= 60 && lane - 60 < nr) part[combo * RPW + row0 + b0 + lane - 60] = wt * tot;
    }
  }
  __syncthreads();
  if (tid < RPW) {
    const int n_combo = n_pieces >> psh;
    float acc = 0.0f;
    for (int c = n_combo_s; c < n_combo; c++) acc += part[c * RPW + tid];      // routed slots in slot order
    for (int c = 0; c < n_combo_s; c++) acc += part[c * RPW + tid];            // then the shared experts
    const size_t n = (size_t)tok * a.d_model + n0 + tid;
    if (a.add_residual) acc += load_act<ACT>(a.x, n);
    store_act<ACT>(a.y, n, acc);
  }
}

template <int ACT, int SCB, int FMT, int RPW>      // RPW output rows per work-group
__global__ __launch_bounds__(DEC_NT) void down_kernel(const int* rec, const float* h, int n_combo_s, int n_pieces, int psh, int f_s,
                                                      int f_r, int ks_s, int ks_r, int inv_ks_s, int inv_ks_r, int nsf,
                                                      DecodeArgs a) {
  extern __shared__ __align__(16) uint8_t dyn[];     // [per wave: h digits of one combo, chunk figures][partials]
  const int tok = blockIdx.y;                          // see gateup_kernel
  if (tok) {
    rec += tok * (int)(sizeof(RouteRec) / 4);
    h += (size_t)tok * DEC_H_STRIDE(nsf, f_r);
  }
  down_body<ACT, SCB, FMT, RPW, false>(rec, h, n_combo_s, n_pieces, psh, f_s, f_r, ks_s, ks_r, inv_ks_s, inv_ks_r, nsf, a, dyn,
                                       (int)blockIdx.x + 8 * (int)blockIdx.z, tok, nullptr, nullptr, nullptr, 0, 0u);
}

// ---------------------------------------------------------------------------------- single-launch kernel
// One token, rows of at most 64 chunks: the gate/up phase of n_wg work-groups, a grid-wide hand-over of
// h, and the down phase in the first n_dn of them, all in one launch (an option of the context; the
// two launches are the default because they measured faster on this hardware: data handed from one
// compute die to another inside a kernel costs several microseconds, the end of a kernel a fraction
// of one).  Same arithmetic in the same order as the two kernels: results are bit-identical.
// (bf16 activations: at most 128 vector registers, so that two work-groups share a CU like those of
// gateup_kernel; the fp32 path keeps 32 activations per lane and gets the full register file, one
// work-group per CU.)
template <int ACT, int SCB, int FMT>
__global__ __launch_bounds__(DEC_NT, ACT == SMOE_F32 ? 2 : 4) void decode_one_kernel(const float* logits, const float* bias, const uint8_t* mask, const void* x_in,
                                                               int E, int k, int do_route, int d_model, int n_wg, int n_se, DecodeArgs a,
                                                               OneArgs o) {
  __shared__ int sel_lds[SMOE_MAX_TOPK], prec_lds[SMOE_MAX_TOPK];
  __shared__ __align__(16) uint8_t xvec[StageTraits<ACT>::COMBO_BYTES];
  __shared__ float2 xcs[64];
  extern __shared__ __align__(16) uint8_t dyn[];
  unsigned par = 0;
  gateup_body<ACT, SCB, FMT, DEC_LEAD_BYTES + (int)sizeof(DecodeArgs) + (int)sizeof(OneArgs), true>(logits, bias, mask, x_in, E, k, do_route, d_model,
                                                                                           n_wg, n_se, a, sel_lds, prec_lds, xvec, xcs, &o.sync, &par);
  // every wave's part of h (and work-group 0's routing record) acknowledged before the work-group counts itself in
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  par = (unsigned)uni((int)par) & 1u;
  __syncthreads();
  const int wg = blockIdx.x;
  if (threadIdx.x == 0) grid_set_flag(o.sync, par, wg);
  if (wg >= o.n_dn) return;
  down_body<ACT, SCB, FMT, DEC_RPW, true>((const int*)a.rec, a.h, o.n_combo_s, o.n_pieces, o.psh, a.f_s, a.f_r, a.ks_s, a.ks_r, a.inv_ks_s,
                                          a.inv_ks_r, a.n_shared * a.f_s, a, dyn, wg, 0, sel_lds, prec_lds, &o, n_wg, par);
}

// ---------------------------------------------------------------------------------- host entry
static int ilog2_exact(int v) {
  int s = 0;
  while ((1 << s) < v) s++;
  return (1 << s) == v ? s : -1;
}

template <int ACT, int SCB, int FMT, int RPW>
static int launch_decode_t(smoe_ctx* ctx, const RouteIn& in, DecodeArgs& a, int n_wg, int T) {
  // down kernel: pieces = combos x parts
  const int n_combo_s = a.n_shared * a.ks_s, n_combo = n_combo_s + a.k * a.ks_r;
  int psh = RPW == 64 ? 6 : RPW == 32 ? 5 : RPW == 16 ? 4 : 3;      // at most RPW parts of one row each
  while (psh > 0 && (n_combo << psh) > DEC_NW) psh--;
  const int n_pieces = n_combo << psh;
  const size_t lds = (size_t)DEC_NW * (StageTraits<ACT>::COMBO_BYTES + 64 * 8) + (size_t)n_combo * RPW * 4;
  if (lds > 160u * 1024u) return SMOE_ESIZE;
  if (lds > 64u * 1024u) {       // beyond the default per-work-group limit: ask for the larger carve-out
    // (kept per context, that is per device: the attribute belongs to the function on the current device)
    size_t& granted = ctx->down_lds_granted[((ACT * 2 + SCB) * 3 + FMT) * 4 + (RPW == 16) + 2 * (RPW == 32) + 3 * (RPW == 64)];
    if (lds > granted) {
      if (hipFuncSetAttribute((const void*)down_kernel<ACT, SCB, FMT, RPW>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess) {
        (void)hipGetLastError();
        return SMOE_ESIZE;
      }
      granted = lds;
    }
  }
  std::vector<hipEvent_t>* evs = (ctx->timing && ctx->timing_events) ? (std::vector<hipEvent_t>*)ctx->timing_events : nullptr;
  const int n_dn = a.d_model / RPW;
  if (T > 1 && ((n_wg & 7) || (n_dn & 7))) return SMOE_ESHAPE;      // the multi-token grid is (8, T, n / 8)
  const dim3 g1 = T > 1 ? dim3(8, T, n_wg / 8) : dim3(n_wg), g2 = T > 1 ? dim3(8, T, n_dn / 8) : dim3(n_dn), blk(DEC_NT);
  const int n_se = a.n_shared * a.cap_s;
  const bool wide = a.d_model > 2048;                 // rows of more than 64 chunks: the k-sliced gate/up kernel
  const int* recw = (const int*)a.rec;
  const int nsf = a.n_shared * a.f_s;
  // ---- single launch, if the context asks for it and the case fits: one token, rows of at most 64
  // chunks, 8 output rows per down work-group, no more down work-groups than gate/up work-groups, the
  // context's own workspace (its hand-over words were cleared when the mode was switched on), and all
  // work-groups resident at once
  if (ctx->one_launch && T == 1 && !wide && RPW == DEC_RPW && n_dn <= n_wg && n_wg <= ONE_MAX_WG && !evs && (uint8_t*)a.rec == ctx->ws + WS_REC_OFF) {
    const size_t lds1 = lds;
    int& per_cu = ctx->one_blocks_per_cu[((ACT * 2 + SCB) * 3 + FMT)];
    size_t& lds_seen = ctx->one_lds_seen[((ACT * 2 + SCB) * 3 + FMT)];
    bool ok = true;
    if (per_cu == 0 || lds1 > lds_seen) {
      if (lds1 > 48u * 1024u &&
          hipFuncSetAttribute((const void*)decode_one_kernel<ACT, SCB, FMT>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds1) != hipSuccess) {
        (void)hipGetLastError();
        ok = false;
      }
      int nb = 0;
      if (ok && hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, (const void*)decode_one_kernel<ACT, SCB, FMT>, DEC_NT, lds1) != hipSuccess) {
        (void)hipGetLastError();
        ok = false;
      }
      if (ok) { per_cu = nb > 0 ? nb : -1; lds_seen = lds1; }
    }
    if (ok && per_cu > 0 && (long)per_cu * ctx->n_cu >= n_wg) {
      OneArgs o{};
      o.sync = (unsigned*)(ctx->ws + WS_SYNC_OFF);
      o.n_combo_s = n_combo_s; o.n_pieces = n_pieces; o.psh = psh; o.n_dn = n_dn;
      o.spin_limit = ctx->one_spin_limit;
      decode_one_kernel<ACT, SCB, FMT><<<g1, blk, lds1, ctx->stream>>>(in.logits, in.bias, in.mask, a.x, in.E, in.k, in.do_route, a.d_model,
                                                                     n_wg, n_se, a, o);
      HIPCHK(ctx, hipGetLastError());
      ctx->one_calls++;
      return SMOE_OK;
    }
  }
  if (evs) {
    // measurement aid: the dispatches themselves carry start/stop events (no extra marker packets)
    hipEvent_t ev[4];
    for (int i = 0; i < 4; i++) { HIPCHK(ctx, hipEventCreate(&ev[i])); evs->push_back(ev[i]); }
    if (wide && a.d_model <= 4096)
      hipExtLaunchKernelGGL((gateup_wide_kernel<ACT, SCB, FMT, 2>), g1, blk, 0, ctx->stream, ev[0], ev[1], 0, in.logits, in.bias, in.mask, a.x,
                            in.E, in.k, in.do_route, a.d_model, n_wg, n_se, a);
    else if (wide)
      hipExtLaunchKernelGGL((gateup_wide_kernel<ACT, SCB, FMT, DEC_WIDE_KS>), g1, blk, 0, ctx->stream, ev[0], ev[1], 0, in.logits, in.bias, in.mask, a.x,
                            in.E, in.k, in.do_route, a.d_model, n_wg, n_se, a);
    else
      hipExtLaunchKernelGGL((gateup_kernel<ACT, SCB, FMT>), g1, blk, 0, ctx->stream, ev[0], ev[1], 0, in.logits, in.bias, in.mask, a.x,
                            in.E, in.k, in.do_route, a.d_model, n_wg, n_se, a);
    hipExtLaunchKernelGGL((down_kernel<ACT, SCB, FMT, RPW>), g2, blk, (unsigned)lds, ctx->stream, ev[2], ev[3], 0, recw, (const float*)a.h,
                          n_combo_s, n_pieces, psh, a.f_s, a.f_r, a.ks_s, a.ks_r, a.inv_ks_s, a.inv_ks_r, nsf, a);
  } else {
    if (wide && a.d_model <= 4096)
      gateup_wide_kernel<ACT, SCB, FMT, 2><<<g1, blk, 0, ctx->stream>>>(in.logits, in.bias, in.mask, a.x, in.E, in.k, in.do_route, a.d_model,
                                                                   n_wg, n_se, a);
    else if (wide)
      gateup_wide_kernel<ACT, SCB, FMT, DEC_WIDE_KS><<<g1, blk, 0, ctx->stream>>>(in.logits, in.bias, in.mask, a.x, in.E, in.k, in.do_route,
                                                                             a.d_model, n_wg, n_se, a);
    else
      gateup_kernel<ACT, SCB, FMT><<<g1, blk, 0, ctx->stream>>>(in.logits, in.bias, in.mask, a.x, in.E, in.k, in.do_route, a.d_model, n_wg, n_se,
                                                           a);
    down_kernel<ACT, SCB, FMT, RPW><<<g2, blk, lds, ctx->stream>>>(recw, (const float*)a.h, n_combo_s, n_pieces, psh, a.f_s, a.f_r, a.ks_s,
                                                         a.ks_r, a.inv_ks_s, a.inv_ks_r, nsf, a);
  }
  HIPCHK(ctx, hipGetLastError());
  return SMOE_OK;
}

// ws: device workspace of ws_bytes (routing records at WS_REC_OFF, SwiGLU vectors from WS_H_OFF on)
static int launch_decode(smoe_ctx* ctx, const smoe_bank* routed, const smoe_bank* shared, int act_dtype, int k,
                         RouteIn in, DecodeArgs& a, int T, uint8_t* ws, size_t ws_bytes) {
  if (!routed && !shared) return SMOE_EINVAL;
  if (routed && routed->device != ctx->device) return SMOE_EINVAL;
  if (shared && shared->device != ctx->device) return SMOE_EINVAL;
  if (routed && shared && routed->desc.d_model != shared->desc.d_model) return SMOE_ESHAPE;
  if (routed && shared && routed->dev.bits != shared->dev.bits) return SMOE_ENOTIMPL;          // one nest per layer
  if (!routed && k != 0) return SMOE_ESHAPE;
  if (routed && (k <= 0 || k > routed->desc.n_experts || k > SMOE_MAX_TOPK)) return SMOE_ESHAPE;
  if (routed && routed->desc.n_experts > SMOE_MAX_EXPERTS) return SMOE_ESHAPE;
  const int ns = shared ? shared->desc.n_experts : 0;
  if (k + ns > SMOE_MAX_SLOTS) return SMOE_ESHAPE;
  const int d_model = routed ? routed->desc.d_model : shared->desc.d_model;
  if (d_model > DEC_WIDE_MAX_D) return SMOE_ENOTIMPL;      // gate/up: at most four 64-chunk k-slices per row
  if (d_model % DEC_RPW) return SMOE_ESHAPE;
  a.f_r = routed ? routed->desc.d_ff : 0;
  a.f_s = shared ? shared->desc.d_ff : 0;
  const int total_f = k * a.f_r + ns * a.f_s;
  if ((size_t)total_f * 4 + WS_H_OFF > ws_bytes) return SMOE_ESIZE;
  if (T < 1 || T > SMOE_MAX_MULTI) return SMOE_ESHAPE;
  if (T > 1 && (size_t)T * DEC_H_STRIDE(ns * a.f_s, a.f_r) * 4 + WS_H_OFF > ws_bytes) return SMOE_ESIZE;
  a.gu_sh_r = a.dn_sh_r = routed ? ilog2_exact(routed->desc.group / 32) : 0;
  a.gu_sh_s = a.dn_sh_s = shared ? ilog2_exact(shared->desc.group / 32) : 0;
  if (a.gu_sh_r < 0 || a.gu_sh_s < 0) return SMOE_ENOTIMPL;   // group must be 32 * 2^n for the decode kernels
  if ((routed && !(routed->dev.gu.fits32 && routed->dev.dn.fits32)) || (shared && !(shared->dev.gu.fits32 && shared->dev.dn.fits32)))
    return SMOE_ENOTIMPL;                                      // decode kernels address a bank section with 32-bit offsets
  HIPCHK(ctx, hipSetDevice(ctx->device));
  auto matk = [](const MatDev& m) { return MatK{m.msb, m.lsb, m.zp, m.sc, m.ps32, m.zs32, m.ss32, m.ng, m.sng, 0}; };
  if (routed) { a.rgu = matk(routed->dev.gu); a.rdn = matk(routed->dev.dn); }
  if (shared) { a.sgu = matk(shared->dev.gu); a.sdn = matk(shared->dev.dn); }
  a.n_shared = ns; a.k = k;
  a.E = routed ? routed->desc.n_experts : 0;
  in.E = a.E; in.k = k;
  a.rec = (RouteRec*)(ws + WS_REC_OFF);
  a.h = (float*)(ws + WS_H_OFF);
  a.d_model = d_model;
  // gate/up split: n_wg work-groups, each takes ceil(f / n_wg) row pairs of every slot
  int n_wg = (total_f + DEC_NW - 1) / DEC_NW;              // at least one row pair per wave
  // Two 8-wave work-groups fit a CU: one token gets two per CU (measured best: 15.0 us per step against
  // 15.9 with one 16-wave work-group per CU and 16.3 - 17.5 with three, five, six or eight halves);
  // several tokens share them, and the work-groups of different tokens run side by side on a CU.
  int wg_cap = 2 * ctx->n_cu;
  if (T > 1) {      // about two per CU over all tokens (measured at 2 .. 16 tokens: better than four or eight per CU)
    wg_cap = ctx->n_cu;
    while (wg_cap > 8 && wg_cap * T > 2 * ctx->n_cu) wg_cap >>= 1;
  }
  n_wg = n_wg < 1 ? 1 : (n_wg > wg_cap ? wg_cap : n_wg);
  if (T > 1) n_wg = n_wg < 8 ? 8 : (n_wg & ~7);            // the multi-token grid is (8, T, n_wg / 8)
  a.cap_r = a.f_r ? (a.f_r + n_wg - 1) / n_wg : 1;
  a.cap_s = a.f_s ? (a.f_s + n_wg - 1) / n_wg : 1;
  a.inv_cap_r = fastdiv_magic(a.cap_r);
  a.inv_cap_s = fastdiv_magic(a.cap_s);
  // (several tokens: no rotation, so that tokens which hold an expert in different slots still read the
  // same rows of it in the same work-group index, i.e. on the same XCD, and share them in its L2)
  a.rot = T > 1 ? 0 : n_wg / (k + ns);
  if (ns * a.cap_s >= SMOE_FASTDIV_LIMIT || k * a.cap_r >= SMOE_FASTDIV_LIMIT) return SMOE_ESIZE;      // entry indices the exact division covers
  a.gu_L = (ns * a.cap_s + k * a.cap_r + DEC_NW - 1) / DEC_NW;
  // down split
  a.ks_r = a.f_r ? (a.f_r / 32 + 63) / 64 : 1;
  a.ks_s = a.f_s ? (a.f_s / 32 + 63) / 64 : 1;
  a.inv_ks_r = (int)fastdiv_magic(a.ks_r);
  a.inv_ks_s = (int)fastdiv_magic(a.ks_s);
  if (ns * a.ks_s >= SMOE_FASTDIV_LIMIT || k * a.ks_r >= SMOE_FASTDIV_LIMIT) return SMOE_ESIZE;
  const int scb = routed ? routed->dev.sc_bf16 : shared->dev.sc_bf16;
  if (routed && shared && routed->dev.sc_bf16 != shared->dev.sc_bf16) return SMOE_ENOTIMPL;   // one scale dtype per layer
  const int bits = routed ? routed->dev.bits : shared->dev.bits;
  // Several tokens per launch: a down work-group owns 8 * 2^n output rows, so that again about two
  // work-groups per CU cover all tokens (8 rows up to 2 tokens, 16 up to 4, 32 up to 8, 64 beyond): with
  // more, smaller work-groups each one pays its own start-up and rewrites h as digits for fewer rows.
  const bool rows16 = T >= 3 && d_model % 128 == 0, rows32 = T >= 6 && d_model % 256 == 0, rows64 = T >= 12 && d_model % 512 == 0;
#define DEC_LAUNCH(A, S, F) (rows64 ? launch_decode_t<A, S, F, 64>(ctx, in, a, n_wg, T) : rows32 ? launch_decode_t<A, S, F, 32>(ctx, in, a, n_wg, T) : rows16 ? launch_decode_t<A, S, F, 16>(ctx, in, a, n_wg, T) : launch_decode_t<A, S, F, DEC_RPW>(ctx, in, a, n_wg, T))
  if (bits == 2) {
    if (act_dtype == SMOE_F32) return scb ? DEC_LAUNCH(SMOE_F32, 1, 1) : DEC_LAUNCH(SMOE_F32, 0, 1);
    return scb ? DEC_LAUNCH(SMOE_BF16, 1, 1) : DEC_LAUNCH(SMOE_BF16, 0, 1);
  }
  if (bits == 3) {
    if (act_dtype == SMOE_F32) return scb ? DEC_LAUNCH(SMOE_F32, 1, 2) : DEC_LAUNCH(SMOE_F32, 0, 2);
    return scb ? DEC_LAUNCH(SMOE_BF16, 1, 2) : DEC_LAUNCH(SMOE_BF16, 0, 2);
  }
  if (act_dtype == SMOE_F32) return scb ? DEC_LAUNCH(SMOE_F32, 1, 0) : DEC_LAUNCH(SMOE_F32, 0, 0);
  return scb ? DEC_LAUNCH(SMOE_BF16, 1, 0) : DEC_LAUNCH(SMOE_BF16, 0, 0);
}

#undef DEC_LAUNCH

// Clears the hand-over words of the single-launch kernel (a kernel, not a memset: the call may sit in
// a stream that is being captured).
__global__ void one_sync_clear_kernel(unsigned* words) {
  for (int i = threadIdx.x; i < ONE_SYNC_WORDS; i += blockDim.x) words[i] = 0u;
}

extern "C" int smoe_ctx_single_launch(smoe_ctx* ctx, int enable, int spin_limit) {
  if (!ctx) return SMOE_EINVAL;
  if (!enable) { ctx->one_launch = 0; return SMOE_OK; }
  if (!ctx->ws || ctx->ws_bytes < (size_t)WS_H_OFF) return SMOE_ESIZE;
  if (spin_limit < 0) return SMOE_EINVAL;
  HIPCHK(ctx, hipSetDevice(ctx->device));
  one_sync_clear_kernel<<<1, 256, 0, ctx->stream>>>((unsigned*)(ctx->ws + WS_SYNC_OFF));
  HIPCHK(ctx, hipGetLastError());
  ctx->one_launch = 1;
  ctx->one_spin_limit = spin_limit ? spin_limit : (1 << 20);
  return SMOE_OK;
}

extern "C" int smoe_ctx_single_launch_status(smoe_ctx* ctx, long long* n_calls, unsigned* n_timeouts) {
  if (!ctx || !n_calls || !n_timeouts) return SMOE_EINVAL;
  *n_calls = ctx->one_calls;
  *n_timeouts = 0;
  if (!ctx->ws) return SMOE_OK;
  HIPCHK(ctx, hipSetDevice(ctx->device));
  HIPCHK(ctx, hipStreamSynchronize(ctx->stream));
  HIPCHK(ctx, hipMemcpy(n_timeouts, ctx->ws + WS_SYNC_OFF + 4 * ONE_TIMEOUTS, 4, hipMemcpyDeviceToHost));
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
  DecodeArgs a{};
  a.idx_in = idx_dev; a.w_in = w_dev; a.tau = tau_head;
  a.x = x_dev; a.shared_gate_w = shared_gate_w_dev; a.prec_out = prec_out_dev; a.y = y_dev; a.add_residual = add_residual;
  const RouteIn in{nullptr, nullptr, slice_mask_dev, 0, 0, 0};
  return launch_decode(ctx, routed, shared, act_dtype, k, in, a, 1, ctx->ws, ctx->ws_bytes);
}

static int decode_layer_impl(smoe_ctx* ctx, const smoe_bank* routed, const smoe_bank* shared, const void* x_dev,
                             int act_dtype, int k, const float* logits_dev, const float* w_router_dev,
                             const float* bias_dev, int norm_topk, float routed_scale,
                             const uint8_t* slice_mask_dev, float tau_head, const void* shared_gate_w_dev,
                             int add_residual, void* y_dev, int32_t* idx_out_dev, float* w_out_dev,
                             uint8_t* prec_out_dev, uint8_t* ws, size_t ws_bytes) {
  if (!ctx || !x_dev || !y_dev || x_dev == y_dev || !routed) return SMOE_EINVAL;
  if (act_dtype != SMOE_F32 && act_dtype != SMOE_BF16) return SMOE_EINVAL;
  if (!logits_dev && !w_router_dev) return SMOE_EINVAL;
  if (!aligned16(x_dev) || !aligned16(y_dev) || !aligned16(logits_dev) || !aligned16(w_router_dev) ||
      !aligned16(bias_dev) || !aligned16(shared_gate_w_dev))
    return SMOE_EALIGN;
  if (!ws || ws_bytes < (size_t)WS_H_OFF) return SMOE_ESIZE;
  const float* logits = logits_dev;
  if (!logits) {
    // router mat-vec into the workspace, then the gate/up prologue selects from those logits
    float* zws = (float*)(ws + WS_IDX_OFF);
    HIPCHK(ctx, hipSetDevice(ctx->device));
    int rc = smoe_launch_router_logits(ctx, routed->desc.n_experts, routed->desc.d_model, x_dev, act_dtype, w_router_dev, zws);
    if (rc) return rc;
    logits = zws;
  }
  DecodeArgs a{};
  a.norm_topk = norm_topk; a.routed_scale = routed_scale;
  a.tau = tau_head; a.x = x_dev; a.shared_gate_w = shared_gate_w_dev;
  const RouteIn in{logits, bias_dev, slice_mask_dev, 0, 0, 1};
  a.idx_out = idx_out_dev; a.w_out = w_out_dev; a.prec_out = prec_out_dev; a.y = y_dev; a.add_residual = add_residual;
  return launch_decode(ctx, routed, shared, act_dtype, k, in, a, 1, ws, ws_bytes);
}

extern "C" int smoe_decode_layer(smoe_ctx* ctx, const smoe_bank* routed, const smoe_bank* shared, const void* x_dev,
                                 int act_dtype, int k, const float* logits_dev, const float* w_router_dev,
                                 const float* bias_dev, int norm_topk, float routed_scale,
                                 const uint8_t* slice_mask_dev, float tau_head, const void* shared_gate_w_dev,
                                 int add_residual, void* y_dev, int32_t* idx_out_dev, float* w_out_dev,
                                 uint8_t* prec_out_dev) {
  if (!ctx) return SMOE_EINVAL;
  return decode_layer_impl(ctx, routed, shared, x_dev, act_dtype, k, logits_dev, w_router_dev, bias_dev, norm_topk, routed_scale,
                           slice_mask_dev, tau_head, shared_gate_w_dev, add_residual, y_dev, idx_out_dev, w_out_dev, prec_out_dev,
                           ctx->ws, ctx->ws_bytes);
}

extern "C" int smoe_decode_layer_multi(smoe_ctx* ctx, const smoe_bank* routed, const smoe_bank* shared, int T,
                                       const void* x_dev, int act_dtype, int k, const float* logits_dev,
                                       const float* bias_dev, int norm_topk, float routed_scale,
                                       const uint8_t* slice_mask_dev, float tau_head, const void* shared_gate_w_dev,
                                       int add_residual, void* y_dev, int32_t* idx_out_dev, float* w_out_dev,
                                       uint8_t* prec_out_dev) {
  if (!ctx || !x_dev || !y_dev || x_dev == y_dev || !routed || !logits_dev) return SMOE_EINVAL;
  if (act_dtype != SMOE_F32 && act_dtype != SMOE_BF16) return SMOE_EINVAL;
  if (T < 1 || T > SMOE_MAX_MULTI) return SMOE_ESHAPE;
  // token rows must keep the 16-byte alignment of the first one
  const int esz = act_dtype == SMOE_BF16 ? 2 : 4;
  if (T > 1 && (((size_t)routed->desc.d_model * esz) & 15u)) return SMOE_ESHAPE;
  if (!aligned16(x_dev) || !aligned16(y_dev) || !aligned16(logits_dev) || !aligned16(bias_dev) || !aligned16(shared_gate_w_dev))
    return SMOE_EALIGN;
  DecodeArgs a{};
  a.norm_topk = norm_topk; a.routed_scale = routed_scale;
  a.tau = tau_head; a.x = x_dev; a.shared_gate_w = shared_gate_w_dev;
  const RouteIn in{logits_dev, bias_dev, slice_mask_dev, 0, 0, 1};
  a.idx_out = idx_out_dev; a.w_out = w_out_dev; a.prec_out = prec_out_dev; a.y = y_dev; a.add_residual = add_residual;
  return launch_decode(ctx, routed, shared, act_dtype, k, in, a, T, ctx->ws, ctx->ws_bytes);
}

// ---------------------------------------------------------------------------------- no-allocation variant
// smoe_decode_layer for callers that cannot allocate device memory at all (code under HIP graph capture,
// serving loops or harnesses that forbid hipMalloc): the workspace of the call -- routing record,
// router logits, SwiGLU vectors -- is this file-scope device array instead of a caller buffer.  Every
// GPU the library runs on holds its own copy of the array, at its own address, until the process ends;
// in host code the array's name is only a handle, so the address is looked up once per device with
// hipGetSymbolAddress and only that pointer is ever handed to a kernel.
static __device__ __align__(256) uint8_t scratch[SMOE_STATIC_SCRATCH_BYTES];

#define SMOE_STATIC_MAX_DEVICES 64
static uint8_t* scratch_dev_ptr[SMOE_STATIC_MAX_DEVICES];      // per device; null until looked up
static std::mutex scratch_lock;

static int static_scratch(smoe_ctx* ctx, uint8_t** out) {
  if (ctx->device < 0 || ctx->device >= SMOE_STATIC_MAX_DEVICES) return SMOE_ESHAPE;
  std::lock_guard<std::mutex> guard(scratch_lock);
  if (!scratch_dev_ptr[ctx->device]) {
    HIPCHK(ctx, hipSetDevice(ctx->device));       // the lookup returns the copy of the current device
    void* p = nullptr;
    HIPCHK(ctx, hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p || (((uintptr_t)p) & 255u)) return SMOE_EALIGN;
    scratch_dev_ptr[ctx->device] = (uint8_t*)p;
  }
  *out = scratch_dev_ptr[ctx->device];
  return SMOE_OK;
}

extern "C" int smoe_static_scratch_bytes(size_t* bytes) {
  if (!bytes) return SMOE_EINVAL;
  *bytes = SMOE_STATIC_SCRATCH_BYTES;
  return SMOE_OK;
}

extern "C" int smoe_decode_layer_static(smoe_ctx* ctx, const smoe_bank* routed, const smoe_bank* shared, const void* x_dev,
                                        int act_dtype, int k, const float* logits_dev, const float* w_router_dev,
                                        const float* bias_dev, int norm_topk, float routed_scale,
                                        const uint8_t* slice_mask_dev, float tau_head, const void* shared_gate_w_dev,
                                        int add_residual, void* y_dev, int32_t* idx_out_dev, float* w_out_dev,
                                        uint8_t* prec_out_dev) {
  if (!ctx || !routed) return SMOE_EINVAL;
  // size check first, with a clear status: the intermediates of the layer must fit the array
  const size_t floats = (size_t)(k > 0 ? k : 0) * (size_t)routed->desc.d_ff +
                        (shared ? (size_t)shared->desc.n_experts * (size_t)shared->desc.d_ff : 0);
  if ((size_t)WS_H_OFF + floats * 4 > SMOE_STATIC_SCRATCH_BYTES) return SMOE_ESIZE;
  uint8_t* ws = nullptr;
  int rc = static_scratch(ctx, &ws);
  if (rc) return rc;
  // (the measurement aid of smoe_ctx_timing creates events: not in this entry point)
  const int timing = ctx->timing;
  ctx->timing = 0;
  rc = decode_layer_impl(ctx, routed, shared, x_dev, act_dtype, k, logits_dev, w_router_dev, bias_dev, norm_topk, routed_scale,
                         slice_mask_dev, tau_head, shared_gate_w_dev, add_residual, y_dev, idx_out_dev, w_out_dev, prec_out_dev,
                         ws, SMOE_STATIC_SCRATCH_BYTES);
  ctx->timing = timing;
  return rc;
}
