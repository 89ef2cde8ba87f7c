// AMAT quantise + slice (paper Section 4.2 and its equation; Table 1 note 1).
//
// One work-group per destination row, one wavefront per quantisation group.  All arithmetic
// that decides an integer (scale, zero-point, code) is plain IEEE fp32 with round-to-nearest-
// even, no fused multiply-add and true division, so codes are reproducible bit for bit.
#include "common.hpp"

#pragma clang fp contract(off)

template <int WDT> __device__ __forceinline__ float load_w(const void* p, size_t i) {
  if (WDT == SMOE_F32) return ((const float*)p)[i];
  return bf16_bits_to_f32(((const uint16_t*)p)[i]);
}

__device__ __forceinline__ float wave_min(float v) {
  for (int m = 32; m >= 1; m >>= 1) v = fminf(v, __shfl_xor(v, m));
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
  for (int m = 32; m >= 1; m >>= 1) v = fmaxf(v, __shfl_xor(v, m));
  return v;
}

// w0/w1: source matrices of the n experts being converted ([n, N/2, K] each when `interleave`,
// else w0 is [n, N, K]).  Destination family `m` already points at expert 0 of the bank.
template <int WDT>
__global__ __launch_bounds__(256) void quantize_rows_kernel(const void* __restrict__ w0, const void* __restrict__ w1,
                                                            MatDev m, int e0, int group, int sc_bf16, int interleave, int symmetric) {
  const int row = blockIdx.x, el = blockIdx.y, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int K = m.K, ng = m.ng;
  const void* src;
  size_t src_row;
  if (interleave) {
    src = (row & 1) ? w1 : w0;
    src_row = (size_t)el * (m.N / 2) + (row >> 1);
  } else {
    src = w0;
    src_row = (size_t)el * m.N + row;
  }
  const size_t sbase = src_row * (size_t)K;
  const size_t e = (size_t)(e0 + el);
  const int bits = m.bits;                             // 4: 8-bit codes, nibble planes; 3: 6-bit codes; 2: 4-bit codes, 2-bit planes
  const float qmax = bits == 4 ? 255.0f : bits == 3 ? 63.0f : 15.0f;
  uint8_t* pm = const_cast<uint8_t*>(m.msb) + e * m.plane_stride + (size_t)row * (K * bits / 8);
  uint8_t* pl = const_cast<uint8_t*>(m.lsb) + e * m.plane_stride + (size_t)row * (K * bits / 8);
  uint8_t* pz = const_cast<uint8_t*>(m.zp) + e * m.zp_stride + (size_t)row * ng;
  uint8_t* ps = const_cast<uint8_t*>(m.sc) + e * m.sc_stride;

  for (int g = wave; g < ng; g += 4) {
    const int k0 = g * group;
    const int gsz = min(group, K - k0);
    const int np = gsz >> 1;
    float lo = 0.0f, hi = 0.0f;                       // the range always contains 0
    for (int p = lane; p < np; p += 64) {
      const float a = load_w<WDT>(src, sbase + k0 + 2 * p), b = load_w<WDT>(src, sbase + k0 + 2 * p + 1);
      lo = fminf(lo, fminf(a, b));
      hi = fmaxf(hi, fmaxf(a, b));
    }
    lo = wave_min(lo);
    hi = wave_max(hi);
    // symmetric variant (Section 6.1 item 1: symmetric integer weights): step from the largest magnitude, the
    // zero-point fixed at mid-range of the unsigned store
    const float half = 0.5f * (qmax + 1.0f);
    float s = symmetric ? fmaxf(hi, -lo) / (half - 1.0f) : (hi - lo) / qmax;
    if (sc_bf16) s = bf16_bits_to_f32(f32_to_bf16_bits(s));
    if (!(s > 0.0f)) s = 1.0f;
    const int zp = symmetric ? (int)half : (int)fminf(fmaxf(rintf((-lo) / s), 0.0f), qmax);
    if (bits == 3) {
      // 6-bit codes: upper three bits = the low-bit code.  A plane keeps the 32 three-bit values of a
      // chunk of 32 columns in 12 bytes, laid out so that a nibble word (one value per nibble, columns
      // 8t .. 8t+7 in word t) comes out of it with a shift and a mask: column 8t + j has its two low
      // bits in word t >> 1 at bits 4j + 2(t & 1), 4j + 2(t & 1) + 1 and its third bit in word 2 at
      // bit 4j + t.  Eight lanes build a chunk: lane j of them takes the columns 8t + j.
      const int nchunk = gsz >> 5, j = lane & 7;
      for (int cb = 0; cb < nchunk; cb += 8) {
        const int c = cb + (lane >> 3);
        uint32_t wm[3] = {0, 0, 0}, wl[3] = {0, 0, 0};
        if (c < nchunk) {
#pragma unroll
          for (int t = 0; t < 4; t++) {
            const float a = load_w<WDT>(src, sbase + k0 + 32 * c + 8 * t + j);
            const int q = min(max((int)rintf(a / s) + zp, 0), 63);
            const uint32_t mv = (uint32_t)q >> 3, lv = (uint32_t)q & 7u;
            wm[t >> 1] |= (mv & 3u) << (4 * j + 2 * (t & 1));
            wl[t >> 1] |= (lv & 3u) << (4 * j + 2 * (t & 1));
            wm[2] |= (mv >> 2) << (4 * j + t);
            wl[2] |= (lv >> 2) << (4 * j + t);
          }
        }
#pragma unroll
        for (int i = 0; i < 3; i++)
          for (int x = 1; x < 8; x <<= 1) {
            wm[i] |= (uint32_t)__shfl_xor((int)wm[i], x);
            wl[i] |= (uint32_t)__shfl_xor((int)wl[i], x);
          }
        if (c < nchunk && j == 0) {
          uint32_t* dm = (uint32_t*)(pm + (size_t)((k0 >> 5) + c) * 12);
          uint32_t* dl = (uint32_t*)(pl + (size_t)((k0 >> 5) + c) * 12);
#pragma unroll
          for (int i = 0; i < 3; i++) { dm[i] = wm[i]; dl[i] = wl[i]; }
        }
      }
    } else if (bits == 2) {
      // 4-bit codes: upper two bits = the low-bit code; four codes per plane byte, column 4j in bits 0-1
      for (int p = lane; p < (gsz >> 2); p += 64) {
        int bm = 0, bl = 0;
#pragma unroll
        for (int c = 0; c < 4; c++) {
          const float a = load_w<WDT>(src, sbase + k0 + 4 * p + c);
          const int q = min(max((int)rintf(a / s) + zp, 0), 15);
          bm |= (q >> 2) << (2 * c);
          bl |= (q & 3) << (2 * c);
        }
        pm[(k0 >> 2) + p] = (uint8_t)bm;
        pl[(k0 >> 2) + p] = (uint8_t)bl;
      }
    } else
    for (int p = lane; p < np; p += 64) {
      const float a = load_w<WDT>(src, sbase + k0 + 2 * p), b = load_w<WDT>(src, sbase + k0 + 2 * p + 1);
      const int qa = min(max((int)rintf(a / s) + zp, 0), 255);
      const int qb = min(max((int)rintf(b / s) + zp, 0), 255);
      // planes keep every nibble n as n - 8 in 4-bit two's complement (n ^ 8): signed 4-bit dot products
      // read them directly
      pm[(k0 >> 1) + p] = (uint8_t)(((qa >> 4) | (qb & 0xF0)) ^ 0x88);          // floor(q/16): the low-bit code
      pl[(k0 >> 1) + p] = (uint8_t)(((qa & 15) | ((qb & 15) << 4)) ^ 0x88);     // the bits truncation drops
    }
    if (lane == 0) {
      pz[g] = (uint8_t)zp;
      const size_t si = (size_t)row * m.sng + g;
      if (sc_bf16) ((uint16_t*)ps)[si] = (uint16_t)f32_to_bf16_bits(s);
      else ((float*)ps)[si] = s;
    }
  }
}

int smoe_launch_quantize(smoe_ctx* ctx, smoe_bank* bank, int e0, int n, const void* wg, const void* wu, const void* wd) {
  const BankDev& b = bank->dev;
  HIPCHK(ctx, hipSetDevice(ctx->device));
  dim3 blk(256);
  if (bank->desc.w_dtype == SMOE_F32) {
    quantize_rows_kernel<SMOE_F32><<<dim3(b.gu.N, n), blk, 0, ctx->stream>>>(wg, wu, b.gu, e0, b.group, b.sc_bf16, 1, bank->desc.symmetric);
    quantize_rows_kernel<SMOE_F32><<<dim3(b.dn.N, n), blk, 0, ctx->stream>>>(wd, nullptr, b.dn, e0, b.group, b.sc_bf16, 0, bank->desc.symmetric);
  } else {
    quantize_rows_kernel<SMOE_BF16><<<dim3(b.gu.N, n), blk, 0, ctx->stream>>>(wg, wu, b.gu, e0, b.group, b.sc_bf16, 1, bank->desc.symmetric);
    quantize_rows_kernel<SMOE_BF16><<<dim3(b.dn.N, n), blk, 0, ctx->stream>>>(wd, nullptr, b.dn, e0, b.group, b.sc_bf16, 0, bank->desc.symmetric);
  }
  HIPCHK(ctx, hipGetLastError());
  return SMOE_OK;
}
