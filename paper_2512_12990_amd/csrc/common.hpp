// Internal declarations shared by the library's translation units (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include "../../include/slicemoe.h"

#define SMOE_MAX_SLOTS 24      // top-k (<= 16) routed + up to 8 shared experts
#define SMOE_MAX_EXPERTS 256
#define SMOE_MAX_MULTI 16          // tokens of one smoe_decode_layer_multi call
#define SMOE_MAX_TOPK 16
#define SMOE_STATIC_SCRATCH_BYTES (512u << 10)   // the file-scope workspace of smoe_decode_layer_static

// ---- host objects -------------------------------------------------------------------------
// Device view of one quantised matrix family inside a bank ("gu": gate and up rows interleaved,
// row 2r = gate r, row 2r+1 = up r, shape [2*d_ff, d_model]; "dn": down, [d_model, d_ff]).
// Per expert e the data starts at base + e * stride.  Planes of the 8/4 nest hold two 4-bit values
// per byte, row-major, low nibble = even column, each value n stored as n ^ 8 (= n - 8 in 4-bit two's
// complement); the 4/2 nest keeps four 2-bit values per byte (column 4j in bits 0-1) and the 6/3 nest
// 32 three-bit values per 12 bytes (layout in quantize.hip), both as plain unsigned values.  Metadata: zp uint8 [N, ng], scale [N, sng] (the first ng of a row are used).
struct MatDev {
  const uint8_t* msb; const uint8_t* lsb; const uint8_t* zp; const uint8_t* sc;
  unsigned long long plane_stride, zp_stride, sc_stride;   // bytes per expert
  int N, K, ng, cpg;                                       // cpg = 32-column chunks per group
  int bits;                                                // bits per code in a plane: 4 (8/4 nest), 3 (6/3) or 2 (4/2)
  int sng;                                                 // scales per row as stored: ng rounded up to even, so that
                                                           // every row of scales starts on a 4-byte boundary
  unsigned ps32, zs32, ss32, fits32;                       // the strides as 32-bit numbers; fits32 = every
                                                           // byte offset inside a section is below 2^31
};

struct BankDev {
  MatDev gu, dn;
  int n_experts, d_model, d_ff, group, sc_bf16;
  int bits;             // plane bits per code (4: 8-bit codes of nibble planes; 3: 6-bit codes; 2: 4-bit codes)
};

struct smoe_ctx {
  int device;
  hipStream_t stream;
  uint8_t* ws;          // the caller's device workspace (borrowed): routing records, router logits, SwiGLU vectors
  size_t ws_bytes;
  int last_hip;
  int n_cu;
  // measurement aid (smoe_ctx_timing): events around the two decode launches of every call
  int timing;
  void* timing_events;   // std::vector<hipEvent_t>*, four events per decode call
  size_t down_lds_granted[48];   // dynamic LDS already granted to each down_kernel instantiation on this device
  size_t route_lds_granted[2];   // likewise for route_batch_kernel (bf16, fp32 activations)
  // single-launch decode (smoe_ctx_single_launch)
  int one_launch;                // the mode is on
  int one_spin_limit;            // polls before a work-group gives up waiting for the others
  long long one_calls;           // decode calls that took the single launch
  int one_blocks_per_cu[12];     // resident work-groups per CU of each decode_one_kernel instantiation (0: not asked yet, -1: none)
  size_t one_lds_seen[12];       // dynamic LDS that figure was asked for
};

struct smoe_bank {
  smoe_bank_desc desc;
  BankDev dev;          // device pointers are non-const views of `store`
  uint8_t* store;
  size_t store_bytes;
  int device;
};

// ---- per-token routing record (device): written by the gate/up kernel, read by the down kernel
struct RouteRec {
  int sel[SMOE_MAX_TOPK];     // selected expert of every slot
  int prec[SMOE_MAX_TOPK];    // 1 = HIGH (MSB+LSB), 0 = LOW (MSB only)
  float w[SMOE_MAX_TOPK];     // gate weights
  float gamma;                // weight of the shared experts
  int pad[15];
};

// workspace layout (offsets in bytes)
#define WS_REC_OFF 0                         // RouteRec
#define WS_SYNC_OFF (8 << 10)                // hand-over words of the single-launch decode kernel (parity, timeouts, two flag arrays)
#define WS_IDX_OFF (16 << 10)                // routing scratch of smoe_decode_layer without given logits
#define WS_H_OFF (64 << 10)                  // float h[total_f]

#define HIPCHK(ctx, expr)                                  \
  do {                                                     \
    hipError_t _e = (expr);                                \
    if (_e != hipSuccess) { (ctx)->last_hip = (int)_e; return SMOE_EHIP; } \
  } while (0)

static inline bool aligned16(const void* p) { return (((uintptr_t)p) & 15u) == 0; }

// ---- device helpers ---------------------------------------------------------------------------
#ifdef __HIPCC__
__device__ __forceinline__ float bf16_bits_to_f32(uint32_t h) { return __uint_as_float(h << 16); }

// round-to-nearest-even fp32 -> bf16 bits (finite inputs)
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

template <int ACT> __device__ __forceinline__ float load_act(const void* p, size_t i) {
  if (ACT == SMOE_F32) return ((const float*)p)[i];
  return bf16_bits_to_f32(((const uint16_t*)p)[i]);
}
template <int ACT> __device__ __forceinline__ void store_act(void* p, size_t i, float v) {
  if (ACT == SMOE_F32) ((float*)p)[i] = v;
  else ((uint16_t*)p)[i] = (uint16_t)f32_to_bf16_bits(v);
}

template <int CTRL> __device__ __forceinline__ float dpp_f32(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, true));
}

// Sum over the 64 lanes of a wavefront; every lane of the wave must call it.  The total is
// returned in all lanes (DPP within rows of 16, then the four row totals are read out).
__device__ __forceinline__ float wave_sum(float v) {
  v += dpp_f32<0xB1>(v);     // quad_perm [1,0,3,2]
  v += dpp_f32<0x4E>(v);     // quad_perm [2,3,0,1]
  v += dpp_f32<0x124>(v);    // row_ror 4
  v += dpp_f32<0x128>(v);    // row_ror 8
  float r0 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 0));
  float r1 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 16));
  float r2 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 32));
  float r3 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 48));
  return (r0 + r1) + (r2 + r3);
}
#endif

// launchers implemented in the .hip files
int smoe_launch_quantize(smoe_ctx* ctx, smoe_bank* bank, int e0, int n, const void* wg, const void* wu, const void* wd);
int smoe_launch_router_logits(smoe_ctx* ctx, int E, int d, const void* x, int act_dtype, const float* w_router, float* z);
struct RouteArgs;
int smoe_launch_route(smoe_ctx* ctx, const RouteArgs& a, int T, int act_dtype);
