// Exact division of a small index by a launch constant, as one multiply-high.
//
// The decode kernels deal the (slot, position) entries of a work-group to waves by index e and need
// slot = floor(e / cap), position = e - slot * cap, with cap fixed per launch.  For n < 2^15 and
// d < 2^15, floor(n / d) = (n * ceil(2^32 / d)) >> 32 exactly (the error term n * (ceil(2^32/d) * d -
// 2^32) stays below 2^32), and floor(e / cap) = floor((2e + 1) / (2 cap)), which keeps the constant
// ceil(2^31 / cap) inside 32 bits for cap = 1 as well.  Valid for 0 <= e < 2^14, 1 <= cap < 2^14.
#pragma once
#include <stdint.h>

#define SMOE_FASTDIV_LIMIT (1 << 14)

#ifdef __HIPCC__
#define SMOE_HD __host__ __device__ __forceinline__
#else
#define SMOE_HD static inline
#endif

SMOE_HD uint32_t fastdiv_magic(int cap) { return (uint32_t)((((uint64_t)1 << 31) + (uint64_t)cap - 1) / (uint64_t)cap); }

SMOE_HD int fastdiv(int e, uint32_t magic) {
#ifdef __HIP_DEVICE_COMPILE__
  return (int)__umulhi(2u * (uint32_t)e + 1u, magic);
#else
  return (int)(((uint64_t)(2u * (uint32_t)e + 1u) * (uint64_t)magic) >> 32);
#endif
}
