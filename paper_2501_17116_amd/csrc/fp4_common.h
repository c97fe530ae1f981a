// Shared device/host helpers for the FP4 linear kernels (gfx950).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "fp4_linear.h"

#if defined(__HIPCC__)
#define FP4_HD __host__ __device__ __forceinline__
#define FP4_D __device__ __forceinline__
#else
#define FP4_HD inline
#define FP4_D inline
#endif

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

FP4_HD uint32_t f2u(float f) {
  union { float f; uint32_t u; } c;
  c.f = f;
  return c.u;
}
FP4_HD float u2f(uint32_t u) {
  union { float f; uint32_t u; } c;
  c.u = u;
  return c.f;
}

// Nearest E2M1 code of an fp32 value, midpoints to the upper neighbour (towards +inf)
// for either sign, saturating, NaN -> +6 (the comparison chain of App. A, evaluated on
// the bit pattern).  On non-negative floats integer order equals value order, so the
// chain's strict '<' tests become integer tests on |v|; lowering a negative value's
// magnitude by one ulp first turns "tie goes towards +inf" into the positive rule.
//   |v| >= 1: one mantissa bit survives; add half of the dropped field and truncate.
//   |v| <  1: the grid is 0, .5, 1 -> two tests at .25 and .75.
FP4_HD uint32_t q_e2m1_code(float v) {
  uint32_t b = f2u(v);
  uint32_t ia = b & 0x7fffffffu;
  uint32_t s = b >> 31;
  if (ia > 0x7f800000u) s = 0;  // NaN: every comparison of the chain fails -> +6
  int32_t x = (int32_t)ia - (int32_t)s;
  // (x + 2^21 - (252 << 22)) >> 22 : exponent/mantissa field re-based so 1.0 -> 2
  int32_t mn = (x - 0x3EE00000) >> 22;
  int32_t ms = (x >= 0x3e800000 ? 1 : 0) + (x >= 0x3f400000 ? 1 : 0);
  int32_t m = mn > ms ? mn : ms;
  m = m < 7 ? m : 7;
  return m ? ((uint32_t)m | (s << 3)) : 0u;
}

// gamma = fl32(6 / amax); 1 for amax == 0 or a non-finite quotient.
FP4_HD float absmax_to_gamma(float amax) {
#if defined(__HIP_DEVICE_COMPILE__)
  float g = __fdiv_rn(6.0f, amax);
#else
  float g = 6.0f / amax;
#endif
  uint32_t gb = f2u(g) & 0x7fffffffu;
  return (amax > 0.0f && gb < 0x7f800000u) ? g : 1.0f;
}

FP4_HD float bf16_bits_to_f32(uint32_t h) { return u2f(h << 16); }

// fp32 -> bf16 bits, round to nearest even (finite inputs; NaN kept quiet).
FP4_HD uint32_t f32_to_bf16_bits(float f) {
  uint32_t u = f2u(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
  return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}

// Order-preserving map fp32 -> uint32 (ascending), and its 16-bit form for bf16 data.
FP4_HD uint32_t f32_order_key(uint32_t bits) {
  return (bits & 0x80000000u) ? ~bits : (bits | 0x80000000u);
}
FP4_HD uint32_t f32_from_order_key(uint32_t key) {
  return (key & 0x80000000u) ? (key & 0x7fffffffu) : ~key;
}

#define FP4_CHECK_LAUNCH()                                   \
  do {                                                       \
    if (hipGetLastError() != hipSuccess) return FP4_ERR_HIP; \
  } while (0)

static inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
static inline bool aligned16(const void* p) { return (((uintptr_t)p) & 15u) == 0; }
