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

#if defined(__HIPCC__)
// Eight values -> eight codes in one word (element e in bits 4e+3..4e), the same codes as
// q_e2m1_code element by element, with the rounding done by the gfx950 FP4 convert, two values
// per instruction.  That instruction rounds to nearest, ties to even; the rule here is ties
// towards +inf.  The two differ only on exact ties, and a tie has a zero low mantissa bit, so:
// lower a negative value's magnitude by one ulp (as q_e2m1_code does: turns "towards +inf" into
// half-up on the magnitude), then set the lowest mantissa bit -- a tie becomes a hair more than
// a tie and rounds up, a value one ulp below a tie already has the bit set and stays below, no
// other value can cross a midpoint by one ulp.  The sign rides along, except that of a NaN
// (-> +6), and is dropped afterwards where the magnitude came out 0 (no -0).  Checked against
// q_e2m1_code on all 2^32 inputs in every position of the word.
FP4_D float q_e2m1_prepare(float v) {
  const uint32_t b = f2u(v);
  const uint32_t neg = ((b - 0x80000000u) <= 0x7f800000u) ? 1u : 0u;   // negative and not a NaN
  const uint32_t m = __builtin_elementwise_sub_sat(b & 0x7fffffffu, neg) | 1u;
  return u2f(m | (neg << 31));
}
// two prepared values -> byte BYTE of w (first value in the low nibble)
#define FP4_CVT_PAIR(w, a, b, BYTE) __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(w, a, b, 1.0f, BYTE)
// eight codes as the convert leaves them -> no sign on a zero magnitude
FP4_D uint32_t q_e2m1_drop_zero_signs(uint32_t w) {
  const uint32_t t = w & 0x77777777u;
  const uint32_t nz = ((t + 0x77777777u) | t) & 0x88888888u;   // bit 3 of every nibble whose magnitude is not 0
  return t | (w & nz);
}
FP4_D uint32_t q_e2m1_pack8(const float (&v)[8]) {
  uint32_t w = 0;
  w = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(w, q_e2m1_prepare(v[0]), q_e2m1_prepare(v[1]), 1.0f, 0);
  w = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(w, q_e2m1_prepare(v[2]), q_e2m1_prepare(v[3]), 1.0f, 1);
  w = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(w, q_e2m1_prepare(v[4]), q_e2m1_prepare(v[5]), 1.0f, 2);
  w = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(w, q_e2m1_prepare(v[6]), q_e2m1_prepare(v[7]), 1.0f, 3);
  return q_e2m1_drop_zero_signs(w);
}

// DGE factor min(cap, f'(x)) of one weight (Sec. 3.1 Eq. 8):
//   f'(x) = (1/k) |2(a-l)/delta - 1|^(1/k-1), a = |w * gamma|, [l, l+delta] the E2M1 interval
//   holding a: delta = .5 below 2, 1 below 4, 2 above (a rounding hair above 6 keeps [4, 6]).
// inv_k = 1/k, pw = 1/k - 1.  t == 0 with pw < 0: log2 = -inf -> exp2(+inf) = inf -> cap.
// pw == 0 (k = 1) is taken out: 0 * log2(0) would be NaN, and |t|^0 = 1 everywhere.
FP4_D float dge_factor(float w, float gamma, float pw, float inv_k, float cap) {
  const float a = fabsf(__fmul_rn(w, gamma));
  float l, s;
  if (a < 2.0f) { l = 0.5f * floorf(a + a); s = 4.0f; }
  else if (a < 4.0f) { l = floorf(a); s = 2.0f; }
  else { l = 4.0f; s = 1.0f; }
  const float t = fabsf(s * (a - l) - 1.0f);
  const float e = pw == 0.0f ? 1.0f : __builtin_amdgcn_exp2f(pw * __builtin_amdgcn_logf(t));
  return fminf(inv_k * e, cap);
}
#endif  // __HIPCC__

// Nearest E4M3 code (OCP FP8: bias 7, largest magnitude 448 = 0x7e, subnormal quantum 2^-9) of a
// finite fp32 value: ties to the even mantissa, sign kept, magnitudes above 448 saturate.  The
// 8-bit operand format of the mixed-format ablations (Sec. 4.3).
FP4_HD uint32_t q_e4m3_code(float v) {
  const uint32_t b = f2u(v);
  const uint32_t s = (b >> 24) & 0x80u;
  uint32_t a = b & 0x7fffffffu;
  if (a > 0x43e00000u) a = 0x43e00000u;                 // 448
  uint32_t code;
  if (a >= 0x3c800000u) {                               // >= 2^-6: a normal number of the format
    const uint32_t r = a + 0x7ffffu + ((a >> 20) & 1u); // nearest even at 3 mantissa bits; a carry moves the exponent
    code = (r >> 20) - (120u << 3);                     // exponent field re-biased from 127 to 7
  } else {                                              // below: multiples of 2^-9, 0 .. 8 (8 = the smallest normal)
#if defined(__HIP_DEVICE_COMPILE__)
    code = (uint32_t)__builtin_rintf(u2f(a) * 512.0f);
#else
    code = (uint32_t)__builtin_rintf(u2f(a) * 512.0f);  // default rounding mode: to nearest even
#endif
  }
  return code | s;
}

// gamma = fl32(fmax / amax) with fmax the largest magnitude of the target format; 1 for amax == 0 or a
// non-finite quotient.
FP4_HD float absmax_to_gamma_of(float amax, float fmax) {
#if defined(__HIP_DEVICE_COMPILE__)
  float g = __fdiv_rn(fmax, amax);
#else
  float g = fmax / amax;
#endif
  uint32_t gb = f2u(g) & 0x7fffffffu;
  return (amax > 0.0f && gb < 0x7f800000u) ? g : 1.0f;
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
