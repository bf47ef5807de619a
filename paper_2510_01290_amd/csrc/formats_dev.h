// Encoders of the paper's number formats (appendix "Quantization Data Formats"): E4M3, E2M1, ternary, and the
// E4M3 group scale.  The arithmetic is binary64 and decision by decision that of the definition: the ratio of
// an element to its scale is one IEEE division, the nearest code is found by exact scaling and round-to-nearest-
// even, so the codes do not depend on who computes them.
#pragma once
#include "common.h"

namespace thinkv {

// nearest code magnitude (ties to the even code, saturating at max_code) of a >= 0 in a format with man_bits
// mantissa bits whose smallest normal number is 2^emin: codes 0 .. 2^man_bits are the multiples of
// 2^(emin - man_bits) up to 2^emin, then every binade has 2^man_bits codes
__device__ inline int minifloat_nearest(double a, int man_bits, int emin, int max_code, double max_val) {
  if (!(a < max_val)) return max_code;
  const int one = 1 << man_bits;
  if (a < ldexp(1.0, emin)) return (int)rint(ldexp(a, man_bits - emin));
  int E = ilogb(a);
  int k = (int)rint(ldexp(a, man_bits - E));   // one .. 2 * one
  if (k == 2 * one) {
    ++E;
    k = one;
  }
  const int code = ((E - emin + 1) << man_bits) | (k - one);
  return code > max_code ? max_code : code;
}

__device__ inline uint32_t e4m3_encode(double r) {   // nearest E4M3 code of r; the sign bit follows the sign of r
  return (uint32_t)minifloat_nearest(fabs(r), 3, -6, 126, 448.0) | (signbit(r) ? 0x80u : 0u);
}
__device__ inline uint32_t e2m1_encode(double r) {   // the sign is dropped from a zero
  const int m = minifloat_nearest(fabs(r), 1, 0, 7, 6.0);
  return (uint32_t)m | ((signbit(r) && m != 0) ? 8u : 0u);
}
__device__ inline uint32_t ternary_encode(double r) {
  const uint32_t m = fabs(r) > 0.5 ? 1u : 0u;
  return (r < 0.0 && m) ? 3u : m;
}

// smallest E4M3 code whose value is >= t (t >= 0; 448 at most): the scale of a group
__device__ inline uint32_t e4m3_code_up(double t) {
  if (!(t > 0.0)) return 0u;
  if (t >= 448.0) return 126u;
  if (t < 0.015625) return (uint32_t)ceil(ldexp(t, 9));
  int E = ilogb(t);
  int k = (int)ceil(ldexp(t, 3 - E));   // 8 .. 16
  if (k == 16) {
    ++E;
    k = 8;
  }
  const uint32_t code = (uint32_t)(((E + 7) << 3) | (k - 8));
  return code > 126u ? 126u : code;
}

}  // namespace thinkv
