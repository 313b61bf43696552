// fp64 <-> fp16 conversions of the offline quantizer, as integer arithmetic that gives the same
// bits on the host and on the device: one rounding to nearest, ties to even, straight from the
// 53-bit significand (a conversion through fp32 would round twice).
#pragma once
#include <stdint.h>
#include <string.h>

#include "layout.h"

namespace lrc {

LRC_HD uint16_t f64_to_f16_bits(double v) {
  uint64_t b;
  memcpy(&b, &v, 8);
  const uint16_t sign = uint16_t((b >> 48) & 0x8000u);
  const int e = int((b >> 52) & 0x7ff);
  const uint64_t m = b & ((uint64_t(1) << 52) - 1);
  if (e == 0x7ff) return uint16_t(sign | 0x7c00u | (m ? 0x200u : 0u));       // infinity, NaN
  if (e == 0) return sign;                                                    // zero and fp64 subnormals
  const int ue = e - 1023;
  if (ue > 15) return uint16_t(sign | 0x7c00u);
  const uint64_t mant = m | (uint64_t(1) << 52);                              // 1.m as a 53-bit integer
  // normal fp16 results keep 11 significant bits; below 2^-14 the unit is fixed at 2^-24
  const int shift = ue >= -14 ? 42 : 42 + (-14 - ue);
  if (shift > 63) return sign;
  uint64_t keep = mant >> shift;
  const uint64_t rem = mant & ((uint64_t(1) << shift) - 1), half = uint64_t(1) << (shift - 1);
  if (rem > half || (rem == half && (keep & 1))) ++keep;
  uint32_t out;
  if (ue >= -14) out = (uint32_t(ue + 15) << 10) + uint32_t(keep - 1024);     // (a carry out of the significand bumps the exponent)
  else out = uint32_t(keep);                                                  // (and a subnormal that rounds up to 2^-14 becomes normal)
  if (out >= 0x7c00u) out = 0x7c00u;
  return uint16_t(sign | out);
}

LRC_HD double f16_bits_to_f64(uint16_t h) {
  const int e = (h >> 10) & 0x1f;
  const uint64_t m = h & 0x3ffu, sign = uint64_t(h & 0x8000u) << 48;
  uint64_t b;
  if (e == 0x1f) {
    b = sign | (uint64_t(0x7ff) << 52) | (m << 42);
  } else if (e != 0) {
    b = sign | (uint64_t(e - 15 + 1023) << 52) | (m << 42);
  } else if (m == 0) {
    b = sign;
  } else {                                           // subnormal: m * 2^-24, normalised
    int k = 0;
    uint64_t mm = m;
    while (!(mm & 0x400u)) { mm <<= 1; ++k; }
    b = sign | (uint64_t(-14 - k + 1023) << 52) | ((mm & 0x3ffu) << 42);
  }
  double v;
  memcpy(&v, &b, 8);
  return v;
}

}  // namespace lrc
