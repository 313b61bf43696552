// Device-side extraction of bit-packed codes (layout.h) into fp16 operand fields.
//
// A "field" is a pair of codes (one per 16-bit half of a dword) sitting somewhere inside the 10
// mantissa bits of an fp16 whose exponent bits are zero: a subnormal with the exact value
// code * 2^-(14+BITS) * 2^-(class * kStepBits).  The class says how far below the top of the
// mantissa the code sits.  Because the value is exact whatever the class, a field needs no shift
// to a common position: fma(field, scale * 2^(class * kStepBits), c) dequantizes it, and the
// kernels keep one pre-multiplied scale per class.  Only the codes stored above bit 9 of a half
// need one shift to come down into the mantissa.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "layout.h"

namespace lrc {

template <int BITS> struct Extract;

// field(w, 4*s+v) is operand register v of MFMA sub-step s (see layout.h)
template <> struct Extract<2> {
  static constexpr int kClasses = 3, kStepBits = 2;
  // field offset 2*i inside a half, i = pair % 8
  __host__ __device__ static constexpr int cls(int pair) {
    constexpr int t[8] = {2, 1, 2, 1, 0, 2, 1, 0};
    return t[pair % 8];
  }
  // `pair` is a compile-time constant after unrolling, so the switch folds away
  __device__ static inline uint32_t field(const uint32_t (&w)[4], int pair) {
    const uint32_t v = w[pair / 8];
    switch (pair % 8) {
      case 0: return (v << 4) & 0x00300030u;   // offset 0  -> 4  (class 2)
      case 1: return (v << 4) & 0x00C000C0u;   // offset 2  -> 6  (class 1)
      case 2: return v & 0x00300030u;          // offset 4        (class 2)
      case 3: return v & 0x00C000C0u;          // offset 6        (class 1)
      case 4: return v & 0x03000300u;          // offset 8        (class 0)
      case 5: return (v >> 6) & 0x00300030u;   // offset 10 -> 4  (class 2)
      case 6: return (v >> 6) & 0x00C000C0u;   // offset 12 -> 6  (class 1)
      default: return (v >> 6) & 0x03000300u;  // offset 14 -> 8  (class 0)
    }
  }
};

template <> struct Extract<3> {
  static constexpr int kClasses = 3, kStepBits = 3;
  // pairs 0..29: field offset 1 + 3*(pair % 5); pairs 30, 31 are assembled at the top (class 0)
  __host__ __device__ static constexpr int cls(int pair) {
    constexpr int t[5] = {2, 1, 0, 1, 0};
    return pair >= 30 ? 0 : t[pair % 5];
  }
  __device__ static inline uint32_t field(const uint32_t (&w)[6], int pair) {
    if (pair >= 30) {                          // spare bit 0 of each half of dwords 3t..3t+2
      const int t = pair - 30;
      return ((w[3 * t] << 7) & 0x00800080u) | ((w[3 * t + 1] << 8) & 0x01000100u) |
             ((w[3 * t + 2] << 9) & 0x02000200u);
    }
    const uint32_t v = w[pair / 5];
    switch (pair % 5) {
      case 0: return v & 0x000E000Eu;          // offset 1        (class 2)
      case 1: return v & 0x00700070u;          // offset 4        (class 1)
      case 2: return v & 0x03800380u;          // offset 7        (class 0)
      case 3: return (v >> 6) & 0x00700070u;   // offset 10 -> 4  (class 1)
      default: return (v >> 6) & 0x03800380u;  // offset 13 -> 7  (class 0)
    }
  }
};

template <> struct Extract<4> {
  static constexpr int kClasses = 4, kStepBits = 2;
  // field offset 4*i inside a half, i = pair % 4
  __host__ __device__ static constexpr int cls(int pair) {
    constexpr int t[4] = {3, 1, 2, 0};
    return t[pair % 4];
  }
  __device__ static inline uint32_t field(const uint32_t (&w)[8], int pair) {
    const uint32_t v = w[pair / 4];
    switch (pair % 4) {
      case 0: return v & 0x000F000Fu;          // offset 0        (class 3)
      case 1: return v & 0x00F000F0u;          // offset 4        (class 1)
      case 2: return (v >> 6) & 0x003C003Cu;   // offset 8  -> 2  (class 2)
      default: return (v >> 6) & 0x03C003C0u;  // offset 12 -> 6  (class 0)
    }
  }
};

// integer code of one half of a field (for the unpack hook)
template <int BITS>
__device__ inline uint32_t field_code(uint32_t half16, int pair) {
  return half16 >> (10 - BITS - Extract<BITS>::cls(pair) * Extract<BITS>::kStepBits);
}

template <int BITS>
__device__ inline void load_codes(const uint32_t* __restrict__ tile, int lane, uint32_t (&w)[2 * BITS]) {
  const uint4 a = reinterpret_cast<const uint4*>(tile)[lane];
  w[0] = a.x; w[1] = a.y; w[2] = a.z; w[3] = a.w;
  if constexpr (BITS == 3) {
    const uint2 b = reinterpret_cast<const uint2*>(tile + 256)[lane];
    w[4] = b.x; w[5] = b.y;
  } else if constexpr (BITS == 4) {
    const uint4 b = reinterpret_cast<const uint4*>(tile + 256)[lane];
    w[4] = b.x; w[5] = b.y; w[6] = b.z; w[7] = b.w;
  }
}

}  // namespace lrc
