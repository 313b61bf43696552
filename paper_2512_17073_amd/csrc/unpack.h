// Device-side extraction of bit-packed codes (layout.h) into fp16 operand fields.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "layout.h"

namespace lrc {

// ---- code extraction: dwords of one lane -> 32 pairs of fields, pair 4*s+v = operand register v
// of sub-step s.  A field is the code placed at the top of an fp16 mantissa (bits 9..10-BITS) with
// zero exponent, i.e. the subnormal code * 2^-(14+BITS).
template <int BITS> struct Extract;

template <> struct Extract<2> {
  static constexpr uint32_t kMask = 0x03000300u;
  __device__ static inline void run(const uint32_t (&w)[4], uint32_t (&f)[32]) {
#pragma unroll
    for (int d = 0; d < 4; ++d)
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const uint32_t t = i < 4 ? (w[d] << (8 - 2 * i)) : (w[d] >> (2 * i - 8));
        f[8 * d + i] = t & kMask;
      }
  }
};

template <> struct Extract<4> {
  static constexpr uint32_t kMask = 0x03C003C0u;
  __device__ static inline void run(const uint32_t (&w)[8], uint32_t (&f)[32]) {
#pragma unroll
    for (int d = 0; d < 8; ++d)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const uint32_t t = i < 2 ? (w[d] << (6 - 4 * i)) : (w[d] >> (4 * i - 6));
        f[4 * d + i] = t & kMask;
      }
  }
};

template <> struct Extract<3> {
  static constexpr uint32_t kMask = 0x03800380u;
  __device__ static inline void run(const uint32_t (&w)[6], uint32_t (&f)[32]) {
#pragma unroll
    for (int d = 0; d < 6; ++d)
#pragma unroll
      for (int i = 0; i < 5; ++i) {
        // field offset 1 + 3*i in each half, wanted at offset 7
        const int sh = 7 - (1 + 3 * i);
        const uint32_t t = sh >= 0 ? (w[d] << sh) : (w[d] >> (-sh));
        f[5 * d + i] = t & kMask;
      }
#pragma unroll
    for (int t = 0; t < 2; ++t)   // pairs 30, 31 from the spare bit 0 of each half
      f[30 + t] = ((w[3 * t] << 7) & 0x00800080u) | ((w[3 * t + 1] << 8) & 0x01000100u) |
                  ((w[3 * t + 2] << 9) & 0x02000200u);
  }
};

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
