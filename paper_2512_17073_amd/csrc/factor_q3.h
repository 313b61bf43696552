// Device-side dequantization of factor units held at 3 bits (layout.h) into fp16 MFMA operands,
// where the units are consumed (Section 3.1 step 2: the factor pairs are stored at INT3).
#pragma once
#include "ffn_common.h"

namespace lrc {
namespace ffn {

// Element pair i (elements 2 i and 2 i + 1 of a lane's eight) as two fp16 subnormals with the codes
// in mantissa bits 7..9: value code * 2^-17 each.
template <int I> __host__ __device__ inline uint32_t q3_field(uint32_t v) {
  if constexpr (I == 0) return (v << 7) & 0x03800380u;
  else if constexpr (I == 1) return (v << 4) & 0x03800380u;
  else if constexpr (I == 2) return (v << 1) & 0x03800380u;
  else return (v >> 2) & 0x03800380u;
}

// A-factor unit: all eight elements share (scale, zero); meta = lo | hi << 16 (layout.h)
__device__ inline half8_t q3_unit_a(uint32_t codes, uint32_t meta) {
  const uint32_t S = (meta & 0xffffu) | (meta << 16), C = (meta >> 16) | (meta & 0xffff0000u);
  return __builtin_bit_cast(half8_t, make_uint4(pk_fma(q3_field<0>(codes), S, C), pk_fma(q3_field<1>(codes), S, C),
                                                pk_fma(q3_field<2>(codes), S, C), pk_fma(q3_field<3>(codes), S, C)));
}

// B-factor unit: `own` is the half of the lane group's 32 bytes of metadata that this lane loaded
// (even lanes the four scale pairs, odd lanes the four offset pairs); the other half comes from
// the neighbouring lane.  Every lane of the wavefront must be active.
__device__ inline half8_t q3_unit_b(uint32_t codes, const uint32_t (&own)[4], bool odd) {
  uint32_t v[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const uint32_t nb = uint32_t(__builtin_amdgcn_mov_dpp(int(own[i]), 0xB1 /* quad_perm [1,0,3,2] */, 0xF, 0xF, false));
    const uint32_t S = odd ? nb : own[i], C = odd ? own[i] : nb;
    const uint32_t f = i == 0 ? q3_field<0>(codes) : i == 1 ? q3_field<1>(codes) : i == 2 ? q3_field<2>(codes) : q3_field<3>(codes);
    v[i] = pk_fma(f, S, C);
  }
  return __builtin_bit_cast(half8_t, make_uint4(v[0], v[1], v[2], v[3]));
}

}  // namespace ffn
}  // namespace lrc
