// Host-side packers for the private layout (see layout.h).
#pragma once
#include "layout.h"

namespace lrc {
// codes [K][N] one per byte -> packed tiles (m.codes_bytes bytes, zero-padded)
void pack_codes(const MatLayout& m, const uint8_t* codes, uint32_t* out);
void unpack_codes(const MatLayout& m, const uint32_t* packed, uint8_t* codes);
// scale/zero fp16 [K/group][N] -> per-n-tile (lo, hi) fp16 pairs; returns lambda
float pack_meta(const MatLayout& m, const uint16_t* scale_f16, const uint16_t* zero_f16, uint32_t* out);
// factors bf16 -> fp16 MFMA-operand order
void pack_factor_a(const MatLayout& m, int rank, const uint16_t* A_bf16, uint16_t* out);
void pack_factor_b(const MatLayout& m, int rank, const uint16_t* B_bf16, uint16_t* out);
// 3-bit factor pair -> transfer blob (q3_offsets in layout.h); codes one per byte, each < 8; returns
// false if a code is out of range.  out: q3_offsets(...)[5] bytes
bool pack_q3_blob(int K, int N, int rank, const uint8_t* a_codes, const uint16_t* a_scale, const uint16_t* a_zero,
                  const uint8_t* b_codes, const uint16_t* b_scale, const uint16_t* b_zero, uint8_t* out);
}  // namespace lrc
