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
// factor pair at 3 bits (codes one per byte, fp16 scale/zero per group of 64 along K for A [K][rank],
// along N for B transposed [N][rank]) -> the unit layout of layout.h, q3_a_bytes / q3_b_bytes bytes.
// Return the power-of-two factor mu folded into the operands (0: a code is out of range).
float pack_factor_a_q3(int K, int rank, const uint8_t* codes, const uint16_t* scale, const uint16_t* zero, uint8_t* out);
float pack_factor_b_q3(int N, int rank, const uint8_t* codes, const uint16_t* scale, const uint16_t* zero, uint8_t* out);
}  // namespace lrc
