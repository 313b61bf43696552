// Private storage layout of the packed experts ("tile-stream layout"), shared by the host packer
// and the device kernels of this library.
//
// One projection W[K][N] (input-dim-major) is cut into tiles of 256 input rows (a "k-step") by 16
// output columns (an "n-tile").  A tile is consumed by one wavefront: lane l = 16*q + c owns output
// column 16*nt + c and the 64 consecutive input rows 256*ks + 64*q .. +63, i.e. exactly one
// quantization group when group == 64.  A lane's 64 codes are stored in 2*bits dwords in the order
// the MFMA operand wants them: code kappa (0..63) is operand element j = kappa % 8 of sub-step
// s = kappa / 8, and the two codes of a pair (kappa even/odd) sit at the same bit offset of the low
// and high 16-bit halves of a dword, so that one shift + one mask places both into the mantissa of
// two packed fp16 values.
//
//   2 bit: dword d = kappa/16, field offset 2*((kappa%16)/2) in each half
//   4 bit: dword d = kappa/8,  field offset 4*((kappa%8)/2)
//   3 bit: pair pi = kappa/2; pi < 30: dword pi/5, field offset 1 + 3*(pi%5) (bit 0 of each half is
//          spare); pairs 30 and 31 are spread over the spare bits: bit j of the code of pair 30+t
//          lives in bit 0 (low half) / bit 16 (high half) of dword 3*t + j.
//
// Tiles are stored k-step-major: tile (ks, nt) sits at index ks * NT + nt.  The wavefronts of a
// launch advance through the k-steps at about the same pace, each on its own n-tile, so at any
// moment the tiles being read form one contiguous sweep of memory that spreads evenly over the HBM
// channels (an n-tile-major order would have every wavefront read at the same large stride).
// Inside a tile, dwords 0..3 of all lanes come first ([lane][4], one 16-byte load per lane), then
// the remaining 2*bits-4 dwords ([lane][2*bits-4]).
//
// Per-group metadata is stored group-major as [K/group][NT][16 columns] pairs of fp16:
//   lo = scale * lambda * 2^(14+bits),  hi = -zero * scale * lambda
// so that fma(field, lo, hi) on the fp16 *subnormal* whose mantissa holds the code at its top bits
// (value code * 2^-(14+bits)) gives lambda * (code - zero) * scale in one packed instruction.
// Codes that sit lower in the mantissa use lo * 2^(their distance from the top) instead.
// lambda is a power of two chosen per projection so that every such multiple of lo stays finite;
// the kernels multiply the accumulators by 1/lambda at the end.
#pragma once
#include <stddef.h>
#include <stdint.h>

#if defined(__HIPCC__) || defined(__HIP__)
#define LRC_HD __host__ __device__ inline
#else
#define LRC_HD inline
#endif

namespace lrc {

constexpr int kTileK = 256;    // input rows per k-step
constexpr int kTileN = 16;     // output columns per n-tile
constexpr int kLaneK = 64;     // consecutive input rows owned by one lane in a k-step
constexpr int kWave = 64;

LRC_HD int dwords_per_lane(int bits) { return 2 * bits; }
LRC_HD int tile_dwords(int bits) { return kWave * 2 * bits; }
LRC_HD int padded_k(int K) { return (K + kTileK - 1) / kTileK * kTileK; }

// Position of lane-local code `kappa` as up to three (dword, bit, width) pieces.
struct CodePiece { int dword, bit, width, src_shift; };

LRC_HD int code_pieces(int bits, int kappa, CodePiece out[3]) {
  const int h = kappa & 1, pi = kappa >> 1;
  if (bits == 2) {
    out[0] = {pi / 8, 16 * h + 2 * (pi % 8), 2, 0};
    return 1;
  }
  if (bits == 4) {
    out[0] = {pi / 4, 16 * h + 4 * (pi % 4), 4, 0};
    return 1;
  }
  if (pi < 30) {
    out[0] = {pi / 5, 16 * h + 1 + 3 * (pi % 5), 3, 0};
    return 1;
  }
  const int t = pi - 30;
  for (int j = 0; j < 3; ++j) out[j] = {3 * t + j, 16 * h, 1, j};
  return 3;
}

// Index of lane `lane`'s dword `d` inside a tile.
LRC_HD int tile_dword_index(int bits, int lane, int d) {
  if (d < 4) return lane * 4 + d;
  const int rest = 2 * bits - 4;
  return kWave * 4 + lane * rest + (d - 4);
}

// Shape-derived sizes of one packed projection.
struct MatLayout {
  int K, N, Kp, KS, NT, G, bits, group, rpad;   // rpad: rank rounded up to 16 (A factor, (in A))
  int ls;                                        // rank steps of 32 of the B factor: ceil(rank / 32)
  size_t codes_bytes, meta_bytes, af_bytes, bf_bytes;
};

inline size_t align256(size_t x) { return (x + 255) & ~size_t(255); }

inline MatLayout make_layout(int K, int N, int bits, int group, int rank) {
  MatLayout m{};
  m.K = K; m.N = N; m.bits = bits; m.group = group;
  m.Kp = padded_k(K); m.KS = m.Kp / kTileK; m.NT = N / kTileN; m.G = m.Kp / group;
  m.rpad = (rank + 15) / 16 * 16;
  m.ls = (rank + 31) / 32;
  m.codes_bytes = align256(size_t(m.NT) * m.KS * tile_dwords(bits) * 4);
  m.meta_bytes = align256(size_t(m.NT) * m.G * kTileN * 4);
  m.af_bytes = align256(size_t(K) * m.rpad * 2);
  m.bf_bytes = align256(size_t(m.ls) * 32 * N * 2);
  return m;
}

// A factor pair held at 3 bits (Section 3.1 step 2) keeps the unit structure of the fp16 layouts
// (pack_factor_a / pack_factor_b): every 16-byte unit of 8 fp16 values per lane becomes one dword
// of 8 codes per lane, the code of element j at bits 3 (j / 2) .. + 2 of half j % 2 of the dword, plus
// metadata from which one packed FMA per element pair rebuilds the fp16 operand
// (mu (code - zero) scale, mu a power of two per factor that keeps the metadata finite in fp16):
//   A [K][r], groups of 64 along K: per (16-column tile, group, column c) one dword
//     lo = scale mu 2^17, hi = -zero scale mu   (every element of a lane shares the group and column)
//   B transposed [N][r], groups of 64 along N: per (rank step, group of 4 n-tiles, lane group q)
//     32 bytes: four pairs scale mu 2^17 of rank indices (8 q + 2 i, 8 q + 2 i + 1), then the four
//     pairs -zero scale mu   (the elements of a lane differ in their rank index)
// Both sections are rank-major like the fp16 ones: codes first, the metadata behind them.
inline size_t q3_a_codes_bytes(int K, int rank) { return size_t((rank + 15) / 16) * (K / 32) * 256; }
inline size_t q3_a_bytes(int K, int rank) { return q3_a_codes_bytes(K, rank) + size_t((rank + 15) / 16) * (K / 64) * 64; }
inline size_t q3_b_codes_bytes(int N, int rank) { return size_t((rank + 31) / 32) * (N / 16) * 256; }
inline size_t q3_b_bytes(int N, int rank) { return q3_b_codes_bytes(N, rank) + size_t((rank + 31) / 32) * (N / 64) * 128; }

}  // namespace lrc
