// Host-side repacking of the canonical artefacts (one code per byte, fp16 scale/zero, bf16 factors)
// into the private tile-stream layout described in layout.h.  Pure host code: no HIP calls.
#include "pack.h"

#include <algorithm>
#include <cmath>
#include <cstring>
#include <thread>
#include <vector>

namespace lrc {

namespace {

inline float f16_bits_to_float(uint16_t b) {
  _Float16 h;
  std::memcpy(&h, &b, 2);
  return (float)h;
}
inline uint16_t float_to_f16_bits(double v) {
  _Float16 h = (_Float16)v;
  uint16_t b;
  std::memcpy(&b, &h, 2);
  return b;
}
inline float bf16_bits_to_float(uint16_t b) {
  uint32_t u = uint32_t(b) << 16;
  float f;
  std::memcpy(&f, &u, 4);
  return f;
}

template <class F>
void parallel_for(int n, F&& body) {
  int nthreads = (int)std::min<unsigned>(std::max(1u, std::thread::hardware_concurrency()), 16u);
  nthreads = std::min(nthreads, n);
  if (nthreads <= 1) {
    for (int i = 0; i < n; ++i) body(i);
    return;
  }
  std::vector<std::thread> pool;
  for (int t = 0; t < nthreads; ++t)
    pool.emplace_back([&, t] {
      for (int i = t; i < n; i += nthreads) body(i);
    });
  for (auto& th : pool) th.join();
}

}  // namespace

void pack_codes(const MatLayout& m, const uint8_t* codes, uint32_t* out) {
  const int bits = m.bits, tdw = tile_dwords(bits);
  std::memset(out, 0, m.codes_bytes);
  // one k-step touches a disjoint set of tiles, so k-steps can be packed in parallel
  parallel_for(m.KS, [&](int ks) {
    for (int q = 0; q < 4; ++q)
      for (int kappa = 0; kappa < kLaneK; ++kappa) {
        const int k = ks * kTileK + q * kLaneK + kappa;
        if (k >= m.K) continue;            // padded rows stay code 0 (their metadata is zero)
        CodePiece pc[3];
        const int np = code_pieces(bits, kappa, pc);
        const uint8_t* row = codes + size_t(k) * m.N;
        for (int n = 0; n < m.N; ++n) {
          const uint32_t code = row[n];
          const int nt = n >> 4, lane = q * 16 + (n & 15);
          uint32_t* tile = out + (size_t(ks) * m.NT + nt) * tdw;
          for (int p = 0; p < np; ++p) {
            const uint32_t piece = (code >> pc[p].src_shift) & ((1u << pc[p].width) - 1u);
            tile[tile_dword_index(bits, lane, pc[p].dword)] |= piece << pc[p].bit;
          }
        }
      }
  });
}

void unpack_codes(const MatLayout& m, const uint32_t* packed, uint8_t* codes) {
  const int bits = m.bits, tdw = tile_dwords(bits);
  parallel_for(m.KS, [&](int ks) {
    for (int q = 0; q < 4; ++q)
      for (int kappa = 0; kappa < kLaneK; ++kappa) {
        const int k = ks * kTileK + q * kLaneK + kappa;
        if (k >= m.K) continue;
        CodePiece pc[3];
        const int np = code_pieces(bits, kappa, pc);
        uint8_t* row = codes + size_t(k) * m.N;
        for (int n = 0; n < m.N; ++n) {
          const int nt = n >> 4, lane = q * 16 + (n & 15);
          const uint32_t* tile = packed + (size_t(ks) * m.NT + nt) * tdw;
          uint32_t code = 0;
          for (int p = 0; p < np; ++p) {
            const uint32_t w = tile[tile_dword_index(bits, lane, pc[p].dword)];
            code |= ((w >> pc[p].bit) & ((1u << pc[p].width) - 1u)) << pc[p].src_shift;
          }
          row[n] = (uint8_t)code;
        }
      }
  });
}

float pack_meta(const MatLayout& m, const uint16_t* scale_f16, const uint16_t* zero_f16, uint32_t* out) {
  const int real_groups = m.K / m.group;
  // lambda: largest power of two <= 1 that keeps scale * 2^(14+bits) * lambda within fp16
  double smax = 0;
  for (size_t i = 0; i < size_t(real_groups) * m.N; ++i) {
    const double s = std::fabs((double)f16_bits_to_float(scale_f16[i]));
    if (std::isfinite(s)) smax = std::max(smax, s);
  }
  const double up = std::ldexp(1.0, 14 + m.bits);
  // the kernels also form scale * 2^(class shift) for codes that sit lower in the mantissa:
  // up to 2^4 (2 bit) or 2^6 (3 and 4 bit) times the stored value must stay finite in fp16
  const double class_max = m.bits == 2 ? 16.0 : 64.0;
  int j = 0;
  while (smax * up * class_max * std::ldexp(1.0, -j) > 32768.0) ++j;
  const double lambda = std::ldexp(1.0, -j);
  std::memset(out, 0, m.meta_bytes);
  for (int nt = 0; nt < m.NT; ++nt)
    for (int g = 0; g < real_groups; ++g)
      for (int c = 0; c < kTileN; ++c) {
        const size_t src = size_t(g) * m.N + nt * kTileN + c;
        const double s = f16_bits_to_float(scale_f16[src]), z = f16_bits_to_float(zero_f16[src]);
        const uint32_t lo = float_to_f16_bits(s * lambda * up);
        const uint32_t hi = float_to_f16_bits(-z * s * lambda);
        out[(size_t(g) * m.NT + nt) * kTileN + c] = lo | (hi << 16);
      }
  return (float)lambda;
}

// Both factors are stored rank-major, so that a smaller rank is a prefix of the same layout: the
// 16-column tiles of A one after the other, the 32-wide rank steps of B one after the other.
void pack_factor_a(const MatLayout& m, int rank, const uint16_t* A_bf16, uint16_t* out) {
  // [rpad/16][K/32][lane][8]: lane (c, q) holds A[32*kk + 8*q + j][16*tile + c], j = 0..7
  const int rt = m.rpad / 16, k32 = m.K / 32;
  std::memset(out, 0, m.af_bytes);
  for (int tile = 0; tile < rt; ++tile)
    for (int kk = 0; kk < k32; ++kk)
      for (int lane = 0; lane < kWave; ++lane) {
        const int c = lane & 15, q = lane >> 4, rho = 16 * tile + c;
        if (rho >= rank) continue;
        uint16_t* dst = out + ((size_t(tile) * k32 + kk) * kWave + lane) * 8;
        for (int j = 0; j < 8; ++j)
          dst[j] = float_to_f16_bits(bf16_bits_to_float(A_bf16[size_t(32 * kk + 8 * q + j) * rank + rho]));
      }
}

void pack_factor_b(const MatLayout& m, int rank, const uint16_t* B_bf16, uint16_t* out) {
  // [ceil(rank/32)][N/16][lane][8]: lane (c, q) holds B[32*st + 8*q + j][16*nt + c], j = 0..7 (zero past
  // the rank): one 16-byte unit per lane, the A operand of a 16x16x32 MFMA step over 32 rank indices
  std::memset(out, 0, m.bf_bytes);
  for (int st = 0; st < m.ls; ++st)
    for (int nt = 0; nt < m.NT; ++nt)
      for (int lane = 0; lane < kWave; ++lane) {
        const int c = lane & 15, q = lane >> 4;
        uint16_t* dst = out + ((size_t(st) * m.NT + nt) * kWave + lane) * 8;
        for (int j = 0; j < 8; ++j) {
          const int rho = 32 * st + 8 * q + j;
          if (rho < rank)
            dst[j] = float_to_f16_bits(bf16_bits_to_float(B_bf16[size_t(rho) * m.N + nt * kTileN + c]));
        }
      }
}

namespace {
// mu: the largest power of two <= 1 that keeps scale * mu * 2^17 finite in fp16
double q3_mu(const uint16_t* scale, size_t n) {
  double smax = 0;
  for (size_t i = 0; i < n; ++i) {
    const double s = std::fabs((double)f16_bits_to_float(scale[i]));
    if (std::isfinite(s)) smax = std::max(smax, s);
  }
  int j = 0;
  while (smax * std::ldexp(1.0, 17 - j) > 32768.0) ++j;
  return std::ldexp(1.0, -j);
}
}  // namespace

float pack_factor_a_q3(int K, int rank, const uint8_t* codes, const uint16_t* scale, const uint16_t* zero, uint8_t* out) {
  const int rt = (rank + 15) / 16, k32 = K / 32, g64 = K / 64;
  std::memset(out, 0, q3_a_bytes(K, rank));
  for (size_t i = 0; i < size_t(K) * rank; ++i)
    if (codes[i] > 7) return 0.f;
  const double mu = q3_mu(scale, size_t(g64) * rank);
  uint32_t* cw = reinterpret_cast<uint32_t*>(out);
  uint32_t* mw = reinterpret_cast<uint32_t*>(out + q3_a_codes_bytes(K, rank));
  for (int tile = 0; tile < rt; ++tile) {
    for (int kk = 0; kk < k32; ++kk)
      for (int lane = 0; lane < kWave; ++lane) {
        const int c = lane & 15, q = lane >> 4, rho = 16 * tile + c;
        if (rho >= rank) continue;
        uint32_t w = 0;
        for (int j = 0; j < 8; ++j)
          w |= uint32_t(codes[size_t(32 * kk + 8 * q + j) * rank + rho]) << (16 * (j & 1) + 3 * (j >> 1));
        cw[(size_t(tile) * k32 + kk) * kWave + lane] = w;
      }
    for (int g = 0; g < g64; ++g)
      for (int c = 0; c < 16; ++c) {
        const int rho = 16 * tile + c;
        if (rho >= rank) continue;
        const double s = f16_bits_to_float(scale[size_t(g) * rank + rho]), z = f16_bits_to_float(zero[size_t(g) * rank + rho]);
        mw[(size_t(tile) * g64 + g) * 16 + c] =
            uint32_t(float_to_f16_bits(s * mu * 131072.0)) | (uint32_t(float_to_f16_bits(-z * s * mu)) << 16);
      }
  }
  return (float)mu;
}

float pack_factor_b_q3(int N, int rank, const uint8_t* codes, const uint16_t* scale, const uint16_t* zero, uint8_t* out) {
  const int ls = (rank + 31) / 32, NT = N / 16, NG = N / 64;
  std::memset(out, 0, q3_b_bytes(N, rank));
  for (size_t i = 0; i < size_t(N) * rank; ++i)
    if (codes[i] > 7) return 0.f;
  const double mu = q3_mu(scale, size_t(NG) * rank);
  uint32_t* cw = reinterpret_cast<uint32_t*>(out);
  uint16_t* mh = reinterpret_cast<uint16_t*>(out + q3_b_codes_bytes(N, rank));
  for (int st = 0; st < ls; ++st) {
    for (int nt = 0; nt < NT; ++nt)
      for (int lane = 0; lane < kWave; ++lane) {
        const int c = lane & 15, q = lane >> 4;
        uint32_t w = 0;
        for (int j = 0; j < 8; ++j) {
          const int rho = 32 * st + 8 * q + j;
          if (rho < rank) w |= uint32_t(codes[size_t(nt * kTileN + c) * rank + rho]) << (16 * (j & 1) + 3 * (j >> 1));
        }
        cw[(size_t(st) * NT + nt) * kWave + lane] = w;
      }
    for (int ng = 0; ng < NG; ++ng)
      for (int q = 0; q < 4; ++q) {
        uint16_t* dst = mh + ((size_t(st) * NG + ng) * 4 + q) * 16;      // 8 halves of scales, then 8 of offsets
        for (int j = 0; j < 8; ++j) {
          const int rho = 32 * st + 8 * q + j;
          if (rho >= rank) continue;
          const double s = f16_bits_to_float(scale[size_t(ng) * rank + rho]), z = f16_bits_to_float(zero[size_t(ng) * rank + rho]);
          dst[j] = float_to_f16_bits(s * mu * 131072.0);
          dst[8 + j] = float_to_f16_bits(-z * s * mu);
        }
      }
  }
  return (float)mu;
}

}  // namespace lrc
