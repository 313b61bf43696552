// (in A) for the rows of the decode flavour: the body shared by xa_rows_kernel (ffn_decode.hip) and
// by the launch that prepares the activations (misc.hip), which runs it for the fused W1|W3
// projections in further blocks.
#pragma once
#include <type_traits>

#include "factor_q3.h"
#include "ffn_common.h"

namespace lrc {
namespace ffn {

constexpr int kXaBatch = 4;     // factor and activation units requested together (8 spill in a 1024-thread block)

// (in A)[row][rho] for the rows of the decode flavour, finished in one launch:
//   P[row][m * ls * 32 + rho] = fp16(lambda_m * sum_k in[row][k] * A_m[k][rho]) for rows that take the
// rank-r term, 0 for the other rows of an expert that has such rows; lambda_m is the projection's
// power-of-two pre-scale.  grid = (16-column tiles of [A1 | A3] or of A2, each padded to ls * 32
// columns; experts); the NW wavefronts of a block split K and add their parts through LDS in a
// fixed order.  A tile past the projection's own rank writes zeros (the FFN kernel reads the columns
// of every rank step its expert runs).  TOKENS: the rows are read from the bf16 tokens through
// row_pair (the launch that prepares the activations runs this body in further blocks); otherwise
// from the fp16 operand-order buffer.
template <bool DUAL, bool TOKENS, int NW, int BATCH = kXaBatch>
__device__ __forceinline__ void xa_rows_body(const KArgs& a, const uint16_t* __restrict__ x_bf16, int tile, int e, int kb,
                                             float4_t (*red)[64] /* [2 * NW][64] */) {
  const int r0 = a.offsets[e], cnt = a.offsets[e + 1] - r0;
  const ExpertDesc& d = a.desc[e];
  if (cnt == 0 || !d.has_factors) return;
  const int lane = threadIdx.x & 63, c = lane & 15, q = lane >> 4;
  {
    // an expert without a row that takes the term is skipped (the FFN kernel does not read its rows
    // of P).  Counted here rather than read from the per-expert counters, which the launch that
    // prepares the activations writes in other blocks of the same launch.
    bool some = false;
    for (int i = lane; i < cnt; i += 64) some |= (a.row_pair[r0 + i] % a.top_k) < a.top_n;
    if (__ballot(some) == 0ull) return;
  }
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int tpm = 2 * a.ls;                        // 16-column tiles per projection (padded to ls * 32 columns)
  const int m = tile / tpm, tl = tile - m * tpm;
  const int mat = DUAL ? m : 2;
  const int pitch = (DUAL ? 2 : 1) * a.ls * 32;
  const int rank = min(d.rank[mat], a.rank);
  const bool live = 16 * tl < rank;
  const float lam = d.xa_scale[mat];
  const half8_t* af = reinterpret_cast<const half8_t*>(d.af[mat]);
  // a pair held at 3 bits (layout.h): one dword of codes per lane and unit, one of metadata per
  // (tile, group of 64 inputs, column), dequantized here
  const bool q3 = __builtin_amdgcn_readfirstlane((d.q3 >> mat) & 1) != 0;
  const uint32_t* aq = reinterpret_cast<const uint32_t*>(d.af[mat]);
  const uint32_t* am = d.afm[mat];
  const int g64 = a.K / 64;
  // this block's K-block (grid.z K-blocks of kb_steps k-steps each; one when kb_steps covers K): the
  // FFN kernel's K-block kb applies the B factor to the part of (in A) summed over its own k-steps
  const int k32 = a.K / 32, kb_lo = min(k32, kb * a.kb_steps * 8), kb_hi = min(k32, (kb + 1) * a.kb_steps * 8);
  const int per = (kb_hi - kb_lo + NW - 1) / NW;
  const int kk0 = kb_lo + wave * per, kk1 = min(kb_hi, kk0 + per);
  _Float16* P = reinterpret_cast<_Float16*>(const_cast<float*>(a.p)) + size_t(kb) * a.total_rows * pitch;
  const half8_t* src = reinterpret_cast<const half8_t*>(a.in);   // operand order: unit (k8, row)
  // Two row tiles share every load of the factor; all loads of a batch are issued before the first
  // is awaited (unconditional loads from clamped addresses, cleared afterwards where they do not count).
  for (int r = 0; r < cnt; r += 32) {
    bool flagged[2];
    int pair[2];
    const uint4* xrow[2];
    float xs2[2] = {1.f, 1.f};
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      const int row = min(r + 16 * t + c, cnt - 1);
      pair[t] = a.row_pair[r0 + row];
      flagged[t] = r + 16 * t + c < cnt && (pair[t] % a.top_k) < a.top_n;
      xrow[t] = TOKENS ? reinterpret_cast<const uint4*>(x_bf16 + size_t(pair[t] / a.top_k) * a.K) : nullptr;
      // the row's power-of-two pre-scale (the fp16 operand-order buffer holds the rows already scaled)
      if constexpr (TOKENS) xs2[t] = pow2i(a.tok_exp ? a.tok_exp[pair[t] / a.top_k] : a.row_exp[r0 + row]);
    }
    const bool any0 = __ballot(flagged[0]) != 0ull, any1 = __ballot(flagged[1]) != 0ull;   // block-uniform
    float4_t acc[2] = {float4_t{0.f, 0.f, 0.f, 0.f}, float4_t{0.f, 0.f, 0.f, 0.f}};
    if (live && (any0 || any1)) {
      // (with rows in the first row tile only, twice as many units are in flight: the second tile's registers are free)
      auto k_loop = [&](auto Q3_, auto TWO_) {
      constexpr bool Q3 = decltype(Q3_)::value, TWO = decltype(TWO_)::value;
      constexpr int NB = TWO ? BATCH : 2 * BATCH, NT = TWO ? 2 : 1;
      for (int kk = kk0; kk < kk1; kk += NB) {
        half8_t wf[NB], xf[NT][NB];
        uint32_t cq[NB], mq[NB];
#pragma unroll
        for (int u = 0; u < NB; ++u) {
          const int ku = max(min(kk + u, kk1 - 1), 0);
          if constexpr (Q3) {
            cq[u] = aq[(size_t(tl) * k32 + ku) * kWave + lane];
            mq[u] = am[(size_t(tl) * g64 + (ku >> 1)) * 16 + c];
          } else {
            wf[u] = af[(size_t(tl) * k32 + ku) * kWave + lane];
          }
#pragma unroll
          for (int t = 0; t < NT; ++t) {
            if constexpr (TOKENS) {
              const uint4 v = xrow[t][4 * ku + q];
              const uint32_t in[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
              for (int i = 0; i < 4; ++i) {
                xf[t][u][2 * i] = (_Float16)(__uint_as_float(in[i] << 16) * xs2[t]);
                xf[t][u][2 * i + 1] = (_Float16)(__uint_as_float(in[i] & 0xffff0000u) * xs2[t]);
              }
            } else {
              xf[t][u] = src[act_unit(4 * ku + q, r0 + min(r + 16 * t + c, cnt - 1), a.in_rt)];
            }
          }
        }
#pragma unroll
        for (int u = 0; u < NB; ++u) {
          if constexpr (Q3) wf[u] = q3_unit_a(cq[u], mq[u]);
          if (kk + u >= kk1) wf[u] = half8_t{0, 0, 0, 0, 0, 0, 0, 0};       // (a step past this wavefront's share)
#pragma unroll
          for (int t = 0; t < NT; ++t) {
            if (!flagged[t]) xf[t][u] = half8_t{0, 0, 0, 0, 0, 0, 0, 0};
            acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_f16(wf[u], xf[t][u], acc[t], 0, 0, 0);
          }
        }
      }
      };
      if (q3) { if (any1) k_loop(std::true_type{}, std::true_type{}); else k_loop(std::true_type{}, std::false_type{}); }
      else { if (any1) k_loop(std::false_type{}, std::true_type{}); else k_loop(std::false_type{}, std::false_type{}); }
      red[wave][lane] = acc[0];
      red[NW + wave][lane] = acc[1];
      __syncthreads();
      if (wave == 0) {
        acc[0] = red[0][lane];
        acc[1] = red[NW][lane];
#pragma unroll
        for (int w = 1; w < NW; ++w) { acc[0] += red[w][lane]; acc[1] += red[NW + w][lane]; }
      }
      __syncthreads();
    }
    // lane (q, c) of wavefront 0 holds columns 16 tl + 4 q .. + 3 of rows r + c and r + 16 + c
    if (wave == 0) {
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        const int row = r + 16 * t + c;
        if (row >= cnt) continue;
        half4_t v = half4_t{0, 0, 0, 0};
        if (flagged[t] && live)
          v = half4_t{to_f16_sat(acc[t][0] * lam), to_f16_sat(acc[t][1] * lam), to_f16_sat(acc[t][2] * lam), to_f16_sat(acc[t][3] * lam)};
        *reinterpret_cast<half4_t*>(P + size_t(r0 + row) * pitch + m * a.ls * 32 + 16 * tl + 4 * q) = v;
      }
    }
  }
}

}  // namespace ffn
}  // namespace lrc
