// (in A) for the rows of the decode flavour: the body shared by xa_rows_kernel (ffn_decode.hip) and
// by the launch that prepares the activations (misc.hip), which runs it for the fused W1|W3
// projections in further blocks.
#pragma once
#include "ffn_common.h"

namespace lrc {
namespace ffn {

// (in A)[row][rho] for the rows of the decode flavour, finished in one launch:
//   P[row][m * ls * 32 + rho] = fp16(lambda_m * sum_k in[row][k] * A_m[k][rho]) for rows that take the
// rank-r term, 0 for the other rows of an expert that has such rows; lambda_m is the projection's
// power-of-two pre-scale.  grid = (16-column tiles of [A1 | A3] or of A2, each padded to ls * 32
// columns; experts); the NW wavefronts of a block split K and add their parts through LDS in a
// fixed order.  A tile past the projection's own rank writes zeros (the FFN kernel reads the columns
// of every rank step its expert runs).  TOKENS: the rows are read from the bf16 tokens through
// row_pair (the launch that prepares the activations runs this body in further blocks); otherwise
// from the fp16 operand-order buffer.
template <bool DUAL, bool TOKENS, int NW>
__device__ __forceinline__ void xa_rows_body(const KArgs& a, const uint16_t* __restrict__ x_bf16, int tile, int e,
                                             float4_t (*red)[64]) {
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
  const float lam = d.lambda[mat];
  const half8_t* af = reinterpret_cast<const half8_t*>(d.af[mat]);
  const int k32 = a.K / 32, per = (k32 + NW - 1) / NW;
  const int kk0 = wave * per, kk1 = min(k32, kk0 + per);
  _Float16* P = reinterpret_cast<_Float16*>(const_cast<float*>(a.p));
  const half8_t* src = reinterpret_cast<const half8_t*>(a.in);   // operand order: unit (k8, row)
  for (int r = 0; r < cnt; r += 16) {
    const int row = r + c;
    bool flagged = false;
    int pair = 0;
    if (row < cnt) { pair = a.row_pair[r0 + row]; flagged = (pair % a.top_k) < a.top_n; }
    const bool any = __ballot(flagged) != 0ull;      // same rows in every wavefront: block-uniform
    float4_t acc = float4_t{0.f, 0.f, 0.f, 0.f};
    if (live && any) {
      const uint4* xrow = TOKENS ? reinterpret_cast<const uint4*>(x_bf16 + size_t(pair / a.top_k) * a.K) : nullptr;
      for (int kk = kk0; kk < kk1; kk += 8) {        // eight steps of loads in flight
        half8_t wf[8], xf[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          wf[u] = half8_t{0, 0, 0, 0, 0, 0, 0, 0};
          xf[u] = half8_t{0, 0, 0, 0, 0, 0, 0, 0};
          if (kk + u < kk1) {
            wf[u] = af[(size_t(tl) * k32 + kk + u) * kWave + lane];
            if (flagged) {
              if constexpr (TOKENS) {
                const uint4 v = xrow[4 * (kk + u) + q];
                const uint32_t in[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                  xf[u][2 * i] = (_Float16)__uint_as_float(in[i] << 16);
                  xf[u][2 * i + 1] = (_Float16)__uint_as_float(in[i] & 0xffff0000u);
                }
              } else {
                xf[u] = src[act_unit(4 * (kk + u) + q, r0 + row, a.in_rt)];
              }
            }
          }
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(wf[u], xf[u], acc, 0, 0, 0);
      }
      red[wave][lane] = acc;
      __syncthreads();
      if (wave == 0) {
        acc = red[0][lane];
#pragma unroll
        for (int w = 1; w < NW; ++w) acc += red[w][lane];
      }
      __syncthreads();
    }
    // lane (q, c) of wavefront 0 holds columns 16 tl + 4 q .. + 3 of row c
    if (wave == 0 && row < cnt) {
      half4_t v = half4_t{0, 0, 0, 0};
      if (flagged && live) v = half4_t{(_Float16)(acc[0] * lam), (_Float16)(acc[1] * lam), (_Float16)(acc[2] * lam), (_Float16)(acc[3] * lam)};
      *reinterpret_cast<half4_t*>(P + size_t(r0 + row) * pitch + m * a.ls * 32 + 16 * tl + 4 * q) = v;
    }
  }
}


}  // namespace ffn
}  // namespace lrc
