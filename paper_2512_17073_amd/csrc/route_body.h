// Device-side pieces of the routing (Section 2.1: w = softmax(G(x)), Top-k) shared by the routing
// kernels and by the launch that prepares the activations, which routes a handful of tokens itself.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "internal.h"

namespace lrc {

__device__ inline double bf16_to_double(uint32_t bits16) {
  return (double)__uint_as_float(bits16 << 16);
}

__device__ inline double wave_sum(double v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off);
  return v;
}

// Top-k of one token's logits by a shuffle arg-max (value descending, ties to the lower index), and
// the softmax weights of the selected experts (Section 2.1), by one wavefront: lane holds the
// logits of experts lane, lane + 64, lane + 128, lane + 192.
__device__ inline void select_topk(const double (&v)[4], int lane, int E, int top_k, int renorm,
                                   int32_t* __restrict__ idx_t, float* __restrict__ w_t) {
  uint32_t taken = 0;
#pragma unroll
  for (int m = 0; m < 4; ++m)
    if (lane + 64 * m >= E) taken |= 1u << m;
  double vmax = 0.0, den = 0.0, sel_sum = 0.0, my_w = 0.0;
  int my_idx = 0;
  for (int j = 0; j < top_k; ++j) {
    double bv = 0.0;
    int bi = 0x7fffffff;
#pragma unroll
    for (int m = 0; m < 4; ++m)
      if (!(taken & (1u << m)) && (bi == 0x7fffffff || v[m] > bv)) { bv = v[m]; bi = lane + 64 * m; }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
      const double ov = __shfl_xor(bv, off);
      const int oi = __shfl_xor(bi, off);
      const bool take = oi != 0x7fffffff && (bi == 0x7fffffff || ov > bv || (ov == bv && oi < bi));
      if (take) { bv = ov; bi = oi; }
    }
    if ((bi & 63) == lane) taken |= 1u << (bi >> 6);
    if (j == 0) {
      vmax = bv;
      double part = 0.0;
#pragma unroll
      for (int m = 0; m < 4; ++m)
        if (lane + 64 * m < E) part += exp(v[m] - vmax);
      den = wave_sum(part);
    }
    const double score = exp(bv - vmax) / den;
    sel_sum += score;
    if (lane == j) { my_w = score; my_idx = bi; }
  }
  if (lane < top_k) {
    idx_t[lane] = my_idx;
    w_t[lane] = (float)(renorm ? my_w / sel_sum : my_w);
  }
}


// The whole routing of a token or two (at most kFusedRoutePairs (token, expert) pairs) by one
// 1024-thread block: every (token, expert) gate dot product by one wavefront, with the lanes walking
// the 16-byte chunks of the rows and adding the exact bf16 x bf16 products in fp64 in the order the
// per-token routing kernel uses (the logits are bit-identical to that kernel's); then one wavefront
// per token takes the Top-k and the softmax weights and writes the token's pre-scale exponent.
// `logit` is LDS, T * E doubles.  Every block that runs this writes the same values; a block reads
// them back after the __syncthreads() the caller follows this with.
__device__ inline void route_small_body(double* logit, const uint16_t* __restrict__ x, const RouteArgs& ra, int T, int H, int E,
                                        int top_k) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, chunks = H / 8;
  for (int p = wave; p < T * E; p += 16) {
    const int t = p / E, e = p - t * E;
    const uint4* xrow = reinterpret_cast<const uint4*>(x + size_t(t) * H);
    const uint4* wrow = reinterpret_cast<const uint4*>(ra.wg + size_t(e) * H);
    double acc = 0.0;
    for (int c0 = lane; c0 < chunks; c0 += 64 * 4) {      // four chunks of both rows in flight
      uint4 xv[4], wv[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int c = c0 + 64 * u;
        xv[u] = c < chunks ? xrow[c] : make_uint4(0, 0, 0, 0);
        wv[u] = c < chunks ? wrow[c] : make_uint4(0, 0, 0, 0);
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {                        // (chunks in increasing order; a chunk of zeros adds nothing)
        const uint32_t xa[4] = {xv[u].x, xv[u].y, xv[u].z, xv[u].w}, wa[4] = {wv[u].x, wv[u].y, wv[u].z, wv[u].w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          acc = fma(bf16_to_double(xa[i] & 0xffffu), bf16_to_double(wa[i] & 0xffffu), acc);
          acc = fma(bf16_to_double(xa[i] >> 16), bf16_to_double(wa[i] >> 16), acc);
        }
      }
    }
    acc = wave_sum(acc);
    if (lane == 0) logit[p] = acc + (ra.bias ? (double)ra.bias[e] : 0.0);
  }
  if (wave < T && ra.tok_exp != nullptr) {       // the token's pre-scale exponent (ffn_common.h)
    const uint4* xrow = reinterpret_cast<const uint4*>(x + size_t(wave) * H);
    uint32_t m = 0;
    for (int c = lane; c < chunks; c += 64) {
      const uint4 xv = xrow[c];
      const uint32_t xa[4] = {xv.x, xv.y, xv.z, xv.w};
#pragma unroll
      for (int i = 0; i < 4; ++i) m = max(m, max(xa[i] & 0x7fffu, (xa[i] >> 16) & 0x7fffu));
    }
#pragma unroll
    for (int d = 32; d > 0; d >>= 1) m = max(m, (uint32_t)__shfl_xor((int)m, d));
    const int eb = int(m >> 7);
    if (lane == 0) ra.tok_exp[wave] = eb == 0 ? 0 : min(60, max(-60, 127 - eb));
  }
  __syncthreads();
  if (wave < T) {
    double v[4];
#pragma unroll
    for (int m = 0; m < 4; ++m) {
      const int e = lane + 64 * m;
      v[m] = e < E ? logit[wave * E + e] : 0.0;
    }
    select_topk(v, lane, E, top_k, ra.renorm, ra.idx + size_t(wave) * top_k, ra.w + size_t(wave) * top_k);
  }
}

}  // namespace lrc
