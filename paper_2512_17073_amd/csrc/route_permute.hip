// Routing (Section 2.1: w = softmax(G(x)), Top-k; Section 3.2: Top-n = first n of the sorted list)
// and the grouping of (token, slot) pairs by expert.
#include "internal.h"
#include "permute_body.h"
#include "route_body.h"

namespace lrc {

namespace {

// One workgroup (NW wavefronts: 4, or 16 when there are many experts) per token.  Wavefront w
// accumulates, in fp64, the gate dot products of experts w, w+NW, ...: every bf16 x bf16 product is exact in fp64, so the logits differ from the
// exact ones by ~1e-13 and the selection equals the exact selection.  The same instruction
// sequence runs for every expert row, so duplicated gate rows give bit-identical logits.
// A lane keeps its 16-byte chunks of the token (chunks lane, lane + 64, ...: CH of them) in
// registers for all experts, and the chunks of the next expert's gate row are in flight while the
// current one is multiplied.  Wavefront 0 then takes the Top-k with a shuffle arg-max (ties to the
// lower index) and the softmax weights of the selected experts.

constexpr int kRouteGroups = 8;     // most blocks that share a token

template <int CH, int NW>
__global__ __launch_bounds__(64 * NW) void route_kernel(const uint16_t* __restrict__ x,
                                                    const uint16_t* __restrict__ wg,
                                                    const float* __restrict__ bias, int T, int H, int E,
                                                    int top_k, int renorm, int32_t* __restrict__ idx,
                                                    float* __restrict__ w, _Float16* __restrict__ xh,
                                                    int32_t* __restrict__ tok_exp, double* __restrict__ logits_g) {
  __shared__ double logit[kMaxExperts];
  const int t = blockIdx.x, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  // Few tokens and many experts: gridDim.y blocks share a token's gate rows (block g takes experts
  // g * epg .. + epg - 1) and leave their logits (without the bias) in logits_g [T][E]; topk_kernel
  // follows in a launch of its own.
  const int G = gridDim.y, g = blockIdx.y;
  const int epg = (E + G - 1) / G, e_lo = g * epg, e_hi = min(E, e_lo + epg);
  const uint4* xrow = reinterpret_cast<const uint4*>(x + size_t(t) * H);
  const int chunks = H / 8;

  if (xh != nullptr && g == 0) {     // fp16 copy of the token for the expert kernels (exact for |x| < 65504)
    for (int c = threadIdx.x; c < chunks; c += 64 * NW) {
      const uint4 v = xrow[c];
      const uint32_t in[4] = {v.x, v.y, v.z, v.w};
      uint32_t o[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const _Float16 lo = (_Float16)__uint_as_float(in[i] << 16);
        const _Float16 hi = (_Float16)__uint_as_float(in[i] & 0xffff0000u);
        o[i] = uint32_t(__builtin_bit_cast(uint16_t, lo)) | (uint32_t(__builtin_bit_cast(uint16_t, hi)) << 16);
      }
      reinterpret_cast<uint4*>(xh + size_t(t) * H)[c] = make_uint4(o[0], o[1], o[2], o[3]);
    }
  }

  uint4 xv[CH];
#pragma unroll
  for (int j = 0; j < CH; ++j) {
    const int c = lane + 64 * j;
    xv[j] = c < chunks ? xrow[c] : make_uint4(0, 0, 0, 0);
  }
  if (tok_exp != nullptr && wave == 0 && g == 0) {
    // exponent of the token's power-of-two pre-scale for the expert kernels: 2^s brings its largest
    // magnitude into [1, 2), s within +-60, 0 for a token of zeros
    uint32_t m = 0;
#pragma unroll
    for (int j = 0; j < CH; ++j) {
      const uint32_t xa[4] = {xv[j].x, xv[j].y, xv[j].z, xv[j].w};
#pragma unroll
      for (int i = 0; i < 4; ++i) m = max(m, max(xa[i] & 0x7fffu, (xa[i] >> 16) & 0x7fffu));
    }
#pragma unroll
    for (int d = 32; d > 0; d >>= 1) m = max(m, (uint32_t)__shfl_xor((int)m, d));
    const int eb = int(m >> 7);
    if (lane == 0) tok_exp[t] = eb == 0 ? 0 : min(60, max(-60, 127 - eb));
  }
  auto load_row = [&](int e, uint4 (&wv)[CH]) {
    const uint4* wrow = reinterpret_cast<const uint4*>(wg + size_t(min(e, E - 1)) * H);
#pragma unroll
    for (int j = 0; j < CH; ++j) {
      const int c = lane + 64 * j;
      wv[j] = c < chunks ? wrow[c] : make_uint4(0, 0, 0, 0);
    }
  };
  uint4 wcur[CH], wnext[CH];
  load_row(e_lo + wave, wcur);
  for (int e = e_lo + wave; e < e_hi; e += NW) {
    load_row(e + NW, wnext);                               // (clamped past the last row; unused then)
    double acc = 0.0;
#pragma unroll
    for (int j = 0; j < CH; ++j) {                        // chunks in increasing order, as a plain loop would
      const uint32_t xa[4] = {xv[j].x, xv[j].y, xv[j].z, xv[j].w}, wa[4] = {wcur[j].x, wcur[j].y, wcur[j].z, wcur[j].w};
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        acc = fma(bf16_to_double(xa[i] & 0xffffu), bf16_to_double(wa[i] & 0xffffu), acc);
        acc = fma(bf16_to_double(xa[i] >> 16), bf16_to_double(wa[i] >> 16), acc);
      }
    }
    acc = wave_sum(acc);
    if (lane == 0) {
      if (G == 1) logit[e] = acc + (bias ? (double)bias[e] : 0.0);
      else logits_g[size_t(t) * E + e] = acc;
    }
#pragma unroll
    for (int j = 0; j < CH; ++j) wcur[j] = wnext[j];
  }
  if (G > 1) return;
  __syncthreads();
  if (wave != 0) return;

  // lane holds experts lane, lane+64, lane+128, lane+192
  double v[4];
#pragma unroll
  for (int m = 0; m < 4; ++m) {
    const int e = lane + 64 * m;
    v[m] = e < E ? logit[e] : 0.0;
  }
  select_topk(v, lane, E, top_k, renorm, idx + size_t(t) * top_k, w + size_t(t) * top_k);
}

// Many tokens: the logits of a 16-token x 16-expert tile on the fp64 matrix cores (every wavefront
// of the other kernel re-reads the whole gate for one token; here a gate row serves 16 tokens).
// v_mfma_f64_16x16x4: experts are the rows, tokens the columns; lane (i = lane % 16, kq = lane / 16)
// supplies gate row i and token i at the k index of the step; it walks quarter kq of the hidden
// dimension in order, eight elements per 16-byte load.  Products of bf16 values are exact in fp64
// and every (expert, token) pair sees the same sequence of operations, so duplicated gate rows
// give bit-identical logits.  Grid: (token tiles, groups of four expert tiles); logits [T][E].
typedef double double4_t __attribute__((ext_vector_type(4)));
__global__ __launch_bounds__(256) void gate_logits_kernel(const uint16_t* __restrict__ x,
                                                          const uint16_t* __restrict__ wg, int T, int H, int E,
                                                          double* __restrict__ logits) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int et = blockIdx.y * 4 + wave;
  if (et * 16 >= E) return;
  const int i = lane & 15, kq = lane >> 4, Hq = H / 4;
  const int token = min((int)blockIdx.x * 16 + i, T - 1), expert = min(et * 16 + i, E - 1);
  const uint4* xp = reinterpret_cast<const uint4*>(x + size_t(token) * H + kq * Hq);
  const uint4* wp = reinterpret_cast<const uint4*>(wg + size_t(expert) * H + kq * Hq);
  double4_t acc = double4_t{0.0, 0.0, 0.0, 0.0};
  const int chunks = Hq / 8;
  for (int c0 = 0; c0 < chunks; c0 += 4) {                  // four loads of each operand in flight
    uint4 xv[4], wv[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      xv[u] = make_uint4(0, 0, 0, 0); wv[u] = make_uint4(0, 0, 0, 0);
      if (c0 + u < chunks) { xv[u] = xp[c0 + u]; wv[u] = wp[c0 + u]; }
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const uint32_t xa[4] = {xv[u].x, xv[u].y, xv[u].z, xv[u].w}, wa[4] = {wv[u].x, wv[u].y, wv[u].z, wv[u].w};
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        acc = __builtin_amdgcn_mfma_f64_16x16x4f64(bf16_to_double(wa[j] & 0xffffu), bf16_to_double(xa[j] & 0xffffu), acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f64_16x16x4f64(bf16_to_double(wa[j] >> 16), bf16_to_double(xa[j] >> 16), acc, 0, 0, 0);
      }
    }
  }
  // register r of lane (i, kq) holds row kq + 4 r of the tile (the fp64 variant interleaves the
  // rows by four), i.e. expert 16 et + kq + 4 r, of token 16 tile + i
  const int t = blockIdx.x * 16 + i;
  if (t < T)
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int e = et * 16 + kq + 4 * r;
      if (e < E) logits[size_t(t) * E + e] = acc[r];
    }
}

// Top-k and softmax weights from stored logits: one wavefront per token.
__global__ __launch_bounds__(256) void topk_kernel(const double* __restrict__ logits, const float* __restrict__ bias,
                                                   int T, int E, int top_k, int renorm, int32_t* __restrict__ idx,
                                                   float* __restrict__ w) {
  const int lane = threadIdx.x & 63, t = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (t >= T) return;
  double v[4];
#pragma unroll
  for (int m = 0; m < 4; ++m) {
    const int e = lane + 64 * m;
    v[m] = e < E ? logits[size_t(t) * E + e] + (bias ? (double)bias[e] : 0.0) : 0.0;
  }
  select_topk(v, lane, E, top_k, renorm, idx + size_t(t) * top_k, w + size_t(t) * top_k);
}

// Grouping: one workgroup of 16 wavefronts (permute_body.h).
__global__ __launch_bounds__(1024) void permute_kernel(const int32_t* __restrict__ idx, int P, int E,
                                                       int top_k, int top_n,
                                                       int32_t* __restrict__ counts,
                                                       int32_t* __restrict__ offsets,
                                                       int32_t* __restrict__ row_pair,
                                                       int32_t* __restrict__ pair_row,
                                                       int32_t* __restrict__ comp_counts) {
  __shared__ PermuteLds lds;
  permute_body(lds, idx, P, E, top_k, top_n, counts, offsets, row_pair, pair_row, comp_counts);
}


// Many pairs: the same grouping by several blocks, in two launches.  Block b owns the pairs
// [b * slice, (b + 1) * slice).  The first launch counts every block's pairs per expert into
// `scratch` ([block][2][E]: all pairs, pairs that take the rank-r term).  The second launch scatters:
// every block first adds up all blocks' counts (block 0 writes counts, offsets and comp_counts) and
// so finds where its own pairs of each expert begin; inside a block as in permute_body (wavefront
// w owns a contiguous run, equal experts of a 64-pair step are ranked by ballots), so the order of
// the pairs (= token order) is kept.  The launch boundary orders the two: no fence, no counter (a
// device-scope fence writes back the whole L2 on this chip).
__global__ __launch_bounds__(1024) void permute_count_kernel(const int32_t* __restrict__ idx, int P, int E, int top_k, int top_n,
                                                             int slice, int32_t* __restrict__ scratch) {
  __shared__ int32_t hist[kMaxExperts], comp[kMaxExperts];
  const int b = blockIdx.x;
  for (int e = threadIdx.x; e < E; e += 1024) { hist[e] = 0; comp[e] = 0; }
  __syncthreads();
  const int begin = b * slice, end = min(P, begin + slice);
  for (int i = begin + (int)threadIdx.x; i < end; i += 1024) {
    const int e = min(max(idx[i], 0), E - 1);
    atomicAdd(&hist[e], 1);
    if (i % top_k < top_n) atomicAdd(&comp[e], 1);
  }
  __syncthreads();
  for (int e = threadIdx.x; e < E; e += 1024) {
    scratch[(b * 2 + 0) * E + e] = hist[e];
    scratch[(b * 2 + 1) * E + e] = comp[e];
  }
}

__global__ __launch_bounds__(1024) void permute_scatter_kernel(const int32_t* __restrict__ idx, int P, int E, int slice,
                                                               const int32_t* __restrict__ scratch, int32_t* __restrict__ counts,
                                                               int32_t* __restrict__ offsets, int32_t* __restrict__ comp_counts,
                                                               int32_t* __restrict__ row_pair, int32_t* __restrict__ pair_row) {
  __shared__ int32_t hist[kPermWaves][kMaxExperts];
  __shared__ int32_t total[kMaxExperts], before[kMaxExperts];
  const int b = blockIdx.x, nb = gridDim.x, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  for (int i = threadIdx.x; i < kPermWaves * kMaxExperts; i += 1024) (&hist[0][0])[i] = 0;
  // every block adds up the counts of all blocks (block 0 writes the sums out) ...
  if ((int)threadIdx.x < E) {
    const int e = threadIdx.x;
    int run = 0, crun = 0, mine = 0;
    for (int bb = 0; bb < nb; ++bb) {
      if (bb == b) mine = run;                              // pairs of this expert in the blocks before this one
      run += scratch[(bb * 2 + 0) * E + e];
      crun += scratch[(bb * 2 + 1) * E + e];
    }
    total[e] = run;
    before[e] = mine;
    if (b == 0) { counts[e] = run; comp_counts[e] = crun; }
  }
  __syncthreads();
  const int s_begin = b * slice, s_end = min(P, s_begin + slice);
  const int per_wave = ((s_end - s_begin + kPermWaves - 1) / kPermWaves + 63) / 64 * 64;
  const int begin = s_begin + wave * per_wave, end = min(s_end, begin + per_wave);
  for (int i = begin + lane; i < end; i += 64) atomicAdd(&hist[wave][min(max(idx[i], 0), E - 1)], 1);
  __syncthreads();
  if ((int)threadIdx.x < E) {
    // ... and finds where its own pairs of each expert begin: the expert's offset, then the blocks before it
    const int e = threadIdx.x;
    int off = 0;
    for (int e2 = 0; e2 < e; ++e2) off += total[e2];
    if (b == 0) {
      offsets[e] = off;
      if (e == E - 1) offsets[E] = off + total[e];
    }
    int run = off + before[e];
    for (int wv = 0; wv < kPermWaves; ++wv) {
      const int c = hist[wv][e];
      hist[wv][e] = run;
      run += c;
    }
  }
  __syncthreads();
  int nbits = 0;
  while ((1 << nbits) < E) ++nbits;
  for (int base = begin; base < end; base += 64) {
    const int i = base + lane;
    const bool valid = i < end;
    const int e = valid ? min(max(idx[i], 0), E - 1) : 0;
    unsigned long long same = __ballot(valid);
    for (int bt = 0; bt < nbits; ++bt) {
      const bool bit = (e >> bt) & 1;
      const unsigned long long bb = __ballot(valid && bit);
      same &= bit ? bb : ~bb;
    }
    const int rank = __popcll(same & ((1ull << lane) - 1ull));
    const int cnt = __popcll(same);
    int pos = 0;
    if (valid) pos = hist[wave][e] + rank;
    __builtin_amdgcn_wave_barrier();
    if (valid && rank == 0) hist[wave][e] = pos + cnt;
    __builtin_amdgcn_wave_barrier();
    if (valid) {
      row_pair[pos] = i;
      pair_row[i] = pos;
    }
  }
}

}  // namespace

bool route_writes_exponents(const moe_lrc_layer* L, int T) {
  return !(T >= 1024 && L->cfg.n_experts >= 128 && L->d_logits != nullptr);
}

hipError_t launch_route(const moe_lrc_layer* L, const void* x, int T, int32_t* idx, float* w,
                        _Float16* xh, int32_t* tok_exp, hipStream_t s) {
  const moe_lrc_config& c = L->cfg;
  // Many tokens and many experts: tiled on the fp64 matrix cores.  (With few expert tiles a tile's
  // chain of H / 4 dependent 64-cycle MFMAs is longer than the per-token kernel takes: measured
  // slower for 8 and 64 experts up to T = 2048.)
  if (T >= 1024 && c.n_experts >= 128 && xh == nullptr && L->d_logits != nullptr) {
    hipLaunchKernelGGL(gate_logits_kernel, dim3((T + 15) / 16, (c.n_experts + 63) / 64), dim3(256), 0, s,
                       (const uint16_t*)x, L->d_wg, T, c.hidden, c.n_experts, L->d_logits);
    hipLaunchKernelGGL(topk_kernel, dim3((T + 3) / 4), dim3(256), 0, s, L->d_logits,
                       L->has_bias ? L->d_bias : nullptr, T, c.n_experts, c.top_k, c.renormalize, idx, w);
    return hipGetLastError();
  }
  const int ch = (c.hidden / 8 + 63) / 64;      // 16-byte chunks of a row per lane
  // 16 wavefronts per token when every wavefront would otherwise walk 16 or more gate rows one
  // after the other, the chunks of a row fit the smaller register budget, and the launch is bound
  // by that latency rather than by throughput (few tokens)
  const bool wide = c.n_experts >= 64 && ch <= 8 && T <= 128;
  // ... and, while the tokens alone leave CUs idle, several blocks per token, each with at least
  // one gate row per wavefront (the fp64 dot products of a token's rows are what the launch takes)
  int G = 1;
  if (wide && L->d_logits != nullptr && T <= c.max_tokens)
    while (G < kRouteGroups && T * G * 2 <= L->n_cu && c.n_experts / (G * 2) >= 16) G *= 2;
  auto go = [&](auto kernel, int nw) {
    hipLaunchKernelGGL(kernel, dim3(T, G), dim3(64 * nw), 0, s, (const uint16_t*)x, L->d_wg,
                       L->has_bias ? L->d_bias : nullptr, T, c.hidden, c.n_experts, c.top_k,
                       c.renormalize, idx, w, xh, tok_exp, L->d_logits);
    if (G > 1)
      hipLaunchKernelGGL(topk_kernel, dim3((T + 3) / 4), dim3(256), 0, s, L->d_logits,
                         L->has_bias ? L->d_bias : nullptr, T, c.n_experts, c.top_k, c.renormalize, idx, w);
  };
  if (ch <= 1) wide ? go(route_kernel<1, 16>, 16) : go(route_kernel<1, 4>, 4);
  else if (ch <= 2) wide ? go(route_kernel<2, 16>, 16) : go(route_kernel<2, 4>, 4);
  else if (ch <= 4) wide ? go(route_kernel<4, 16>, 16) : go(route_kernel<4, 4>, 4);
  // (eight wavefronts when that gives every gate row a wavefront of its own and the tokens are few)
  else if (ch <= 8) wide ? go(route_kernel<8, 16>, 16) : (c.n_experts <= 8 && T <= 256) ? go(route_kernel<8, 8>, 8) : go(route_kernel<8, 4>, 4);
  else if (ch <= 16) go(route_kernel<16, 4>, 4);
  else if (ch <= 32) go(route_kernel<32, 4>, 4);
  else return hipErrorInvalidValue;             // hidden > 16384 (layer_create rejects it)
  return hipGetLastError();
}

hipError_t launch_permute(const moe_lrc_layer* L, const int32_t* idx, int T, int32_t* counts,
                          int32_t* offsets, int32_t* row_pair, int32_t* pair_row,
                          int32_t* comp_counts, hipStream_t s) {
  const moe_lrc_config& c = L->cfg;
  const int P = T * c.top_k;
  if (P > kPermuteOneBlockPairs && L->d_perm != nullptr) {
    // several blocks (at most kPermuteMaxBlocks), each with a slice of at least 2048 pairs
    const int slice = std::max(2048, ((P + kPermuteMaxBlocks - 1) / kPermuteMaxBlocks + 63) / 64 * 64);
    const int nb = (P + slice - 1) / slice;
    hipLaunchKernelGGL(permute_count_kernel, dim3(nb), dim3(1024), 0, s, idx, P, c.n_experts, c.top_k, c.top_n, slice,
                       L->d_perm);
    hipLaunchKernelGGL(permute_scatter_kernel, dim3(nb), dim3(1024), 0, s, idx, P, c.n_experts, slice, L->d_perm, counts,
                       offsets, comp_counts, row_pair, pair_row);
    return hipGetLastError();
  }
  hipLaunchKernelGGL(permute_kernel, dim3(1), dim3(1024), 0, s, idx, P, c.n_experts,
                     c.top_k, c.top_n, counts, offsets, row_pair, pair_row, comp_counts);
  return hipGetLastError();
}

}  // namespace lrc
