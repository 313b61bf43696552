// Weighted combine (Section 2.1: y = sum_{i in TopK} w_i E_i(x)), the fp16 activation copy with the
// per-call expert statistics, and the unpack hook that reads the private packed layout back.
#include <algorithm>

#include "decode_index.h"
#include "internal.h"
#include "permute_body.h"
#include "plan.h"
#include "route_body.h"
#include "unpack.h"
#include "xa_rows.h"

namespace lrc {

namespace {

__device__ inline float bf16_lo(uint32_t v) { return __uint_as_float(v << 16); }
__device__ inline float bf16_hi(uint32_t v) { return __uint_as_float(v & 0xffff0000u); }
__device__ inline uint32_t pack_bf16(float a, float b) {
  uint32_t ua = __float_as_uint(a), ub = __float_as_uint(b);
  ua += 0x7fffu + ((ua >> 16) & 1u);
  ub += 0x7fffu + ((ub >> 16) & 1u);
  return (ua >> 16) | (ub & 0xffff0000u);
}

// out[t] = sum_j w[t][j] * y_rows[pair_row[t*k+j]] + sum_s y_shared[s*T+t]; slots in order j = 0..k-1,
// then the shared experts: a fixed order, so two runs give identical bits.  With y_part, row R's
// output is the sum over the K-blocks kb = 0.. of y_part[kb][R] (fp32, in that order) instead of
// the bf16 row y_rows[R].
// PARTS: the rows come as K-block parts (y_part); else as bf16 rows (y_rows).
template <bool PARTS>
__global__ __launch_bounds__(256) void combine_kernel(const uint16_t* __restrict__ y_rows,
                                                      const float* __restrict__ y_part, int kblocks, size_t kb_stride,
                                                      const float* __restrict__ w,
                                                      const int32_t* __restrict__ pair_row,
                                                      const uint16_t* __restrict__ y_shared,
                                                      const uint16_t* __restrict__ residual, int T, int H,
                                                      int top_k, int n_shared, uint16_t* __restrict__ out) {
  // (grid.y walks the 8-column chunks of a row in steps of the block size: few tokens still make many blocks)
  const int t = blockIdx.x;
  for (int ch = blockIdx.y * 256 + threadIdx.x; ch < H / 8; ch += 256 * gridDim.y) {
    float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    for (int j = 0; j < top_k; ++j) {
      const int row = pair_row[t * top_k + j];
      const float wj = w[t * top_k + j];
      if constexpr (PARTS) {
        // every K-block's part is requested before the first is added; the additions keep the
        // order kb = 0, 1, ...
        float4 pl[kMaxKBlocks], ph[kMaxKBlocks];
#pragma unroll
        for (int kb = 0; kb < kMaxKBlocks; ++kb) {
          if (kb < kblocks) {
            const float4* s2 = reinterpret_cast<const float4*>(y_part + kb * kb_stride + size_t(row) * H) + 2 * ch;
            pl[kb] = s2[0]; ph[kb] = s2[1];
          }
        }
        float4 lo = pl[0], hi = ph[0];
#pragma unroll
        for (int kb = 1; kb < kMaxKBlocks; ++kb) {
          if (kb >= kblocks) break;
          const float4 a = pl[kb], b = ph[kb];
          lo.x += a.x; lo.y += a.y; lo.z += a.z; lo.w += a.w;
          hi.x += b.x; hi.y += b.y; hi.z += b.z; hi.w += b.w;
        }
        acc[0] = fmaf(wj, lo.x, acc[0]); acc[1] = fmaf(wj, lo.y, acc[1]); acc[2] = fmaf(wj, lo.z, acc[2]); acc[3] = fmaf(wj, lo.w, acc[3]);
        acc[4] = fmaf(wj, hi.x, acc[4]); acc[5] = fmaf(wj, hi.y, acc[5]); acc[6] = fmaf(wj, hi.z, acc[6]); acc[7] = fmaf(wj, hi.w, acc[7]);
      } else {
        const uint4 v = reinterpret_cast<const uint4*>(y_rows + size_t(row) * H)[ch];
        const uint32_t a[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          acc[2 * i] = fmaf(wj, bf16_lo(a[i]), acc[2 * i]);
          acc[2 * i + 1] = fmaf(wj, bf16_hi(a[i]), acc[2 * i + 1]);
        }
      }
    }
    for (int s = 0; s < n_shared; ++s) {
      const uint4 v = reinterpret_cast<const uint4*>(y_shared + (size_t(s) * T + t) * H)[ch];
      const uint32_t a[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        acc[2 * i] += bf16_lo(a[i]);
        acc[2 * i + 1] += bf16_hi(a[i]);
      }
    }
    if (residual != nullptr) {                 // a stack of layers: out = x + layer(x)
      const uint4 v = reinterpret_cast<const uint4*>(residual + size_t(t) * H)[ch];
      const uint32_t a[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        acc[2 * i] += bf16_lo(a[i]);
        acc[2 * i + 1] += bf16_hi(a[i]);
      }
    }
    reinterpret_cast<uint4*>(out + size_t(t) * H)[ch] =
        make_uint4(pack_bf16(acc[0], acc[1]), pack_bf16(acc[2], acc[3]), pack_bf16(acc[4], acc[5]),
                   pack_bf16(acc[6], acc[7]));
  }
}

// Blocks 0..ceil(rows/16)-1 write the fp16 copy of sixteen rows' tokens in operand order (the layout
// the FFN kernels stage from, see act_unit in ffn_common.h): row R of the routed rows is the token
// of pair row_pair[R]; without row_pair, row R is token R.  Thread (row r = t % 16, column lane
// t / 16) converts the 16-byte units t / 16, t / 16 + 64, ... of its row: a wavefront reads 64
// contiguous bytes of each of its rows and writes runs of 256 bytes (sixteen rows of one unit).
// The blocks after those count, one wavefront per expert, the routed rows and the rows that take
// the rank-r term (what the router-guided transfer must bring in): stat = [-, -, rows[E], comp rows[E]].
// (and compact the latter for the grouped (in A) kernels, CompactArgs).
// Then one block makes the block tables of the decode launches (plan.h), and xa_tiles * E further
// blocks compute (x A1 | x A3) for the decode flavour of the fused projection from the bf16 tokens
// (xa_rows.h), so that no launch of its own stands between this one and the W1|W3 kernel.
constexpr int kPrepThreads = 1024;
// With a token or two every block first routes them itself (route.wg != null).
// With few pairs, every block first groups the pairs by expert itself (perm.idx != null: the body of
// the permute kernel, writing the same values from every block) instead of a launch of its own
// doing it beforehand; offsets and row_pair are then this block's own writes, read back after a
// barrier (hence no __restrict__ on them).
__global__ __launch_bounds__(kPrepThreads) void prep_kernel(const uint16_t* __restrict__ x, int rows, int H,
                                                   uint4* __restrict__ xg, int rt,
                                                   const int32_t* offsets,
                                                   const int32_t* row_pair, int E, int top_k,
                                                   int top_n, int32_t* __restrict__ stat, PlanSpec plan0,
                                                   PlanSpec plan1, int xa_tiles, ffn::KArgs xa,
                                                   const int32_t* tok_exp, int32_t* __restrict__ row_exp,
                                                   PermuteArgs perm, CompactArgs cmp, RouteArgs route, ZeroRowsArgs zr) {
  __shared__ ffn::float4_t red[2 * kPrepThreads / 64][64];
  __shared__ uint32_t row_max[16];
  if (route.wg != nullptr) {
    // a token or two: every block routes them itself (route_body.h) instead of a launch of its
    // own doing it beforehand; perm.idx and tok_exp are then this block's own writes
    route_small_body(reinterpret_cast<double*>(&red[0][0]), x, route, perm.P / top_k, H, E, top_k);
    __syncthreads();
  }
  if (perm.idx != nullptr) {
    PermuteLds& pl = *reinterpret_cast<PermuteLds*>(&red[0][0]);     // (the reduction buffer is not in use yet)
    static_assert(sizeof(PermuteLds) <= sizeof(red), "the permutation tables must fit the reduction buffer");
    permute_body(pl, perm.idx, perm.P, E, top_k, top_n, perm.counts, perm.offsets, perm.row_pair, perm.pair_row, perm.comp_counts);
    __syncthreads();
  }
  constexpr int kWavesPerBlock = kPrepThreads / 64, kColLanes = kPrepThreads / 16;
  const int row_blocks = (rows + 15) / 16;
  const int stat_blocks = stat ? (E + kWavesPerBlock - 1) / kWavesPerBlock : 0, plan_block = plan0.B + plan1.B > 0 ? 1 : 0;
  if ((int)blockIdx.x == (int)gridDim.x - 1) {                              // the zero rows (the last block)
    const int n = blockIdx.y * kPrepThreads + threadIdx.x, step = kPrepThreads * gridDim.y;
    const int xu = (H + kTileK - 1) / kTileK * (kTileK / 8);               // 16-byte units per row
    for (int i = n; i < xu * dec::kZeroRows; i += step)
      xg[size_t(i / dec::kZeroRows) * rt + rt - dec::kZeroRows + i % dec::kZeroRows] = make_uint4(0, 0, 0, 0);
    if (zr.h != nullptr)
      for (int i = n; i < zr.Fp / 8 * dec::kZeroRows; i += step)
        zr.h[size_t(i / dec::kZeroRows) * zr.h_rt + zr.h_rt - dec::kZeroRows + i % dec::kZeroRows] = make_uint4(0, 0, 0, 0);
    return;
  }
  if ((int)blockIdx.x >= row_blocks + stat_blocks + plan_block) {          // (x A1 | x A3)
    const int i = (int)blockIdx.x - (row_blocks + stat_blocks + plan_block);
    if (blockIdx.y == 0) ffn::xa_rows_body<true, true, kWavesPerBlock>(xa, x, i % xa_tiles, i / xa_tiles, 0, red);
    return;
  }
  if (plan_block && (int)blockIdx.x == row_blocks + stat_blocks) {         // the block tables (plan.h)
    if (blockIdx.y == 0 && threadIdx.x < 128) make_plan(offsets, E, threadIdx.x < 64 ? plan0 : plan1, threadIdx.x & 63);
    return;
  }
  if ((int)blockIdx.x >= row_blocks) {
    const int e = ((int)blockIdx.x - row_blocks) * kWavesPerBlock + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    if (e >= E || blockIdx.y != 0) return;
    const int b = offsets[e], n = offsets[e + 1] - b;
    // the expert's rows that take the rank-r term, counted and (for the grouped (in A) kernels,
    // CompactArgs) compacted in row order by ballot
    int comp = 0;
    for (int r0 = 0; r0 < n; r0 += 64) {
      const int r = r0 + lane;
      const bool f = r < n && (row_pair[b + min(r, n - 1)] % top_k) < top_n;
      const unsigned long long m = __ballot(f);
      if (cmp.index != nullptr) {
        const int at = b + comp + __popcll(m & ((1ull << lane) - 1ull));
        if (r < n) cmp.index[b + r] = f ? at : -1;
        if (f) cmp.list[at] = b + r;
      }
      comp += __popcll(m);
    }
    if (lane == 0) { stat[2 + e] = n; stat[2 + E + e] = comp; }
    return;
  }
  const int R = blockIdx.x * 16 + (threadIdx.x & 15);
  const int t = R < rows ? (row_pair ? row_pair[R] / top_k : R) : 0;
  const uint4* xrow = reinterpret_cast<const uint4*>(x + size_t(t) * H);
  // The row's power-of-two pre-scale (ffn_common.h): from the routing kernel's per-token exponents,
  // or, without them, from a pass of this block over its sixteen rows.
  int se = 0;
  if (tok_exp != nullptr) {
    se = tok_exp[t];
  } else {
    if (threadIdx.x < 16) row_max[threadIdx.x] = 0;
    __syncthreads();
    uint32_t m = 0;
    if (R < rows)
      for (int k8 = threadIdx.x >> 4; k8 < H / 8; k8 += kColLanes) {
        const uint4 v = xrow[k8];
        const uint32_t in[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) m = max(m, max(in[i] & 0x7fffu, (in[i] >> 16) & 0x7fffu));
      }
    atomicMax(&row_max[threadIdx.x & 15], m);
    __syncthreads();
    se = ffn::row_exponent(row_max[threadIdx.x & 15]);
  }
  if (R >= rows) return;
  if (blockIdx.y == 0 && (threadIdx.x >> 4) == 0) row_exp[R] = se;
  const float sc = ffn::pow2i(se);
  // (grid.y splits the columns when there are few rows, so that the launch still fills the chip)
  // (two adjacent units per thread: a wavefront reads 128 contiguous bytes of each of its rows; H / 8 is even)
  for (int k8p = 2 * (blockIdx.y * kColLanes + (threadIdx.x >> 4)); k8p < H / 8; k8p += 2 * kColLanes * gridDim.y) {
    const uint4 vv[2] = {xrow[k8p], xrow[k8p + 1]};
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const uint32_t in[4] = {vv[u].x, vv[u].y, vv[u].z, vv[u].w};
      uint32_t o[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const _Float16 lo = (_Float16)(bf16_lo(in[i]) * sc);
        const _Float16 hi = (_Float16)(bf16_hi(in[i]) * sc);
        o[i] = uint32_t(__builtin_bit_cast(uint16_t, lo)) | (uint32_t(__builtin_bit_cast(uint16_t, hi)) << 16);
      }
      const int k8 = k8p + u, ks = k8 >> 5, q = (k8 >> 3) & 3, s = k8 & 7;
      xg[size_t((ks * 8 + s) * 4 + q) * rt + R] = make_uint4(o[0], o[1], o[2], o[3]);
    }
  }
}

// One wavefront per packed tile: runs the same field extraction as the FFN kernels and writes the
// integer codes back as one byte each.
template <int BITS>
__global__ __launch_bounds__(64) void unpack_kernel(const uint32_t* __restrict__ packed, int K, int N,
                                                    int KS, uint8_t* __restrict__ codes) {
  const int tile = blockIdx.x, NT = N / kTileN, ks = tile / NT, nt = tile % NT, lane = threadIdx.x;
  uint32_t w[2 * BITS];
  load_codes<BITS>(packed + size_t(tile) * kWave * 2 * BITS, lane, w);
  const int n = nt * kTileN + (lane & 15), kbase = ks * kTileK + (lane >> 4) * kLaneK;
#pragma unroll
  for (int pi = 0; pi < 32; ++pi) {
    const uint32_t f = Extract<BITS>::field(w, pi);
    const int k = kbase + 2 * pi;
    if (k < K) codes[size_t(k) * N + n] = (uint8_t)field_code<BITS>(f & 0xffffu, pi);
    if (k + 1 < K) codes[size_t(k + 1) * N + n] = (uint8_t)field_code<BITS>(f >> 16, pi);
  }
}

}  // namespace

hipError_t launch_combine(const moe_lrc_layer* L, const void* y_rows, const float* y_part, int kblocks, const float* w,
                          const int32_t* pair_row, const void* y_shared, const void* residual, int T, void* out,
                          hipStream_t s) {
  const moe_lrc_config& c = L->cfg;
  // enough blocks for the chip when there are few tokens: up to one per 256 chunks of 8 columns
  const int gy = std::max(1, std::min((c.hidden / 8 + 255) / 256, (2 * L->n_cu + T - 1) / T));
  auto kernel = y_part != nullptr ? combine_kernel<true> : combine_kernel<false>;
  hipLaunchKernelGGL(kernel, dim3(T, gy), dim3(256), 0, s, (const uint16_t*)y_rows, y_part, kblocks,
                     size_t(T) * c.top_k * c.hidden, w, pair_row,
                     (const uint16_t*)y_shared, (const uint16_t*)residual, T, c.hidden, c.top_k, c.n_shared, (uint16_t*)out);
  return hipGetLastError();
}

hipError_t launch_convert_x(const moe_lrc_layer* L, const void* x_bf16, int T, _Float16* xg, int rt,
                            const int32_t* offsets, const int32_t* row_pair, int32_t* stat,
                            const PlanSpec* plans, const FfnArgs* xa13, const int32_t* tok_exp, int32_t* row_exp,
                            const PermuteArgs* perm, const CompactArgs* cmp, const RouteArgs* route, const ZeroRowsArgs& zr,
                            hipStream_t s) {
  const moe_lrc_config& c = L->cfg;
  const int rows = row_pair ? T * c.top_k : T;
  const int row_blocks = (rows + 15) / 16;
  // (a block pass covers 16 * kPrepThreads / 16 columns: two 8-column units per thread)
  const int ky = std::max(1, std::min(c.hidden / (16 * (kPrepThreads / 16)), L->n_cu / std::max(1, row_blocks)));
  const PlanSpec none{0, 0, 0, nullptr};
  const PlanSpec p0 = plans ? plans[0] : none, p1 = plans ? plans[1] : none;
  const int plan_block = p0.B + p1.B > 0 ? 1 : 0;
  // (x A1 | x A3) of the decode flavour: 16-column tiles of both factors, each padded to ls * 32 columns
  ffn::KArgs xa{};
  int xa_tiles = 0;
  if (xa13 && xa13->rank > 0 && xa13->top_n > 0 && row_pair) {
    const FfnArgs& f = *xa13;
    xa.desc = f.desc; xa.offsets = f.offsets; xa.row_pair = f.row_pair; xa.top_k = f.top_k; xa.top_n = f.top_n;
    xa.rank = f.rank; xa.ls = (f.rank + 31) / 32; xa.K = f.H; xa.p = f.p13; xa.total_rows = f.total_rows;
    xa.kb_steps = (f.H + kTileK - 1) / kTileK;
    xa.tok_exp = tok_exp; xa.row_exp = row_exp;
    xa_tiles = 4 * xa.ls;
  }
  const int stat_blocks = stat ? (c.n_experts + kPrepThreads / 64 - 1) / (kPrepThreads / 64) : 0;
  const int cmp_block = (cmp && row_pair && stat) ? 1 : 0;     // (the compaction rides the per-expert counting)
  // (+ 1: the block that keeps the zero rows)
  hipLaunchKernelGGL(prep_kernel, dim3(row_blocks + stat_blocks + plan_block + xa_tiles * c.n_experts + 1, ky),
                     dim3(kPrepThreads), 0, s, (const uint16_t*)x_bf16, rows, c.hidden, reinterpret_cast<uint4*>(xg), rt, offsets,
                     row_pair, c.n_experts, c.top_k, c.top_n, stat, p0, p1, xa_tiles, xa, tok_exp, row_exp,
                     perm ? *perm : PermuteArgs{nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, 0},
                     cmp_block ? *cmp : CompactArgs{nullptr, nullptr},
                     (route && perm) ? *route : RouteArgs{nullptr, nullptr, nullptr, nullptr, nullptr, 0}, zr);
  return hipGetLastError();
}

hipError_t launch_debug_unpack(const uint32_t* packed, const MatLayout& m, uint8_t* codes_dev,
                               hipStream_t s) {
  const dim3 grid(m.NT * m.KS), block(64);
  switch (m.bits) {
    case 2: hipLaunchKernelGGL(unpack_kernel<2>, grid, block, 0, s, packed, m.K, m.N, m.KS, codes_dev); break;
    case 3: hipLaunchKernelGGL(unpack_kernel<3>, grid, block, 0, s, packed, m.K, m.N, m.KS, codes_dev); break;
    case 4: hipLaunchKernelGGL(unpack_kernel<4>, grid, block, 0, s, packed, m.K, m.N, m.KS, codes_dev); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace lrc
