// Expert FFN on grouped rows (Sections 2.3 and 3.2):
//   g = x D1 + c (x A1) B1,  u = x D3 + c (x A3) B3,  h = silu(g) * u,  y = h D2 + c (h A2) B2
// with D = Qinv(Q(W)) unpacked from the bit-packed codes inside the wavefront's registers and
// c = 1 only for rows that hold a Top-n (token, expert) pair.
//
// Kernel design (gfx950): the packed weights are the large, read-once operand, so they never touch
// LDS.  A wavefront owns one n-tile (16 output columns) of a projection and streams its k-steps
// from HBM; each lane unpacks the 64 codes it loaded into packed fp16 pairs with one mask and one
// v_pk_fma_f16 per pair (scale and zero folded into the fma, see unpack.h), which are exactly the
// A-operand registers of v_mfma_f32_16x16x32_f16.  The activations (a few rows, re-used by every
// wavefront) are the operand staged through LDS, already in B-operand register order.
// The rank-r term is appended as r/16 extra MFMA steps on (x A), which a small MFMA kernel
// computes beforehand as split-K partial sums that are added in a fixed order (no atomics).
#include <algorithm>

#include "ffn_common.h"

namespace lrc {

namespace {

using namespace ffn;


// One pass over all k-steps for up to MAXMT row tiles (16 rows each) starting at expert-local row `r`.
//   - activations: staged chunk by chunk (kc k-steps) into LDS in MFMA B-operand order; two
//     barriers per chunk, none inside it;
//   - weights: each wavefront streams its own tiles HBM -> registers through a two-slot ring
//     (the tile of its next-but-one k-step is in flight while it unpacks the current one).
template <int BITS, bool DUAL, int MAXMT>
__device__ inline void ffn_pass(const KArgs& a, const ExpertDesc& d, uint4* xs, int r0, int cnt, int r,
                                int nt, int kw, bool wave_ok) {
  constexpr int NM = DUAL ? 2 : 1;
  constexpr int DW = 2 * BITS;
  constexpr int NC = Extract<BITS>::kClasses;
  constexpr int kRing = ring_depth(BITS, DUAL);
  const int lane = threadIdx.x & 63, th = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(th >> 6);
  const int tdw = kWave * DW;
  const int q = lane >> 4, c = lane & 15;
  const int mt_n = min(MAXMT, (cnt - r + 15) >> 4);
  // k-steps per chunk: as many as fit the LDS buffer for this many row tiles (a power of two)
  const int kc = max(1, (kLdsUnits / 512) >> (mt_n == 1 ? 0 : (mt_n == 2 ? 1 : (mt_n <= 4 ? 2 : 3))));

  // Buffer resources over this wavefront's tile stream and metadata of each projection: a load
  // past the end (a k-step beyond the last, or a wavefront without an n-tile) returns zeros and
  // touches no memory, so every step can issue its refill unconditionally and the count of loads
  // in flight is known statically.
  __amdgpu_buffer_rsrc_t code_rs[NM], meta_rs[NM];
#pragma unroll
  for (int m = 0; m < NM; ++m) {
    const int mat = DUAL ? m : 2;
    code_rs[m] = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint32_t*>(d.codes[mat]), 0,
                                                   wave_ok ? a.KS * a.NT * tdw * 4 : 0, 0x00020000);
    meta_rs[m] = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint32_t*>(d.meta[mat]), 0,
                                                   wave_ok ? a.G * a.NT * kTileN * 4 : 0, 0x00020000);
  }
  const int groups_per_step = kTileK >> a.group_shift;      // 4, 2 or 1
  auto fetch = [&](int ks, Slot<BITS, NM>& sl) {
    // wave-uniform byte offsets of tile (ks, nt) and of its first metadata row; a k-step past the
    // end lands beyond the resource (k-step-major order), so the loads return zeros
    // (offsets go into the per-lane offset operand: that is the one the hardware range-checks)
    const bool ok = ks < a.KS;
    const int tile_off = (ok ? (ks * a.NT + nt) * (tdw * 4) : a.KS * a.NT * tdw * 4) + lane * 16;
    const int tile_off2 = (ok ? (ks * a.NT + nt) * (tdw * 4) : a.KS * a.NT * tdw * 4) + 1024 + lane * (BITS == 3 ? 8 : 16);
    const int meta_off = (ok ? (ks * groups_per_step * a.NT + nt) * (kTileN * 4) : a.G * a.NT * kTileN * 4) +
                         ((q * kLaneK) >> a.group_shift) * (a.NT * kTileN * 4) + c * 4;
#pragma unroll
    for (int m = 0; m < NM; ++m) {
      const u32x4 v0 = __builtin_amdgcn_raw_buffer_load_b128(code_rs[m], tile_off, 0, 0);
      sl.cw[m][0] = v0[0]; sl.cw[m][1] = v0[1]; sl.cw[m][2] = v0[2]; sl.cw[m][3] = v0[3];
      if constexpr (BITS == 3) {
        const u32x2 v1 = __builtin_amdgcn_raw_buffer_load_b64(code_rs[m], tile_off2, 0, 0);
        sl.cw[m][4] = v1[0]; sl.cw[m][5] = v1[1];
      } else if constexpr (BITS == 4) {
        const u32x4 v1 = __builtin_amdgcn_raw_buffer_load_b128(code_rs[m], tile_off2, 0, 0);
        sl.cw[m][4] = v1[0]; sl.cw[m][5] = v1[1]; sl.cw[m][6] = v1[2]; sl.cw[m][7] = v1[3];
      }
      sl.mw[m] = __builtin_amdgcn_raw_buffer_load_b32(meta_rs[m], meta_off, 0, 0);
    }
  };

  // staging: the chunk is mt_n * nk * 512 units of 16 bytes (8 activations of one row); unit u is
  // row u%16 of row tile (u/512)/nk, 8-element column (u/16)%32 of k-step (u/512)%nk.  The input
  // is in operand order (act_unit): rows are contiguous, so 16 lanes read one 256-byte run.  Rows
  // past the expert's last one read whatever follows (their output columns are never stored);
  // columns past K read as zero.
  constexpr int kThreads = 64 * block_waves(MAXMT);
  const int rowl = th & 15;
  const int rin = ((DUAL && !a.offsets) ? 0 : r0) + r;
  const uint4* in_units = reinterpret_cast<const uint4*>(a.in);
  auto stage = [&](int ks0, int nk) {
    const int total = mt_n * nk * 512;
    constexpr int kMaxUnits = (kLdsUnits + kThreads - 1) / kThreads;    // per thread
#pragma unroll
    for (int b = 0; b < kMaxUnits; b += 4) {
      if (th + b * kThreads >= total) break;
      uint4 reg[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int u = th + (b + i) * kThreads;
        reg[i] = make_uint4(0, 0, 0, 0);
        if (u < total) {
          const int k8l = (u >> 4) & 31, mk = u >> 9, mt = mk / nk, kl = mk - mt * nk;
          const int k8 = (ks0 + kl) * 32 + k8l;
          if (k8 * 8 < a.K) reg[i] = in_units[act_unit(k8, rin + 16 * mt + rowl, a.in_rt)];
        }
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int u = th + (b + i) * kThreads;
        if (u < total) {
          const int k8l = (u >> 4) & 31, mk = u >> 9, mt = mk / nk, kl = mk - mt * nk;
          xs[((mt * kc + kl) * 8 + (k8l & 7)) * 64 + (k8l >> 3) * 16 + rowl] = reg[i];
        }
      }
    }
  };

  float4_t acc[MAXMT][NM];
#pragma unroll
  for (int mt = 0; mt < MAXMT; ++mt)
#pragma unroll
    for (int m = 0; m < NM; ++m) acc[mt][m] = float4_t{0.f, 0.f, 0.f, 0.f};

  auto compute = [&](const Slot<BITS, NM>& cur, int kl) {
    const uint4* xk = xs + size_t(kl) * 8 * 64 + lane;
    uint32_t s2[NM][NC], c2[NM];
#pragma unroll
    for (int m = 0; m < NM; ++m) {
      s2[m][0] = (cur.mw[m] & 0xffffu) | (cur.mw[m] << 16);
      c2[m] = (cur.mw[m] >> 16) | (cur.mw[m] & 0xffff0000u);
      constexpr uint32_t step = Extract<BITS>::kStepBits == 2 ? 0x44004400u : 0x48004800u;   // 4.0 or 8.0
#pragma unroll
      for (int p = 1; p < NC; ++p) s2[m][p] = pk_mul(s2[m][p - 1], step);
    }
#pragma unroll
    for (int s = 0; s < 8; ++s) {
      half8_t wf[NM];
#pragma unroll
      for (int m = 0; m < NM; ++m) {
        uint32_t v[4];
#pragma unroll
        for (int j = 0; j < 4; ++j)
          v[j] = pk_fma(Extract<BITS>::field(cur.cw[m], 4 * s + j), s2[m][Extract<BITS>::cls(4 * s + j)], c2[m]);
        wf[m] = __builtin_bit_cast(half8_t, make_uint4(v[0], v[1], v[2], v[3]));
      }
#pragma unroll
      for (int mt = 0; mt < MAXMT; ++mt)
        if (mt < mt_n) {
          const half8_t xf = __builtin_bit_cast(half8_t, xk[(size_t(mt) * kc * 8 + s) * 64]);
#pragma unroll
          for (int m = 0; m < NM; ++m)
            acc[mt][m] = __builtin_amdgcn_mfma_f32_16x16x32_f16(wf[m], xf, acc[mt][m], 0, 0, 0);
        }
      // keep the sub-steps in order: hoisting later unpacks above these MFMAs only costs registers,
      // the other wavefronts of the SIMD hide the latency
      if (MAXMT <= 2 && (s & 1)) __builtin_amdgcn_sched_barrier(0);
    }
  };

  // Ring of kRing slots, walked by a loop unrolled kRing times so that every slot index is static:
  // slot i holds this wavefront's own k-steps i, i + kRing, ...  A slot is refilled right after it
  // has been consumed, so kRing - 1 tiles stay in flight during an unpack.  All wavefronts of the
  // block take the same number of steps (the k-steps of one step lie in the same chunk because
  // the chunk length is a multiple of kw), so the barriers around the staging are uniform.
  Slot<BITS, NM> ring[kRing];
#pragma unroll
  for (int i = 0; i < kRing; ++i) fetch(kw + i * a.kw, ring[i]);
  const int n_steps = (a.KS + a.kw - 1) / a.kw;
  for (int j0 = 0; j0 < n_steps; j0 += kRing) {
#pragma unroll
    for (int i = 0; i < kRing; ++i) {
      const int ksb = (j0 + i) * a.kw;     // first k-step of this step, block-uniform
      if (ksb < a.KS) {
        if (ksb % kc == 0) {
          __syncthreads();                 // everyone is done with the previous chunk
          stage(ksb, min(kc, a.KS - ksb));
          __syncthreads();
        }
#ifndef LRC_EXP_NOCOMPUTE
        if (wave_ok && ksb + kw < a.KS) compute(ring[i], (ksb + kw) % kc);
#else
        if (wave_ok && ksb + kw < a.KS) { acc[0][0][0] += __uint_as_float(ring[i].cw[0][0] ^ ring[i].cw[NM-1][3] ^ ring[i].mw[0]); }
#endif
      }
#ifndef LRC_EXP_NOFETCH
      fetch(ksb + kw + kRing * a.kw, ring[i]);
#endif
    }
  }

  // ---- wavefronts that shared an n-tile add up their partial sums through LDS ----
  if (a.kw > 1) {
    float4_t* red = reinterpret_cast<float4_t*>(xs);
    __syncthreads();
    if (kw != 0) {
#pragma unroll
      for (int mt = 0; mt < MAXMT; ++mt)
        if (mt < mt_n)
#pragma unroll
          for (int m = 0; m < NM; ++m) red[((wave * MAXMT + mt) * NM + m) * 64 + lane] = acc[mt][m];
    }
    __syncthreads();
    if (kw == 0) {
      for (int j = 1; j < a.kw; ++j)
#pragma unroll
        for (int mt = 0; mt < MAXMT; ++mt)
          if (mt < mt_n)
#pragma unroll
            for (int m = 0; m < NM; ++m) acc[mt][m] += red[(((wave + j) * MAXMT + mt) * NM + m) * 64 + lane];
    }
  }
  if (kw != 0 || !wave_ok) return;

  // ---- rank-r term: r/16 more MFMA steps, weights = packed B factor, activations = (in A) ----
  const int PW = DUAL ? 2 * a.rpad : a.rpad;
#pragma unroll
  for (int mt = 0; mt < MAXMT; ++mt) {
    if (mt >= mt_n) continue;
    const int row = r + 16 * mt + c;   // this lane's token column of the tile
    bool flagged = false;
    if (a.rank > 0 && d.has_factors && a.row_pair != nullptr && row < cnt)
      flagged = (a.row_pair[r0 + row] % a.top_k) < a.top_n;
    if (__ballot(flagged) != 0ull) {
      const int rs = a.rpad / 16;
#pragma unroll
      for (int m = 0; m < NM; ++m) {
        const int mat = DUAL ? m : 2;
        const float lam = d.lambda[mat];
        for (int st = 0; st < rs; ++st) {
          float4_t pv = float4_t{0.f, 0.f, 0.f, 0.f};
          if (flagged) {
            const float* pp = a.p + size_t(r0 + row) * PW + m * a.rpad + 16 * st + 4 * q;
            for (int sp = 0; sp < a.ksplit; ++sp)
              pv += *reinterpret_cast<const float4_t*>(pp + size_t(sp) * a.total_rows * PW);
          }
          const half4_t pf = half4_t{(_Float16)(pv[0] * lam), (_Float16)(pv[1] * lam),
                                     (_Float16)(pv[2] * lam), (_Float16)(pv[3] * lam)};
          // B factor: [N/16][ceil(rank/32)][lane][8], 32 rank indices per unit row; this step's 16
          const int ls = (a.rank + 31) / 32;
          const half4_t bfr = *reinterpret_cast<const half4_t*>(
              d.bf[mat] + ((size_t(nt) * ls + (st >> 1)) * kWave + (2 * (st & 1) + (q >> 1)) * 16 + c) * 8 + 4 * (q & 1));
          acc[mt][m] = __builtin_amdgcn_mfma_f32_16x16x16f16(bfr, pf, acc[mt][m], 0, 0, 0);
        }
      }
    }
  }

  // ---- epilogue: lane holds output columns 16*nt + 4*q .. +3 of token column c ----
#pragma unroll
  for (int mt = 0; mt < MAXMT; ++mt) {
    const int row = r + 16 * mt + c;
    if (mt >= mt_n || row >= cnt) continue;
    const size_t o = size_t(r0 + row) * a.N + nt * kTileN + 4 * q;
    if constexpr (DUAL) {
      const float i1 = d.inv_lambda[0], i3 = d.inv_lambda[1];
      half4_t hv;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float g = acc[mt][0][i] * i1, u = acc[mt][1][i] * i3;
        hv[i] = (_Float16)(g * __builtin_amdgcn_rcpf(1.0f + __expf(-g)) * u);
      }
      const int f = nt * kTileN + 4 * q;      // h in operand order for the W2 kernel
      *reinterpret_cast<half4_t*>(reinterpret_cast<_Float16*>(a.out) + act_unit(f >> 3, r0 + row, a.out_rt) * 8 + (f & 7)) = hv;
    } else {
      const float i2 = d.inv_lambda[2];
      uint2 yv;
      yv.x = f32x2_to_bf16x2(acc[mt][0][0] * i2, acc[mt][0][1] * i2);
      yv.y = f32x2_to_bf16x2(acc[mt][0][2] * i2, acc[mt][0][3] * i2);
      *reinterpret_cast<uint2*>(reinterpret_cast<uint16_t*>(a.out) + o) = yv;
    }
  }
}

// grid = (ceil(NT * kw / waves), experts); a block of `waves` wavefronts covers waves / kw n-tiles.
// MAXMT = 2: decode flavour, 128 registers, 16 wavefronts per CU.  MAXMT = 8: many rows per expert,
// one unpack serves up to 128 rows, 256 registers.
template <int BITS, bool DUAL, int MAXMT>
__global__ __launch_bounds__(64 * block_waves(MAXMT), MAXMT <= 2 ? LRC_DECODE_MINW : 2) void qgemm_kernel(KArgs a) {
  __shared__ uint4 xs[kLdsUnits];
  const int e = blockIdx.y;
  const int r0 = a.offsets ? a.offsets[e] : e * a.T;
  const int cnt = a.offsets ? a.offsets[e + 1] - r0 : a.T;
  if (cnt == 0) return;
  const ExpertDesc& d = a.desc[e];
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int kw = wave % a.kw;
  const int nt = blockIdx.x * (block_waves(MAXMT) / a.kw) + wave / a.kw;
  const bool wave_ok = nt < a.NT;
  for (int r = 0; r < cnt; r += 16 * MAXMT) ffn_pass<BITS, DUAL, MAXMT>(a, d, xs, r0, cnt, r, nt, kw, wave_ok);
}

// p[sp][row][rho] = sum over k-slice sp of in[row][k] * A[k][rho], for rows that take the rank-r
// term.  grid = (ksplit, experts); wavefronts loop over 16-column tiles of the factor(s).
template <bool DUAL>
__global__ __launch_bounds__(256) void xa_kernel(KArgs a) {
  const int e = blockIdx.y, sp = blockIdx.x;
  const int r0 = a.offsets[e], cnt = a.offsets[e + 1] - r0;
  const ExpertDesc& d = a.desc[e];
  if (cnt == 0 || !d.has_factors) return;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, c = lane & 15, q = lane >> 4;
  const int rt = a.rpad / 16, tiles = DUAL ? 2 * rt : rt, PW = tiles * 16;
  const int k32 = a.K / 32, per = (k32 + a.ksplit - 1) / a.ksplit;
  const int kk0 = sp * per, kk1 = min(k32, kk0 + per);
  for (int r = 0; r < cnt; r += 16) {
    const int row = r + c;
    bool flagged = false;
    if (row < cnt) flagged = (a.row_pair[r0 + row] % a.top_k) < a.top_n;
    if (__ballot(flagged) == 0ull) continue;
    const half8_t* src = reinterpret_cast<const half8_t*>(a.in);   // operand order: unit (k8, row)
    for (int tile = wave; tile < tiles; tile += 4) {
      const int mat = DUAL ? (tile >= rt ? 1 : 0) : 2;
      const int tl = DUAL && tile >= rt ? tile - rt : tile;
      const _Float16* af = d.af[mat];
      float4_t acc = float4_t{0.f, 0.f, 0.f, 0.f};
      for (int kk = kk0; kk < kk1; ++kk) {
        const half8_t wf = *reinterpret_cast<const half8_t*>(af + ((size_t(kk) * rt + tl) * kWave + lane) * 8);
        half8_t xf = half8_t{0, 0, 0, 0, 0, 0, 0, 0};
        if (flagged) xf = src[act_unit(4 * kk + q, r0 + row, a.in_rt)];
        acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(wf, xf, acc, 0, 0, 0);
      }
      if (flagged)
        *reinterpret_cast<float4_t*>(const_cast<float*>(a.p) + (size_t(sp) * a.total_rows + r0 + row) * PW +
                                     16 * tile + 4 * q) = acc;
    }
  }
}

// Wavefronts per n-tile: enough split-K that the launch fills the chip (~16 wavefronts per CU)
// even when few experts are active.
int pick_kw(int tasks, int waves, int cap) {
  int best = 1;
  for (int kw = 1; kw <= cap; kw *= 2)
    if (waves % kw == 0) {
      best = kw;
      if (tasks * kw >= 3072) break;
    }
  return best;
}

template <int BITS, int MAXMT>
hipError_t launch_bits(const FfnArgs& f, hipStream_t s) {
  int gs = 0;
  while ((1 << gs) < f.group) ++gs;
  KArgs a{};
  a.desc = f.desc; a.offsets = f.offsets; a.row_pair = f.row_pair;
  a.group_shift = gs; a.top_k = f.top_k; a.top_n = f.top_n; a.T = f.T;
  a.rank = f.rank; a.rpad = f.rpad; a.total_rows = f.total_rows;
  const bool comp = f.rank > 0 && f.top_n > 0 && f.row_pair != nullptr;
  // experts that can be active at all: at most one per routed pair
  const int max_active = f.offsets ? std::min(f.n_exp, f.T * f.top_k) : f.n_exp;
  // an expert can hold up to T rows; with more than 16 a chunk holds fewer k-steps than 8, and the
  // split-K partial sums of a block must fit its 64 KB of LDS
  const int kc_max = kLdsUnits / 512;
  const int kw_cap = f.T <= 16 ? kc_max : (f.T <= 32 ? kc_max / 2 : (MAXMT <= 2 ? std::max(1, kc_max / 4) : 1));
  constexpr int kWaves = block_waves(MAXMT);   // kw must divide both this and the chunk length

  // W1 | W3 with the SwiGLU epilogue
  a.in = f.xh; a.out = f.h; a.K = f.H; a.N = f.F; a.NT = f.F / kTileN;
  a.in_rt = f.x_rt; a.out_rt = f.h_rt;
  a.KS = padded_k(f.H) / kTileK; a.G = padded_k(f.H) / f.group;
  a.p = f.p13; a.ksplit = f.ksplit13;
  a.kw = pick_kw(max_active * a.NT, kWaves, std::min(kw_cap, a.KS));
  if (comp) hipLaunchKernelGGL(xa_kernel<true>, dim3(a.ksplit, f.n_exp), dim3(256), 0, s, a);
  if (f.marks) (void)hipEventRecord(f.marks[0], s);
  hipLaunchKernelGGL((qgemm_kernel<BITS, true, MAXMT>), dim3((a.NT * a.kw + kWaves - 1) / kWaves, f.n_exp),
                     dim3(64 * kWaves), 0, s, a);
  if (f.marks) (void)hipEventRecord(f.marks[1], s);
  // W2
  a.in = f.h; a.out = f.y_rows; a.K = f.F; a.N = f.H; a.NT = f.H / kTileN;
  a.in_rt = f.h_rt; a.out_rt = 0;
  a.KS = padded_k(f.F) / kTileK; a.G = padded_k(f.F) / f.group;
  a.p = f.p2; a.ksplit = f.ksplit2;
  a.kw = pick_kw(max_active * a.NT, kWaves, std::min(kw_cap, a.KS));
  if (comp) hipLaunchKernelGGL(xa_kernel<false>, dim3(a.ksplit, f.n_exp), dim3(256), 0, s, a);
  if (f.marks) (void)hipEventRecord(f.marks[2], s);
  hipLaunchKernelGGL((qgemm_kernel<BITS, false, MAXMT>), dim3((a.NT * a.kw + kWaves - 1) / kWaves, f.n_exp),
                     dim3(64 * kWaves), 0, s, a);
  if (f.marks) (void)hipEventRecord(f.marks[3], s);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_expert_ffn(const FfnArgs& f, hipStream_t s) {
  // expected rows per expert under uniform routing decides the flavour
  const int rows = f.offsets ? (f.T * f.top_k + f.n_exp - 1) / f.n_exp : f.T;
  if (rows <= 24) return launch_decode_ffn(f, s);
  switch (f.bits) {
    case 2: return launch_bits<2, 8>(f, s);
    case 3: return launch_bits<3, 8>(f, s);
    case 4: return launch_bits<4, 8>(f, s);
  }
  return hipErrorInvalidValue;
}

}  // namespace lrc
