// Expert FFN on grouped rows (Sections 2.3 and 3.2):
//   g = x D1 + c (x A1) B1,  u = x D3 + c (x A3) B3,  h = silu(g) * u,  y = h D2 + c (h A2) B2
// with D = Qinv(Q(W)) unpacked from the bit-packed codes inside the wavefront's registers and
// c = 1 only for rows that hold a Top-n (token, expert) pair.
//
// Kernel design (gfx950): the packed weights are the large, read-once operand, so they never touch
// LDS.  A wavefront owns one n-tile (16 output columns) of a projection and streams its k-steps
// from HBM; each lane unpacks the 64 codes it loaded into packed fp16 pairs with one shift, one mask
// and one v_pk_fma_f16 per pair (scale and zero folded into the fma), which are exactly the
// A-operand registers of v_mfma_f32_16x16x32_f16.  The activations (a few rows, re-used by every
// wavefront) are the operand staged through LDS, already in B-operand register order.
// The rank-r term is appended as r/16 extra MFMA steps on (x A), which a small MFMA kernel
// computes beforehand as split-K partial sums that are added in a fixed order (no atomics).
#include "internal.h"
#include "unpack.h"

namespace lrc {

namespace {

typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef float float4_t __attribute__((ext_vector_type(4)));

constexpr int kMT = 2;            // row tiles (16 rows each) a block handles per pass
constexpr int kBlockWaves = 4;    // n-tiles per block

__device__ inline uint32_t pk_fma(uint32_t q, uint32_t s, uint32_t c) {
  const half2_t r = __builtin_elementwise_fma(__builtin_bit_cast(half2_t, q),
                                              __builtin_bit_cast(half2_t, s),
                                              __builtin_bit_cast(half2_t, c));
  return __builtin_bit_cast(uint32_t, r);
}

struct KArgs {
  const ExpertDesc* desc;
  const int32_t* offsets;    // null: shared experts, expert e owns rows e*T .. e*T+T-1
  const int32_t* row_pair;   // null: rows are tokens
  const _Float16* in;        // DUAL: xh [T][K];  else h [rows][K]
  void* out;                 // DUAL: h [rows][N] fp16; else y_rows [rows][N] bf16
  const float* p;            // split-K partials of (in A): [ksplit][total_rows][PW]
  int K, N, KS, G, group_shift, top_k, top_n, T, rank, rpad, ksplit, total_rows;
};

__device__ inline uint32_t f32x2_to_bf16x2(float a, float b) {
  uint32_t ua = __float_as_uint(a), ub = __float_as_uint(b);
  ua += 0x7fffu + ((ua >> 16) & 1u);
  ub += 0x7fffu + ((ub >> 16) & 1u);
  return (ua >> 16) | (ub & 0xffff0000u);
}

// One pass over all k-steps for MT row tiles starting at expert-local row `r`.
template <int BITS, bool DUAL, int MT>
__device__ inline void ffn_pass(const KArgs& a, const ExpertDesc& d, uint4 (*xs)[kMT][8][64], int r0,
                                int cnt, int r, int nt) {
  constexpr int NM = DUAL ? 2 : 1;
  constexpr int DW = 2 * BITS;
  const int lane = threadIdx.x & 63, th = threadIdx.x;
  const int tdw = kWave * DW;

  const uint32_t* codes[NM];
  const uint32_t* meta[NM];
#pragma unroll
  for (int m = 0; m < NM; ++m) {
    const int mat = DUAL ? m : 2;
    codes[m] = d.codes[mat] + size_t(nt) * a.KS * tdw;
    meta[m] = d.meta[mat] + size_t(nt) * a.G * kTileN;
  }

  // staging assignment: unit i of this thread is (row tile i/2, row th%16, 8-element column th/16 + 16*(i%2))
  const int rowl = th & 15;
  const _Float16* src[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    const int row = r + 16 * mt + rowl;
    src[mt] = nullptr;
    if (row < cnt) {
      const int R = r0 + row;
      int in_row;
      if (DUAL) in_row = a.row_pair ? a.row_pair[R] / a.top_k : (R % a.T);
      else in_row = R;
      src[mt] = a.in + size_t(in_row) * a.K;
    }
  }
  auto stage_load = [&](int ks, uint4 (&reg)[2 * MT]) {
#pragma unroll
    for (int i = 0; i < 2 * MT; ++i) {
      const int k = ks * kTileK + 8 * ((th >> 4) + 16 * (i & 1));
      reg[i] = make_uint4(0, 0, 0, 0);
      if (src[i >> 1] != nullptr && k < a.K) reg[i] = *reinterpret_cast<const uint4*>(src[i >> 1] + k);
    }
  };
  auto stage_store = [&](int buf, const uint4 (&reg)[2 * MT]) {
#pragma unroll
    for (int i = 0; i < 2 * MT; ++i) {
      const int k8 = (th >> 4) + 16 * (i & 1);
      xs[buf][i >> 1][k8 & 7][(k8 >> 3) * 16 + rowl] = reg[i];
    }
  };

  float4_t acc[MT][NM];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int m = 0; m < NM; ++m) acc[mt][m] = float4_t{0.f, 0.f, 0.f, 0.f};

  uint32_t cw[NM][DW], cw_next[NM][DW], mw[NM], mw_next[NM];
  uint4 xreg[2 * MT];
  const int q = lane >> 4, c = lane & 15;
  auto fetch = [&](int ks, uint32_t (&cwd)[NM][DW], uint32_t (&mwd)[NM]) {
#pragma unroll
    for (int m = 0; m < NM; ++m) {
      load_codes<BITS>(codes[m] + size_t(ks) * tdw, lane, cwd[m]);
      mwd[m] = meta[m][((ks * kTileK + q * kLaneK) >> a.group_shift) * kTileN + c];
    }
  };

  stage_load(0, xreg);
  fetch(0, cw_next, mw_next);
  stage_store(0, xreg);
  __syncthreads();

  for (int ks = 0; ks < a.KS; ++ks) {
#pragma unroll
    for (int m = 0; m < NM; ++m) {
#pragma unroll
      for (int i = 0; i < DW; ++i) cw[m][i] = cw_next[m][i];
      mw[m] = mw_next[m];
    }
    const bool more = ks + 1 < a.KS;
    if (more) {
      fetch(ks + 1, cw_next, mw_next);
      stage_load(ks + 1, xreg);
    }
    const int buf = ks & 1;
#pragma unroll
    for (int m = 0; m < NM; ++m) {
      uint32_t f[32];
      Extract<BITS>::run(cw[m], f);
      const uint32_t s2 = (mw[m] & 0xffffu) | (mw[m] << 16);
      const uint32_t c2 = (mw[m] >> 16) | (mw[m] & 0xffff0000u);
#pragma unroll
      for (int s = 0; s < 8; ++s) {
        const uint4 wv = make_uint4(pk_fma(f[4 * s], s2, c2), pk_fma(f[4 * s + 1], s2, c2),
                                    pk_fma(f[4 * s + 2], s2, c2), pk_fma(f[4 * s + 3], s2, c2));
        const half8_t wf = __builtin_bit_cast(half8_t, wv);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
          const half8_t xf = __builtin_bit_cast(half8_t, xs[buf][mt][s][lane]);
          acc[mt][m] = __builtin_amdgcn_mfma_f32_16x16x32_f16(wf, xf, acc[mt][m], 0, 0, 0);
        }
      }
    }
    if (more) stage_store(buf ^ 1, xreg);
    __syncthreads();
  }

  // ---- rank-r term: r/16 more MFMA steps, weights = packed B factor, activations = (in A) ----
  const int PW = DUAL ? 2 * a.rpad : a.rpad;
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
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
          const half4_t bfr = *reinterpret_cast<const half4_t*>(
              d.bf[mat] + ((size_t(nt) * rs + st) * kWave + lane) * 4);
          acc[mt][m] = __builtin_amdgcn_mfma_f32_16x16x16f16(bfr, pf, acc[mt][m], 0, 0, 0);
        }
      }
    }
  }

  // ---- epilogue: lane holds output columns 16*nt + 4*q .. +3 of token column c ----
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    const int row = r + 16 * mt + c;
    if (row >= cnt) continue;
    const size_t o = size_t(r0 + row) * a.N + nt * kTileN + 4 * q;
    if constexpr (DUAL) {
      const float i1 = d.inv_lambda[0], i3 = d.inv_lambda[1];
      half4_t hv;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float g = acc[mt][0][i] * i1, u = acc[mt][1][i] * i3;
        hv[i] = (_Float16)(g / (1.0f + expf(-g)) * u);
      }
      *reinterpret_cast<half4_t*>(reinterpret_cast<_Float16*>(a.out) + o) = hv;
    } else {
      const float i2 = d.inv_lambda[2];
      uint2 yv;
      yv.x = f32x2_to_bf16x2(acc[mt][0][0] * i2, acc[mt][0][1] * i2);
      yv.y = f32x2_to_bf16x2(acc[mt][0][2] * i2, acc[mt][0][3] * i2);
      *reinterpret_cast<uint2*>(reinterpret_cast<uint16_t*>(a.out) + o) = yv;
    }
  }
}

template <int BITS, bool DUAL>
__global__ __launch_bounds__(256) void qgemm_kernel(KArgs a) {
  __shared__ uint4 xs[2][kMT][8][64];     // activations in MFMA B-operand order, double buffered
  const int e = blockIdx.y;
  const int r0 = a.offsets ? a.offsets[e] : e * a.T;
  const int cnt = a.offsets ? a.offsets[e + 1] - r0 : a.T;
  if (cnt == 0) return;
  const ExpertDesc& d = a.desc[e];
  const int nt = blockIdx.x * kBlockWaves + (threadIdx.x >> 6);
  for (int r = 0; r < cnt; r += 16 * kMT) {
    if (cnt - r <= 16) ffn_pass<BITS, DUAL, 1>(a, d, xs, r0, cnt, r, nt);
    else ffn_pass<BITS, DUAL, kMT>(a, d, xs, r0, cnt, r, nt);
  }
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
    const _Float16* src = nullptr;
    if (row < cnt) {
      const int pair = a.row_pair[r0 + row];
      flagged = (pair % a.top_k) < a.top_n;
      src = a.in + size_t(DUAL ? pair / a.top_k : r0 + row) * a.K;
    }
    if (__ballot(flagged) == 0ull) continue;
    for (int tile = wave; tile < tiles; tile += 4) {
      const int mat = DUAL ? (tile >= rt ? 1 : 0) : 2;
      const int tl = DUAL && tile >= rt ? tile - rt : tile;
      const _Float16* af = d.af[mat];
      float4_t acc = float4_t{0.f, 0.f, 0.f, 0.f};
      for (int kk = kk0; kk < kk1; ++kk) {
        const half8_t wf = *reinterpret_cast<const half8_t*>(af + ((size_t(kk) * rt + tl) * kWave + lane) * 8);
        half8_t xf = half8_t{0, 0, 0, 0, 0, 0, 0, 0};
        if (flagged) xf = *reinterpret_cast<const half8_t*>(src + 32 * kk + 8 * q);
        acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(wf, xf, acc, 0, 0, 0);
      }
      if (flagged)
        *reinterpret_cast<float4_t*>(const_cast<float*>(a.p) + (size_t(sp) * a.total_rows + r0 + row) * PW +
                                     16 * tile + 4 * q) = acc;
    }
  }
}

template <int BITS>
hipError_t launch_bits(const FfnArgs& f, hipStream_t s) {
  int gs = 0;
  while ((1 << gs) < f.group) ++gs;
  KArgs a{};
  a.desc = f.desc; a.offsets = f.offsets; a.row_pair = f.row_pair;
  a.group_shift = gs; a.top_k = f.top_k; a.top_n = f.top_n; a.T = f.T;
  a.rank = f.rank; a.rpad = f.rpad; a.total_rows = f.total_rows;
  const bool comp = f.rank > 0 && f.top_n > 0 && f.row_pair != nullptr;

  // W1 | W3 with the SwiGLU epilogue
  a.in = f.xh; a.out = f.h; a.K = f.H; a.N = f.F;
  a.KS = padded_k(f.H) / kTileK; a.G = padded_k(f.H) / f.group;
  a.p = f.p13; a.ksplit = f.ksplit13;
  if (comp) hipLaunchKernelGGL(xa_kernel<true>, dim3(a.ksplit, f.n_exp), dim3(256), 0, s, a);
  if (f.marks) (void)hipEventRecord(f.marks[0], s);
  hipLaunchKernelGGL((qgemm_kernel<BITS, true>), dim3(f.F / (kTileN * kBlockWaves), f.n_exp), dim3(256), 0, s, a);
  if (f.marks) (void)hipEventRecord(f.marks[1], s);
  // W2
  a.in = f.h; a.out = f.y_rows; a.K = f.F; a.N = f.H;
  a.KS = padded_k(f.F) / kTileK; a.G = padded_k(f.F) / f.group;
  a.p = f.p2; a.ksplit = f.ksplit2;
  if (comp) hipLaunchKernelGGL(xa_kernel<false>, dim3(a.ksplit, f.n_exp), dim3(256), 0, s, a);
  if (f.marks) (void)hipEventRecord(f.marks[2], s);
  hipLaunchKernelGGL((qgemm_kernel<BITS, false>), dim3(f.H / (kTileN * kBlockWaves), f.n_exp), dim3(256), 0, s, a);
  if (f.marks) (void)hipEventRecord(f.marks[3], s);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_expert_ffn(const FfnArgs& f, hipStream_t s) {
  switch (f.bits) {
    case 2: return launch_bits<2>(f, s);
    case 3: return launch_bits<3>(f, s);
    case 4: return launch_bits<4>(f, s);
  }
  return hipErrorInvalidValue;
}

}  // namespace lrc
