// Decode flavour of the expert FFN (Sections 2.3 and 3.2): few rows per expert, so the layer is a
// stream of packed weights and the job is to keep HBM busy.
//
//   - one block of 16 wavefronts per CU; the grid is (blocks per expert, experts) and the host picks
//     the blocks per expert so that the active experts alone fill the chip;
//   - the activations of the expert (up to 32 rows) are staged into 128 KB of LDS once per phase of
//     16 (or 8) k-steps, every load of a phase issued before the first is awaited: the W1|W3 kernel
//     of a 4096-wide model has a single phase, i.e. one barrier pair per block;
//   - a block's n-tiles are dealt to its wavefronts (two tiles each when there are more than 16,
//     several wavefronts per tile, each taking every kw-th k-step, when there are fewer);
//   - each wavefront streams its packed tiles HBM -> registers with buffer loads through a
//     ring of register slots walked by straight-line code: a load past the end of the resource returns
//     zeros, so refills are unconditional and the number of loads in flight is static;
//   - codes are unpacked in registers (unpack.h) straight into MFMA A-operands; the rank-r term is
//     r/16 more MFMA steps on the pre-computed (x A): xa_split_kernel leaves K-block partial sums,
//     which a block adds in a fixed order into LDS when it starts.
#include <algorithm>

#include "ffn_common.h"

namespace lrc {

namespace {

using namespace ffn;

constexpr int kDecodeWaves = 16;
constexpr int kDecodeLdsUnits = 8192;     // 128 KB in 16-byte units
constexpr int kTPW = 2;                   // n-tiles per wavefront (at most)
constexpr int kDMT = 2;                   // row tiles per pass
// packed tiles a wavefront holds in registers (one being unpacked, the others in flight), chosen
// per kernel so that it stays within 128 registers at 16 wavefronts per CU
#ifndef LRC_DRING_DUAL2
#define LRC_DRING_DUAL2 2
#endif
#ifndef LRC_DRING_DUALW
#define LRC_DRING_DUALW 2
#endif
#ifndef LRC_DRING_SINGLE
#define LRC_DRING_SINGLE 4
#endif
__host__ __device__ constexpr int decode_ring(int bits, bool dual) {
  return dual ? (bits == 2 ? LRC_DRING_DUAL2 : LRC_DRING_DUALW) : LRC_DRING_SINGLE;
}

#ifdef LRC_TIMELINE
// development aid (variant builds only): per-block time stamps of the last decode kernels
__device__ long long g_timeline[2][4096][16];
#define LRC_STAMP(slot)                                                                         \
  do {                                                                                          \
    if (threadIdx.x == 0 && blockIdx.y * gridDim.x + blockIdx.x < 4096)                         \
      g_timeline[DUAL ? 0 : 1][blockIdx.y * gridDim.x + blockIdx.x][slot] = wall_clock64();     \
  } while (0)
#else
#define LRC_STAMP(slot) do {} while (0)
#endif

template <int BITS, bool DUAL>
__global__ __launch_bounds__(64 * kDecodeWaves, 4) void qgemm_decode_kernel(KArgs a) {
  extern __shared__ uint4 xs[];
  constexpr int NM = DUAL ? 2 : 1;
  constexpr int DW = 2 * BITS;
  constexpr int NC = Extract<BITS>::kClasses;
  constexpr int RING = decode_ring(BITS, DUAL);
  const int e = blockIdx.y;
  const int r0 = a.offsets ? a.offsets[e] : e * a.T;
  const int cnt = a.offsets ? a.offsets[e + 1] - r0 : a.T;
  if (cnt == 0) return;
  const ExpertDesc& d = a.desc[e];
  const int th = threadIdx.x, lane = th & 63;
  const int wave = __builtin_amdgcn_readfirstlane(th >> 6);
  const int q = lane >> 4, c = lane & 15, rowl = th & 15;
  const int tdw = kWave * DW;
  LRC_STAMP(0);

  // this block's n-tiles, and how they are dealt to the 16 wavefronts
  const int G = gridDim.x, b = blockIdx.x;
  const int t0 = (int)((long long)b * a.NT / G), t1 = (int)((long long)(b + 1) * a.NT / G);
  const int nt_b = t1 - t0;
  if (nt_b == 0) return;
  int kw = 1;
  while (kw < kDecodeWaves && nt_b * kw * 2 <= kDecodeWaves) kw *= 2;
  const int groups = kDecodeWaves / kw;              // wavefront groups, one n-tile (per slot) each
  const int grp = wave / kw, kwi = wave % kw;

  // this block's K-block: k-steps ks_lo .. ks_lo + KSl - 1
  const int kb = blockIdx.z, ks_lo = kb * a.kb_steps, KSl = min(a.KS, ks_lo + a.kb_steps) - ks_lo;
  const int code_bytes = a.KS * a.NT * tdw * 4, meta_bytes = a.G * a.NT * kTileN * 4;
  __amdgpu_buffer_rsrc_t code_rs[NM], meta_rs[NM];
#pragma unroll
  for (int m = 0; m < NM; ++m) {
    const int mat = DUAL ? m : 2;
    code_rs[m] = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint32_t*>(d.codes[mat]), 0, code_bytes, 0x00020000);
    meta_rs[m] = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint32_t*>(d.meta[mat]), 0, meta_bytes, 0x00020000);
  }
  const int gps = kTileK >> a.group_shift;           // groups per k-step
  const int meta_lane = ((q * kLaneK) >> a.group_shift) * (a.NT * kTileN * 4) + c * 4;

  for (int r = 0; r < cnt; r += 16 * kDMT) {
    const int mt_n = min(kDMT, (cnt - r + 15) >> 4);
    const int KP = (kDecodeLdsUnits / 512) / mt_n;   // k-steps per phase: 16 or 8
    const int n_ph = (KSl + KP - 1) / KP;
    const int spw = (KP + kw - 1) / kw;              // own steps per (tile, phase) segment
    const int SP = (spw + RING - 1) / RING * RING;   // padded to the ring depth: slot indices stay static
    const int n_total = n_ph * kTPW * SP;

    // flat step n -> (phase, tile slot, own step); a step that does not exist loads from past the
    // end of the resources and gets zeros
    auto fetch = [&](int n, Slot<BITS, NM>& sl) {
      const int seg = n / SP, si = n - seg * SP, ph = seg / kTPW, ts = seg - ph * kTPW;
      const int kl = si * kw + kwi, ksl = ph * KP + kl, ks = ks_lo + ksl, tile = t0 + grp + ts * groups;
      const bool ok = n < n_total && kl < KP && ksl < KSl && tile < t1;
      // the offsets go into the per-lane offset operand: that is the one the hardware range-checks
      const int tile_off = (ok ? (ks * a.NT + tile) * (tdw * 4) : code_bytes) + lane * 16;
      const int tile_off2 = (ok ? (ks * a.NT + tile) * (tdw * 4) : code_bytes) + 1024 + lane * (BITS == 3 ? 8 : 16);
      const int meta_off = (ok ? (ks * gps * a.NT + tile) * (kTileN * 4) : meta_bytes) + meta_lane;
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

    // first input row of this pass (shared experts all read the token rows 0..T-1), and whether
    // this lane's token column (th%16 of each row tile) takes the rank-r term
    const int rin = ((DUAL && !a.offsets) ? 0 : r0) + r;
    bool flag[kDMT];
    const bool lowrank = a.rank > 0 && d.has_factors && a.row_pair != nullptr && kb == 0;
#pragma unroll
    for (int mt = 0; mt < kDMT; ++mt) {
      const int row = r + 16 * mt + rowl;
      flag[mt] = false;
      if (lowrank && mt < mt_n && row < cnt) flag[mt] = (a.row_pair[r0 + row] % a.top_k) < a.top_n;
    }
    // (in A) of this pass's rows: the K-block partial sums of xa_split_kernel are added here, in
    // K-block order, and kept in LDS as fp16 behind the activations (zero for rows without the term)
    const int PW = DUAL ? 2 * a.rpad : a.rpad;
    _Float16* p_lds = reinterpret_cast<_Float16*>(xs + kDecodeLdsUnits);
    auto load_p = [&]() {
      for (int e2 = th; e2 < 16 * PW; e2 += 64 * kDecodeWaves) {      // pairs of adjacent columns
        const int row = (2 * e2) / PW, col = (2 * e2) - row * PW;
        float sx = 0.f, sy = 0.f;
        if (r + row < cnt && (a.row_pair[r0 + r + row] % a.top_k) < a.top_n) {
          const float* pp = a.p + size_t(r0 + r + row) * PW + col;
          for (int kb2 = 0; kb2 < a.ksplit; ++kb2) {
            const float2 v = *reinterpret_cast<const float2*>(pp + size_t(kb2) * a.total_rows * PW);
            sx += v.x; sy += v.y;
          }
        }
        *reinterpret_cast<half2_t*>(p_lds + 2 * e2) = half2_t{(_Float16)sx, (_Float16)sy};
      }
    };
    // The B-factor tiles of this wavefront's n-tiles are needed only after the last k-step, by loads
    // that would then miss every cache: touch their lines now (one dword per 64 bytes, one lane per
    // line) so that they wait in L2.  The value is only kept alive, never used.
    uint32_t touch = 0;
    if (lowrank && kwi == 0) {
      const int rs_ = a.rpad / 16, lines = rs_ * 8;           // 64-byte lines per (tile, projection)
      const int per = (64 / (kTPW * NM));                     // lanes available per (tile, projection)
      const int ts = lane / (per * NM), m = (lane / per) % NM, line = lane % per;
      const int tile = t0 + grp + ts * groups;
      if (tile < t1 && line < lines)
        touch = *reinterpret_cast<const uint32_t*>(reinterpret_cast<const char*>(d.bf[DUAL ? m : 2]) +
                                                   size_t(tile) * rs_ * 512 + line * 64);
    }
    // A phase is mt_n * nk * 8 fragments of 64 units (16 rows x 4 column groups of one MFMA sub-step);
    // wavefront w copies fragments w, w + 16, ...: four 256-byte runs of the operand-order buffer
    // into 1 KB of LDS, lane-linear.  Rows past the expert's last one read whatever follows (other
    // rows or the padding): their output columns are never stored.  Columns past K read as zero.
    const uint4* in_units = reinterpret_cast<const uint4*>(a.in);
    auto stage = [&](int ph, int nk) {
      const int nfrag = mt_n * nk * 8;
      uint4 reg[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int fb = wave + i * kDecodeWaves;
        reg[i] = make_uint4(0, 0, 0, 0);
        if (fb < nfrag) {
          const int s = fb & 7, mk = fb >> 3, mt = mk / nk, kl = mk - mt * nk;
          const int k8 = (ks_lo + ph * KP + kl) * 32 + q * 8 + s;
          if (k8 * 8 < a.K) reg[i] = in_units[act_unit(k8, rin + 16 * mt + rowl, a.in_rt)];
        }
      }
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int fb = wave + i * kDecodeWaves;
        if (fb < nfrag) {
          const int s = fb & 7, mk = fb >> 3, mt = mk / nk, kl = mk - mt * nk;
          xs[((mt * KP + kl) * 8 + s) * 64 + lane] = reg[i];
        }
      }
    };

    LRC_STAMP(11);
    float4_t acc[kTPW][kDMT][NM];
#pragma unroll
    for (int ts = 0; ts < kTPW; ++ts)
#pragma unroll
      for (int mt = 0; mt < kDMT; ++mt)
#pragma unroll
        for (int m = 0; m < NM; ++m) acc[ts][mt][m] = float4_t{0.f, 0.f, 0.f, 0.f};

    auto compute = [&](const Slot<BITS, NM>& cur, int kl, float4_t (&ac)[kDMT][NM]) {
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
        for (int mt = 0; mt < kDMT; ++mt)
          if (mt < mt_n) {
            const half8_t xf = __builtin_bit_cast(half8_t, xk[(size_t(mt) * KP * 8 + s) * 64]);
#pragma unroll
            for (int m = 0; m < NM; ++m)
              ac[mt][m] = __builtin_amdgcn_mfma_f32_16x16x32_f16(wf[m], xf, ac[mt][m], 0, 0, 0);
          }
      }
    };

    Slot<BITS, NM> ring[RING];
#pragma unroll
    for (int i = 0; i < RING; ++i) fetch(i, ring[i]);
    LRC_STAMP(12);
    int n = 0;
    for (int ph = 0; ph < n_ph; ++ph) {
      const int nk = min(KP, KSl - ph * KP);
      if (ph > 0 || r > 0) __syncthreads();   // everyone is done with the previous phase
      if (ph == 0 && lowrank) load_p();
      if (ph < 5) LRC_STAMP(1 + 2 * ph);
      stage(ph, nk);
      __syncthreads();
      if (ph < 5) LRC_STAMP(2 + 2 * ph);
#pragma unroll
      for (int ts = 0; ts < kTPW; ++ts) {
        const bool tile_ok = t0 + grp + ts * groups < t1;
        for (int si = 0; si < SP; si += RING) {
#pragma unroll
          for (int i = 0; i < RING; ++i) {   // slot i: consumed, then refilled RING steps ahead
            if (tile_ok && (si + i) * kw + kwi < nk) compute(ring[i], (si + i) * kw + kwi, acc[ts]);
            fetch(n + i + RING, ring[i]);
          }
          n += RING;
        }
      }
    }

    LRC_STAMP(13);
    // ---- wavefronts that shared an n-tile add up their partial sums through LDS ----
    if (kw > 1) {
      float4_t* red = reinterpret_cast<float4_t*>(xs);
      __syncthreads();
      if (kwi != 0) {
#pragma unroll
        for (int mt = 0; mt < kDMT; ++mt)
          if (mt < mt_n)
#pragma unroll
            for (int m = 0; m < NM; ++m) red[((wave * kDMT + mt) * NM + m) * 64 + lane] = acc[0][mt][m];
      }
      __syncthreads();
      if (kwi == 0) {
        for (int j = 1; j < kw; ++j)
#pragma unroll
          for (int mt = 0; mt < kDMT; ++mt)
            if (mt < mt_n)
#pragma unroll
              for (int m = 0; m < NM; ++m) acc[0][mt][m] += red[(((wave + j) * kDMT + mt) * NM + m) * 64 + lane];
      }
    }
    LRC_STAMP(14);
    if (kwi != 0) continue;                  // (the next pass starts with a barrier every wavefront reaches)

    // ---- rank-r term: r/16 more MFMA steps on (in A), two at a time with every load of the pair
    //      of steps (B-factor tiles of both n-tiles, (in A) fragments of both row tiles) issued first
    const int rs = a.rpad / 16;
    bool any = false;
#pragma unroll
    for (int mt = 0; mt < kDMT; ++mt) any = any || __ballot(flag[mt]) != 0ull;
    if (any) {
      for (int st0 = 0; st0 < rs; st0 += 2) {
        half4_t bfr[kTPW][NM][2], pf[kDMT][NM][2];
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
          for (int m = 0; m < NM; ++m) {
            const int mat = DUAL ? m : 2, st = st0 + j;
#pragma unroll
            for (int ts = 0; ts < kTPW; ++ts) {
              const int tile = t0 + grp + ts * groups;
              bfr[ts][m][j] = half4_t{0, 0, 0, 0};
              if (tile < t1 && st < rs)
                bfr[ts][m][j] = *reinterpret_cast<const half4_t*>(d.bf[mat] + ((size_t(tile) * rs + st) * kWave + lane) * 4);
            }
#pragma unroll
            for (int mt = 0; mt < kDMT; ++mt) {
              pf[mt][m][j] = half4_t{0, 0, 0, 0};
              if (flag[mt] && st < rs)
                pf[mt][m][j] = *reinterpret_cast<const half4_t*>(p_lds + (16 * mt + c) * PW + m * a.rpad + 16 * st + 4 * q);
            }
          }
#pragma unroll
        for (int m = 0; m < NM; ++m) {
          const _Float16 lam = (_Float16)d.lambda[DUAL ? m : 2];
#pragma unroll
          for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int ts = 0; ts < kTPW; ++ts)
#pragma unroll
              for (int mt = 0; mt < kDMT; ++mt)
                if (mt < mt_n)
                  acc[ts][mt][m] = __builtin_amdgcn_mfma_f32_16x16x16f16(bfr[ts][m][j], pf[mt][m][j] * lam, acc[ts][mt][m], 0, 0, 0);
        }
      }
    }

    // ---- epilogue: lane holds output columns 16*tile + 4*q .. +3 of token column c ----
#pragma unroll
    for (int ts = 0; ts < kTPW; ++ts) {
      const int tile = t0 + grp + ts * groups;
      if (tile >= t1) continue;
#pragma unroll
      for (int mt = 0; mt < kDMT; ++mt) {
        const int row = r + 16 * mt + c;
        if (mt >= mt_n || row >= cnt) continue;
        const size_t o = size_t(r0 + row) * a.N + tile * kTileN + 4 * q;
        if constexpr (DUAL) {
          const float i1 = d.inv_lambda[0], i3 = d.inv_lambda[1];
          half4_t hv;
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const float g = acc[ts][mt][0][i] * i1, u = acc[ts][mt][1][i] * i3;
            hv[i] = (_Float16)(g * __builtin_amdgcn_rcpf(1.0f + __expf(-g)) * u);
          }
          // h in operand order for the W2 kernel: columns f .. f+3 are half of one 16-byte unit
          const int f = tile * kTileN + 4 * q;
          *reinterpret_cast<half4_t*>(reinterpret_cast<_Float16*>(a.out) + act_unit(f >> 3, r0 + row, a.out_rt) * 8 + (f & 7)) = hv;
        } else {
          const float i2 = d.inv_lambda[2];
          if (a.partial != nullptr) {          // K-blocks: fp32 partial sums, added up by reduce_kernel
            *reinterpret_cast<float4_t*>(a.partial + size_t(kb) * a.total_rows * a.N + o) = acc[ts][mt][0] * i2;
          } else {
            uint2 yv;
            yv.x = f32x2_to_bf16x2(acc[ts][mt][0][0] * i2, acc[ts][mt][0][1] * i2);
            yv.y = f32x2_to_bf16x2(acc[ts][mt][0][2] * i2, acc[ts][mt][0][3] * i2);
            *reinterpret_cast<uint2*>(reinterpret_cast<uint16_t*>(a.out) + o) = yv;
          }
        }
      }
    }
    asm volatile("" ::"v"(touch));
    LRC_STAMP(15);
  }
}

// Partial (in A): pk[kb2][row][rho] = sum over K-block kb2 of in[row][k] * A[k][rho] in fp32, for the
// rows that take the rank-r term.  grid = (16-column tiles of the factor(s), experts, K-blocks); the
// 8 wavefronts of a block split their K-block and add their parts through LDS in a fixed order.
// The FFN kernel adds the K-blocks (in order) when it starts.
template <bool DUAL>
__global__ __launch_bounds__(512) void xa_split_kernel(KArgs a) {
  __shared__ float4_t red[8][64];
  const int e = blockIdx.y, tile = blockIdx.x, kb2 = blockIdx.z;
  const int r0 = a.offsets[e], cnt = a.offsets[e + 1] - r0;
  const ExpertDesc& d = a.desc[e];
  if (cnt == 0 || !d.has_factors) return;
  const int lane = threadIdx.x & 63, c = lane & 15, q = lane >> 4;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int rt = a.rpad / 16, PW = (DUAL ? 2 : 1) * a.rpad;
  const int mat = DUAL ? (tile >= rt ? 1 : 0) : 2;
  const int tl = DUAL && tile >= rt ? tile - rt : tile;
  const half8_t* af = reinterpret_cast<const half8_t*>(d.af[mat]);
  const int k32 = a.K / 32, per_b = (k32 + a.ksplit - 1) / a.ksplit, per = (per_b + 7) / 8;
  const int kk0 = kb2 * per_b + wave * per, kk1 = min(min(k32, (kb2 + 1) * per_b), kk0 + per);
  float* pout = const_cast<float*>(a.p) + size_t(kb2) * a.total_rows * PW;
  const half8_t* src = reinterpret_cast<const half8_t*>(a.in);   // operand order: unit (k8, row)
  for (int r = 0; r < cnt; r += 16) {
    const int row = r + c;
    bool flagged = false;
    if (row < cnt) flagged = (a.row_pair[r0 + row] % a.top_k) < a.top_n;
    if (__ballot(flagged) == 0ull) continue;      // same rows in every wavefront: block-uniform
    float4_t acc = float4_t{0.f, 0.f, 0.f, 0.f};
    for (int kk = kk0; kk < kk1; kk += 8) {        // eight steps of loads in flight
      half8_t wf[8], xf[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        wf[u] = half8_t{0, 0, 0, 0, 0, 0, 0, 0};
        xf[u] = half8_t{0, 0, 0, 0, 0, 0, 0, 0};
        if (kk + u < kk1) {
          wf[u] = af[(size_t(kk + u) * rt + tl) * kWave + lane];
          if (flagged) xf[u] = src[act_unit(4 * (kk + u) + q, r0 + row, a.in_rt)];
        }
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(wf[u], xf[u], acc, 0, 0, 0);
    }
    red[wave][lane] = acc;
    __syncthreads();
    if (wave == 0 && flagged) {
      float4_t sum = red[0][lane];
#pragma unroll
      for (int w = 1; w < 8; ++w) sum += red[w][lane];
      *reinterpret_cast<float4_t*>(pout + size_t(r0 + row) * PW + 16 * tile + 4 * q) = sum;
    }
    __syncthreads();
  }
}

// y_rows[R][n] = bf16(sum over K-blocks of partial[kb][R][n]), K-blocks in order (deterministic).
__global__ __launch_bounds__(256) void reduce_kernel(const float* __restrict__ partial, int kblocks, size_t stride,
                                                     size_t units, uint2* __restrict__ y) {
  const size_t u = size_t(blockIdx.x) * 256 + threadIdx.x;       // one unit = 4 outputs
  if (u >= units) return;
  float4_t sum = *reinterpret_cast<const float4_t*>(partial + u * 4);
  for (int kb = 1; kb < kblocks; ++kb) sum += *reinterpret_cast<const float4_t*>(partial + kb * stride + u * 4);
  uint2 v;
  v.x = f32x2_to_bf16x2(sum[0], sum[1]);
  v.y = f32x2_to_bf16x2(sum[2], sum[3]);
  y[u] = v;
}

template <int BITS>
hipError_t launch_bits(const FfnArgs& f, hipStream_t s) {
  static bool attr_set = false;
  if (!attr_set) {
    // 128 KB of activations + up to 32 KB of (in A) for 32 rows at rank 256 = all 160 KB of a CU
    hipError_t e1 = hipFuncSetAttribute(reinterpret_cast<const void*>(&qgemm_decode_kernel<BITS, true>),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, kDecodeLdsUnits * 16 + 32768);
    hipError_t e2 = hipFuncSetAttribute(reinterpret_cast<const void*>(&qgemm_decode_kernel<BITS, false>),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, kDecodeLdsUnits * 16 + 32768);
    if (e1 != hipSuccess) return e1;
    if (e2 != hipSuccess) return e2;
    attr_set = true;
  }
  int gs = 0;
  while ((1 << gs) < f.group) ++gs;
  KArgs a{};
  a.desc = f.desc; a.offsets = f.offsets; a.row_pair = f.row_pair;
  a.group_shift = gs; a.top_k = f.top_k; a.top_n = f.top_n; a.T = f.T;
  a.rank = f.rank; a.rpad = f.rpad; a.total_rows = f.total_rows; a.kw = 1; a.ksplit = 1;
  const bool comp = f.rank > 0 && f.top_n > 0 && f.row_pair != nullptr;
  // experts that can be active at all: at most one per routed pair; the blocks of the active
  // experts alone should cover the 256 CUs, and a block takes at most 32 n-tiles
  const int max_active = f.offsets ? std::min(f.n_exp, f.T * f.top_k) : f.n_exp;
  auto blocks_per_expert = [&](int NT, int kblocks) {
    int g = (256 + max_active * kblocks - 1) / (max_active * kblocks);
    g = std::max(g, (NT + 16 * kTPW - 1) / (16 * kTPW));
    return std::min(g, NT);
  };
  auto lds_bytes = [&](int pw) { return size_t(kDecodeLdsUnits) * 16 + (comp ? size_t(32) * pw * 2 : 0); };
  auto xa_blocks = [](int K) { return std::max(1, std::min(8, K / 1024)); };   // K-blocks of the (in A) kernels

  // W1 | W3 with the SwiGLU epilogue
  a.in = f.xh; a.out = f.h; a.K = f.H; a.N = f.F; a.NT = f.F / kTileN;
  a.in_rt = f.x_rt; a.out_rt = f.h_rt;
  a.KS = padded_k(f.H) / kTileK; a.G = padded_k(f.H) / f.group;
  a.p = f.p13; a.ksplit = std::min(f.ksplit13, xa_blocks(f.H));
  if (comp) hipLaunchKernelGGL(xa_split_kernel<true>, dim3(2 * f.rpad / 16, f.n_exp, a.ksplit), dim3(512), 0, s, a);
  if (f.marks) (void)hipEventRecord(f.marks[0], s);
  a.kb_steps = a.KS; a.partial = nullptr;
  hipLaunchKernelGGL((qgemm_decode_kernel<BITS, true>), dim3(blocks_per_expert(a.NT, 1), f.n_exp, 1),
                     dim3(64 * kDecodeWaves), lds_bytes(2 * f.rpad), s, a);
  if (f.marks) (void)hipEventRecord(f.marks[1], s);
  // W2
  a.in = f.h; a.out = f.y_rows; a.K = f.F; a.N = f.H; a.NT = f.H / kTileN;
  a.in_rt = f.h_rt; a.out_rt = 0;
  a.KS = padded_k(f.F) / kTileK; a.G = padded_k(f.F) / f.group;
  a.p = f.p2; a.ksplit = std::min(f.ksplit2, xa_blocks(f.F));
  if (comp) hipLaunchKernelGGL(xa_split_kernel<false>, dim3(f.rpad / 16, f.n_exp, a.ksplit), dim3(512), 0, s, a);
  if (f.marks) (void)hipEventRecord(f.marks[2], s);
  // a long K (many phases of staged activations) is split into K-blocks of one 16-k-step phase each;
  // their fp32 partial outputs are added by reduce_kernel
  const int kblocks = f.y_part ? std::min(kMaxKBlocks, (a.KS + 15) / 16) : 1;
  a.kb_steps = (a.KS + kblocks - 1) / kblocks;
  a.partial = kblocks > 1 ? f.y_part : nullptr;
  hipLaunchKernelGGL((qgemm_decode_kernel<BITS, false>), dim3(blocks_per_expert(a.NT, kblocks), f.n_exp, kblocks),
                     dim3(64 * kDecodeWaves), lds_bytes(f.rpad), s, a);
  if (kblocks > 1) {
    const size_t units = size_t(f.total_rows) * f.H / 4;
    hipLaunchKernelGGL(reduce_kernel, dim3((unsigned)((units + 255) / 256)), dim3(256), 0, s, f.y_part, kblocks,
                       size_t(f.total_rows) * f.H, units, reinterpret_cast<uint2*>(f.y_rows));
  }
  if (f.marks) (void)hipEventRecord(f.marks[3], s);
  return hipGetLastError();
}

}  // namespace

#ifdef LRC_TIMELINE
extern "C" int moe_lrc_debug_timeline(long long* host_out) {
  return (int)hipMemcpyFromSymbol(host_out, HIP_SYMBOL(g_timeline), sizeof(long long) * 2 * 4096 * 16);
}
#endif

hipError_t launch_decode_ffn(const FfnArgs& f, hipStream_t s) {
  switch (f.bits) {
    case 2: return launch_bits<2>(f, s);
    case 3: return launch_bits<3>(f, s);
    case 4: return launch_bits<4>(f, s);
  }
  return hipErrorInvalidValue;
}

}  // namespace lrc
