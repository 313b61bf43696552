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
#include <type_traits>

#include "ffn_common.h"
#include "plan.h"

namespace lrc {

namespace {

using namespace ffn;

constexpr int kDecodeWaves = 16;
constexpr int kDecodeLdsUnits = 8192;     // 128 KB in 16-byte units
constexpr int kTPW = 2;                   // n-tiles per wavefront (at most)
// packed tiles a wavefront holds in registers (one being unpacked, the others in flight): two for
// the fused W1|W3 kernel (two projections per slot), four for W2.  Blocks with more in flight take a
// larger share of a saturated memory system, so the depths are the same for one and two row tiles
// per pass (measured: deeper rings for one row tile slow the whole kernel down).
__host__ __device__ constexpr int decode_ring(bool dual) { return dual ? 2 : 4; }

// One expert's share of a block: MT = row tiles per pass (1 when the expert has at most 16 rows).
template <int BITS, bool DUAL, int MT>
__device__ __forceinline__ void decode_body(const KArgs& a, uint4* xs, const int e, const int r0, const int cnt,
                                            const int b, const int G) {
  constexpr int NM = DUAL ? 2 : 1;
  constexpr int DW = 2 * BITS;
  constexpr int NC = Extract<BITS>::kClasses;
  constexpr int RING = decode_ring(DUAL);
  constexpr int kDMT = MT;
  const ExpertDesc& d = a.desc[e];
  const int th = threadIdx.x, lane = th & 63;
  const int wave = __builtin_amdgcn_readfirstlane(th >> 6);
  const int q = lane >> 4, c = lane & 15, rowl = th & 15;
  const int tdw = kWave * DW;

  // this block's n-tiles (block b of the G that share the expert), and how they are dealt to the 16 wavefronts
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
    // (the pointers are read once, into scalar registers: a buffer resource must be wave-uniform)
    code_rs[m] = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint32_t*>(uniform_ptr(d.codes[mat])), 0, code_bytes, 0x00020000);
    meta_rs[m] = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint32_t*>(uniform_ptr(d.meta[mat])), 0, meta_bytes, 0x00020000);
  }
  // The rank-r term rides the same stream: the B factor of an n-tile is LS more steps of 32 rank
  // indices, whose 16-byte units (fp16, MFMA operand order) take the place of the packed codes in a
  // ring slot and go into the MFMA as they are, against (in A) instead of the activations.  A
  // resource of size zero (no factors, or not this K-block's job) makes those steps read zeros.
  const bool has_factors = __builtin_amdgcn_readfirstlane(d.has_factors) != 0;
  const bool lowrank = a.rank > 0 && has_factors && a.row_pair != nullptr && blockIdx.z == 0 &&
                       __builtin_amdgcn_readfirstlane(a.comp_rows[e]) > 0;
  const int LS = lowrank ? a.ls : 0;
  float lam[NM];
#pragma unroll
  for (int m = 0; m < NM; ++m) lam[m] = __uint_as_float(__builtin_amdgcn_readfirstlane(__float_as_uint(d.lambda[DUAL ? m : 2])));
  __amdgpu_buffer_rsrc_t bf_rs[NM];
#pragma unroll
  for (int m = 0; m < NM; ++m)
    bf_rs[m] = __builtin_amdgcn_make_buffer_rsrc(const_cast<_Float16*>(uniform_ptr(d.bf[DUAL ? m : 2])), 0,
                                                 lowrank ? a.NT * a.ls * 1024 : 0, 0x00020000);
  const int bf_bytes = a.NT * a.ls * 1024;
  const int gps = kTileK >> a.group_shift;           // groups per k-step
  const int meta_lane = ((q * kLaneK) >> a.group_shift) * (a.NT * kTileN * 4) + c * 4;
  const int PW = DUAL ? 2 * a.rpad : a.rpad;
  uint4* p_lds = xs + kDecodeLdsUnits;               // (in A) fragments: [m][rank step][row tile][lane]

  for (int r = 0; r < cnt; r += 16 * kDMT) {
    // every pass computes all MT row tiles (a last pass with fewer rows computes columns nobody stores)
    constexpr int KP = (kDecodeLdsUnits / 512) / kDMT;   // k-steps per phase: 16 or 8
    const int n_ph = (KSl + KP - 1) / KP;
    // A wavefront's steps, in order: [phase][tile slot][own k-step], then [own rank step][tile slot].
    // Each segment is padded to a multiple of the ring depth, so that slot indices stay static.
    const int spw = (KP + kw - 1) / kw;                  // own k-steps per (tile, phase) segment
    const int SP = (spw + RING - 1) / RING * RING;
    const int n_reg = n_ph * kTPW * SP;
    static_assert(RING % kTPW == 0, "the rank steps alternate between the tile slots: even ring depths only");
    const int LSP = (kTPW * ((LS + kw - 1) / kw) + RING - 1) / RING * RING;

    // step n -> (phase, tile slot, own step); a step that does not exist loads from past the end of
    // the resources and gets zeros
    auto fetch = [&](int n, Slot<BITS, NM>& sl) {
      const bool reg = n < n_reg;
      const int l = n - n_reg;                                           // index among the rank steps
      const int seg = n / SP, si = n - seg * SP, ph = seg / kTPW;
      const int ts = reg ? seg - ph * kTPW : l % kTPW;
      const int kl = si * kw + kwi, tile = t0 + grp + ts * groups;
      const int st = (l / kTPW) * kw + kwi;                              // rank step
      const bool ok = reg && tile < t1 && kl < KP && ph * KP + kl < KSl;     // a k-step of packed codes
      const bool lr = !reg && l < LSP && tile < t1 && st < LS;               // a rank step of the B factor
      const int ks = ks_lo + ph * KP + kl;
      // the offsets go into the per-lane offset operand: that is the one the hardware range-checks
      const int tile_off = (ok ? (ks * a.NT + tile) * (tdw * 4) : lr ? (st * a.NT + tile) * 1024 : max(code_bytes, bf_bytes)) + lane * 16;
      const int tile_off2 = (ok ? (ks * a.NT + tile) * (tdw * 4) : code_bytes) + 1024 + lane * (BITS == 3 ? 8 : 16);
      const int meta_off = (ok ? (ks * gps * a.NT + tile) * (kTileN * 4) : meta_bytes) + meta_lane;
#pragma unroll
      for (int m = 0; m < NM; ++m) {
        const u32x4 v0 = __builtin_amdgcn_raw_buffer_load_b128(lr ? bf_rs[m] : code_rs[m], tile_off, 0, 0);
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

    // first input row of this pass (shared experts all read the token rows 0..T-1)
    const int rin = ((DUAL && !a.offsets) ? 0 : r0) + r;

    // A phase is MT * nk * 8 fragments of 64 units (16 rows x 4 column groups of one MFMA sub-step);
    // four 256-byte runs of the operand-order buffer become 1 KB of LDS, lane-linear.  Rows past the
    // expert's last one read whatever follows (other rows or the padding): their output columns are
    // never stored.  The copy is asynchronous and takes no registers:
    // each lane's 16 bytes go from global memory straight to LDS (wave-uniform LDS base + 16 * lane),
    // counted by vmcnt like any other load.
    const uint4* in_units = reinterpret_cast<const uint4*>(a.in);
    auto stage_issue = [&](int ph, int nk) {
      const int s = wave & 7;                  // fragment (mt, kl, s): wavefront w takes s = w % 8, kl = w / 8, w / 8 + 2, ...
      for (int mt = 0; mt < kDMT; ++mt)
        for (int kl = wave >> 3; kl < nk; kl += 2) {
          // (columns past K: the padded weights there are exact zeros, any finite value will do)
          const int k8 = min((ks_lo + ph * KP + kl) * 32 + q * 8 + s, a.K / 8 - 1);
          uint4* dst = xs + ((mt * KP + kl) * 8 + s) * 64;
          __builtin_amdgcn_global_load_lds(
              reinterpret_cast<const __attribute__((address_space(1))) void*>(
                  reinterpret_cast<uintptr_t>(in_units + act_unit(k8, rin + 16 * mt + rowl, a.in_rt))),
              reinterpret_cast<__attribute__((address_space(3))) void*>(reinterpret_cast<uintptr_t>(dst)), 16, 0, 0);
        }
    };

    // ---- start of a pass.  The K-block partial sums of (in A) are read and added first (a few KB,
    //      one round trip); then the activations of phase 0 (straight to LDS) and the first packed
    //      tiles are issued, and only the packed tiles are still in flight when the first barrier is
    //      passed.
    if (r > 0) __syncthreads();               // everyone is done with the previous pass's LDS
    // (in A) of this pass's rows, times the projection's power-of-two pre-scale, as fp16 in MFMA
    // operand order: unit ((m * LS + st) * MT + mt) * 64 + lane holds columns 32 st + 8 q .. + 7 of
    // row 16 mt + lane % 16 (zero for rows without the term and past the rank).  The partial sums of
    // xa_split_kernel are added in K-block order.  They are read whether or not the row takes the
    // term (a row inside the expert's range is always inside the buffer) and selected afterwards,
    // so that the loads do not wait for the flag.
    const int p_pairs = NM * LS * kDMT * 64 * 4;     // pairs of adjacent columns
    auto p_load = [&](int e2, int& rp, float2 (&v)[4], int kb0) {
      const int u = e2 >> 2, ln = u & 63, g = u >> 6, mt = g % kDMT, st = (g / kDMT) % max(LS, 1), m = g / (kDMT * max(LS, 1));
      const int rho = 32 * st + 8 * (ln >> 4) + 2 * (e2 & 3);
      const int rr = r0 + min(r + 16 * mt + (ln & 15), cnt - 1);
      rp = a.row_pair[rr];
      const float* pp = a.p + size_t(rr) * PW + m * a.rpad + min(rho, a.rpad - 2);
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        v[j] = make_float2(0.f, 0.f);
        if (kb0 + j < a.ksplit) v[j] = *reinterpret_cast<const float2*>(pp + size_t(kb0 + j) * a.total_rows * PW);
      }
    };
    auto p_store = [&](int e2, int rp, float sx, float sy) {
      const int u = e2 >> 2, ln = u & 63, g = u >> 6, mt = g % kDMT, st = (g / kDMT) % max(LS, 1), m = g / (kDMT * max(LS, 1));
      const int rho = 32 * st + 8 * (ln >> 4) + 2 * (e2 & 3);
      const bool on = r + 16 * mt + (ln & 15) < cnt && (rp % a.top_k) < a.top_n && rho < a.rpad;
      const float lm = NM == 2 && m == 1 ? lam[NM - 1] : lam[0];
      reinterpret_cast<half2_t*>(p_lds)[e2] = on ? half2_t{(_Float16)(sx * lm), (_Float16)(sy * lm)} : half2_t{0, 0};
    };
    for (int e2 = th; e2 < p_pairs; e2 += 64 * kDecodeWaves) {
      float sx = 0.f, sy = 0.f;
      int rp = 0;
      for (int kb0 = 0; kb0 < a.ksplit; kb0 += 4) {       // four K-blocks' loads in flight, added in order
        float2 v[4];
        p_load(e2, rp, v, kb0);
#pragma unroll
        for (int j = 0; j < 4; ++j) { sx += v[j].x; sy += v[j].y; }
      }
      p_store(e2, rp, sx, sy);
    }
    const int nk0 = min(KP, KSl);
    stage_issue(0, nk0);                      // (no registers)
    __builtin_amdgcn_sched_barrier(0);        // (the wait below counts the packed tiles as the only later loads)
    Slot<BITS, NM> ring[RING];
#pragma unroll
    for (int i = 0; i < RING; ++i) fetch(i, ring[i]);
    // everything but the packed tiles issued last has arrived: the activations are in LDS
    // The barrier is written out: a __syncthreads() here would first wait for every load in flight,
    // the packed tiles included.  LDS writes of this wavefront are awaited by lgkmcnt(0).
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(RING * NM * (BITS == 2 ? 2 : 3)) : "memory");

    float4_t acc[kTPW][kDMT][NM];
#pragma unroll
    for (int ts = 0; ts < kTPW; ++ts)
#pragma unroll
      for (int mt = 0; mt < kDMT; ++mt)
#pragma unroll
        for (int m = 0; m < NM; ++m) acc[ts][mt][m] = float4_t{0.f, 0.f, 0.f, 0.f};

    // a rank step of one n-tile: the slot holds B-factor units, which meet (in A) as they are
    auto compute_lr = [&](const Slot<BITS, NM>& cur, int st, float4_t (&ac)[kDMT][NM]) {
      const uint4* pk = p_lds + size_t(st) * kDMT * 64 + lane;
#pragma unroll
      for (int m = 0; m < NM; ++m) {
        const half8_t bfrag = __builtin_bit_cast(half8_t, make_uint4(cur.cw[m][0], cur.cw[m][1], cur.cw[m][2], cur.cw[m][3]));
#pragma unroll
        for (int mt = 0; mt < kDMT; ++mt) {
          const half8_t pf = __builtin_bit_cast(half8_t, pk[(size_t(m) * LS * kDMT + mt) * 64]);
          ac[mt][m] = __builtin_amdgcn_mfma_f32_16x16x32_f16(bfrag, pf, ac[mt][m], 0, 0, 0);
        }
      }
    };
    // a k-step of packed codes of one n-tile
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
      // One sub-step: 32 rows of the weight tile are unpacked into the MFMA operand while the
      // activation fragments wait in registers.  Where the registers allow (XB == 2) the fragments of
      // sub-step s + 1 are requested from LDS before sub-step s is unpacked; the reads and the waits
      // are written out, because the compiler would move each read down to its use.
      constexpr int XB = (kDMT == 1 || BITS == 2) ? 2 : 1;
      half8_t xf[XB][kDMT];
      uint32_t xaddr[kDMT];
#pragma unroll
      for (int mt = 0; mt < kDMT; ++mt) xaddr[mt] = uint32_t(reinterpret_cast<uintptr_t>(xk)) + mt * KP * 8 * 1024;
      if constexpr (XB == 2) {
#pragma unroll
        for (int mt = 0; mt < kDMT; ++mt) xf[0][mt] = lds_read16<0>(xaddr[mt]);
      }
      auto substep = [&](auto S) {
        constexpr int s = decltype(S)::value;
        if constexpr (XB == 2) {
          if constexpr (s < 7) {
#pragma unroll
            for (int mt = 0; mt < kDMT; ++mt) xf[(s + 1) & 1][mt] = lds_read16<(s + 1) * 1024>(xaddr[mt]);
          }
        } else {
#pragma unroll
          for (int mt = 0; mt < kDMT; ++mt) xf[0][mt] = __builtin_bit_cast(half8_t, xk[(size_t(mt) * KP * 8 + s) * 64]);
        }
        half8_t wf[NM];
#pragma unroll
        for (int m = 0; m < NM; ++m) {
          uint32_t v[4];
#pragma unroll
          for (int j = 0; j < 4; ++j)
            v[j] = pk_fma(Extract<BITS>::field(cur.cw[m], 4 * s + j), s2[m][Extract<BITS>::cls(4 * s + j)], c2[m]);
          wf[m] = __builtin_bit_cast(half8_t, make_uint4(v[0], v[1], v[2], v[3]));
        }
        if constexpr (XB == 2) {
          // the fragments of this sub-step are older than the kDMT reads just issued
          if constexpr (kDMT == 1) lds_wait<(s < 7 ? 1 : 0)>(xf[s & 1][0]);
          else lds_wait<(s < 7 ? 2 : 0)>(xf[s & 1][0], xf[s & 1][kDMT - 1]);
        }
#pragma unroll
        for (int mt = 0; mt < kDMT; ++mt)
#pragma unroll
          for (int m = 0; m < NM; ++m)
            ac[mt][m] = __builtin_amdgcn_mfma_f32_16x16x32_f16(wf[m], xf[XB == 2 ? (s & 1) : 0][mt], ac[mt][m], 0, 0, 0);
      };
      substep(std::integral_constant<int, 0>{}); substep(std::integral_constant<int, 1>{});
      substep(std::integral_constant<int, 2>{}); substep(std::integral_constant<int, 3>{});
      substep(std::integral_constant<int, 4>{}); substep(std::integral_constant<int, 5>{});
      substep(std::integral_constant<int, 6>{}); substep(std::integral_constant<int, 7>{});
    };

    int n = 0;
    for (int ph = 0; ph < n_ph; ++ph) {
      const int nk = min(KP, KSl - ph * KP);
      if (ph > 0) {
        __syncthreads();                      // everyone is done with the previous phase
        stage_issue(ph, nk);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
      }
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
    for (int l0 = 0; l0 < LSP; l0 += RING) {   // the rank steps (none unless this block adds the term)
#pragma unroll
      for (int i = 0; i < RING; ++i) {
        const int st = ((l0 + i) / kTPW) * kw + kwi;
        if (t0 + grp + (i % kTPW) * groups < t1 && st < LS) compute_lr(ring[i], st, acc[i % kTPW]);
        fetch(n + i + RING, ring[i]);
      }
      n += RING;
    }
    // ---- wavefronts that shared an n-tile add up their partial sums through LDS ----
    if (kw > 1) {
      float4_t* red = reinterpret_cast<float4_t*>(xs);
      __syncthreads();
      if (kwi != 0) {
#pragma unroll
        for (int mt = 0; mt < kDMT; ++mt)
#pragma unroll
          for (int m = 0; m < NM; ++m) red[((wave * kDMT + mt) * NM + m) * 64 + lane] = acc[0][mt][m];
      }
      __syncthreads();
      if (kwi == 0) {
        for (int j = 1; j < kw; ++j)
#pragma unroll
          for (int mt = 0; mt < kDMT; ++mt)
#pragma unroll
            for (int m = 0; m < NM; ++m) acc[0][mt][m] += red[(((wave + j) * kDMT + mt) * NM + m) * 64 + lane];
      }
    }
    if (kwi != 0) continue;                  // (the next pass starts with a barrier every wavefront reaches)

    // ---- epilogue: lane holds output columns 16*tile + 4*q .. +3 of token column c ----
#pragma unroll
    for (int ts = 0; ts < kTPW; ++ts) {
      const int tile = t0 + grp + ts * groups;
      if (tile >= t1) continue;
#pragma unroll
      for (int mt = 0; mt < kDMT; ++mt) {
        const int row = r + 16 * mt + c;
        if (row >= cnt) continue;
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
  }
}

template <int BITS, bool DUAL>
__global__ __launch_bounds__(64 * kDecodeWaves, 4) void qgemm_decode_kernel(KArgs a) {
  extern __shared__ uint4 xs[];
  int e = blockIdx.y, b = blockIdx.x, G = gridDim.x;
  if (a.plan != nullptr) {                   // shares by table (plan_kernel)
    const int4 pe = reinterpret_cast<const int4*>(a.plan)[blockIdx.x];
    e = __builtin_amdgcn_readfirstlane(pe.x); b = __builtin_amdgcn_readfirstlane(pe.y); G = __builtin_amdgcn_readfirstlane(pe.z);
    if (e < 0) return;
  }
  const int r0 = a.offsets ? a.offsets[e] : e * a.T;
  const int cnt = a.offsets ? a.offsets[e + 1] - r0 : a.T;
  if (cnt == 0) return;
  if (cnt <= 16) decode_body<BITS, DUAL, 1>(a, xs, e, r0, cnt, b, G);
  else decode_body<BITS, DUAL, 2>(a, xs, e, r0, cnt, b, G);
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
          wf[u] = af[(size_t(tl) * k32 + kk + u) * kWave + lane];
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

// Block tables pay when experts are likely to be without rows or to differ much in rows: many
// experts, or few pairs per expert.  Otherwise (e.g. 8 experts, 64 tokens) every expert gets the
// same share of a (blocks per expert x experts) grid.
static bool use_plan(const FfnArgs& f) {
  return f.offsets != nullptr && f.plan != nullptr && (f.n_exp >= 32 || f.T * f.top_k < 4 * f.n_exp);
}

template <int BITS>
hipError_t launch_bits(const FfnArgs& f, hipStream_t s, int which) {
  int gs = 0;
  while ((1 << gs) < f.group) ++gs;
  KArgs a{};
  a.desc = f.desc; a.offsets = f.offsets; a.row_pair = f.row_pair; a.comp_rows = f.comp_rows;
  a.group_shift = gs; a.top_k = f.top_k; a.top_n = f.top_n; a.T = f.T;
  a.rank = f.rank; a.rpad = f.rpad; a.ls = (f.rank + 31) / 32; a.total_rows = f.total_rows; a.kw = 1; a.ksplit = 1;
  const bool comp = f.rank > 0 && f.top_n > 0 && f.row_pair != nullptr;
  // experts that can be active at all: at most one per routed pair; the blocks of the active
  // experts alone should cover the CUs, and a block takes at most 32 n-tiles
  const int max_active = f.offsets ? std::min(f.n_exp, f.T * f.top_k) : f.n_exp;
  auto blocks_per_expert = [&](int NT, int kblocks) {
    int g = (f.n_cu + max_active * kblocks - 1) / (max_active * kblocks);
    g = std::max(g, (NT + 16 * kTPW - 1) / (16 * kTPW));
    return std::min(g, NT);
  };
  // activations + the (in A) fragments: [projections][rank steps][2 row tiles] KB
  auto lds_bytes = [&](int nm) { return size_t(kDecodeLdsUnits) * 16 + (comp ? size_t(nm) * a.ls * 2 * 1024 : 0); };
  auto xa_blocks = [](int K) { return std::max(1, std::min(8, K / 1024)); };   // K-blocks of the (in A) kernels
  // the blocks are shared out among the experts that have rows by the tables the launch that
  // prepared the activations has left (plan.h)
  const bool by_table = use_plan(f);

  if (which & 1) {
  // W1 | W3 with the SwiGLU epilogue
  a.in = f.xh; a.out = f.h; a.K = f.H; a.N = f.F; a.NT = f.F / kTileN;
  a.in_rt = f.x_rt; a.out_rt = f.h_rt;
  a.KS = padded_k(f.H) / kTileK; a.G = padded_k(f.H) / f.group;
  a.p = f.p13; a.ksplit = std::min(f.ksplit13, xa_blocks(f.H));
  if (comp) hipLaunchKernelGGL(xa_split_kernel<true>, dim3(2 * f.rpad / 16, f.n_exp, a.ksplit), dim3(512), 0, s, a);
  if (f.marks) (void)hipEventRecord(f.marks[0], s);
  a.kb_steps = a.KS; a.partial = nullptr;
  if (by_table) {
    const int B = plan_blocks(f.n_exp, f.T * f.top_k, a.NT, f.n_cu);
    a.plan = f.plan;
    hipLaunchKernelGGL((qgemm_decode_kernel<BITS, true>), dim3(B, 1, 1), dim3(64 * kDecodeWaves), lds_bytes(2), s, a);
    a.plan = nullptr;
  } else {
    hipLaunchKernelGGL((qgemm_decode_kernel<BITS, true>), dim3(blocks_per_expert(a.NT, 1), f.n_exp, 1),
                       dim3(64 * kDecodeWaves), lds_bytes(2), s, a);
  }
  if (f.marks) (void)hipEventRecord(f.marks[1], s);
  }
  if (which & 2) {
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
  if (by_table) {
    // (second table behind the first; every K-block uses the same shares)
    int32_t* plan2 = f.plan + 4 * plan_blocks(f.n_exp, f.T * f.top_k, f.F / kTileN, f.n_cu);
    const int B = plan_blocks(f.n_exp, f.T * f.top_k, a.NT, (f.n_cu + kblocks - 1) / kblocks);
    a.plan = plan2;
    hipLaunchKernelGGL((qgemm_decode_kernel<BITS, false>), dim3(B, 1, kblocks), dim3(64 * kDecodeWaves), lds_bytes(1), s, a);
    a.plan = nullptr;
  } else {
    hipLaunchKernelGGL((qgemm_decode_kernel<BITS, false>), dim3(blocks_per_expert(a.NT, kblocks), f.n_exp, kblocks),
                       dim3(64 * kDecodeWaves), lds_bytes(1), s, a);
  }
  if (kblocks > 1) {
    const size_t units = size_t(f.total_rows) * f.H / 4;
    hipLaunchKernelGGL(reduce_kernel, dim3((unsigned)((units + 255) / 256)), dim3(256), 0, s, f.y_part, kblocks,
                       size_t(f.total_rows) * f.H, units, reinterpret_cast<uint2*>(f.y_rows));
  }
  if (f.marks) (void)hipEventRecord(f.marks[3], s);
  }
  return hipGetLastError();
}

}  // namespace

void decode_plan_specs(const FfnArgs& f, int which, PlanSpec& p13, PlanSpec& p2) {
  p13 = PlanSpec{0, 0, 0, nullptr};
  p2 = PlanSpec{0, 0, 0, nullptr};
  if (!use_plan(f)) return;
  const int pairs = f.T * f.top_k, NT13 = f.F / kTileN, NT2 = f.H / kTileN;
  const int B13 = plan_blocks(f.n_exp, pairs, NT13, f.n_cu);
  if (which & 1) p13 = PlanSpec{B13, (NT13 + 31) / 32, f.n_cu, f.plan};
  if (which & 2) {
    const int KS2 = padded_k(f.F) / kTileK, kb2 = f.y_part ? std::min(kMaxKBlocks, (KS2 + 15) / 16) : 1;
    const int target2 = (f.n_cu + kb2 - 1) / kb2;
    p2 = PlanSpec{plan_blocks(f.n_exp, pairs, NT2, target2), (NT2 + 31) / 32, target2, f.plan + 4 * B13};
  }
}

hipError_t decode_init_device() {
  // 128 KB of activations + up to 32 KB of (in A) for 32 rows at rank 256 = all 160 KB of a CU
  const void* fns[6] = {reinterpret_cast<const void*>(&qgemm_decode_kernel<2, true>), reinterpret_cast<const void*>(&qgemm_decode_kernel<2, false>),
                        reinterpret_cast<const void*>(&qgemm_decode_kernel<3, true>), reinterpret_cast<const void*>(&qgemm_decode_kernel<3, false>),
                        reinterpret_cast<const void*>(&qgemm_decode_kernel<4, true>), reinterpret_cast<const void*>(&qgemm_decode_kernel<4, false>)};
  for (const void* fn : fns) {
    hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, kDecodeLdsUnits * 16 + 32768);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

hipError_t launch_decode_ffn(const FfnArgs& f, hipStream_t s, int which) {
  switch (f.bits) {
    case 2: return launch_bits<2>(f, s, which);
    case 3: return launch_bits<3>(f, s, which);
    case 4: return launch_bits<4>(f, s, which);
  }
  return hipErrorInvalidValue;
}

}  // namespace lrc
