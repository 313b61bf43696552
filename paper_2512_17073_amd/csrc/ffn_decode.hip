// Decode flavour of the expert FFN (Sections 2.3 and 3.2): few rows per expert, so the layer is a
// stream of packed weights and the job is to keep HBM busy.
//
//   - one block of 16 wavefronts per CU.  For routed experts every block reads which expert it
//     serves, which share of the expert's n-tiles and where the expert's rows are from one 32-byte
//     entry of a table the preparing launch has made (plan.h): experts without rows get no blocks,
//     experts whose rows need several 32-row passes get more;
//   - the activations of the expert (up to 32 rows) are staged into 128 KB of LDS once per phase of
//     16 (or 8) k-steps by direct global -> LDS copies, issued together with the first packed tiles
//     and the (in A) fragments: one memory round trip before the first multiply;
//   - a ring slot of a wavefront holds one k-step of two streams: the W1 and W3 tiles of one n-tile
//     in the fused kernel, two adjacent n-tiles in the W2 kernel.  An activation fragment read from
//     LDS meets both streams;
//   - each wavefront streams its packed tiles HBM -> registers with buffer loads through a ring of
//     register slots walked by straight-line code: a load past the end of the resource returns
//     zeros, so refills are unconditional and the number of loads in flight is static;
//   - codes are unpacked in registers (unpack.h) straight into MFMA A-operands; the rank-r term is
//     ceil(r / 32) more steps per stream on the B factor's fp16 units against (in A), which
//     xa_rows_kernel has left in global memory; the rank is the projection's own (Section 3.1
//     allocates a rank per expert matrix): a stream with fewer rank steps reads zeros past its factor;
//   - a long K (W2) is split into K-blocks (grid.z) of one or two phases whose fp32 partial outputs
//     the combine (or reduce_kernel, for the stand-alone call) adds in a fixed order.
#include <algorithm>
#include <type_traits>

#include "decode_index.h"
#include "factor_q3.h"
#include "ffn_common.h"
#include "plan.h"
#include "xa_rows.h"

namespace lrc {

namespace {

using namespace ffn;
using namespace dec;


// One expert's share of a block: MT = row tiles per pass (1 when the expert has at most 16 rows).
// (A pass of 32 rows can be put on v_mfma_f32_32x32x16_f16, which has the same peak rate as the
// 16x16x32 shape used here and needs half as many instructions, by swapping 16-lane rows between the
// two streams' registers; measured, the four swaps per sub-step cost this kernel more than the two
// matrix instructions save.)
// Q3: some factor pair of the layer is held at 3 bits (layout.h): a rank step of such a pair brings
// the unit's code dword in the slot's metadata register and the lane's half of the unit's metadata in
// its first four code registers, and is dequantized into the fp16 unit before it is used.
template <int BITS, bool DUAL, int MT, bool Q3>
__device__ __forceinline__ void decode_body(const KArgs& a, uint4* xs, const int e, const int r0, const int cnt,
                                            const int b, const int G) {
  constexpr int NS = kStreams;
  constexpr int TS = DUAL ? 2 : 1;
  constexpr int NC = Extract<BITS>::kClasses;
  constexpr int RING = kRing;
  const ExpertDesc& d = a.desc[e];
  const int th = threadIdx.x, lane = th & 63;
  const int wave = __builtin_amdgcn_readfirstlane(th >> 6);
  const int q = lane >> 4, c = lane & 15, rowl = th & 15;

  // this block's n-tiles and how their units are dealt to the 16 wavefronts
  int t0, t1;
  block_tiles(b, G, a.NT, t0, t1);
  const int nt_b = t1 - t0;
  if (nt_b == 0) return;
  const int units = block_units(nt_b, DUAL);
  const int kw = waves_per_unit(units);
  const int groups = kWaves / kw, grp = wave / kw, kwi = wave % kw;

  // this block's K-block: k-steps ks_lo .. ks_lo + KSl - 1
  const int kb = blockIdx.z, ks_lo = kb * a.kb_steps, KSl = min(a.KS, ks_lo + a.kb_steps) - ks_lo;
  const uint32_t code_bytes = uint32_t(a.KS) * a.NT * (kWave * 2 * BITS * 4), meta_bytes = uint32_t(a.G) * a.NT * kTileN * 4;

  // The rank-r term rides the same stream (B-factor units in place of packed codes, against (in A)
  // instead of the activations).  With K-blocks, every K-block meets the part of (in A) summed over
  // its own k-steps (the term is linear in it).  Each stream has the rank of its own projection; a
  // resource of the size its rank fills makes later steps read zeros.
  const bool lowrank = a.rank > 0 && a.row_pair != nullptr && __builtin_amdgcn_readfirstlane(d.has_factors) != 0 &&
                       __builtin_amdgcn_readfirstlane(a.comp_rows[e]) > 0;
  int LSm[NS];
#pragma unroll
  for (int m = 0; m < NS; ++m) {
    const int rk = __builtin_amdgcn_readfirstlane(d.rank[DUAL ? m : 2]);
    LSm[m] = lowrank ? (min(rk, a.rank) + 31) / 32 : 0;
  }
  const int LS = max(LSm[0], LSm[1]);
  const uint32_t bf_bytes_max = uint32_t(a.NT) * a.ls * 1024;

  __amdgpu_buffer_rsrc_t code_rs[NS], meta_rs[NS], bf_rs[NS], bc_rs[NS];
  bool q3m[NS];
#pragma unroll
  for (int m = 0; m < NS; ++m) {
    const int mat = DUAL ? m : 2;
    q3m[m] = Q3 && __builtin_amdgcn_readfirstlane((d.q3 >> mat) & 1) != 0;
    // (the pointers are read once, into scalar registers: a buffer resource must be wave-uniform)
    code_rs[m] = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint32_t*>(uniform_ptr(d.codes[mat])), 0, code_bytes, 0x00020000);
    meta_rs[m] = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint32_t*>(uniform_ptr(d.meta[mat])), 0, meta_bytes, 0x00020000);
    // (3-bit pair: the B section's metadata, 128 bytes per rank step and group of four n-tiles)
    bf_rs[m] = __builtin_amdgcn_make_buffer_rsrc(const_cast<_Float16*>(uniform_ptr(d.bf[mat])), 0,
                                                 q3m[m] ? uint32_t(a.NT / 4) * LSm[m] * 128 : uint32_t(a.NT) * LSm[m] * 1024, 0x00020000);
    if constexpr (Q3)     // the code dwords of a 3-bit pair's B units (no bytes for an fp16 pair: every read gives zero)
      bc_rs[m] = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint32_t*>(uniform_ptr(q3m[m] ? d.bfc[mat] : d.codes[mat])), 0,
                                                   q3m[m] ? uint32_t(a.NT) * LSm[m] * 256 : 0u, 0x00020000);
  }
  // (in A) fragments: [projection][rank step][row tile][lane].  Up to 32 of them sit behind the staged
  // activations from the start of a pass; more (ranks above 256) take the place of the activations
  // after the last k-step.
  // (the two streams of the W2 kernel are tiles of one projection: they meet the same fragments)
  constexpr int NP = DUAL ? 2 : 1;
  const int p_frags = NP * LS * MT;
  const bool p_late = p_frags * 64 > kSpareUnits;
  uint4* p_lds = p_late ? xs : xs + kLdsUnits;
  const int pitch = NP * a.ls * 32;                  // halves per row of (in A): [A1 | A3], or A2

  for (int r = 0; r < cnt; r += 16 * MT) {
    // every pass computes all MT row tiles (a last pass with fewer rows computes columns nobody stores)
    const StepPlan sp = step_plan(KSl, MT, kw, LS, DUAL);
    const int KP = sp.KP;

    // (the steps are fetched in order, RING of them ahead of their use and RING past the last one)
    StepCursor cursor = cursor_start();
    auto fetch = [&](Slot<BITS, NS>& sl) {
      const StepRef ref = cursor_ref(cursor, sp, grp, groups, kwi, kw, units, ks_lo, KSl, LS);
      cursor_advance(cursor, sp);
#pragma unroll
      for (int m = 0; m < NS; ++m) {
        const int tile = stream_tile(t0, ref.unit, m, DUAL);
        const LaneOffsets o = lane_offsets(ref, tile, tile < t1, lane, BITS, a.NT, a.group_shift, code_bytes, meta_bytes, bf_bytes_max,
                                           Q3 && q3m[m]);
        const bool lr = ref.lr;
        const u32x4 v0 = __builtin_amdgcn_raw_buffer_load_b128(lr ? bf_rs[m] : code_rs[m], lr ? o.bf : o.code0, 0, 0);
        sl.cw[m][0] = v0[0]; sl.cw[m][1] = v0[1]; sl.cw[m][2] = v0[2]; sl.cw[m][3] = v0[3];
        if constexpr (BITS == 3) {
          const u32x2 v1 = __builtin_amdgcn_raw_buffer_load_b64(code_rs[m], o.code1, 0, 0);
          sl.cw[m][4] = v1[0]; sl.cw[m][5] = v1[1];
        } else if constexpr (BITS == 4) {
          const u32x4 v1 = __builtin_amdgcn_raw_buffer_load_b128(code_rs[m], o.code1, 0, 0);
          sl.cw[m][4] = v1[0]; sl.cw[m][5] = v1[1]; sl.cw[m][6] = v1[2]; sl.cw[m][7] = v1[3];
        }
        if constexpr (Q3) sl.mw[m] = __builtin_amdgcn_raw_buffer_load_b32(lr ? bc_rs[m] : meta_rs[m], lr ? o.bc : o.meta, 0, 0);
        else sl.mw[m] = __builtin_amdgcn_raw_buffer_load_b32(meta_rs[m], o.meta, 0, 0);
      }
    };

    // first input row of this pass (shared experts all read the token rows 0..T-1)
    const int rin = ((DUAL && !a.offsets) ? 0 : r0) + r;

    // A phase is MT * nk * 8 fragments of 64 units (16 rows x 4 column groups of one MFMA sub-step);
    // four 256-byte runs of the operand-order buffer become 1 KB of LDS, lane-linear.  Rows past the
    // expert's last one read the zero rows at the end of the buffer (staged_row): their output
    // columns are never stored.  The copy is asynchronous and takes no registers: each lane's 16 bytes go from
    // global memory straight to LDS (wave-uniform LDS base + 16 * lane), counted by vmcnt.
    const uint4* in_units = reinterpret_cast<const uint4*>(a.in);
    auto stage_issue = [&](int ph, int nk) {
      const int s = wave & 7;                  // fragment (mt, kl, s): wavefront w takes s = w % 8, kl = w / 8, w / 8 + 2, ...
      for (int mt = 0; mt < MT; ++mt)
        for (int kl = wave >> 3; kl < nk; kl += 2) {
          // (columns past K: the padded weights there are exact zeros, any finite value will do)
          const int k8 = min((ks_lo + ph * KP + kl) * 32 + q * 8 + s, a.K / 8 - 1);
          uint4* dst = xs + act_frag_unit(mt, kl, s, KP);
          __builtin_amdgcn_global_load_lds(
              reinterpret_cast<const __attribute__((address_space(1))) void*>(
                  reinterpret_cast<uintptr_t>(in_units + act_unit(k8, staged_row(rin, r, mt, rowl, cnt, a.in_rt), a.in_rt))),
              reinterpret_cast<__attribute__((address_space(3))) void*>(reinterpret_cast<uintptr_t>(dst)), 16, 0, 0);
        }
    };
    // (in A) of this pass's rows: fp16 row-major in global memory, already multiplied by the
    // projection's power-of-two pre-scale and zero for rows without the term.  Fragment
    // (m, st, mt): lane (q, c) copies columns 32 st + 8 q .. + 7 of row 16 mt + c.  A row past the
    // expert's last one is clamped to a valid row (its output column is never stored).
    const _Float16* P = reinterpret_cast<const _Float16*>(a.p) + size_t(kb) * a.total_rows * pitch;
    auto p_issue = [&]() {
      for (int f = wave; f < p_frags; f += kWaves) {
        const int mt = f % MT, g = f / MT, st = g % LS, m = g / LS;
        const int row = r0 + min(r + 16 * mt + c, cnt - 1);
        const _Float16* src = P + size_t(row) * pitch + m * a.ls * 32 + 32 * st + 8 * q;
        __builtin_amdgcn_global_load_lds(
            reinterpret_cast<const __attribute__((address_space(1))) void*>(reinterpret_cast<uintptr_t>(src)),
            reinterpret_cast<__attribute__((address_space(3))) void*>(reinterpret_cast<uintptr_t>(p_lds + p_frag_unit(m, st, mt, LS, MT))), 16, 0, 0);
      }
    };

    // ---- start of a pass: activations of phase 0, the (in A) fragments and the first packed tiles
    //      are all requested before anything is awaited ----
    if (r > 0) __syncthreads();               // everyone is done with the previous pass's LDS
    stage_issue(0, min(KP, KSl));
    if (!p_late) p_issue();
    Slot<BITS, NS> ring[RING];
#pragma unroll
    for (int i = 0; i < RING; ++i) fetch(ring[i]);
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");

    float4_t acc[TS][MT][NS];
#pragma unroll
    for (int ts = 0; ts < TS; ++ts)
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int m = 0; m < NS; ++m) acc[ts][mt][m] = float4_t{0.f, 0.f, 0.f, 0.f};

    // a rank step of one unit: the slot holds B-factor units, which meet (in A) as they are
    auto compute_lr = [&](const Slot<BITS, NS>& cur, int st, float4_t (&ac)[MT][NS]) {
#pragma unroll
      for (int m = 0; m < NS; ++m) {
        if (st >= LSm[m]) continue;
        half8_t bfrag = __builtin_bit_cast(half8_t, make_uint4(cur.cw[m][0], cur.cw[m][1], cur.cw[m][2], cur.cw[m][3]));
        if constexpr (Q3) {
          if (q3m[m]) {
            const uint32_t own[4] = {cur.cw[m][0], cur.cw[m][1], cur.cw[m][2], cur.cw[m][3]};
            bfrag = q3_unit_b(cur.mw[m], own, (c & 1) != 0);
          }
        }
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
          const half8_t pf = __builtin_bit_cast(half8_t, p_lds[p_frag_unit(DUAL ? m : 0, st, mt, LS, MT) + lane]);
          ac[mt][m] = __builtin_amdgcn_mfma_f32_16x16x32_f16(bfrag, pf, ac[mt][m], 0, 0, 0);
        }
      }
    };
    // a k-step of packed codes of one unit
    auto compute = [&](const Slot<BITS, NS>& cur, int kl, float4_t (&ac)[MT][NS]) {
      const uint4* xk = xs + size_t(kl) * 8 * 64 + lane;
      uint32_t s2[NS][NC], c2[NS];
#pragma unroll
      for (int m = 0; m < NS; ++m) {
        s2[m][0] = (cur.mw[m] & 0xffffu) | (cur.mw[m] << 16);
        c2[m] = (cur.mw[m] >> 16) | (cur.mw[m] & 0xffff0000u);
        constexpr uint32_t step = Extract<BITS>::kStepBits == 2 ? 0x44004400u : 0x48004800u;   // 4.0 or 8.0
#pragma unroll
        for (int p = 1; p < NC; ++p) s2[m][p] = pk_mul(s2[m][p - 1], step);
      }
      // One sub-step: 32 rows of both weight tiles are unpacked into MFMA operands while the
      // activation fragments wait in registers.  Where the registers allow (XB == 2) the fragments of
      // sub-step s + 1 are requested from LDS before sub-step s is unpacked; the reads and the waits
      // are written out, because the compiler would move each read down to its use.
      constexpr int XB = (MT == 1 || BITS == 2) ? 2 : 1;
      half8_t xf[XB][MT];
      uint32_t xaddr[MT];
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) xaddr[mt] = uint32_t(reinterpret_cast<uintptr_t>(xk)) + mt * KP * 8 * 1024;
      if constexpr (XB == 2) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) xf[0][mt] = lds_read16<0>(xaddr[mt]);
      }
      auto substep = [&](auto S) {
        constexpr int s = decltype(S)::value;
        if constexpr (XB == 2) {
          if constexpr (s < 7) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) xf[(s + 1) & 1][mt] = lds_read16<(s + 1) * 1024>(xaddr[mt]);
          }
        } else {
#pragma unroll
          for (int mt = 0; mt < MT; ++mt) xf[0][mt] = __builtin_bit_cast(half8_t, xk[(size_t(mt) * KP * 8 + s) * 64]);
        }
        half8_t wf[NS];
#pragma unroll
        for (int m = 0; m < NS; ++m) {
          uint32_t v[4];
#pragma unroll
          for (int j = 0; j < 4; ++j)
            v[j] = pk_fma(Extract<BITS>::field(cur.cw[m], 4 * s + j), s2[m][Extract<BITS>::cls(4 * s + j)], c2[m]);
          wf[m] = __builtin_bit_cast(half8_t, make_uint4(v[0], v[1], v[2], v[3]));
        }
        if constexpr (XB == 2) {
          // the fragments of this sub-step are older than the MT reads just issued
          if constexpr (MT == 1) lds_wait<(s < 7 ? 1 : 0)>(xf[s & 1][0]);
          else lds_wait<(s < 7 ? 2 : 0)>(xf[s & 1][0], xf[s & 1][MT - 1]);
        }
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
          for (int m = 0; m < NS; ++m)
            ac[mt][m] = __builtin_amdgcn_mfma_f32_16x16x32_f16(wf[m], xf[XB == 2 ? (s & 1) : 0][mt], ac[mt][m], 0, 0, 0);
      };
      substep(std::integral_constant<int, 0>{}); substep(std::integral_constant<int, 1>{});
      substep(std::integral_constant<int, 2>{}); substep(std::integral_constant<int, 3>{});
      substep(std::integral_constant<int, 4>{}); substep(std::integral_constant<int, 5>{});
      substep(std::integral_constant<int, 6>{}); substep(std::integral_constant<int, 7>{});
    };

    for (int ph = 0; ph < sp.n_ph; ++ph) {
      const int nk = min(KP, KSl - ph * KP);
      if (ph > 0) {
        __syncthreads();                      // everyone is done with the previous phase
        stage_issue(ph, nk);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
      }
#pragma unroll
      for (int ts = 0; ts < TS; ++ts) {
        const bool unit_ok = grp + ts * groups < units;
        for (int si = 0; si < sp.SP; si += RING) {
#pragma unroll
          for (int i = 0; i < RING; ++i) {   // slot i: consumed, then refilled RING steps ahead
            if (unit_ok && (si + i) * kw + kwi < nk) compute(ring[i], (si + i) * kw + kwi, acc[ts]);
            fetch(ring[i]);
          }
        }
      }
    }
    if (p_late && LS > 0) {                   // many rank steps: their (in A) fragments replace the activations
      __syncthreads();
      p_issue();
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      __syncthreads();
    }
#pragma unroll
    for (int ts = 0; ts < TS; ++ts) {         // the rank steps (none unless this block adds the term)
      const bool unit_ok = grp + ts * groups < units;
      for (int l0 = 0; l0 < sp.LSS; l0 += RING) {
#pragma unroll
        for (int i = 0; i < RING; ++i) {
          const int st = (l0 + i) * kw + kwi;
          if (unit_ok && st < LS) compute_lr(ring[i], st, acc[ts]);
          fetch(ring[i]);
        }
      }
    }

    // ---- wavefronts that shared a unit add up their partial sums through LDS ----
    if (kw > 1) {
      float4_t* red = reinterpret_cast<float4_t*>(xs);
      __syncthreads();
      if (kwi != 0) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
          for (int m = 0; m < NS; ++m) red[((wave * MT + mt) * NS + m) * 64 + lane] = acc[0][mt][m];
      }
      __syncthreads();
      if (kwi == 0) {
        for (int j = 1; j < kw; ++j)
#pragma unroll
          for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int m = 0; m < NS; ++m) acc[0][mt][m] += red[(((wave + j) * MT + mt) * NS + m) * 64 + lane];
      }
    }
    if (kwi != 0) continue;                  // (the next pass starts with a barrier every wavefront reaches)

    // ---- epilogue: lane holds output columns 16*tile + 4*q .. +3 of token column c ----
#pragma unroll
    for (int ts = 0; ts < TS; ++ts) {
      const int unit = grp + ts * groups;
      if (unit >= units) continue;
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        const int row = r + 16 * mt + c;
        if (row >= cnt) continue;
        const int se = a.row_exp[(a.offsets ? r0 : 0) + row];      // the row's inputs were scaled by 2^se
        if constexpr (DUAL) {
          const int tile = t0 + unit;
          const float dn = pow2i(-se), up = pow2i(2 * se);
          const float i1 = d.inv_lambda[0] * dn, i3 = d.inv_lambda[1] * dn;
          half4_t hv;
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const float g = acc[ts][mt][0][i] * i1, u = acc[ts][mt][1][i] * i3;
            hv[i] = to_f16_sat(g * __builtin_amdgcn_rcpf(1.0f + __expf(-g)) * u * up);
          }
          // h in operand order for the W2 kernel: columns f .. f+3 are half of one 16-byte unit
          const int f = tile * kTileN + 4 * q;
          *reinterpret_cast<half4_t*>(reinterpret_cast<_Float16*>(a.out) + act_unit(f >> 3, r0 + row, a.out_rt) * 8 + (f & 7)) = hv;
        } else {
          const float i2 = d.inv_lambda[2] * pow2i(-2 * se);       // (h was stored times 2^(2 se))
#pragma unroll
          for (int m = 0; m < NS; ++m) {
            const int tile = t0 + 2 * unit + m;
            if (tile >= t1) continue;
            const size_t o = size_t(r0 + row) * a.N + tile * kTileN + 4 * q;
            if (a.partial != nullptr) {          // K-blocks: fp32 partial sums, added up by the combine or by reduce_kernel
              *reinterpret_cast<float4_t*>(a.partial + size_t(kb) * a.total_rows * a.N + o) = acc[ts][mt][m] * i2;
            } else {
              uint2 yv;
              yv.x = f32x2_to_bf16x2(acc[ts][mt][m][0] * i2, acc[ts][mt][m][1] * i2);
              yv.y = f32x2_to_bf16x2(acc[ts][mt][m][2] * i2, acc[ts][mt][m][3] * i2);
              *reinterpret_cast<uint2*>(reinterpret_cast<uint16_t*>(a.out) + o) = yv;
            }
          }
        }
      }
    }
  }
}

template <int BITS, bool DUAL, bool Q3>
__global__ __launch_bounds__(64 * kWaves, 4) void qgemm_decode_kernel(KArgs a) {
  extern __shared__ uint4 xs[];
  int e = blockIdx.y, b = blockIdx.x, G = gridDim.x, r0, cnt;
  if (a.plan != nullptr) {                   // shares by table (plan.h): one 32-byte entry per block
    const PlanEntry* pe = reinterpret_cast<const PlanEntry*>(a.plan) + blockIdx.x;
    e = __builtin_amdgcn_readfirstlane(pe->e); b = __builtin_amdgcn_readfirstlane(pe->b); G = __builtin_amdgcn_readfirstlane(pe->G);
    r0 = __builtin_amdgcn_readfirstlane(pe->r0); cnt = __builtin_amdgcn_readfirstlane(pe->cnt);
    if (e < 0) return;
  } else {
    r0 = a.offsets ? a.offsets[e] : e * a.T;
    cnt = a.offsets ? a.offsets[e + 1] - r0 : a.T;
  }
  if (cnt == 0) return;
  if (cnt <= 16) decode_body<BITS, DUAL, 1, Q3>(a, xs, e, r0, cnt, b, G);
  else decode_body<BITS, DUAL, 2, Q3>(a, xs, e, r0, cnt, b, G);
}

template <bool DUAL>
__global__ __launch_bounds__(1024) void xa_rows_kernel(KArgs a) {
  __shared__ float4_t red[32][64];
  xa_rows_body<DUAL, false, 16>(a, nullptr, blockIdx.x, blockIdx.y, blockIdx.z, red);
}

// (x A1 | x A3) from the bf16 tokens in a launch of its own: the same body, block size and summation
// order as the blocks of the preparing launch that normally do this, so that a layer whose factors
// arrive late (staged residency) gets the same bits.
__global__ __launch_bounds__(1024) void xa13_tokens_kernel(KArgs a, const uint16_t* __restrict__ x_bf16) {
  __shared__ float4_t red[32][64];
  xa_rows_body<true, true, 16>(a, x_bf16, blockIdx.x, blockIdx.y, 0, red);
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
hipError_t launch_bits(const FfnArgs& f, hipStream_t s, int which) {
  int gs = 0;
  while ((1 << gs) < f.group) ++gs;
  KArgs a{};
  a.desc = f.desc; a.offsets = f.offsets; a.row_pair = f.row_pair; a.comp_rows = f.comp_rows;
  a.row_exp = f.row_exp; a.tok_exp = f.tok_exp;
  a.group_shift = gs; a.top_k = f.top_k; a.top_n = f.top_n; a.T = f.T;
  a.rank = f.rank; a.rpad = f.rpad; a.ls = (f.rank + 31) / 32; a.total_rows = f.total_rows;
  const bool comp = f.rank > 0 && f.top_n > 0 && f.row_pair != nullptr;
  // shared experts (no routing): a (blocks per expert x experts) grid; the blocks of the experts
  // together should cover the CUs, and a block takes at most 32 n-tiles
  auto blocks_per_expert = [&](int NT, int kblocks) {
    int g = (f.n_cu + f.n_exp * kblocks - 1) / (f.n_exp * kblocks);
    g = std::max(g, (NT + 31) / 32);
    return std::min(g, NT);
  };
  // activations + the (in A) fragments of small ranks
  const size_t lds = size_t(kLdsUnits + kSpareUnits) * 16;
  // routed experts: the blocks are shared out among the experts that have rows by the tables the
  // launch that prepared the activations has left (plan.h)
  const bool by_table = f.offsets != nullptr && f.plan != nullptr;
  const int pairs = f.T * f.top_k;
  // (the kernels that can dequantize 3-bit factor pairs, where the layer holds any)
  const bool q3 = comp && f.q3;
  auto k13 = q3 ? qgemm_decode_kernel<BITS, true, true> : qgemm_decode_kernel<BITS, true, false>;
  auto k2 = q3 ? qgemm_decode_kernel<BITS, false, true> : qgemm_decode_kernel<BITS, false, false>;

  if (which & 1) {
    // W1 | W3 with the SwiGLU epilogue
    a.in = f.xh; a.out = f.h; a.K = f.H; a.N = f.F; a.NT = f.F / kTileN;
    a.in_rt = f.x_rt; a.out_rt = f.h_rt;
    a.KS = padded_k(f.H) / kTileK; a.G = padded_k(f.H) / f.group;
    a.p = f.p13;
    a.kb_steps = a.KS; a.partial = nullptr;
    // ((x A1 | x A3) has been made by the launch that prepared the activations, unless it is asked for here)
    if (comp && f.xa13_here)
      hipLaunchKernelGGL(xa13_tokens_kernel, dim3(4 * a.ls, f.n_exp), dim3(1024), 0, s, a, (const uint16_t*)f.x_tokens);
    if (f.marks) (void)hipEventRecord(f.marks[0], s);
    if (by_table) {
      a.plan = f.plan;
      hipLaunchKernelGGL(k13, dim3(plan_blocks(f.n_exp, pairs, a.NT, f.n_cu), 1, 1), dim3(64 * kWaves), lds, s, a);
      a.plan = nullptr;
    } else {
      hipLaunchKernelGGL(k13, dim3(blocks_per_expert(a.NT, 1), f.n_exp, 1), dim3(64 * kWaves), lds, s, a);
    }
    if (f.marks) (void)hipEventRecord(f.marks[1], s);
  }
  if (which & 2) {
    // W2
    a.in = f.h; a.out = f.y_rows; a.K = f.F; a.N = f.H; a.NT = f.H / kTileN;
    a.in_rt = f.h_rt; a.out_rt = 0;
    a.KS = padded_k(f.F) / kTileK; a.G = padded_k(f.F) / f.group;
    a.p = f.p2;
    // a long K (many phases of staged activations) is split into K-blocks of one 16-k-step phase each;
    // their fp32 partial outputs are added by the combine, or by reduce_kernel when y_rows is wanted.
    // The rank-r term is linear in (h A2): every K-block adds B2 times the part of (h A2) over its own
    // k-steps, so (h A2) needs no sum over the K-blocks either.
    const int kblocks = decode_w2_kblocks(f);
    a.kb_steps = (a.KS + kblocks - 1) / kblocks;
    a.partial = kblocks > 1 ? f.y_part : nullptr;
    if (comp) hipLaunchKernelGGL(xa_rows_kernel<false>, dim3(2 * a.ls, f.n_exp, kblocks), dim3(1024), 0, s, a);
    if (f.marks) (void)hipEventRecord(f.marks[2], s);
    if (by_table) {
      // (second table behind the first; every K-block uses the same shares)
      a.plan = f.plan + kPlanEntryInts * plan_blocks(f.n_exp, pairs, f.F / kTileN, f.n_cu);
      const int B = plan_blocks(f.n_exp, pairs, a.NT, (f.n_cu + kblocks - 1) / kblocks);
      hipLaunchKernelGGL(k2, dim3(B, 1, kblocks), dim3(64 * kWaves), lds, s, a);
      a.plan = nullptr;
    } else {
      hipLaunchKernelGGL(k2, dim3(blocks_per_expert(a.NT, kblocks), f.n_exp, kblocks), dim3(64 * kWaves), lds, s, a);
    }
    if (kblocks > 1 && !f.keep_partials) {
      const size_t units = size_t(f.total_rows) * f.H / 4;
      hipLaunchKernelGGL(reduce_kernel, dim3((unsigned)((units + 255) / 256)), dim3(256), 0, s, f.y_part, kblocks,
                         size_t(f.total_rows) * f.H, units, reinterpret_cast<uint2*>(f.y_rows));
    }
    if (f.marks) (void)hipEventRecord(f.marks[3], s);
  }
  return hipGetLastError();
}

}  // namespace

// K-blocks of the decode flavour's W2 launch: one 16-k-step phase each, at most kMaxKBlocks
int decode_w2_kblocks(const FfnArgs& f) {
  const int KS2 = padded_k(f.F) / kTileK;
  return f.y_part ? std::min(kMaxKBlocks, (KS2 + 15) / 16) : 1;
}

void decode_plan_specs(const FfnArgs& f, int which, PlanSpec& p13, PlanSpec& p2) {
  p13 = PlanSpec{0, 0, 0, nullptr};
  p2 = PlanSpec{0, 0, 0, nullptr};
  if (f.offsets == nullptr || f.plan == nullptr) return;
  const int pairs = f.T * f.top_k, NT13 = f.F / kTileN, NT2 = f.H / kTileN;
  const int B13 = plan_blocks(f.n_exp, pairs, NT13, f.n_cu);
  if (which & 1) p13 = PlanSpec{B13, NT13, f.n_cu, f.plan};
  if (which & 2) {
    const int kb2 = decode_w2_kblocks(f);
    const int target2 = (f.n_cu + kb2 - 1) / kb2;
    p2 = PlanSpec{plan_blocks(f.n_exp, pairs, NT2, target2), NT2, target2, f.plan + kPlanEntryInts * B13};
  }
}

hipError_t decode_init_device() {
  // 128 KB of activations + 32 KB of (in A) fragments = all 160 KB of a CU
  const void* fns[12] = {
      reinterpret_cast<const void*>(&qgemm_decode_kernel<2, true, false>), reinterpret_cast<const void*>(&qgemm_decode_kernel<2, false, false>),
      reinterpret_cast<const void*>(&qgemm_decode_kernel<3, true, false>), reinterpret_cast<const void*>(&qgemm_decode_kernel<3, false, false>),
      reinterpret_cast<const void*>(&qgemm_decode_kernel<4, true, false>), reinterpret_cast<const void*>(&qgemm_decode_kernel<4, false, false>),
      reinterpret_cast<const void*>(&qgemm_decode_kernel<2, true, true>), reinterpret_cast<const void*>(&qgemm_decode_kernel<2, false, true>),
      reinterpret_cast<const void*>(&qgemm_decode_kernel<3, true, true>), reinterpret_cast<const void*>(&qgemm_decode_kernel<3, false, true>),
      reinterpret_cast<const void*>(&qgemm_decode_kernel<4, true, true>), reinterpret_cast<const void*>(&qgemm_decode_kernel<4, false, true>)};
  for (const void* fn : fns) {
    hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (kLdsUnits + kSpareUnits) * 16);
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
