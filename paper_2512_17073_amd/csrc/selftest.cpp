// Host-only self-check of the decode-flavour FFN kernels' index arithmetic (no device needed).
// The kernels form every buffer offset and LDS address through the functions of decode_index.h;
// this file walks the same functions for every block, wavefront, lane and step of a launch and
// checks each result against the size of what it addresses, and that the blocks and wavefronts
// together read every packed tile of the expert exactly once per pass.
#include <cstdio>
#include <string>
#include <vector>

#include <cmath>
#include <cstring>

#include "decode_index.h"
#include "factor_q3.h"
#include "ffn_common.h"
#include "internal.h"
#include "pack.h"

namespace lrc {

namespace {

using namespace dec;

struct Shape {
  int K, N, bits, group, ls_max, LSm[2], r0, cnt, total_rows, G, kblocks;
  bool dual;
};

#define SELF_FAIL(...)                                 \
  do {                                                 \
    char buf_[512];                                    \
    std::snprintf(buf_, sizeof buf_, __VA_ARGS__);     \
    return std::string(buf_);                          \
  } while (0)

// "" if every index of one launch shape is in range, else the first violation
std::string check_shape(const Shape& sh) {
  const int Kp = padded_k(sh.K), KS = Kp / kTileK, NT = sh.N / kTileN, Gr = Kp / sh.group;
  int gs = 0;
  while ((1 << gs) < sh.group) ++gs;
  const uint32_t code_bytes = uint32_t(KS) * NT * (kWave * 2 * sh.bits * 4), meta_bytes = uint32_t(Gr) * NT * kTileN * 4;
  const uint32_t bf_bytes_max = uint32_t(NT) * sh.ls_max * 1024;
  const int rt = sh.total_rows + kActPadRows;                       // rows of the operand-order activation buffers
  const size_t in_units = size_t(rt) * Kp / 8;
  const int kb_steps = (KS + sh.kblocks - 1) / sh.kblocks;
  const int MT = sh.cnt <= 16 ? 1 : 2, NP = sh.dual ? 2 : 1;
  const int pitch = NP * sh.ls_max * 32;
  for (int kb = 0; kb < sh.kblocks; ++kb) {
    const int ks_lo = kb * kb_steps, KSl = std::min(KS, ks_lo + kb_steps) - ks_lo;
    if (KSl <= 0) SELF_FAIL("K-block %d of %d has no k-step", kb, sh.kblocks);
    const bool lowrank = sh.LSm[0] > 0 || sh.LSm[1] > 0;
    const int LS = lowrank ? std::max(sh.LSm[0], sh.LSm[1]) : 0;
    std::vector<int> seen(size_t(KSl) * NT * 2, 0), seen_lr(size_t(std::max(LS, 1)) * NT * 2, 0);
    for (int b = 0; b < sh.G; ++b) {
      int t0, t1;
      block_tiles(b, sh.G, NT, t0, t1);
      const int nt_b = t1 - t0;
      if (nt_b == 0) continue;
      if (nt_b > max_block_tiles(MT)) SELF_FAIL("block %d of %d owns %d n-tiles (at most %d)", b, sh.G, nt_b, max_block_tiles(MT));
      const int units = block_units(nt_b, sh.dual), kw = waves_per_unit(units), groups = kWaves / kw;
      if (units > groups * unit_slots(sh.dual, MT)) SELF_FAIL("%d units do not fit %d wavefront groups", units, groups);
      const StepPlan sp = step_plan(KSl, MT, kw, LS, sh.dual);
      const int p_frags = NP * LS * MT;
      const bool p_late = p_frags * 64 > kSpareUnits;
      if (p_frags * 64 > (p_late ? kLdsUnits : kSpareUnits)) SELF_FAIL("%d (in A) fragments exceed their LDS region", p_frags);
      if (kw > 1 && ((kWaves * MT) * kStreams) * 64 > kLdsUnits) SELF_FAIL("reduction buffer exceeds LDS");
      for (int r = 0; r < sh.cnt; r += 16 * MT) {
        // staging: LDS units and global units
        for (int ph = 0; ph < sp.n_ph; ++ph) {
          const int nk = std::min(sp.KP, KSl - ph * sp.KP);
          for (int wave = 0; wave < kWaves; ++wave)
            for (int mt = 0; mt < MT; ++mt)
              for (int kl = wave >> 3; kl < nk; kl += 2)
                for (int lane = 0; lane < 64; ++lane) {
                  const int q = lane >> 4, rowl = lane & 15, s = wave & 7;
                  const int k8 = std::min((ks_lo + ph * sp.KP + kl) * 32 + q * 8 + s, sh.K / 8 - 1);
                  if (act_frag_unit(mt, kl, s, sp.KP) + 64 > kLdsUnits) SELF_FAIL("staged fragment (mt %d, kl %d, s %d) leaves LDS", mt, kl, s);
                  const int row = staged_row(sh.r0 + r, r, mt, rowl, sh.cnt, rt);
                  if (row < 0 || row >= rt) SELF_FAIL("staging reads row %d of %d", row, rt);
                  if (r + 16 * mt + rowl < sh.cnt ? row != sh.r0 + r + 16 * mt + rowl : row < sh.total_rows + kActPadRows - kZeroRows)
                    SELF_FAIL("staging reads row %d for row %d of an expert with %d rows at %d", row, r + 16 * mt + rowl, sh.cnt, sh.r0);
                  const size_t u = ffn::act_unit(k8, row, rt);
                  if (u >= in_units) SELF_FAIL("staging reads unit %zu of %zu (row %d of %d)", u, in_units, row, rt);
                }
        }
        // (in A) fragments
        for (int f = 0; f < p_frags; ++f) {
          const int mt = f % MT, g = f / MT, st = g % LS, m = g / LS;
          if (p_frag_unit(m, st, mt, LS, MT) + 64 > (p_late ? kLdsUnits : kSpareUnits)) SELF_FAIL("(in A) fragment %d leaves its LDS region", f);
          for (int lane = 0; lane < 64; ++lane) {
            const int q = lane >> 4, c = lane & 15;
            const int row = sh.r0 + std::min(r + 16 * mt + c, sh.cnt - 1);
            const size_t h = size_t(row) * pitch + m * sh.ls_max * 32 + 32 * st + 8 * q;
            if (h + 8 > size_t(sh.total_rows) * pitch) SELF_FAIL("(in A) copy reads half %zu of %zu", h, size_t(sh.total_rows) * pitch);
          }
        }
        // the steps of every wavefront (the kernel fetches RING steps past the last one)
        if (r > 0) continue;                  // (the steps do not depend on the pass)
        for (int wave = 0; wave < kWaves; ++wave) {
          const int grp = wave / kw, kwi = wave % kw;
          StepCursor cur = cursor_start();
          for (int n = 0; n < sp.n_reg + sp.LSP + kRing; ++n) {
            // the kernel walks the steps with the cursor; step_ref is the closed form it must agree with
            const StepRef want = step_ref(n, sp, grp, groups, kwi, kw, units, ks_lo, KSl, LS, sh.dual);
            const StepRef ref = cursor_ref(cur, sp, grp, groups, kwi, kw, units, ks_lo, KSl, LS);
            cursor_advance(cur, sp);
            if (ref.reg != want.reg || ref.lr != want.lr) SELF_FAIL("step %d: the cursor disagrees on what kind of step it is", n);
            if (ref.reg && (ref.unit != want.unit || ref.ks != want.ks || ref.kl != want.kl || ref.ts != want.ts))
              SELF_FAIL("step %d: the cursor is at k-step %d of unit %d, the closed form at %d of %d", n, ref.ks, ref.unit, want.ks, want.unit);
            if (ref.lr && (ref.unit != want.unit || ref.st != want.st || ref.ts != want.ts))
              SELF_FAIL("step %d: the cursor is at rank step %d of unit %d, the closed form at %d of %d", n, ref.st, ref.unit, want.st, want.unit);
            if (ref.reg && ref.lr) SELF_FAIL("step %d is both a k-step and a rank step", n);
            for (int m = 0; m < kStreams; ++m) {
              const int tile = stream_tile(t0, ref.unit, m, sh.dual);
              const bool tile_ok = tile < t1;
              const uint32_t bf_size = uint32_t(NT) * (lowrank ? sh.LSm[sh.dual ? m : 0] : 0) * 1024;
              for (int lane = 0; lane < 64; ++lane) {
                const LaneOffsets o = lane_offsets(ref, tile, tile_ok, lane, sh.bits, NT, gs, code_bytes, meta_bytes, bf_bytes_max);
                const uint32_t w1 = sh.bits == 3 ? 8 : 16;
                if (ref.reg && tile_ok) {
                  if (ref.ks < ks_lo || ref.ks >= ks_lo + KSl || tile < t0) SELF_FAIL("step %d reads k-step %d tile %d outside the block's share", n, ref.ks, tile);
                  if (o.code0 + 16 > code_bytes) SELF_FAIL("code load at %u + 16 > %u", o.code0, code_bytes);
                  if (sh.bits > 2 && o.code1 + w1 > code_bytes) SELF_FAIL("second code load at %u > %u", o.code1, code_bytes);
                  if (o.meta + 4 > meta_bytes) SELF_FAIL("metadata load at %u + 4 > %u", o.meta, meta_bytes);
                  const uint32_t tdw = kWave * 2 * sh.bits * 4;
                  if (o.code0 != (uint32_t(ref.ks) * NT + tile) * tdw + lane * 16) SELF_FAIL("code offset does not address tile (%d, %d)", ref.ks, tile);
                  if (lane == 0) ++seen[(size_t(ref.ks - ks_lo) * NT + tile) * 2 + (sh.dual ? m : 0)];
                } else {
                  // (the kernel takes the first load from the B factor's resource on a rank step, else from the codes')
                  const uint32_t off1 = ref.lr ? o.bf : o.code0, size1 = ref.lr ? bf_size : code_bytes;
                  if (!(ref.lr && tile_ok) && off1 < size1) SELF_FAIL("idle step %d loads inside a resource (offset %u of %u)", n, off1, size1);
                  if (o.code1 < code_bytes) SELF_FAIL("idle step %d: second code load inside the resource", n);
                  if (o.meta < meta_bytes) SELF_FAIL("idle step %d: metadata load inside the resource", n);
                }
                if (ref.lr && tile_ok) {
                  // inside the stream's own factor, or wholly past it (zeros): never astride its end
                  const bool inside = o.bf + 16 <= bf_size, outside = o.bf >= bf_size;
                  if (!inside && !outside) SELF_FAIL("rank step %d straddles the end of the B factor", ref.st);
                  if ((ref.st < (lowrank ? sh.LSm[sh.dual ? m : 0] : 0)) != inside) SELF_FAIL("rank step %d of stream %d: wrong side of the factor's end", ref.st, m);
                  if (inside && lane == 0) ++seen_lr[(size_t(ref.st) * NT + tile) * 2 + (sh.dual ? m : 0)];
                }
                // the same step of a stream whose pair is held at 3 bits: metadata through `bf`, codes through `bc`
                {
                  const int LSq = lowrank ? sh.LSm[sh.dual ? m : 0] : 0;
                  const uint32_t bm_size = uint32_t(NT / 4) * LSq * 128, bc_size = uint32_t(NT) * LSq * 256;
                  const LaneOffsets oq = lane_offsets(ref, tile, tile_ok, lane, sh.bits, NT, gs, code_bytes, meta_bytes, bf_bytes_max, true);
                  if (oq.code0 != o.code0 || oq.code1 != o.code1 || oq.meta != o.meta) SELF_FAIL("3-bit pairs change the k-step offsets of step %d", n);
                  if (ref.lr && tile_ok && ref.st < LSq) {
                    const uint32_t q = lane >> 4, c = lane & 15;
                    if (oq.bf != ((uint32_t(ref.st) * (NT / 4) + tile / 4) * 4 + q) * 32 + (c & 1) * 16 || oq.bf + 16 > bm_size)
                      SELF_FAIL("rank step %d: metadata of a 3-bit unit at %u of %u", ref.st, oq.bf, bm_size);
                    if (oq.bc != (uint32_t(ref.st) * NT + tile) * 256 + lane * 4 || oq.bc + 4 > bc_size)
                      SELF_FAIL("rank step %d: codes of a 3-bit unit at %u of %u", ref.st, oq.bc, bc_size);
                  } else {
                    if (ref.lr && oq.bf < bm_size) SELF_FAIL("step %d reads 3-bit metadata it should not (offset %u of %u)", n, oq.bf, bm_size);
                    // (the kernel reads through `bc` on rank steps only, from the codes' resource)
                    if (ref.lr && oq.bc < bc_size) SELF_FAIL("step %d reads 3-bit codes it should not (offset %u of %u)", n, oq.bc, bc_size);
                  }
                }
              }
            }
          }
        }
      }
    }
    // every packed tile of the K-block exactly once (both streams of a dual launch)
    for (int ks = 0; ks < KSl; ++ks)
      for (int t = 0; t < NT; ++t)
        for (int m = 0; m < (sh.dual ? 2 : 1); ++m)
          if (seen[(size_t(ks) * NT + t) * 2 + m] != 1)
            SELF_FAIL("K-block %d: tile (k-step %d, n-tile %d, stream %d) read %d times", kb, ks, t, m, seen[(size_t(ks) * NT + t) * 2 + m]);
    for (int st = 0; st < LS; ++st)
      for (int t = 0; t < NT; ++t)
        for (int m = 0; m < (sh.dual ? 2 : 1); ++m) {
          const int want = st < sh.LSm[sh.dual ? m : 0] ? 1 : 0;
          if (seen_lr[(size_t(st) * NT + t) * 2 + m] != want)
            SELF_FAIL("rank step %d n-tile %d stream %d read %d times (want %d)", st, t, m, seen_lr[(size_t(st) * NT + t) * 2 + m], want);
        }
  }
  return "";
}

}  // namespace

}  // namespace lrc

using namespace lrc;

extern "C" int moe_lrc_selftest_decode_index(int hidden, int ffn, int bits, int group, int layer_rank, int rank1,
                                             int rank3, int rank2, int first_row, int rows, int total_rows,
                                             int blocks_w13, int blocks_w2, int kblocks_w2) {
  if (hidden <= 0 || ffn <= 0 || hidden % 64 || ffn % 64 || bits < 2 || bits > 4 ||
      (group != 64 && group != 128 && group != 256) || layer_rank < 0 || layer_rank > 1024 || rank1 < 0 ||
      rank3 < 0 || rank2 < 0 || rank1 > layer_rank || rank3 > layer_rank || rank2 > layer_rank || rows < 1 ||
      first_row < 0 || first_row + rows > total_rows || blocks_w13 < 1 || blocks_w2 < 1 || kblocks_w2 < 1 ||
      kblocks_w2 > kMaxKBlocks)
    return set_error(MOE_LRC_EINVAL, "selftest_decode_index: argument out of range");
  const int ls = (layer_rank + 31) / 32;
  Shape a{hidden, ffn, bits, group, ls, {(rank1 + 31) / 32, (rank3 + 31) / 32}, first_row, rows, total_rows, blocks_w13, 1, true};
  std::string err = check_shape(a);
  if (!err.empty()) return set_error(MOE_LRC_ESHAPE, "selftest_decode_index (W1|W3): " + err);
  Shape b{ffn, hidden, bits, group, ls, {(rank2 + 31) / 32, (rank2 + 31) / 32}, first_row, rows, total_rows, blocks_w2, kblocks_w2, false};
  err = check_shape(b);
  if (!err.empty()) return set_error(MOE_LRC_ESHAPE, "selftest_decode_index (W2): " + err);
  return MOE_LRC_OK;
}

namespace {
// one half of a packed fp16 FMA as the device computes it: exact product and sum, one rounding
float half_fma(uint16_t f, uint16_t s, uint16_t c) {
  auto h = [](uint16_t b) { _Float16 v; std::memcpy(&v, &b, 2); return (double)v; };
  return (float)(_Float16)std::fma(h(f), h(s), h(c));
}
uint32_t q3_field_rt(uint32_t v, int i) {
  return i == 0 ? ffn::q3_field<0>(v) : i == 1 ? ffn::q3_field<1>(v) : i == 2 ? ffn::q3_field<2>(v) : ffn::q3_field<3>(v);
}
}  // namespace

extern "C" int moe_lrc_selftest_factor_pair(int K, int N, int rank, const uint8_t* a_codes, const uint16_t* a_scale,
                                          const uint16_t* a_zero, const uint8_t* b_codes, const uint16_t* b_scale,
                                          const uint16_t* b_zero, float* A_out, float* B_out) {
  if (!a_codes || !a_scale || !a_zero || !b_codes || !b_scale || !b_zero || !A_out || !B_out)
    return set_error(MOE_LRC_EINVAL, "selftest_factor_pair: null argument");
  if (K <= 0 || N <= 0 || K % 64 || N % 64 || rank <= 0 || rank > 1024 || rank % 8)
    return set_error(MOE_LRC_ESHAPE, "selftest_factor_pair: K and N must be multiples of 64, rank a multiple of 8 in 8..1024");
  std::vector<uint8_t> abuf(q3_a_bytes(K, rank)), bbuf(q3_b_bytes(N, rank));
  const float mu_a = pack_factor_a_q3(K, rank, a_codes, a_scale, a_zero, abuf.data());
  const float mu_b = pack_factor_b_q3(N, rank, b_codes, b_scale, b_zero, bbuf.data());
  if (mu_a == 0.f || mu_b == 0.f) return set_error(MOE_LRC_EINVAL, "selftest_factor_pair: code out of range (3 bits)");
  // A: the reads of the (in A) kernels: unit (tile, kk), lane (q, c); codes dword, metadata dword of (tile, kk / 2, c)
  const int k32 = K / 32, g64 = K / 64, NT = N / 16, NG = N / 64;
  const uint32_t* acw = reinterpret_cast<const uint32_t*>(abuf.data());
  const uint32_t* amw = reinterpret_cast<const uint32_t*>(abuf.data() + q3_a_codes_bytes(K, rank));
  for (int tile = 0; tile < (rank + 15) / 16; ++tile)
    for (int kk = 0; kk < k32; ++kk)
      for (int lane = 0; lane < 64; ++lane) {
        const int q = lane >> 4, c = lane & 15, rho = 16 * tile + c;
        const uint32_t codes = acw[(size_t(tile) * k32 + kk) * 64 + lane], meta = amw[(size_t(tile) * g64 + (kk >> 1)) * 16 + c];
        for (int j = 0; j < 8; ++j) {
          const uint32_t f = q3_field_rt(codes, j >> 1);
          const float v = half_fma(uint16_t(j & 1 ? f >> 16 : f), uint16_t(meta), uint16_t(meta >> 16)) / mu_a;
          if (rho < rank) A_out[size_t(32 * kk + 8 * q + j) * rank + rho] = v;
          else if (v != 0.f) return set_error(MOE_LRC_ESHAPE, "selftest_factor_pair: a column of A past the rank is not zero");
        }
      }
  // B: the reads of the FFN kernels' rank steps: unit (st, nt), lane (q, c); codes dword, 32 bytes of
  // metadata of (st, nt / 4, q): eight scale halves, then eight offset halves
  const uint32_t* bcw = reinterpret_cast<const uint32_t*>(bbuf.data());
  const uint16_t* bmh = reinterpret_cast<const uint16_t*>(bbuf.data() + q3_b_codes_bytes(N, rank));
  for (int st = 0; st < (rank + 31) / 32; ++st)
    for (int nt = 0; nt < NT; ++nt)
      for (int lane = 0; lane < 64; ++lane) {
        const int q = lane >> 4, c = lane & 15;
        const uint32_t codes = bcw[(size_t(st) * NT + nt) * 64 + lane];
        const uint16_t* mh = bmh + ((size_t(st) * NG + nt / 4) * 4 + q) * 16;
        for (int j = 0; j < 8; ++j) {
          const uint32_t f = q3_field_rt(codes, j >> 1);
          const float v = half_fma(uint16_t(j & 1 ? f >> 16 : f), mh[j], mh[8 + j]) / mu_b;
          const int rho = 32 * st + 8 * q + j;
          if (rho < rank) B_out[size_t(rho) * N + nt * 16 + c] = v;
          else if (v != 0.f) return set_error(MOE_LRC_ESHAPE, "selftest_factor_pair: a row of B past the rank is not zero");
        }
      }
  return MOE_LRC_OK;
}
