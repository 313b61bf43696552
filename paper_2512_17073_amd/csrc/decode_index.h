// Index arithmetic of the decode-flavour FFN kernels (ffn_decode.hip), as plain integer functions
// that compile for the device and for the host.  The kernels call them; moe_lrc_selftest_decode_index
// (host only) sweeps shapes, ranks and block shares through the same functions and checks every
// offset against the size of the buffer resource or LDS region it addresses.
#pragma once
#include <stdint.h>

#include "layout.h"

namespace lrc {
namespace dec {

constexpr int kWaves = 16;            // wavefronts of a block
constexpr int kLdsUnits = 8192;       // 16-byte units of staged activations (128 KB)
constexpr int kSpareUnits = 2048;     // 16-byte units behind them (32 KB): (in A) fragments of small ranks
constexpr int kRing = 2;              // ring slots of a wavefront (each holds one k-step of two streams)
constexpr int kStreams = 2;           // streams of a slot: (W1, W3) tiles of one n-tile, or two n-tiles of W2

// A block's n-tiles: block b of the G that share an expert owns tiles [t0, t1).
LRC_HD void block_tiles(int b, int G, int NT, int& t0, int& t1) {
  t0 = (int)((long long)b * NT / G);
  t1 = (int)((long long)(b + 1) * NT / G);
}

// Work units of a block: an n-tile of both projections (DUAL) or a pair of adjacent n-tiles (W2).
LRC_HD int block_units(int nt_b, bool dual) { return dual ? nt_b : (nt_b + 1) / 2; }
// Unit slots a wavefront visits one after the other.
LRC_HD int unit_slots(bool dual, int mt) { (void)mt; return dual ? 2 : 1; }
// n-tiles a block can own
LRC_HD int max_block_tiles(int mt) { (void)mt; return 32; }

// Wavefronts that share one unit, each taking every kw-th k-step (power of two, 1..16).
LRC_HD int waves_per_unit(int units) {
  int kw = 1;
  while (kw < kWaves && units * kw * 2 <= kWaves) kw *= 2;
  return kw;
}

// n-tile of stream m of unit u (block-relative unit index): DUAL: tile t0 + u for both streams;
// W2: tiles t0 + 2u and t0 + 2u + 1.
LRC_HD int stream_tile(int t0, int u, int m, bool dual) { return dual ? t0 + u : t0 + 2 * u + m; }

// Steps of a wavefront, in order: [phase][unit slot][own k-step], then [unit slot][own rank step];
// each innermost segment is padded to a multiple of the ring depth, so that ring slots are indexed
// statically.
struct StepPlan {
  int TS;        // unit slots
  int KP;        // k-steps per phase (16 with one row tile, 8 with two)
  int n_ph;      // phases of this K-block
  int SP;        // padded own k-steps per (unit slot, phase) segment
  int n_reg;     // regular steps in all
  int LSS;       // padded own rank steps per unit slot
  int LSP;       // padded rank steps in all
};
LRC_HD StepPlan step_plan(int KSl, int mt, int kw, int LS, bool dual) {
  StepPlan p;
  p.TS = unit_slots(dual, mt);
  p.KP = (kLdsUnits / 512) / mt;
  p.n_ph = (KSl + p.KP - 1) / p.KP;
  const int spw = (p.KP + kw - 1) / kw;
  p.SP = (spw + kRing - 1) / kRing * kRing;
  p.n_reg = p.n_ph * p.TS * p.SP;
  p.LSS = ((LS + kw - 1) / kw + kRing - 1) / kRing * kRing;
  p.LSP = p.TS * p.LSS;
  return p;
}

// What step n of a wavefront (group grp of `groups`, k-share kwi of kw) reads.
struct StepRef {
  bool reg;      // a k-step of packed codes (else a rank step, or nothing)
  bool lr;       // a rank step of the B factor
  int ts;        // unit slot
  int unit;      // block-relative unit
  int ks;        // absolute k-step (reg)
  int kl;        // k-step within the phase (reg)
  int st;        // rank step (lr)
};
LRC_HD StepRef step_ref(int n, const StepPlan& p, int grp, int groups, int kwi, int kw, int units, int ks_lo, int KSl,
                        int LS, bool dual) {
  StepRef r{};
  const int TS = p.TS;
  (void)dual;
  if (n < p.n_reg) {
    const int seg = n / p.SP, si = n - seg * p.SP, ph = seg / TS;
    r.ts = seg - ph * TS;
    r.unit = grp + r.ts * groups;
    r.kl = si * kw + kwi;
    r.ks = ks_lo + ph * p.KP + r.kl;
    r.reg = r.unit < units && r.kl < p.KP && ph * p.KP + r.kl < KSl;
  } else {
    const int l = n - p.n_reg;
    r.ts = p.LSS > 0 ? l / p.LSS : 0;
    r.unit = grp + r.ts * groups;
    r.st = (p.LSS > 0 ? l - r.ts * p.LSS : 0) * kw + kwi;
    r.lr = l < p.LSP && r.unit < units && r.st < LS;
  }
  return r;
}

// The same sequence walked one step at a time, without divisions: the kernel fetches the steps
// 0, 1, 2, ... of a pass in order, two of them past the last one.  cursor_ref gives what step_ref
// gives for the cursor's step (for a step that reads nothing only `reg` and `lr`, both false, are
// meant to agree).
struct StepCursor {
  int part;      // 0: k-steps, 1: rank steps
  int ph;        // phase (k-steps)
  int ts;        // unit slot (past the last one: nothing left)
  int si;        // index within the (phase, unit slot) or (unit slot) segment
};
LRC_HD StepCursor cursor_start() { return StepCursor{0, 0, 0, 0}; }
LRC_HD StepRef cursor_ref(const StepCursor& c, const StepPlan& p, int grp, int groups, int kwi, int kw, int units, int ks_lo,
                          int KSl, int LS) {
  StepRef r{};
  r.ts = c.ts;
  r.unit = grp + c.ts * groups;
  const int own = c.si * kw + kwi;
  if (c.part == 0) {
    r.kl = own;
    r.ks = ks_lo + c.ph * p.KP + own;
    r.reg = r.unit < units && own < p.KP && c.ph * p.KP + own < KSl;
  } else {
    r.st = own;
    r.lr = c.ts < p.TS && c.si < p.LSS && r.unit < units && own < LS;
  }
  return r;
}
LRC_HD void cursor_advance(StepCursor& c, const StepPlan& p) {
  ++c.si;
  if (c.si == (c.part ? p.LSS : p.SP)) { c.si = 0; ++c.ts; }
  if (c.part == 0 && c.ts == p.TS) {
    c.ts = 0;
    ++c.ph;
    if (c.ph == p.n_ph) c.part = 1;
  }
}

// Byte offsets of a lane's loads of one stream of a step (the hardware range-checks offset + size
// against the resource; a step that reads nothing gets an offset at the end of every resource).
// q3: the stream's factor pair is held at 3 bits (layout.h).  A rank step then reads, through `bf`,
// the lane's half of the 32 bytes of metadata of (rank step, group of four n-tiles, lane group) from
// a resource of (NT / 4) * LS * 128 bytes, and through `bc` the unit's code dword from a resource of
// NT * LS * 256 bytes; `bc` of any other step lies past every resource.
struct LaneOffsets { uint32_t code0, code1, meta, bf, bc; };
LRC_HD LaneOffsets lane_offsets(const StepRef& r, int tile, bool tile_ok, int lane, int bits, int NT, int group_shift,
                                uint32_t code_bytes, uint32_t meta_bytes, uint32_t bf_bytes_max, bool q3 = false) {
  const uint32_t tdw = kWave * 2 * bits, q = lane >> 4, c = lane & 15;
  const uint32_t gps = kTileK >> group_shift;
  const uint32_t meta_lane = ((q * kLaneK) >> group_shift) * (uint32_t(NT) * kTileN * 4) + c * 4;
  LaneOffsets o;
  const bool ok = r.reg && tile_ok, lr = r.lr && tile_ok;
  const uint32_t past = code_bytes > bf_bytes_max ? code_bytes : bf_bytes_max;
  const uint32_t tile_base = (uint32_t(r.ks) * NT + tile) * (tdw * 4);
  o.code0 = (ok ? tile_base : past) + lane * 16;
  o.code1 = (ok ? tile_base : code_bytes) + 1024 + lane * (bits == 3 ? 8 : 16);
  o.meta = (ok ? (uint32_t(r.ks) * gps * NT + tile) * (kTileN * 4) : meta_bytes) + meta_lane;
  // (selects on wave-uniform conditions rather than branches: the loads of a step stay in one block)
  const bool lq = q3 && lr;
  const uint32_t unit = uint32_t(r.st) * NT + tile, group4 = uint32_t(r.st) * (NT / 4) + (tile >> 2);
  o.bf = (lq ? group4 * 128 : lr ? unit * 1024 : past) + (lq ? q * 32 + (c & 1) * 16 : lane * 16);
  o.bc = (lq ? unit * 256 : 0xfffffe00u) + lane * 4;
  return o;
}

// Row of the operand-order activation buffer (in_rt rows) that lane row `rowl` of row tile mt stages
// in the pass that starts at the expert's row r (rin: that row's index in the buffer).  Past the
// expert's last row the MFMA columns are never stored: they read the buffer's last 16 rows, which
// the preparing launch keeps at zero (multiplying zeros costs the matrix cores the least).
constexpr int kZeroRows = 16;
LRC_HD int staged_row(int rin, int r, int mt, int rowl, int cnt, int in_rt) {
  return r + 16 * mt + rowl < cnt ? rin + 16 * mt + rowl : in_rt - kZeroRows + rowl;
}

// LDS unit of staged activation fragment (row tile mt, k-step kl of the phase, sub-step s).
LRC_HD int act_frag_unit(int mt, int kl, int s, int KP) { return ((mt * KP + kl) * 8 + s) * 64; }
// LDS unit (relative to the fragment region) of (in A) fragment (stream m, rank step st, row tile mt).
LRC_HD int p_frag_unit(int m, int st, int mt, int LS, int MT) { return ((m * LS + st) * MT + mt) * 64; }


}  // namespace dec
}  // namespace lrc
