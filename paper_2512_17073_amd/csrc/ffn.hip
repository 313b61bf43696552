// Expert FFN on grouped rows (Sections 2.3 and 3.2), many-rows flavour (prefill):
//   g = x D1 + c (x A1) B1,  u = x D3 + c (x A3) B3,  h = silu(g) * u,  y = h D2 + c (h A2) B2
// with D = Qinv(Q(W)) unpacked from the bit-packed codes inside the wavefront's registers and
// c = 1 only for rows that hold a Top-n (token, expert) pair.
//
// With hundreds of rows per expert the work is a grouped GEMM and the matrix cores are the bound.
// Kernel design (gfx950):
//   - a block of 8 wavefronts owns 128 rows of one expert x 256 output columns (of both W1 and W3
//     in the fused kernel); a wavefront owns two n-tiles (16 columns each) for all 128 rows, so a
//     tile of weights unpacked once in registers (unpack.h) feeds all the rows;
//   - the products run on v_mfma_f32_32x32x16_f16 (the same peak rate as the 16x16x32 shape, half
//     as many MFMA and LDS-read instructions per flop, and on this chip the matrix pipe and the
//     vector ALU share the wavefront's issue slots, so instructions saved are time saved): two
//     streams of 16 output columns that meet the same activations (W1 and W3 of one n-tile, or two
//     n-tiles of W2) become the 32 rows of one A operand by a swap of 16-lane rows between their
//     registers, which puts the same inputs of both streams side by side; the activations are
//     staged as fragments of 32 rows;
//   - the packed weights never touch LDS: each wavefront streams its tiles HBM -> registers through
//     a two-slot ring of buffer loads (a load past the end of the resource returns zeros, so the
//     refills are unconditional and the waits static);
//   - the activations of one k-step (128 rows x 256 columns, 64 KB, MFMA operand order) are
//     double-buffered in LDS: the copy of the next k-step goes from global memory straight to LDS
//     (no registers) while the current one is multiplied; one barrier per k-step;
//   - the rank-r term rides the same stream as extra steps: the B factor's 32-wide units take the
//     place of the codes in a ring slot and meet (in A), which a small kernel of the same shape
//     (xa_tile_kernel: fp16 factor tiles instead of packed codes) has left in global memory.
// Experts with few rows (decode) take the other flavour, ffn_decode.hip.
#include <algorithm>
#include <type_traits>
#include <utility>

#include "decode_index.h"
#include "factor_q3.h"
#include "ffn_common.h"
#include "plan.h"

namespace lrc {

namespace {

using namespace ffn;

constexpr int kTileWaves = 8;             // wavefronts per block
constexpr int kBM = 128;                  // rows of an expert per block
constexpr int kTMT = kBM / 16;            // row tiles
constexpr int kStepUnits = kTMT * 8 * 64; // 16-byte units of one k-step of activations (64 KB)
// Work item `item` of a launch -> (expert, first row of its 128-row chunk).  Routed experts: the
// items enumerate the chunks of the experts in order (an expert with cnt rows has ceil(cnt / 128));
// shared experts: every expert has the same T rows.
struct Chunk { int e, r0, cnt, r; };
__device__ inline bool find_chunk(const KArgs& a, int item, Chunk& c) {
  if (!a.offsets) {
    const int per = (a.T + kBM - 1) / kBM;
    c.e = item / per; c.r = (item - c.e * per) * kBM; c.r0 = c.e * a.T; c.cnt = a.T;
    return c.e < a.n_exp;
  }
  // 64 experts at a time: every lane counts the chunks of one expert, a prefix sum over the
  // wavefront finds the one that holds the item (every wavefront of the block does the same)
  const int lane = threadIdx.x & 63;
  int base = 0;
  for (int e0 = 0; e0 < a.n_exp; e0 += 64) {
    const int e = e0 + lane;
    int r0 = 0, cnt = 0;
    if (e < a.n_exp) { r0 = a.offsets[e]; cnt = a.row_list ? a.comp_rows[e] : a.offsets[e + 1] - r0; }
    const int n = (cnt + kBM - 1) / kBM;
    int incl = n;
#pragma unroll
    for (int dlt = 1; dlt < 64; dlt *= 2) {
      const int t = __shfl_up(incl, dlt);
      if (lane >= dlt) incl += t;
    }
    const int total = __shfl(incl, 63);
    if (item < base + total) {
      const unsigned long long hit = __ballot(base + incl > item);
      const int first = __ffsll(hit) - 1;
      c.e = e0 + first;
      c.r0 = __shfl(r0, first); c.cnt = __shfl(cnt, first);
      c.r = (item - base - __shfl(incl - n, first)) * kBM;
      return true;
    }
    base += total;
  }
  return false;
}

// Copy of the activations of k-step ks for the 128 rows of a chunk into `buf`, as 64 fragments (row
// tile mt, sub-step s) of 64 units: wavefront w copies the fragments with s = w, each lane its own 16
// bytes from global memory straight to LDS; R[mt] is this lane's input row of row tile mt.  A column
// past the end is clamped to a valid unit (the padded weights of such columns are exact zeros).
__device__ inline void stage_step_rows(const KArgs& a, uint4* buf, int ks, const int (&R)[kTMT], int mt_n, int wave, int lane) {
  const uint4* in_units = reinterpret_cast<const uint4*>(a.in);
  const int q = lane >> 4, s = wave;
  const int k8 = min(ks * 32 + q * 8 + s, a.K / 8 - 1);
#pragma unroll
  for (int mt = 0; mt < kTMT; ++mt)
    if (mt < mt_n)        // (row tiles past the chunk's last row are not read)
    __builtin_amdgcn_global_load_lds(
        reinterpret_cast<const __attribute__((address_space(1))) void*>(reinterpret_cast<uintptr_t>(in_units + act_unit(k8, R[mt], a.in_rt))),
        reinterpret_cast<__attribute__((address_space(3))) void*>(reinterpret_cast<uintptr_t>(buf + (mt * 8 + s) * 64)), 16, 0, 0);
}

typedef float float16_t __attribute__((ext_vector_type(16)));
constexpr int kRP = kBM / 32;             // 32-row fragments ("row pairs") of a chunk
constexpr int kTileLdsAhead = 2;          // LDS fragment reads in flight ahead of the MFMAs (1 to 4 measured alike)

// fn(std::integral_constant<int, 0>{}) ... fn(std::integral_constant<int, N - 1>{})
template <int... I, class Fn> __device__ inline void static_for_impl(std::integer_sequence<int, I...>, Fn&& fn) {
  (fn(std::integral_constant<int, I>{}), ...);
}
template <int N, class Fn> __device__ inline void static_for(Fn&& fn) { static_for_impl(std::make_integer_sequence<int, N>{}, fn); }

// The same k-step as fragments for the 32x32x16 products: fragment (row pair rp, sub-step s, operand p)
// at unit ((rp * 8 + s) * 2 + p) * 64; lane l holds, of row 32 rp + l % 32, the 8 inputs of lane
// group q = p + 2 (l / 32) of sub-step s.  (After the row swap, operand p of a sub-step holds in
// lanes 0..31 the weights of lane group q = p and in lanes 32..63 those of q = p + 2.)  Wavefront w
// of the block's WAVES copies the fragments of sub-steps s = w, w + WAVES, ...
// Only the first rp_n row pairs are copied (the others hold no rows of the expert and are not read);
// `rows` of the chunk's rows are the expert's.
template <int WAVES>
__device__ inline void stage_step32(const KArgs& a, uint4* buf, int ks, int rin, int rows, int rp_n, int wave, int lane) {
  const uint4* in_units = reinterpret_cast<const uint4*>(a.in);
  const int n = lane & 31, h = lane >> 5;
#pragma unroll
  for (int s0 = 0; s0 < 8; s0 += WAVES) {
    const int s = s0 + wave;
#pragma unroll
    for (int p = 0; p < 2; ++p) {
      const int k8 = min(ks * 32 + (p + 2 * h) * 8 + s, a.K / 8 - 1);
#pragma unroll
      for (int rp = 0; rp < kRP; ++rp) {
        if (rp >= rp_n) continue;
        // (a row past the chunk's last one: one of the zero rows at the end of the buffer, see staged_row)
        const int R = 32 * rp + n < rows ? rin + 32 * rp + n : a.in_rt - dec::kZeroRows + (n & 15);
        __builtin_amdgcn_global_load_lds(
            reinterpret_cast<const __attribute__((address_space(1))) void*>(reinterpret_cast<uintptr_t>(in_units + act_unit(k8, R, a.in_rt))),
            reinterpret_cast<__attribute__((address_space(3))) void*>(reinterpret_cast<uintptr_t>(buf + ((rp * 8 + s) * 2 + p) * 64)), 16, 0, 0);
      }
    }
  }
}

// (in A) fragments of a rank step for the 32x32x16 products: V variants per rank step (4 fused, 2
// for W2).  Variant v, lane l (half h = l / 32) holds the 8 rank indices of group `grp` of
// projection m's (in A).  The fused projections meet different (in A): the A operand of variant v
// keeps W1's columns in input half h = v & 1 and W3's in the other, so the fragment holds A1's part
// where W1 sits and A3's where W3 sits.
__device__ inline void rank_frag_source(int v, int lane, bool dual, int& m, int& grp) {
  const int h = lane >> 5;
  if (dual) { m = h ^ (v & 1); grp = (v >> 1) + 2 * h; }
  else { m = 0; grp = v + 2 * h; }
}

// Codes and metadata of one k-step of a wavefront's two n-tiles.
template <int BITS, int NM, int NTW> struct Slot2 { Slot<BITS, NM> t[NTW]; };

// WAVES wavefronts per block.  8 (two per SIMD, 256 registers each) is what the launches use: with 4
// (one per SIMD with 512 registers and twice the n-tiles, so that a fragment read from LDS feeds
// twice the MFMAs) the fused kernel measured 19 % slower: nothing fills a wavefront's waits.
// Q3: some factor pair of the layer is held at 3 bits (layout.h): the rank steps of such a pair fetch
// the unit's code dword and the lane's half of the unit's metadata with loads of their own, one rank
// step ahead (the ring and the k-loop are those of the plain kernel), and dequantize them into the
// fp16 unit before it is used.
template <int BITS, bool DUAL, int NTW, int WAVES = kTileWaves, bool Q3 = false>
__global__ __launch_bounds__(64 * WAVES, WAVES == 4 ? 1 : 2) void qgemm_tile_kernel(KArgs a) {
  extern __shared__ uint4 xs[];           // two k-steps of activations; afterwards the (in A) fragments
  constexpr int NM = DUAL ? 2 : 1;
  constexpr int kNTW = NTW;                              // n-tiles per wavefront
  constexpr int DW = 2 * BITS;
  constexpr int NC = Extract<BITS>::kClasses;
  constexpr int LPS = BITS == 2 ? 2 : 3;                 // loads per tile and projection
  constexpr int kSlotOps = kNTW * NM * LPS;              // loads of one ring slot
  Chunk ch;
  if (!find_chunk(a, blockIdx.y, ch)) return;
  const int e = ch.e, r0 = ch.r0, cnt = ch.cnt, r = ch.r;
  const ExpertDesc& d = a.desc[e];
  const int th = threadIdx.x, lane = th & 63;
  const int wave = __builtin_amdgcn_readfirstlane(th >> 6);
  const int q = lane >> 4, c = lane & 15;
  const int tdw = kWave * DW;
  const int tile0 = (blockIdx.x * WAVES + wave) * kNTW;

  const int code_bytes = a.KS * a.NT * tdw * 4, meta_bytes = a.G * a.NT * kTileN * 4;
  const bool lowrank = a.rank > 0 && __builtin_amdgcn_readfirstlane(d.has_factors) != 0 && a.row_pair != nullptr &&
                       __builtin_amdgcn_readfirstlane(a.comp_rows[e]) > 0;
  // every projection has the rank of its own factor pair (Section 3.1): the expert runs the rank
  // steps of the larger one, a resource of the size its rank fills makes the other read zeros
  int LSm[NM];
  const int bf_bytes = a.NT * a.ls * 1024;
  __amdgpu_buffer_rsrc_t code_rs[NM], meta_rs[NM], bf_rs[NM];
  bool q3m[NM];
  float lam[NM];
#pragma unroll
  for (int m = 0; m < NM; ++m) {
    const int mat = DUAL ? m : 2;
    LSm[m] = lowrank ? (min(__builtin_amdgcn_readfirstlane(d.rank[mat]), a.rank) + 31) / 32 : 0;
    q3m[m] = Q3 && __builtin_amdgcn_readfirstlane((d.q3 >> mat) & 1) != 0;
    code_rs[m] = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint32_t*>(uniform_ptr(d.codes[mat])), 0, code_bytes, 0x00020000);
    meta_rs[m] = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint32_t*>(uniform_ptr(d.meta[mat])), 0, meta_bytes, 0x00020000);
    // (a 3-bit pair does not ride the ring: its rank steps read zeros here and fetch their units themselves)
    bf_rs[m] = __builtin_amdgcn_make_buffer_rsrc(const_cast<_Float16*>(uniform_ptr(d.bf[mat])), 0,
                                                 q3m[m] ? 0 : a.NT * LSm[m] * 1024, 0x00020000);
    lam[m] = __uint_as_float(__builtin_amdgcn_readfirstlane(__float_as_uint(d.inv_lambda[mat])));
  }
  const int LS = max(LSm[0], LSm[NM - 1]);
  const int gps = kTileK >> a.group_shift;               // groups per k-step
  const int meta_lane = ((q * kLaneK) >> a.group_shift) * (a.NT * kTileN * 4) + c * 4;

  // step < KS: the packed tiles of k-step `step`; KS <= step < KS + LS: the B-factor units of rank
  // step (step - KS); anything else (and an n-tile past the last) reads zeros past the resources
  auto fetch = [&](int step, Slot2<BITS, NM, kNTW>& sl) {
#pragma unroll
    for (int t = 0; t < kNTW; ++t) {
      const int tile = tile0 + t;
      const bool ok = step < a.KS && tile < a.NT;
      const bool lr = step >= a.KS && step < a.KS + LS && tile < a.NT;
      const int tile_off = (ok ? (step * a.NT + tile) * (tdw * 4) : lr ? ((step - a.KS) * a.NT + tile) * 1024 : max(code_bytes, bf_bytes)) + lane * 16;
      const int tile_off2 = (ok ? (step * a.NT + tile) * (tdw * 4) : code_bytes) + 1024 + lane * (BITS == 3 ? 8 : 16);
      const int meta_off = (ok ? (step * gps * a.NT + tile) * (kTileN * 4) : meta_bytes) + meta_lane;
#pragma unroll
      for (int m = 0; m < NM; ++m) {
        Slot<BITS, NM>& s1 = sl.t[t];
        const u32x4 v0 = __builtin_amdgcn_raw_buffer_load_b128(lr ? bf_rs[m] : code_rs[m], tile_off, 0, 0);
        s1.cw[m][0] = v0[0]; s1.cw[m][1] = v0[1]; s1.cw[m][2] = v0[2]; s1.cw[m][3] = v0[3];
        if constexpr (BITS == 3) {
          const u32x2 v1 = __builtin_amdgcn_raw_buffer_load_b64(code_rs[m], tile_off2, 0, 0);
          s1.cw[m][4] = v1[0]; s1.cw[m][5] = v1[1];
        } else if constexpr (BITS == 4) {
          const u32x4 v1 = __builtin_amdgcn_raw_buffer_load_b128(code_rs[m], tile_off2, 0, 0);
          s1.cw[m][4] = v1[0]; s1.cw[m][5] = v1[1]; s1.cw[m][6] = v1[2]; s1.cw[m][7] = v1[3];
        }
        s1.mw[m] = __builtin_amdgcn_raw_buffer_load_b32(meta_rs[m], meta_off, 0, 0);
      }
    }
  };

  // first input row of this chunk (shared experts all read the token rows 0..T-1)
  const int rin = ((DUAL && !a.offsets) ? 0 : r0) + r;

  // Streams (16 output columns that meet the same activations) are paired into the 32 rows of an A
  // operand: (W1, W3) of n-tile j in the fused kernel, n-tiles 2j and 2j + 1 otherwise.
  constexpr int NPAIR = kNTW * NM / 2;
  // acc[j][rp]: the 32 x 32 result of pair j and row pair rp; register i of lane l holds, of row
  // 32 rp + l % 32, stream i / 8, column 8 ((i / 4) % 2) + 4 (l / 32) + i % 4 of the stream's n-tile
  float16_t acc[NPAIR][kRP];
#pragma unroll
  for (int j = 0; j < NPAIR; ++j)
#pragma unroll
    for (int rp = 0; rp < kRP; ++rp)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[j][rp][i] = 0.f;
  const int rp_n = min(kRP, (cnt - r + 31) >> 5);         // row pairs that hold rows of this expert

  // the two streams of pair j: (tile slot, projection)
  auto pair_stream = [](int j, int side, int& t, int& m) {
    if constexpr (DUAL) { t = j; m = side; }
    else { t = 2 * j + side; m = 0; }
  };

  // One k-step for a chunk with RPN row pairs that hold rows.  A sub-step (32 inputs per lane
  // group) has F = 2 RPN fragments of activations, operand p major; fragment g of the k-step's
  // 8 F is read from LDS kPF fragments ahead of its two MFMAs (one per pair), and the weights of
  // the next sub-step are unpacked, a piece per fragment, behind the MFMAs of the current one, so
  // that the matrix pipe, the LDS reads and the unpacking run side by side within a wavefront.
  constexpr int kPF = kTileLdsAhead;
  auto compute = [&](auto RPN_, const Slot2<BITS, NM, kNTW>& cur, const uint4* buf) {
    constexpr int RPN = decltype(RPN_)::value;
    constexpr int F = 2 * RPN, G = 8 * F;
    uint32_t s2[kNTW][NM][NC], c2[kNTW][NM];
#pragma unroll
    for (int t = 0; t < kNTW; ++t)
#pragma unroll
      for (int m = 0; m < NM; ++m) {
        const uint32_t mw = cur.t[t].mw[m];
        s2[t][m][0] = (mw & 0xffffu) | (mw << 16);
        c2[t][m] = (mw >> 16) | (mw & 0xffff0000u);
        constexpr uint32_t step = Extract<BITS>::kStepBits == 2 ? 0x44004400u : 0x48004800u;   // 4.0 or 8.0
#pragma unroll
        for (int p = 1; p < NC; ++p) s2[t][m][p] = pk_mul(s2[t][m][p - 1], step);
      }
    const uint32_t base = uint32_t(reinterpret_cast<uintptr_t>(buf + lane));
    // LDS byte offset of fragment g: sub-step g / F, operand (g % F) / RPN, row pair (g % F) % RPN
    auto frag_off = [](int g) constexpr { return (g / F) * 2048 + ((g % F) % RPN) * 16384 + ((g % F) / RPN) * 1024; };
    half8_t xf[kPF + 1];
    static_for<(kPF < G ? kPF : G)>([&](auto g) { xf[g] = lds_read16<frag_off(g)>(base); });
    // piece (j, i) of a sub-step: operand register i of the two streams of pair j, before the swap
    uint32_t v[NPAIR][2][4];
    auto unpack_piece = [&](int s, int piece) {
      const int j = piece / 4, i = piece % 4;
#pragma unroll
      for (int side = 0; side < 2; ++side) {
        int t, m;
        pair_stream(j, side, t, m);
        v[j][side][i] = pk_fma(Extract<BITS>::field(cur.t[t].cw[m], 4 * s + i), s2[t][m][Extract<BITS>::cls(4 * s + i)], c2[t][m]);
      }
    };
    constexpr int PIECES = NPAIR * 4;
    static_for<PIECES>([&](auto pc) { unpack_piece(0, pc); });
    static_for<8>([&](auto S) {
      constexpr int s = decltype(S)::value;
      // rows of 16 lanes swapped between the two streams of a pair: operand 0 = lane groups q = 0, 2
      // of both streams side by side, operand 1 = q = 1, 3
      uint32_t A[2][NPAIR][4];
#pragma unroll
      for (int j = 0; j < NPAIR; ++j)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const auto sw = __builtin_amdgcn_permlane16_swap(v[j][0][i], v[j][1][i], false, false);
          A[0][j][i] = sw[0]; A[1][j][i] = sw[1];
        }
      __builtin_amdgcn_sched_barrier(0);
      static_for<F>([&](auto Fi) {
        constexpr int f = decltype(Fi)::value, g = s * F + f, p = f / RPN, rp = f % RPN;
        if constexpr (g + kPF < G) xf[(g + kPF) % (kPF + 1)] = lds_read16<frag_off(g + kPF)>(base);
        lds_wait<(G - 1 - g < kPF ? G - 1 - g : kPF)>(xf[g % (kPF + 1)]);
#pragma unroll
        for (int j = 0; j < NPAIR; ++j) {
          const half8_t av = __builtin_bit_cast(half8_t, make_uint4(A[p][j][0], A[p][j][1], A[p][j][2], A[p][j][3]));
          acc[j][rp] = __builtin_amdgcn_mfma_f32_32x32x16_f16(av, xf[g % (kPF + 1)], acc[j][rp], 0, 0, 0);
        }
        if constexpr (s < 7) {
#pragma unroll
          for (int pc = PIECES * f / F; pc < PIECES * (f + 1) / F; ++pc) unpack_piece(s + 1, pc);
        }
        __builtin_amdgcn_sched_barrier(0);
      });
    });
  };

  // ---- prologue: the first k-step of activations and the first two ring slots
  Slot2<BITS, NM, kNTW> ring[2];
  stage_step32<WAVES>(a, xs, 0, rin, cnt - r, rp_n, wave, lane);
  __builtin_amdgcn_sched_barrier(0);
  fetch(0, ring[0]);
  fetch(1, ring[1]);
  // only the packed tiles are still in flight when the barrier is passed (written out: a
  // __syncthreads() would first wait for every load in flight)
  asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(2 * kSlotOps) : "memory");

  // ---- the k-steps, two per trip so that the ring slots are indexed statically.  In a step: the
  //      copy of the next step's activations is issued into the other half of LDS (free since the
  //      barrier that ended the previous step), the current step is multiplied, its slot refilled;
  //      then only that refill may still be in flight (the copy has landed) and the barrier ends
  //      the step.  One copy of the loop per number of row pairs, so that every count is static.
  const int steps = a.KS;
  auto k_loop = [&](auto RPN_) {
    for (int s0 = 0; s0 < steps; s0 += 2) {
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const int step = s0 + i;
        if (step < steps) {
          stage_step32<WAVES>(a, xs + ((step + 1) & 1) * kStepUnits, step + 1, rin, cnt - r, decltype(RPN_)::value, wave, lane);
          __builtin_amdgcn_sched_barrier(0);     // (the wait below counts the refill as the only later loads)
          compute(RPN_, ring[i], xs + (step & 1) * kStepUnits);
          fetch(step + 2, ring[i]);
          asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(kSlotOps) : "memory");
        }
      }
    }
  };
  if (rp_n == 4) k_loop(std::integral_constant<int, 4>{});
  else if (rp_n == 3) k_loop(std::integral_constant<int, 3>{});
  else if (rp_n == 2) k_loop(std::integral_constant<int, 2>{});
  else k_loop(std::integral_constant<int, 1>{});

  // ---- rank steps.  (in A) of the chunk's rows, fp16 row-major in global memory (xa_tile_kernel
  //      has scaled it and zeroed the rows without the term), is copied into LDS as fragments of 32
  //      rows, kRankChunk rank steps at a time (all of them for ranks up to 256): fragment (rank step
  //      st, variant v, row pair rp) at unit (((st - c0) * V + v) * 4 + rp) * 64 (rank_frag_source).
  constexpr int V = DUAL ? 4 : 2;
  constexpr int kRankChunk = 2 * kStepUnits / (V * kRP * 64);       // 8 (fused) or 16 rank steps fill the 128 KB
  // 3-bit pairs: the code dword and the lane's half of the metadata (layout.h) of every stream's unit
  // of one rank step; zeros for fp16 pairs, past the stream's own rank and past the last n-tile
  struct QUnits { uint32_t codes[kNTW][NM]; uint32_t meta[kNTW][NM][4]; };
  auto q_load = [&](int st, QUnits& qu) {
#pragma unroll
    for (int t = 0; t < kNTW; ++t)
#pragma unroll
      for (int m = 0; m < NM; ++m) {
        qu.codes[t][m] = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i) qu.meta[t][m][i] = 0;
        if constexpr (Q3) {
          const int tile = tile0 + t;
          if (q3m[m] && st < LSm[m] && tile < a.NT) {
            const int mat = DUAL ? m : 2;
            qu.codes[t][m] = uniform_ptr(d.bfc[mat])[(size_t(st) * a.NT + tile) * kWave + lane];
            const uint4 v = *reinterpret_cast<const uint4*>(reinterpret_cast<const uint8_t*>(uniform_ptr(d.bf[mat])) +
                                                            ((size_t(st) * (a.NT / 4) + (tile >> 2)) * 4 + q) * 32 + (c & 1) * 16);
            qu.meta[t][m][0] = v.x; qu.meta[t][m][1] = v.y; qu.meta[t][m][2] = v.z; qu.meta[t][m][3] = v.w;
          }
        }
      }
  };
  QUnits qnext;
  for (int c0 = 0; c0 < LS; c0 += kRankChunk) {
    const int c1 = min(LS, c0 + kRankChunk);
    q_load(c0, qnext);                       // (arrives with the copies below)
    asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");   // (everyone is done with what LDS held)
    const _Float16* P = reinterpret_cast<const _Float16*>(a.p);
    const int pitch = NM * a.ls * 32;                                // halves per row
    for (int f = wave; f < (c1 - c0) * V * kRP; f += WAVES) {
      const int rp = f % kRP, g = f / kRP, v = g % V, sl = g / V;
      int m, grp;
      rank_frag_source(v, lane, DUAL, m, grp);
      const int row = min(r0 + r + 32 * rp + (lane & 31), a.total_rows - 1);
      const _Float16* src = P + size_t(row) * pitch + m * a.ls * 32 + 32 * (c0 + sl) + 8 * grp;
      __builtin_amdgcn_global_load_lds(
          reinterpret_cast<const __attribute__((address_space(1))) void*>(reinterpret_cast<uintptr_t>(src)),
          reinterpret_cast<__attribute__((address_space(3))) void*>(reinterpret_cast<uintptr_t>(xs + ((size_t(sl) * V + v) * kRP + rp) * 64)), 16, 0, 0);
    }
    // (the ring slots are refilled below, after this wait: only the copies just issued and the two
    // slots requested before them are outstanding)
    asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");
    // the fp16 B-factor unit of stream (t, m) of a rank step: from the slot, or rebuilt from a 3-bit unit
    auto b_unit = [&](const Slot2<BITS, NM, kNTW>& cur, const QUnits& qu, int t, int m, uint32_t (&u)[4]) {
#pragma unroll
      for (int i = 0; i < 4; ++i) u[i] = cur.t[t].cw[m][i];
      if constexpr (Q3) {
        if (q3m[m]) {
          const uint32_t own[4] = {qu.meta[t][m][0], qu.meta[t][m][1], qu.meta[t][m][2], qu.meta[t][m][3]};
          const uint4 v = __builtin_bit_cast(uint4, q3_unit_b(qu.codes[t][m], own, (c & 1) != 0));
          u[0] = v.x; u[1] = v.y; u[2] = v.z; u[3] = v.w;
        }
      }
    };
    auto rank_step = [&](const Slot2<BITS, NM, kNTW>& cur, const QUnits& qu, int st) {
#pragma unroll
      for (int j = 0; j < NPAIR; ++j) {
        // the B-factor units of the pair's two streams, 16-lane rows swapped: r0 = rank groups 0 and 2
        // of both streams side by side, r1 = groups 1 and 3 (a stream past its own rank holds zeros)
        int t0s, m0s, t1s, m1s;
        pair_stream(j, 0, t0s, m0s);
        pair_stream(j, 1, t1s, m1s);
        uint32_t u0[4], u1[4], r0v[4], r1v[4];
        b_unit(cur, qu, t0s, m0s, u0);
        b_unit(cur, qu, t1s, m1s, u1);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const auto sw = __builtin_amdgcn_permlane16_swap(u0[i], u1[i], false, false);
          r0v[i] = sw[0]; r1v[i] = sw[1];
        }
#pragma unroll
        for (int v = 0; v < V; ++v) {
          uint32_t av[4];
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            if constexpr (DUAL) {
              // W1 and W3 meet different (in A): W1's columns keep one half of the inputs, W3's the
              // other (lane rows 0, 3 or 1, 2), zero elsewhere
              const bool keep = (v & 1) ? (q == 1 || q == 2) : (q == 0 || q == 3);
              av[i] = keep ? (v < 2 ? r0v[i] : r1v[i]) : 0u;
            } else {
              av[i] = v == 0 ? r0v[i] : r1v[i];
            }
          }
          const half8_t avh = __builtin_bit_cast(half8_t, make_uint4(av[0], av[1], av[2], av[3]));
#pragma unroll
          for (int rp = 0; rp < kRP; ++rp)
            if (rp < rp_n) {
              const half8_t pf = __builtin_bit_cast(half8_t, xs[((size_t(st - c0) * V + v) * kRP + rp) * 64 + lane]);
              acc[j][rp] = __builtin_amdgcn_mfma_f32_32x32x16_f16(avh, pf, acc[j][rp], 0, 0, 0);
            }
        }
      }
    };
    // the slot of step KS + st is ring[(KS + st) % 2]: walk the chunk's steps in aligned pairs
    for (int s0 = (steps + c0) & ~1; s0 < steps + c1; s0 += 2) {
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const int step = s0 + i;
        if (step >= steps + c0 && step < steps + c1) {
          const QUnits qcur = qnext;
          q_load(step - steps + 1 < c1 ? step - steps + 1 : LS, qnext);   // (LS: nothing to fetch)
          rank_step(ring[i], qcur, step - steps);
          fetch(step + 2, ring[i]);
        }
      }
    }
  }

  // ---- epilogue: lane l holds, of row 32 rp + l % 32, columns 8 g + 4 (l / 32) .. + 3 (g = 0, 1) of
  //      both streams of every pair ----
  const int hh = lane >> 5;
#pragma unroll
  for (int j = 0; j < NPAIR; ++j)
#pragma unroll
    for (int rp = 0; rp < kRP; ++rp) {
      const int row = r + 32 * rp + (lane & 31);
      if (rp >= rp_n || row >= cnt) continue;
      const int se = a.row_exp[(a.offsets ? r0 : 0) + row];        // the row's inputs were scaled by 2^se
      const float dn = pow2i(DUAL ? -se : -2 * se), up = pow2i(2 * se);
#pragma unroll
      for (int g = 0; g < 2; ++g) {
        const int col4 = 8 * g + 4 * hh;
        if constexpr (DUAL) {
          const int tile = tile0 + j;
          if (tile >= a.NT) continue;
          half4_t hv;
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const float gg = acc[j][rp][4 * g + i] * (lam[0] * dn), uu = acc[j][rp][8 + 4 * g + i] * (lam[NM - 1] * dn);
            hv[i] = to_f16_sat(gg * __builtin_amdgcn_rcpf(1.0f + __expf(-gg)) * uu * up);
          }
          // h in operand order for the W2 kernel: columns f .. f+3 are half of one 16-byte unit
          const int f = tile * kTileN + col4;
          *reinterpret_cast<half4_t*>(reinterpret_cast<_Float16*>(a.out) + act_unit(f >> 3, r0 + row, a.out_rt) * 8 + (f & 7)) = hv;
        } else {
#pragma unroll
          for (int side = 0; side < 2; ++side) {
            const int tile = tile0 + 2 * j + side;
            if (tile >= a.NT) continue;
            const size_t o = size_t(r0 + row) * a.N + tile * kTileN + col4;
            uint2 yv;
            const float l2 = lam[0] * dn;
            yv.x = f32x2_to_bf16x2(acc[j][rp][8 * side + 4 * g] * l2, acc[j][rp][8 * side + 4 * g + 1] * l2);
            yv.y = f32x2_to_bf16x2(acc[j][rp][8 * side + 4 * g + 2] * l2, acc[j][rp][8 * side + 4 * g + 3] * l2);
            *reinterpret_cast<uint2*>(reinterpret_cast<uint16_t*>(a.out) + o) = yv;
          }
        }
      }
    }
}

// (in A)[row][rho] for the 128-row chunks of every expert, in two launches.
// xa_tile_kernel: K-block partial sums in fp32, [K-block][row][NM * ls * 32 columns] ([A1 | A3] in
// the fused case, each padded to a multiple of 32), already multiplied by the projection's
// power-of-two pre-scale.  Same shape as the kernel above (activations through double-buffered LDS,
// eight row tiles per fragment of weights), with the fp16 factor tiles [rpad/16][K/32][lane][8] as
// the weight operand: wavefront w owns the 16-column factor tiles w, w + 8, ... (at most four);
// grid.x splits K so that the launch fills the chip.
// xa_finish_kernel: adds the K-blocks in order, zeroes the rows without the rank-r term and the
// padding columns, writes fp16 row-major.
// Only the rows that take the term are computed: the chunks run over the compact rows the preparing
// launch has made of them (CompactArgs: the front of every expert's row range), the partial sums
// are indexed by compact row, and the finish kernel puts every routed row's sum (or zeros) in its
// place.
// Q3: some factor pair of the layer is held at 3 bits (layout.h); such a pair's units are fetched as
// (codes, metadata) dwords and dequantized when their k-step comes up.
template <bool DUAL, int NT, bool Q3>
__global__ __launch_bounds__(64 * kTileWaves, 2) void xa_tile_kernel(KArgs a) {
  extern __shared__ uint4 xs[];
  constexpr int NM = DUAL ? 2 : 1;
  constexpr int kMaxT = NT;                              // factor tiles per wavefront (2 or 4); grid.z: groups of 8 * NT tiles
  constexpr bool kAhead = NT <= 2;                       // registers for the factor units of a whole k-step ahead
  Chunk ch;
  if (!find_chunk(a, blockIdx.y, ch)) return;
  const int e = ch.e, r0 = ch.r0, cnt = ch.cnt, r = ch.r;
  const ExpertDesc& d = a.desc[e];
  if (!d.has_factors || a.comp_rows[e] == 0) return;
  const int th = threadIdx.x, lane = th & 63;
  const int wave = __builtin_amdgcn_readfirstlane(th >> 6);
  const int q = lane >> 4, c = lane & 15;
  const int mt_n = min(kTMT, (cnt - r + 15) >> 4);
  const int rt = a.rpad / 16, tiles = NM * rt;           // 16-column factor tiles in all
  const int pitch = NM * a.ls * 32;
  // The chunk's rows are compact rows (the rows of the expert that take the rank-r term, in row
  // order): row_list names the routed row whose activations each one reads.  A row past the
  // expert's last compact row reads one of the zero rows at the end of the buffer (its results are
  // never stored).
  int Rm[kTMT];
#pragma unroll
  for (int mt = 0; mt < kTMT; ++mt) {
    const int i = r0 + min(r + 16 * mt + c, cnt - 1);
    Rm[mt] = r + 16 * mt + c < cnt ? (a.row_list ? a.row_list[i] : i) : a.in_rt - dec::kZeroRows + c;
  }

  float4_t acc[kMaxT][kTMT];
#pragma unroll
  for (int t = 0; t < kMaxT; ++t)
#pragma unroll
    for (int mt = 0; mt < kTMT; ++mt) acc[t][mt] = float4_t{0.f, 0.f, 0.f, 0.f};
  // A fragment of activations (k-step ks, sub-step s) holds, in lane (q, row), the columns
  // 256 ks + 64 q + 8 s + j: the factor unit that meets it is the one with those K rows, unit
  // (8 ks + 2 q + s / 4, tile) of the packed factor, lane (s % 4, c) of it.
  const half8_t* af[kMaxT];
  const uint32_t* am[kMaxT];                 // 3-bit pairs: the tile's metadata, [group of 64 inputs][16 columns]
  bool q3t[kMaxT], valid[kMaxT];             // (a tile past the projection's own rank holds nothing: its columns stay zero)
  int nmine = 0;
#pragma unroll
  for (int t = 0; t < kMaxT; ++t) {
    const int tile = blockIdx.z * (kTileWaves * kMaxT) + wave + t * kTileWaves;
    af[t] = nullptr; am[t] = nullptr; q3t[t] = false; valid[t] = false;
    if (tile < tiles) {
      const int m = tile / rt, tl = tile - m * rt, mat = DUAL ? m : 2;
      valid[t] = 16 * tl < __builtin_amdgcn_readfirstlane(d.rank[mat]);
      q3t[t] = Q3 && __builtin_amdgcn_readfirstlane((d.q3 >> mat) & 1) != 0;
      if (q3t[t]) {
        af[t] = reinterpret_cast<const half8_t*>(reinterpret_cast<const uint32_t*>(uniform_ptr(d.af[mat])) + size_t(tl) * (a.K / 32) * kWave + c);
        am[t] = uniform_ptr(d.afm[mat]) + size_t(tl) * (a.K / 64) * 16 + c;
      } else {
        af[t] = reinterpret_cast<const half8_t*>(uniform_ptr(d.af[mat])) + size_t(tl) * (a.K / 32) * kWave + c;
      }
      nmine = t + 1;
    }
  }

  const int all_steps = (a.K + kTileK - 1) / kTileK, per_kb = (all_steps + gridDim.x - 1) / gridDim.x;
  const int step_lo = blockIdx.x * per_kb, steps = min(all_steps, step_lo + per_kb);
  if (step_lo >= steps) return;              // (the finish kernel reads only K-blocks that exist)
  // the factor units of sub-step s of k-step `step` for this lane (zero past K)
  auto load_unit = [&](int step, int s, int t) {
    const int kk = step * 8 + 2 * q + (s >> 2);          // this lane's 32-row unit of the factor
    u32x4 v = u32x4{0, 0, 0, 0};
    if (valid[t] && kk * 32 < a.K) {
      if (Q3 && q3t[t]) {
        v[0] = reinterpret_cast<const uint32_t*>(af[t])[size_t(kk) * kWave + (s & 3) * 16];
      } else {
        v = __builtin_bit_cast(u32x4, af[t][size_t(kk) * kWave + (s & 3) * 16]);
      }
    }
    return v;
  };
  // 3-bit pairs: a lane's eight units of a k-step lie in one group of 64 inputs (rows 256 step + 64 q ..):
  // one dword of metadata per k-step and tile
  auto load_meta = [&](int step, int t) {
    uint32_t mv = 0;
    if (Q3 && q3t[t] && valid[t] && (step * 4 + q) * 64 < a.K) mv = am[t][(step * 4 + q) * 16];
    return mv;
  };
  // the operand of a fetched unit (a unit that was not fetched is all zeros in either format)
  auto operand = [&](const u32x4& v, uint32_t mv, int t) {
    if (Q3 && q3t[t]) return q3_unit_a(v[0], mv);
    return __builtin_bit_cast(half8_t, v);
  };
  u32x4 wnext[kAhead ? 8 : 1][kMaxT];
  uint32_t mnext[kMaxT];
#pragma unroll
  for (int t = 0; t < kMaxT; ++t) mnext[t] = load_meta(step_lo, t);
  if constexpr (kAhead) {
#pragma unroll
    for (int s = 0; s < 8; ++s)
#pragma unroll
      for (int t = 0; t < kMaxT; ++t) wnext[s][t] = load_unit(step_lo, s, t);
  }
  stage_step_rows(a, xs + (step_lo & 1) * kStepUnits, step_lo, Rm, mt_n, wave, lane);
  asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");
  for (int step = step_lo; step < steps; ++step) {
    stage_step_rows(a, xs + ((step + 1) & 1) * kStepUnits, step + 1, Rm, mt_n, wave, lane);
    const uint4* buf = xs + (step & 1) * kStepUnits;
    half8_t wcur[kAhead ? 8 : 1][kMaxT];
    uint32_t mcur[kMaxT];
#pragma unroll
    for (int t = 0; t < kMaxT; ++t) { mcur[t] = mnext[t]; mnext[t] = load_meta(step + 1, t); }
    if constexpr (kAhead) {                  // this step's units have arrived; ask for the next step's
#pragma unroll
      for (int s = 0; s < 8; ++s)
#pragma unroll
        for (int t = 0; t < kMaxT; ++t) wcur[s][t] = operand(wnext[s][t], mcur[t], t);
#pragma unroll
      for (int s = 0; s < 8; ++s)
#pragma unroll
        for (int t = 0; t < kMaxT; ++t) wnext[s][t] = load_unit(step + 1, s, t);
    }
#pragma unroll
    for (int s = 0; s < 8; ++s) {
      half8_t wf[kMaxT];
#pragma unroll
      for (int t = 0; t < kMaxT; ++t) {
        if constexpr (kAhead) wf[t] = wcur[s][t];
        else wf[t] = operand(load_unit(step, s, t), mcur[t], t);
      }
#pragma unroll
      for (int mt = 0; mt < kTMT; ++mt)
        if (mt < mt_n) {
          const half8_t xf = __builtin_bit_cast(half8_t, buf[(mt * 8 + s) * 64 + lane]);
#pragma unroll
          for (int t = 0; t < kMaxT; ++t)
            if (t < nmine) acc[t][mt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(wf[t], xf, acc[t][mt], 0, 0, 0);
        }
    }
    // the copy of the next step has landed; everyone is done with this step's half of LDS
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
  }

  // lane holds columns 16*tile + 4*q .. +3 of row 16 mt + c
  float* part = a.partial + size_t(blockIdx.x) * a.total_rows * pitch;
#pragma unroll
  for (int t = 0; t < kMaxT; ++t) {
    const int tile = blockIdx.z * (kTileWaves * kMaxT) + wave + t * kTileWaves;
    if (tile >= tiles) continue;
    const int m = tile / rt, tl = tile - m * rt;
    const float lam = d.xa_scale[DUAL ? m : 2];
#pragma unroll
    for (int mt = 0; mt < kTMT; ++mt) {
      const int row = r + 16 * mt + c;
      if (mt >= mt_n || row >= cnt) continue;
      *reinterpret_cast<float4_t*>(part + size_t(r0 + row) * pitch + m * a.ls * 32 + 16 * tl + 4 * q) = acc[t][mt] * lam;
    }
  }
}

// P[row][col] = fp16(sum over K-blocks of part[kb][row][col]) for rows that take the rank-r term and
// columns below the rank rounded up to 16; zero elsewhere.  One thread per four columns.
__global__ __launch_bounds__(256) void xa_finish_kernel(const float* __restrict__ part, int kblocks, int rows, int pitch,
                                                        int ls32, int rpad, const int32_t* __restrict__ comp_index,
                                                        int comp_rows, _Float16* __restrict__ P) {
  const size_t i = size_t(blockIdx.x) * 256 + threadIdx.x;       // index of a group of four columns
  const int per_row = pitch / 4;
  if (i >= size_t(rows) * per_row) return;
  const int row = int(i / per_row), col = int(i - size_t(row) * per_row) * 4;
  half4_t v = half4_t{0, 0, 0, 0};
  const int ci = comp_index[row];                                // the row's place among the rows with the term (-1: none)
  if (ci >= 0 && (col % ls32) < rpad) {
    float4_t sum = *reinterpret_cast<const float4_t*>(part + size_t(ci) * pitch + col);
    for (int kb = 1; kb < kblocks; ++kb)
      sum += *reinterpret_cast<const float4_t*>(part + (size_t(kb) * comp_rows + ci) * pitch + col);
    v = half4_t{(_Float16)sum[0], (_Float16)sum[1], (_Float16)sum[2], (_Float16)sum[3]};
  }
  *reinterpret_cast<half4_t*>(P + size_t(row) * pitch + col) = v;
}

template <int BITS>
hipError_t launch_bits(const FfnArgs& f, hipStream_t s, int which) {
  int gs = 0;
  while ((1 << gs) < f.group) ++gs;
  KArgs a{};
  a.desc = f.desc; a.offsets = f.offsets; a.row_pair = f.row_pair; a.comp_rows = f.comp_rows; a.n_exp = f.n_exp;
  a.row_exp = f.row_exp; a.tok_exp = f.tok_exp;
  a.group_shift = gs; a.top_k = f.top_k; a.top_n = f.top_n; a.T = f.T;
  a.rank = f.rank; a.rpad = f.rpad; a.ls = (f.rank + 31) / 32; a.total_rows = f.total_rows;
  const bool comp = f.rank > 0 && f.top_n > 0 && f.row_pair != nullptr;
  // 128-row chunks: at most one partly filled chunk per expert
  const int items = f.offsets ? f.total_rows / kBM + f.n_exp : f.n_exp * ((f.T + kBM - 1) / kBM);
  const size_t lds = size_t(2) * kStepUnits * 16;

  // (in A): fp16 result at the start of the buffer, the K-block partial sums behind it
  auto xa = [&](auto k2, auto k4, float* buf, int nm, int ksplit) {
    const int per_wave = (nm * f.rpad / 16 + kTileWaves - 1) / kTileWaves;   // factor tiles per wavefront
    const int pitch = nm * a.ls * 32, steps = (a.K + kTileK - 1) / kTileK;
    const int per_kb = (steps + std::max(1, ksplit) - 1) / std::max(1, ksplit);
    const int kblocks = (steps + per_kb - 1) / per_kb;      // no K-block without a k-step
    a.p = buf;
    // the kernel's rows are the compact rows of the pairs that take the term (T * top_n in all), at
    // the front of every expert's row range
    KArgs ax = a;
    ax.row_list = f.cmp_list;
    ax.partial = buf + (size_t(f.total_rows) * pitch / 2 + 63) / 64 * 64;
    const int xitems = f.T * f.top_n / kBM + f.n_exp;
    // (more than 32 factor tiles, i.e. ranks above 256: further groups of 32 tiles in grid.z)
    if (per_wave <= 2) hipLaunchKernelGGL(k2, dim3(kblocks, xitems), dim3(64 * kTileWaves), lds, s, ax);
    else hipLaunchKernelGGL(k4, dim3(kblocks, xitems, (per_wave + 3) / 4), dim3(64 * kTileWaves), lds, s, ax);
    const size_t groups = size_t(f.total_rows) * pitch / 4;
    hipLaunchKernelGGL(xa_finish_kernel, dim3((unsigned)((groups + 255) / 256)), dim3(256), 0, s, ax.partial, kblocks,
                       f.total_rows, pitch, a.ls * 32, a.rpad, f.cmp_index, f.total_rows, reinterpret_cast<_Float16*>(buf));
  };
  if (which & 1) {
  // W1 | W3 with the SwiGLU epilogue
  a.in = f.xh; a.out = f.h; a.K = f.H; a.N = f.F; a.NT = f.F / kTileN;
  a.in_rt = f.x_rt; a.out_rt = f.h_rt;
  a.KS = padded_k(f.H) / kTileK; a.G = padded_k(f.H) / f.group;
  if (comp && f.q3) xa(xa_tile_kernel<true, 2, true>, xa_tile_kernel<true, 4, true>, f.p13, 2, f.ksplit13);
  else if (comp) xa(xa_tile_kernel<true, 2, false>, xa_tile_kernel<true, 4, false>, f.p13, 2, f.ksplit13);
  if (f.marks) (void)hipEventRecord(f.marks[0], s);
  if (comp && f.q3) hipLaunchKernelGGL((qgemm_tile_kernel<BITS, true, 2, kTileWaves, true>), dim3((a.NT + 15) / 16, items), dim3(64 * kTileWaves), lds, s, a);
  else hipLaunchKernelGGL((qgemm_tile_kernel<BITS, true, 2>), dim3((a.NT + 15) / 16, items), dim3(64 * kTileWaves), lds, s, a);
  if (f.marks) (void)hipEventRecord(f.marks[1], s);
  }
  if (which & 2) {
  // W2
  a.in = f.h; a.out = f.y_rows; a.K = f.F; a.N = f.H; a.NT = f.H / kTileN;
  a.in_rt = f.h_rt; a.out_rt = 0;
  a.KS = padded_k(f.F) / kTileK; a.G = padded_k(f.F) / f.group;
  if (comp && f.q3) xa(xa_tile_kernel<false, 2, true>, xa_tile_kernel<false, 4, true>, f.p2, 1, f.ksplit2);
  else if (comp) xa(xa_tile_kernel<false, 2, false>, xa_tile_kernel<false, 4, false>, f.p2, 1, f.ksplit2);
  if (f.marks) (void)hipEventRecord(f.marks[2], s);
  // four n-tiles per wavefront use a fragment of activations twice as often as two, but make
  // blocks twice as large: take the one with fewer (weighted) rounds of blocks over the 256 CUs
  // (expected number of chunks: about half of the experts end with a partly filled one)
  const int chunks = std::max(1, f.offsets ? f.total_rows / kBM + (f.n_exp + 1) / 2 : f.n_exp * ((f.T + kBM - 1) / kBM));
  auto rounds = [&](int ntw) { return (chunks * ((a.NT + 8 * ntw - 1) / (8 * ntw)) + f.n_cu - 1) / f.n_cu * ntw; };
  const bool q3 = comp && f.q3;
  if (rounds(4) * 100 <= rounds(2) * 108) {
    if (q3) hipLaunchKernelGGL((qgemm_tile_kernel<BITS, false, 4, kTileWaves, true>), dim3((a.NT + 31) / 32, items), dim3(64 * kTileWaves), lds, s, a);
    else hipLaunchKernelGGL((qgemm_tile_kernel<BITS, false, 4>), dim3((a.NT + 31) / 32, items), dim3(64 * kTileWaves), lds, s, a);
  } else {
    if (q3) hipLaunchKernelGGL((qgemm_tile_kernel<BITS, false, 2, kTileWaves, true>), dim3((a.NT + 15) / 16, items), dim3(64 * kTileWaves), lds, s, a);
    else hipLaunchKernelGGL((qgemm_tile_kernel<BITS, false, 2>), dim3((a.NT + 15) / 16, items), dim3(64 * kTileWaves), lds, s, a);
  }
  if (f.marks) (void)hipEventRecord(f.marks[3], s);
  }
  return hipGetLastError();
}

}  // namespace

// Which flavour a projection takes (measured on Mixtral, DeepSeek and Qwen3 shapes): the decode
// flavour up to 24 rows per expert; beyond that the grouped GEMM as soon as it is efficient: the
// fused W1|W3 from about 40 rows per expert on, W2 (whose grid has few column blocks) once its grid
// of (128-row chunk, 256 columns) blocks covers the 256 CUs.
constexpr int kDecodeMaxRows13 = 40;

// bit 0: W1|W3 takes the decode flavour, bit 1: W2 does
static int decode_parts(const FfnArgs& f) {
  // expected rows per expert under uniform routing decides the flavour of each projection
  const int rows = f.offsets ? (f.T * f.top_k + f.n_exp - 1) / f.n_exp : f.T;
  const int chunks = f.offsets ? f.total_rows / kBM + (f.n_exp + 1) / 2 : f.n_exp * ((f.T + kBM - 1) / kBM);
  const bool w2_grid_full = chunks * ((f.H / kTileN + 15) / 16) >= f.n_cu;
  const bool d13 = rows <= kDecodeMaxRows13;
  // (beyond 128 rows per expert the decode flavour would stream the weights five times or more)
  const bool d2 = rows <= 24 || (!w2_grid_full && rows <= 128);
  return (d13 ? 1 : 0) | (d2 ? 2 : 0);
}

template <int BITS> static hipError_t tile_init_bits() {
  const void* fns[6] = {reinterpret_cast<const void*>(&qgemm_tile_kernel<BITS, true, 2>),
                        reinterpret_cast<const void*>(&qgemm_tile_kernel<BITS, false, 4>),
                        reinterpret_cast<const void*>(&qgemm_tile_kernel<BITS, false, 2>),
                        reinterpret_cast<const void*>(&qgemm_tile_kernel<BITS, true, 2, kTileWaves, true>),
                        reinterpret_cast<const void*>(&qgemm_tile_kernel<BITS, false, 4, kTileWaves, true>),
                        reinterpret_cast<const void*>(&qgemm_tile_kernel<BITS, false, 2, kTileWaves, true>)};
  for (const void* fn : fns) {
    hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, 2 * kStepUnits * 16);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

hipError_t ffn_init_device() {
  const void* fns[8] = {reinterpret_cast<const void*>(&xa_tile_kernel<true, 2, false>), reinterpret_cast<const void*>(&xa_tile_kernel<false, 2, false>),
                        reinterpret_cast<const void*>(&xa_tile_kernel<true, 4, false>), reinterpret_cast<const void*>(&xa_tile_kernel<false, 4, false>),
                        reinterpret_cast<const void*>(&xa_tile_kernel<true, 2, true>), reinterpret_cast<const void*>(&xa_tile_kernel<false, 2, true>),
                        reinterpret_cast<const void*>(&xa_tile_kernel<true, 4, true>), reinterpret_cast<const void*>(&xa_tile_kernel<false, 4, true>)};
  for (const void* fn : fns) {
    hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, 2 * kStepUnits * 16);
    if (e != hipSuccess) return e;
  }
  hipError_t e = tile_init_bits<2>();
  if (e == hipSuccess) e = tile_init_bits<3>();
  if (e == hipSuccess) e = tile_init_bits<4>();
  if (e == hipSuccess) e = decode_init_device();
  return e;
}

int expert_ffn_path(const FfnArgs& f) { return 3 & ~decode_parts(f); }

void expert_ffn_plan_specs(const FfnArgs& f, PlanSpec& p13, PlanSpec& p2) { decode_plan_specs(f, decode_parts(f), p13, p2); }

hipError_t launch_expert_ffn(const FfnArgs& f, hipStream_t s) {
  auto tile = [&](int which) {
    switch (f.bits) {
      case 2: return launch_bits<2>(f, s, which);
      case 3: return launch_bits<3>(f, s, which);
      case 4: return launch_bits<4>(f, s, which);
    }
    return hipErrorInvalidValue;
  };
  const int dp = decode_parts(f);
  if (dp == 3) return launch_decode_ffn(f, s, 3);
  hipError_t e = (dp & 1) ? launch_decode_ffn(f, s, 1) : tile(1);
  if (e != hipSuccess) return e;
  return (dp & 2) ? launch_decode_ffn(f, s, 2) : tile(2);
}

}  // namespace lrc
