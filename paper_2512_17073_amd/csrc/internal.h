// Internal declarations shared by the host API and the kernel translation units.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <string>
#include <vector>

#include "../../include/moe_lrc.h"
#include "layout.h"

namespace lrc {

// Device-visible description of one expert: where its packed projections live.
struct ExpertDesc {
  const uint32_t* codes[3];
  const uint32_t* meta[3];
  const _Float16* af[3];      // packed A factor (null if none); a pair held at 3 bits: the code dwords of its units
  const _Float16* bf[3];      // packed B factor; at 3 bits: the metadata of its units
  const uint32_t* afm[3];     // pairs held at 3 bits (layout.h): metadata of the A units ...
  const uint32_t* bfc[3];     // ... and code dwords of the B units
  float lambda[3];            // power-of-two pre-scale folded into the metadata
  float inv_lambda[3];
  float xa_scale[3];          // what (in A) is multiplied by: lambda, over the power-of-two factors folded into a
                              // 3-bit pair's operands
  int32_t rank[3];            // rank of each projection's factor pair (0: none); a prefix of the factor sections
  int32_t has_factors;
  int32_t q3;                 // bit m: projection m's pair is held at 3 bits
};

// Byte offsets of the sections of an expert's two blobs (weights: codes+meta; factors: A+B).
struct BlobLayout {
  MatLayout mat[3];
  size_t off_codes[3], off_meta[3], off_af[3], off_bf[3];
  size_t w_bytes, f_bytes;
};

struct Workspace {       // carved out of the caller's buffer; all offsets 256-byte aligned
  size_t topk_idx, topk_w, counts, offsets, comp_counts, row_pair, pair_row;
  size_t y_rows, xh, xh_sh, h, p13, p2, y_part, sh_y_part, sh_h, sh_y, plan, tok_exp, row_exp, row_exp_sh;
  size_t cmp_index, cmp_list, total;
};

}  // namespace lrc

struct moe_lrc_stack;

struct moe_lrc_layer {
  moe_lrc_config cfg;
  int device;
  moe_lrc_stack* pool = nullptr;       // pooled residency: the stack whose slot pool serves this layer
  int pool_index = -1;                 // ... and the layer's place in it
  size_t dev_w_base = 0;               // device pointer of expert e's weights: d_w + w_off[e] - dev_w_base (pooled
                                       // residency keeps only the shared experts on the device)
  int n_cu = 0;                        // compute units of `device`
  lrc::BlobLayout routed, shared;
  int n_total;                         // E + S
  uint8_t* d_w = nullptr;              // device: weight blobs (resident) or slot pool (staged)
  uint8_t* d_f = nullptr;              // device: factor blobs / slots
  uint8_t* h_w = nullptr;              // pinned host pool (staged only)
  uint8_t* h_f = nullptr;
  std::vector<size_t> w_off, f_off;    // per-expert offsets into the pools
  lrc::ExpertDesc* d_desc = nullptr;
  std::vector<lrc::ExpertDesc> h_desc;
  uint16_t* d_wg = nullptr;
  float* d_bias = nullptr;
  double* d_logits = nullptr;          // [max_tokens][E] gate logits of the routing paths that go through memory (many experts)
  bool gate_set = false, has_bias = false;
  std::vector<uint8_t> mat_set;        // [n_total*3]
  std::vector<int> mat_rank;           // [n_total*3] rank of each projection's factor pair (Section 3.1: may differ)
  std::vector<uint8_t> mat_q3;         // [n_total*3] 1: the pair is held at 3 bits (layout.h), in the projection's own
                                       // factor sections, and dequantized by the kernels that consume it
  std::vector<float> mat_inv_mu;       // [n_total*3] 1 / (the power-of-two factors folded into a 3-bit pair's operands)
  int n_q3 = 0;                        // projections held at 3 bits (0: the launches take the kernels without that path)
  size_t f_total = 0;                  // bytes of d_f (and of h_f)
  int32_t* d_perm = nullptr;           // block counters of the grouping of many pairs by several blocks (kPermuteScratchInts)
  int32_t* d_stat = nullptr;           // [2 + 2E]: active, comp-active, counts, comp counts
  int32_t* h_stat = nullptr;           // pinned mirror
  hipStream_t side = nullptr;
  hipEvent_t ev_t0 = nullptr, ev_t1 = nullptr;   // bracket the staged copies on the side stream
  hipEvent_t ev_fork = nullptr, ev_join = nullptr;   // shared experts on the side stream (resident mode)
  moe_lrc_stats stats{};
  bool stats_valid = false;
  int ksplit13 = 1, ksplit2 = 1;
  bool profile = false, profile_valid = false;
  hipEvent_t marks[MOE_LRC_N_STAGES + 1] = {};   // stage i runs between marks[i] and marks[i+1]
};

namespace lrc {

int set_error(int code, const std::string& msg);
// returns MOE_LRC_EHIP (with the call's text and HIP's message as the last error) if a HIP call fails
#define LRC_HIP(expr)                                                                       \
  do {                                                                                      \
    hipError_t e_ = (expr);                                                                 \
    if (e_ != hipSuccess)                                                                   \
      return lrc::set_error(MOE_LRC_EHIP, std::string(#expr) + ": " + hipGetErrorString(e_)); \
  } while (0)
Workspace plan_workspace(const moe_lrc_layer* L, int T);

// ---- kernel launchers (each returns hipError_t of the launch) ------------------------------
// tok_exp (may be null): receives every token's pre-scale exponent (ffn_common.h) if
// route_writes_exponents(L, T), else it is left untouched
hipError_t launch_route(const moe_lrc_layer* L, const void* x, int T, int32_t* idx, float* w,
                        _Float16* xh /*may be null*/, int32_t* tok_exp, hipStream_t s);
bool route_writes_exponents(const moe_lrc_layer* L, int T);
hipError_t launch_permute(const moe_lrc_layer* L, const int32_t* idx, int T, int32_t* counts,
                          int32_t* offsets, int32_t* row_pair, int32_t* pair_row,
                          int32_t* comp_counts, hipStream_t s);
struct PlanSpec;   // plan.h
// the grouping of the pairs by expert run inside the preparing launch (few pairs): the routing
// kernel's indices in, the five arrays of moe_lrc_permute out
struct PermuteArgs { const int32_t* idx; int32_t *counts, *offsets, *row_pair, *pair_row, *comp_counts; int P; };
constexpr int kFusedPermuteMaxPairs = 1024;
// the routing of a token or two run inside the preparing launch as well (forward only): gate
// [E][H] bf16 and bias (or null) in, the outputs of moe_lrc_route and the tokens' pre-scale exponents out
struct RouteArgs { const uint16_t* wg; const float* bias; int32_t* idx; float* w; int32_t* tok_exp; int renorm; };
constexpr int kFusedRoutePairs = 16;      // (token, expert) gate products: one per wavefront of a block
// above this many pairs several blocks group them (two launches); their counters live in the layer
constexpr int kPermuteOneBlockPairs = 8192, kPermuteMaxBlocks = 64;
constexpr int kPermuteScratchInts = kPermuteMaxBlocks * 2 * 256 + 64;
// The routed rows that take the rank-r term (Section 3.2: the Top-n pairs), compacted per expert in
// row order by the preparing launch for the grouped (in A) kernels, which then touch only those
// rows.  Expert e's compact rows are offsets[e] .. offsets[e] + (its number of such rows) - 1, i.e.
// the front of its own row range: list [T * k] names the routed row of each compact row, index
// [T * k] the compact row of each routed row (-1 for a row without the term).
struct CompactArgs { int32_t *index, *list; };
// The last rows of the operand-order buffers, which the decode flavour stages in place of rows past
// an expert's last one (decode_index.h, staged_row), are kept at zero by one block of the preparing
// launch: those of its own output and, if given, of the buffer `h` (h_rt rows, Fp columns) that the
// fused projection writes next.
struct ZeroRowsArgs { uint4* h; int h_rt, Fp; };
// fp16 copy of the activations in operand order, every row times its power-of-two pre-scale
// (ffn_common.h; exponents to row_exp, taken from tok_exp per token if given): one row per routed
// pair (row_pair given) or one per token (row_pair null); with `stat`, one more block counts the
// per-expert rows
struct FfnArgs;
// xa13: the arguments of the expert-FFN launches that follow, when their fused W1|W3 projection takes
// the decode flavour and wants (x A1 | x A3) made by further blocks of this launch; else null
hipError_t launch_convert_x(const moe_lrc_layer* L, const void* x_bf16, int T, _Float16* xg, int rt,
                            const int32_t* offsets, const int32_t* row_pair, int32_t* stat,
                            const PlanSpec* plans /* two, or null */, const FfnArgs* xa13,
                            const int32_t* tok_exp /* or null */, int32_t* row_exp,
                            const PermuteArgs* perm /* or null: offsets and row_pair are ready */,
                            const CompactArgs* cmp /* or null */, const RouteArgs* route /* or null: perm->idx is ready */,
                            const ZeroRowsArgs& zr,
                            hipStream_t s);
constexpr int kMaxKBlocks = 8;    // most K-blocks the decode W2 kernel splits into
// blocks (per K-block) of a decode launch that shares its blocks out by a table: `target` (the
// device's CUs over the K-blocks), or enough for ceil(NT / 32) blocks per expert that can be active
inline int plan_blocks(int n_exp, int pairs, int NT, int target) {
  const int active = n_exp < pairs ? n_exp : pairs, base = (NT + 31) / 32;
  return active * base > target ? active * base : target;
}

constexpr int kActPadRows = 32;   // rows past the last one that a 32-row staging pass may read

struct FfnArgs {
  const ExpertDesc* desc;     // device array, already offset to the first expert of this launch
  int n_exp;                  // experts in this launch (grid.y)
  int bits, group, rank, rpad;
  int H, F, top_k, top_n, T;
  const int32_t* offsets;     // [n_exp+1] or null: shared experts, rows e*T .. e*T+T-1
  const int32_t* row_pair;    // null for shared experts (row -> token = row % T)
  const int32_t* comp_rows;   // [n_exp] rows that take the rank-r term (written by the prep kernel), or null
  const _Float16* xh;         // gathered activations in operand order, x_rt rows (routed: one per pair)
  _Float16* h;                // SwiGLU output in operand order, h_rt rows
  int x_rt, h_rt;
  float* p13;                 // [ksplit13][rows][2*rpad]
  float* p2;                  // [ksplit2][rows][rpad]
  void* y_rows;               // [rows][H] bf16
  float* y_part;              // fp32 partial outputs of the W2 K-blocks (decode flavour), or null
  int32_t* plan;              // decode flavour, routed experts: the block tables (plan.h) of the two projections
  const void* x_tokens;       // the bf16 tokens [T][H] (routed launches)
  int xa13_here;              // decode flavour of W1|W3: (x A1 | x A3) is made by a launch of its own in front of the
                              // FFN kernel (staged layers: the factors arrive after the preparing launch) instead
                              // of by further blocks of the preparing launch
  int keep_partials;          // decode flavour, W2 split into K-blocks: leave the fp32 partial sums in y_part for
                              // the combine instead of adding them into y_rows
  int ksplit13, ksplit2, total_rows;
  int n_cu;                   // compute units of the device (the launches size their grids to fill them)
  int q3;                     // some factor pair of the layer is held at 3 bits: the launches take the kernels that
                              // can dequantize such pairs
  const PermuteArgs* perm;    // forward with few pairs: the preparing launch groups the pairs itself (else null)
  const int32_t *cmp_index, *cmp_list;   // CompactArgs of this call (null: none made)
  int32_t* row_exp;           // per input row (routed: per routed row; shared: per token): pre-scale exponent
  const int32_t* tok_exp;     // per token, from the routing kernel, or null
  hipEvent_t* marks;          // null, or 4 events recorded after xa13, w13, xa2, w2
};
hipError_t launch_expert_ffn(const FfnArgs& a, hipStream_t s);
// K-blocks the decode flavour splits W2 into (1: none); the W2 output of a launch is y_rows, or with
// keep_partials that many fp32 partial sums [kb][rows][H] in y_part
int decode_w2_kblocks(const FfnArgs& a);
// bit 0: the fused W1|W3 projection takes the grouped GEMM (else the decode flavour), bit 1: W2 does
int expert_ffn_path(const FfnArgs& a);
// once per device, before the first launch: lets the FFN kernels use the whole LDS of a CU
hipError_t ffn_init_device();
hipError_t decode_init_device();
// the block tables (plan.h) that launch_expert_ffn(a) will read: to be made by launch_convert_x
void expert_ffn_plan_specs(const FfnArgs& a, PlanSpec& p13, PlanSpec& p2);
// y_part != null: the expert outputs are the sums over `kblocks` fp32 partial sums [kb][T*k][H]
// (the decode flavour's W2 K-blocks) instead of the bf16 rows y_rows
// residual != null: out = residual + (the weighted sum), rounded once
hipError_t launch_combine(const moe_lrc_layer* L, const void* y_rows, const float* y_part, int kblocks, const float* w,
                          const int32_t* pair_row, const void* y_shared, const void* residual, int T, void* out,
                          hipStream_t s);
// ---- host API internals shared with the layer stack (stack.hip) ----
const BlobLayout& blob_of(const moe_lrc_layer* L, int expert);
void factor_section_bytes(const moe_lrc_layer* L, int e, int mat, size_t& a_bytes, size_t& b_bytes);
void set_factor_ptrs(const moe_lrc_layer* L, int e, int mat, ExpertDesc& d, const uint8_t* a_base, const uint8_t* b_base);
void fill_algorithmic_stats(moe_lrc_layer* L, const int32_t* stat);
// moe_lrc_forward after its argument checks; residual as in launch_combine
int forward_impl(moe_lrc_layer* L, const void* x, int T, void* out, void* ws, hipStream_t s, const void* residual);
// pooled residency, inside the expert FFN after the preparing launch: reads the per-expert counts
// back, brings the experts that received rows into slots of the stack's pool, points the layer's
// expert table at them and makes `s` wait for the copies
int pool_stage(moe_lrc_layer* L, const void* x, int T, hipStream_t s);
hipError_t launch_debug_unpack(const uint32_t* packed, const MatLayout& m, uint8_t* codes_dev,
                               hipStream_t s);
}  // namespace lrc
