// Host side of the C ABI declared in include/moe_lrc.h: argument checking, the layer object and its
// packed-weight storage, workspace carving, the router-guided staging of packed experts and
// factors from the pinned pool (Sections 3.2 and 4.3 case 1), and the launch sequence.
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>

#include "internal.h"
#include "plan.h"
#include "pack.h"

using namespace lrc;

namespace lrc {

static thread_local std::string g_last_error;

int set_error(int code, const std::string& msg) {
  g_last_error = msg;
  return code;
}

static BlobLayout make_blob(const moe_lrc_config& c, int bits, int rank) {
  BlobLayout b{};
  size_t w = 0, f = 0;
  for (int mat = 0; mat < 3; ++mat) {
    const int K = mat == 2 ? c.ffn : c.hidden, N = mat == 2 ? c.hidden : c.ffn;
    b.mat[mat] = make_layout(K, N, bits, c.group, rank);
    b.off_codes[mat] = w; w += b.mat[mat].codes_bytes;
    b.off_meta[mat] = w;  w += b.mat[mat].meta_bytes;
    if (rank > 0) {
      b.off_af[mat] = f; f += b.mat[mat].af_bytes;
      b.off_bf[mat] = f; f += b.mat[mat].bf_bytes;
    }
  }
  b.w_bytes = w;
  b.f_bytes = f;
  return b;
}

static int check_config(const moe_lrc_config& c) {
  auto bad = [](const char* what) { return set_error(MOE_LRC_EINVAL, std::string("config: ") + what); };
  auto shape = [](const char* what) { return set_error(MOE_LRC_ESHAPE, std::string("config: ") + what); };
  if (c.hidden <= 0 || c.ffn <= 0) return bad("hidden and ffn must be positive");
  if (c.hidden > 16384 || c.ffn > 65536) return shape("hidden above 16384 or ffn above 65536");
  if (c.n_experts < 1 || c.n_experts > 256) return bad("n_experts must be in 1..256");
  if (c.n_shared < 0 || c.n_shared > 8) return bad("n_shared must be in 0..8");
  if (c.top_k < 1 || c.top_k > 16 || c.top_k > c.n_experts) return bad("top_k must be in 1..min(n_experts,16)");
  if (c.top_n < 0 || c.top_n > c.top_k) return bad("top_n must be in 0..top_k");
  if (c.bits < 2 || c.bits > 4) return bad("bits must be 2, 3 or 4");
  if (c.n_shared > 0 && (c.shared_bits < 2 || c.shared_bits > 4)) return bad("shared_bits must be 2, 3 or 4");
  if (c.rank < 0 || c.rank > 1024 || c.rank % 8) return bad("rank must be a multiple of 8 in 0..1024");
  if (c.renormalize != 0 && c.renormalize != 1) return bad("renormalize must be 0 or 1");
  if (c.max_tokens < 1 || (long long)c.max_tokens * c.top_k > (1 << 24)) return bad("max_tokens out of range");
  if (c.residency != MOE_LRC_RESIDENT && c.residency != MOE_LRC_STAGED && c.residency != MOE_LRC_POOLED)
    return bad("residency must be MOE_LRC_RESIDENT, MOE_LRC_STAGED or MOE_LRC_POOLED");
  if (c.group != 64 && c.group != 128 && c.group != 256) return shape("group must be 64, 128 or 256");
  if (c.hidden % 64 || c.ffn % 64) return shape("hidden and ffn must be multiples of 64");
  if (c.hidden % c.group || c.ffn % c.group) return shape("hidden and ffn must be multiples of group");
  return MOE_LRC_OK;
}

Workspace plan_workspace(const moe_lrc_layer* L, int T) {
  const moe_lrc_config& c = L->cfg;
  const size_t P = size_t(T) * c.top_k, E = c.n_experts;
  const size_t rpad = L->routed.mat[0].rpad;
  Workspace w{};
  size_t o = 0;
  auto take = [&](size_t bytes) { size_t at = o; o += align256(bytes); return at; };
  w.topk_idx = take(P * 4);  w.topk_w = take(P * 4);
  w.counts = take(E * 4);    w.offsets = take((E + 1) * 4);  w.comp_counts = take(E * 4);
  w.row_pair = take(P * 4);  w.pair_row = take(P * 4);
  w.y_rows = take(P * c.hidden * 2);
  // activations in operand order: whole k-steps (256 columns) and kActPadRows rows of slack
  const size_t Hp = padded_k(c.hidden), Fp = padded_k(c.ffn);
  w.xh = take((P + kActPadRows) * Hp * 2);
  w.xh_sh = take(c.n_shared ? (size_t(T) + kActPadRows) * Hp * 2 : 0);
  w.h = take((P + kActPadRows) * Fp * 2);
  // (in A): K-block partial sums in fp32 and, in the many-rows flavour, the fp16 result in front of
  // them, both with the columns padded to a multiple of 32
  w.p13 = take(size_t(L->ksplit13 + 1) * P * 2 * (rpad + 16) * 4 + 256);
  // (the decode flavour keeps one fp16 (h A2) per W2 K-block)
  w.p2 = take(std::max(size_t(L->ksplit2 + 1) * P * (rpad + 16) * 4, size_t(kMaxKBlocks) * P * (rpad + 16) * 2) + 256);
  w.y_part = take(size_t(kMaxKBlocks) * P * c.hidden * 4);
  w.sh_y_part = take(size_t(kMaxKBlocks) * c.n_shared * T * c.hidden * 4);   // (shared experts run beside the routed ones)
  w.sh_h = take(c.n_shared ? (size_t(c.n_shared) * T + kActPadRows) * Fp * 2 : 0);
  w.sh_y = take(size_t(c.n_shared) * T * c.hidden * 2);
  w.tok_exp = take(size_t(T) * 4);
  w.row_exp = take((P + kActPadRows) * 4);
  w.row_exp_sh = take(c.n_shared ? (size_t(T) + kActPadRows) * 4 : 0);
  w.plan = take(size_t(plan_blocks(c.n_experts, int(P), c.ffn / 16, L->n_cu) + plan_blocks(c.n_experts, int(P), c.hidden / 16, L->n_cu)) * kPlanEntryInts * 4);
  w.cmp_index = take(P * 4);  w.cmp_list = take(P * 4);
  w.total = o;
  return w;
}

const BlobLayout& blob_of(const moe_lrc_layer* L, int expert) {
  return expert < L->cfg.n_experts ? L->routed : L->shared;
}

static int check_hot(const moe_lrc_layer* L, int T, const char* fn) {
  if (!L) return set_error(MOE_LRC_EINVAL, std::string(fn) + ": layer is null");
  if (T < 0 || T > L->cfg.max_tokens)
    return set_error(MOE_LRC_ESTATE, std::string(fn) + ": T outside 0..max_tokens");
  return MOE_LRC_OK;
}

static int check_uploaded(const moe_lrc_layer* L, const char* fn, bool routed, bool shared) {
  const int E = L->cfg.n_experts;
  for (int e = routed ? 0 : E; e < (shared ? L->n_total : E); ++e)
    for (int m = 0; m < 3; ++m)
      if (!L->mat_set[e * 3 + m])
        return set_error(MOE_LRC_ESTATE, std::string(fn) + ": expert " + std::to_string(e) +
                                             " projection " + std::to_string(m) + " not uploaded");
  return MOE_LRC_OK;
}

static int check_ws(const moe_lrc_layer* L, int T, const void* ws, size_t ws_bytes, const char* fn) {
  if (!ws) return set_error(MOE_LRC_EINVAL, std::string(fn) + ": workspace is null");
  if ((uintptr_t)ws & 255) return set_error(MOE_LRC_EINVAL, std::string(fn) + ": workspace must be 256-byte aligned");
  if (ws_bytes < plan_workspace(L, T).total)
    return set_error(MOE_LRC_ENOMEM, std::string(fn) + ": workspace smaller than moe_lrc_workspace_bytes");
  return MOE_LRC_OK;
}

void fill_algorithmic_stats(moe_lrc_layer* L, const int32_t* stat) {
  const moe_lrc_config& c = L->cfg;
  const uint64_t P = 3ull * c.hidden * c.ffn;
  moe_lrc_stats& s = L->stats;
  int active = 0, comp = 0;
  for (int e = 0; e < c.n_experts; ++e) {
    active += stat[2 + e] > 0;
    comp += stat[2 + c.n_experts + e] > 0;
  }
  s.active_experts = active;
  s.comp_experts = (c.rank > 0 && c.top_n > 0) ? comp : 0;
  s.bytes_codes = uint64_t(active) * (P * c.bits / 8) + uint64_t(c.n_shared) * (P * c.shared_bits / 8);
  s.bytes_meta = uint64_t(active + c.n_shared) * (P / c.group * 4);
  s.bytes_factors = 0;
  if (c.rank > 0 && c.top_n > 0)
    for (int e = 0; e < c.n_experts; ++e)
      if (stat[2 + c.n_experts + e] > 0)
        for (int mat = 0; mat < 3; ++mat)      // A [K][r] and B [r][N]: r (K + N) values, as bf16 or as 3-bit codes
          s.bytes_factors += L->mat_q3[e * 3 + mat]
                                 ? uint64_t(L->mat_rank[e * 3 + mat]) * (c.hidden + c.ffn) * 4 / 8 +      // a code per 4-bit cell
                                       uint64_t(L->mat_rank[e * 3 + mat]) * (c.hidden + c.ffn) / 64 * 4     // fp16 scale + zero
                                 : uint64_t(L->mat_rank[e * 3 + mat]) * (c.hidden + c.ffn) * 2;
  L->stats_valid = true;
}

// Bytes at the start of the A and of the B section of (expert, projection) that its factor pair
// fills: the prefix its own rank takes, in the format it is held in.  (The A and B sections of a
// projection are adjacent; a 3-bit pair is one piece that starts with the A section.)
void factor_section_bytes(const moe_lrc_layer* L, int e, int mat, size_t& a_bytes, size_t& b_bytes) {
  const MatLayout& m = blob_of(L, e).mat[mat];
  const int r = L->mat_rank[e * 3 + mat];
  a_bytes = b_bytes = 0;
  if (r == 0) return;
  if (L->mat_q3[e * 3 + mat]) {      // one piece: the B part lies right behind the A part, at the start of the A section
    a_bytes = align256(q3_a_bytes(m.K, r)) + q3_b_bytes(m.N, r);
  } else {
    const MatLayout fm = make_layout(m.K, m.N, m.bits, m.group, r);
    a_bytes = fm.af_bytes; b_bytes = fm.bf_bytes;
  }
}

// Points projection `mat` of an expert table entry at its factor sections (a_base, b_base: the
// starts of the projection's A and B sections on the device).
void set_factor_ptrs(const moe_lrc_layer* L, int e, int mat, ExpertDesc& d, const uint8_t* a_base, const uint8_t* b_base) {
  const MatLayout& m = blob_of(L, e).mat[mat];
  const int r = L->mat_rank[e * 3 + mat];
  d.afm[mat] = nullptr; d.bfc[mat] = nullptr;
  if (L->mat_q3[e * 3 + mat]) {
    const uint8_t* bq = a_base + align256(q3_a_bytes(m.K, r));      // (the B part follows the A part)
    d.af[mat] = reinterpret_cast<const _Float16*>(a_base);
    d.afm[mat] = reinterpret_cast<const uint32_t*>(a_base + q3_a_codes_bytes(m.K, r));
    d.bfc[mat] = reinterpret_cast<const uint32_t*>(bq);
    d.bf[mat] = reinterpret_cast<const _Float16*>(bq + q3_b_codes_bytes(m.N, r));
  } else {
    d.af[mat] = reinterpret_cast<const _Float16*>(a_base);
    d.bf[mat] = reinterpret_cast<const _Float16*>(b_base);
  }
}

// Copies the packed blobs of every expert that received a row, and the factor blobs of every expert
// that received a Top-n row, from the pinned pool into the device slots on the side stream.
static int stage_selected(moe_lrc_layer* L, hipStream_t stream) {
  const moe_lrc_config& c = L->cfg;
  const int E = c.n_experts;
  LRC_HIP(hipMemcpyAsync(L->h_stat, L->d_stat, (2 + 2 * E) * 4, hipMemcpyDeviceToHost, stream));
  LRC_HIP(hipStreamSynchronize(stream));       // the one host read-back: which experts are needed
  fill_algorithmic_stats(L, L->h_stat);
  LRC_HIP(hipEventRecord(L->ev_t0, L->side));
  for (int e = 0; e < E; ++e) {
    const BlobLayout& b = blob_of(L, e);
    if (L->h_stat[2 + e] > 0)
      LRC_HIP(hipMemcpyAsync(L->d_w + L->w_off[e], L->h_w + L->w_off[e], b.w_bytes, hipMemcpyHostToDevice, L->side));
    if (b.f_bytes && c.top_n > 0 && L->h_stat[2 + E + e] > 0) {
      const int* r = &L->mat_rank[e * 3];
      const uint8_t* q3 = &L->mat_q3[e * 3];
      if (!(q3[0] | q3[1] | q3[2]) && r[0] == c.rank && r[1] == c.rank && r[2] == c.rank) {   // the whole factor blob in one piece
        LRC_HIP(hipMemcpyAsync(L->d_f + L->f_off[e], L->h_f + L->f_off[e], b.f_bytes, hipMemcpyHostToDevice, L->side));
      } else {
        for (int mat = 0; mat < 3; ++mat) {      // the prefixes the projection's rank fills, in the format it is held in
          size_t ab, bb;
          factor_section_bytes(L, e, mat, ab, bb);
          const size_t aoff = L->f_off[e] + b.off_af[mat], boff = L->f_off[e] + b.off_bf[mat];
          if (ab) LRC_HIP(hipMemcpyAsync(L->d_f + aoff, L->h_f + aoff, ab, hipMemcpyHostToDevice, L->side));
          if (bb) LRC_HIP(hipMemcpyAsync(L->d_f + boff, L->h_f + boff, bb, hipMemcpyHostToDevice, L->side));
        }
      }
    }
  }
  LRC_HIP(hipEventRecord(L->ev_t1, L->side));
  LRC_HIP(hipStreamWaitEvent(stream, L->ev_t1, 0));
  return MOE_LRC_OK;
}

static int run_expert_ffn(moe_lrc_layer* L, const void* x, int T, const int32_t* offsets,
                          const int32_t* row_pair, void* y_rows, uint8_t* ws, hipStream_t stream,
                          bool mark = false, bool keep_partials = false, int* kblocks_out = nullptr,
                          const int32_t* tok_exp = nullptr, const PermuteArgs* perm = nullptr, const RouteArgs* route = nullptr) {
  const moe_lrc_config& c = L->cfg;
  const Workspace w = plan_workspace(L, T);
  _Float16* xh = reinterpret_cast<_Float16*>(ws + w.xh);
  const int P = T * c.top_k;
  FfnArgs a{};
  a.desc = L->d_desc; a.n_exp = c.n_experts; a.bits = c.bits; a.group = c.group;
  a.rank = c.rank; a.rpad = L->routed.mat[0].rpad;
  a.H = c.hidden; a.F = c.ffn; a.top_k = c.top_k; a.top_n = c.top_n; a.T = T;
  a.offsets = offsets; a.row_pair = row_pair; a.xh = xh;
  a.comp_rows = L->d_stat + 2 + c.n_experts;
  a.h = reinterpret_cast<_Float16*>(ws + w.h);
  a.x_rt = P + kActPadRows; a.h_rt = P + kActPadRows;
  a.p13 = reinterpret_cast<float*>(ws + w.p13); a.p2 = reinterpret_cast<float*>(ws + w.p2);
  a.y_part = reinterpret_cast<float*>(ws + w.y_part);
  a.plan = reinterpret_cast<int32_t*>(ws + w.plan);
  a.y_rows = y_rows; a.ksplit13 = L->ksplit13; a.ksplit2 = L->ksplit2; a.total_rows = T * c.top_k;
  a.n_cu = L->n_cu;
  a.q3 = L->n_q3 > 0;
  a.row_exp = reinterpret_cast<int32_t*>(ws + w.row_exp);
  a.tok_exp = tok_exp;
  const int path = expert_ffn_path(a);
  // the combine can add the K-block partial sums of a decode-flavour W2 itself
  const int kblocks = (path & 2) ? 1 : decode_w2_kblocks(a);
  a.keep_partials = keep_partials && kblocks > 1;
  if (kblocks_out) *kblocks_out = a.keep_partials ? kblocks : 1;
  // the launch that converts the activations also makes the block tables of the decode launches
  // and, for the decode flavour of the fused projection, (x A1 | x A3)
  PlanSpec plans[2];
  expert_ffn_plan_specs(a, plans[0], plans[1]);
  // ((x A1 | x A3) from the tokens inside the preparing launch needs the exponents beforehand)
  a.xa13_here = c.residency != MOE_LRC_RESIDENT || tok_exp == nullptr;
  a.x_tokens = x;
  // (the grouped (in A) kernels work on the rows that take the rank-r term only: their compact order)
  const bool comp = c.rank > 0 && c.top_n > 0 && path != 0;
  const CompactArgs cmp{reinterpret_cast<int32_t*>(ws + w.cmp_index), reinterpret_cast<int32_t*>(ws + w.cmp_list)};
  if (comp) { a.cmp_index = cmp.index; a.cmp_list = cmp.list; }
  LRC_HIP(launch_convert_x(L, x, T, xh, P + kActPadRows, offsets, row_pair, L->d_stat, plans,
                           ((path & 1) || a.xa13_here) ? nullptr : &a, tok_exp, a.row_exp, perm, comp ? &cmp : nullptr, route,
                           ZeroRowsArgs{reinterpret_cast<uint4*>(a.h), a.h_rt, padded_k(c.ffn)}, stream));
  L->stats_valid = false;
  L->stats.stage_ms = 0.f;
  if (c.residency == MOE_LRC_STAGED) {
    const int rc = stage_selected(L, stream);
    if (rc) return rc;
  } else if (c.residency == MOE_LRC_POOLED) {
    const int rc = pool_stage(L, x, T, stream);
    if (rc) return rc;
  }
  if (mark) LRC_HIP(hipEventRecord(L->marks[MOE_LRC_STAGE_XA13], stream));
  a.marks = mark ? &L->marks[MOE_LRC_STAGE_W13] : nullptr;
  LRC_HIP(launch_expert_ffn(a, stream));
  L->stats.path = path;
  return MOE_LRC_OK;
}

static int run_shared(moe_lrc_layer* L, const void* x, int T, uint8_t* ws, hipStream_t stream) {
  const moe_lrc_config& c = L->cfg;
  const Workspace w = plan_workspace(L, T);
  _Float16* xh = reinterpret_cast<_Float16*>(ws + w.xh_sh);
  int32_t* row_exp = reinterpret_cast<int32_t*>(ws + w.row_exp_sh);
  LRC_HIP(launch_convert_x(L, x, T, xh, T + kActPadRows, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, row_exp, nullptr, nullptr, nullptr,
                           ZeroRowsArgs{reinterpret_cast<uint4*>(ws + w.sh_h), c.n_shared * T + kActPadRows, padded_k(c.ffn)}, stream));
  FfnArgs a{};
  a.desc = L->d_desc + c.n_experts; a.n_exp = c.n_shared; a.bits = c.shared_bits; a.group = c.group;
  a.rank = 0; a.rpad = 0; a.H = c.hidden; a.F = c.ffn; a.top_k = c.top_k; a.top_n = 0; a.T = T;
  a.offsets = nullptr; a.row_pair = nullptr; a.xh = xh;
  a.h = reinterpret_cast<_Float16*>(ws + w.sh_h);
  a.x_rt = T + kActPadRows; a.h_rt = c.n_shared * T + kActPadRows;
  a.y_part = reinterpret_cast<float*>(ws + w.sh_y_part);
  a.y_rows = ws + w.sh_y; a.ksplit13 = 1; a.ksplit2 = 1; a.total_rows = T * c.n_shared;
  a.n_cu = L->n_cu;
  a.row_exp = row_exp; a.tok_exp = nullptr;
  LRC_HIP(launch_expert_ffn(a, stream));
  return MOE_LRC_OK;
}

}  // namespace lrc

extern "C" {

const char* moe_lrc_last_error(void) { return g_last_error.c_str(); }

int moe_lrc_layer_create(const moe_lrc_config* cfg, moe_lrc_layer** out) {
  if (!cfg || !out) return set_error(MOE_LRC_EINVAL, "layer_create: null argument");
  int rc = check_config(*cfg);
  if (rc) return rc;
  int dev = 0;
  LRC_HIP(hipGetDevice(&dev));
  moe_lrc_layer* L = new (std::nothrow) moe_lrc_layer();
  if (!L) return set_error(MOE_LRC_ENOMEM, "layer_create: out of host memory");
  L->cfg = *cfg;
  L->device = dev;
  {
    // once per device: the FFN kernels are allowed the whole LDS of a CU
    static std::mutex mu;
    static bool ready[64] = {};
    std::lock_guard<std::mutex> lock(mu);
    if (dev >= 0 && dev < 64 && !ready[dev]) {
      hipError_t e = ffn_init_device();
      if (e != hipSuccess) {
        delete L;
        return set_error(MOE_LRC_EHIP, std::string("layer_create: kernel attributes: ") + hipGetErrorString(e));
      }
      ready[dev] = true;
    }
  }
  if (hipDeviceGetAttribute(&L->n_cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || L->n_cu <= 0) {
    delete L;
    return set_error(MOE_LRC_EHIP, "layer_create: cannot read the device's compute unit count");
  }
  L->n_total = cfg->n_experts + cfg->n_shared;
  L->routed = make_blob(*cfg, cfg->bits, cfg->rank);
  L->shared = make_blob(*cfg, cfg->n_shared ? cfg->shared_bits : cfg->bits, 0);
  L->ksplit13 = std::max(1, std::min(8, cfg->hidden / 512));
  L->ksplit2 = std::max(1, std::min(16, cfg->ffn / 512));
  L->mat_set.assign(size_t(L->n_total) * 3, 0);
  L->mat_rank.assign(size_t(L->n_total) * 3, 0);
  L->mat_q3.assign(size_t(L->n_total) * 3, 0);
  L->mat_inv_mu.assign(size_t(L->n_total) * 3, 1.f);
  size_t w = 0, f = 0;
  for (int e = 0; e < L->n_total; ++e) {
    L->w_off.push_back(w); L->f_off.push_back(f);
    w += blob_of(L, e).w_bytes; f += blob_of(L, e).f_bytes;
  }
  const bool pooled = cfg->residency == MOE_LRC_POOLED, host_homed = cfg->residency != MOE_LRC_RESIDENT;
  // pooled residency: only the shared experts (always on) own device memory here
  L->dev_w_base = !pooled ? 0 : cfg->n_shared > 0 ? L->w_off[cfg->n_experts] : w;
  const size_t w_dev = w - L->dev_w_base, f_dev = pooled ? 0 : f;
  auto fail = [&](int code) { moe_lrc_layer_destroy(L); return code; };
#define LRC_TRY(expr)                                                                             \
  do {                                                                                            \
    hipError_t e_ = (expr);                                                                       \
    if (e_ != hipSuccess)                                                                         \
      return fail(set_error(e_ == hipErrorOutOfMemory ? MOE_LRC_ENOMEM : MOE_LRC_EHIP,            \
                            std::string(#expr) + ": " + hipGetErrorString(e_)));                  \
  } while (0)
  LRC_TRY(hipMalloc((void**)&L->d_w, std::max<size_t>(w_dev, 256)));
  L->f_total = std::max<size_t>(f, 256);
  LRC_TRY(hipMalloc((void**)&L->d_f, std::max<size_t>(f_dev, 256)));
  // (a projection uploaded with a smaller rank fills a prefix of its sections: the rest stays zero)
  LRC_TRY(hipMemset(L->d_f, 0, std::max<size_t>(f_dev, 256)));
  if (host_homed) {
    LRC_TRY(hipHostMalloc((void**)&L->h_w, std::max<size_t>(w, 256), hipHostMallocDefault));
    LRC_TRY(hipHostMalloc((void**)&L->h_f, std::max<size_t>(f, 256), hipHostMallocDefault));
    // (pooled residency copies an expert's factor blob whole: what lies behind a smaller rank's prefix is zero)
    std::memset(L->h_f, 0, std::max<size_t>(f, 256));
    LRC_TRY(hipEventCreate(&L->ev_t0));
    LRC_TRY(hipEventCreate(&L->ev_t1));
  }
  if (cfg->residency == MOE_LRC_STAGED || cfg->n_shared > 0) {   // side stream: copies, or the shared experts
    LRC_TRY(hipStreamCreateWithFlags(&L->side, hipStreamNonBlocking));
    LRC_TRY(hipEventCreateWithFlags(&L->ev_fork, hipEventDisableTiming));
    LRC_TRY(hipEventCreateWithFlags(&L->ev_join, hipEventDisableTiming));
  }
  LRC_TRY(hipMalloc((void**)&L->d_desc, sizeof(ExpertDesc) * L->n_total));
  LRC_TRY(hipMalloc((void**)&L->d_wg, size_t(cfg->n_experts) * cfg->hidden * 2));
  LRC_TRY(hipMalloc((void**)&L->d_bias, size_t(cfg->n_experts) * 4));
  if (cfg->n_experts >= 128) {
    LRC_TRY(hipMalloc((void**)&L->d_logits, size_t(cfg->max_tokens) * cfg->n_experts * 8));
  }
  LRC_TRY(hipMalloc((void**)&L->d_perm, kPermuteScratchInts * 4));
  LRC_TRY(hipMemset(L->d_perm, 0, kPermuteScratchInts * 4));
  LRC_TRY(hipMalloc((void**)&L->d_stat, (2 + 2 * cfg->n_experts) * 4));
  LRC_TRY(hipMemset(L->d_stat, 0, (2 + 2 * cfg->n_experts) * 4));
  LRC_TRY(hipHostMalloc((void**)&L->h_stat, (2 + 2 * cfg->n_experts) * 4, hipHostMallocDefault));
  L->h_desc.resize(L->n_total);
  for (int e = 0; e < L->n_total; ++e) {
    const BlobLayout& b = blob_of(L, e);
    ExpertDesc& d = L->h_desc[e];
    std::memset(&d, 0, sizeof(d));
    for (int m = 0; m < 3; ++m) {
      if (pooled && e < cfg->n_experts) {        // pointers come from the stack's slots, call by call
        d.lambda[m] = d.inv_lambda[m] = d.xa_scale[m] = 1.f;
        continue;
      }
      d.codes[m] = reinterpret_cast<const uint32_t*>(L->d_w + L->w_off[e] - L->dev_w_base + b.off_codes[m]);
      d.meta[m] = reinterpret_cast<const uint32_t*>(L->d_w + L->w_off[e] - L->dev_w_base + b.off_meta[m]);
      if (b.f_bytes) {
        d.af[m] = reinterpret_cast<const _Float16*>(L->d_f + L->f_off[e] + b.off_af[m]);
        d.bf[m] = reinterpret_cast<const _Float16*>(L->d_f + L->f_off[e] + b.off_bf[m]);
      }
      d.lambda[m] = d.inv_lambda[m] = d.xa_scale[m] = 1.f;
    }
    d.has_factors = b.f_bytes ? 1 : 0;
  }
  LRC_TRY(hipMemcpy(L->d_desc, L->h_desc.data(), sizeof(ExpertDesc) * L->n_total, hipMemcpyHostToDevice));
#undef LRC_TRY
  *out = L;
  return MOE_LRC_OK;
}

int moe_lrc_layer_destroy(moe_lrc_layer* L) {
  if (!L) return MOE_LRC_OK;
  (void)hipDeviceSynchronize();
  if (L->d_w) (void)hipFree(L->d_w);
  if (L->d_f) (void)hipFree(L->d_f);
  if (L->h_w) (void)hipHostFree(L->h_w);
  if (L->h_f) (void)hipHostFree(L->h_f);
  if (L->d_desc) (void)hipFree(L->d_desc);
  if (L->d_wg) (void)hipFree(L->d_wg);
  if (L->d_bias) (void)hipFree(L->d_bias);
  if (L->d_stat) (void)hipFree(L->d_stat);
  if (L->d_perm) (void)hipFree(L->d_perm);
  if (L->d_logits) (void)hipFree(L->d_logits);
  if (L->h_stat) (void)hipHostFree(L->h_stat);
  if (L->side) (void)hipStreamDestroy(L->side);
  if (L->ev_t0) (void)hipEventDestroy(L->ev_t0);
  if (L->ev_t1) (void)hipEventDestroy(L->ev_t1);
  if (L->ev_fork) (void)hipEventDestroy(L->ev_fork);
  if (L->ev_join) (void)hipEventDestroy(L->ev_join);
  for (auto ev : L->marks)
    if (ev) (void)hipEventDestroy(ev);
  delete L;
  return MOE_LRC_OK;
}

int moe_lrc_set_gate(moe_lrc_layer* L, const uint16_t* wg, const float* bias) {
  if (!L || !wg) return set_error(MOE_LRC_EINVAL, "set_gate: null argument");
  const moe_lrc_config& c = L->cfg;
  LRC_HIP(hipMemcpy(L->d_wg, wg, size_t(c.n_experts) * c.hidden * 2, hipMemcpyHostToDevice));
  if (bias) LRC_HIP(hipMemcpy(L->d_bias, bias, size_t(c.n_experts) * 4, hipMemcpyHostToDevice));
  L->has_bias = bias != nullptr;
  L->gate_set = true;
  return MOE_LRC_OK;
}

int moe_lrc_set_expert_ranked(moe_lrc_layer* L, int expert, int mat, const uint8_t* codes,
                              const uint16_t* scale, const uint16_t* zero, const uint16_t* A, const uint16_t* B,
                              int rank) {
  if (!L || !codes || !scale || !zero) return set_error(MOE_LRC_EINVAL, "set_expert: null argument");
  if (expert < 0 || expert >= L->n_total) return set_error(MOE_LRC_EINVAL, "set_expert: expert out of range");
  if (mat < 0 || mat > 2) return set_error(MOE_LRC_EINVAL, "set_expert: mat must be 0, 1 or 2");
  const moe_lrc_config& c = L->cfg;
  const BlobLayout& b = blob_of(L, expert);
  const MatLayout& m = b.mat[mat];
  const int max_rank = b.f_bytes > 0 ? c.rank : 0;
  if (rank < 0 || rank > max_rank || rank % 8)
    return set_error(MOE_LRC_EINVAL, "set_expert: rank must be a multiple of 8 in 0..layer rank (0 for shared experts)");
  const bool wants = rank > 0;
  if (wants && (!A || !B)) return set_error(MOE_LRC_EINVAL, "set_expert: factors required when rank > 0");
  if (!wants && (A || B)) return set_error(MOE_LRC_EINVAL, "set_expert: factors given for rank 0 or a shared expert");
  const uint32_t limit = 1u << m.bits;
  for (size_t i = 0; i < size_t(m.K) * m.N; ++i)
    if (codes[i] >= limit) return set_error(MOE_LRC_EINVAL, "set_expert: code out of range for the bit width");

  std::vector<uint8_t> wbuf(m.codes_bytes + m.meta_bytes);
  pack_codes(m, codes, reinterpret_cast<uint32_t*>(wbuf.data()));
  const float lambda = pack_meta(m, scale, zero, reinterpret_cast<uint32_t*>(wbuf.data() + m.codes_bytes));
  // codes and meta sections of one projection are adjacent in the blob
  // (shared experts serve every token of every call: their slots are filled here, once, also in
  // staged residency; only routed experts live in the pinned pool)
  const size_t woff = L->w_off[expert] + b.off_codes[mat];
  const bool host_homed = c.residency != MOE_LRC_RESIDENT, pooled = c.residency == MOE_LRC_POOLED;
  if (host_homed && expert < c.n_experts) std::memcpy(L->h_w + woff, wbuf.data(), wbuf.size());
  else LRC_HIP(hipMemcpy(L->d_w + woff - L->dev_w_base, wbuf.data(), wbuf.size(), hipMemcpyHostToDevice));

  // Factors: the layouts are rank-major, so the pair of rank `rank` is a prefix of the projection's A
  // section and a prefix of its B section; only the prefixes are staged.  (The kernels take each
  // projection's own rank from the expert table and read nothing past it; the rest of both sections
  // is kept zero in the device slot all the same.)
  if (b.f_bytes > 0) {
    const MatLayout fm = make_layout(m.K, m.N, m.bits, m.group, rank);     // sizes of the prefixes
    const size_t aoff = L->f_off[expert] + b.off_af[mat], boff = L->f_off[expert] + b.off_bf[mat];
    std::vector<uint8_t> abuf(fm.af_bytes), bbuf(fm.bf_bytes);
    if (wants) {
      pack_factor_a(fm, rank, A, reinterpret_cast<uint16_t*>(abuf.data()));
      pack_factor_b(fm, rank, B, reinterpret_cast<uint16_t*>(bbuf.data()));
    }
    if (host_homed) {
      if (wants) { std::memcpy(L->h_f + aoff, abuf.data(), abuf.size()); std::memcpy(L->h_f + boff, bbuf.data(), bbuf.size()); }
      if (pooled) {                    // (the blob is copied whole: keep what lies behind the prefixes zero)
        std::memset(L->h_f + aoff + fm.af_bytes, 0, m.af_bytes - fm.af_bytes);
        std::memset(L->h_f + boff + fm.bf_bytes, 0, m.bf_bytes - fm.bf_bytes);
      }
    } else if (wants) {
      LRC_HIP(hipMemcpy(L->d_f + aoff, abuf.data(), abuf.size(), hipMemcpyHostToDevice));
      LRC_HIP(hipMemcpy(L->d_f + boff, bbuf.data(), bbuf.size(), hipMemcpyHostToDevice));
    }
    // what an earlier upload with a larger rank may have left behind the prefixes
    if (!pooled && m.af_bytes > fm.af_bytes) LRC_HIP(hipMemset(L->d_f + aoff + fm.af_bytes, 0, m.af_bytes - fm.af_bytes));
    if (!pooled && m.bf_bytes > fm.bf_bytes) LRC_HIP(hipMemset(L->d_f + boff + fm.bf_bytes, 0, m.bf_bytes - fm.bf_bytes));
  }
  L->mat_rank[expert * 3 + mat] = rank;
  L->n_q3 -= L->mat_q3[expert * 3 + mat];
  L->mat_q3[expert * 3 + mat] = 0;
  L->mat_inv_mu[expert * 3 + mat] = 1.f;
  ExpertDesc& d = L->h_desc[expert];
  d.rank[mat] = rank;
  d.lambda[mat] = lambda;
  d.inv_lambda[mat] = 1.0f / lambda;
  d.xa_scale[mat] = lambda;
  d.q3 &= ~(1 << mat);
  if (b.f_bytes > 0 && !(pooled && expert < c.n_experts))
    set_factor_ptrs(L, expert, mat, d, L->d_f + L->f_off[expert] + b.off_af[mat], L->d_f + L->f_off[expert] + b.off_bf[mat]);
  LRC_HIP(hipMemcpy(L->d_desc + expert, &d, sizeof(ExpertDesc), hipMemcpyHostToDevice));
  L->mat_set[expert * 3 + mat] = 1;
  return MOE_LRC_OK;
}

int moe_lrc_set_expert(moe_lrc_layer* L, int expert, int mat, const uint8_t* codes,
                       const uint16_t* scale, const uint16_t* zero, const uint16_t* A, const uint16_t* B) {
  if (!L) return set_error(MOE_LRC_EINVAL, "set_expert: null argument");
  const bool routed = expert >= 0 && expert < L->cfg.n_experts;
  return moe_lrc_set_expert_ranked(L, expert, mat, codes, scale, zero, A, B, routed ? L->cfg.rank : 0);
}

int moe_lrc_set_expert_factors_quantized(moe_lrc_layer* L, int expert, int mat, int rank,
                                  const uint8_t* a_codes, const uint16_t* a_scale, const uint16_t* a_zero,
                                  const uint8_t* b_codes, const uint16_t* b_scale, const uint16_t* b_zero) {
  if (!L || !a_codes || !a_scale || !a_zero || !b_codes || !b_scale || !b_zero)
    return set_error(MOE_LRC_EINVAL, "set_expert_factors_quantized: null argument");
  const moe_lrc_config& c = L->cfg;
  if (expert < 0 || expert >= c.n_experts) return set_error(MOE_LRC_EINVAL, "set_expert_factors_quantized: not a routed expert");
  if (mat < 0 || mat > 2) return set_error(MOE_LRC_EINVAL, "set_expert_factors_quantized: mat must be 0, 1 or 2");
  if (rank <= 0 || rank > c.rank || rank % 8)
    return set_error(MOE_LRC_EINVAL, "set_expert_factors_quantized: rank must be a multiple of 8 in 8..layer rank");
  if (!L->mat_set[expert * 3 + mat])
    return set_error(MOE_LRC_ESTATE, "set_expert_factors_quantized: upload the projection's codes with set_expert first");
  const BlobLayout& b = L->routed;
  const MatLayout& m = b.mat[mat];
  // The pair goes into the projection's own A and B sections, in the unit layout the kernels
  // dequantize from (layout.h): smaller than the fp16 pair of the same rank, so it always fits.
  std::vector<uint8_t> abuf(q3_a_bytes(m.K, rank)), bbuf(q3_b_bytes(m.N, rank));
  const float mu_a = pack_factor_a_q3(m.K, rank, a_codes, a_scale, a_zero, abuf.data());
  const float mu_b = pack_factor_b_q3(m.N, rank, b_codes, b_scale, b_zero, bbuf.data());
  if (mu_a == 0.f || mu_b == 0.f) return set_error(MOE_LRC_EINVAL, "set_expert_factors_quantized: code out of range (3 bits)");
  // one piece at the start of the projection's A section (the B section follows it in the blob): the
  // A part, then the B part at the next multiple of 256 bytes; one copy brings it in
  const size_t aoff = L->f_off[expert] + b.off_af[mat];
  if (b.off_bf[mat] != b.off_af[mat] + m.af_bytes) return set_error(MOE_LRC_ESTATE, "set_expert_factors_quantized: factor sections not adjacent");
  std::vector<uint8_t> piece(align256(abuf.size()) + bbuf.size(), 0);
  std::memcpy(piece.data(), abuf.data(), abuf.size());
  std::memcpy(piece.data() + align256(abuf.size()), bbuf.data(), bbuf.size());
  const size_t span = m.af_bytes + m.bf_bytes;
  const bool host_homed = c.residency != MOE_LRC_RESIDENT, pooled = c.residency == MOE_LRC_POOLED;
  if (host_homed) std::memcpy(L->h_f + aoff, piece.data(), piece.size());
  else LRC_HIP(hipMemcpy(L->d_f + aoff, piece.data(), piece.size(), hipMemcpyHostToDevice));
  // what an earlier upload may have left behind the pair
  if (pooled) std::memset(L->h_f + aoff + piece.size(), 0, span - piece.size());
  else LRC_HIP(hipMemset(L->d_f + aoff + piece.size(), 0, span - piece.size()));
  L->mat_rank[expert * 3 + mat] = rank;
  L->n_q3 += 1 - L->mat_q3[expert * 3 + mat];
  L->mat_q3[expert * 3 + mat] = 1;
  L->mat_inv_mu[expert * 3 + mat] = 1.0f / (mu_a * mu_b);
  ExpertDesc& d = L->h_desc[expert];
  d.rank[mat] = rank;
  d.xa_scale[mat] = d.lambda[mat] * L->mat_inv_mu[expert * 3 + mat];
  d.q3 |= 1 << mat;
  if (!pooled) set_factor_ptrs(L, expert, mat, d, L->d_f + aoff, L->d_f + L->f_off[expert] + b.off_bf[mat]);
  LRC_HIP(hipMemcpy(L->d_desc + expert, &d, sizeof(ExpertDesc), hipMemcpyHostToDevice));
  return MOE_LRC_OK;
}

size_t moe_lrc_workspace_bytes(const moe_lrc_layer* L, int T) {
  if (!L || T < 0) return 0;
  return plan_workspace(L, T).total;
}

int moe_lrc_route(moe_lrc_layer* L, const void* x, int T, int32_t* idx, float* w, void* stream) {
  int rc = check_hot(L, T, "route");
  if (rc) return rc;
  if (!L->gate_set) return set_error(MOE_LRC_ESTATE, "route: gate not uploaded");
  if (T == 0) return MOE_LRC_OK;                 // (an empty batch: the per-token buffers may be null)
  if (!x || !idx || !w) return set_error(MOE_LRC_EINVAL, "route: null argument");
  LRC_HIP(launch_route(L, x, T, idx, w, nullptr, nullptr, (hipStream_t)stream));
  return MOE_LRC_OK;
}

int moe_lrc_permute(moe_lrc_layer* L, const int32_t* idx, int T, int32_t* counts, int32_t* offsets,
                    int32_t* row_pair, int32_t* pair_row, int32_t* comp_counts, void* stream) {
  int rc = check_hot(L, T, "permute");
  if (rc) return rc;
  if (!counts || !offsets || !comp_counts || (T > 0 && (!idx || !row_pair || !pair_row)))
    return set_error(MOE_LRC_EINVAL, "permute: null argument");
  LRC_HIP(launch_permute(L, idx, T, counts, offsets, row_pair, pair_row, comp_counts, (hipStream_t)stream));
  return MOE_LRC_OK;
}

int moe_lrc_expert_ffn(moe_lrc_layer* L, const void* x, int T, const int32_t* offsets,
                       const int32_t* row_pair, void* y_rows, void* ws, size_t ws_bytes, void* stream) {
  int rc = check_hot(L, T, "expert_ffn");
  if (rc) return rc;
  if ((rc = check_uploaded(L, "expert_ffn", true, false))) return rc;
  if (L->cfg.residency == MOE_LRC_POOLED)
    return set_error(MOE_LRC_ESTATE, "expert_ffn: a pooled layer runs through moe_lrc_stack_step only");
  if (T == 0) return MOE_LRC_OK;
  if (!x || !offsets || !row_pair || !y_rows) return set_error(MOE_LRC_EINVAL, "expert_ffn: null argument");
  if ((rc = check_ws(L, T, ws, ws_bytes, "expert_ffn"))) return rc;
  return run_expert_ffn(L, x, T, offsets, row_pair, y_rows, (uint8_t*)ws, (hipStream_t)stream);
}

int moe_lrc_combine(moe_lrc_layer* L, const void* y_rows, const float* w, const int32_t* pair_row,
                    const void* x, int T, void* out, void* ws, size_t ws_bytes, void* stream) {
  int rc = check_hot(L, T, "combine");
  if (rc) return rc;
  const bool shared = L->cfg.n_shared > 0;
  if (T == 0) return (shared && (rc = check_uploaded(L, "combine", false, true))) ? rc : MOE_LRC_OK;
  if (!y_rows || !w || !pair_row || !out) return set_error(MOE_LRC_EINVAL, "combine: null argument");
  if (shared) {
    if (!x) return set_error(MOE_LRC_EINVAL, "combine: x is required when the layer has shared experts");
    if ((rc = check_ws(L, T, ws, ws_bytes, "combine"))) return rc;
    if ((rc = check_uploaded(L, "combine", false, true))) return rc;
  }
  if (T == 0) return MOE_LRC_OK;
  const void* y_shared = nullptr;
  if (shared) {
    if (L->cfg.residency != MOE_LRC_RESIDENT && (rc = check_uploaded(L, "combine", true, true))) return rc;
    if ((rc = run_shared(L, x, T, (uint8_t*)ws, (hipStream_t)stream))) return rc;
    y_shared = (uint8_t*)ws + plan_workspace(L, T).sh_y;
  }
  LRC_HIP(launch_combine(L, y_rows, nullptr, 1, w, pair_row, y_shared, nullptr, T, out, (hipStream_t)stream));
  return MOE_LRC_OK;
}

int moe_lrc_forward(moe_lrc_layer* L, const void* x, int T, void* out, void* ws, size_t ws_bytes, void* stream) {
  int rc = check_hot(L, T, "forward");
  if (rc) return rc;
  if (!L->gate_set) return set_error(MOE_LRC_ESTATE, "forward: gate not uploaded");
  if ((rc = check_uploaded(L, "forward", true, true))) return rc;
  if (L->cfg.residency == MOE_LRC_POOLED)
    return set_error(MOE_LRC_ESTATE, "forward: a pooled layer runs through moe_lrc_stack_step only");
  if (T == 0) return MOE_LRC_OK;
  if (!x || !out) return set_error(MOE_LRC_EINVAL, "forward: null argument");
  if ((rc = check_ws(L, T, ws, ws_bytes, "forward"))) return rc;
  return forward_impl(L, x, T, out, ws, (hipStream_t)stream, nullptr);
}

}  // extern "C"

namespace lrc {
int forward_impl(moe_lrc_layer* L, const void* x, int T, void* out, void* ws, hipStream_t s, const void* residual) {
  int rc = MOE_LRC_OK;
  uint8_t* b = (uint8_t*)ws;
  const Workspace w = plan_workspace(L, T);
  int32_t* idx = (int32_t*)(b + w.topk_idx);
  float* tw = (float*)(b + w.topk_w);
  int32_t* offsets = (int32_t*)(b + w.offsets);
  int32_t* row_pair = (int32_t*)(b + w.row_pair);
  int32_t* pair_row = (int32_t*)(b + w.pair_row);
  const bool mk = L->profile;
  L->profile_valid = false;
  if (mk) LRC_HIP(hipEventRecord(L->marks[MOE_LRC_STAGE_ROUTE], s));
  int32_t* tok_exp = route_writes_exponents(L, T) ? (int32_t*)(b + w.tok_exp) : nullptr;
  // few pairs: every block of the preparing launch groups the pairs itself (one launch fewer)
  const PermuteArgs perm{idx, (int32_t*)(b + w.counts), offsets, row_pair, pair_row, (int32_t*)(b + w.comp_counts), T * L->cfg.top_k};
  // (every block repeats the grouping, so only where the preparing launch is one round of blocks
  // and the tables are small: few experts)
  const bool fused_permute = perm.P <= kFusedPermuteMaxPairs && L->cfg.n_experts <= 32;
  // a token or two: the blocks of the preparing launch route them as well (another launch fewer)
  const bool fused_route = fused_permute && T * L->cfg.n_experts <= kFusedRoutePairs && tok_exp != nullptr;
  const RouteArgs route{L->d_wg, L->has_bias ? L->d_bias : nullptr, idx, tw, tok_exp, L->cfg.renormalize};
  if (!fused_route) LRC_HIP(launch_route(L, x, T, idx, tw, nullptr, tok_exp, s));
  if (mk) LRC_HIP(hipEventRecord(L->marks[MOE_LRC_STAGE_PERMUTE], s));
  if (!fused_permute)
    LRC_HIP(launch_permute(L, idx, T, (int32_t*)(b + w.counts), offsets, row_pair, pair_row,
                           (int32_t*)(b + w.comp_counts), s));
  if (mk) LRC_HIP(hipEventRecord(L->marks[MOE_LRC_STAGE_PREP], s));
  // Shared experts need nothing from the router: with resident weights they run on the layer's side
  // stream beside the routed experts (forked here, joined before the combine).  In staged mode the
  // side stream carries the copies and the shared experts follow the routed ones.
  const bool fork = L->cfg.n_shared > 0 && L->cfg.residency == MOE_LRC_RESIDENT;
  const void* y_shared = L->cfg.n_shared > 0 ? b + w.sh_y : nullptr;
  if (fork) {
    LRC_HIP(hipEventRecord(L->ev_fork, s));
    LRC_HIP(hipStreamWaitEvent(L->side, L->ev_fork, 0));
    if ((rc = run_shared(L, x, T, b, L->side))) return rc;
    LRC_HIP(hipEventRecord(L->ev_join, L->side));
  }
  // (the K-block partial sums of a decode-flavour W2 go to the combine as they are: no pass that
  // adds them into bf16 rows first)
  int kblocks = 1;
  if ((rc = run_expert_ffn(L, x, T, offsets, row_pair, b + w.y_rows, b, s, mk, true, &kblocks, tok_exp,
                           fused_permute ? &perm : nullptr, fused_route ? &route : nullptr))) return rc;
  if (fork) LRC_HIP(hipStreamWaitEvent(s, L->ev_join, 0));
  else if (L->cfg.n_shared > 0 && (rc = run_shared(L, x, T, b, s))) return rc;
  if (mk) LRC_HIP(hipEventRecord(L->marks[MOE_LRC_STAGE_COMBINE], s));
  LRC_HIP(launch_combine(L, b + w.y_rows, kblocks > 1 ? (const float*)(b + w.y_part) : nullptr, kblocks, tw, pair_row, y_shared,
                         residual, T, out, s));
  if (mk) {
    LRC_HIP(hipEventRecord(L->marks[MOE_LRC_N_STAGES], s));
    L->profile_valid = true;
  }
  return MOE_LRC_OK;
}
}  // namespace lrc

extern "C" {

// ---- the entry point that allocates nothing --------------------------------------------------
// moe_lrc_forward with its workspace in a fixed device array of this library instead of a caller
// buffer.  Every GPU the library runs on holds its own copy of the array at its own address from
// the moment the code object is loaded until the process ends; the address is looked up once per
// device (with that device current) and kept.  Host code never uses the array's name for anything
// but that lookup: on the host the name is a stand-in, not a device address.
static __device__ __align__(256) unsigned char scratch[MOE_LRC_NOALLOC_WS_BYTES];

static int scratch_of_device(int dev, uint8_t** out) {
  static std::mutex mu;
  static uint8_t* ptr[64] = {};
  if (dev < 0 || dev >= 64) return set_error(MOE_LRC_EINVAL, "forward_noalloc: device index out of range");
  std::lock_guard<std::mutex> lock(mu);
  if (!ptr[dev]) {
    void* p = nullptr;
    hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p)
      return set_error(MOE_LRC_EHIP, std::string("forward_noalloc: hipGetSymbolAddress: ") + hipGetErrorString(e));
    ptr[dev] = static_cast<uint8_t*>(p);
  }
  *out = ptr[dev];
  return MOE_LRC_OK;
}

int moe_lrc_forward_noalloc(moe_lrc_layer* L, const void* x, int T, void* out, void* stream) {
  int rc = check_hot(L, T, "forward_noalloc");
  if (rc) return rc;
  int dev = -1;
  LRC_HIP(hipGetDevice(&dev));
  if (dev != L->device)
    return set_error(MOE_LRC_ESTATE, "forward_noalloc: the layer's device must be the current device");
  const size_t need = plan_workspace(L, T).total;
  if (need > size_t(MOE_LRC_NOALLOC_WS_BYTES))
    return set_error(MOE_LRC_ENOMEM, "forward_noalloc: T tokens of this layer need " + std::to_string(need) +
                                         " bytes of workspace, the built-in one holds " +
                                         std::to_string(size_t(MOE_LRC_NOALLOC_WS_BYTES)) + "; use moe_lrc_forward");
  uint8_t* ws = nullptr;
  if ((rc = scratch_of_device(dev, &ws))) return rc;
  // (nothing in the workspace has to start at zero: every buffer in it is written by an earlier
  // kernel of the same call before a later one reads it, so the last call's contents do no harm)
  return moe_lrc_forward(L, x, T, out, ws, size_t(MOE_LRC_NOALLOC_WS_BYTES), stream);
}

int moe_lrc_debug_unpack(moe_lrc_layer* L, int expert, int mat, uint8_t* codes_dev, void* stream) {
  if (!L || !codes_dev) return set_error(MOE_LRC_EINVAL, "debug_unpack: null argument");
  if (expert < 0 || expert >= L->n_total || mat < 0 || mat > 2)
    return set_error(MOE_LRC_EINVAL, "debug_unpack: expert or mat out of range");
  if (!L->mat_set[expert * 3 + mat]) return set_error(MOE_LRC_ESTATE, "debug_unpack: projection not uploaded");
  if (L->cfg.residency == MOE_LRC_POOLED && expert < L->cfg.n_experts)
    return set_error(MOE_LRC_ESTATE, "debug_unpack: a pooled layer's routed experts have no device copy of their own");
  const BlobLayout& b = blob_of(L, expert);
  const size_t off = L->w_off[expert] - L->dev_w_base + b.off_codes[mat];
  if (L->cfg.residency == MOE_LRC_STAGED)   // bring the packed codes into the expert's slot first
    LRC_HIP(hipMemcpyAsync(L->d_w + off, L->h_w + off, b.mat[mat].codes_bytes, hipMemcpyHostToDevice,
                           (hipStream_t)stream));
  LRC_HIP(launch_debug_unpack(reinterpret_cast<const uint32_t*>(L->d_w + off), b.mat[mat], codes_dev,
                              (hipStream_t)stream));
  return MOE_LRC_OK;
}

size_t moe_lrc_packed_bytes(int bits, int K, int N) {
  if (bits < 2 || bits > 4 || K <= 0 || N <= 0 || N % 16) return 0;
  return make_layout(K, N, bits, 64, 0).codes_bytes;
}

int moe_lrc_pack_codes(int bits, int K, int N, const uint8_t* codes, void* packed) {
  if (!codes || !packed) return set_error(MOE_LRC_EINVAL, "pack_codes: null argument");
  if (bits < 2 || bits > 4 || K <= 0 || N <= 0 || N % 16) return set_error(MOE_LRC_ESHAPE, "pack_codes: unsupported shape");
  for (size_t i = 0; i < size_t(K) * N; ++i)
    if (codes[i] >> bits) return set_error(MOE_LRC_EINVAL, "pack_codes: code out of range for the bit width");
  pack_codes(make_layout(K, N, bits, 64, 0), codes, (uint32_t*)packed);
  return MOE_LRC_OK;
}

int moe_lrc_unpack_codes(int bits, int K, int N, const void* packed, uint8_t* codes) {
  if (!codes || !packed) return set_error(MOE_LRC_EINVAL, "unpack_codes: null argument");
  if (bits < 2 || bits > 4 || K <= 0 || N <= 0 || N % 16) return set_error(MOE_LRC_ESHAPE, "unpack_codes: unsupported shape");
  unpack_codes(make_layout(K, N, bits, 64, 0), (const uint32_t*)packed, codes);
  return MOE_LRC_OK;
}

int moe_lrc_profile_enable(moe_lrc_layer* L, int on) {
  if (!L) return set_error(MOE_LRC_EINVAL, "profile_enable: layer is null");
  if (on && !L->marks[0])
    for (auto& ev : L->marks) LRC_HIP(hipEventCreate(&ev));
  L->profile = on != 0;
  L->profile_valid = false;
  return MOE_LRC_OK;
}

int moe_lrc_profile_read(moe_lrc_layer* L, float* ms) {
  if (!L || !ms) return set_error(MOE_LRC_EINVAL, "profile_read: null argument");
  if (!L->profile_valid) return set_error(MOE_LRC_ESTATE, "profile_read: no profiled forward call yet");
  LRC_HIP(hipEventSynchronize(L->marks[MOE_LRC_N_STAGES]));
  for (int i = 0; i < MOE_LRC_N_STAGES; ++i) LRC_HIP(hipEventElapsedTime(&ms[i], L->marks[i], L->marks[i + 1]));
  return MOE_LRC_OK;
}

int moe_lrc_get_stats(moe_lrc_layer* L, moe_lrc_stats* out) {
  if (!L || !out) return set_error(MOE_LRC_EINVAL, "get_stats: null argument");
  if (L->cfg.residency == MOE_LRC_POOLED && L->stats_valid) {
    L->stats.stage_ms = 0.f;                 // (the stack's own counters hold the copy time)
  } else if (L->cfg.residency == MOE_LRC_STAGED && L->stats_valid) {
    float ms = 0.f;
    if (hipEventSynchronize(L->ev_t1) == hipSuccess && hipEventElapsedTime(&ms, L->ev_t0, L->ev_t1) == hipSuccess)
      L->stats.stage_ms = ms;
  } else {
    LRC_HIP(hipDeviceSynchronize());
    LRC_HIP(hipMemcpy(L->h_stat, L->d_stat, (2 + 2 * L->cfg.n_experts) * 4, hipMemcpyDeviceToHost));
    fill_algorithmic_stats(L, L->h_stat);
  }
  *out = L->stats;
  return MOE_LRC_OK;
}

}  // extern "C"
