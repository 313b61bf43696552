// A stack of MoE layers decoding from host-resident experts (Section 4.3, case study 1): a device
// slot pool shared by the layers and kept across steps, on-demand copies of what each layer's router
// selects (packed experts of activated pairs, factors of Top-n pairs only: Section 3.2), and copies
// ahead for the next layer on a guess of its routing while the current layer computes.
//
// Order of events for layer l (stream s = the caller's, c = the stack's copy stream):
//   s: route, permute, preparing launch of layer l; the gate of layer l+1 on layer l's input (the guess)
//   s: read back the per-expert counts and the guess, host waits                    (one per layer)
//   host: hits are pinned; every miss gets the least recently used slot that is not pinned
//   c: copies of the misses; event R;          s: waits for R, expert table of layer l -> device
//   c: copies ahead for layer l+1 (slots not pinned, not used by layer l)
//   s: FFN kernels, combine of layer l
// Every kernel of the layers before l has finished when the host chooses slots (the wait above
// follows them on s), so a copy never overwrites a slot a running kernel reads; the copies ahead
// spare the slots layer l is about to use.
#include <chrono>
#include <cstring>
#include <mutex>

#include "internal.h"

using namespace lrc;

struct moe_lrc_stack {
  struct Slot {
    int layer = -1, expert = -1;
    bool has_f = false;          // the expert's factor pair is in the slot too
    bool fresh = false;          // filled by a copy ahead and not used since
    uint64_t tick = 0;           // last use (0: never)
    uint64_t pin = 0;            // epoch in which the slot must stay
  };
  std::vector<moe_lrc_layer*> layers;
  int flags = 0, n_slots = 0, max_tokens = 0, hidden = 0, device = 0;
  size_t slot_w = 0, slot_f = 0;           // bytes of a slot's two parts
  uint8_t* d_pool = nullptr;
  std::vector<Slot> slots;
  std::vector<std::vector<int>> where;     // [layer][expert] -> slot or -1
  uint64_t tick = 0, epoch = 0;
  hipStream_t copy = nullptr;
  hipEvent_t ev_ready = nullptr, ev_c0 = nullptr, ev_c1 = nullptr;
  bool copied_this_step = false, c0_recorded = false;
  uint8_t* ws = nullptr;
  size_t ws_bytes = 0;
  uint8_t* xbuf[2] = {nullptr, nullptr};
  ExpertDesc* h_desc = nullptr;            // pinned, [layer][max E]: source of the asynchronous table uploads
  int max_e = 0;
  int32_t* d_guess_idx = nullptr;
  float* d_guess_w = nullptr;
  int32_t* h_guess = nullptr;              // pinned
  moe_lrc_stack_stats st{};
};

namespace {

uint8_t* slot_w_ptr(const moe_lrc_stack* S, int slot) { return S->d_pool + size_t(slot) * (S->slot_w + S->slot_f); }
uint8_t* slot_f_ptr(const moe_lrc_stack* S, int slot) { return slot_w_ptr(S, slot) + S->slot_w; }

// The slot to fill among those no need of this epoch holds: an empty one, else one filled ahead and
// never used, else the least recently used (lowest index on ties); -1 if every slot is pinned.
int pick_victim(moe_lrc_stack* S) {
  int best = -1;
  auto older = [&](const moe_lrc_stack::Slot& a, const moe_lrc_stack::Slot& b) {
    const bool ae = a.layer < 0, be = b.layer < 0;
    return ae != be ? ae : a.tick < b.tick;
  };
  for (int i = 0; i < S->n_slots; ++i) {
    const auto& sl = S->slots[i];
    if (sl.pin == S->epoch) continue;
    if (best < 0 || older(sl, S->slots[best])) best = i;
  }
  return best;
}

hipError_t note_copy(moe_lrc_stack* S) {
  if (!S->c0_recorded) {
    hipError_t e = hipEventRecord(S->ev_c0, S->copy);
    if (e != hipSuccess) return e;
    S->c0_recorded = true;
  }
  S->copied_this_step = true;
  return hipSuccess;
}

// brings (layer li, expert e) into `slot` on the copy stream: the packed weights unless they are there, the factors if wanted
int fill_slot(moe_lrc_stack* S, int li, int e, int slot, bool weights, bool factors) {
  moe_lrc_layer* L = S->layers[li];
  const BlobLayout& b = L->routed;
  if (weights) {
    LRC_HIP(note_copy(S));
    LRC_HIP(hipMemcpyAsync(slot_w_ptr(S, slot), L->h_w + L->w_off[e], b.w_bytes, hipMemcpyHostToDevice, S->copy));
    S->st.bytes_h2d += b.w_bytes;
  }
  if (factors && b.f_bytes) {
    LRC_HIP(note_copy(S));
    const uint8_t* q3 = &L->mat_q3[e * 3];
    if (q3[0] | q3[1] | q3[2]) {             // pairs held at 3 bits fill a part of their sections only
      for (int mat = 0; mat < 3; ++mat) {
        size_t ab, bb;
        factor_section_bytes(L, e, mat, ab, bb);
        if (ab) LRC_HIP(hipMemcpyAsync(slot_f_ptr(S, slot) + b.off_af[mat], L->h_f + L->f_off[e] + b.off_af[mat], ab, hipMemcpyHostToDevice, S->copy));
        if (bb) LRC_HIP(hipMemcpyAsync(slot_f_ptr(S, slot) + b.off_bf[mat], L->h_f + L->f_off[e] + b.off_bf[mat], bb, hipMemcpyHostToDevice, S->copy));
        S->st.bytes_h2d += ab + bb;
      }
    } else {
      LRC_HIP(hipMemcpyAsync(slot_f_ptr(S, slot), L->h_f + L->f_off[e], b.f_bytes, hipMemcpyHostToDevice, S->copy));
      S->st.bytes_h2d += b.f_bytes;
    }
    S->st.factor_copies++;
    S->slots[slot].has_f = true;
  }
  return MOE_LRC_OK;
}

void evict(moe_lrc_stack* S, int slot) {
  auto& sl = S->slots[slot];
  if (sl.layer >= 0) S->where[sl.layer][sl.expert] = -1;
  sl = moe_lrc_stack::Slot{};
}

}  // namespace

namespace lrc {

int pool_stage(moe_lrc_layer* L, const void* x, int T, hipStream_t s) {
  moe_lrc_stack* S = L->pool;
  if (!S) return set_error(MOE_LRC_ESTATE, "a pooled layer runs through moe_lrc_stack_step only");
  const moe_lrc_config& c = L->cfg;
  const int E = c.n_experts, li = L->pool_index;
  moe_lrc_layer* next = ((S->flags & MOE_LRC_STACK_PREFETCH) && li + 1 < (int)S->layers.size()) ? S->layers[li + 1] : nullptr;
  if (next) LRC_HIP(launch_route(next, x, T, S->d_guess_idx, S->d_guess_w, nullptr, nullptr, s));
  LRC_HIP(hipMemcpyAsync(L->h_stat, L->d_stat, (2 + 2 * E) * 4, hipMemcpyDeviceToHost, s));
  if (next) LRC_HIP(hipMemcpyAsync(S->h_guess, S->d_guess_idx, size_t(T) * next->cfg.top_k * 4, hipMemcpyDeviceToHost, s));
  LRC_HIP(hipStreamSynchronize(s));
  fill_algorithmic_stats(L, L->h_stat);
  const int32_t* rows = L->h_stat + 2;
  const int32_t* comp = L->h_stat + 2 + E;
  const bool factors_used = c.rank > 0 && c.top_n > 0 && L->routed.f_bytes > 0;

  // ---- this layer's needs: hits first (they pin their slots), then a slot for every miss
  ++S->epoch;
  for (int e = 0; e < E; ++e) {
    if (rows[e] <= 0) continue;
    S->st.expert_uses++;
    const int slot = S->where[li][e];
    if (slot < 0) continue;
    auto& sl = S->slots[slot];
    sl.pin = S->epoch; sl.tick = ++S->tick;
    S->st.hits++;
    if (sl.fresh) { S->st.prefetch_hits++; sl.fresh = false; }
  }
  for (int e = 0; e < E; ++e) {
    if (rows[e] <= 0) continue;
    int slot = S->where[li][e];
    const bool miss = slot < 0;
    if (miss) {
      slot = pick_victim(S);
      if (slot < 0) return set_error(MOE_LRC_ENOMEM, "stack_step: fewer slots than one layer's active experts");
      evict(S, slot);
      auto& sl = S->slots[slot];
      sl.layer = li; sl.expert = e; sl.pin = S->epoch; sl.tick = ++S->tick;
      S->where[li][e] = slot;
      S->st.misses++;
    }
    const bool want_f = factors_used && comp[e] > 0 && !S->slots[slot].has_f;
    const int rc = fill_slot(S, li, e, slot, miss, want_f);
    if (rc) return rc;
  }
  LRC_HIP(hipEventRecord(S->ev_ready, S->copy));
  LRC_HIP(hipStreamWaitEvent(s, S->ev_ready, 0));

  // ---- the layer's expert table: experts with rows point into their slots (the others, which no
  //      kernel touches, at slot 0)
  ExpertDesc* hd = S->h_desc + size_t(li) * S->max_e;
  for (int e = 0; e < E; ++e) {
    ExpertDesc d = L->h_desc[e];
    const int slot = S->where[li][e] >= 0 ? S->where[li][e] : 0;
    const BlobLayout& b = L->routed;
    for (int m = 0; m < 3; ++m) {
      d.codes[m] = reinterpret_cast<const uint32_t*>(slot_w_ptr(S, slot) + b.off_codes[m]);
      d.meta[m] = reinterpret_cast<const uint32_t*>(slot_w_ptr(S, slot) + b.off_meta[m]);
      d.af[m] = d.bf[m] = nullptr;
      if (b.f_bytes) set_factor_ptrs(L, e, m, d, slot_f_ptr(S, slot) + b.off_af[m], slot_f_ptr(S, slot) + b.off_bf[m]);
    }
    hd[e] = d;
  }
  LRC_HIP(hipMemcpyAsync(L->d_desc, hd, sizeof(ExpertDesc) * E, hipMemcpyHostToDevice, s));

  // ---- copies ahead for the next layer, into slots this layer does not use
  if (next) {
    const moe_lrc_config& nc = next->cfg;
    const bool nf = nc.rank > 0 && nc.top_n > 0 && next->routed.f_bytes > 0;
    std::vector<uint8_t> want(nc.n_experts, 0);       // bit 0: weights, bit 1: factors
    for (int t = 0; t < T; ++t)
      for (int j = 0; j < nc.top_k; ++j) {
        const int e = S->h_guess[t * nc.top_k + j];
        if (e < 0 || e >= nc.n_experts) continue;
        want[e] |= 1 | ((nf && j < nc.top_n) ? 2 : 0);
      }
    for (int e = 0; e < nc.n_experts; ++e) {
      if (!want[e]) continue;
      int slot = S->where[li + 1][e];
      const bool absent = slot < 0;
      if (absent) {
        slot = pick_victim(S);
        if (slot < 0) break;                           // every slot is spoken for
        evict(S, slot);
        auto& sl = S->slots[slot];
        // (least recently used until its layer really uses it: a wrong guess is the first to go)
        sl.layer = li + 1; sl.expert = e; sl.fresh = true; sl.tick = 0;
        S->where[li + 1][e] = slot;
        S->st.prefetched++;
      }
      S->slots[slot].pin = S->epoch;                   // (a later copy ahead of this layer must not take it)
      const int rc = fill_slot(S, li + 1, e, slot, absent, (want[e] & 2) && !S->slots[slot].has_f);
      if (rc) return rc;
    }
  }
  return MOE_LRC_OK;
}

}  // namespace lrc

extern "C" {

int moe_lrc_stack_destroy(moe_lrc_stack* S) {
  if (!S) return MOE_LRC_OK;
  (void)hipDeviceSynchronize();
  for (auto* L : S->layers)
    if (L && L->pool == S) { L->pool = nullptr; L->pool_index = -1; }
  if (S->d_pool) (void)hipFree(S->d_pool);
  if (S->ws) (void)hipFree(S->ws);
  if (S->xbuf[0]) (void)hipFree(S->xbuf[0]);
  if (S->xbuf[1]) (void)hipFree(S->xbuf[1]);
  if (S->d_guess_idx) (void)hipFree(S->d_guess_idx);
  if (S->d_guess_w) (void)hipFree(S->d_guess_w);
  if (S->h_desc) (void)hipHostFree(S->h_desc);
  if (S->h_guess) (void)hipHostFree(S->h_guess);
  if (S->copy) (void)hipStreamDestroy(S->copy);
  if (S->ev_ready) (void)hipEventDestroy(S->ev_ready);
  if (S->ev_c0) (void)hipEventDestroy(S->ev_c0);
  if (S->ev_c1) (void)hipEventDestroy(S->ev_c1);
  delete S;
  return MOE_LRC_OK;
}

int moe_lrc_stack_create(moe_lrc_layer* const* layers, int n_layers, int slots, int flags, moe_lrc_stack** out) {
  if (!layers || !out) return set_error(MOE_LRC_EINVAL, "stack_create: null argument");
  if (n_layers < 1 || n_layers > 1024) return set_error(MOE_LRC_EINVAL, "stack_create: n_layers outside 1..1024");
  if (flags & ~(MOE_LRC_STACK_PREFETCH | MOE_LRC_STACK_RESIDUAL)) return set_error(MOE_LRC_EINVAL, "stack_create: unknown flag");
  int dev = 0;
  LRC_HIP(hipGetDevice(&dev));
  size_t slot_w = 0, slot_f = 0, ws_bytes = 0;
  int need = 0, max_e = 0, max_k = 0;
  for (int i = 0; i < n_layers; ++i) {
    const moe_lrc_layer* L = layers[i];
    if (!L) return set_error(MOE_LRC_EINVAL, "stack_create: null layer");
    if (L->cfg.residency != MOE_LRC_POOLED) return set_error(MOE_LRC_EINVAL, "stack_create: layers must have residency MOE_LRC_POOLED");
    if (L->pool) return set_error(MOE_LRC_ESTATE, "stack_create: a layer already belongs to a stack");
    if (L->device != dev) return set_error(MOE_LRC_ESTATE, "stack_create: a layer lives on another device");
    if (L->cfg.hidden != layers[0]->cfg.hidden || L->cfg.max_tokens != layers[0]->cfg.max_tokens)
      return set_error(MOE_LRC_ESHAPE, "stack_create: layers differ in hidden size or max_tokens");
    for (int j = 0; j < i; ++j)
      if (layers[j] == L) return set_error(MOE_LRC_EINVAL, "stack_create: a layer is listed twice");
    slot_w = std::max(slot_w, (L->routed.w_bytes + 255) & ~size_t(255));
    slot_f = std::max(slot_f, (L->routed.f_bytes + 255) & ~size_t(255));
    ws_bytes = std::max(ws_bytes, moe_lrc_workspace_bytes(L, L->cfg.max_tokens));
    const long long pairs = (long long)L->cfg.max_tokens * L->cfg.top_k;
    need = std::max(need, (int)std::min<long long>(L->cfg.n_experts, pairs));
    max_e = std::max(max_e, L->cfg.n_experts);
    max_k = std::max(max_k, L->cfg.top_k);
  }
  if (slots < need || slots > (1 << 20))
    return set_error(MOE_LRC_EINVAL, "stack_create: slots must be at least min(n_experts, max_tokens * top_k) of the widest layer");
  moe_lrc_stack* S = new (std::nothrow) moe_lrc_stack();
  if (!S) return set_error(MOE_LRC_ENOMEM, "stack_create: out of host memory");
  S->flags = flags; S->n_slots = slots; S->device = dev;
  S->max_tokens = layers[0]->cfg.max_tokens; S->hidden = layers[0]->cfg.hidden;
  S->slot_w = slot_w; S->slot_f = slot_f; S->ws_bytes = ws_bytes; S->max_e = max_e;
  S->slots.resize(slots);
  S->where.resize(n_layers);
  for (int i = 0; i < n_layers; ++i) S->where[i].assign(layers[i]->cfg.n_experts, -1);
  auto fail = [&](int code) { moe_lrc_stack_destroy(S); return code; };
#define STK_TRY(expr)                                                                             \
  do {                                                                                            \
    hipError_t e_ = (expr);                                                                       \
    if (e_ != hipSuccess)                                                                         \
      return fail(set_error(e_ == hipErrorOutOfMemory ? MOE_LRC_ENOMEM : MOE_LRC_EHIP,            \
                            std::string("stack_create: ") + #expr + ": " + hipGetErrorString(e_))); \
  } while (0)
  const size_t xbytes = std::max<size_t>(size_t(S->max_tokens) * S->hidden * 2, 256);
  STK_TRY(hipMalloc((void**)&S->d_pool, size_t(slots) * (slot_w + slot_f)));
  STK_TRY(hipMalloc((void**)&S->ws, std::max<size_t>(ws_bytes, 256)));
  STK_TRY(hipMalloc((void**)&S->xbuf[0], xbytes));
  STK_TRY(hipMalloc((void**)&S->xbuf[1], xbytes));
  STK_TRY(hipMalloc((void**)&S->d_guess_idx, std::max<size_t>(size_t(S->max_tokens) * max_k * 4, 256)));
  STK_TRY(hipMalloc((void**)&S->d_guess_w, std::max<size_t>(size_t(S->max_tokens) * max_k * 4, 256)));
  STK_TRY(hipHostMalloc((void**)&S->h_desc, sizeof(ExpertDesc) * size_t(n_layers) * max_e, hipHostMallocDefault));
  STK_TRY(hipHostMalloc((void**)&S->h_guess, std::max<size_t>(size_t(S->max_tokens) * max_k * 4, 256), hipHostMallocDefault));
  STK_TRY(hipStreamCreateWithFlags(&S->copy, hipStreamNonBlocking));
  STK_TRY(hipEventCreateWithFlags(&S->ev_ready, hipEventDisableTiming));
  STK_TRY(hipEventCreate(&S->ev_c0));
  STK_TRY(hipEventCreate(&S->ev_c1));
#undef STK_TRY
  for (int i = 0; i < n_layers; ++i) {
    S->layers.push_back(layers[i]);
    layers[i]->pool = S;
    layers[i]->pool_index = i;
  }
  *out = S;
  return MOE_LRC_OK;
}

int moe_lrc_stack_reset(moe_lrc_stack* S) {
  if (!S) return set_error(MOE_LRC_EINVAL, "stack_reset: stack is null");
  LRC_HIP(hipStreamSynchronize(S->copy));
  for (auto& sl : S->slots) sl = moe_lrc_stack::Slot{};
  for (auto& w : S->where) std::fill(w.begin(), w.end(), -1);
  S->tick = 0; S->epoch = 0;
  S->st = moe_lrc_stack_stats{};
  S->copied_this_step = false;
  return MOE_LRC_OK;
}

int moe_lrc_stack_step(moe_lrc_stack* S, const void* x, int T, void* out, void* layer_inputs, void* stream) {
  if (!S) return set_error(MOE_LRC_EINVAL, "stack_step: null argument");
  if (T < 0 || T > S->max_tokens) return set_error(MOE_LRC_ESTATE, "stack_step: T outside 0..max_tokens");
  int dev = 0;
  LRC_HIP(hipGetDevice(&dev));
  if (dev != S->device) return set_error(MOE_LRC_ESTATE, "stack_step: the stack lives on another device");
  for (auto* L : S->layers) {
    if (!L->gate_set) return set_error(MOE_LRC_ESTATE, "stack_step: a layer's gate is not uploaded");
    for (size_t i = 0; i < L->mat_set.size(); ++i)
      if (!L->mat_set[i]) return set_error(MOE_LRC_ESTATE, "stack_step: an expert projection is not uploaded");
  }
  if (T == 0) return MOE_LRC_OK;                 // (an empty batch: the per-token buffers may be null)
  if (!x || !out) return set_error(MOE_LRC_EINVAL, "stack_step: null argument");
  hipStream_t s = (hipStream_t)stream;
  const auto t0 = std::chrono::steady_clock::now();
  S->c0_recorded = false;
  S->copied_this_step = false;
  const size_t xbytes = size_t(T) * S->hidden * 2;
  const void* cur = x;
  const int n = (int)S->layers.size();
  for (int li = 0; li < n; ++li) {
    void* dst = li == n - 1 ? out : S->xbuf[li & 1];
    if (layer_inputs)
      LRC_HIP(hipMemcpyAsync((uint8_t*)layer_inputs + size_t(li) * xbytes, cur, xbytes, hipMemcpyDeviceToDevice, s));
    const int rc = forward_impl(S->layers[li], cur, T, dst, S->ws, s, (S->flags & MOE_LRC_STACK_RESIDUAL) ? cur : nullptr);
    if (rc) return rc;
    cur = dst;
  }
  if (S->copied_this_step) LRC_HIP(hipEventRecord(S->ev_c1, S->copy));
  S->st.steps++;
  S->st.last_step_ms = std::chrono::duration<float, std::milli>(std::chrono::steady_clock::now() - t0).count();
  return MOE_LRC_OK;
}

int moe_lrc_stack_get_stats(moe_lrc_stack* S, moe_lrc_stack_stats* out) {
  if (!S || !out) return set_error(MOE_LRC_EINVAL, "stack_get_stats: null argument");
  S->st.last_copy_ms = 0.f;
  if (S->copied_this_step) {
    float ms = 0.f;
    if (hipEventSynchronize(S->ev_c1) == hipSuccess && hipEventElapsedTime(&ms, S->ev_c0, S->ev_c1) == hipSuccess)
      S->st.last_copy_ms = ms;
  }
  *out = S->st;
  return MOE_LRC_OK;
}

}  // extern "C"
