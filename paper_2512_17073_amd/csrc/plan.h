// Sharing a decode launch's blocks out among the experts that have rows.
//
// With a fixed number of blocks per expert, experts without rows leave CUs idle and experts with
// several 32-row passes finish last.  One wavefront (part of the launch that prepares the
// activations) writes, for every block of the later launch, which expert it serves: each expert with
// rows gets `base` blocks (enough for 32 n-tiles per block), the rest of `target` blocks go by
// weight (the number of 32-row passes the expert's rows need: every pass streams its weights
// again), dealt by the running sum of the weights.  Entry i of the table (PlanEntry, 32 bytes, read by block i with one scalar
// load): expert (or -1: the block exits), index of the block within the expert, blocks of the expert,
// first row and number of rows of the expert.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace lrc {

struct PlanSpec { int B, NT, target; int32_t* plan; };     // B entries for a projection of NT n-tiles; plan == null: no table wanted
struct PlanEntry { int32_t e, b, G, r0, cnt, pad0, pad1, pad2; };
constexpr int kPlanEntryInts = 8;

__device__ inline void make_plan(const int32_t* __restrict__ offsets, int E, const PlanSpec sp, int lane) {
  if (sp.plan == nullptr) return;
  const int B = sp.B, target = sp.target;
  int32_t* __restrict__ plan = sp.plan;
  // what an expert's rows cost: every 32-row pass streams the expert's weights again
  auto weight = [](int cnt) { return (cnt + 31) / 32; };
  // fewest blocks an expert needs: a block owns at most 32 n-tiles
  auto base_of = [&](int cnt) { return cnt == 0 ? 0 : (sp.NT + 31) / 32; };
  auto scan = [&](int v) {
#pragma unroll
    for (int dlt = 1; dlt < 64; dlt *= 2) {
      const int t = __shfl_up(v, dlt);
      if (lane >= dlt) v += t;
    }
    return v;
  };
  int n_active = 0, wsum = 0, base_sum = 0;
  for (int e0 = 0; e0 < E; e0 += 64) {
    const int e = e0 + lane;
    const int cnt = e < E ? offsets[e + 1] - offsets[e] : 0;
    n_active += __popcll(__ballot(cnt > 0));
    wsum += __shfl(scan(weight(cnt)), 63);
    base_sum += __shfl(scan(base_of(cnt)), 63);
  }
  // as many blocks as fill the chip (`target`), more only if the experts with rows need them; the
  // rest of the grid exits at once.  Every expert gets its fewest blocks or its share by weight of
  // all the blocks, whichever is more (the shares by weight are then scaled down to what is left).
  const int total = min(B, max(target, base_sum));
  int over = 0;                                  // sum over experts of max(0, share by weight - fewest)
  for (int e0 = 0; e0 < E; e0 += 64) {
    const int e = e0 + lane;
    const int cnt = e < E ? offsets[e + 1] - offsets[e] : 0;
    const int want = wsum > 0 ? int((long long)total * weight(cnt) / wsum) : 0;
    over += __shfl(scan(max(0, want - base_of(cnt))), 63);
  }
  const long long extra = total - base_sum;
  int act_before = 0, w_before = 0, b_before = 0;
  for (int e0 = 0; e0 < E; e0 += 64) {
    const int e = e0 + lane;
    const int cnt = e < E ? offsets[e + 1] - offsets[e] : 0;
    const int r0 = e < E ? offsets[e] : 0;
    const int act = cnt > 0 ? 1 : 0, ai = scan(act), base = base_of(cnt), bi = scan(base);
    // this expert's claim on the blocks beyond the fewest: what its share by weight exceeds them by
    const int want = wsum > 0 ? int((long long)total * weight(cnt) / wsum) : 0;
    const int w = max(0, want - base), wi = scan(w);
    int lo = 0, hi = 0;
    if (act) {
      lo = b_before + bi - base + (over > 0 ? int(extra * (w_before + wi - w) / over) : 0);
      hi = b_before + bi + (over > 0 ? int(extra * (w_before + wi) / over) : 0);
    }
    const unsigned long long with_rows = __ballot(act != 0);
    if (__popcll(with_rows) <= 8) {
      // few experts with many blocks each: the whole wavefront writes one expert's entries after the other's
      for (unsigned long long todo = with_rows; todo; todo &= todo - 1) {
        const int j = __ffsll(todo) - 1;
        const int lo_j = __shfl(lo, j), G_j = __shfl(hi, j) - lo_j, hi_j = min(lo_j + G_j, B);
        const int r0_j = __shfl(r0, j), cnt_j = __shfl(cnt, j);
        for (int i = lo_j + lane; i < hi_j; i += 64)
          reinterpret_cast<PlanEntry*>(plan)[i] = PlanEntry{e0 + j, i - lo_j, G_j, r0_j, cnt_j, 0, 0, 0};
      }
    } else if (act) {
      // many experts with few blocks each: every lane writes its own expert's entries
      for (int i = lo; i < hi && i < B; ++i) reinterpret_cast<PlanEntry*>(plan)[i] = PlanEntry{e, i - lo, hi - lo, r0, cnt, 0, 0, 0};
    }
    act_before += __shfl(ai, 63); w_before += __shfl(wi, 63); b_before += __shfl(bi, 63);
  }
  (void)act_before;
  const int used = n_active > 0 ? base_sum + (over > 0 ? int(extra) : 0) : 0;
  for (int i = used + lane; i < B; i += 64) reinterpret_cast<PlanEntry*>(plan)[i] = PlanEntry{-1, 0, 1, 0, 0, 0, 0, 0};
}

}  // namespace lrc
