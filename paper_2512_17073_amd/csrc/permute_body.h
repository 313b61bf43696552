// Grouping of the (token, slot) pairs by expert: the body of the permute kernel, also run by every
// block of the launch that prepares the activations when there are few pairs (no launch of its own
// then).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace lrc {

constexpr int kMaxExperts = 256;
constexpr int kPermWaves = 16;
struct PermuteLds {
  int32_t hist[kPermWaves][kMaxExperts];
  int32_t comp[kMaxExperts];
  int32_t total[kMaxExperts];
};

// One workgroup of 16 wavefronts (1024 threads).  Wavefront w owns a contiguous run of pair ids, so
// pair order (= token order) is kept by walking the run in order and ranking equal experts inside
// each 64-pair step with ballots; per-(wavefront, expert) counters in LDS carry the positions.
// Ends with every result written (by this block) but not yet fenced: callers that read them back
// follow with __syncthreads().
// (idx carries no __restrict__: the caller may have written it itself just before)
__device__ inline void permute_body(PermuteLds& L, const int32_t* idx, int P, int E, int top_k, int top_n,
                                    int32_t* __restrict__ counts, int32_t* __restrict__ offsets,
                                    int32_t* __restrict__ row_pair, int32_t* __restrict__ pair_row,
                                    int32_t* __restrict__ comp_counts) {
  auto& hist = L.hist;
  auto& comp = L.comp;
  auto& total = L.total;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  for (int i = threadIdx.x; i < kPermWaves * kMaxExperts; i += 1024) (&hist[0][0])[i] = 0;
  for (int i = threadIdx.x; i < kMaxExperts; i += 1024) comp[i] = 0;
  __syncthreads();

  const int per_wave = ((P + kPermWaves - 1) / kPermWaves + 63) / 64 * 64;
  const int begin = wave * per_wave, end = min(P, begin + per_wave);
  for (int i = begin + lane; i < end; i += 64) {
    const int e = min(max(idx[i], 0), E - 1);     // out-of-range ids cannot leave the LDS tables
    atomicAdd(&hist[wave][e], 1);
    if (i % top_k < top_n) atomicAdd(&comp[e], 1);
  }
  __syncthreads();

  if (threadIdx.x < E) {
    int run = 0;
    for (int wv = 0; wv < kPermWaves; ++wv) {
      const int c = hist[wv][threadIdx.x];
      hist[wv][threadIdx.x] = run;
      run += c;
    }
    total[threadIdx.x] = run;
    counts[threadIdx.x] = run;
    comp_counts[threadIdx.x] = comp[threadIdx.x];
  }
  __syncthreads();
  if (threadIdx.x < E) {
    int off = 0;
    for (int e = 0; e < (int)threadIdx.x; ++e) off += total[e];
    offsets[threadIdx.x] = off;
    if ((int)threadIdx.x == E - 1) offsets[E] = off + total[threadIdx.x];
    for (int wv = 0; wv < kPermWaves; ++wv) hist[wv][threadIdx.x] += off;
  }
  __syncthreads();

  int nbits = 0;
  while ((1 << nbits) < E) ++nbits;
  for (int base = begin; base < end; base += 64) {
    const int i = base + lane;
    const bool valid = i < end;
    const int e = valid ? min(max(idx[i], 0), E - 1) : 0;
    unsigned long long same = __ballot(valid);
    for (int b = 0; b < nbits; ++b) {
      const bool bit = (e >> b) & 1;
      const unsigned long long bb = __ballot(valid && bit);
      same &= bit ? bb : ~bb;
    }
    const int rank = __popcll(same & ((1ull << lane) - 1ull));
    const int cnt = __popcll(same);
    int pos = 0;
    if (valid) pos = hist[wave][e] + rank;
    __builtin_amdgcn_wave_barrier();
    if (valid && rank == 0) hist[wave][e] = pos + cnt;
    __builtin_amdgcn_wave_barrier();
    if (valid) {
      row_pair[pos] = i;
      pair_row[i] = pos;
    }
  }
}

}  // namespace lrc
