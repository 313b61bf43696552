// Shared device helpers and argument block of the expert-FFN kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "internal.h"
#include "unpack.h"

namespace lrc {
namespace ffn {

typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef float float4_t __attribute__((ext_vector_type(4)));

__device__ inline uint32_t pk_fma(uint32_t q, uint32_t s, uint32_t c) {
  const half2_t r = __builtin_elementwise_fma(__builtin_bit_cast(half2_t, q),
                                              __builtin_bit_cast(half2_t, s),
                                              __builtin_bit_cast(half2_t, c));
  return __builtin_bit_cast(uint32_t, r);
}
__device__ inline uint32_t pk_mul(uint32_t a, uint32_t b) {
  const half2_t r = __builtin_bit_cast(half2_t, a) * __builtin_bit_cast(half2_t, b);
  return __builtin_bit_cast(uint32_t, r);
}

struct KArgs {
  const ExpertDesc* desc;
  const int32_t* offsets;    // null: shared experts, expert e owns rows e*T .. e*T+T-1
  const int32_t* row_pair;   // null: rows are tokens
  const int32_t* comp_rows;  // per expert: rows that take the rank-r term (an expert with none skips it:
                             // in staged residency its factors were not brought in)
  const _Float16* in;        // activations in operand order (act_unit), in_rt rows: gathered x, or h
  void* out;                 // DUAL: h in operand order (out_rt rows); else y_rows [rows][N] bf16
  int in_rt, out_rt;         // row counts (incl. padding) of the operand-order buffers
  const float* p;            // (in A): fp16 [total_rows][projections * ls * 32], scaled by the projections' pre-scales,
                             // zero for rows without the rank-r term (written by the (in A) kernels)
  int K, N, KS, G, NT, group_shift, top_k, top_n, T, rank, rpad, total_rows;
  int ls;                    // rank steps of 32 of the B factor: ceil(rank / 32)
  int n_exp;                 // experts of this launch (many-rows flavour: the grid enumerates row chunks)
  int kb_steps;              // decode flavour: k-steps per K-block (grid.z blocks split K; KS if one)
  float* partial;            // decode flavour, more than one K-block: fp32 partial outputs [kb][rows][N]
  const int32_t* plan;       // decode flavour: null (grid = blocks per expert x experts), or the block table
                             // (PlanEntry per block, plan.h)
  const int32_t* row_exp;    // per input row: the exponent s of its power-of-two pre-scale (row_exponent below);
                             // routed launches: one per routed row; shared experts: one per token
  const int32_t* tok_exp;    // the same per token, where a kernel reads the bf16 tokens itself (or null)
  const int32_t* row_list;   // grouped (in A) kernel: an expert's rows are the first comp_rows[e] of its range, the
                             // compact rows of the pairs that take the rank-r term; row_list names the routed row
                             // of each (CompactArgs); null: the rows are the routed rows
};

// Range of the fp16 operands.  The activations cross the ABI as bf16 (8 exponent bits); the matrix
// cores take fp16 (5).  Every input row is therefore multiplied by 2^s, s chosen so that its largest
// magnitude lands in [1, 2) (exact: a power of two), the fused projection's fp32 results are
// multiplied by 2^-s before the SwiGLU, its output h (at most quadratic in the scale, since
// |silu(g)| <= |g|) is stored times 2^(2s), and the down projection's fp32 results are multiplied
// by 2^(-2s).  s is clamped to +-60, which covers inputs from 2^-60 to 2^60.
__device__ inline float pow2i(int k) { return __uint_as_float(uint32_t(127 + k) << 23); }   // 2^k, -126 <= k <= 127
// from the largest (bits & 0x7fff) over a row of bf16 values
__device__ inline int row_exponent(uint32_t max_abs_bits) {
  const int e = int(max_abs_bits >> 7);          // biased exponent of the largest magnitude (0: zero or subnormal)
  return e == 0 ? 0 : min(60, max(-60, 127 - e));
}
// fp32 -> fp16 that saturates at the largest finite value instead of giving infinity
__device__ inline _Float16 to_f16_sat(float v) { return (_Float16)__builtin_fminf(__builtin_fmaxf(v, -65504.f), 65504.f); }

__device__ inline uint32_t f32x2_to_bf16x2(float a, float b) {
  uint32_t ua = __float_as_uint(a), ub = __float_as_uint(b);
  ua += 0x7fffu + ((ua >> 16) & 1u);
  ub += 0x7fffu + ((ub >> 16) & 1u);
  return (ua >> 16) | (ub & 0xffff0000u);
}


// Operand-order activations: the 8 consecutive elements k8*8 .. k8*8+7 of row R form one 16-byte
// unit at index ((ks*8 + s)*4 + q) * rt + R, where k8 = ks*32 + q*8 + s.  For a fixed (ks, s, q) the
// rows are contiguous, so the 16 rows x 4 q of one MFMA B-operand fragment are four 256-byte runs
// and staging a fragment into LDS is a lane-linear copy.
__host__ __device__ inline size_t act_unit(int k8, int R, int rt) {
  const int ks = k8 >> 5, q = (k8 >> 3) & 3, s = k8 & 7;
  return size_t((ks * 8 + s) * 4 + q) * rt + R;
}

// LDS read of one 16-byte unit per lane whose result is awaited by lds_wait, not by the compiler
// (which would move each read down to its use).
template <int OFF> __device__ inline half8_t lds_read16(uint32_t addr) {
  half8_t v;
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF));
  return v;
}
// Waits until at most N LDS operations issued after the wanted ones are outstanding (LDS returns in
// order), and ties the wanted registers to the wait so that their uses stay behind it.
template <int N> __device__ inline void lds_wait(half8_t& a) { asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(a) : "n"(N)); }
template <int N> __device__ inline void lds_wait(half8_t& a, half8_t& b) {
  asm volatile("s_waitcnt lgkmcnt(%2)" : "+v"(a), "+v"(b) : "n"(N));
}

// A pointer read from memory, moved into scalar registers (a buffer resource must be wave-uniform).
template <class T> __device__ inline const T* uniform_ptr(const T* p) {
  const uint64_t v = reinterpret_cast<uint64_t>(p);
  const uint32_t lo = __builtin_amdgcn_readfirstlane(uint32_t(v)), hi = __builtin_amdgcn_readfirstlane(uint32_t(v >> 32));
  return reinterpret_cast<const T*>((uint64_t(hi) << 32) | lo);
}

// Codes and metadata of one k-step of one wavefront (both projections when DUAL), in registers.
template <int BITS, int NM> struct Slot {
  uint32_t cw[NM][2 * BITS];
  uint32_t mw[NM];
};

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

}  // namespace ffn

// decode flavour (ffn_decode.hip): few rows per expert, one 16-wavefront block per CU.
// which: bit 0 = the fused W1|W3 projection (with its (x A) kernel), bit 1 = W2 (with its (h A) kernel)
hipError_t launch_decode_ffn(const FfnArgs& f, hipStream_t s, int which);
// the block tables (plan.h) a decode launch of the projections in `which` reads
void decode_plan_specs(const FfnArgs& f, int which, PlanSpec& p13, PlanSpec& p2);

}  // namespace lrc
