/*
 * moe_lrc — one MoE layer's forward pass with router-guided low-rank compensation, for MI355X.
 *
 * The layer follows the paper's statement of the problem:
 *   routing        w = softmax(G(x)), the k highest-scored experts are activated     (Section 2.1)
 *   Top-n marking  the n < k highest-scored of those k take the compensator          (Section 3.2)
 *   expert weights W_hat_e = Qinv(Q(W_e)) + U_e V_e for a Top-n (token, expert) pair,
 *                  Qinv(Q(W_e)) for every other activated pair                       (Sections 2.3, 3.2)
 *   output         y = sum_{i in TopK} w_i E_i(x), plus always-on shared experts      (Section 2.1, Table 1)
 *   transfer       packed low-bit experts of every activated expert and the factors of
 *                  Top-n experts only are brought host -> device on demand           (Sections 3.2, 4.3 case 1)
 *
 * Conventions
 *   - plain C ABI; every call returns 0 on success or a negative MOE_LRC_E* code; the text of the
 *     last error on the calling thread is available from moe_lrc_last_error().
 *   - "host" / "device" in a parameter comment says where the memory lives.  Device buffers are
 *     owned by the caller (activations, indices, outputs, workspace); the library owns the layer
 *     object, its packed weights, the pinned host pool and the device slot pool.  set_* calls copy
 *     out of the caller's host memory before they return and keep no pointer.
 *   - hot-path calls are asynchronous on `stream` (a hipStream_t passed as void*, NULL = default
 *     stream), allocate nothing and do not synchronise, with one exception: a layer created with
 *     residency = MOE_LRC_STAGED reads the per-expert counts back (<= 2 KiB) inside
 *     moe_lrc_expert_ffn / moe_lrc_forward to decide which experts to copy, and therefore
 *     synchronises `stream` once per call.
 *   - argument errors are reported before any device work is issued.
 *   - a layer serves one hot-path call at a time: calls on the same layer must be ordered on one
 *     stream (they share the layer's counters and, with shared experts or staged residency, its
 *     side stream).  moe_lrc_forward on a layer with shared experts forks to that side stream and
 *     joins it before the combine, so everything it does is ordered before later work on `stream`;
 *     it can be captured into a HIP graph (resident layers only: staged ones synchronise).
 *   - matrices are input-dim-major: W[K_in][N_out], y = x W.  mat 0 = W1 (gate projection,
 *     [H][F]), 1 = W3 (up projection, [H][F]), 2 = W2 (down projection, [F][H]);
 *     E_i(x) = (silu(x W1) * (x W3)) W2.
 *   - bf16 / fp16 values cross the ABI as their uint16_t bit patterns.
 *   - range: activations and outputs are bf16; inside, the matrix cores take fp16 operands and
 *     accumulate in fp32.  Every input row x is multiplied by a power of two 2^s (s an integer within
 *     +-60) that brings its largest magnitude into [1, 2), the fp32 results are multiplied by 2^-s
 *     again, and the SwiGLU output h = silu(x W1) * (x W3) is held as fp16(h * 2^(2s)).  Consequences:
 *     a row scaled by any power of two gives the correspondingly exact result while its largest
 *     magnitude is between 2^-60 and 2^60; elements below 2^-14 of their row's largest magnitude lose
 *     bits and those below 2^-24 of it count as zero; |h| * 2^(2s) saturates at 65504 (so with inputs of
 *     order one, |h| up to 6e4; not reached by weights of the magnitudes of Section 4.1's models);
 *     non-finite inputs give unspecified finite or non-finite outputs.
 */
#ifndef MOE_LRC_H
#define MOE_LRC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MOE_LRC_OK       0
#define MOE_LRC_EINVAL  -1   /* null pointer or value out of range                      */
#define MOE_LRC_ESHAPE  -2   /* shape not supported by the kernels                       */
#define MOE_LRC_ESTATE  -3   /* call order: gate or an expert not uploaded, T too large  */
#define MOE_LRC_ENOMEM  -4   /* allocation failed, or workspace too small                */
#define MOE_LRC_EHIP    -5   /* a HIP runtime call failed (no device, launch error)      */

#define MOE_LRC_RESIDENT 0   /* packed experts live in device memory                      */
#define MOE_LRC_STAGED   1   /* packed experts live in pinned host memory and are copied  */
                             /* per call through a device slot pool on a side stream      */
#define MOE_LRC_POOLED   2   /* packed experts live in pinned host memory; the layer owns  */
                             /* no device slots: it runs only as a member of a             */
                             /* moe_lrc_stack, whose slot pool its experts share with the  */
                             /* other layers and keep across calls                         */

typedef struct {
  int32_t hidden;       /* H, multiple of 64, at most 16384                               */
  int32_t ffn;          /* F, multiple of 64, at most 65536                               */
  int32_t n_experts;    /* E routed experts, 1..256                                       */
  int32_t n_shared;     /* S always-on shared experts (Table 1 note), 0..8                */
  int32_t top_k;        /* k, 1..min(E,16)                                                */
  int32_t top_n;        /* n, 0..k: slots 0..n-1 of a token's sorted list are compensated */
  int32_t bits;         /* code width of routed experts: 2, 3 or 4                        */
  int32_t shared_bits;  /* code width of shared experts: 2, 3 or 4 (ignored if S == 0)    */
  int32_t group;        /* quantization group along the input dim: 64, 128 or 256         */
  int32_t rank;         /* compensator rank r >= 0, multiple of 8, <= 1024 (the largest bucket of
                           Section 3.1): the rank of moe_lrc_set_expert, the largest
                           moe_lrc_set_expert_ranked takes                                   */
  int32_t renormalize;  /* 0: routing weights are the softmax-over-all scores (Section 2.1)
                           1: divided by their sum over the k selected                    */
  int32_t max_tokens;   /* largest T any call will pass                                   */
  int32_t residency;    /* MOE_LRC_RESIDENT, MOE_LRC_STAGED or MOE_LRC_POOLED             */
} moe_lrc_config;

typedef struct moe_lrc_layer moe_lrc_layer;

/* Thread-local text of the last error returned on this thread ("" if none). */
const char* moe_lrc_last_error(void);

/* Creates a layer on the current HIP device.  Allocates the packed-weight storage (device, or
 * pinned host + device slots when staged).  *out is set only on success. */
int moe_lrc_layer_create(const moe_lrc_config* cfg, moe_lrc_layer** out);
int moe_lrc_layer_destroy(moe_lrc_layer* layer);

/* Gate G(x) = x Wg^T (+ bias) of Section 2.1.  wg_bf16: host [E][H].  bias_f32: host [E] or NULL
 * (added to the logits before the softmax). */
int moe_lrc_set_gate(moe_lrc_layer* layer, const uint16_t* wg_bf16, const float* bias_f32);

/* Stored artefacts of one projection of one expert (Sections 2.3, 3.1 step 2), all host memory:
 *   codes      one code per byte, [K][N], each < 2^bits
 *   scale_f16  [K/group][N];  zero_f16 [K/group][N];  Qinv(q) = (q - zero) * scale
 *   A_bf16     [K][r] = U sqrt(S);  B_bf16 [r][N] = sqrt(S) V^T   (both NULL when rank == 0 or the
 *              expert is shared; shared experts are never compensated)
 * expert in [0,E) is routed, [E,E+S) shared.  The library repacks into its private bit-packed
 * layout (dense `bits` per weight); moe_lrc_debug_unpack reads it back. */
int moe_lrc_set_expert(moe_lrc_layer* layer, int expert, int mat, const uint8_t* codes,
                       const uint16_t* scale_f16, const uint16_t* zero_f16,
                       const uint16_t* A_bf16, const uint16_t* B_bf16);

/* The same with a rank of its own for this projection (Section 3.1: the rank budget is spread over
 * the expert matrices by their kurtosis, so ranks differ from matrix to matrix and may be 0).
 * rank: multiple of 8, 0..cfg.rank; A_bf16 [K][rank], B_bf16 [rank][N], both NULL when rank == 0.
 * Only `rank` columns/rows are stored in the pinned pool and moved by the staged mode (the byte
 * counters of moe_lrc_get_stats follow), and the expert kernels run only the rank steps of the
 * projection's own rank and read only that many rows of B (a rank-0 projection costs nothing).
 * moe_lrc_set_expert is this call with rank = cfg.rank (0 for shared experts). */
int moe_lrc_set_expert_ranked(moe_lrc_layer* layer, int expert, int mat, const uint8_t* codes,
                              const uint16_t* scale_f16, const uint16_t* zero_f16,
                              const uint16_t* A_bf16, const uint16_t* B_bf16, int rank);

/* Factor pair of one routed projection at 3 bits (Section 3.1 step 2 stores the factors at INT3; the
 * paper gives no group format, this is ours): A [K][rank] quantized in groups of 64 along K, B kept
 * transposed [N][rank] and quantized in groups of 64 along N, both like the weights
 * (value = (code - zero) * scale).  All host memory:
 *   a_codes [K][rank], b_codes [N][rank]   one code per byte, each < 8
 *   a_scale, a_zero  fp16 [K/64][rank];  b_scale, b_zero  fp16 [N/64][rank]
 * rank: multiple of 8 in 8..cfg.rank.  Call after moe_lrc_set_expert(_ranked) of the same projection
 * (with A = B = NULL, rank 0), which uploads the codes of the weights.  The pair stays at 3 bits
 * everywhere: in the pinned pool of a staged or pooled layer, on the bus and in device memory; the
 * kernels that consume it (the (in A) products and the rank steps of the expert FFN, both
 * flavours) rebuild the fp16 operands in registers, one packed FMA per two elements.  On the device
 * a code occupies a 4-bit cell (one dword per eight-element operand unit of a lane), so a pair
 * takes 4 bits + scale/zero (0.5 bit) per value, 3.6 times fewer bytes than the fp16 pair; the byte
 * counters of moe_lrc_get_stats count that.  Projections with fp16 pairs and projections with
 * 3-bit pairs may share a layer, even an expert. */
int moe_lrc_set_expert_factors_quantized(moe_lrc_layer* layer, int expert, int mat, int rank,
                                  const uint8_t* a_codes, const uint16_t* a_scale_f16, const uint16_t* a_zero_f16,
                                  const uint8_t* b_codes, const uint16_t* b_scale_f16, const uint16_t* b_zero_f16);

/* Bytes of device workspace the hot-path calls need for T tokens (the largest over all calls). */
size_t moe_lrc_workspace_bytes(const moe_lrc_layer* layer, int T);

/* An empty batch (T = 0) is accepted by every hot-path call: it launches nothing and returns
 * MOE_LRC_OK; the per-token buffers (x, topk_idx, topk_w, row_pair, pair_row, y_rows, out, the
 * workspace) are not touched and may be null.  moe_lrc_permute still writes counts, offsets and
 * comp_counts (all zero). */
/* Routing (Section 2.1) and Top-n order (Section 3.2).
 *   x_bf16    device [T][H]
 *   topk_idx  device [T][k] int32, experts in descending score order, ties to the lower index;
 *             slots 0..n-1 are the token's Top-n experts
 *   topk_w    device [T][k] float, the routing weights of those experts
 * The gate dot products are accumulated in fp64 so that the selection equals the exact one. */
int moe_lrc_route(moe_lrc_layer* layer, const void* x_bf16, int T,
                  int32_t* topk_idx, float* topk_w, void* stream);

/* Groups the T*k (token, slot) pairs by expert; rows are sorted by (expert asc, token asc).
 * All arrays device int32: counts[E], offsets[E+1] (exclusive scan, offsets[E] = T*k),
 * row_pair[T*k] (row -> t*k+j), pair_row[T*k] (inverse), comp_counts[E] (pairs with j < n). */
int moe_lrc_permute(moe_lrc_layer* layer, const int32_t* topk_idx, int T,
                    int32_t* counts, int32_t* offsets, int32_t* row_pair, int32_t* pair_row,
                    int32_t* comp_counts, void* stream);

/* Expert FFN on the grouped rows (Sections 2.3, 3.2): for row p holding pair (t, j) of expert e,
 *   y_rows[p] = E_e(x_t) with W_hat = Qinv(Q(W)) + [j < n] A B for each of the three projections,
 * the low-rank term applied as (x A) B.  y_rows_bf16: device [T*k][H].  ws: device workspace of
 * at least moe_lrc_workspace_bytes(layer, T) bytes, 256-byte aligned. */
int moe_lrc_expert_ffn(moe_lrc_layer* layer, const void* x_bf16, int T,
                       const int32_t* offsets, const int32_t* row_pair,
                       void* y_rows_bf16, void* ws, size_t ws_bytes, void* stream);

/* out[t] = sum_j topk_w[t][j] * y_rows[pair_row[t*k+j]]  (+ sum over shared experts of E_s(x_t),
 * weight 1, which is why x is passed).  Fixed summation order, no atomics.  out_bf16: device [T][H]. */
int moe_lrc_combine(moe_lrc_layer* layer, const void* y_rows_bf16, const float* topk_w,
                    const int32_t* pair_row, const void* x_bf16, int T,
                    void* out_bf16, void* ws, size_t ws_bytes, void* stream);

/* The whole layer: route -> permute -> (stage) -> expert_ffn -> combine, intermediates in ws.
 * Indices equal those of the four separate calls; `out` equals theirs up to rounding: when the
 * skinny W2 kernel splits its long K into blocks, the combine adds the fp32 partial sums itself
 * instead of reading expert rows that were rounded to bf16 first (one rounding fewer). */
int moe_lrc_forward(moe_lrc_layer* layer, const void* x_bf16, int T, void* out_bf16,
                    void* ws, size_t ws_bytes, void* stream);

/* moe_lrc_forward for callers that cannot allocate device memory or hand over a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The intermediates
 * live in a fixed device array inside the library (MOE_LRC_NOALLOC_WS_BYTES, held by every GPU the
 * library is loaded on until the process ends) instead of a caller workspace; the caller still owns
 * x and out.  Calls no allocator.  Returns MOE_LRC_ENOMEM, before any device work, when
 * moe_lrc_workspace_bytes(layer, T) exceeds the array (the Mixtral-shaped layer fits up to T = 64),
 * MOE_LRC_ESTATE when the layer's device is not the current device.  Every call on a GPU shares that
 * GPU's array: calls that overlap on one GPU (two streams, two layers) race; order them on one
 * stream.  Same result as moe_lrc_forward, bit for bit. */
#define MOE_LRC_NOALLOC_WS_BYTES (32u << 20)
int moe_lrc_forward_noalloc(moe_lrc_layer* layer, const void* x_bf16, int T, void* out_bf16, void* stream);

/* ---- a stack of layers decoding from host-resident experts (Section 4.3, case study 1) -------- */

/* The regime of the paper's GPU-only offloading figures: the packed experts and compensators of
 * every layer stay in (pinned) host memory, the device holds `slots` expert-sized slots shared by
 * all layers, and a decode step walks the layers in order, bringing in what each layer's router
 * selects: the packed codes of every expert that received a row, the factor pair only of experts
 * that received a Top-n row (Section 3.2).  An expert found in a slot is not copied again (slots are
 * kept across layers and steps, least recently used first out).  With MOE_LRC_STACK_PREFETCH, while
 * layer l computes, layer l+1's gate is applied to layer l's input as a guess of its routing and the
 * guessed experts are copied ahead on the copy stream; the guess never decides what is computed
 * (the layer's own routing does), only what is already in a slot when it is needed.
 * With MOE_LRC_STACK_RESIDUAL layer l+1's input is x_l + layer_l(x_l) (rounded once to bf16), else
 * layer_l(x_l). */
typedef struct moe_lrc_stack moe_lrc_stack;
#define MOE_LRC_STACK_PREFETCH 1
#define MOE_LRC_STACK_RESIDUAL 2

/* layers: host array of n_layers (1..1024) layer handles created with residency MOE_LRC_POOLED on
 * the current device, all with the same hidden size and max_tokens; a layer belongs to one stack.
 * The stack does not own them: destroy the stack first, then the layers.  slots: device slots, at
 * least min(n_experts, max_tokens * top_k) of the widest layer (what one layer can need at once);
 * each holds one expert's packed codes, scales and zeros and its factor pair.  Allocates the slot
 * pool, a workspace and two activation buffers on the device. */
int moe_lrc_stack_create(moe_lrc_layer* const* layers, int n_layers, int slots, int flags, moe_lrc_stack** out);
int moe_lrc_stack_destroy(moe_lrc_stack* stack);

/* One decode step: x [T][hidden] bf16 (device) through every layer, result to out [T][hidden] bf16
 * (device).  layer_inputs (device, [n_layers][T][hidden] bf16, or NULL) receives the input of every
 * layer (layer 0's is x).  Synchronises `stream` once per layer (the read-back of the per-expert
 * counts that decides the copies); all kernels run on `stream`, the copies on the stack's own stream.
 * MOE_LRC_ESTATE if a layer's gate or an expert is not uploaded or T exceeds max_tokens. */
int moe_lrc_stack_step(moe_lrc_stack* stack, const void* x_bf16, int T, void* out_bf16, void* layer_inputs, void* stream);

typedef struct {
  uint64_t steps;
  uint64_t expert_uses;     /* (layer, expert) pairs that received a row, over all layers and steps      */
  uint64_t hits;            /* ... whose packed weights were already in a slot                            */
  uint64_t misses;          /* ... copied on demand, the layer's kernels waiting                          */
  uint64_t prefetched;      /* experts copied ahead on the guess                                          */
  uint64_t prefetch_hits;   /* hits on a slot that such a copy had filled and nothing had used yet        */
  uint64_t factor_copies;   /* factor pairs copied, on demand or ahead                                    */
  uint64_t bytes_h2d;       /* bytes copied host -> device by all of the above                            */
  float    last_step_ms;    /* host wall time of the last step, read-backs included                       */
  float    last_copy_ms;    /* first to last copy of the last step on the copy stream (0: none)           */
} moe_lrc_stack_stats;
/* Counters since moe_lrc_stack_create (or the last reset); waits for the last step's copies. */
int moe_lrc_stack_get_stats(moe_lrc_stack* stack, moe_lrc_stack_stats* out);
/* Empties every slot and zeroes the counters (a cold start). */
int moe_lrc_stack_reset(moe_lrc_stack* stack);

/* ---- the offline half of the method on the device (Sections 2.3 and 3.1) ---------------------- */

/* These calls prepare a model once; they are not part of the hot path: moe_lrc_offline_factors and
 * moe_lrc_offline_kurtosis allocate their own device buffers, run on the default stream and
 * synchronise.  All arithmetic is fp64.
 *
 * moe_lrc_offline_quantize: Q(W) of Section 2.3 for W [K][N] (device, fp64, input-dim-major): per
 * group of `group` consecutive input rows of one output column, scale = fp16((max - min) / (2^bits - 1)),
 * zero = fp16(-min / scale), code = clamp(round-half-even(w / scale + zero), 0, 2^bits - 1) with the
 * scale and zero already rounded; a constant group (or a scale that leaves fp16's range) gets
 * scale 1, zero = fp16(-min), codes 0.  codes_dev [K][N] one code per byte, scale_dev / zero_dev
 * [K/group][N] fp16 bit patterns: the arrays moe_lrc_set_expert takes.  residual_dev (or NULL)
 * receives E = W - (code - zero) * scale, [K][N] fp64.  Asynchronous on `stream`. */
int moe_lrc_offline_quantize(const double* W_dev, int K, int N, int bits, int group, uint8_t* codes_dev,
                             uint16_t* scale_dev, uint16_t* zero_dev, double* residual_dev, void* stream);

/* moe_lrc_offline_quantize with the zero points refined by a half-quadratic solver (Section 3.1
 * step 2: "HQQ-style weight optimization"; the paper gives no parameters, the customary ones are
 * iters = 20, p = 0.7, beta = 10, kappa = 1.01).  Per group, with the min/max scale kept and a
 * real-valued zero point z, `iters` times: q = clamp(round(w / scale + z)); e = shrink(w - (q - z) scale)
 * with shrink(x) = sign(x) max(|x| - |x|^(p-1) / beta, 0); z = mean over the group of
 * (q - (w - e) / scale); beta *= kappa.  Then z is rounded to fp16 and the codes are chosen for the
 * stored values.  iters = 0 gives moe_lrc_offline_quantize.  Same outputs; asynchronous on `stream`. */
int moe_lrc_offline_quantize_refined(const double* W_dev, int K, int N, int bits, int group, int iters, double p, double beta,
                                     double kappa, uint8_t* codes_dev, uint16_t* scale_dev, uint16_t* zero_dev,
                                     double* residual_dev, void* stream);

/* Rank-`rank` factors of E [K][N] (device, fp64), Section 3.1 step 2: A = U sqrt(S) [K][rank] and
 * B = sqrt(S) V^T [rank][N] (device, fp64) for the `rank` leading singular triplets, found by a
 * subspace iteration from the test matrix omega_dev [N][l] (device, fp64; standard normal entries,
 * rank <= l <= min(K, N, 1088), l = rank + 8 is the usual choice) with `power_iters` (0..8) passes over
 * E and E^T; the singular values go to sigma_host [rank] (or NULL), in descending order.  The signs
 * of a pair (column i of A, row i of B) are arbitrary; their product is not.  A_bf16_dev /
 * B_bf16_dev (or NULL) receive the factors rounded to bf16, the form moe_lrc_set_expert takes.
 * MOE_LRC_ESHAPE if the sketch loses rank (E of rank below l) or the rotations do not converge. */
int moe_lrc_offline_factors(const double* E_dev, int K, int N, int rank, const double* omega_dev, int l, int power_iters,
                            double* A_dev, double* B_dev, double* sigma_host, uint16_t* A_bf16_dev, uint16_t* B_bf16_dev);

/* Kurtosis of the n entries of a matrix (device, fp64), Section 3.1 step 1:
 * kappa = mean((w - mu)^4) / mean((w - mu)^2)^2, to *kappa (host). */
int moe_lrc_offline_kurtosis(const double* W_dev, size_t n, double* kappa);

/* Host-only (no device): the greedy bucketed rank allocation of Section 3.1 step 1.  In descending
 * order of kurtosis (kappa_host [n]; equal values in index order) every matrix takes the largest
 * value of buckets_host [n_buckets] (the paper's {0, 16, 32, 128, 256, 512, 1024}) that keeps the sum
 * of the ranks given out so far within n * r_avg; ranks_host [n] receives them (0 if none fits). */
int moe_lrc_offline_allocate_ranks(const double* kappa_host, int n, int r_avg, const int32_t* buckets_host, int n_buckets,
                                   int32_t* ranks_host);

/* Host-only: the quantizer's fp64 -> fp16 rounding (to nearest, ties to even, one rounding) of n
 * values, for checking against another implementation. */
int moe_lrc_selftest_half_rounding(const double* in_host, size_t n, uint16_t* out_host);

/* ---- evidence and test hooks ------------------------------------------------------------- */

/* Unpacks the layer's private copy of one projection back to one code per byte, device [K][N]. */
int moe_lrc_debug_unpack(moe_lrc_layer* layer, int expert, int mat, uint8_t* codes_dev, void* stream);

/* Host-only packing round trip (no device needed): packs codes [K][N] into the private layout
 * (packed must hold moe_lrc_packed_bytes(bits, K, N) bytes) and back. */
size_t moe_lrc_packed_bytes(int bits, int K, int N);
int moe_lrc_pack_codes(int bits, int K, int N, const uint8_t* codes, void* packed);
int moe_lrc_unpack_codes(int bits, int K, int N, const void* packed, uint8_t* codes);

typedef struct {
  uint64_t bytes_codes;    /* packed code bytes of experts with at least one routed pair         */
  uint64_t bytes_meta;     /* fp16 scale+zero bytes of those experts                             */
  uint64_t bytes_factors;  /* bf16 factor bytes of experts with at least one Top-n pair          */
  int32_t  active_experts;
  int32_t  comp_experts;
  int32_t  path;           /* kernel flavour of the last expert_ffn's routed projections:
                              bit 0 set: W1|W3 ran as the grouped GEMM (many rows per expert),
                              bit 1 set: W2 did; a clear bit: the skinny decode flavour            */
  float    stage_ms;       /* staged mode: time of the last call's host->device copies, else 0   */
} moe_lrc_stats;

/* Counters of the last moe_lrc_expert_ffn / moe_lrc_forward on this layer.  In staged mode they
 * are exact (the counts are read back anyway); in resident mode this call synchronises the device
 * and reads the counts of the last call. */
int moe_lrc_get_stats(moe_lrc_layer* layer, moe_lrc_stats* out);

/* Per-stage timing of moe_lrc_forward with HIP events recorded on the caller's stream between the
 * kernels (measurement hook for the roofline figures; off by default, adds ~10 event records per
 * call when on).  Stages, in launch order: */
#define MOE_LRC_STAGE_ROUTE    0   /* gate + softmax + Top-k                          */
#define MOE_LRC_STAGE_PERMUTE  1   /* grouping of pairs by expert                     */
#define MOE_LRC_STAGE_PREP     2   /* fp16 activation copy, per-expert counters, staging */
#define MOE_LRC_STAGE_XA13     3   /* (x A1 | x A3) for Top-n rows                    */
#define MOE_LRC_STAGE_W13      4   /* packed W1|W3 projections + SwiGLU               */
#define MOE_LRC_STAGE_XA2      5   /* (h A2) for Top-n rows                           */
#define MOE_LRC_STAGE_W2       6   /* packed W2 projection                            */
#define MOE_LRC_STAGE_SHARED   7   /* shared experts                                  */
#define MOE_LRC_STAGE_COMBINE  8   /* weighted sum                                    */
#define MOE_LRC_N_STAGES       9
int moe_lrc_profile_enable(moe_lrc_layer* layer, int on);
/* Waits for the last moe_lrc_forward of this layer and writes its stage durations in
 * milliseconds to ms[MOE_LRC_N_STAGES] (host). */
int moe_lrc_profile_read(moe_lrc_layer* layer, float* ms);

/* Host-only self-check of the index arithmetic of the skinny (decode) FFN kernels; needs no device.
 * The kernels form every buffer offset and LDS address through a small set of integer functions;
 * this call walks the same functions for every block, wavefront, lane and step of the two launches
 * (fused W1|W3, then W2 in `kblocks_w2` K-blocks) that serve one expert with `rows` rows starting at
 * `first_row` of `total_rows`, the expert's n-tiles shared by `blocks_w13` / `blocks_w2` blocks, and
 * checks every offset against the size of what it addresses, and that every packed tile and every
 * rank step of each projection (rank1, rank3, rank2 <= layer_rank <= 1024: Section 3.1 gives every
 * expert matrix a rank of its own) is read exactly once.  Returns 0, or MOE_LRC_ESHAPE with the first
 * violation in moe_lrc_last_error(). */
int moe_lrc_selftest_decode_index(int hidden, int ffn, int bits, int group, int layer_rank, int rank1,
                                  int rank3, int rank2, int first_row, int rows, int total_rows,
                                  int blocks_w13, int blocks_w2, int kblocks_w2);

/* Host-only model of how the kernels read a factor pair held at 3 bits (Section 3.1 step 2): packs
 * the pair as moe_lrc_set_expert_factors_quantized does, then rebuilds every element the way the
 * consuming kernels do (the same unit and metadata indices, the same field extraction, one fp16 FMA
 * with a single rounding per element) into A_out [K][rank] and B_out [rank][N] (host, fp32). */
int moe_lrc_selftest_factor_pair(int K, int N, int rank, const uint8_t* a_codes, const uint16_t* a_scale,
                               const uint16_t* a_zero, const uint8_t* b_codes, const uint16_t* b_scale,
                               const uint16_t* b_zero, float* A_out, float* B_out);

/* What the current device sustains on the resources the roofline figures are priced against
 * (Section 2.2's roofline remark: offloaded MoE decoding is bound by moving expert weights).
 * Measurement hook: allocates its own buffers, runs on the default stream and synchronises.
 *   MOE_LRC_CAL_HBM_READ  streaming read of a `bytes`-sized device buffer (use several times the
 *                         256 MB last-level cache), *result = GB/s of the median of `reps` passes
 *   MOE_LRC_CAL_H2D       copy of `bytes` from pinned host memory to the device, GB/s
 *   MOE_LRC_CAL_MFMA_F16  dense v_mfma_f32_16x16x32_f16 issue rate on registers, TFLOP/s (`bytes` unused)
 *   MOE_LRC_CAL_MFMA_F16_32  the same with v_mfma_f32_32x32x16_f16
 *   MOE_LRC_CAL_MFMA_VALU  two wavefronts per SIMD issue v_mfma_f32_16x16x32_f16, each followed by
 *                         `bytes` (0, 2, 4, 8 or 16) independent packed fp16 FMAs: *result = ns per
 *                         MFMA with its FMAs on one SIMD (how far vector work hides behind MFMAs)
 *   MOE_LRC_CAL_SUBSTEP   four wavefronts per SIMD run a loop shaped like a sub-step of the decode
 *                         flavour of the expert FFN: 8 mask and 8 packed-FMA operations make two
 *                         operands, then 2 MT MFMAs use them.  bytes = MT (1 or 2 row tiles) + 16 *
 *                         mode (0: both, 1: the MFMAs alone, 2: the vector operations alone);
 *                         *result = ns of SIMD time per sub-step of one wavefront
 * result: host pointer to one double. */
#define MOE_LRC_CAL_HBM_READ 0
#define MOE_LRC_CAL_H2D      1
#define MOE_LRC_CAL_MFMA_F16 2
#define MOE_LRC_CAL_MFMA_F16_32 3
#define MOE_LRC_CAL_MFMA_VALU 4
#define MOE_LRC_CAL_SUBSTEP 5
int moe_lrc_calibrate(int kind, size_t bytes, int reps, double* result);

#ifdef __cplusplus
}
#endif
#endif /* MOE_LRC_H */
