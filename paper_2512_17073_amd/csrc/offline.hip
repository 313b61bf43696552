// The offline half of the method on the device, in fp64: group-wise uniform quantization of a weight
// matrix (Section 2.3), its residual E = W - Qinv(Q(W)), the rank-r factors of the residual
// (Section 3.1 step 2: SVD_r(E) = U S V^T, stored as A = U sqrt(S), B = sqrt(S) V^T) and the kurtosis of
// a matrix (Section 3.1 step 1).  Not part of the hot path: these calls allocate their own buffers
// and synchronise.
//
// Factors: a randomized subspace iteration (Halko, Martinsson, Tropp) driven by a caller-supplied
// test matrix Omega, so that both sides of a comparison can use the same random numbers:
//   Y = E Omega;  repeat `power_iters` times:  Y <- E (E^T orth(Y));  Q = orth(Y);  Bm = Q^T E  (l x N)
//   SVD of the small matrix Bm by one-sided Jacobi rotations of its rows (Hestenes), which leaves
//   rows sigma_i w_i^T and accumulates the rotations G: Bm = G diag(sigma) W^T, so U = Q G.
// orth() is a Cholesky QR applied twice (Gram matrix, Cholesky factor, triangular solve): the
// residual of a quantizer is close to white noise, its leading singular values are nearly flat, and
// the Gram matrix of l such directions is well conditioned.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <numeric>
#include <vector>

#include "internal.h"
#include "offline_round.h"

namespace lrc {
namespace {

// ---------------------------------------------------------------------------------- quantizer
// One thread per (group, column): minimum and maximum of the group's `group` entries, then scale and
// zero rounded to fp16 before the codes are chosen (so the codes are optimal for the stored values),
// then the codes and, if wanted, the residual.  A constant group, or one whose scale rounds to zero
// or overflows in fp16, gets scale 1, zero = -min and codes 0.
__global__ __launch_bounds__(256) void quantize_kernel(const double* __restrict__ W, int K, int N, int bits, int group,
                                                       uint8_t* __restrict__ codes, uint16_t* __restrict__ scale,
                                                       uint16_t* __restrict__ zero, double* __restrict__ resid) {
#pragma clang fp contract(off)      // every product and sum rounded on its own, as written
  const int n = blockIdx.x * 256 + threadIdx.x, g = blockIdx.y;
  if (n >= N) return;
  const double* w = W + size_t(g) * group * N + n;
  double lo = w[0], hi = w[0];
  for (int i = 1; i < group; ++i) {
    const double v = w[size_t(i) * N];
    lo = v < lo ? v : lo;
    hi = v > hi ? v : hi;
  }
  const int levels = (1 << bits) - 1;
  uint16_t sb = f64_to_f16_bits((hi - lo) / double(levels));
  double s = f16_bits_to_f64(sb);
  const bool degenerate = !(s > 0.0) || (sb & 0x7fffu) >= 0x7c00u;
  uint16_t zb;
  if (degenerate) {
    sb = 0x3c00u; s = 1.0;
    zb = f64_to_f16_bits(-lo);
  } else {
    zb = f64_to_f16_bits(-lo / s);
  }
  const double z = f16_bits_to_f64(zb);
  scale[size_t(g) * N + n] = sb;
  zero[size_t(g) * N + n] = zb;
  for (int i = 0; i < group; ++i) {
    const size_t at = (size_t(g) * group + i) * N + n;
    const double v = w[size_t(i) * N];
    double q = degenerate ? 0.0 : __builtin_rint(v / s + z);      // round half to even
    q = q < 0.0 ? 0.0 : (q > double(levels) ? double(levels) : q);
    if (!(q == q)) q = 0.0;
    codes[at] = uint8_t(int(q));
    if (resid) resid[at] = v - (q - z) * s;
  }
}

// The same with the zero points refined by a half-quadratic solver ("HQQ-style weight optimization",
// Section 3.1 step 2; the published scheme: l_p error, p < 1, penalty beta growing by kappa per step).
// Per group, scale fixed, zero point z real-valued:
//   q = clamp(round(w / s + z));  e = shrink(w - (q - z) s);  z = mean(q - (w - e) / s);  beta *= kappa
// with shrink(x) = sign(x) max(|x| - |x|^(p-1) / beta, 0); then z is rounded to fp16 and the codes are
// chosen for the stored values.  The group's entries are re-read from memory in every step (they stay
// in cache); sums run in index order.
__global__ __launch_bounds__(256) void quantize_refined_kernel(const double* __restrict__ W, int K, int N, int bits, int group,
                                                               int iters, double p, double beta, double kappa,
                                                               uint8_t* __restrict__ codes, uint16_t* __restrict__ scale,
                                                               uint16_t* __restrict__ zero, double* __restrict__ resid) {
#pragma clang fp contract(off)
  const int n = blockIdx.x * 256 + threadIdx.x, g = blockIdx.y;
  if (n >= N) return;
  const double* w = W + size_t(g) * group * N + n;
  double lo = w[0], hi = w[0];
  for (int i = 1; i < group; ++i) {
    const double v = w[size_t(i) * N];
    lo = v < lo ? v : lo;
    hi = v > hi ? v : hi;
  }
  const int levels = (1 << bits) - 1;
  uint16_t sb = f64_to_f16_bits((hi - lo) / double(levels));
  double s = f16_bits_to_f64(sb);
  const bool degenerate = !(s > 0.0) || (sb & 0x7fffu) >= 0x7c00u;
  double z;
  if (degenerate) { sb = 0x3c00u; s = 1.0; z = -lo; }
  else z = -lo / s;
  if (!degenerate) {
    double b = beta;
    for (int it = 0; it < iters; ++it) {
      double sum = 0.0;
      for (int i = 0; i < group; ++i) {
        const double v = w[size_t(i) * N];
        double q = __builtin_rint(v / s + z);
        q = q < 0.0 ? 0.0 : (q > double(levels) ? double(levels) : q);
        const double x = v - (q - z) * s, ax = fabs(x);
        double e = 0.0;
        if (ax > 0.0) {
          const double t = ax - pow(ax, p - 1.0) / b;
          e = t > 0.0 ? (x < 0.0 ? -t : t) : 0.0;
        }
        sum += q - (v - e) / s;
      }
      z = sum / double(group);
      b *= kappa;
    }
  }
  const uint16_t zb = f64_to_f16_bits(z);
  z = f16_bits_to_f64(zb);
  scale[size_t(g) * N + n] = sb;
  zero[size_t(g) * N + n] = zb;
  for (int i = 0; i < group; ++i) {
    const size_t at = (size_t(g) * group + i) * N + n;
    const double v = w[size_t(i) * N];
    double q = degenerate ? 0.0 : __builtin_rint(v / s + z);
    q = q < 0.0 ? 0.0 : (q > double(levels) ? double(levels) : q);
    if (!(q == q)) q = 0.0;
    codes[at] = uint8_t(int(q));
    if (resid) resid[at] = v - (q - z) * s;
  }
}

// ---------------------------------------------------------------------------------- kurtosis
// Partial sums of one pass in fp64: blocks of 256 threads over a grid-stride range, one partial per
// block, added up on the host in block order (deterministic).
__global__ __launch_bounds__(256) void moment_kernel(const double* __restrict__ w, size_t n, double mu, int power,
                                                     double* __restrict__ partial) {
  __shared__ double red[256];
  double acc = 0.0;
  for (size_t i = size_t(blockIdx.x) * 256 + threadIdx.x; i < n; i += size_t(gridDim.x) * 256) {
    const double d = w[i] - mu;
    acc += power == 1 ? d : power == 2 ? d * d : (d * d) * (d * d);
  }
  red[threadIdx.x] = acc;
  __syncthreads();
  for (int s = 128; s > 0; s >>= 1) {
    if ((int)threadIdx.x < s) red[threadIdx.x] += red[threadIdx.x + s];
    __syncthreads();
  }
  if (threadIdx.x == 0) partial[blockIdx.x] = red[0];
}

// ---------------------------------------------------------------------------------- dense fp64 products
// C[M][Nc] = op(A) B with op(A)[i][k] = TRANS ? A[k * lda + i] : A[i * lda + k] and B[k * ldb + j]:
// 64 x 64 tiles of C per block of 256 threads (a 4 x 4 block of C each), k in steps of 16 through LDS,
// sums in increasing k.  Plain vector fp64 FMAs: the products here are tall and skinny and run once.
template <bool TRANS>
__global__ __launch_bounds__(256) void dgemm_kernel(int M, int Nc, int Kd, const double* __restrict__ A, int lda,
                                                    const double* __restrict__ B, int ldb, double* __restrict__ C, int ldc) {
  __shared__ double As[16][65], Bs[16][65];
  const int t = threadIdx.x, tx = t & 15, ty = t >> 4;
  const int i0 = blockIdx.y * 64, j0 = blockIdx.x * 64;
  double acc[4][4] = {};
  for (int k0 = 0; k0 < Kd; k0 += 16) {
    if (TRANS) {
      const int kk = t >> 4, r4 = (t & 15) * 4;
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int i = i0 + r4 + u, k = k0 + kk;
        As[kk][r4 + u] = (i < M && k < Kd) ? A[size_t(k) * lda + i] : 0.0;
      }
    } else {
      const int r = t >> 2, k4 = (t & 3) * 4;
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int i = i0 + r, k = k0 + k4 + u;
        As[k4 + u][r] = (i < M && k < Kd) ? A[size_t(i) * lda + k] : 0.0;
      }
    }
    {
      const int kk = t >> 4, c4 = (t & 15) * 4;
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int j = j0 + c4 + u, k = k0 + kk;
        Bs[kk][c4 + u] = (j < Nc && k < Kd) ? B[size_t(k) * ldb + j] : 0.0;
      }
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < 16; ++kk) {
      double a[4], b[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) { a[u] = As[kk][ty * 4 + u]; b[u] = Bs[kk][tx * 4 + u]; }
#pragma unroll
      for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int v = 0; v < 4; ++v) acc[u][v] = fma(a[u], b[v], acc[u][v]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int u = 0; u < 4; ++u)
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int i = i0 + ty * 4 + u, j = j0 + tx * 4 + v;
      if (i < M && j < Nc) C[size_t(i) * ldc + j] = acc[u][v];
    }
}

template <bool TRANS>
void dgemm(int M, int Nc, int Kd, const double* A, int lda, const double* B, int ldb, double* C, int ldc) {
  hipLaunchKernelGGL(dgemm_kernel<TRANS>, dim3((Nc + 63) / 64, (M + 63) / 64), dim3(256), 0, nullptr, M, Nc, Kd, A, lda, B, ldb, C, ldc);
}

// ---------------------------------------------------------------------------------- Cholesky QR
// In-place lower Cholesky factor of the l x l matrix G (one block; right-looking): *bad is set if a
// pivot is not positive.
__global__ __launch_bounds__(1024) void cholesky_kernel(double* __restrict__ G, int l, int* __restrict__ bad) {
  __shared__ double d_sh;
  for (int j = 0; j < l; ++j) {
    if (threadIdx.x == 0) {
      const double p = G[size_t(j) * l + j];
      if (!(p > 0.0)) *bad = 1;
      d_sh = sqrt(p > 0.0 ? p : 1.0);
      G[size_t(j) * l + j] = d_sh;
    }
    __syncthreads();
    const double d = d_sh;
    for (int i = j + 1 + threadIdx.x; i < l; i += 1024) G[size_t(i) * l + j] /= d;
    __syncthreads();
    const int n = l - j - 1;
    for (long long idx = threadIdx.x; idx < (long long)n * n; idx += 1024) {
      const int i = j + 1 + int(idx / n), k = j + 1 + int(idx % n);
      if (k <= i) G[size_t(i) * l + k] -= G[size_t(i) * l + j] * G[size_t(k) * l + j];
    }
    __syncthreads();
  }
}

// Y <- Y L^-T for the lower-triangular L (l x l): one thread per row of Y (K rows), forward substitution.
__global__ __launch_bounds__(256) void trsm_kernel(double* __restrict__ Y, int K, int l, const double* __restrict__ L) {
  const int r = blockIdx.x * 256 + threadIdx.x;
  if (r >= K) return;
  double* y = Y + size_t(r) * l;
  for (int j = 0; j < l; ++j) {
    double s = y[j];
    for (int k = 0; k < j; ++k) s -= y[k] * L[size_t(j) * l + k];
    y[j] = s / L[size_t(j) * l + j];
  }
}

// ---------------------------------------------------------------------------------- one-sided Jacobi
// One step of a sweep: block b rotates rows (p, q) = pairs[2b], pairs[2b + 1] of Bm (l x N) so that
// they become orthogonal, and applies the same rotation to rows p, q of Gt (l x l).  *off receives
// the largest |<p, q>| / (|p| |q|) seen (as the bits of a non-negative float, by atomicMax).
__global__ __launch_bounds__(256) void jacobi_kernel(double* __restrict__ Bm, int N, double* __restrict__ Gt, int l,
                                                     const int* __restrict__ pairs, unsigned* __restrict__ off) {
  __shared__ double red[3][256];
  __shared__ double cs[2];
  const int p = pairs[2 * blockIdx.x], q = pairs[2 * blockIdx.x + 1];
  if (p < 0 || q < 0) return;
  double* bp = Bm + size_t(p) * N;
  double* bq = Bm + size_t(q) * N;
  double a = 0.0, b = 0.0, g = 0.0;
  for (int i = threadIdx.x; i < N; i += 256) {
    const double x = bp[i], y = bq[i];
    a = fma(x, x, a); b = fma(y, y, b); g = fma(x, y, g);
  }
  red[0][threadIdx.x] = a; red[1][threadIdx.x] = b; red[2][threadIdx.x] = g;
  __syncthreads();
  for (int s = 128; s > 0; s >>= 1) {
    if ((int)threadIdx.x < s)
      for (int m = 0; m < 3; ++m) red[m][threadIdx.x] += red[m][threadIdx.x + s];
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    const double alpha = red[0][0], beta = red[1][0], gamma = red[2][0];
    const double denom = sqrt(alpha * beta);
    const double rel = denom > 0.0 ? fabs(gamma) / denom : 0.0;
    atomicMax(off, __float_as_uint(float(rel)));
    double c = 1.0, s = 0.0;
    if (rel > 1e-16) {
      const double zeta = (beta - alpha) / (2.0 * gamma);
      const double t = (zeta >= 0.0 ? 1.0 : -1.0) / (fabs(zeta) + sqrt(1.0 + zeta * zeta));
      c = 1.0 / sqrt(1.0 + t * t);
      s = c * t;
    }
    cs[0] = c; cs[1] = s;
  }
  __syncthreads();
  const double c = cs[0], s = cs[1];
  if (s == 0.0) return;
  for (int i = threadIdx.x; i < N; i += 256) {
    const double x = bp[i], y = bq[i];
    bp[i] = c * x - s * y;
    bq[i] = s * x + c * y;
  }
  double* gp = Gt + size_t(p) * l;
  double* gq = Gt + size_t(q) * l;
  for (int i = threadIdx.x; i < l; i += 256) {
    const double x = gp[i], y = gq[i];
    gp[i] = c * x - s * y;
    gq[i] = s * x + c * y;
  }
}

__global__ __launch_bounds__(256) void row_norm2_kernel(const double* __restrict__ Bm, int N, double* __restrict__ out) {
  __shared__ double red[256];
  const double* b = Bm + size_t(blockIdx.x) * N;
  double a = 0.0;
  for (int i = threadIdx.x; i < N; i += 256) a = fma(b[i], b[i], a);
  red[threadIdx.x] = a;
  __syncthreads();
  for (int s = 128; s > 0; s >>= 1) {
    if ((int)threadIdx.x < s) red[threadIdx.x] += red[threadIdx.x + s];
    __syncthreads();
  }
  if (threadIdx.x == 0) out[blockIdx.x] = red[0];
}

// B[i][n] = Bm[sel[i]][n] * mul[i]
__global__ __launch_bounds__(256) void pick_rows_kernel(const double* __restrict__ Bm, int N, const int* __restrict__ sel,
                                                        const double* __restrict__ mul, double* __restrict__ B) {
  const int i = blockIdx.y, n = blockIdx.x * 256 + threadIdx.x;
  if (n < N) B[size_t(i) * N + n] = Bm[size_t(sel[i]) * N + n] * mul[i];
}

__global__ __launch_bounds__(256) void to_bf16_kernel(const double* __restrict__ in, size_t n, uint16_t* __restrict__ out) {
  const size_t i = size_t(blockIdx.x) * 256 + threadIdx.x;
  if (i >= n) return;
  // (through fp32, as the stored factors are defined: exact for the magnitudes of a residual's factors)
  uint32_t u = __float_as_uint(float(in[i]));
  u += 0x7fffu + ((u >> 16) & 1u);
  out[i] = uint16_t(u >> 16);
}

}  // namespace
}  // namespace lrc

using namespace lrc;

#define OFF_HIP(expr)                                                                                \
  do {                                                                                               \
    hipError_t e_ = (expr);                                                                          \
    if (e_ != hipSuccess) {                                                                          \
      rc = set_error(e_ == hipErrorOutOfMemory ? MOE_LRC_ENOMEM : MOE_LRC_EHIP,                      \
                     std::string("offline: ") + #expr + ": " + hipGetErrorString(e_));               \
      goto done;                                                                                     \
    }                                                                                                \
  } while (0)

extern "C" {

int moe_lrc_offline_quantize(const double* W_dev, int K, int N, int bits, int group, uint8_t* codes_dev,
                             uint16_t* scale_dev, uint16_t* zero_dev, double* residual_dev, void* stream) {
  if (!W_dev || !codes_dev || !scale_dev || !zero_dev) return set_error(MOE_LRC_EINVAL, "offline_quantize: null argument");
  if (bits < 2 || bits > 4) return set_error(MOE_LRC_EINVAL, "offline_quantize: bits must be 2, 3 or 4");
  if (K <= 0 || N <= 0 || group <= 0 || K % group) return set_error(MOE_LRC_ESHAPE, "offline_quantize: K must be a positive multiple of group");
  hipLaunchKernelGGL(quantize_kernel, dim3((N + 255) / 256, K / group), dim3(256), 0, (hipStream_t)stream, W_dev, K, N, bits, group,
                     codes_dev, scale_dev, zero_dev, residual_dev);
  LRC_HIP(hipGetLastError());
  return MOE_LRC_OK;
}

int moe_lrc_offline_quantize_refined(const double* W_dev, int K, int N, int bits, int group, int iters, double p, double beta,
                                     double kappa, uint8_t* codes_dev, uint16_t* scale_dev, uint16_t* zero_dev,
                                     double* residual_dev, void* stream) {
  if (!W_dev || !codes_dev || !scale_dev || !zero_dev) return set_error(MOE_LRC_EINVAL, "offline_quantize_refined: null argument");
  if (bits < 2 || bits > 4) return set_error(MOE_LRC_EINVAL, "offline_quantize_refined: bits must be 2, 3 or 4");
  if (iters < 0 || iters > 1000 || !(p > 0.0 && p <= 1.0) || !(beta > 0.0) || !(kappa >= 1.0))
    return set_error(MOE_LRC_EINVAL, "offline_quantize_refined: need 0 <= iters <= 1000, 0 < p <= 1, beta > 0, kappa >= 1");
  if (K <= 0 || N <= 0 || group <= 0 || K % group) return set_error(MOE_LRC_ESHAPE, "offline_quantize_refined: K must be a positive multiple of group");
  hipLaunchKernelGGL(quantize_refined_kernel, dim3((N + 255) / 256, K / group), dim3(256), 0, (hipStream_t)stream, W_dev, K, N, bits, group,
                     iters, p, beta, kappa, codes_dev, scale_dev, zero_dev, residual_dev);
  LRC_HIP(hipGetLastError());
  return MOE_LRC_OK;
}

int moe_lrc_offline_kurtosis(const double* W_dev, size_t n, double* kappa) {
  if (!W_dev || !kappa || n == 0) return set_error(MOE_LRC_EINVAL, "offline_kurtosis: null argument or empty matrix");
  int rc = MOE_LRC_OK;
  const int blocks = 1024;
  double* d_part = nullptr;
  std::vector<double> part(blocks);
  double mu = 0.0, m2 = 0.0, m4 = 0.0;
  auto pass = [&](double center, int power, double& out) -> hipError_t {
    hipLaunchKernelGGL(moment_kernel, dim3(blocks), dim3(256), 0, nullptr, W_dev, n, center, power, d_part);
    hipError_t e = hipMemcpy(part.data(), d_part, blocks * sizeof(double), hipMemcpyDeviceToHost);
    out = 0.0;
    for (double v : part) out += v;
    return e;
  };
  OFF_HIP(hipMalloc((void**)&d_part, blocks * sizeof(double)));
  OFF_HIP(pass(0.0, 1, mu));
  mu /= double(n);
  OFF_HIP(pass(mu, 2, m2));
  OFF_HIP(pass(mu, 4, m4));
  m2 /= double(n); m4 /= double(n);
  *kappa = m4 / (m2 * m2);
done:
  if (d_part) (void)hipFree(d_part);
  return rc;
}

int moe_lrc_offline_factors(const double* E_dev, int K, int N, int rank, const double* omega_dev, int l, int power_iters,
                            double* A_dev, double* B_dev, double* sigma_host, uint16_t* A_bf16_dev, uint16_t* B_bf16_dev) {
  if (!E_dev || !omega_dev || !A_dev || !B_dev) return set_error(MOE_LRC_EINVAL, "offline_factors: null argument");
  if (K <= 0 || N <= 0 || rank <= 0 || l < rank || l > K || l > N || l > 1088)
    return set_error(MOE_LRC_ESHAPE, "offline_factors: need 0 < rank <= l <= min(K, N, 1088)");
  if (power_iters < 0 || power_iters > 8) return set_error(MOE_LRC_EINVAL, "offline_factors: power_iters outside 0..8");
  int rc = MOE_LRC_OK;
  double *Y = nullptr, *Z = nullptr, *G = nullptr, *Bm = nullptr, *Gt = nullptr, *norm2 = nullptr, *M = nullptr, *mul = nullptr;
  int *bad = nullptr, *pairs = nullptr, *sel = nullptr;
  unsigned* off = nullptr;
  const int lp = l + (l & 1);                       // rows of the tournament (an odd l gets a bye)
  std::vector<int> h_pairs(size_t(lp - 1) * lp, -1), order(l);
  std::vector<double> h_norm2(l), h_Gt, h_M, h_mul(rank);
  std::vector<int> h_sel(rank);
  int h_bad = 0;
  // orth(Y): Cholesky QR, twice
  auto orth = [&]() -> int {
    for (int rep = 0; rep < 2; ++rep) {
      dgemm<true>(l, l, K, Y, l, Y, l, G, l);
      hipLaunchKernelGGL(cholesky_kernel, dim3(1), dim3(1024), 0, nullptr, G, l, bad);
      hipLaunchKernelGGL(trsm_kernel, dim3((K + 255) / 256), dim3(256), 0, nullptr, Y, K, l, G);
    }
    if (hipMemcpy(&h_bad, bad, sizeof(int), hipMemcpyDeviceToHost) != hipSuccess) return -1;
    return h_bad;
  };
  OFF_HIP(hipMalloc((void**)&Y, size_t(K) * l * 8));
  OFF_HIP(hipMalloc((void**)&Z, size_t(N) * l * 8));
  OFF_HIP(hipMalloc((void**)&G, size_t(l) * l * 8));
  OFF_HIP(hipMalloc((void**)&Bm, size_t(l) * N * 8));
  OFF_HIP(hipMalloc((void**)&Gt, size_t(l) * l * 8));
  OFF_HIP(hipMalloc((void**)&norm2, size_t(l) * 8));
  OFF_HIP(hipMalloc((void**)&M, size_t(l) * rank * 8));
  OFF_HIP(hipMalloc((void**)&mul, size_t(rank) * 8));
  OFF_HIP(hipMalloc((void**)&bad, sizeof(int)));
  OFF_HIP(hipMalloc((void**)&off, sizeof(unsigned)));
  OFF_HIP(hipMalloc((void**)&pairs, h_pairs.size() * sizeof(int)));
  OFF_HIP(hipMalloc((void**)&sel, size_t(rank) * sizeof(int)));
  OFF_HIP(hipMemset(bad, 0, sizeof(int)));

  // ---- range finder
  dgemm<false>(K, l, N, E_dev, N, omega_dev, l, Y, l);                  // Y = E Omega
  for (int it = 0; it < power_iters; ++it) {
    if (orth() != 0) { rc = set_error(MOE_LRC_ESHAPE, "offline_factors: the sketch lost rank (Gram matrix not positive definite)"); goto done; }
    dgemm<true>(N, l, K, E_dev, N, Y, l, Z, l);                         // Z = E^T Q
    dgemm<false>(K, l, N, E_dev, N, Z, l, Y, l);                        // Y = E Z
  }
  if (orth() != 0) { rc = set_error(MOE_LRC_ESHAPE, "offline_factors: the sketch lost rank (Gram matrix not positive definite)"); goto done; }
  dgemm<true>(l, N, K, Y, l, E_dev, N, Bm, N);                          // Bm = Q^T E

  // ---- SVD of Bm: sweeps of a round-robin tournament over the row pairs
  for (int s = 0; s < lp - 1; ++s) {
    int* row = h_pairs.data() + size_t(s) * lp;
    for (int k = 0; k < lp / 2; ++k) {
      int a = k == 0 ? lp - 1 : (s + k) % (lp - 1), b = (s - k + (lp - 1)) % (lp - 1);
      if (a >= l || b >= l) { a = -1; b = -1; }
      row[2 * k] = a; row[2 * k + 1] = b;
    }
  }
  OFF_HIP(hipMemcpy(pairs, h_pairs.data(), h_pairs.size() * sizeof(int), hipMemcpyHostToDevice));
  h_Gt.assign(size_t(l) * l, 0.0);
  for (int i = 0; i < l; ++i) h_Gt[size_t(i) * l + i] = 1.0;
  OFF_HIP(hipMemcpy(Gt, h_Gt.data(), h_Gt.size() * 8, hipMemcpyHostToDevice));
  for (int sweep = 0; sweep < 30; ++sweep) {
    unsigned h_off = 0;
    OFF_HIP(hipMemset(off, 0, sizeof(unsigned)));
    for (int s = 0; s < lp - 1; ++s)
      hipLaunchKernelGGL(jacobi_kernel, dim3(lp / 2), dim3(256), 0, nullptr, Bm, N, Gt, l, pairs + size_t(s) * lp, off);
    OFF_HIP(hipMemcpy(&h_off, off, sizeof(unsigned), hipMemcpyDeviceToHost));
    float rel;
    std::memcpy(&rel, &h_off, 4);
    if (rel < 1e-14f) break;
    if (sweep == 29) { rc = set_error(MOE_LRC_ESHAPE, "offline_factors: Jacobi sweeps did not converge"); goto done; }
  }
  hipLaunchKernelGGL(row_norm2_kernel, dim3(l), dim3(256), 0, nullptr, Bm, N, norm2);
  OFF_HIP(hipMemcpy(h_norm2.data(), norm2, size_t(l) * 8, hipMemcpyDeviceToHost));
  OFF_HIP(hipMemcpy(h_Gt.data(), Gt, h_Gt.size() * 8, hipMemcpyDeviceToHost));

  // ---- the `rank` largest singular values, in descending order; A = Q G_sel sqrt(sigma), B = rows / sqrt(sigma)
  std::iota(order.begin(), order.end(), 0);
  std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return h_norm2[a] > h_norm2[b]; });
  h_M.assign(size_t(l) * rank, 0.0);
  for (int i = 0; i < rank; ++i) {
    const int src = order[i];
    const double sigma = std::sqrt(h_norm2[src]), root = std::sqrt(sigma);
    if (sigma_host) sigma_host[i] = sigma;
    h_sel[i] = src;
    h_mul[i] = sigma > 0.0 ? 1.0 / root : 0.0;
    for (int j = 0; j < l; ++j) h_M[size_t(j) * rank + i] = h_Gt[size_t(src) * l + j] * root;   // G[j][src] = Gt[src][j]
  }
  OFF_HIP(hipMemcpy(M, h_M.data(), h_M.size() * 8, hipMemcpyHostToDevice));
  OFF_HIP(hipMemcpy(mul, h_mul.data(), size_t(rank) * 8, hipMemcpyHostToDevice));
  OFF_HIP(hipMemcpy(sel, h_sel.data(), size_t(rank) * sizeof(int), hipMemcpyHostToDevice));
  dgemm<false>(K, rank, l, Y, l, M, rank, A_dev, rank);
  hipLaunchKernelGGL(pick_rows_kernel, dim3((N + 255) / 256, rank), dim3(256), 0, nullptr, Bm, N, sel, mul, B_dev);
  if (A_bf16_dev) hipLaunchKernelGGL(to_bf16_kernel, dim3((unsigned)((size_t(K) * rank + 255) / 256)), dim3(256), 0, nullptr, A_dev, size_t(K) * rank, A_bf16_dev);
  if (B_bf16_dev) hipLaunchKernelGGL(to_bf16_kernel, dim3((unsigned)((size_t(rank) * N + 255) / 256)), dim3(256), 0, nullptr, B_dev, size_t(rank) * N, B_bf16_dev);
  OFF_HIP(hipGetLastError());
  OFF_HIP(hipDeviceSynchronize());
done:
  for (void* p : {(void*)Y, (void*)Z, (void*)G, (void*)Bm, (void*)Gt, (void*)norm2, (void*)M, (void*)mul, (void*)bad, (void*)off, (void*)pairs, (void*)sel})
    if (p) (void)hipFree(p);
  return rc;
}

int moe_lrc_offline_allocate_ranks(const double* kappa_host, int n, int r_avg, const int32_t* buckets_host, int n_buckets,
                                   int32_t* ranks_host) {
  if (!kappa_host || !buckets_host || !ranks_host) return set_error(MOE_LRC_EINVAL, "offline_allocate_ranks: null argument");
  if (n <= 0 || n_buckets <= 0 || r_avg < 0) return set_error(MOE_LRC_EINVAL, "offline_allocate_ranks: n, n_buckets must be positive, r_avg not negative");
  for (int i = 0; i < n_buckets; ++i)
    if (buckets_host[i] < 0) return set_error(MOE_LRC_EINVAL, "offline_allocate_ranks: negative bucket value");
  // in descending kurtosis order (equal values: lower index first), every matrix takes the largest
  // bucket value that keeps the running total within n * r_avg
  std::vector<int> order(n);
  std::iota(order.begin(), order.end(), 0);
  std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return kappa_host[a] > kappa_host[b]; });
  const long long budget = (long long)n * r_avg;
  long long used = 0;
  for (int i : order) {
    int best = 0;
    bool any = false;
    for (int j = 0; j < n_buckets; ++j)
      if (used + buckets_host[j] <= budget && (!any || buckets_host[j] > best)) { best = buckets_host[j]; any = true; }
    ranks_host[i] = any ? best : 0;
    used += ranks_host[i];
  }
  return MOE_LRC_OK;
}

int moe_lrc_selftest_half_rounding(const double* in_host, size_t n, uint16_t* out_host) {
  if (!in_host || !out_host) return set_error(MOE_LRC_EINVAL, "selftest_half_rounding: null argument");
  for (size_t i = 0; i < n; ++i) out_host[i] = f64_to_f16_bits(in_host[i]);
  return MOE_LRC_OK;
}

}  // extern "C"
