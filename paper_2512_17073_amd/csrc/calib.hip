// Measurement hook: what this device sustains on the three resources the roofline figures of the
// layer are priced against: streaming reads of device memory (the decode path's bound), pinned
// host -> device copies (the staged mode's bound) and dense f16 matrix-core throughput (the
// many-rows path's bound).  Not part of the hot path: allocates its own buffers and synchronises.
#include <algorithm>
#include <cstring>
#include <vector>

#include "internal.h"

namespace lrc {

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float4_t __attribute__((ext_vector_type(4)));

// Every wavefront reads 1 KB pieces (16 bytes per lane) of the buffer, DEPTH pieces in flight, the
// wavefronts of the launch sweeping the buffer together: piece i of round r is read by wavefront
// (i mod waves).  The xor of everything read is stored only if it has an improbable value, which
// keeps the loads alive without a write stream.
template <int DEPTH>
__global__ __launch_bounds__(256) void stream_read_kernel(const u32x4* __restrict__ buf, size_t pieces, uint32_t* __restrict__ sink) {
  const int lane = threadIdx.x & 63;
  const size_t wave = (size_t(blockIdx.x) * 256 + threadIdx.x) >> 6, waves = size_t(gridDim.x) * 4;
  u32x4 acc = u32x4{0, 0, 0, 0};
  for (size_t p = wave; p < pieces; p += waves * DEPTH) {
    u32x4 v[DEPTH];
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) {
      const size_t q = p + size_t(d) * waves;
      v[d] = q < pieces ? __builtin_nontemporal_load(buf + q * 64 + lane) : u32x4{0, 0, 0, 0};
    }
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) acc ^= v[d];
  }
  const uint32_t x = acc[0] ^ acc[1] ^ acc[2] ^ acc[3];
  if (x == 0x9e3779b9u) sink[0] = x;
}

// Dense f16 matrix-core rate: every wavefront issues `iters` rounds of eight independent
// v_mfma_f32_16x16x32_f16 on registers (no memory traffic).  The scheduling barriers keep the eight
// accumulators apart (left alone, the compiler rotates them through overlapping registers, which
// chains the instructions and halves the rate).
__global__ __launch_bounds__(256) void mfma_rate_kernel(int iters, float* __restrict__ sink) {
  half8_t a, b;
#pragma unroll
  for (int i = 0; i < 8; ++i) { a[i] = (_Float16)(0.001f * float((threadIdx.x + i) & 63)); b[i] = (_Float16)(0.002f * float(i + 1)); }
  float4_t acc[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) acc[j] = float4_t{0.f, 0.f, 0.f, 0.f};
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, acc[j], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  float s = 0.f;
#pragma unroll
  for (int j = 0; j < 8; ++j) s += acc[j][0] + acc[j][1] + acc[j][2] + acc[j][3];
  if (s == 12345.678f) sink[0] = s;
}

// The same with v_mfma_f32_32x32x16_f16 (four independent 32x32 accumulators per wavefront).
typedef float float16_t __attribute__((ext_vector_type(16)));
__global__ __launch_bounds__(256) void mfma_rate32_kernel(int iters, float* __restrict__ sink) {
  half8_t a, b;
#pragma unroll
  for (int i = 0; i < 8; ++i) { a[i] = (_Float16)(0.001f * float((threadIdx.x + i) & 63)); b[i] = (_Float16)(0.002f * float(i + 1)); }
  float16_t acc[4];
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[j][i] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, acc[j], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  float s = 0.f;
#pragma unroll
  for (int j = 0; j < 4; ++j) s += acc[j][0] + acc[j][5] + acc[j][10] + acc[j][15];
  if (s == 12345.678f) sink[0] = s;
}

// How far vector ALU work hides behind MFMAs: two wavefronts per SIMD (512 threads, one block per
// CU) issue rounds of eight independent v_mfma_f32_16x16x32_f16, each followed by NV independent
// packed fp16 FMAs (the instruction the kernels dequantize with).
template <int NV>
__global__ __launch_bounds__(512) void mfma_valu_kernel(int iters, float* __restrict__ sink) {
  half8_t a, b;
#pragma unroll
  for (int i = 0; i < 8; ++i) { a[i] = (_Float16)(0.001f * float((threadIdx.x + i) & 63)); b[i] = (_Float16)(0.002f * float(i + 1)); }
  float4_t acc[8];
  uint32_t v[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) { acc[j] = float4_t{0.f, 0.f, 0.f, 0.f}; v[j] = threadIdx.x * 77u + j; }
  const uint32_t c1 = 0x3c003c00u, c2 = 0x00010001u;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, acc[j], 0, 0, 0);
#pragma unroll
      for (int n = 0; n < NV; ++n) asm volatile("v_pk_fma_f16 %0, %0, %1, %2" : "+v"(v[(j * NV + n) & 7]) : "v"(c1), "v"(c2));
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  float s = 0.f;
  uint32_t x = 0;
#pragma unroll
  for (int j = 0; j < 8; ++j) { s += acc[j][0] + acc[j][3]; x ^= v[j]; }
  if (s == 12345.678f || x == 0x12345u) sink[0] = s;
}

// A loop shaped like a sub-step of the decode-flavour FFN kernel, four wavefronts per SIMD (one
// 1024-thread block per CU): 8 mask and 8 packed-FMA operations make the A operands of two streams,
// then 2 MT MFMAs (v_mfma_f32_16x16x32_f16) multiply them with MT activation fragments.  MODE 0: both,
// 1: the MFMAs alone, 2: the vector operations alone.
template <int MT, int MODE>
__global__ __launch_bounds__(1024) void substep_kernel(int iters, float* __restrict__ sink) {
  half8_t b[MT];
  float4_t acc[MT][2];
  uint32_t cw[2][4], v[2][4];
#pragma unroll
  for (int t = 0; t < MT; ++t) {
#pragma unroll
    for (int i = 0; i < 8; ++i) b[t][i] = (_Float16)(0.001f * float((threadIdx.x & 15) + i + t));
#pragma unroll
    for (int m = 0; m < 2; ++m) acc[t][m] = float4_t{0.f, 0.f, 0.f, 0.f};
  }
#pragma unroll
  for (int m = 0; m < 2; ++m)
#pragma unroll
    for (int j = 0; j < 4; ++j) { cw[m][j] = threadIdx.x * 2654435761u + 97u * (4 * m + j); v[m][j] = 0x3c003c00u; }
  const uint32_t mask = 0x00300030u, c1 = 0x64006400u, c2 = 0x00010001u;
  for (int it = 0; it < iters; ++it) {
    if (MODE != 1) {
#pragma unroll
      for (int m = 0; m < 2; ++m)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          uint32_t f;
          asm volatile("v_and_b32 %0, %1, %2" : "=v"(f) : "v"(cw[m][j]), "v"(mask));
          asm volatile("v_pk_fma_f16 %0, %1, %2, %3" : "=v"(v[m][j]) : "v"(f), "v"(c1), "v"(c2));
        }
    }
    if (MODE != 2) {
#pragma unroll
      for (int t = 0; t < MT; ++t)
#pragma unroll
        for (int m = 0; m < 2; ++m)
          acc[t][m] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8_t, make_uint4(v[m][0], v[m][1], v[m][2], v[m][3])),
                                                            b[t], acc[t][m], 0, 0, 0);
    }
    __builtin_amdgcn_sched_barrier(0);
  }
  float s = 0.f;
  uint32_t x = 0;
#pragma unroll
  for (int t = 0; t < MT; ++t)
#pragma unroll
    for (int m = 0; m < 2; ++m) { s += acc[t][m][0] + acc[t][m][3]; x ^= v[m][t]; }
  if (s == 12345.678f || x == 0x12345u) sink[0] = s;
}

}  // namespace

}  // namespace lrc

using namespace lrc;

#define CAL_HIP(expr)                                                                               \
  do {                                                                                              \
    hipError_t e_ = (expr);                                                                         \
    if (e_ != hipSuccess) {                                                                         \
      rc = set_error(MOE_LRC_EHIP, std::string("calibrate: ") + #expr + ": " + hipGetErrorString(e_)); \
      goto done;                                                                                    \
    }                                                                                               \
  } while (0)

extern "C" int moe_lrc_calibrate(int kind, size_t bytes, int reps, double* result) {
  if (!result || reps < 1 || reps > 1000) return set_error(MOE_LRC_EINVAL, "calibrate: result is null or reps outside 1..1000");
  if (kind < MOE_LRC_CAL_HBM_READ || kind > MOE_LRC_CAL_SUBSTEP) return set_error(MOE_LRC_EINVAL, "calibrate: unknown kind");
  if (kind == MOE_LRC_CAL_SUBSTEP && ((bytes & 15) < 1 || (bytes & 15) > 2 || (bytes >> 4) > 2))
    return set_error(MOE_LRC_EINVAL, "calibrate: sub-step: bytes = row tiles (1 or 2) + 16 * mode (0, 1 or 2)");
  if (kind == MOE_LRC_CAL_MFMA_VALU && bytes != 0 && bytes != 2 && bytes != 4 && bytes != 8 && bytes != 16)
    return set_error(MOE_LRC_EINVAL, "calibrate: the number of FMAs per MFMA must be 0, 2, 4, 8 or 16");
  if (kind < MOE_LRC_CAL_MFMA_F16 && (bytes < (1u << 20) || bytes > (size_t(16) << 30)))
    return set_error(MOE_LRC_EINVAL, "calibrate: bytes must be between 1 MiB and 16 GiB");
  int rc = MOE_LRC_OK, dev = 0, n_cu = 0;
  void *dbuf = nullptr, *hbuf = nullptr;
  uint32_t* sink = nullptr;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  std::vector<float> ms;
  float t = 0.f;
  CAL_HIP(hipGetDevice(&dev));
  CAL_HIP(hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev));
  CAL_HIP(hipEventCreate(&e0));
  CAL_HIP(hipEventCreate(&e1));
  CAL_HIP(hipMalloc((void**)&sink, 256));
  if (kind == MOE_LRC_CAL_HBM_READ) {
    // the buffer should be several times the last-level cache, so that every pass comes from HBM
    bytes &= ~size_t(1023);
    CAL_HIP(hipMalloc(&dbuf, bytes));
    CAL_HIP(hipMemset(dbuf, 1, bytes));
    CAL_HIP(hipDeviceSynchronize());
    for (int i = 0; i < reps + 1; ++i) {          // (first pass untimed)
      CAL_HIP(hipEventRecord(e0, nullptr));
      hipLaunchKernelGGL(stream_read_kernel<4>, dim3(n_cu * 8), dim3(256), 0, nullptr, (const u32x4*)dbuf, bytes / 1024, sink);
      CAL_HIP(hipEventRecord(e1, nullptr));
      CAL_HIP(hipEventSynchronize(e1));
      CAL_HIP(hipEventElapsedTime(&t, e0, e1));
      if (i > 0) ms.push_back(t);
    }
    std::sort(ms.begin(), ms.end());
    *result = double(bytes) / (ms[ms.size() / 2] * 1e-3) / 1e9;      // GB/s, median pass
  } else if (kind == MOE_LRC_CAL_H2D) {
    CAL_HIP(hipHostMalloc(&hbuf, bytes, hipHostMallocDefault));
    memset(hbuf, 1, bytes);
    CAL_HIP(hipMalloc(&dbuf, bytes));
    for (int i = 0; i < reps + 1; ++i) {
      CAL_HIP(hipEventRecord(e0, nullptr));
      CAL_HIP(hipMemcpyAsync(dbuf, hbuf, bytes, hipMemcpyHostToDevice, nullptr));
      CAL_HIP(hipEventRecord(e1, nullptr));
      CAL_HIP(hipEventSynchronize(e1));
      CAL_HIP(hipEventElapsedTime(&t, e0, e1));
      if (i > 0) ms.push_back(t);
    }
    std::sort(ms.begin(), ms.end());
    *result = double(bytes) / (ms[ms.size() / 2] * 1e-3) / 1e9;      // GB/s
  } else if (kind == MOE_LRC_CAL_SUBSTEP) {
    const int iters = 8192, mt = int(bytes & 15), mode = int(bytes >> 4);
    for (int i = 0; i < reps + 1; ++i) {
      CAL_HIP(hipEventRecord(e0, nullptr));
      const dim3 g(n_cu), b(1024);
      if (mt == 1 && mode == 0) hipLaunchKernelGGL((substep_kernel<1, 0>), g, b, 0, nullptr, iters, (float*)sink);
      else if (mt == 1 && mode == 1) hipLaunchKernelGGL((substep_kernel<1, 1>), g, b, 0, nullptr, iters, (float*)sink);
      else if (mt == 1) hipLaunchKernelGGL((substep_kernel<1, 2>), g, b, 0, nullptr, iters, (float*)sink);
      else if (mode == 0) hipLaunchKernelGGL((substep_kernel<2, 0>), g, b, 0, nullptr, iters, (float*)sink);
      else if (mode == 1) hipLaunchKernelGGL((substep_kernel<2, 1>), g, b, 0, nullptr, iters, (float*)sink);
      else hipLaunchKernelGGL((substep_kernel<2, 2>), g, b, 0, nullptr, iters, (float*)sink);
      CAL_HIP(hipEventRecord(e1, nullptr));
      CAL_HIP(hipEventSynchronize(e1));
      CAL_HIP(hipEventElapsedTime(&t, e0, e1));
      if (i > 0) ms.push_back(t);
    }
    std::sort(ms.begin(), ms.end());
    *result = ms[ms.size() / 2] * 1e6 / (double(iters) * 4);         // ns of SIMD time per sub-step of one wavefront
  } else if (kind == MOE_LRC_CAL_MFMA_VALU) {
    const int iters = 4096;
    for (int i = 0; i < reps + 1; ++i) {
      CAL_HIP(hipEventRecord(e0, nullptr));
      switch (bytes) {
        case 0: hipLaunchKernelGGL(mfma_valu_kernel<0>, dim3(n_cu), dim3(512), 0, nullptr, iters, (float*)sink); break;
        case 2: hipLaunchKernelGGL(mfma_valu_kernel<2>, dim3(n_cu), dim3(512), 0, nullptr, iters, (float*)sink); break;
        case 4: hipLaunchKernelGGL(mfma_valu_kernel<4>, dim3(n_cu), dim3(512), 0, nullptr, iters, (float*)sink); break;
        case 8: hipLaunchKernelGGL(mfma_valu_kernel<8>, dim3(n_cu), dim3(512), 0, nullptr, iters, (float*)sink); break;
        default: hipLaunchKernelGGL(mfma_valu_kernel<16>, dim3(n_cu), dim3(512), 0, nullptr, iters, (float*)sink); break;
      }
      CAL_HIP(hipEventRecord(e1, nullptr));
      CAL_HIP(hipEventSynchronize(e1));
      CAL_HIP(hipEventElapsedTime(&t, e0, e1));
      if (i > 0) ms.push_back(t);
    }
    std::sort(ms.begin(), ms.end());
    *result = ms[ms.size() / 2] * 1e6 / (double(iters) * 8 * 2);      // ns per MFMA (and its FMAs) on one SIMD
  } else {
    const int iters = 4096, blocks = n_cu * 8;
    for (int i = 0; i < reps + 1; ++i) {
      CAL_HIP(hipEventRecord(e0, nullptr));
      if (kind == MOE_LRC_CAL_MFMA_F16) hipLaunchKernelGGL(mfma_rate_kernel, dim3(blocks), dim3(256), 0, nullptr, iters, (float*)sink);
      else hipLaunchKernelGGL(mfma_rate32_kernel, dim3(blocks), dim3(256), 0, nullptr, iters, (float*)sink);
      CAL_HIP(hipEventRecord(e1, nullptr));
      CAL_HIP(hipEventSynchronize(e1));
      CAL_HIP(hipEventElapsedTime(&t, e0, e1));
      if (i > 0) ms.push_back(t);
    }
    std::sort(ms.begin(), ms.end());
    const double flops = double(blocks) * 4 * iters * (kind == MOE_LRC_CAL_MFMA_F16 ? 8 * (2.0 * 16 * 16 * 32) : 4 * (2.0 * 32 * 32 * 16));
    *result = flops / (ms[ms.size() / 2] * 1e-3) / 1e12;             // TFLOP/s
  }
  CAL_HIP(hipGetLastError());
done:
  if (dbuf) (void)hipFree(dbuf);
  if (hbuf) (void)hipHostFree(hbuf);
  if (sink) (void)hipFree(sink);
  if (e0) (void)hipEventDestroy(e0);
  if (e1) (void)hipEventDestroy(e1);
  return rc;
}
