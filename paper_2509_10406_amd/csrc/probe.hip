// Measurement aid, not part of the method: what a plain streaming copy and a loop of independent bf16 MFMAs reach on
// the device the library runs on.  The roofline fractions a benchmark reports against the published peaks (8 TB/s,
// 2.5 PFLOP/s) can then be read against what the box delivers to the simplest possible kernel of each kind.
#include "common.h"

namespace {

// every thread moves 16 bytes per step; consecutive lanes take consecutive vectors, a workgroup strides the grid
__global__ void __launch_bounds__(256) k_probe_copy(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n) {
  const size_t stride = (size_t)gridDim.x * 256;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += stride) dst[i] = src[i];
}

// four independent accumulator tiles per wave: the matrix pipe always has an instruction whose operands are ready
__global__ void __launch_bounds__(256) k_probe_mfma(float* __restrict__ out, int iters) {
  bf16x8_t a, b;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    a[e] = (__bf16)(float)((threadIdx.x + e) % 3);
    b[e] = (__bf16)(float)((threadIdx.x + 2 * e) % 5);
  }
  f32x16_t c[4];
#pragma unroll
  for (int t = 0; t < 4; ++t)
#pragma unroll
    for (int e = 0; e < 16; ++e) c[t][e] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int t = 0; t < 4; ++t) c[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c[t], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int t = 0; t < 4; ++t)
#pragma unroll
    for (int e = 0; e < 16; ++e) s += c[t][e];
  out[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
}

struct Events {
  hipEvent_t a = nullptr, b = nullptr;
  ~Events() {
    if (a) (void)hipEventDestroy(a);
    if (b) (void)hipEventDestroy(b);
  }
};

}  // namespace

extern "C" int muse_probe_peaks(void* buf, size_t bytes, double* copy_gbps, double* mfma_bf16_tflops, void* stream) {
  constexpr int kGrid = 256 * 8, kIters = 4096, kReps = 5;
  if (!buf || !copy_gbps || !mfma_bf16_tflops) return MUSE_ERR_INVALID_ARG;
  if (((uintptr_t)buf & 255) != 0) return MUSE_ERR_INVALID_ARG;
  if (bytes < ((size_t)1 << 30)) return MUSE_ERR_WORKSPACE_TOO_SMALL;  // well beyond the 256 MB last-level cache
  hipStream_t st = (hipStream_t)stream;
  Events ev;
  MUSE_HIP_CHECK(hipEventCreate(&ev.a));
  MUSE_HIP_CHECK(hipEventCreate(&ev.b));
  const size_t half = (bytes / 2) & ~(size_t)255, n = half / 16;
  const uint4* src = (const uint4*)buf;
  uint4* dst = (uint4*)((char*)buf + half);
  float best_copy = 0.f, best_mfma = 0.f;
  for (int rep = 0; rep < kReps + 1; ++rep) {  // the first repetition warms up
    MUSE_HIP_CHECK(hipEventRecord(ev.a, st));
    hipLaunchKernelGGL(k_probe_copy, dim3(kGrid * 4), dim3(256), 0, st, src, dst, n);
    MUSE_HIP_CHECK(hipEventRecord(ev.b, st));
    MUSE_HIP_CHECK(hipEventSynchronize(ev.b));
    float ms = 0.f;
    MUSE_HIP_CHECK(hipEventElapsedTime(&ms, ev.a, ev.b));
    if (rep > 0 && (best_copy == 0.f || ms < best_copy)) best_copy = ms;
  }
  for (int rep = 0; rep < kReps + 1; ++rep) {
    MUSE_HIP_CHECK(hipEventRecord(ev.a, st));
    hipLaunchKernelGGL(k_probe_mfma, dim3(kGrid), dim3(256), 0, st, (float*)buf, kIters);
    MUSE_HIP_CHECK(hipEventRecord(ev.b, st));
    MUSE_HIP_CHECK(hipEventSynchronize(ev.b));
    float ms = 0.f;
    MUSE_HIP_CHECK(hipEventElapsedTime(&ms, ev.a, ev.b));
    if (rep > 0 && (best_mfma == 0.f || ms < best_mfma)) best_mfma = ms;
  }
  MUSE_HIP_CHECK(hipGetLastError());
  *copy_gbps = 2.0 * (double)half / (best_copy * 1e-3) / 1e9;  // bytes read plus bytes written
  const double flop = (double)kGrid * 4 /*waves*/ * kIters * 4 /*tiles*/ * (2.0 * 32 * 32 * 16);
  *mfma_bf16_tflops = flop / (best_mfma * 1e-3) / 1e12;
  return MUSE_OK;
}
