// Plain fp32-arithmetic causal attention (Sec. 3, Eq. 1-2) restricted to the query's own spatial
// block (Sec. 3.3 "Local attention"; Bs = N gives exact attention), forward and backward.
// Used for fp32 inputs, where no MFMA type holds the operands exactly; four lanes share a query
// (or a key, in the dK/dV kernel) and split the head dimension.
#include "common.h"

namespace {


template <typename T, int D>
__global__ void __launch_bounds__(256) k_attn_fwd_simple(const T* __restrict__ Q, const T* __restrict__ K,
                                                          const T* __restrict__ V, const float* __restrict__ ff,
                                                          T* __restrict__ O, float* __restrict__ LSE, int N, int Bs,
                                                          int Hq, int Hkv, float scale) {
  constexpr int DL = D / 4;
  constexpr int kTile = 4096 / D;  // keys (or queries) staged in LDS per step
  __shared__ float ks[kTile][D + 4];
  __shared__ float vs[kTile][D + 4];
  const int hq = blockIdx.y, b = blockIdx.z, hk = hq / (Hq / Hkv);
  const size_t qh = ((size_t)b * Hq + hq) * N, kh = ((size_t)b * Hkv + hk) * N;
  const int q0 = blockIdx.x * 64;
  const int n = q0 + threadIdx.x / 4, part = threadIdx.x % 4;
  const bool live = n < N;
  float q[DL], acc[DL];
#pragma unroll
  for (int d = 0; d < DL; ++d) {
    q[d] = live ? scale * Elem<T>::ld(Q, (qh + n) * D + part * DL + d) : 0.f;
    acc[d] = 0.f;
  }
  float m = MUSE_NEG_INF, l = 0.f;
  const int kbeg = (q0 / Bs) * Bs;
  const int kend = min(q0 + 64, N);
  const int myb = live ? (n / Bs) * Bs : 0;
  for (int k0 = kbeg; k0 < kend; k0 += kTile) {
    __syncthreads();
    for (int t = threadIdx.x; t < kTile * D; t += 256) {
      int kk = t / D, d = t % D;
      bool ok = k0 + kk < N;
      ks[kk][d] = ok ? Elem<T>::ld(K, (kh + k0 + kk) * D + d) : 0.f;
      vs[kk][d] = ok ? Elem<T>::ld(V, (kh + k0 + kk) * D + d) : 0.f;
    }
    __syncthreads();
    int lim = min(kTile, kend - k0);
    for (int kk = 0; kk < lim; ++kk) {
      float s = 0.f;
#pragma unroll
      for (int d = 0; d < DL; ++d) s = fmaf(q[d], ks[kk][part * DL + d], s);
      s += __shfl_xor(s, 1, 64);
      s += __shfl_xor(s, 2, 64);
      int mpos = k0 + kk;
      if (!live || mpos > n || mpos < myb) continue;
      float mn = fmaxf(m, s);
      float a = __expf(m - mn), p = __expf(s - mn);
      l = l * a + p;
#pragma unroll
      for (int d = 0; d < DL; ++d) acc[d] = acc[d] * a + p * vs[kk][part * DL + d];
      m = mn;
    }
  }
  if (!live) return;
  if (ff) {  // merge the far-field partial softmax state (max, sum, acc[D])
    const float* f = ff + (qh + n) * D;                                   // [acc | (max,sum)] planes
    const float* fm = ff + (size_t)gridDim.z * Hq * N * D + (qh + n) * 2;
    float mf = fm[0], lf = fm[1];
    if (lf > 0.f) {
      float mn = fmaxf(m, mf);
      float a = __expf(m - mn), c = __expf(mf - mn);
      l = l * a + lf * c;
#pragma unroll
      for (int d = 0; d < DL; ++d) acc[d] = acc[d] * a + c * f[part * DL + d];
      m = mn;
    }
  }
  float inv = 1.f / l;
#pragma unroll
  for (int d = 0; d < DL; ++d) Elem<T>::st(O, (qh + n) * D + part * DL + d, acc[d] * inv);
  if (part == 0) LSE[qh + n] = m + __logf(l);
}

template <typename T, int D>
__global__ void __launch_bounds__(256) k_delta(const T* __restrict__ O, const T* __restrict__ dO,
                                                float* __restrict__ delta, size_t rows) {
  size_t row = (size_t)blockIdx.x * 4 + threadIdx.x / 64;
  if (row >= rows) return;
  int lane = threadIdx.x % 64;
  float s = 0.f;
  for (int d = lane; d < D; d += 64) s += Elem<T>::ld(O, row * D + d) * Elem<T>::ld(dO, row * D + d);
  s = wave_sum(s);
  if (lane == 0) delta[row] = s;
}

// dQ: four lanes per query, loop over its keys
template <typename T, int D>
__global__ void __launch_bounds__(256) k_attn_bwd_dq_simple(const T* __restrict__ Q, const T* __restrict__ K,
                                                             const T* __restrict__ V, const T* __restrict__ dO,
                                                             const float* __restrict__ LSE, const float* __restrict__ delta,
                                                             float* __restrict__ dQ, int N, int Bs, int Hq, int Hkv,
                                                             float scale) {
  constexpr int DL = D / 4;
  constexpr int kTile = 4096 / D;  // keys (or queries) staged in LDS per step
  __shared__ float ks[kTile][D + 4];
  __shared__ float vs[kTile][D + 4];
  const int hq = blockIdx.y, b = blockIdx.z, hk = hq / (Hq / Hkv);
  const size_t qh = ((size_t)b * Hq + hq) * N, kh = ((size_t)b * Hkv + hk) * N;
  const int q0 = blockIdx.x * 64;
  const int n = q0 + threadIdx.x / 4, part = threadIdx.x % 4;
  const bool live = n < N;
  float q[DL], g[DL], acc[DL];
#pragma unroll
  for (int d = 0; d < DL; ++d) {
    q[d] = live ? scale * Elem<T>::ld(Q, (qh + n) * D + part * DL + d) : 0.f;
    g[d] = live ? Elem<T>::ld(dO, (qh + n) * D + part * DL + d) : 0.f;
    acc[d] = 0.f;
  }
  const float lse = live ? LSE[qh + n] : 0.f, dl = live ? delta[qh + n] : 0.f;
  const int kbeg = (q0 / Bs) * Bs, kend = min(q0 + 64, N);
  const int myb = live ? (n / Bs) * Bs : 0;
  for (int k0 = kbeg; k0 < kend; k0 += kTile) {
    __syncthreads();
    for (int t = threadIdx.x; t < kTile * D; t += 256) {
      int kk = t / D, d = t % D;
      bool ok = k0 + kk < N;
      ks[kk][d] = ok ? Elem<T>::ld(K, (kh + k0 + kk) * D + d) : 0.f;
      vs[kk][d] = ok ? Elem<T>::ld(V, (kh + k0 + kk) * D + d) : 0.f;
    }
    __syncthreads();
    int lim = min(kTile, kend - k0);
    for (int kk = 0; kk < lim; ++kk) {
      float s = 0.f, dp = 0.f;
#pragma unroll
      for (int d = 0; d < DL; ++d) {
        s = fmaf(q[d], ks[kk][part * DL + d], s);
        dp = fmaf(g[d], vs[kk][part * DL + d], dp);
      }
      s += __shfl_xor(s, 1, 64); s += __shfl_xor(s, 2, 64);
      dp += __shfl_xor(dp, 1, 64); dp += __shfl_xor(dp, 2, 64);
      int mpos = k0 + kk;
      if (!live || mpos > n || mpos < myb) continue;
      float ds = __expf(s - lse) * (dp - dl);
#pragma unroll
      for (int d = 0; d < DL; ++d) acc[d] = fmaf(ds, ks[kk][part * DL + d], acc[d]);
    }
  }
  if (!live) return;
#pragma unroll
  for (int d = 0; d < DL; ++d) dQ[(qh + n) * D + part * DL + d] += scale * acc[d];
}

// dK, dV: four lanes per key, loop over the query heads of the group and their queries n >= m
template <typename T, int D>
__global__ void __launch_bounds__(256) k_attn_bwd_dkv_simple(const T* __restrict__ Q, const T* __restrict__ K,
                                                              const T* __restrict__ V, const T* __restrict__ dO,
                                                              const float* __restrict__ LSE, const float* __restrict__ delta,
                                                              float* __restrict__ dK, float* __restrict__ dV, int N, int Bs,
                                                              int Hq, int Hkv, float scale) {
  constexpr int DL = D / 4;
  constexpr int kTile = 4096 / D;  // keys (or queries) staged in LDS per step
  __shared__ float qs[kTile][D + 4];
  __shared__ float gs[kTile][D + 4];
  __shared__ float ls[kTile], ds_[kTile];
  const int hk = blockIdx.y, b = blockIdx.z, G = Hq / Hkv;
  const size_t kh = ((size_t)b * Hkv + hk) * N;
  const int k0 = blockIdx.x * 64;
  const int m = k0 + threadIdx.x / 4, part = threadIdx.x % 4;
  const bool live = m < N;
  float k[DL], v[DL], ak[DL], av[DL];
#pragma unroll
  for (int d = 0; d < DL; ++d) {
    k[d] = live ? Elem<T>::ld(K, (kh + m) * D + part * DL + d) : 0.f;
    v[d] = live ? Elem<T>::ld(V, (kh + m) * D + part * DL + d) : 0.f;
    ak[d] = av[d] = 0.f;
  }
  const int qend = min(((k0 / Bs) + 1) * Bs, N);  // queries of the same spatial block as the key tile start
  // a tile of 64 keys may straddle blocks when Bs < 64: extend to the block of the last key
  const int qend2 = min(((min(k0 + 63, N - 1) / Bs) + 1) * Bs, N);
  const int myend = live ? min(((m / Bs) + 1) * Bs, N) : 0;
  (void)qend;
  for (int g = 0; g < G; ++g) {
    const size_t qh = ((size_t)b * Hq + (size_t)hk * G + g) * N;
    for (int q0 = k0; q0 < qend2; q0 += kTile) {
      __syncthreads();
      for (int t = threadIdx.x; t < kTile * D; t += 256) {
        int qq = t / D, d = t % D;
        bool ok = q0 + qq < N;
        qs[qq][d] = ok ? scale * Elem<T>::ld(Q, (qh + q0 + qq) * D + d) : 0.f;
        gs[qq][d] = ok ? Elem<T>::ld(dO, (qh + q0 + qq) * D + d) : 0.f;
      }
      if (threadIdx.x < kTile) {
        bool ok = q0 + threadIdx.x < N;
        ls[threadIdx.x] = ok ? LSE[qh + q0 + threadIdx.x] : 0.f;
        ds_[threadIdx.x] = ok ? delta[qh + q0 + threadIdx.x] : 0.f;
      }
      __syncthreads();
      int lim = min(kTile, qend2 - q0);
      for (int qq = 0; qq < lim; ++qq) {
        float s = 0.f, dp = 0.f;
#pragma unroll
        for (int d = 0; d < DL; ++d) {
          s = fmaf(qs[qq][part * DL + d], k[d], s);
          dp = fmaf(gs[qq][part * DL + d], v[d], dp);
        }
        s += __shfl_xor(s, 1, 64); s += __shfl_xor(s, 2, 64);
        dp += __shfl_xor(dp, 1, 64); dp += __shfl_xor(dp, 2, 64);
        int n = q0 + qq;
        if (!live || n < m || n >= myend) continue;
        float p = __expf(s - ls[qq]);
        float dsv = p * (dp - ds_[qq]);
#pragma unroll
        for (int d = 0; d < DL; ++d) {
          ak[d] = fmaf(dsv, qs[qq][part * DL + d], ak[d]);
          av[d] = fmaf(p, gs[qq][part * DL + d], av[d]);
        }
      }
    }
  }
  if (!live) return;
#pragma unroll
  for (int d = 0; d < DL; ++d) {
    dK[(kh + m) * D + part * DL + d] += ak[d];
    dV[(kh + m) * D + part * DL + d] += av[d];
  }
}

template <typename T>
__global__ void k_cast(const float* __restrict__ src, T* __restrict__ dst, size_t n, float mul) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) Elem<T>::st(dst, i, src[i] * mul);
}

__global__ void k_fill_i32(int32_t* __restrict__ dst, size_t n, int32_t v) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) dst[i] = v;
}

__global__ void k_fill(float* __restrict__ dst, size_t n, float v) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) dst[i] = v;
}

}  // namespace

// implemented in attn_mfma.hip
int muse_launch_attn_fwd_mfma(const MuseDims& d, int Bs, const void* Q, const void* K, const void* V,
                              const float* ff, void* O, float* LSE, hipStream_t st);
int muse_launch_attn_bwd_mfma(const MuseDims& d, int Bs, const void* Q, const void* K, const void* V,
                              const void* dO, const float* LSE, const float* delta, float* dQacc,
                              float* dKacc, float* dVacc, hipStream_t st);

int muse_launch_attn_fwd(const MuseDims& d, int Bs, const void* Q, const void* K, const void* V,
                         const float* ff, void* O, float* LSE, hipStream_t st) {
  if (d.dtype == MUSE_DTYPE_BF16) return muse_launch_attn_fwd_mfma(d, Bs, Q, K, V, ff, O, LSE, st);
  dim3 g((d.N + 63) / 64, d.Hq, d.B);
  if (d.D == 64)
    { MuseProf prof_("k_attn_fwd_simple", st); hipLaunchKernelGGL((k_attn_fwd_simple<float, 64>), g, dim3(256), 0, st, (const float*)Q, (const float*)K,
                       (const float*)V, ff, (float*)O, LSE, d.N, Bs, d.Hq, d.Hkv, d.scale); }
  else
    { MuseProf prof_("k_attn_fwd_simple", st); hipLaunchKernelGGL((k_attn_fwd_simple<float, 128>), g, dim3(256), 0, st, (const float*)Q, (const float*)K,
                       (const float*)V, ff, (float*)O, LSE, d.N, Bs, d.Hq, d.Hkv, d.scale); }
  MUSE_LAUNCH_CHECK();
  return MUSE_OK;
}

int muse_launch_delta(const MuseDims& d, const void* O, const void* dO, float* delta, hipStream_t st) {
  size_t rows = (size_t)d.B * d.Hq * d.N;
  dim3 g((unsigned)((rows + 3) / 4));
  if (d.dtype == MUSE_DTYPE_BF16) {
    if (d.D == 64) { MuseProf prof_("k_delta", st); hipLaunchKernelGGL((k_delta<bf16_t, 64>), g, dim3(256), 0, st, (const bf16_t*)O, (const bf16_t*)dO, delta, rows); }
    else { MuseProf prof_("k_delta", st); hipLaunchKernelGGL((k_delta<bf16_t, 128>), g, dim3(256), 0, st, (const bf16_t*)O, (const bf16_t*)dO, delta, rows); }
  } else {
    if (d.D == 64) { MuseProf prof_("k_delta", st); hipLaunchKernelGGL((k_delta<float, 64>), g, dim3(256), 0, st, (const float*)O, (const float*)dO, delta, rows); }
    else { MuseProf prof_("k_delta", st); hipLaunchKernelGGL((k_delta<float, 128>), g, dim3(256), 0, st, (const float*)O, (const float*)dO, delta, rows); }
  }
  MUSE_LAUNCH_CHECK();
  return MUSE_OK;
}

int muse_launch_attn_bwd(const MuseDims& d, int Bs, const void* Q, const void* K, const void* V,
                         const void* dO, const float* LSE, const float* delta, float* dQacc,
                         float* dKacc, float* dVacc, hipStream_t st) {
  if (d.dtype == MUSE_DTYPE_BF16)  // the matrix-core kernels write every row once
    return muse_launch_attn_bwd_mfma(d, Bs, Q, K, V, dO, LSE, delta, dQacc, dKacc, dVacc, st);
  {  // the fp32 kernels add to their rows
    const size_t q = (size_t)d.B * d.Hq * d.N * d.D, k = (size_t)d.B * d.Hkv * d.N * d.D;
    int rc;
    if ((rc = muse_launch_fill(dQacc, q, 0.f, st)) || (rc = muse_launch_fill(dKacc, k, 0.f, st)) ||
        (rc = muse_launch_fill(dVacc, k, 0.f, st)))
      return rc;
  }
  dim3 gq((d.N + 63) / 64, d.Hq, d.B), gk((d.N + 63) / 64, d.Hkv, d.B);
  const float *q = (const float*)Q, *k = (const float*)K, *v = (const float*)V, *g = (const float*)dO;
  if (d.D == 64) {
    { MuseProf prof_("k_attn_bwd_dq_simple", st); hipLaunchKernelGGL((k_attn_bwd_dq_simple<float, 64>), gq, dim3(256), 0, st, q, k, v, g, LSE, delta, dQacc, d.N, Bs, d.Hq, d.Hkv, d.scale); }
    { MuseProf prof_("k_attn_bwd_dkv_simple", st); hipLaunchKernelGGL((k_attn_bwd_dkv_simple<float, 64>), gk, dim3(256), 0, st, q, k, v, g, LSE, delta, dKacc, dVacc, d.N, Bs, d.Hq, d.Hkv, d.scale); }
  } else {
    { MuseProf prof_("k_attn_bwd_dq_simple", st); hipLaunchKernelGGL((k_attn_bwd_dq_simple<float, 128>), gq, dim3(256), 0, st, q, k, v, g, LSE, delta, dQacc, d.N, Bs, d.Hq, d.Hkv, d.scale); }
    { MuseProf prof_("k_attn_bwd_dkv_simple", st); hipLaunchKernelGGL((k_attn_bwd_dkv_simple<float, 128>), gk, dim3(256), 0, st, q, k, v, g, LSE, delta, dKacc, dVacc, d.N, Bs, d.Hq, d.Hkv, d.scale); }
  }
  MUSE_LAUNCH_CHECK();
  return MUSE_OK;
}

int muse_launch_cast(const float* src, void* dst, size_t n, int dst_dtype, float mul, hipStream_t st) {
  unsigned blocks = (unsigned)((n + 1023) / 1024 > 65535 * 16 ? 65535 * 16 : (n + 1023) / 1024);
  if (blocks == 0) return MUSE_OK;
  if (dst_dtype == MUSE_DTYPE_BF16) { MuseProf prof_("k_cast", st); hipLaunchKernelGGL(k_cast<bf16_t>, dim3(blocks), dim3(256), 0, st, src, (bf16_t*)dst, n, mul); }
  else { MuseProf prof_("k_cast", st); hipLaunchKernelGGL(k_cast<float>, dim3(blocks), dim3(256), 0, st, src, (float*)dst, n, mul); }
  MUSE_LAUNCH_CHECK();
  return MUSE_OK;
}

int muse_launch_fill(float* dst, size_t n, float v, hipStream_t st) {
  unsigned blocks = (unsigned)((n + 1023) / 1024 > 65535 * 16 ? 65535 * 16 : (n + 1023) / 1024);
  if (blocks == 0) return MUSE_OK;
  { MuseProf prof_("k_fill", st); hipLaunchKernelGGL(k_fill, dim3(blocks), dim3(256), 0, st, dst, n, v); }
  MUSE_LAUNCH_CHECK();
  return MUSE_OK;
}

int muse_launch_fill_i32(int32_t* dst, size_t n, int32_t v, hipStream_t st) {
  unsigned blocks = (unsigned)((n + 1023) / 1024 > 65535 * 16 ? 65535 * 16 : (n + 1023) / 1024);
  if (blocks == 0) return MUSE_OK;
  { MuseProf prof_("k_fill_i32", st); hipLaunchKernelGGL(k_fill_i32, dim3(blocks), dim3(256), 0, st, dst, n, v); }
  MUSE_LAUNCH_CHECK();
  return MUSE_OK;
}
