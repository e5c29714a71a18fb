// Dipole correction of the monopole-only mode (App. B "Dipole Correction", Eq. "premerge", with the shared
// untilted covariances of "Untilted (Partially Specialized) Covariances"), forward only, r = 0.
//
// Causal form: the key set of cluster j seen from query block b is its keys in the blocks before b (the set the
// accumulated summaries describe).  Three stages:
//   1. k_dipole_cov    Cov_0jb(v,k) = E[v k^T] - E[v] E[k]^T over that set, equal weights, for every (kv head, key
//                      block prefix, key cluster): running sums over the bucketed key rows, one workgroup per cluster;
//   2. k_dipole_merge  C-bar_ib = sum_j p_ib(j) Cov_0jb,  p_ib = softmax_j of the accumulated log-masses A-mu_ijb:
//                      a [Cq x Ck] x [Ck x D^2] product per (head, block);
//   3. k_dipole_apply  per query n of block b >= 1:  acc_n += l_n C-bar_ib q~_n, where (acc, l) is the far-field
//                      partial softmax state (acc = sum_j e^(score_j - m) v-bar_j, l = sum_j e^(score_j - m)); the
//                      block-diagonal kernel then merges it with the local block, which weights the correction with
//                      the far field's share of the softmax mass.  The masses (scores) are left unchanged.
// All arithmetic is fp32.
#include "ff_common.h"

namespace {

// thread t owns the 4 x 4 (D = 64) or 8 x 8 (D = 128) block of the D x D matrix at rows (value dims) RB * (t / (D/RB)),
// columns (key dims) RB * (t % (D/RB)); D*D = 256 RB^2
template <typename T, int D>
__global__ void __launch_bounds__(256) k_dipole_cov(const T* __restrict__ Ks, const T* __restrict__ Vs,
                                                     const int32_t* __restrict__ off_k, float* __restrict__ cov,
                                                     int N, int nb, int Ck) {
  constexpr int RB = D / 16, CH = 16;  // keys staged per step
  __shared__ float kk[CH][D], vv[CH][D];
  const int j = blockIdx.x, hk = blockIdx.y, NBm = nb - 1;
  const int t = threadIdx.x, a0 = RB * (t / (D / RB)), c0 = RB * (t % (D / RB));
  const int32_t* ok = off_k + (size_t)hk * ((size_t)nb * Ck + 1);
  float svk[RB][RB], sv[RB], sk[RB];
#pragma unroll
  for (int a = 0; a < RB; ++a) {
    sv[a] = 0.f; sk[a] = 0.f;
#pragma unroll
    for (int c = 0; c < RB; ++c) svk[a][c] = 0.f;
  }
  int cnt = 0;
  for (int b = 0; b < NBm; ++b) {
    const int lo = ok[b * Ck + j], hi = ok[b * Ck + j + 1];
    for (int m0 = lo; m0 < hi; m0 += CH) {
      const int rows = min(CH, hi - m0);
      __syncthreads();
      for (int e = t; e < rows * D; e += 256) {
        const int r = e / D, d = e % D;
        kk[r][d] = Elem<T>::ld(Ks, ((size_t)hk * N + m0 + r) * D + d);
        vv[r][d] = Elem<T>::ld(Vs, ((size_t)hk * N + m0 + r) * D + d);
      }
      __syncthreads();
      for (int r = 0; r < rows; ++r) {
        float kv[RB], vl[RB];
#pragma unroll
        for (int x = 0; x < RB; ++x) { kv[x] = kk[r][c0 + x]; vl[x] = vv[r][a0 + x]; }
#pragma unroll
        for (int a = 0; a < RB; ++a) {
          sv[a] += vl[a]; sk[a] += kv[a];
#pragma unroll
          for (int c = 0; c < RB; ++c) svk[a][c] = fmaf(vl[a], kv[c], svk[a][c]);
        }
      }
    }
    cnt += hi - lo;
    // the keys of blocks 0..b are what query block b + 1 sees
    float* out = cov + ((((size_t)hk * NBm + b) * Ck + j) * D) * D;
    const float inv = cnt > 0 ? 1.f / (float)cnt : 0.f;
#pragma unroll
    for (int a = 0; a < RB; ++a)
#pragma unroll
      for (int c = 0; c < RB; ++c)
        out[(size_t)(a0 + a) * D + c0 + c] = svk[a][c] * inv - (sv[a] * inv) * (sk[c] * inv);
  }
}

// C-bar[h][b][i][:] = sum_j softmax_j(A_mu[h][b][i][:])[j] cov[hk][b][j][:]; a workgroup takes 16 query clusters x 256
// matrix entries, a thread one entry for the 16 query clusters
__global__ void __launch_bounds__(256) k_dipole_merge(const float* __restrict__ A_mu, const float* __restrict__ cov,
                                                       float* __restrict__ cbar, int h0, int NBm, int Cq, int Ck, int DD,
                                                       int Hq, int Hkv) {
  constexpr int TI = 16, JC = 32;
  __shared__ float ps[TI][JC];
  __shared__ float mx_s[TI], zi_s[TI];
  const int hl = blockIdx.z / NBm, b = blockIdx.z % NBm, hq = h0 + hl;
  const int hk = (hq / Hq) * Hkv + (hq % Hq) / (Hq / Hkv);
  const int i0 = blockIdx.y * TI, col = blockIdx.x * 256 + threadIdx.x;
  const int t = threadIdx.x, wave = t / 64, lane = t % 64;
  const float* am = A_mu + (((size_t)hl * NBm + b) * Cq) * Ck;
  // softmax statistics of the 16 rows: wave w takes rows 4 w .. 4 w + 3
  for (int rr = 0; rr < 4; ++rr) {
    const int row = 4 * wave + rr, i = i0 + row;
    float m = MUSE_NEG_INF;
    if (i < Cq)
      for (int jj = lane; jj < Ck; jj += 64) m = fmaxf(m, am[(size_t)i * Ck + jj]);
    m = wave_max(m);
    float z = 0.f;
    if (i < Cq && m > MUSE_NEG_INF)
      for (int jj = lane; jj < Ck; jj += 64) z += __expf(am[(size_t)i * Ck + jj] - m);
    z = wave_sum(z);
    if (lane == 0) { mx_s[row] = m; zi_s[row] = z > 0.f ? 1.f / z : 0.f; }
  }
  float acc[TI];
#pragma unroll
  for (int r = 0; r < TI; ++r) acc[r] = 0.f;
  const float* cv = cov + (((size_t)hk * NBm + b) * Ck) * DD;
  for (int j0 = 0; j0 < Ck; j0 += JC) {
    __syncthreads();
    for (int e = t; e < TI * JC; e += 256) {
      const int row = e / JC, jj = j0 + e % JC, i = i0 + row;
      float p = 0.f;
      if (i < Cq && jj < Ck && zi_s[row] > 0.f) p = __expf(am[(size_t)i * Ck + jj] - mx_s[row]) * zi_s[row];
      ps[row][e % JC] = p;
    }
    __syncthreads();
    if (col < DD) {
      const int jn = min(JC, Ck - j0);
      for (int jj = 0; jj < jn; ++jj) {
        const float c = cv[(size_t)(j0 + jj) * DD + col];
#pragma unroll
        for (int r = 0; r < TI; ++r) acc[r] = fmaf(ps[r][jj], c, acc[r]);
      }
    }
  }
  if (col < DD)
#pragma unroll
    for (int r = 0; r < TI; ++r)
      if (i0 + r < Cq) cbar[((((size_t)hl * NBm + b) * Cq + i0 + r) * DD) + col] = acc[r];
}

// one wave per query of blocks >= 1 (bucketed order, so that neighbours share the matrix): acc_n += l_n C-bar q~_n
template <typename T, int D>
__global__ void __launch_bounds__(256) k_dipole_apply(const T* __restrict__ Q, const float* __restrict__ qc,
                                                       const float* __restrict__ cbar, const int32_t* __restrict__ perm_q,
                                                       const int32_t* __restrict__ aq, float* __restrict__ ff_acc,
                                                       const float* __restrict__ ff_ml, int h0, int N, int Bs, int nb,
                                                       int Cq, float scale) {
  __shared__ float qts[4][D];
  const int hl = blockIdx.y, hq = h0 + hl, NBm = nb - 1;
  const int wave = threadIdx.x / 64, lane = threadIdx.x % 64;
  const int pos = Bs + blockIdx.x * 4 + wave;  // position in the bucketed order (blocks >= 1 follow block 0)
  if (pos >= N) return;                        // whole waves leave; no workgroup barrier below
  const int n = perm_q[(size_t)hq * N + pos];
  const int b = n / Bs, i = aq[(size_t)hq * N + n];
  const float l = ff_ml[((size_t)hq * N + n) * 2 + 1];
  if (!(l > 0.f)) return;  // wave-uniform: this query has no far field
  const float* qci = qc + ((size_t)hq * Cq + i) * D;
  for (int d = lane; d < D; d += 64) qts[wave][d] = scale * (Elem<T>::ld(Q, ((size_t)hq * N + n) * D + d) - qci[d]);
  wave_lds_fence();
  const float* cm = cbar + (((size_t)hl * NBm + (b - 1)) * Cq + i) * (size_t)D * D;
  for (int a = lane; a < D; a += 64) {
    const float* row = cm + (size_t)a * D;
    float s = 0.f;
#pragma unroll 8
    for (int c = 0; c < D; c += 4) {
      const float4 r4 = *reinterpret_cast<const float4*>(row + c);
      s = fmaf(r4.x, qts[wave][c], s); s = fmaf(r4.y, qts[wave][c + 1], s);
      s = fmaf(r4.z, qts[wave][c + 2], s); s = fmaf(r4.w, qts[wave][c + 3], s);
    }
    ff_acc[((size_t)hq * N + n) * D + a] += l * s;
  }
}

}  // namespace

size_t muse_dipole_fixed_bytes(const MuseDims& d) {
  const size_t NBm = d.nb > 1 ? d.nb - 1 : 1;
  return ff_al((size_t)d.B * d.Hkv * NBm * d.Ck * d.D * d.D * 4);
}
size_t muse_dipole_head_bytes(const MuseDims& d) {
  const size_t NBm = d.nb > 1 ? d.nb - 1 : 1;
  return ff_al(NBm * d.Cq * (size_t)d.D * d.D * 4);
}

template <typename T>
int muse_dipole_covariances(const MuseDims& d, FFWorkspace& w, hipStream_t st) {
  dim3 g(d.Ck, d.B * d.Hkv);
  if (d.D == 64)
    { MuseProf prof_("k_dipole_cov", st); hipLaunchKernelGGL((k_dipole_cov<T, 64>), g, dim3(256), 0, st, (const T*)w.Ks, (const T*)w.Vs, w.off_k, w.dip_cov, d.N, d.nb, d.Ck); }
  else
    { MuseProf prof_("k_dipole_cov", st); hipLaunchKernelGGL((k_dipole_cov<T, 128>), g, dim3(256), 0, st, (const T*)w.Ks, (const T*)w.Vs, w.off_k, w.dip_cov, d.N, d.nb, d.Ck); }
  MUSE_LAUNCH_CHECK();
  return MUSE_OK;
}

template <typename T>
int muse_dipole_apply(const MuseDims& d, const T* Q, const float* qc, const int32_t* aq, FFWorkspace& w, int h0, int hn,
                      hipStream_t st) {
  const int NBm = d.nb - 1, DD = d.D * d.D;
  dim3 gm((DD + 255) / 256, (d.Cq + 15) / 16, hn * NBm);
  { MuseProf prof_("k_dipole_merge", st); hipLaunchKernelGGL(k_dipole_merge, gm, dim3(256), 0, st, w.A_mu, w.dip_cov, w.dip_cbar, h0, NBm, d.Cq, d.Ck, DD, d.Hq, d.Hkv); }
  dim3 ga((d.N - d.Bs + 3) / 4, hn);
  if (d.D == 64)
    { MuseProf prof_("k_dipole_apply", st); hipLaunchKernelGGL((k_dipole_apply<T, 64>), ga, dim3(256), 0, st, Q, qc, w.dip_cbar, w.perm_q, aq, w.ff_acc, w.ff_ml, h0, d.N, d.Bs, d.nb, d.Cq, d.scale); }
  else
    { MuseProf prof_("k_dipole_apply", st); hipLaunchKernelGGL((k_dipole_apply<T, 128>), ga, dim3(256), 0, st, Q, qc, w.dip_cbar, w.perm_q, aq, w.ff_acc, w.ff_ml, h0, d.N, d.Bs, d.nb, d.Cq, d.scale); }
  MUSE_LAUNCH_CHECK();
  return MUSE_OK;
}

template int muse_dipole_covariances<float>(const MuseDims&, FFWorkspace&, hipStream_t);
template int muse_dipole_covariances<bf16_t>(const MuseDims&, FFWorkspace&, hipStream_t);
template int muse_dipole_apply<float>(const MuseDims&, const float*, const float*, const int32_t*, FFWorkspace&, int, int, hipStream_t);
template int muse_dipole_apply<bf16_t>(const MuseDims&, const bf16_t*, const float*, const int32_t*, FFWorkspace&, int, int, hipStream_t);
