// Clustering stage (Sec. 3 "Clustering", App. C): Lloyd K-means per head at a fixed iteration
// count, nearest centroid by ||c||^2 - 2<x,c> (App. C, "Balanced Assignment": the ||x||^2 term
// cancels), and the stable bucketing by (spatial block, cluster) that both the centroid update
// and the attention stages use.
//
//   assign (bf16): the N x C x D similarity is a dense contraction -> MFMA 32x32x16 bf16 with the
//                  argmin kept in the accumulator layout (one query point per lane column).
//   assign (fp32): plain FMA kernel, used for fp32 inputs only.
//   bucket:        one workgroup per (head, spatial block), LDS histograms per wave, ballot-based
//                  stable ranks -> no global atomics, order inside a segment = ascending position.
//   update:        one wave per (head, cluster): fixed-order sum over its segments.
//   streaming pass (App. C "Centroid Computation") and balanced assignment (App. C "Balanced Assignment"):
//                  the paper's own clustering, behind flags; see k_stream_kmeans and k_balance.
#include "common.h"

namespace {

// ------------------------------------------------------------------------------------------
// centroid gather / preparation
// ------------------------------------------------------------------------------------------
template <typename T>
__global__ void k_init_centroids(const T* __restrict__ X, const int32_t* __restrict__ init_idx,
                                 float* __restrict__ cent, int N, int D, int C) {
  int h = blockIdx.y, j = blockIdx.x;
  int row = init_idx[(size_t)h * C + j];
  for (int d = threadIdx.x; d < D; d += blockDim.x)
    cent[((size_t)h * C + j) * D + d] = Elem<T>::ld(X, ((size_t)h * N + row) * D + d);
}

// chat [H,C,D]: centroid in the scoring type; nhc2 [H,C] = -0.5 * ||chat||^2 (fp32 of the rounded values)
template <typename T>
__global__ void k_prep_centroids(const float* __restrict__ cent, T* __restrict__ chat,
                                 float* __restrict__ nhc2, int D, int total) {
  int row = blockIdx.x * (blockDim.x / 64) + threadIdx.x / 64;
  int lane = threadIdx.x % 64;
  if (row >= total) return;
  float s = 0.f;
  for (int d = lane; d < D; d += 64) {
    float c = cent[(size_t)row * D + d];
    Elem<T>::st(chat, (size_t)row * D + d, c);
    float cr = Elem<T>::ld(chat, (size_t)row * D + d);
    s += cr * cr;
  }
  s = wave_sum(s);
  if (lane == 0) nhc2[row] = -0.5f * s;
}

// ------------------------------------------------------------------------------------------
// assignment, fp32 inputs: one thread per point, centroid tiles in LDS
// ------------------------------------------------------------------------------------------
template <int D>
__global__ void __launch_bounds__(256) k_assign_f32(const float* __restrict__ X,
                                                     const float* __restrict__ chat,
                                                     const float* __restrict__ nhc2,
                                                     int32_t* __restrict__ assign, int N, int C) {
  constexpr int CT = 32;
  __shared__ float cs[CT][D + 1];
  __shared__ float c2s[CT];
  int h = blockIdx.y;
  int n = blockIdx.x * 256 + threadIdx.x;
  float x[D];
  if (n < N) {
#pragma unroll
    for (int d = 0; d < D; ++d) x[d] = X[((size_t)h * N + n) * D + d];
  }
  float best = MUSE_NEG_INF;
  int bj = 0;
  for (int j0 = 0; j0 < C; j0 += CT) {
    __syncthreads();
    for (int t = threadIdx.x; t < CT * D; t += 256) {
      int jj = t / D, d = t % D;
      cs[jj][d] = (j0 + jj < C) ? chat[((size_t)h * C + j0 + jj) * D + d] : 0.f;
    }
    if ((int)threadIdx.x < CT) c2s[threadIdx.x] = (j0 + (int)threadIdx.x < C) ? nhc2[(size_t)h * C + j0 + threadIdx.x] : MUSE_NEG_INF;
    __syncthreads();
    if (n < N) {
      for (int jj = 0; jj < CT && j0 + jj < C; ++jj) {
        float acc = c2s[jj];
#pragma unroll
        for (int d = 0; d < D; ++d) acc = fmaf(x[d], cs[jj][d], acc);
        if (acc > best) { best = acc; bj = j0 + jj; }
      }
    }
  }
  if (n < N) assign[(size_t)h * N + n] = bj;
}

// ------------------------------------------------------------------------------------------
// assignment, bf16 inputs: S^T = Chat X^T on MFMA, accumulator preloaded with -||c||^2/2, so the
// nearest centroid is the row-argmax.  Each wave owns PT tiles of 32 points (one point per lane
// column, two lane halves hold different centroid rows).  The four waves of a block share the
// centroids: chunks of CCH rows go through LDS (two buffers, the next chunk's loads are in flight
// while this one is scored), so the inner loop has no global-memory round trip.
// ------------------------------------------------------------------------------------------
template <int D, int PT>
__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(D == 64 ? 2 : 1, 2))) k_assign_bf16(const bf16_t* __restrict__ X,
                                                      const bf16_t* __restrict__ chat,
                                                      const float* __restrict__ nhc2,
                                                      int32_t* __restrict__ assign, int N, int C) {
  constexpr int KS = D / 16, CCH = 8192 / D, CPR = D / 8, NLD = CCH * CPR / 256;
  __shared__ __attribute__((aligned(16))) bf16_t cs[2][CCH][D + 8];
  __shared__ __attribute__((aligned(16))) float c2s[2][CCH];
  const int h = blockIdx.y;
  const int wave = threadIdx.x / 64, lane = threadIdx.x % 64;
  const int col = lane % 32, half = lane / 32;
  const int p0 = (blockIdx.x * 4 + wave) * (32 * PT);
  const bf16_t* Xh = X + (size_t)h * N * D;
  const bf16_t* Ch = chat + (size_t)h * C * D;
  const float* c2h = nhc2 + (size_t)h * C;

  bf16x8_t xb[PT][KS];
#pragma unroll
  for (int t = 0; t < PT; ++t) {
    int n = p0 + 32 * t + col;
    n = n < N ? n : N - 1;
#pragma unroll
    for (int s = 0; s < KS; ++s)
      xb[t][s] = *reinterpret_cast<const bf16x8_t*>(Xh + (size_t)n * D + 16 * s + 8 * half);
  }
  float best[PT][16];
  int btile[PT][16];
#pragma unroll
  for (int t = 0; t < PT; ++t)
#pragma unroll
    for (int e = 0; e < 16; ++e) { best[t][e] = MUSE_NEG_INF; btile[t][e] = 0; }

  uint4 stg[NLD];
  float stg2 = MUSE_NEG_INF;
  auto load_chunk = [&](int c0) {  // this thread's share of rows c0 .. c0+CCH-1 (zero rows / -inf past C)
#pragma unroll
    for (int u = 0; u < NLD; ++u) {
      const int c = threadIdx.x + 256 * u, row = c / CPR, cc = c % CPR;
      stg[u] = c0 + row < C ? *reinterpret_cast<const uint4*>(Ch + (size_t)(c0 + row) * D + cc * 8) : make_uint4(0u, 0u, 0u, 0u);
    }
    if (threadIdx.x < CCH) stg2 = c0 + (int)threadIdx.x < C ? c2h[c0 + threadIdx.x] : MUSE_NEG_INF;
  };
  auto store_chunk = [&](int buf) {
#pragma unroll
    for (int u = 0; u < NLD; ++u) {
      const int c = threadIdx.x + 256 * u, row = c / CPR, cc = c % CPR;
      *reinterpret_cast<uint4*>(&cs[buf][row][cc * 8]) = stg[u];
    }
    if (threadIdx.x < CCH) c2s[buf][threadIdx.x] = stg2;
  };
  const int nch = (C + CCH - 1) / CCH;
  load_chunk(0);
  store_chunk(0);
  __syncthreads();
  for (int ch = 0; ch < nch; ++ch) {
    const int buf = ch & 1;
    if (ch + 1 < nch) load_chunk((ch + 1) * CCH);
#pragma unroll 2
    for (int ct = 0; ct < CCH / 32; ++ct) {
      bf16x8_t ca[KS];
#pragma unroll
      for (int s = 0; s < KS; ++s) ca[s] = *reinterpret_cast<const bf16x8_t*>(&cs[buf][ct * 32 + col][16 * s + 8 * half]);
      f32x16_t init;
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const float4 c4 = *reinterpret_cast<const float4*>(&c2s[buf][ct * 32 + 8 * g + 4 * half]);
        init[4 * g] = c4.x; init[4 * g + 1] = c4.y; init[4 * g + 2] = c4.z; init[4 * g + 3] = c4.w;
      }
      const int gt_ = ch * (CCH / 32) + ct;  // global centroid tile
#pragma unroll
      for (int t = 0; t < PT; ++t) {
        f32x16_t acc = init;
#pragma unroll
        for (int s = 0; s < KS; ++s) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ca[s], xb[t][s], acc, 0, 0, 0);
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          bool gt = acc[e] > best[t][e];
          best[t][e] = gt ? acc[e] : best[t][e];
          btile[t][e] = gt ? gt_ : btile[t][e];
        }
      }
    }
    if (ch + 1 < nch) store_chunk(buf ^ 1);
    __syncthreads();
  }
#pragma unroll
  for (int t = 0; t < PT; ++t) {
    float bv = MUSE_NEG_INF;
    int bj = 0x7fffffff;
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      int j = btile[t][e] * 32 + 8 * (e / 4) + 4 * half + (e % 4);
      bool take = best[t][e] > bv || (best[t][e] == bv && j < bj);
      bv = take ? best[t][e] : bv;
      bj = take ? j : bj;
    }
    float ov = __shfl_xor(bv, 32, 64);
    int oj = __shfl_xor(bj, 32, 64);
    if (ov > bv || (ov == bv && oj < bj)) { bv = ov; bj = oj; }
    int n = p0 + 32 * t + col;
    if (half == 0 && n < N) assign[(size_t)h * N + n] = bj;
  }
}

// ------------------------------------------------------------------------------------------
// The same assignment with ALL centroids of the head resident in LDS (C (D + 8) 2 + 4 C bytes <= 160 KB: every
// shape but the largest C x D).  One workgroup of 8 waves per CU fills the LDS once and then walks batches of
// 512 points (64 per wave), the rows of the next batch in flight while this one is scored: no chunk pipeline, no
// barrier after the fill, and the fill is paid once per eight or so batches.  (D = 128: 32 points per wave.)
// Running argmax in the accumulator layout, one (value, run) pair per accumulator element.  Inside a run of 16
// centroid tiles the tile number rides in the low four mantissa bits of the score (15 - tile % 16, so the earlier
// tile wins among scores equal above those bits): one v_and_or and half a v_max3 per score instead of a compare
// and two selects.  The four bits cost a relative 2^-19 of a score, below the margin at which an assignment is
// defined.  At the end of a run the packed maximum is folded into (gbest, grun) with compare and selects.
// ------------------------------------------------------------------------------------------
constexpr float kPadScore = -3.0e38f;  // score of the padding rows past C: finite, so that tagging its low bits keeps it a number
constexpr int kResWaves = 8;
template <int D>
__global__ void __launch_bounds__(64 * kResWaves) __attribute__((amdgpu_waves_per_eu(2, 2))) k_assign_res(
    const bf16_t* __restrict__ X, const bf16_t* __restrict__ chat, const float* __restrict__ nhc2,
    int32_t* __restrict__ assign, int N, int C, int Cpad) {
  constexpr int KS = D / 16, CPR = D / 8, PT = D == 64 ? 2 : 1, LDW = D + 8;
  extern __shared__ __attribute__((aligned(16))) unsigned char res_lds[];
  bf16_t* cs = reinterpret_cast<bf16_t*>(res_lds);                          // [Cpad][D + 8]
  float* c2s = reinterpret_cast<float*>(res_lds + (size_t)Cpad * LDW * 2);  // [Cpad]
  const int h = blockIdx.y;
  const int wave = threadIdx.x / 64, lane = threadIdx.x % 64, col = lane % 32, half = lane / 32;
  const bf16_t* Xh = X + (size_t)h * N * D;
  const bf16_t* Ch = chat + (size_t)h * C * D;
  for (int idx = threadIdx.x; idx < Cpad * CPR; idx += 64 * kResWaves) {
    const int row = idx / CPR, cc = idx % CPR;
    *reinterpret_cast<uint4*>(&cs[(size_t)row * LDW + cc * 8]) =
        row < C ? *reinterpret_cast<const uint4*>(Ch + (size_t)row * D + cc * 8) : make_uint4(0u, 0u, 0u, 0u);
  }
  for (int row = threadIdx.x; row < Cpad; row += 64 * kResWaves) c2s[row] = row < C ? nhc2[(size_t)h * C + row] : kPadScore;
  __syncthreads();

  constexpr int BP = kResWaves * 32 * PT;  // points per batch
  const int nbatch = (N + BP - 1) / BP;
  auto load_x = [&](bf16x8_t (&xb)[PT][KS], int batch) {
#pragma unroll
    for (int t = 0; t < PT; ++t) {
      int n = batch * BP + (wave * PT + t) * 32 + col;
      n = n < N ? n : N - 1;
#pragma unroll
      for (int s = 0; s < KS; ++s) xb[t][s] = *reinterpret_cast<const bf16x8_t*>(Xh + (size_t)n * D + 16 * s + 8 * half);
    }
  };
  auto tag = [](float v, uint32_t code) { return __uint_as_float((__float_as_uint(v) & 0xfffffff0u) | code); };
  bf16x8_t xn[PT][KS];
  if ((int)blockIdx.x < nbatch) load_x(xn, blockIdx.x);
  for (int batch = blockIdx.x; batch < nbatch; batch += gridDim.x) {
    bf16x8_t xb[PT][KS];
#pragma unroll
    for (int t = 0; t < PT; ++t)
#pragma unroll
      for (int s = 0; s < KS; ++s) xb[t][s] = xn[t][s];
    if (batch + (int)gridDim.x < nbatch) load_x(xn, batch + gridDim.x);
    float sbest[PT][16], gbest[PT][16];
    int grun[PT][16];
#pragma unroll
    for (int t = 0; t < PT; ++t)
#pragma unroll
      for (int e = 0; e < 16; ++e) { sbest[t][e] = MUSE_NEG_INF; gbest[t][e] = MUSE_NEG_INF; grun[t][e] = 0; }
    const int ntile = Cpad / 32;  // even
    for (int ct = 0; ct < ntile; ct += 2) {
      bf16x8_t ca[2][KS];
#pragma unroll
      for (int z = 0; z < 2; ++z)
#pragma unroll
        for (int s = 0; s < KS; ++s)
          ca[z][s] = *reinterpret_cast<const bf16x8_t*>(&cs[(size_t)((ct + z) * 32 + col) * LDW + 16 * s + 8 * half]);
      auto init = [&](int z) {  // -||c||^2 / 2 of the tile's rows: read again for every point tile (registers are scarcer than LDS reads)
        f32x16_t v;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const float4 c4 = *reinterpret_cast<const float4*>(&c2s[(ct + z) * 32 + 8 * g + 4 * half]);
          v[4 * g] = c4.x; v[4 * g + 1] = c4.y; v[4 * g + 2] = c4.z; v[4 * g + 3] = c4.w;
        }
        return v;
      };
      uint32_t code0 = 15u - (uint32_t)(ct & 15), code1 = code0 - 1u;
      // opaque to the optimiser, which otherwise rewrites "| code" as per-element additions of its terms
      asm volatile("" : "+s"(code0), "+s"(code1));
#pragma unroll
      for (int t = 0; t < PT; ++t) {
        asm volatile("" ::: "memory");  // keeps the two point tiles' reads of the bias rows apart
        f32x16_t a0 = init(0), a1 = init(1);
#pragma unroll
        for (int s = 0; s < KS; ++s) {
          a0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ca[0][s], xb[t][s], a0, 0, 0, 0);
          a1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ca[1][s], xb[t][s], a1, 0, 0, 0);
        }
#pragma unroll
        for (int e = 0; e < 16; ++e) sbest[t][e] = fmaxf(fmaxf(sbest[t][e], tag(a0[e], code0)), tag(a1[e], code1));
      }
      if ((ct & 15) == 14 || ct + 2 >= ntile) {  // a run of 16 tiles, or the last one, is complete
        const int run = ct >> 4;
#pragma unroll
        for (int t = 0; t < PT; ++t)
#pragma unroll
          for (int e = 0; e < 16; ++e) {
            const bool gt = sbest[t][e] > gbest[t][e];
            gbest[t][e] = gt ? sbest[t][e] : gbest[t][e];
            grun[t][e] = gt ? run : grun[t][e];
            sbest[t][e] = MUSE_NEG_INF;
          }
      }
    }
#pragma unroll
    for (int t = 0; t < PT; ++t) {
      float bv = MUSE_NEG_INF;
      int bj = 0x7fffffff;
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int tile = grun[t][e] * 16 + 15 - (int)(__float_as_uint(gbest[t][e]) & 15u);
        const int j = tile * 32 + 8 * (e / 4) + 4 * half + (e % 4);
        const bool take = gbest[t][e] > bv || (gbest[t][e] == bv && j < bj);
        bv = take ? gbest[t][e] : bv;
        bj = take ? j : bj;
      }
      const float ov = __shfl_xor(bv, 32, 64);
      const int oj = __shfl_xor(bj, 32, 64);
      if (ov > bv || (ov == bv && oj < bj)) { bv = ov; bj = oj; }
      const int n = batch * BP + (wave * PT + t) * 32 + col;
      if (half == 0 && n < N) assign[(size_t)h * N + n] = bj;
    }
  }
}

// ------------------------------------------------------------------------------------------
// stable bucketing by (block, cluster): grid (nb, heads), 1024 threads = 16 waves
// ------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(1024) k_bucket(const int32_t* __restrict__ assign,
                                                  int32_t* __restrict__ perm,
                                                  int32_t* __restrict__ off, int N, int Bs, int C) {
  extern __shared__ uint32_t smem[];
  uint32_t* hist = smem;               // [16][C]
  uint32_t* tot = smem + 16 * C;       // [C]
  __shared__ uint32_t wsum[16];
  const int b = blockIdx.x, h = blockIdx.y, nb = gridDim.x;
  const int wave = threadIdx.x / 64, lane = threadIdx.x % 64;
  const int32_t* a = assign + (size_t)h * N + (size_t)b * Bs;
  const int sub = (Bs + 15) / 16;
  const int lo = wave * sub, hi = min(lo + sub, Bs);

  for (int t = threadIdx.x; t < 17 * C; t += 1024) smem[t] = 0;
  __syncthreads();
  // entries outside [0, C) are the caller's error; clamped here so that they cannot index outside the histograms
  for (int i = lo + lane; i < hi; i += 64) atomicAdd(&hist[wave * C + min(max(a[i], 0), C - 1)], 1u);
  __syncthreads();
  // per cluster: exclusive prefix over the waves, total per cluster
  for (int c = threadIdx.x; c < C; c += 1024) {
    uint32_t run = 0;
    for (int w = 0; w < 16; ++w) {
      uint32_t v = hist[w * C + c];
      hist[w * C + c] = run;
      run += v;
    }
    tot[c] = run;
  }
  __syncthreads();
  // exclusive scan of tot over clusters; every thread owns a contiguous run of clusters
  const int per = (C + 1023) / 1024;
  uint32_t mine = 0;
  for (int u = 0; u < per; ++u) {
    int c = threadIdx.x * per + u;
    if (c < C) mine += tot[c];
  }
  uint32_t incl = mine;
  for (int o = 1; o < 64; o <<= 1) {
    uint32_t v = __shfl_up(incl, o, 64);
    if (lane >= o) incl += v;
  }
  if (lane == 63) wsum[wave] = incl;
  __syncthreads();
  uint32_t base = 0;
  for (int w = 0; w < wave; ++w) base += wsum[w];
  uint32_t run = base + incl - mine;
  for (int u = 0; u < per; ++u) {
    int c = threadIdx.x * per + u;
    if (c < C) {
      uint32_t v = tot[c];
      tot[c] = run;
      off[(size_t)h * ((size_t)nb * C + 1) + (size_t)b * C + c] = b * Bs + (int)run;
      run += v;
    }
  }
  if (b == nb - 1 && threadIdx.x == 0) off[(size_t)h * ((size_t)nb * C + 1) + (size_t)nb * C] = N;
  __syncthreads();
  // placement: each wave walks its sub-chunk in order; equal keys inside a group of 64 are ranked
  // by lane with ballots over the key bits
  for (int i0 = lo; i0 < hi; i0 += 64) {
    int i = i0 + lane;
    bool act = i < hi;
    int key = act ? min(max(a[i], 0), C - 1) : 0;
    unsigned long long m = __ballot(act);
#pragma unroll
    for (int bit = 0; bit < 12; ++bit) {
      unsigned long long bb = __ballot((key >> bit) & 1);
      m &= ((key >> bit) & 1) ? bb : ~bb;
    }
    unsigned long long below = m & ((1ull << lane) - 1ull);
    int rank = __popcll(below), cnt = __popcll(m);
    if (act) {
      uint32_t start = hist[wave * C + key];
      perm[(size_t)h * N + (size_t)b * Bs + tot[key] + start + rank] = b * Bs + i;
      if (rank == cnt - 1) hist[wave * C + key] = start + cnt;
    }
  }
}

// ------------------------------------------------------------------------------------------
// centroid update: one wave per (head, cluster); RL lanes cover one row with 16-byte loads, the
// 64/RL row slots run over the members in order, slots are combined in a fixed tree.
// ------------------------------------------------------------------------------------------
template <typename T>
__global__ void __launch_bounds__(256) k_update(const T* __restrict__ X, const int32_t* __restrict__ perm,
                                                 const int32_t* __restrict__ off, float* __restrict__ cent,
                                                 int N, int D, int C, int nb, int total) {
  constexpr int EPL = 16 / Elem<T>::kBytes;  // elements per lane
  int wid = blockIdx.x * 4 + threadIdx.x / 64;
  if (wid >= total) return;
  const int lane = threadIdx.x % 64;
  const int h = wid / C, j = wid % C;
  const int RL = D / EPL, slots = 64 / RL;
  const int slot = lane / RL, chunk = lane % RL;
  const T* Xh = X + (size_t)h * N * D;
  const int32_t* ph = perm + (size_t)h * N;
  const int32_t* oh = off + (size_t)h * ((size_t)nb * C + 1);
  float acc[EPL];
#pragma unroll
  for (int e = 0; e < EPL; ++e) acc[e] = 0.f;
  // a row slot takes every slots-th spatial block and walks its members MPI at a time; the positions of the
  // next MPI are requested together with the rows of these (one round trip per MPI members)
  constexpr int MPI = 16;
  int count = 0;
  for (int b = slot; b < nb; b += slots) {
    const int lo = oh[b * C + j], hi = oh[b * C + j + 1];
    count += hi - lo;
    if (lo >= hi) continue;
    int rown[MPI];
#pragma unroll
    for (int u = 0; u < MPI; ++u) rown[u] = ph[lo + u < hi ? lo + u : hi - 1];
    for (int p = lo; p < hi; p += MPI) {
      int row[MPI];
#pragma unroll
      for (int u = 0; u < MPI; ++u) {
        row[u] = rown[u];
        rown[u] = ph[p + MPI + u < hi ? p + MPI + u : hi - 1];
      }
      if constexpr (EPL == 8) {
        uint4 v[MPI];
#pragma unroll
        for (int u = 0; u < MPI; ++u) v[u] = *reinterpret_cast<const uint4*>(Xh + (size_t)row[u] * D + chunk * 8);
#pragma unroll
        for (int u = 0; u < MPI; ++u) {
          if (p + u >= hi) continue;
          const uint32_t w[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            acc[2 * e] += __uint_as_float(w[e] << 16);
            acc[2 * e + 1] += __uint_as_float(w[e] & 0xffff0000u);
          }
        }
      } else {
        float4 v[MPI];
#pragma unroll
        for (int u = 0; u < MPI; ++u) v[u] = *reinterpret_cast<const float4*>(Xh + (size_t)row[u] * D + chunk * 4);
#pragma unroll
        for (int u = 0; u < MPI; ++u) {
          if (p + u >= hi) continue;
          acc[0] += v[u].x; acc[1] += v[u].y; acc[2] += v[u].z; acc[3] += v[u].w;
        }
      }
    }
  }
  for (int o = RL; o < 64; o <<= 1) count += __shfl_xor(count, o, 64);
  for (int o = RL; o < 64; o <<= 1)
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[e] += __shfl_xor(acc[e], o, 64);
  if (slot == 0 && count > 0) {
    float inv = (float)count;
#pragma unroll
    for (int e = 0; e < EPL; ++e) cent[((size_t)h * C + j) * D + chunk * EPL + e] = acc[e] / inv;
  }
}

// ------------------------------------------------------------------------------------------
// Streaming centroid pass (App. C "Centroid Computation", step 2): one pass over the rows of a head in
// sequence order, minibatches of 64.  Every row of a minibatch is assigned to its nearest centroid as the
// centroids stand when the minibatch starts; then, row by row, the total and the count of the row's centroid
// decay and absorb it: t <- beta t + x, c <- beta c + 1 (beta = 0.9), centroid = t / c.
//
// The pass is sequential over the N / 64 minibatches, so one workgroup (8 waves, two per SIMD) owns a head from
// start to end; a minibatch is a chain of dependent steps, and what counts is their latency, not throughput.
// Rows and centroids enter the similarity as binary16 (App. C: the clustering runs in float16) on MFMA 32x32x16
// f16 with fp32 accumulation that starts at -||c^||^2 / 2: centroid tiles are the A operand, the 64 rows of the
// minibatch the B operand (LDS), each wave takes every eighth tile of 32 centroids and keeps a running argmax
// (value, tile, accumulator element) per lane.  The state t, c stays fp32 (one fma per update, one division per
// centroid); only the centroids that a minibatch touches are rewritten: centroid j belongs to wave j % 8, which
// finds the distinct ones among its rows by ballots, requests all their totals before it uses any, and reduces
// their norms with DPP row sums.  While C D is small the whole state sits in LDS (no global round trip inside
// the pass); otherwise it sits in the workspace, L2-resident, and is re-read through the CU's L1 after the
// workgroup barrier that ends a minibatch.
// ------------------------------------------------------------------------------------------
typedef __attribute__((ext_vector_type(8))) _Float16 kf16x8_t;

constexpr int kStreamMB = 64;
constexpr int kStreamNW = 8;  // waves of the workgroup that owns a head (two per SIMD)
constexpr float kStreamBeta = 0.9f;
// operands of TB tiles of 32 centroids: this lane's row of each tile (its half of every 16 dims) and the
// -||c^||^2 / 2 of the 16 centroids whose scores land in this lane
template <int D, int TB_>
struct CentBatch {
  static constexpr int TB = TB_;
  kf16x8_t ca[TB][D / 16];
  f32x16_t nv[TB];
};

// TBN: tiles per batch (two batches are live: registers).  LS: the whole state (totals, counts, binary16
// centroids, their norms) lives in dynamic LDS instead of the L2-resident workspace arrays: no global round
// trips inside the pass; possible while C D is small enough (the host decides).
template <typename T, int D, int TBN, bool LS>
__global__ void __launch_bounds__(64 * kStreamNW) __attribute__((amdgpu_waves_per_eu(kStreamNW / 4, kStreamNW / 4)))
k_stream_kmeans(const T* __restrict__ X, const int32_t* __restrict__ init_idx, float* __restrict__ cent,
                float* __restrict__ tst, float* __restrict__ cst, _Float16* __restrict__ chat,
                float* __restrict__ nhc2, int32_t* __restrict__ trace, float* __restrict__ counts_out, int N, int C) {
  // cst and nhc2 are [heads][CS], CS = C rounded up to a whole tile of 32 (16-byte reads of a tile's 32 values)
  constexpr int KS = D / 16, DL = D / 64;         // k-steps of the similarity; dims per lane in the update
  constexpr int NW = kStreamNW, NT = 64 * NW;
  constexpr int CPR = D / 8, NCH = 64 * CPR / NT;  // 16-byte (bf16) / 32-byte (fp32) chunks of a minibatch per thread
  __shared__ __attribute__((aligned(16))) _Float16 xs[kStreamMB][D + 8];
  __shared__ float bval[kStreamNW][kStreamMB];
  __shared__ int bidx[kStreamNW][kStreamMB];
  const int h = blockIdx.x;
  const int tid = threadIdx.x, lane = tid % 64, col = lane % 32, half = lane / 32;
  const int wave = __builtin_amdgcn_readfirstlane(tid / 64);  // in a scalar register: loops and branches on it are uniform
  const T* Xh = X + (size_t)h * N * D;
  const int CS = (C + 31) / 32 * 32;
  extern __shared__ __attribute__((aligned(16))) unsigned char stream_lds[];
  constexpr int HS = LS ? D + 8 : D;  // row stride of the binary16 centroids (padded in LDS: conflict-free 16-byte reads)
  float* th = LS ? reinterpret_cast<float*>(stream_lds) : tst + (size_t)h * C * D;
  _Float16* hh = LS ? reinterpret_cast<_Float16*>(stream_lds + (size_t)C * D * 4) : chat + (size_t)h * C * D;
  float* ch_ = LS ? reinterpret_cast<float*>(stream_lds + (size_t)C * D * 4 + (size_t)C * HS * 2) : cst + (size_t)h * CS;
  float* nh = LS ? ch_ + CS : nhc2 + (size_t)h * CS;
  float* ce = cent + (size_t)h * C * D;

  // ---- initial state: t = the initial centroid (as binary16 values), c = 1 ----
  for (int j = wave; j < C; j += NW) {
    float s = 0.f;
#pragma unroll
    for (int x = 0; x < DL; ++x) {
      const int d = lane + 64 * x;
      float v = init_idx ? Elem<T>::ld(Xh, (size_t)init_idx[(size_t)h * C + j] * D + d) : ce[(size_t)j * D + d];
      const _Float16 vh = (_Float16)v;
      if (init_idx) v = (float)vh;
      th[(size_t)j * D + d] = v;
      hh[(size_t)j * HS + d] = vh;
      s += (float)vh * (float)vh;
    }
    s = wave_sum(s);
    if (lane == 0) {
      ch_[j] = 1.f;
      nh[j] = -0.5f * s;
    }
  }
  // the last tile's entries past C: never the nearest (their rows repeat the centroid C - 1)
  for (int j = C + tid; j < CS; j += NT) nh[j] = MUSE_NEG_INF;

  // raw rows of a minibatch, this thread's chunks (row = c % 64, 8 dims from 8 (c / 64)); rows past N repeat N - 1
  auto row_ptr = [&](int v0, int it) {
    const int c = tid + NT * it;
    int gr = v0 + c % 64;
    gr = gr < N ? gr : N - 1;
    return Xh + (size_t)gr * D + (c / 64) * 8;
  };
  uint4 ra[NCH], rb[sizeof(T) == 4 ? NCH : 1];
#pragma unroll
  for (int it = 0; it < NCH; ++it) {
    ra[it] = *reinterpret_cast<const uint4*>(row_ptr(0, it));
    if constexpr (sizeof(T) == 4) rb[it] = *reinterpret_cast<const uint4*>(row_ptr(0, it) + 4);
  }
  const int ntile = (C + 31) / 32;
  const int nmb = (N + kStreamMB - 1) / kStreamMB;
  for (int mbi = 0; mbi < nmb; ++mbi) {
    const int v0 = mbi * kStreamMB;
    __syncthreads();  // state of the previous minibatch is written; xs is free
    // ---- the minibatch as binary16 in LDS ----
#pragma unroll
    for (int it = 0; it < NCH; ++it) {
      const int c = tid + NT * it, row = c % 64, cc = c / 64;
      kf16x8_t o;
      if constexpr (sizeof(T) == 2) {
        const uint32_t w[4] = {ra[it].x, ra[it].y, ra[it].z, ra[it].w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          o[2 * e] = (_Float16)__uint_as_float(w[e] << 16);
          o[2 * e + 1] = (_Float16)__uint_as_float(w[e] & 0xffff0000u);
        }
      } else {
        const uint32_t w[8] = {ra[it].x, ra[it].y, ra[it].z, ra[it].w, rb[it].x, rb[it].y, rb[it].z, rb[it].w};
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] = (_Float16)__uint_as_float(w[e]);
      }
      *reinterpret_cast<kf16x8_t*>(&xs[row][cc * 8]) = o;
    }
    __syncthreads();
    // next minibatch's rows: independent of the state, in flight during this one
    {
      const int vn = mbi + 1 < nmb ? v0 + kStreamMB : v0;
#pragma unroll
      for (int it = 0; it < NCH; ++it) {
        ra[it] = *reinterpret_cast<const uint4*>(row_ptr(vn, it));
        if constexpr (sizeof(T) == 4) rb[it] = *reinterpret_cast<const uint4*>(row_ptr(vn, it) + 4);
      }
    }
    // ---- similarity x^ . c^ - ||c^||^2 / 2 against every centroid, running argmax per lane ----
    kf16x8_t xb[2][KS];
#pragma unroll
    for (int hf = 0; hf < 2; ++hf)
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) xb[hf][ks] = *reinterpret_cast<const kf16x8_t*>(&xs[32 * hf + col][16 * ks + 8 * half]);
    // running argmax per lane and half-minibatch: value, tile and the accumulator element (row of the tile)
    float best[2] = {MUSE_NEG_INF, MUSE_NEG_INF};
    int bt[2] = {0x3fffff, 0x3fffff}, be[2] = {0, 0};
    // this wave's tiles jt = wave + NW k in batches of TB: the operands of a whole batch are requested before the
    // first is used, and the next batch is in flight while this one is scored (loads are unconditional: tiles
    // past the end re-read the last one and are skipped when scoring)
    auto load_cb = [&](CentBatch<D, TBN>& cb, int k0) {
#pragma unroll
      for (int tb = 0; tb < CentBatch<D, TBN>::TB; ++tb) {
        int jt = wave + NW * (k0 + tb);
        jt = jt < ntile ? jt : ntile - 1;
        const int j0 = jt * 32;
        const int jr = j0 + col < C ? j0 + col : C - 1;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
          cb.ca[tb][ks] = *reinterpret_cast<const kf16x8_t*>(hh + (size_t)jr * HS + 16 * ks + 8 * half);
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const float4 n4 = *reinterpret_cast<const float4*>(nh + j0 + 8 * g + 4 * half);
          cb.nv[tb][4 * g] = n4.x; cb.nv[tb][4 * g + 1] = n4.y; cb.nv[tb][4 * g + 2] = n4.z; cb.nv[tb][4 * g + 3] = n4.w;
        }
      }
    };
    // Tiles past the end were loaded as copies of the last tile: scoring a tile twice changes nothing (only a
    // strictly larger score replaces the best), so a batch is scored without branches and its independent
    // MFMA chains (TB tiles x 2 halves) can be interleaved with the comparisons.
    auto score_cb = [&](const CentBatch<D, TBN>& cb, int k0) {
      constexpr int TB = CentBatch<D, TBN>::TB;
      f32x16_t acc[TB][2];
#pragma unroll
      for (int tb = 0; tb < TB; ++tb)
#pragma unroll
        for (int hf = 0; hf < 2; ++hf)  // the accumulator starts at -||c^||^2 / 2 of its row's centroid
          acc[tb][hf] = __builtin_amdgcn_mfma_f32_32x32x16_f16(cb.ca[tb][0], xb[hf][0], cb.nv[tb], 0, 0, 0);
#pragma unroll
      for (int ks = 1; ks < KS; ++ks)
#pragma unroll
        for (int tb = 0; tb < TB; ++tb)
#pragma unroll
          for (int hf = 0; hf < 2; ++hf)
            acc[tb][hf] = __builtin_amdgcn_mfma_f32_32x32x16_f16(cb.ca[tb][ks], xb[hf][ks], acc[tb][hf], 0, 0, 0);
#pragma unroll
      for (int tb = 0; tb < TB; ++tb) {
        int jt = wave + NW * (k0 + tb);
        jt = jt < ntile ? jt : ntile - 1;
#pragma unroll
        for (int hf = 0; hf < 2; ++hf) {
          const float before = best[hf];
#pragma unroll
          for (int e = 0; e < 16; ++e) {  // rows in increasing centroid order: the first of equal scores stays
            const bool up = acc[tb][hf][e] > best[hf];
            be[hf] = up ? e : be[hf];
            best[hf] = up ? acc[tb][hf][e] : best[hf];
          }
          bt[hf] = best[hf] > before ? jt : bt[hf];
        }
      }
    };
    {
      const int nk = (ntile - wave + NW - 1) / NW;  // tiles of this wave
      constexpr int TB = CentBatch<D, TBN>::TB;
      CentBatch<D, TBN> ba, bb;
      load_cb(ba, 0);
      for (int k0 = 0; k0 < nk; k0 += 2 * TB) {
        load_cb(bb, k0 + TB);
        score_cb(ba, k0);
        load_cb(ba, k0 + 2 * TB);
        if (k0 + TB < nk) score_cb(bb, k0 + TB);
      }
    }
    int bj[2];
#pragma unroll
    for (int hf = 0; hf < 2; ++hf) bj[hf] = 32 * bt[hf] + 8 * (be[hf] / 4) + 4 * half + (be[hf] % 4);
    // the two halves of a row's centroids, then the four waves; ties go to the lowest index
#pragma unroll
    for (int hf = 0; hf < 2; ++hf) {
      const float ov = __shfl_xor(best[hf], 32, 64);
      const int oj = __shfl_xor(bj[hf], 32, 64);
      if (ov > best[hf] || (ov == best[hf] && oj < bj[hf])) {
        best[hf] = ov;
        bj[hf] = oj;
      }
    }
    if (half == 0) {
      bval[wave][col] = best[0]; bidx[wave][col] = bj[0];
      bval[wave][32 + col] = best[1]; bidx[wave][32 + col] = bj[1];
    }
    __syncthreads();
    // every wave derives the assignment of all 64 rows (lane = row of the minibatch)
    int a;
    {
      float bv = bval[0][lane];
      a = bidx[0][lane];
#pragma unroll
      for (int w = 1; w < NW; ++w) {
        const float ov = bval[w][lane];
        const int oj = bidx[w][lane];
        if (ov > bv || (ov == bv && oj < a)) {
          bv = ov;
          a = oj;
        }
      }
    }
    const bool live = v0 + lane < N;
    if (wave == 0 && live && trace) trace[(size_t)h * N + v0 + lane] = a;
    if (!live) a = -1 - lane;  // a class of its own that nobody updates
    // ---- updates.  A centroid j belongs to wave j % NW; the wave walks the distinct centroids among its rows
    //      (first row of each, then a ballot for the rows that share it) in rounds of up to MAXL: all loads of
    //      a round are issued before any is used, and the reductions of a round run in lockstep.  A lane owns
    //      the dims lane + 64 x. ----
    constexpr int MAXL = 8;
    unsigned long long rem = __ballot(live && (a & (NW - 1)) == wave);  // wave-uniform
    while (rem) {
      int lj[MAXL];
      unsigned long long lm[MAXL];
      float tv[MAXL][DL], cv[MAXL], x0[MAXL][DL];
      int nl = 0;
#pragma unroll
      for (int q = 0; q < MAXL; ++q) {
        if (rem) {
          const int u = __ffsll((long long)rem) - 1;
          const int j = __builtin_amdgcn_readlane(a, u);
          const unsigned long long m = __ballot(a == j);
          lj[q] = j;
          lm[q] = m & (m - 1);  // rows after the first
#pragma unroll
          for (int x = 0; x < DL; ++x) {
            tv[q][x] = th[(size_t)j * D + lane + 64 * x];
            x0[q][x] = (float)xs[u][lane + 64 * x];
          }
          cv[q] = ch_[j];
          nl = q + 1;
          rem &= ~m;
        }
      }
      float sq[MAXL];
#pragma unroll
      for (int q = 0; q < MAXL; ++q) {
        sq[q] = 0.f;
        if (q < nl) {
          const int j = lj[q];
          unsigned long long m = lm[q];
          float c = fmaf(kStreamBeta, cv[q], 1.f);
          float t[DL];
#pragma unroll
          for (int x = 0; x < DL; ++x) t[x] = fmaf(kStreamBeta, tv[q][x], x0[q][x]);
          while (m) {  // further rows of the class, in order
            const int u = __ffsll((long long)m) - 1;
            m &= m - 1;
#pragma unroll
            for (int x = 0; x < DL; ++x) t[x] = fmaf(kStreamBeta, t[x], (float)xs[u][lane + 64 * x]);
            c = fmaf(kStreamBeta, c, 1.f);
          }
          cv[q] = c;
#pragma unroll
          for (int x = 0; x < DL; ++x) {
            th[(size_t)j * D + lane + 64 * x] = t[x];
            const _Float16 vh = (_Float16)(t[x] / c);
            hh[(size_t)j * HS + lane + 64 * x] = vh;
            sq[q] += (float)vh * (float)vh;
          }
        }
      }
      // ||c^||^2 of the round's centroids: sums inside the rows of 16 lanes by DPP, then the four rows
#pragma unroll
      for (int q = 0; q < MAXL; ++q) sq[q] = wave_sum_dpp(sq[q]);
      {  // lane q writes the scalars of the round's q-th centroid
        int jq = 0;
        float cq = 0.f, sv = 0.f;
#pragma unroll
        for (int q = 0; q < MAXL; ++q)
          if (q < nl && lane == q) {
            jq = lj[q];
            cq = cv[q];
            sv = sq[q];
          }
        if (lane < nl) {
          ch_[jq] = cq;
          nh[jq] = -0.5f * sv;
        }
      }
    }
  }
  __syncthreads();
  // ---- centroids of the raw rows: t / c ----
  for (int j = wave; j < C; j += NW) {
    const float c = ch_[j];
#pragma unroll
    for (int x = 0; x < DL; ++x) ce[(size_t)j * D + lane + 64 * x] = th[(size_t)j * D + lane + 64 * x] / c;
    if (lane == 0 && counts_out) counts_out[(size_t)h * C + j] = c;
  }
}

// ------------------------------------------------------------------------------------------
// Balanced assignment (App. C "Balanced Assignment"): inside a spatial block a cluster holds at most `cap` rows.
// Phase A is the nearest-centroid assignment already in `assign`, bucketed by (block, cluster) in position
// order: the first cap rows of a segment keep their cluster.  Phase B, here: the other rows of the block, one
// after the other in position order, go to the nearest centroid that still has room (same score as the
// assignment kernels: x . c^ - ||c^||^2 / 2 on the scoring-type centroids, fp32 sums, lowest index on ties).
// One workgroup per (head, block); phase B is sequential by definition, a thread owns the centroids
// tid + 256 k and the row being placed is staged in LDS one row ahead.
// ------------------------------------------------------------------------------------------
template <typename T, int D>
__global__ void __launch_bounds__(256) k_balance(const T* __restrict__ X, const T* __restrict__ chat,
                                                 const float* __restrict__ nhc2, const int32_t* __restrict__ perm,
                                                 const int32_t* __restrict__ off, int32_t* __restrict__ assign,
                                                 int N, int Bs, int C, int cap) {
  extern __shared__ int bal_lds[];
  int* count = bal_lds;                                        // [C] rows held per cluster
  unsigned* bits = reinterpret_cast<unsigned*>(count + C);     // [Bs / 32 (+1)] displaced rows of the block
  unsigned short* evl = reinterpret_cast<unsigned short*>(bits + (Bs + 31) / 32);  // [Bs] the same, in order
  __shared__ float xs[2][D];
  __shared__ float rv[4];
  __shared__ int rj[4];
  __shared__ int wsum[4];
  const int b = blockIdx.x, h = blockIdx.y, nbk = N / Bs;
  const int tid = threadIdx.x, lane = tid % 64, wave = tid / 64;
  const int32_t* oh = off + (size_t)h * ((size_t)nbk * C + 1) + (size_t)b * C;
  const int32_t* ph = perm + (size_t)h * N;
  int32_t* ah = assign + (size_t)h * N;
  const T* Xh = X + (size_t)h * N * D;
  const int nw = (Bs + 31) / 32;
  for (int j = tid; j < C; j += 256) count[j] = min(oh[j + 1] - oh[j], cap);
  for (int w = tid; w < nw; w += 256) bits[w] = 0u;
  __syncthreads();
  // rank of a row inside its segment = its index in the bucketed order minus the segment's start
  for (int t = tid; t < Bs; t += 256) {
    const int idx = b * Bs + t;
    const int row = ph[idx];
    const int j = ah[row];
    if (idx - oh[j] >= cap) atomicOr(&bits[(row - b * Bs) >> 5], 1u << ((row - b * Bs) & 31));
  }
  __syncthreads();
  // the displaced rows in position order
  int nev = 0;
  for (int w0 = 0; w0 < nw; w0 += 256) {
    const int w = w0 + tid;
    const unsigned word = w < nw ? bits[w] : 0u;
    const int c = __popc(word);
    int incl = c;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const int v = __shfl_up(incl, o, 64);
      if (lane >= o) incl += v;
    }
    if (lane == 63) wsum[wave] = incl;
    __syncthreads();
    int base = nev;
    for (int q = 0; q < wave; ++q) base += wsum[q];
    const int total = wsum[0] + wsum[1] + wsum[2] + wsum[3];
    int pos = base + incl - c;
    unsigned rest = word;
    while (rest) {
      evl[pos++] = (unsigned short)(32 * w + __ffs(rest) - 1);
      rest &= rest - 1;
    }
    nev += total;
    __syncthreads();
  }
  if (nev == 0) return;
  if (tid < D) xs[0][tid] = Elem<T>::ld(Xh, (size_t)(b * Bs + evl[0]) * D + tid);
  __syncthreads();
  const T* ch = chat + (size_t)h * C * D;
  const float* nh = nhc2 + (size_t)h * C;
  for (int i = 0; i < nev; ++i) {
    const int row = b * Bs + evl[i];
    float xn = 0.f;  // next row, requested before this one is scored
    if (tid < D && i + 1 < nev) xn = Elem<T>::ld(Xh, (size_t)(b * Bs + evl[i + 1]) * D + tid);
    const float* x = xs[i & 1];
    float best = MUSE_NEG_INF;
    int bj = 0x7fffffff;
    for (int j = tid; j < C; j += 256) {
      if (count[j] >= cap) continue;
      float acc = 0.f;
#pragma unroll
      for (int d0 = 0; d0 < D; d0 += 4) {
        float c4[4];
        ld4(ch, (size_t)j * D + d0, c4);
        const float4 x4 = *reinterpret_cast<const float4*>(x + d0);
        acc = fmaf(c4[0], x4.x, acc); acc = fmaf(c4[1], x4.y, acc);
        acc = fmaf(c4[2], x4.z, acc); acc = fmaf(c4[3], x4.w, acc);
      }
      acc += nh[j];
      if (acc > best) {  // j increases: the first of equal scores stays
        best = acc;
        bj = j;
      }
    }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) {
      const float ov = __shfl_xor(best, o, 64);
      const int oj = __shfl_xor(bj, o, 64);
      if (ov > best || (ov == best && oj < bj)) {
        best = ov;
        bj = oj;
      }
    }
    if (lane == 0) {
      rv[wave] = best;
      rj[wave] = bj;
    }
    if (tid < D) xs[(i + 1) & 1][tid] = xn;
    __syncthreads();
    if (tid == 0) {
      float bv = rv[0];
      int j = rj[0];
      for (int q = 1; q < 4; ++q)
        if (rv[q] > bv || (rv[q] == bv && rj[q] < j)) {
          bv = rv[q];
          j = rj[q];
        }
      if (j < C) {  // always: a place is free somewhere, C cap >= Bs is checked by the host
        ah[row] = j;
        count[j] += 1;
      }
    }
    __syncthreads();
  }
}

size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

template <typename T>
int cluster_impl(const MuseDims& d, const T* X, int H, int C, const int32_t* init_idx, float* cent,
                 int32_t* assign, int32_t* trace, float* counts, void* ws, hipStream_t st) {
  const int N = d.N, D = d.D, heads = d.B * H;
  char* w = (char*)ws;
  T* chat = (T*)w;                w += align256((size_t)heads * C * D * sizeof(T));
  float* nhc2 = (float*)w;        w += align256((size_t)heads * C * sizeof(float));
  int32_t* perm = (int32_t*)w;    w += align256((size_t)heads * N * sizeof(int32_t));
  int32_t* off = (int32_t*)w;   w += align256((size_t)heads * ((size_t)d.nb * C + 1) * sizeof(int32_t));
  if (d.streaming) {
    // App. C "Centroid Computation": the streaming pass gives the centroids, one final assignment follows
    const size_t CS = (size_t)(C + 31) / 32 * 32;
    float* tst = (float*)w;        w += align256((size_t)heads * C * D * sizeof(float));
    float* cst = (float*)w;        w += align256((size_t)heads * CS * sizeof(float));
    _Float16* shat = (_Float16*)w; w += align256((size_t)heads * C * D * sizeof(_Float16));
    float* snh = (float*)w;
    const int per_wave = ((C + 31) / 32 + kStreamNW - 1) / kStreamNW;  // centroid tiles of a wave
    const int tbn = per_wave >= 4 && D == 64 ? 2 : 1;
    // state in LDS when it fits beside the kernel's static arrays (totals fp32, centroids binary16 with padded rows,
    // counts and norms)
    const size_t lds_state = (size_t)C * D * 4 + (size_t)C * (D + 8) * 2 + 2 * CS * 4;
    const bool ls = lds_state <= 128 * 1024;
#define MUSE_STREAM_LAUNCH(DD, TT)                                                                                  \
  {                                                                                                                 \
    MuseProf prof_("k_stream_kmeans", st);                                                                          \
    if (ls) {                                                                                                       \
      static bool attr_ = false;                                                                                    \
      if (!attr_) {                                                                                                 \
        MUSE_HIP_CHECK(hipFuncSetAttribute((const void*)k_stream_kmeans<T, DD, 1, true>,                            \
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 128 * 1024));                \
        attr_ = true;                                                                                               \
      }                                                                                                             \
      hipLaunchKernelGGL((k_stream_kmeans<T, DD, 1, true>), dim3(heads), dim3(64 * kStreamNW), lds_state, st, X,    \
                         init_idx, cent, tst, cst, shat, snh, trace, counts, N, C);                                 \
    } else {                                                                                                        \
      hipLaunchKernelGGL((k_stream_kmeans<T, DD, TT, false>), dim3(heads), dim3(64 * kStreamNW), 0, st, X, init_idx, \
                         cent, tst, cst, shat, snh, trace, counts, N, C);                                           \
    }                                                                                                               \
  }
    if (D == 64) {
      if (tbn == 2) MUSE_STREAM_LAUNCH(64, 2) else MUSE_STREAM_LAUNCH(64, 1)
    } else {
      MUSE_STREAM_LAUNCH(128, 1)
    }
#undef MUSE_STREAM_LAUNCH
    MUSE_LAUNCH_CHECK();
    if (!assign) return MUSE_OK;
  }
  const int T_ = d.streaming ? 0 : d.T;
  if (init_idx && !d.streaming) {
    { MuseProf prof_("k_init_centroids", st); hipLaunchKernelGGL(k_init_centroids<T>, dim3(C, heads), dim3(64), 0, st, X, init_idx, cent, N, D, C); }
    MUSE_LAUNCH_CHECK();
  }
  for (int it = 0; it <= T_; ++it) {
    int rows = heads * C;
    { MuseProf prof_("k_prep_centroids", st); hipLaunchKernelGGL(k_prep_centroids<T>, dim3((rows + 3) / 4), dim3(256), 0, st, cent, chat, nhc2, D, rows); }
    MUSE_LAUNCH_CHECK();
    if constexpr (sizeof(T) == 4) {
      dim3 g((N + 255) / 256, heads);
      if (D == 64) { MuseProf prof_("k_assign_f32", st); hipLaunchKernelGGL(k_assign_f32<64>, g, dim3(256), 0, st, (const float*)X, (const float*)chat, nhc2, assign, N, C); }
      else { MuseProf prof_("k_assign_f32", st); hipLaunchKernelGGL(k_assign_f32<128>, g, dim3(256), 0, st, (const float*)X, (const float*)chat, nhc2, assign, N, C); }
    } else {
      // all centroids resident in LDS when they fit (rows padded to a multiple of 64 for the tile pairs)
      const int Cpad = (C + 63) / 64 * 64;
      const size_t res_bytes = (size_t)Cpad * (D + 8) * 2 + (size_t)Cpad * 4;
      if (res_bytes <= 160 * 1024) {
        static bool attr_set = false;
        if (!attr_set) {
          MUSE_HIP_CHECK(hipFuncSetAttribute((const void*)k_assign_res<64>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
          MUSE_HIP_CHECK(hipFuncSetAttribute((const void*)k_assign_res<128>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
          attr_set = true;
        }
        const int bp = (D == 64 ? 64 : 32) * kResWaves;  // points per batch
        const int nbatch = (N + bp - 1) / bp;
        int gx = (256 + heads - 1) / heads;  // about one workgroup per CU over all heads
        gx = gx > nbatch ? nbatch : gx;
        dim3 g(gx, heads);
        if (D == 64) { MuseProf prof_("k_assign_bf16", st); hipLaunchKernelGGL(k_assign_res<64>, g, dim3(64 * kResWaves), res_bytes, st, (const bf16_t*)X, (const bf16_t*)chat, nhc2, assign, N, C, Cpad); }
        else { MuseProf prof_("k_assign_bf16", st); hipLaunchKernelGGL(k_assign_res<128>, g, dim3(64 * kResWaves), res_bytes, st, (const bf16_t*)X, (const bf16_t*)chat, nhc2, assign, N, C, Cpad); }
      } else {
        constexpr int PT = 2;
        dim3 g((N + 4 * 32 * PT - 1) / (4 * 32 * PT), heads);
        if (D == 64) { MuseProf prof_("k_assign_bf16", st); hipLaunchKernelGGL((k_assign_bf16<64, PT>), g, dim3(256), 0, st, (const bf16_t*)X, (const bf16_t*)chat, nhc2, assign, N, C); }
        else { MuseProf prof_("k_assign_bf16", st); hipLaunchKernelGGL((k_assign_bf16<128, PT>), g, dim3(256), 0, st, (const bf16_t*)X, (const bf16_t*)chat, nhc2, assign, N, C); }
      }
    }
    MUSE_LAUNCH_CHECK();
    if (it == T_ && d.balanced) {
      // App. C "Balanced Assignment": the nearest-centroid assignment bucketed by (block, cluster), then the rows
      // beyond the cap of their segment are placed again
      const int cap = (int)((4LL * d.Bs) / C);
      if (cap < 1 || (long long)cap * C < d.Bs) return MUSE_ERR_UNSUPPORTED;
      int rc = muse_launch_bucket(assign, heads, N, d.Bs, C, perm, off, st);
      if (rc) return rc;
      const size_t lds = (size_t)C * 4 + (size_t)((d.Bs + 31) / 32) * 4 + (size_t)d.Bs * 2 + 16;
      if (D == 64) { MuseProf prof_("k_balance", st); hipLaunchKernelGGL((k_balance<T, 64>), dim3(d.nb, heads), dim3(256), lds, st, X, chat, nhc2, perm, off, assign, N, d.Bs, C, cap); }
      else { MuseProf prof_("k_balance", st); hipLaunchKernelGGL((k_balance<T, 128>), dim3(d.nb, heads), dim3(256), lds, st, X, chat, nhc2, perm, off, assign, N, d.Bs, C, cap); }
      MUSE_LAUNCH_CHECK();
    }
    if (it == T_) break;
    int rc = muse_launch_bucket(assign, heads, N, d.Bs, C, perm, off, st);
    if (rc) return rc;
    { MuseProf prof_("k_update", st); hipLaunchKernelGGL(k_update<T>, dim3((rows + 3) / 4), dim3(256), 0, st, X, perm, off, cent, N, D, C, d.nb, rows); }
    MUSE_LAUNCH_CHECK();
  }
  return MUSE_OK;
}

}  // namespace

size_t muse_cluster_ws_bytes(const MuseDims& d) {
  size_t heads = (size_t)d.B * (d.Hq > d.Hkv ? d.Hq : d.Hkv);
  size_t C = d.Cq > d.Ck ? d.Cq : d.Ck;
  size_t CS = (C + 31) / 32 * 32;
  return align256(heads * C * d.D * 4) + align256(heads * C * 4) + align256(heads * d.N * 4) +
         align256(heads * ((size_t)d.nb * C + 1) * 4) +
         // state of the streaming pass: totals, counts, binary16 centroids and their -||c^||^2 / 2
         align256(heads * C * d.D * 4) + align256(heads * CS * 4) + align256(heads * C * d.D * 2) + align256(heads * CS * 4);
}

int muse_launch_bucket(const int32_t* assign, int heads, int N, int Bs, int C, int32_t* perm,
                       int32_t* off, hipStream_t st) {
  static_assert((size_t)17 * MUSE_MAX_CLUSTERS * sizeof(uint32_t) <= 150 * 1024, "histograms of the largest accepted C fit the LDS");
  size_t lds = (size_t)17 * C * sizeof(uint32_t);
  if (C > MUSE_MAX_CLUSTERS) return MUSE_ERR_UNSUPPORTED;  // the entry points have checked this already
  static bool attr_set = false;
  if (!attr_set) {
    MUSE_HIP_CHECK(hipFuncSetAttribute((const void*)k_bucket, hipFuncAttributeMaxDynamicSharedMemorySize, 150 * 1024));
    attr_set = true;
  }
  { MuseProf prof_("k_bucket", st); hipLaunchKernelGGL(k_bucket, dim3(N / Bs, heads), dim3(1024), lds, st, assign, perm, off, N, Bs, C); }
  MUSE_LAUNCH_CHECK();
  return MUSE_OK;
}

int muse_launch_cluster(const MuseDims& d, const void* X, int H, int C, const int32_t* init_idx,
                        float* cent, int32_t* assign, int32_t* trace, float* counts, void* ws, hipStream_t st) {
  if (d.dtype == MUSE_DTYPE_FP32) return cluster_impl<float>(d, (const float*)X, H, C, init_idx, cent, assign, trace, counts, ws, st);
  return cluster_impl<bf16_t>(d, (const bf16_t*)X, H, C, init_idx, cent, assign, trace, counts, ws, st);
}
