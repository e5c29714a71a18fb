// Far-field backward: gradient of the forward of Sec. 3.1-3.3 with the assignments, the selections
// and the query centroids held fixed (App. C "Centroid Gradient Flow"); gradient flows into K and
// V through the tilted aggregation weights (App. C "Aggregation Weight Gradient Flow", default).
//
// With p_u = exp(logit_u - LSE), delta = dO.O, dl_u = p_u (dO.value_u - delta) per virtual key:
//   summary keys (component 1 on accumulated cells, component 2 on per-block cells):
//     dq~ += dl kappa,  g_k[cell] += dl q~,  g_v[cell] += p dO,  g_mu[cell] += dl
//   a cell in unnormalised form (S = e^mu, Ksum = S kappa, Vsum = S vbar) receives
//     dKsum = g_k/S, dVsum = g_v/S, dS = c/S with c = g_mu - g_k.kappa - g_v.vbar,
//   accumulated cells are plain sums of per-block (S, Ksum, Vsum), and for a key m of a per-block
//   cell with w = exp(qbar.k_m - mu):  dv_m += w G_v,  dk_m += w G_k + w (G_c + G_k.k_m + G_v.v_m) qbar,
//   where G = own gradient + sum over later accumulated cells a of exp(mu - Amu[a]) gA[a].
// Every reduction has one owner (no float atomics): cells by (query cluster, key-cluster tile),
// keys by (key block, key-cluster tile).
#include <type_traits>

#include "ff_common.h"

namespace {

// The exported selections, re-indexed by bucketed query position p (consecutive p = one (block, cluster)
// group, so that every later read is coalesced):
//   slotinfo[hq][p][t] = j | (bitmask of the retrieved key blocks) << 16 for slot t, -1 when the slot is empty
//   selmask[hq][j/32][p]: bit j%32 set when query p retrieved key cluster j
__global__ void __launch_bounds__(256) k_selinfo(const int32_t* __restrict__ selc, const int32_t* __restrict__ selb,
                                                  const int32_t* __restrict__ perm_q, uint32_t* __restrict__ mask,
                                                  int32_t* __restrict__ slotinfo, int N, int r, int k2e, int W) {
  const size_t hq = blockIdx.y;
  const int p = blockIdx.x * 256 + threadIdx.x;
  if (p >= N) return;
  const size_t q = hq * N + perm_q[hq * N + p];
  int32_t* si = slotinfo + (hq * N + p) * r;
  int info[8];
#pragma unroll
  for (int t = 0; t < 8; ++t) info[t] = -1;
  if (r <= 8 && k2e == 1) {
    // the usual shape: the query's selections are requested together
    int jj[8], bb[8];
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      jj[t] = t < r ? selc[q * r + t] : -1;
      bb[t] = t < r ? selb[q * r + t] : -1;
    }
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      info[t] = jj[t] >= 0 ? (int)((uint32_t)jj[t] | ((bb[t] >= 0 ? 1u << bb[t] : 0u) << 16)) : -1;
      if (t < r) si[t] = info[t];
    }
  } else {
    for (int t = 0; t < r; ++t) {
      const int j = selc[q * r + t];
      int v = -1;
      if (j >= 0) {
        uint32_t bm = 0;
        for (int u = 0; u < k2e; ++u) {
          const int bb = selb[(q * r + t) * k2e + u];
          bm |= bb >= 0 ? 1u << bb : 0u;
        }
        v = (int)((uint32_t)j | (bm << 16));
      }
      si[t] = v;
#pragma unroll
      for (int k = 0; k < 8; ++k)
        if (k == t) info[k] = v;
    }
  }
  for (int w = 0; w < W; ++w) {
    uint32_t m = 0;
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      const int j = info[k] & 0xffff;
      if (info[k] >= 0 && (j >> 5) == w) m |= 1u << (j & 31);
    }
    for (int t = 8; t < r; ++t) {
      const int v = si[t], j = v & 0xffff;
      if (v >= 0 && (j >> 5) == w) m |= 1u << (j & 31);
    }
    mask[(hq * W + w) * N + p] = m;
  }
}

// ------------------------------------------------------------------------------------------
// dQ of the far field, one wave per query tile (same tiling as the forward kernel)
// ------------------------------------------------------------------------------------------
template <typename T, int D>
__global__ void __launch_bounds__(64) __attribute__((amdgpu_waves_per_eu(D == 64 ? 2 : 1, 2))) k_ff_bwd_dq(
    const T* __restrict__ Q, const T* __restrict__ dO, const float* __restrict__ qc, const T* __restrict__ Ks,
    const T* __restrict__ Vs, const float* __restrict__ L, const float* __restrict__ s_mu,
    const float* __restrict__ s_k, const T* __restrict__ s_v, const float* __restrict__ A_mu,
    const float* __restrict__ A_k, const T* __restrict__ A_v, const bf16_t* __restrict__ A_kb,
    const int32_t* __restrict__ perm_q,
    const int32_t* __restrict__ off_q, const int32_t* __restrict__ off_k, const int32_t* __restrict__ tile_off,
    const float* __restrict__ LSE, const float* __restrict__ delta, const uint32_t* __restrict__ selmask,
    const int32_t* __restrict__ selc, const int32_t* __restrict__ selb, const float* __restrict__ dqpart,
    float* __restrict__ dQ, int h0, int N, int nb, int Cq, int Ck, int r, int k2e, int Hq, int Hkv, float scale) {
  constexpr int U = D / 8, DT = D / 32;
  const int hl = blockIdx.z, hq = h0 + hl;
  const int hk = (hq / Hq) * Hkv + (hq % Hq) / (Hq / Hkv);
  const int b = blockIdx.y + 1, NBm = nb - 1;
  const int lane = threadIdx.x, col = lane % 32, half = lane / 32;
  const int W = (Ck + 31) / 32;

  const int32_t* to = tile_off + ((size_t)hq * nb + b) * (Cq + 1);
  // x % 8 is the XCD (grid x extent a multiple of 8): each XCD takes a contiguous run of the tiles, so the
  // tiles of one (block, query cluster) group share its L2
  const int ntl = to[Cq], run = (ntl + 7) / 8;
  const int tile = (blockIdx.x % 8) * run + blockIdx.x / 8;
  if ((int)blockIdx.x / 8 >= run || tile >= ntl) return;
  int lo_ = 0, hi_ = Cq;
  while (hi_ - lo_ > 1) {
    int mid = (lo_ + hi_) >> 1;
    if (to[mid] <= tile) lo_ = mid; else hi_ = mid;
  }
  const int i = lo_, tt = tile - to[lo_];
  const int32_t* oq = off_q + (size_t)hq * ((size_t)nb * Cq + 1);
  const int32_t* ok = off_k + (size_t)hk * ((size_t)nb * Ck + 1);
  const int qlo = oq[b * Cq + i], qhi = oq[b * Cq + i + 1];
  int pos = qlo + 32 * tt + col;
  const bool valid = pos < qhi;
  pos = valid ? pos : qlo + 32 * tt;
  const int n = perm_q[(size_t)hq * N + pos];
  const size_t qn = (size_t)hq * N + n;

  float qt[U][4], gt[U][4];
  {
    const float* qci = qc + ((size_t)hq * Cq + i) * D;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      float x[4];
      ld4(Q, qn * D + 8 * u + 4 * half, x);
      float4 c = *reinterpret_cast<const float4*>(qci + 8 * u + 4 * half);
      qt[u][0] = scale * (x[0] - c.x); qt[u][1] = scale * (x[1] - c.y);
      qt[u][2] = scale * (x[2] - c.z); qt[u][3] = scale * (x[3] - c.w);
      ld4(dO, qn * D + 8 * u + 4 * half, gt[u]);
    }
  }
  const float lse = LSE[qn], dl = delta[qn];
  const size_t acell = (((size_t)hl * NBm + (b - 1)) * Cq + i) * Ck;
  const float* Amu = A_mu + acell;
  const float* Ak = A_k + acell * D;
  const float* Avf = reinterpret_cast<const float*>(A_v) + acell * D;   // fp32 inputs
  const bf16_t* Akh = A_kb + acell * D;                                  // bf16 inputs
  const bf16_t* Avh = reinterpret_cast<const bf16_t*>(A_v) + acell * D;
  const int ntile = (Ck + 31) / 32;

  f32x16_t dq[DT];
#pragma unroll
  for (int t = 0; t < DT; ++t) dq[t] = zero16();
  // component 1
  if (sizeof(T) == 2) {
    // bf16 inputs: operands rounded to bf16 for the matrix cores (gradients only)
    constexpr int KS = D / 16;
    bf16x8_t qb[KS], gb[KS];
    // the bf16 operand order (8 consecutive dims per lane half) differs from the fp32 row pattern of qt/gt
    {
      const float* qci = qc + ((size_t)hq * Cq + i) * D;
#pragma unroll
      for (int x = 0; x < KS; ++x) {
        float q8[8], g8[8];
        ld4(Q, qn * D + 16 * x + 8 * half, q8); ld4(Q, qn * D + 16 * x + 8 * half + 4, q8 + 4);
        ld4(dO, qn * D + 16 * x + 8 * half, g8); ld4(dO, qn * D + 16 * x + 8 * half + 4, g8 + 4);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          qb[x][e] = (__bf16)(scale * (q8[e] - qci[16 * x + 8 * half + e]));
          gb[x][e] = (__bf16)g8[e];
        }
      }
    }
    // a tile's operands: this lane's k-bar and v-bar rows (cluster j0 + col, its half of every 16 dims), the
    // mu-bar of the 16 clusters whose scores land in this lane, and the retrieved-cluster mask of its query.
    // Two buffers: the next tile's loads are in flight while this one is used; loads are unconditional (a tile
    // index past the end repeats the last tile) and the values stay raw until they are used.
    struct BT {
      uint4 k[KS], v[KS];
      float mu[16];
      uint32_t mw;
    };
    auto load_bt = [&](BT& t, int jt) {
      jt = jt < ntile ? jt : ntile - 1;
      const int j0 = jt * 32;
      int c = j0 + col;
      c = c < Ck ? c : Ck - 1;
#pragma unroll
      for (int x = 0; x < KS; ++x) {
        t.k[x] = *reinterpret_cast<const uint4*>(Akh + (size_t)c * D + 16 * x + 8 * half);
        t.v[x] = *reinterpret_cast<const uint4*>(Avh + (size_t)c * D + 16 * x + 8 * half);
      }
      if ((Ck & 3) == 0) {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          int base = j0 + 8 * g + 4 * half;
          base = base < Ck ? base : Ck - 4;
          const float4 m4 = *reinterpret_cast<const float4*>(Amu + base);
          t.mu[4 * g] = m4.x; t.mu[4 * g + 1] = m4.y; t.mu[4 * g + 2] = m4.z; t.mu[4 * g + 3] = m4.w;
        }
      } else {
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int jr = j0 + 8 * (e / 4) + 4 * half + (e % 4);
          t.mu[e] = Amu[jr < Ck ? jr : Ck - 1];
        }
      }
      t.mw = selmask[((size_t)hq * W + jt) * N + pos];
    };
    // k-bar tile transposed ([dim][cluster]) for the dq contraction; lanes run along the clusters: 2-byte stores
    // into consecutive banks
    __shared__ __attribute__((aligned(16))) bf16_t kt[D][32 + 4];
    auto process = [&](const BT& t, int jt) {
      const int j0 = jt * 32;
      f32x16_t s, dp;
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        s[e] = t.mu[e];
        dp[e] = 0.f;
      }
#pragma unroll
      for (int x = 0; x < KS; ++x) {
        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, t.k[x]), qb[x], s, 0, 0, 0);
        dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, t.v[x]), gb[x], dp, 0, 0, 0);
      }
      wave_lds_fence();
#pragma unroll
      for (int x = 0; x < KS; ++x) {
        const uint32_t w4[4] = {t.k[x].x, t.k[x].y, t.k[x].z, t.k[x].w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          kt[16 * x + 8 * half + 2 * e][col] = (bf16_t)(w4[e] & 0xffffu);
          kt[16 * x + 8 * half + 2 * e + 1][col] = (bf16_t)(w4[e] >> 16);
        }
      }
      wave_lds_fence();
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int row = 8 * (e / 4) + 4 * half + (e % 4);
        const bool off_ = ((t.mw >> row) & 1u) || j0 + row >= Ck;  // retrieved, or past the last cluster
        const float p = off_ ? 0.f : __expf(s[e] - lse);
        s[e] = p * (dp[e] - dl);
      }
#pragma unroll
      for (int G = 0; G < 2; ++G) {
        const bf16x8_t df = pack8(s, 2 * G, 2 * G + 1);
#pragma unroll
        for (int x = 0; x < DT; ++x)
          dq[x] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ld_tr8(&kt[32 * x + col][0], 16 * G, half), df, dq[x], 0, 0, 0);
      }
    };
    BT ta, tb;
    load_bt(ta, 0);
    for (int jt = 0; jt < ntile; jt += 2) {
      load_bt(tb, jt + 1);
      process(ta, jt);
      if (jt + 1 < ntile) {
        load_bt(ta, jt + 2);
        process(tb, jt + 1);
      }
    }
  } else
  for (int jt = 0; jt < ntile; ++jt) {
    const int j0 = jt * 32;
    f32x16_t s = score_tile<D>(Amu, Ak, j0, Ck, qt, col, half);
    int c = j0 + col;
    c = c < Ck ? c : Ck - 1;
    f32x16_t dp = mfma_rows<D>(zero16(), Avf + (size_t)c * D + 4 * half, gt);
    const uint32_t mw = selmask[((size_t)hq * W + jt) * N + pos];
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      int row = 8 * (e / 4) + 4 * half + (e % 4);
      float p = ((mw >> row) & 1u) ? 0.f : __expf(s[e] - lse);
      s[e] = p * (dp[e] - dl);
    }
#pragma unroll
    for (int g = 0; g < 4; ++g)
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        int jr = j0 + 8 * g + 4 * half + t;
        jr = jr < Ck ? jr : Ck - 1;
        const float* krow = Ak + (size_t)jr * D + col;
#pragma unroll
        for (int x = 0; x < DT; ++x) dq[x] = mfma32(krow[32 * x], s[4 * g + t], dq[x]);
      }
  }
  // components 2 and 3 (fp32 inputs; bf16 inputs take them in the per-query and per-pair kernels)
  for (int t = 0; t < (sizeof(T) == 4 ? r : 0); ++t) {
    const int j = selc[qn * r + t];
    if (j < 0) continue;
    unsigned selbits = 0;
    for (int u = 0; u < k2e; ++u) {
      int bb = selb[(qn * r + t) * k2e + u];
      if (bb >= 0) selbits |= 1u << bb;
    }
    for (int bp = 0; bp < b; ++bp) {
      const size_t cell = (((size_t)hl * NBm + bp) * Cq + i) * Ck + j;
      const float mu = s_mu[cell];
      if (!(mu > MUSE_NEG_INF)) continue;
      if (!((selbits >> bp) & 1u)) {
        const float* kr = s_k + cell * D + 4 * half;
        float part = 0.f, dpp = 0.f;
        float4 k4[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
          k4[u] = *reinterpret_cast<const float4*>(kr + 8 * u);
          float v4[4];
          ld4(s_v, cell * D + 4 * half + 8 * u, v4);
          part = fmaf(qt[u][0], k4[u].x, part); part = fmaf(qt[u][1], k4[u].y, part);
          part = fmaf(qt[u][2], k4[u].z, part); part = fmaf(qt[u][3], k4[u].w, part);
          dpp = fmaf(gt[u][0], v4[0], dpp); dpp = fmaf(gt[u][1], v4[1], dpp);
          dpp = fmaf(gt[u][2], v4[2], dpp); dpp = fmaf(gt[u][3], v4[3], dpp);
        }
        part += __shfl_xor(part, 32, 64);
        dpp += __shfl_xor(dpp, 32, 64);
        float p = __expf(part + mu - lse);
        float dlg = p * (dpp - dl);
#pragma unroll
        for (int u = 0; u < U; ++u) {
          dq[u / 4][4 * (u % 4) + 0] += dlg * k4[u].x; dq[u / 4][4 * (u % 4) + 1] += dlg * k4[u].y;
          dq[u / 4][4 * (u % 4) + 2] += dlg * k4[u].z; dq[u / 4][4 * (u % 4) + 3] += dlg * k4[u].w;
        }
      } else if (sizeof(T) == 4) {
        const int klo = ok[bp * Ck + j], khi = ok[bp * Ck + j + 1];
        for (int p_ = klo; p_ < khi; ++p_) {
          const size_t krow = ((size_t)hk * N + p_) * D + 4 * half;
          float part = 0.f, dpp = 0.f;
          float k4[U][4];
#pragma unroll
          for (int u = 0; u < U; ++u) {
            float v4[4];
            ld4(Ks, krow + 8 * u, k4[u]);
            ld4(Vs, krow + 8 * u, v4);
#pragma unroll
            for (int x = 0; x < 4; ++x) {
              part = fmaf(qt[u][x], k4[u][x], part);
              dpp = fmaf(gt[u][x], v4[x], dpp);
            }
          }
          part += __shfl_xor(part, 32, 64);
          dpp += __shfl_xor(dpp, 32, 64);
          float p = __expf(part + L[((size_t)hl * Cq + i) * N + p_] - lse);
          float dlg = p * (dpp - dl);
#pragma unroll
          for (int u = 0; u < U; ++u)
#pragma unroll
            for (int x = 0; x < 4; ++x) dq[u / 4][4 * (u % 4) + x] += dlg * k4[u][x];
        }
      }
    }
  }
  if (!valid) return;
  float res[U][4];
#pragma unroll
  for (int u = 0; u < U; ++u)
#pragma unroll
    for (int x = 0; x < 4; ++x) res[u][x] = scale * dq[u / 4][4 * (u % 4) + x];
  float* out = dQ + qn * D + 4 * half;
#pragma unroll
  for (int u = 0; u < U; ++u)
    *reinterpret_cast<float4*>(out + 8 * u) = make_float4(res[u][0], res[u][1], res[u][2], res[u][3]);
}

// ------------------------------------------------------------------------------------------
// dQ of component 2 for bf16 inputs, per query (16 lanes, dims 64 x + 4 l16 + t, bucketed order, as in the
// forward): for every retrieved cluster, the summaries of the preceding blocks that were NOT retrieved
// contribute  dl k-bar  with  dl = p (dO.v-bar - delta),  p = exp(q~.k-bar + mu-bar - LSE).  The retrieval's
// per-pair dq partials are added here too, and the sum is added to the row the tile kernel wrote.
// ------------------------------------------------------------------------------------------
template <int D, int NBC>
__global__ void __launch_bounds__(256) k_comp2_bwd_dq(
    const bf16_t* __restrict__ Q, const bf16_t* __restrict__ dO, const float* __restrict__ qc,
    const float* __restrict__ s_mu, const float* __restrict__ s_k, const bf16_t* __restrict__ s_v,
    const int32_t* __restrict__ perm_q, const int32_t* __restrict__ aq, const float* __restrict__ LSE,
    const float* __restrict__ delta, const int32_t* __restrict__ slotinfo, const float* __restrict__ dqpart,
    float* __restrict__ dQ, int h0, int N, int nb, int Bs, int Cq, int Ck, int r, int k2e, float scale) {
  constexpr int NG = D / 64;
  const int hl = blockIdx.y, hq = h0 + hl;
  const int l16 = threadIdx.x % 16;
  // Workgroups go to the 8 XCDs round-robin by their linear id (the grid's x extent is a multiple of 256): an XCD
  // takes runs of 32 consecutive workgroups of the bucketed order, so the queries of one cluster, which read the
  // same summary rows, meet in one L2, while the late blocks (more work per query) still spread over all XCDs.
  const int sq = blockIdx.x / 8;
  const int wg = ((sq / 32) * 8 + blockIdx.x % 8) * 32 + sq % 32;
  const int pos = Bs + wg * 16 + threadIdx.x / 16;  // bucketed order is block-major: block 0 comes first
  if (pos >= N) return;
  const int n = perm_q[(size_t)hq * N + pos];
  const size_t qn = (size_t)hq * N + n;
  const int b = pos / Bs, NBm = nb - 1;
  const int i = aq[qn];
  const float lse = LSE[qn], dl = delta[qn];
  float qt[NG][4], gt[NG][4], dq[NG][4];
#pragma unroll
  for (int x = 0; x < NG; ++x) {
    float q4[4];
    ld4(Q, qn * D + 64 * x + 4 * l16, q4);
    ld4(dO, qn * D + 64 * x + 4 * l16, gt[x]);
    const float4 c4 = *reinterpret_cast<const float4*>(qc + ((size_t)hq * Cq + i) * D + 64 * x + 4 * l16);
    qt[x][0] = scale * (q4[0] - c4.x); qt[x][1] = scale * (q4[1] - c4.y);
    qt[x][2] = scale * (q4[2] - c4.z); qt[x][3] = scale * (q4[3] - c4.w);
#pragma unroll
    for (int t = 0; t < 4; ++t) dq[x][t] = 0.f;
  }
  const int32_t* si = slotinfo + ((size_t)hq * N + pos) * r;
  // the row this kernel adds to is requested now and used at the end
  float4 oldq[NG];
#pragma unroll
  for (int x = 0; x < NG; ++x) oldq[x] = *reinterpret_cast<const float4*>(dQ + qn * D + 64 * x + 4 * l16);
  // the four queries of a wave are neighbours in the block-major order: the largest b among them (wave-uniform)
  // bounds the block loops
  // (the bound is a template constant of the loop body below: one straight-line body per value, loads batched)
  int bwv = b;
  bwv = max(bwv, __shfl_xor(bwv, 16, 64));
  bwv = max(bwv, __shfl_xor(bwv, 32, 64));
  bwv = __builtin_amdgcn_readfirstlane(bwv);
  auto run = [&](auto bw_c) {
  constexpr int bw = decltype(bw_c)::value;
  for (int t = 0; t < r; ++t) {
    const int info = si[t];
    if (info < 0) continue;
    const int j = info & 0xffff;
    const unsigned selbits = (unsigned)info >> 16;
#pragma unroll
    for (int c0 = 0; c0 < 8 * NBC; c0 += 8) {
      if (c0 >= bw) break;
      float mu[8], part[8], dpp[8];
      float4 kr[8][NG];
      float vr[8][NG][4];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        if (c0 + u >= bw) break;
        const int bp = c0 + u < b ? c0 + u : b - 1;
        const size_t cell = (((size_t)hl * NBm + bp) * Cq + i) * Ck + j;
        mu[u] = s_mu[cell];
#pragma unroll
        for (int x = 0; x < NG; ++x) {
          kr[u][x] = *reinterpret_cast<const float4*>(s_k + cell * D + 64 * x + 4 * l16);
          ld4(s_v, cell * D + 64 * x + 4 * l16, vr[u][x]);
        }
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        if (c0 + u >= bw) break;
        float pa = 0.f, pd = 0.f;
#pragma unroll
        for (int x = 0; x < NG; ++x) {
          pa = fmaf(qt[x][0], kr[u][x].x, pa); pa = fmaf(qt[x][1], kr[u][x].y, pa);
          pa = fmaf(qt[x][2], kr[u][x].z, pa); pa = fmaf(qt[x][3], kr[u][x].w, pa);
          pd = fmaf(gt[x][0], vr[u][x][0], pd); pd = fmaf(gt[x][1], vr[u][x][1], pd);
          pd = fmaf(gt[x][2], vr[u][x][2], pd); pd = fmaf(gt[x][3], vr[u][x][3], pd);
        }
        part[u] = pa; dpp[u] = pd;
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        if (c0 + u >= bw) break;
        part[u] = group_sum<16>(part[u]);
        dpp[u] = group_sum<16>(dpp[u]);
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        if (c0 + u >= bw) break;
        const bool use = c0 + u < b && mu[u] > MUSE_NEG_INF && !((selbits >> (c0 + u)) & 1u);
        const float p = use ? __expf(part[u] + mu[u] - lse) : 0.f;
        const float dlg = p * (dpp[u] - dl);
#pragma unroll
        for (int x = 0; x < NG; ++x) {
          dq[x][0] = fmaf(dlg, kr[u][x].x, dq[x][0]); dq[x][1] = fmaf(dlg, kr[u][x].y, dq[x][1]);
          dq[x][2] = fmaf(dlg, kr[u][x].z, dq[x][2]); dq[x][3] = fmaf(dlg, kr[u][x].w, dq[x][3]);
        }
      }
    }
  }
  };
  if (NBC == 1) {
    switch (bwv) {
      case 1: run(std::integral_constant<int, 1>{}); break;
      case 2: run(std::integral_constant<int, 2>{}); break;
      case 3: run(std::integral_constant<int, 3>{}); break;
      case 4: run(std::integral_constant<int, 4>{}); break;
      case 5: run(std::integral_constant<int, 5>{}); break;
      case 6: run(std::integral_constant<int, 6>{}); break;
      case 7: run(std::integral_constant<int, 7>{}); break;
      default: run(std::integral_constant<int, 8>{}); break;
    }
  } else {
    run(std::integral_constant<int, 8 * NBC>{});
  }
#pragma unroll
  for (int x = 0; x < NG; ++x)
#pragma unroll
    for (int t = 0; t < 4; ++t) dq[x][t] *= scale;
  // retrieval part, computed per retrieved pair (already scaled); a slot's pair u exists iff its block bit is set
  if (k2e == 1 && r <= 8) {
    // the usual shape: the partial rows of all slots are requested together and added in slot order
    int inf[8];
#pragma unroll
    for (int t = 0; t < 8; ++t) inf[t] = t < r ? si[t] : -1;
    float4 v[8][NG];
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      const bool ok = inf[t] >= 0 && ((unsigned)inf[t] >> 16) != 0u;
#pragma unroll
      for (int x = 0; x < NG; ++x)
        v[t][x] = ok ? *reinterpret_cast<const float4*>(dqpart + (qn * r + t) * D + 64 * x + 4 * l16) : make_float4(0.f, 0.f, 0.f, 0.f);
    }
#pragma unroll
    for (int t = 0; t < 8; ++t)
#pragma unroll
      for (int x = 0; x < NG; ++x) { dq[x][0] += v[t][x].x; dq[x][1] += v[t][x].y; dq[x][2] += v[t][x].z; dq[x][3] += v[t][x].w; }
  } else {
    for (int t = 0; t < r; ++t) {
      const int info = si[t];
      if (info < 0 || ((unsigned)info >> 16) == 0u) continue;
      for (int u = 0; u < k2e; ++u) {
        const float* pp = dqpart + (qn * r * k2e + t * k2e + u) * D;
        if (u < (int)__popc((unsigned)info >> 16)) {
#pragma unroll
          for (int x = 0; x < NG; ++x) {
            const float4 v = *reinterpret_cast<const float4*>(pp + 64 * x + 4 * l16);
            dq[x][0] += v.x; dq[x][1] += v.y; dq[x][2] += v.z; dq[x][3] += v.w;
          }
        }
      }
    }
  }
#pragma unroll
  for (int x = 0; x < NG; ++x) {
    float4* out = reinterpret_cast<float4*>(dQ + qn * D + 64 * x + 4 * l16);
    float4 o = oldq[x];
    o.x += dq[x][0]; o.y += dq[x][1]; o.z += dq[x][2]; o.w += dq[x][3];
    *out = o;
  }
}

// ------------------------------------------------------------------------------------------
// gradients of the accumulated cells (component 1): one wave per (query block b, query cluster i,
// tile of 32 key clusters); loops over the queries of the group.  Writes every cell it owns:
//   g_A_k = sum dl q~,  g_A_v = sum p dO,  g_A_c = sum [dl (1 - q~.kappa) - p dO.vbar]
// ------------------------------------------------------------------------------------------
template <typename T, int D>
__global__ void __launch_bounds__(64) k_ff_bwd_cells(
    const T* __restrict__ Q, const T* __restrict__ dO, const float* __restrict__ qc, const float* __restrict__ A_mu,
    const float* __restrict__ A_k, const float* __restrict__ A_v, const int32_t* __restrict__ perm_q,
    const int32_t* __restrict__ off_q, const float* __restrict__ LSE, const float* __restrict__ delta,
    const uint32_t* __restrict__ selmask, float* __restrict__ g_A_c, float* __restrict__ g_A_k,
    float* __restrict__ g_A_v, int h0, int N, int nb, int Cq, int Ck, float scale) {
  constexpr int U = D / 8, DT = D / 32;
  __shared__ int ns[32];
  __shared__ float ls[32], ds[32];
  __shared__ uint32_t mws[32];
  const int hl = blockIdx.z, hq = h0 + hl;
  const int NBm = nb - 1;
  const int b = blockIdx.y / Cq + 1, i = blockIdx.y % Cq;
  const int jt = blockIdx.x, j0 = jt * 32;
  const int lane = threadIdx.x, col = lane % 32, half = lane / 32;
  const int W = (Ck + 31) / 32;
  const int32_t* oq = off_q + (size_t)hq * ((size_t)nb * Cq + 1);
  const int qlo = oq[b * Cq + i], qhi = oq[b * Cq + i + 1];
  const size_t acell = (((size_t)hl * NBm + (b - 1)) * Cq + i) * Ck;
  const int jc = j0 + col;
  const bool jvalid = jc < Ck;
  const int jcc = jvalid ? jc : Ck - 1;
  // B operands: this lane's key cluster
  float kt[U][4], vt[U][4];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    float4 a = *reinterpret_cast<const float4*>(A_k + (acell + jcc) * D + 8 * u + 4 * half);
    float4 c = *reinterpret_cast<const float4*>(A_v + (acell + jcc) * D + 8 * u + 4 * half);
    kt[u][0] = a.x; kt[u][1] = a.y; kt[u][2] = a.z; kt[u][3] = a.w;
    vt[u][0] = c.x; vt[u][1] = c.y; vt[u][2] = c.z; vt[u][3] = c.w;
  }
  const float amu = jvalid ? A_mu[acell + jcc] : MUSE_NEG_INF;
  const float* qci = qc + ((size_t)hq * Cq + i) * D;
  f32x16_t gk[DT], gv[DT];
#pragma unroll
  for (int t = 0; t < DT; ++t) { gk[t] = zero16(); gv[t] = zero16(); }
  float csum = 0.f;
  for (int q0 = qlo; q0 < qhi; q0 += 32) {
    __syncthreads();
    if (half == 0) {
      int pos = q0 + col;
      bool ok_ = pos < qhi;
      int n = perm_q[(size_t)hq * N + (ok_ ? pos : q0)];
      ns[col] = n;
      ls[col] = ok_ ? LSE[(size_t)hq * N + n] : __builtin_huge_valf();  // +inf -> p = 0 for padding rows
      ds[col] = delta[(size_t)hq * N + n];
      mws[col] = selmask[((size_t)hq * W + jt) * N + (ok_ ? pos : q0)];
    }
    __syncthreads();
    // A operands (row pattern): this lane's query row
    const size_t qn = (size_t)hq * N + ns[col];
    f32x16_t s = zero16(), dp = zero16();
#pragma unroll
    for (int u = 0; u < U; ++u) {
      float x[4], g[4];
      ld4(Q, qn * D + 8 * u + 4 * half, x);
      ld4(dO, qn * D + 8 * u + 4 * half, g);
      float4 c = *reinterpret_cast<const float4*>(qci + 8 * u + 4 * half);
      s = mfma32(scale * (x[0] - c.x), kt[u][0], s); s = mfma32(scale * (x[1] - c.y), kt[u][1], s);
      s = mfma32(scale * (x[2] - c.z), kt[u][2], s); s = mfma32(scale * (x[3] - c.w), kt[u][3], s);
      dp = mfma32(g[0], vt[u][0], dp); dp = mfma32(g[1], vt[u][1], dp);
      dp = mfma32(g[2], vt[u][2], dp); dp = mfma32(g[3], vt[u][3], dp);
    }
    f32x16_t pr;
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      int row = 8 * (e / 4) + 4 * half + (e % 4);
      float p = __expf(s[e] + amu - ls[row]);   // amu = -inf or lse = +inf -> 0
      p = ((mws[row] >> col) & 1u) ? 0.f : p;
      float dlg = p * (dp[e] - ds[row]);
      csum += p > 0.f ? dlg * (1.f - s[e]) - p * dp[e] : 0.f;
      pr[e] = p;
      s[e] = dlg;
    }
    // g_k^T [D x clusters] += q~^T dl,  g_v^T += dO^T p  (column pattern over the query rows)
#pragma unroll
    for (int g = 0; g < 4; ++g)
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        const size_t rn = (size_t)hq * N + ns[8 * g + 4 * half + t];
#pragma unroll
        for (int x = 0; x < DT; ++x) {
          float qv = scale * (Elem<T>::ld(Q, rn * D + 32 * x + col) - qci[32 * x + col]);
          float gvv = Elem<T>::ld(dO, rn * D + 32 * x + col);
          gk[x] = mfma32(qv, s[4 * g + t], gk[x]);
          gv[x] = mfma32(gvv, pr[4 * g + t], gv[x]);
        }
      }
  }
  csum += __shfl_xor(csum, 32, 64);
  if (!jvalid) return;
  float* ok_ = g_A_k + (acell + jc) * D;
  float* ov_ = g_A_v + (acell + jc) * D;
#pragma unroll
  for (int x = 0; x < DT; ++x)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      int d = 32 * x + 8 * g + 4 * half;
      *reinterpret_cast<float4*>(ok_ + d) = make_float4(gk[x][4 * g], gk[x][4 * g + 1], gk[x][4 * g + 2], gk[x][4 * g + 3]);
      *reinterpret_cast<float4*>(ov_ + d) = make_float4(gv[x][4 * g], gv[x][4 * g + 1], gv[x][4 * g + 2], gv[x][4 * g + 3]);
    }
  if (half == 0) g_A_c[acell + jc] = csum;
}

// ------------------------------------------------------------------------------------------
// Gradients of the per-block cells from those of the accumulated cells: one block of 256 threads per (query
// cluster i, tile of 32 key clusters); wave w owns the 8 chains (i, j, all blocks), j = 32 jt + 8 w + c.  A
// wave is 8 groups of 8 lanes; a lane holds D/8 elements of a row (d = 32 x + 4 l8 + t); group c owns chain c.
// Reverse accumulation over the key blocks a = nb-2 .. 0, in registers:
//      R[a] = gA[a] + exp(Amu[a] - Amu[a+1]) R[a+1],   G[a] = exp(mu[a] - Amu[a]) R[a]   (written out)
// All factors are <= 1.  One owner per cell.  Component 2 is added afterwards by k_chain_grads.
// ------------------------------------------------------------------------------------------
template <typename T, int D>
__global__ void __launch_bounds__(256) k_cell_grads(
    const float* __restrict__ s_mu, const float* __restrict__ A_mu, const float* __restrict__ g_A_c,
    const T* __restrict__ g_A_k, const T* __restrict__ g_A_v, float* __restrict__ G_c, T* __restrict__ G_k,
    T* __restrict__ G_v, int nb, int Cq, int Ck) {
  constexpr int NV = D / 32;
  using F4 = Frag<T, 4>;
  const int hl = blockIdx.z;
  const int i = blockIdx.y, jt = blockIdx.x;
  const int tid = threadIdx.x, lane = tid % 64, wave = tid / 64, s8 = lane / 8, l8 = lane % 8;
  const int NBm = nb - 1;

  const int jown = jt * 32 + 8 * wave + s8;
  const bool jok = jown < Ck;
  {
    float Rk[NV][4], Rv[NV][4], an = 0.f, rc = 0.f;
#pragma unroll
    for (int x = 0; x < NV; ++x)
#pragma unroll
      for (int t = 0; t < 4; ++t) { Rk[x][t] = 0.f; Rv[x][t] = 0.f; }
    struct Step {
      float Am, mu, gac;
      typename F4::raw gak[NV], gav[NV];
    };
    auto load_step = [&](int a, Step& st) {
      const size_t cell = (((size_t)hl * NBm + a) * Cq + i) * Ck + (jok ? jown : Ck - 1);
      st.Am = A_mu[cell]; st.mu = s_mu[cell]; st.gac = g_A_c[cell];
#pragma unroll
      for (int x = 0; x < NV; ++x) {
        st.gak[x] = F4::ld(g_A_k, cell * D + 32 * x + 4 * l8);
        st.gav[x] = F4::ld(g_A_v, cell * D + 32 * x + 4 * l8);
      }
    };
    // the loads of up to 8 steps are issued together: the recurrence itself is a few multiply-adds per step
    for (int a1 = NBm - 1; a1 >= 0; a1 -= 8) {
      Step st[8];
#pragma unroll
      for (int u = 0; u < 8; ++u)
        if (a1 - u >= 0) load_step(a1 - u, st[u]);
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int a = a1 - u;
        if (a < 0 || !jok) continue;
        const Step& cur = st[u];
        const size_t cell = (((size_t)hl * NBm + a) * Cq + i) * Ck + jown;
        const float f = (a < NBm - 1 && cur.Am > MUSE_NEG_INF) ? __expf(cur.Am - an) : 0.f;
        const float wgt = cur.mu > MUSE_NEG_INF ? __expf(cur.mu - cur.Am) : 0.f;
        rc = cur.gac + f * rc;
        an = cur.Am;
        if (l8 == 0) G_c[cell] = wgt * rc;
#pragma unroll
        for (int x = 0; x < NV; ++x) {
          float ok4[4], ov4[4];
#pragma unroll
          for (int t = 0; t < 4; ++t) {
            Rk[x][t] = F4::get(cur.gak[x], t) + f * Rk[x][t];
            Rv[x][t] = F4::get(cur.gav[x], t) + f * Rv[x][t];
            ok4[t] = wgt * Rk[x][t];
            ov4[t] = wgt * Rv[x][t];
          }
          st4(G_k, cell * D + 32 * x + 4 * l8, ok4);
          st4(G_v, cell * D + 32 * x + 4 * l8, ov4);
        }
      }
    }
  }
}

// ------------------------------------------------------------------------------------------
// Component 2 of the per-block cell gradients: every query of cluster i in a later block that retrieved
// cluster j but not block a adds  g_k += dl q~,  g_v += p dO,  g_c += dl (1 - q~.kbar) - p dO.vbar  to the
// cell (a, i, j) that k_cell_grads wrote.  One block of 256 threads per (head, query cluster i): it takes the
// cluster's queries (bucketed order, blocks >= 1) a chunk at a time, stages their Q and dO rows, LSE and delta
// in LDS once, lists the (query, slot) entries by chain j with a counting sort over all Ck chains, and gives
// each non-empty chain to a wave.  About one chain in ten has entries, and those that do have many.  For a
// chain, the 8-lane group g takes key block a = g, so that the loads of all its blocks are one round trip; a
// lane holds D/8 elements of a row (d = 32 x + 4 l8 + t).  The counting sort places entries in arrival order;
// the wave that owns a chain then orders them by query, so every sum has a fixed order.  One owner per cell
// (chain j -> wave (j / 64) % 4, block a -> group): no atomics on floats.
// ------------------------------------------------------------------------------------------
template <typename T, int D>
__global__ void __launch_bounds__(256) k_chain_grads(
    const T* __restrict__ Q, const T* __restrict__ dO, const float* __restrict__ qc, const float* __restrict__ s_mu,
    const float* __restrict__ s_k, const T* __restrict__ s_v, const int32_t* __restrict__ perm_q,
    const int32_t* __restrict__ off_q, const float* __restrict__ LSE, const float* __restrict__ delta,
    const int32_t* __restrict__ slotinfo, float* __restrict__ G_c, T* __restrict__ G_k, T* __restrict__ G_v, int h0,
    int N, int nb, int Bs, int Cq, int Ck, int r, float scale) {
  constexpr int NV = D / 32;
  constexpr int POOL = 1024;                                   // entries per chunk
  constexpr int CHB = 32768 / (2 * D * (int)sizeof(T));        // queries whose rows fit 32 KB
  constexpr int CHMAX = CHB < 128 ? CHB : 128;                 // at most two entries of a chain per lane
  using F4 = Frag<T, 4>;
  __shared__ int2 pool[POOL];                                  // x = query of the chunk, y = its block << 16 | retrieved blocks
  __shared__ __attribute__((aligned(16))) T qS[CHMAX][D];
  __shared__ __attribute__((aligned(16))) T gS[CHMAX][D];
  __shared__ float2 ldS[CHMAX];                                // (LSE, delta)
  __shared__ int nS[CHMAX];
  __shared__ int bins[kMaxCk + 1];
  __shared__ int wsum[4];
  __shared__ int cum[18];                                      // cum[b] = queries of cluster i in blocks 1 .. b-1
  const int hl = blockIdx.y, hq = h0 + hl, i = blockIdx.x;
  const int tid = threadIdx.x, lane = tid % 64, wave = tid / 64, s8 = lane / 8, l8 = lane % 8;
  const int NBm = nb - 1;
  const int32_t* oq = off_q + (size_t)hq * ((size_t)nb * Cq + 1);
  const int CH = POOL / r < CHMAX ? POOL / r : CHMAX;          // queries per chunk
  if (tid == 0) {
    int run = 0;
    cum[0] = 0;
    cum[1] = 0;
    for (int b = 1; b < nb; ++b) {
      run += oq[b * Cq + i + 1] - oq[b * Cq + i];
      cum[b + 1] = run;
    }
  }
  __syncthreads();
  const int Tq = cum[nb];
  float qcv[NV][4];
#pragma unroll
  for (int x = 0; x < NV; ++x) {
    float4 c4 = *reinterpret_cast<const float4*>(qc + ((size_t)hq * Cq + i) * D + 32 * x + 4 * l8);
    qcv[x][0] = c4.x; qcv[x][1] = c4.y; qcv[x][2] = c4.z; qcv[x][3] = c4.w;
  }
  for (int c0 = 0; c0 < Tq; c0 += CH) {
    const int nq = Tq - c0 < CH ? Tq - c0 : CH;
    __syncthreads();  // the previous chunk is consumed
    for (int t = tid; t <= Ck; t += 256) bins[t] = 0;
    // this thread's query: position, block, slots
    int mybq = 0;
    int info[8];
#pragma unroll
    for (int t = 0; t < 8; ++t) info[t] = -1;
    const int32_t* si = slotinfo;
    if (tid < nq) {
      const int idx = c0 + tid;
      int b = 1;
      while (idx >= cum[b + 1]) ++b;
      const int pq = oq[b * Cq + i] + idx - cum[b];
      const int n = perm_q[(size_t)hq * N + pq];
      mybq = b;
      si = slotinfo + ((size_t)hq * N + pq) * r;
#pragma unroll
      for (int t = 0; t < 8; ++t)
        if (t < r) info[t] = si[t];
      nS[tid] = n;
      ldS[tid] = make_float2(LSE[(size_t)hq * N + n], delta[(size_t)hq * N + n]);
    }
    __syncthreads();
    if (tid < nq) {
      for (int t = 0; t < r; ++t) {
        const int x = t < 8 ? info[t] : si[t];
        if (x >= 0) atomicAdd(&bins[x & 0xffff], 1);
      }
    }
    {
      constexpr int CPR = D * (int)sizeof(T) / 16;
      for (int idx = tid; idx < nq * CPR; idx += 256) {
        const int e = idx / CPR, cc = idx % CPR;
        const size_t qn = (size_t)hq * N + nS[e];
        reinterpret_cast<uint4*>(&qS[e][0])[cc] = reinterpret_cast<const uint4*>(Q + qn * D)[cc];
        reinterpret_cast<uint4*>(&gS[e][0])[cc] = reinterpret_cast<const uint4*>(dO + qn * D)[cc];
      }
    }
    __syncthreads();
    // exclusive scan of the chain counts: bins[j] becomes the cursor of chain j
    {
      const int per = (Ck + 255) / 256, base = tid * per;
      int loc = 0;
      for (int k = 0; k < per; ++k) loc += base + k < Ck ? bins[base + k] : 0;
      int incl = loc;
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) {
        const int v = __shfl_up(incl, o, 64);
        if (lane >= o) incl += v;
      }
      if (lane == 63) wsum[wave] = incl;
      __syncthreads();
      int run = incl - loc;
      for (int w_ = 0; w_ < wave; ++w_) run += wsum[w_];
      for (int k = 0; k < per; ++k) {
        if (base + k < Ck) {
          const int c = bins[base + k];
          bins[base + k] = run;
          run += c;
        }
      }
    }
    __syncthreads();
    if (tid < nq) {
      for (int t = 0; t < r; ++t) {
        const int x = t < 8 ? info[t] : si[t];
        if (x >= 0) pool[atomicAdd(&bins[x & 0xffff], 1)] = make_int2(tid, (int)(((uint32_t)mybq << 16) | ((uint32_t)x >> 16)));
      }
    }
    __syncthreads();
    // chain j now is pool[bins[j-1] .. bins[j])
    for (int jb = 64 * wave; jb < Ck; jb += 256) {
      const int jmine = jb + lane;
      const int e1m = jmine < Ck ? bins[jmine] : 0;
      const int e0m = jmine < Ck ? (jmine > 0 ? bins[jmine - 1] : 0) : 0;
      unsigned long long todo = __ballot(e1m > e0m);
      while (todo) {
        const int src = __ffsll((long long)todo) - 1;
        todo &= todo - 1;
        const int j = jb + src;
        const int e0 = __builtin_amdgcn_readlane(e0m, src), e1 = __builtin_amdgcn_readlane(e1m, src);
        const int ne = e1 - e0;
        for (int a0 = 0; a0 < NBm; a0 += 8) {
          const int a = a0 + s8;
          const bool act = a < NBm;
          const size_t cell = (((size_t)hl * NBm + (act ? a : 0)) * Cq + i) * Ck + j;
          const float mu = s_mu[cell];  // an empty cell has mu = -inf and zero rows: p = 0, nothing is added
          float4 kv[NV];
          float vv[NV][4];
          typename F4::raw ogk[NV], ogv[NV];  // the row written by k_cell_grads
          const float ogc = G_c[cell];
#pragma unroll
          for (int x = 0; x < NV; ++x) {
            kv[x] = *reinterpret_cast<const float4*>(s_k + cell * D + 32 * x + 4 * l8);
            ld4(s_v, cell * D + 32 * x + 4 * l8, vv[x]);
            ogk[x] = F4::ld(G_k, cell * D + 32 * x + 4 * l8);
            ogv[x] = F4::ld(G_v, cell * D + 32 * x + 4 * l8);
          }
          if (a0 == 0 && ne > 1) {
            // order the chain's entries by query (each lane ranks up to two of them against all)
            int2 mine[2];
            int rank[2] = {0, 0};
#pragma unroll
            for (int u = 0; u < 2; ++u) mine[u] = e0 + lane + 64 * u < e1 ? pool[e0 + lane + 64 * u] : make_int2(0x7fffffff, 0);
            for (int e = e0; e < e1; ++e) {
              const int k = pool[e].x;
              rank[0] += k < mine[0].x;
              rank[1] += k < mine[1].x;
            }
            wave_lds_fence();
#pragma unroll
            for (int u = 0; u < 2; ++u)
              if (e0 + lane + 64 * u < e1) pool[e0 + rank[u]] = mine[u];
            wave_lds_fence();
          }
          float gk[NV][4], gv[NV][4], gc = 0.f;
#pragma unroll
          for (int x = 0; x < NV; ++x)
#pragma unroll
            for (int t = 0; t < 4; ++t) { gk[x][t] = 0.f; gv[x][t] = 0.f; }
          bool any = false;
          // two entries per step: their LDS reads and 8-lane reductions are independent and overlap
          for (int e = e0; e < e1; e += 2) {
            int2 en[2];
            bool use[2];
#pragma unroll
            for (int z = 0; z < 2; ++z) {
              en[z] = e + z < e1 ? pool[e + z] : make_int2(0, 0);  // block 0: precedes no key block
              use[z] = act && (en[z].y >> 16) > a && !((en[z].y >> a) & 1);
            }
            if (!use[0] && !use[1]) continue;
            any = true;
            float qv[2][NV][4], dv[2][NV][4];
            float2 ld2[2];
            float part[2] = {0.f, 0.f}, dpp[2] = {0.f, 0.f};
#pragma unroll
            for (int z = 0; z < 2; ++z) {
#pragma unroll
              for (int x = 0; x < NV; ++x) {
                ld4(&qS[en[z].x][0], 32 * x + 4 * l8, qv[z][x]);
                ld4(&gS[en[z].x][0], 32 * x + 4 * l8, dv[z][x]);
              }
              ld2[z] = ldS[en[z].x];
            }
#pragma unroll
            for (int z = 0; z < 2; ++z)
#pragma unroll
              for (int x = 0; x < NV; ++x) {
#pragma unroll
                for (int t = 0; t < 4; ++t) qv[z][x][t] = scale * (qv[z][x][t] - qcv[x][t]);
                part[z] = fmaf(qv[z][x][0], kv[x].x, part[z]); part[z] = fmaf(qv[z][x][1], kv[x].y, part[z]);
                part[z] = fmaf(qv[z][x][2], kv[x].z, part[z]); part[z] = fmaf(qv[z][x][3], kv[x].w, part[z]);
                dpp[z] = fmaf(dv[z][x][0], vv[x][0], dpp[z]); dpp[z] = fmaf(dv[z][x][1], vv[x][1], dpp[z]);
                dpp[z] = fmaf(dv[z][x][2], vv[x][2], dpp[z]); dpp[z] = fmaf(dv[z][x][3], vv[x][3], dpp[z]);
              }
#pragma unroll
            for (int z = 0; z < 2; ++z) {
              part[z] = group_sum<8>(part[z]);
              dpp[z] = group_sum<8>(dpp[z]);
            }
#pragma unroll
            for (int z = 0; z < 2; ++z) {  // entry e first, then e + 1: the order of the sums stays that of the list
              const float p = use[z] ? __expf(part[z] + mu - ld2[z].x) : 0.f;
              const float dlg = p * (dpp[z] - ld2[z].y);
#pragma unroll
              for (int x = 0; x < NV; ++x)
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                  gk[x][t] = fmaf(dlg, qv[z][x][t], gk[x][t]);
                  gv[x][t] = fmaf(p, dv[z][x][t], gv[x][t]);
                }
              gc += dlg * (1.f - part[z]) - p * dpp[z];
            }
          }
          if (any) {
            if (l8 == 0) G_c[cell] = ogc + gc;
#pragma unroll
            for (int x = 0; x < NV; ++x) {
              float ok4[4], ov4[4];
#pragma unroll
              for (int t = 0; t < 4; ++t) {
                ok4[t] = F4::get(ogk[x], t) + gk[x][t];
                ov4[t] = F4::get(ogv[x], t) + gv[x][t];
              }
              st4(G_k, cell * D + 32 * x + 4 * l8, ok4);
              st4(G_v, cell * D + 32 * x + 4 * l8, ov4);
            }
          }
        }
      }
    }
  }
}

// ------------------------------------------------------------------------------------------
// summary gradients -> keys and values: one wave per (kv head, key block b', key cluster j); loops
// over the query heads of the group and over tiles of 32 query clusters.
//   W[i,m] = exp(L[i,m] - mu[i]),  T[i,m] = G_c[i] + G_k[i].k_m + G_v[i].v_m
//   dv_m += sum_i W G_v[i],  dk_m += sum_i W G_k[i] + (W T) qbar_i
// ------------------------------------------------------------------------------------------
template <typename T, int D>
__global__ void __launch_bounds__(64) k_cells_to_keys(const T* __restrict__ Ks, const T* __restrict__ Vs,
                                                       const float* __restrict__ qc, const float* __restrict__ L,
                                                       const float* __restrict__ s_mu, const float* __restrict__ G_c,
                                                       const float* __restrict__ G_k, const float* __restrict__ G_v,
                                                       const int32_t* __restrict__ off_k, float* __restrict__ dKs,
                                                       float* __restrict__ dVs, int h0, int N, int nb, int Cq, int Ck,
                                                       int Hq, int Hkv, float scale, int frozen) {
  constexpr int U = D / 8, DT = D / 32;
  const int G_ = Hq / Hkv;
  const int hkl = blockIdx.z;                 // kv head inside the chunk
  const int hq0 = h0 + hkl * G_;              // first query head of the group (global flat index)
  const int hk = (hq0 / Hq) * Hkv + (hq0 % Hq) / G_;
  const int bp = blockIdx.y, j = blockIdx.x, NBm = nb - 1;
  const int lane = threadIdx.x, col = lane % 32, half = lane / 32;
  const int32_t* ok = off_k + (size_t)hk * ((size_t)nb * Ck + 1);
  const int klo = ok[bp * Ck + j], khi = ok[bp * Ck + j + 1];
  for (int m0 = klo; m0 < khi; m0 += 32) {
    const int pm = m0 + col;
    const bool mvalid = pm < khi;
    const int pmc = mvalid ? pm : m0;
    // B operands (row pattern): this lane's key
    float kb[U][4], vb[U][4];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      ld4(Ks, ((size_t)hk * N + pmc) * D + 8 * u + 4 * half, kb[u]);
      ld4(Vs, ((size_t)hk * N + pmc) * D + 8 * u + 4 * half, vb[u]);
    }
    f32x16_t dk[DT], dv[DT];
#pragma unroll
    for (int t = 0; t < DT; ++t) { dk[t] = zero16(); dv[t] = zero16(); }
    for (int g = 0; g < G_; ++g) {
      const int hl = hkl * G_ + g, hq = h0 + hl;
      for (int i0 = 0; i0 < Cq; i0 += 32) {
        const int ic = i0 + col < Cq ? i0 + col : Cq - 1;  // A-operand row of this lane
        const size_t cellA = (((size_t)hl * NBm + bp) * Cq + ic) * Ck + j;
        f32x16_t tacc, wv;
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          int ir = i0 + 8 * (e / 4) + 4 * half + (e % 4);
          bool iv = ir < Cq;
          int irc = iv ? ir : Cq - 1;
          const size_t cell = (((size_t)hl * NBm + bp) * Cq + irc) * Ck + j;
          tacc[e] = G_c[cell];
          float w = __expf(L[((size_t)hl * Cq + irc) * N + pmc] - s_mu[cell]);
          wv[e] = (iv && mvalid) ? w : 0.f;
        }
        tacc = mfma_rows<D>(tacc, G_k + cellA * D + 4 * half, kb);
        tacc = mfma_rows<D>(tacc, G_v + cellA * D + 4 * half, vb);
        // frozen aggregation weights: nothing flows through W (the T term drops out)
#pragma unroll
        for (int e = 0; e < 16; ++e) tacc[e] = (wv[e] > 0.f && !frozen) ? wv[e] * tacc[e] : 0.f;
#pragma unroll
        for (int gg = 0; gg < 4; ++gg)
#pragma unroll
          for (int t = 0; t < 4; ++t) {
            int ir = i0 + 8 * gg + 4 * half + t;
            ir = ir < Cq ? ir : Cq - 1;
            const size_t cell = (((size_t)hl * NBm + bp) * Cq + ir) * Ck + j;
#pragma unroll
            for (int x = 0; x < DT; ++x) {
              float gkv = G_k[cell * D + 32 * x + col];
              float gvv = G_v[cell * D + 32 * x + col];
              float qb = scale * qc[((size_t)hq * Cq + ir) * D + 32 * x + col];
              dv[x] = mfma32(gvv, wv[4 * gg + t], dv[x]);
              dk[x] = mfma32(gkv, wv[4 * gg + t], dk[x]);
              dk[x] = mfma32(qb, tacc[4 * gg + t], dk[x]);
            }
          }
      }
    }
    if (mvalid) {
      float* ok_ = dKs + ((size_t)hk * N + pm) * D;
      float* ov_ = dVs + ((size_t)hk * N + pm) * D;
#pragma unroll
      for (int x = 0; x < DT; ++x)
#pragma unroll
        for (int gg = 0; gg < 4; ++gg) {
          int d = 32 * x + 8 * gg + 4 * half;
          float4 a = *reinterpret_cast<float4*>(ok_ + d), c = *reinterpret_cast<float4*>(ov_ + d);
          a.x += dk[x][4 * gg]; a.y += dk[x][4 * gg + 1]; a.z += dk[x][4 * gg + 2]; a.w += dk[x][4 * gg + 3];
          c.x += dv[x][4 * gg]; c.y += dv[x][4 * gg + 1]; c.z += dv[x][4 * gg + 2]; c.w += dv[x][4 * gg + 3];
          *reinterpret_cast<float4*>(ok_ + d) = a;
          *reinterpret_cast<float4*>(ov_ + d) = c;
        }
    }
  }
}

// ------------------------------------------------------------------------------------------
// retrieval (component 3) -> keys and values: one wave per (kv head, key block b', tile of 32 key
// clusters) owns those keys.  Phase 1 scans the queries of later blocks (all heads of the group),
// collecting (query, cluster) hits into LDS; phase 2 accumulates per cluster in registers and adds
// the result to the bucketed gradient rows.  When the list fills, phase 2 runs and scanning resumes.
// ------------------------------------------------------------------------------------------
constexpr int kHitCap = 2048;

// stable counting sort of the hits by their 5-bit cluster id (single wave): sorted[], start[33]
__device__ __forceinline__ void c3_sort_hits(const uint32_t* hits, int nh, uint32_t* sorted, int* start, int* cursor) {
  const int lane = threadIdx.x;
  if (lane < 33) start[lane] = 0;
  __syncthreads();
  for (int i = lane; i < nh; i += 64) atomicAdd(&start[(hits[i] & 31u) + 1], 1);
  __syncthreads();
  if (lane == 0)
    for (int k = 0; k < 32; ++k) start[k + 1] += start[k];
  __syncthreads();
  if (lane < 32) cursor[lane] = start[lane];
  __syncthreads();
  for (int i0 = 0; i0 < nh; i0 += 64) {
    const int i = i0 + lane;
    const bool act = i < nh;
    const uint32_t h = act ? hits[i] : 0u;
    const int key = h & 31u;
    unsigned long long m = __ballot(act);
#pragma unroll
    for (int bit = 0; bit < 5; ++bit) {
      unsigned long long bb = __ballot((key >> bit) & 1);
      m &= ((key >> bit) & 1) ? bb : ~bb;
    }
    const int rank = __popcll(m & ((1ull << lane) - 1ull)), cnt = __popcll(m);
    if (act) {
      const int base = cursor[key];
      sorted[base + rank] = h;
      if (rank == cnt - 1) cursor[key] = base + cnt;
    }
  }
  __syncthreads();
}

template <typename T, int D>
__device__ __forceinline__ void c3_flush(const uint32_t* hits, const int* start, const T* __restrict__ Q,
                                         const T* __restrict__ dO, const T* __restrict__ Ks, const T* __restrict__ Vs,
                                         const float* __restrict__ LSE, const float* __restrict__ delta,
                                         const int32_t* __restrict__ ok, float* __restrict__ dKs,
                                         float* __restrict__ dVs, int hk, int hqbase, int N, int Ck, int bp, int jt,
                                         float scale) {
  constexpr int CH = D / 8, KSL = 64 / CH;  // lanes per key, keys per step
  const int lane = threadIdx.x, slot = lane / CH, chunk = lane % CH;
  for (int jl = 0; jl < 32; ++jl) {
    const int j = jt * 32 + jl;
    if (j >= Ck) break;
    const int klo = ok[bp * Ck + j], khi = ok[bp * Ck + j + 1];
    for (int kb = klo; kb < khi; kb += KSL) {
      const int pk = kb + slot;
      const bool kvalid = pk < khi;
      const size_t krow = ((size_t)hk * N + (kvalid ? pk : klo)) * D + 8 * chunk;
      float k8[8], v8[8], ak[8], av[8];
      ld4(Ks, krow, k8); ld4(Ks, krow + 4, k8 + 4);
      ld4(Vs, krow, v8); ld4(Vs, krow + 4, v8 + 4);
#pragma unroll
      for (int x = 0; x < 8; ++x) { ak[x] = 0.f; av[x] = 0.f; }
      for (int hI = start[jl]; hI < start[jl + 1]; ++hI) {
        const uint32_t hit = hits[hI];
        const int g = (hit >> 5) & 7, n = hit >> 8;
        const size_t qn = ((size_t)hqbase + g) * N + n;
        float q8[8], g8[8];
        ld4(Q, qn * D + 8 * chunk, q8); ld4(Q, qn * D + 8 * chunk + 4, q8 + 4);
        ld4(dO, qn * D + 8 * chunk, g8); ld4(dO, qn * D + 8 * chunk + 4, g8 + 4);
        float part = 0.f, dpp = 0.f;
#pragma unroll
        for (int x = 0; x < 8; ++x) {
          q8[x] *= scale;
          part = fmaf(q8[x], k8[x], part);
          dpp = fmaf(g8[x], v8[x], dpp);
        }
        part = group_sum<CH>(part);
        dpp = group_sum<CH>(dpp);
        const float p = kvalid ? __expf(part - LSE[qn]) : 0.f;
        const float dlg = p * (dpp - delta[qn]);
#pragma unroll
        for (int x = 0; x < 8; ++x) {
          ak[x] = fmaf(dlg, q8[x], ak[x]);
          av[x] = fmaf(p, g8[x], av[x]);
        }
      }
      if (kvalid) {
        float* ok_ = dKs + krow;
        float* ov_ = dVs + krow;
#pragma unroll
        for (int x = 0; x < 8; ++x) { ok_[x] += ak[x]; ov_[x] += av[x]; }
      }
    }
  }
}

template <typename T, int D>
__global__ void __launch_bounds__(64) k_c3_keys(const T* __restrict__ Q, const T* __restrict__ dO,
                                                 const T* __restrict__ Ks, const T* __restrict__ Vs,
                                                 const float* __restrict__ LSE, const float* __restrict__ delta,
                                                 const uint32_t* __restrict__ pmask, const int32_t* __restrict__ off_k,
                                                 float* __restrict__ dKs, float* __restrict__ dVs, int N, int Bs, int nb,
                                                 int Ck, int Hq, int Hkv, float scale) {
  __shared__ uint32_t hits[kHitCap];
  __shared__ uint32_t sorted[kHitCap];
  __shared__ int start[33], cursor[32];
  const int hk = blockIdx.z, bp = blockIdx.y, jt = blockIdx.x;
  const int G_ = Hq / Hkv;
  const int hqbase = (hk / Hkv) * Hq + (hk % Hkv) * G_;
  const int lane = threadIdx.x;
  const int W = (Ck + 31) / 32;
  const int32_t* ok = off_k + (size_t)hk * ((size_t)nb * Ck + 1);
  // nothing to do when the tile has no keys in this block
  {
    int jhi = min(jt * 32 + 32, Ck);
    if (ok[bp * Ck + jt * 32] == ok[bp * Ck + jhi]) return;
  }
  int nh = 0;
  for (int g = 0; g < G_; ++g) {
    const size_t hq = (size_t)hqbase + g;
    for (int n0 = (bp + 1) * Bs; n0 < N; n0 += 64) {
      const int n = n0 + lane;
      uint32_t keep = n < N ? pmask[((hq * (nb - 1) + bp) * W + jt) * N + n] : 0u;
      // append (n, g, jl) for every kept bit, in lane order
      int cnt = __popc(keep);
      unsigned long long any = __ballot(cnt > 0);
      if (!any) continue;
      int incl = cnt;
      for (int o = 1; o < 64; o <<= 1) {
        int v = __shfl_up(incl, o, 64);
        if (lane >= o) incl += v;
      }
      const int total = __shfl(incl, 63, 64);
      if (nh + total > kHitCap) {
        __syncthreads();
        c3_sort_hits(hits, nh, sorted, start, cursor);
        c3_flush<T, D>(sorted, start, Q, dO, Ks, Vs, LSE, delta, ok, dKs, dVs, hk, hqbase, N, Ck, bp, jt, scale);
        __syncthreads();
        nh = 0;
      }
      int at = nh + incl - cnt;
      while (keep) {
        const int jl = __ffs((int)keep) - 1;
        keep &= keep - 1;
        hits[at++] = ((uint32_t)n << 8) | ((uint32_t)g << 5) | (uint32_t)jl;
      }
      nh += total;
    }
  }
  __syncthreads();
  c3_sort_hits(hits, nh, sorted, start, cursor);
  c3_flush<T, D>(sorted, start, Q, dO, Ks, Vs, LSE, delta, ok, dKs, dVs, hk, hqbase, N, Ck, bp, jt, scale);
}

// rows back to sequence order, added to what the block-diagonal kernels left: dst[perm[p]] += src[p]
__global__ void __launch_bounds__(256) k_scatter_rows(const float* __restrict__ src, const int32_t* __restrict__ perm,
                                                       float* __restrict__ dst, int N, int D) {
  const int CPR = D / 4;
  size_t h = blockIdx.y;
  size_t c = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (c >= (size_t)N * CPR) return;
  int p = (int)(c / CPR), cc = (int)(c % CPR);
  int to = perm[h * N + p];
  float4* o = reinterpret_cast<float4*>(dst + (h * N + to) * D) + cc;
  const float4 a = reinterpret_cast<const float4*>(src + (h * N + p) * D)[cc];
  float4 v = *o;
  v.x += a.x; v.y += a.y; v.z += a.z; v.w += a.w;
  *o = v;
}

// dst[h][n] += src[h][n] for the rows n >= n0 of every head (the queries that have a far field)
__global__ void __launch_bounds__(256) k_add_rows(const float* __restrict__ src, float* __restrict__ dst, int N, int n0,
                                                   int D) {
  const size_t per = (size_t)(N - n0) * (D / 4);
  const size_t c = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (c >= per) return;
  const size_t o = ((size_t)blockIdx.y * N + n0) * (D / 4) + c;
  const float4 a = reinterpret_cast<const float4*>(src)[o];
  float4 v = reinterpret_cast<float4*>(dst)[o];
  v.x += a.x; v.y += a.y; v.z += a.z; v.w += a.w;
  reinterpret_cast<float4*>(dst)[o] = v;
}

template <typename T, int D>
int run_bwd_chunk(const MuseDims& d, const T* Q, const T* dO, const float* qc, const int32_t* aq, const float* LSE,
                  const int32_t* selc, const int32_t* selb, FFWorkspace& w, int h0, int hn, hipStream_t sq_, hipStream_t sk_) {
  // the far-field part of dQ goes to stream sq_, the cell gradients and what they give to keys and values to
  // stream sk_: the two share inputs only
  const int NBm = d.nb - 1;
  const int W = (d.Ck + 31) / 32;
  dim3 gt((d.Bs / 32 + d.Cq + 1 + 7) / 8 * 8, NBm, hn);
  hipStream_t st = sq_;
  { MuseProf prof_("k_ff_bwd_dq", st); hipLaunchKernelGGL((k_ff_bwd_dq<T, D>), gt, dim3(64), 0, st, Q, dO, qc, (const T*)w.Ks, (const T*)w.Vs, w.L, w.s_mu,
                     w.s_k, (const T*)w.s_v, w.A_mu, w.A_k, (const T*)w.A_v, (const bf16_t*)w.A_kb, w.perm_q, w.off_q, w.off_k, w.tile_off, LSE, w.delta,
                     w.selmask, selc, selb, w.ret_part, w.dQff, h0, d.N, d.nb, d.Cq, d.Ck, d.r, d.k2e, d.Hq, d.Hkv, d.scale); }
  if (sizeof(T) == 2 && d.r > 0) {
    dim3 g2(((d.N - d.Bs + 15) / 16 + 255) / 256 * 256, hn);  // a multiple of 256 (see the kernel)
    if (d.nb <= 9)
      { MuseProf prof_("k_comp2_bwd_dq", st); hipLaunchKernelGGL((k_comp2_bwd_dq<D, 1>), g2, dim3(256), 0, st, (const bf16_t*)Q, (const bf16_t*)dO, qc, w.s_mu, w.s_k, (const bf16_t*)w.s_v,
                         w.perm_q, aq, LSE, w.delta, w.slotinfo, w.ret_part, w.dQff, h0, d.N, d.nb, d.Bs, d.Cq, d.Ck, d.r, d.k2e, d.scale); }
    else
      { MuseProf prof_("k_comp2_bwd_dq", st); hipLaunchKernelGGL((k_comp2_bwd_dq<D, 2>), g2, dim3(256), 0, st, (const bf16_t*)Q, (const bf16_t*)dO, qc, w.s_mu, w.s_k, (const bf16_t*)w.s_v,
                         w.perm_q, aq, LSE, w.delta, w.slotinfo, w.ret_part, w.dQff, h0, d.N, d.nb, d.Bs, d.Cq, d.Ck, d.r, d.k2e, d.scale); }
  }
  st = sk_;
  if (sizeof(T) == 2) {
    int rc2 = muse_launch_ff_bwd_cells_mx(d, Q, dO, qc, w.A_mu, w.A_kb, w.A_v, w.perm_q, w.off_q, LSE, w.delta, w.selmask,
                                          w.g_A_c, w.g_A_k, w.g_A_v, h0, hn, st);
    if (rc2) return rc2;
  } else
  { MuseProf prof_("k_ff_bwd_cells", st); hipLaunchKernelGGL((k_ff_bwd_cells<T, D>), dim3(W, NBm * d.Cq, hn), dim3(64), 0, st, Q, dO, qc, w.A_mu, w.A_k, (const float*)w.A_v,
                     w.perm_q, w.off_q, LSE, w.delta, w.selmask, w.g_A_c, (float*)w.g_A_k, (float*)w.g_A_v, h0, d.N, d.nb, d.Cq, d.Ck,
                     d.scale); }
  { MuseProf prof_("k_cell_grads", st); hipLaunchKernelGGL((k_cell_grads<T, D>), dim3(W, d.Cq, hn), dim3(256), 0, st, w.s_mu, w.A_mu, w.g_A_c,
                     (const T*)w.g_A_k, (const T*)w.g_A_v, w.g_s_c, (T*)w.g_s_k, (T*)w.g_s_v, d.nb, d.Cq, d.Ck); }
  if (d.r > 0)
    { MuseProf prof_("k_chain_grads", st); hipLaunchKernelGGL((k_chain_grads<T, D>), dim3(d.Cq, hn), dim3(256), 0, st, Q, dO, qc, w.s_mu, w.s_k,
                       (const T*)w.s_v, w.perm_q, w.off_q, LSE, w.delta, w.slotinfo, w.g_s_c, (T*)w.g_s_k, (T*)w.g_s_v, h0, d.N,
                       d.nb, d.Bs, d.Cq, d.Ck, d.r, d.scale); }
  const int G_ = d.Hq / d.Hkv;
  if (sizeof(T) == 2) {
    int rc2 = muse_launch_cells_to_keys_mx(d, w.Ks, w.Vs, qc, w.qcT, w.L, w.s_mu, w.g_s_c, w.g_s_k, w.g_s_v, w.off_k, w.dKs, w.dVs,
                                           h0, hn, st);
    if (rc2) return rc2;
  } else
  { MuseProf prof_("k_cells_to_keys", st); hipLaunchKernelGGL((k_cells_to_keys<T, D>), dim3(d.Ck, NBm, hn / G_), dim3(64), 0, st, (const T*)w.Ks, (const T*)w.Vs,
                     qc, w.L, w.s_mu, w.g_s_c, (const float*)w.g_s_k, (const float*)w.g_s_v, w.off_k, w.dKs, w.dVs, h0, d.N, d.nb, d.Cq, d.Ck, d.Hq,
                     d.Hkv, d.scale, d.frozen_weights ? 1 : 0); }
  MUSE_LAUNCH_CHECK();
  return MUSE_OK;
}

template <typename T>
int run_bwd_typed(const MuseDims& d, const T* Q, const T* K, const T* V, const T* O, const float* LSE, const T* dO,
                  const float* qc, const int32_t* aq, const int32_t* ak, const int32_t* selc, const int32_t* selb,
                  void* dQ, void* dK, void* dV, FFWorkspace& w, hipStream_t st) {
  const int HQ = d.B * d.Hq, HK = d.B * d.Hkv, N = d.N, D = d.D;
  const size_t nq = (size_t)HQ * N, nk = (size_t)HK * N;
  int rc;
  const bool reuse = d.keep_state;  // bucketing, bucketed copies and summaries are still in the workspace
  if (!reuse && (rc = muse_ff_prepare<T>(d, K, V, aq, ak, w, st))) return rc;
  if ((rc = muse_launch_delta(d, O, dO, w.delta, st))) return rc;
  // the block-diagonal backward (matrix-core bound) runs beside the far field (memory bound) on a second
  // stream; it writes the accumulators and the far-field results are added after the join
  MuseAux& ax = muse_aux_stream();
  const bool two = ax.state == 1 && !muse_profiling();
  hipStream_t sb = two ? ax.s : st;
  // on every way out after the fork, the caller's stream waits for what the second stream was given
  struct AuxJoin {
    MuseAux& ax; hipStream_t st, sb; bool armed;
    ~AuxJoin() {
      if (armed && hipEventRecord(ax.join, sb) == hipSuccess) (void)hipStreamWaitEvent(st, ax.join, 0);
    }
  } guard{ax, st, sb, false};
  if (two) {
    MUSE_HIP_CHECK(hipEventRecord(ax.fork, st));
    MUSE_HIP_CHECK(hipStreamWaitEvent(sb, ax.fork, 0));
    guard.armed = true;
  }
  if ((rc = muse_launch_attn_bwd(d, d.Bs, Q, K, V, dO, LSE, w.delta, w.dQacc, w.dKacc, w.dVacc, sb))) return rc;
  // With all heads in one chunk the far-field part of dQ follows on the second stream (it needs the selection
  // info and the inverse index, which the first stream builds: event `mid`), beside the cell gradients.
  const bool split = two && w.hc >= HQ;
  if (two && !split) MUSE_HIP_CHECK(hipEventRecord(ax.join, sb));
  if ((rc = muse_launch_fill(w.dKs, nk * D, 0.f, st))) return rc;
  if ((rc = muse_launch_fill(w.dVs, nk * D, 0.f, st))) return rc;
  if (d.nb > 1) {
    const int W = (d.Ck + 31) / 32;
    if (d.r > 0) {
      { MuseProf prof_("k_selinfo", st); hipLaunchKernelGGL(k_selinfo, dim3((N + 255) / 256, HQ), dim3(256), 0, st, selc, selb, w.perm_q, w.selmask, w.slotinfo, N, d.r, d.k2e, W); }
    } else {
      if ((rc = muse_launch_fill_i32((int32_t*)w.selmask, nq * W, 0, st))) return rc;
    }
    MUSE_LAUNCH_CHECK();
    if (d.r > 0) {
      // retrieval (component 3): inverse index (kept from the forward when the state is reused), then per pair
      if (!reuse || sizeof(T) == 4)
        if ((rc = muse_ff_build_inverse_index(d, selc, selb, w, sizeof(T) == 2, st))) return rc;
      if (sizeof(T) == 2) {
        if ((rc = muse_launch_c3_pairs(d, Q, dO, w.Ks, w.Vs, LSE, w.delta, w.off_k, w.pair_off, w.c3_off, w.c3_map, w.run_cap, w.hits,
                                       w.hit_cap, w.dKs, w.dVs, w.c3_part, st)))
          return rc;
        if (split) {
          MUSE_HIP_CHECK(hipEventRecord(ax.mid, st));
          MUSE_HIP_CHECK(hipStreamWaitEvent(sb, ax.mid, 0));
        }
        if ((rc = muse_launch_ret_bwd_dq_pairs(d, Q, dO, w.Ks, w.Vs, LSE, w.delta, w.off_k, w.run_off, w.run_map, w.run_cap, w.hits,
                                               w.hit_cap, w.ret_part, split ? sb : st)))
          return rc;
      } else {
        dim3 g((d.Ck + 31) / 32, d.nb - 1, HK);
        if (D == 64)
          { MuseProf prof_("k_c3_keys", st); hipLaunchKernelGGL((k_c3_keys<T, 64>), g, dim3(64), 0, st, Q, dO, (const T*)w.Ks, (const T*)w.Vs, LSE, w.delta,
                             w.pairmask, w.off_k, w.dKs, w.dVs, N, d.Bs, d.nb, d.Ck, d.Hq, d.Hkv, d.scale); }
        else
          { MuseProf prof_("k_c3_keys", st); hipLaunchKernelGGL((k_c3_keys<T, 128>), g, dim3(64), 0, st, Q, dO, (const T*)w.Ks, (const T*)w.Vs, LSE, w.delta,
                             w.pairmask, w.off_k, w.dKs, w.dVs, N, d.Bs, d.nb, d.Ck, d.Hq, d.Hkv, d.scale); }
        MUSE_LAUNCH_CHECK();
      }
    }
    for (int h0 = 0; h0 < HQ; h0 += w.hc) {
      int hn = HQ - h0 < w.hc ? HQ - h0 : w.hc;
      if (!reuse && (rc = muse_ff_summaries<T>(d, qc, w, h0, hn, st))) return rc;
      if (!reuse && (rc = muse_ff_block_summaries<T>(d, selc, aq, w, h0, hn, st))) return rc;
      if (split) {  // everything the dQ side reads is now queued on the first stream
        MUSE_HIP_CHECK(hipEventRecord(ax.mid, st));
        MUSE_HIP_CHECK(hipStreamWaitEvent(sb, ax.mid, 0));
      }
      if (D == 64) rc = run_bwd_chunk<T, 64>(d, Q, dO, qc, aq, LSE, selc, selb, w, h0, hn, split ? sb : st, st);
      else rc = run_bwd_chunk<T, 128>(d, Q, dO, qc, aq, LSE, selc, selb, w, h0, hn, split ? sb : st, st);
      if (rc) return rc;
    }
  }
  if (split) MUSE_HIP_CHECK(hipEventRecord(ax.join, sb));
  if (two) MUSE_HIP_CHECK(hipStreamWaitEvent(st, ax.join, 0));
  guard.armed = false;
  {
    dim3 g((unsigned)(((size_t)N * (D / 4) + 255) / 256), HK);
    { MuseProf prof_("k_scatter_rows", st); hipLaunchKernelGGL(k_scatter_rows, g, dim3(256), 0, st, w.dKs, w.perm_k, w.dKacc, N, D); }
    { MuseProf prof_("k_scatter_rows", st); hipLaunchKernelGGL(k_scatter_rows, g, dim3(256), 0, st, w.dVs, w.perm_k, w.dVacc, N, D); }
    MUSE_LAUNCH_CHECK();
  }
  if (d.nb > 1) {
    dim3 g((unsigned)(((size_t)(N - d.Bs) * (D / 4) + 255) / 256), HQ);
    { MuseProf prof_("k_add_rows", st); hipLaunchKernelGGL(k_add_rows, g, dim3(256), 0, st, w.dQff, w.dQacc, N, d.Bs, D); }
    MUSE_LAUNCH_CHECK();
  }
  if (d.grad_dtype != MUSE_DTYPE_FP32) {
    if ((rc = muse_launch_cast(w.dQacc, dQ, nq * D, d.grad_dtype, 1.f, st))) return rc;
    if ((rc = muse_launch_cast(w.dKacc, dK, nk * D, d.grad_dtype, 1.f, st))) return rc;
    if ((rc = muse_launch_cast(w.dVacc, dV, nk * D, d.grad_dtype, 1.f, st))) return rc;
  }
  return MUSE_OK;
}

}  // namespace

int muse_run_bwd(const MuseDims& d, const void* Q, const void* K, const void* V, const void* O, const float* LSE,
                 const void* dO, const float* qc, const int32_t* aq, const int32_t* ak, const int32_t* selc,
                 const int32_t* selb, void* dQ, void* dK, void* dV, void* ws, size_t ws_bytes, hipStream_t st) {
  FFWorkspace w;
  if (!muse_ff_carve(d, true, ws, ws_bytes, &w, dQ, dK, dV)) return MUSE_ERR_WORKSPACE_TOO_SMALL;
  if (d.keep_state && w.hc < d.B * d.Hq) return MUSE_ERR_WORKSPACE_TOO_SMALL;
  if (d.dtype == MUSE_DTYPE_FP32)
    return run_bwd_typed<float>(d, (const float*)Q, (const float*)K, (const float*)V, (const float*)O, LSE,
                                (const float*)dO, qc, aq, ak, selc, selb, dQ, dK, dV, w, st);
  return run_bwd_typed<bf16_t>(d, (const bf16_t*)Q, (const bf16_t*)K, (const bf16_t*)V, (const bf16_t*)O, LSE,
                               (const bf16_t*)dO, qc, aq, ak, selc, selb, dQ, dK, dV, w, st);
}
