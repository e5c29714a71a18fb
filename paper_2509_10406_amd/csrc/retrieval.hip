// Exact retrieval (Sec. 3.3): the inverse index "retrieved (key cluster, key block) pair -> queries" and
// the merge of the per-pair forward partial states into the far-field state of every query.
//
//   pairmask[hq][b'][j/32][n]  bit j%32 set iff query n of head hq retrieved the pair (j, b')
//   hits[hk][pair_off[hk][b'*Ck + j] ...]  the queries of all heads of the KV group that retrieved the
//                                           pair, ascending (head, position): x = n | g << 22, y = slot*k2e + u
// Ordered lists (ballot ranks, no atomics on the order) keep every later sum reproducible.
#include "ff_common.h"

namespace {

__global__ void __launch_bounds__(256) k_pairmask(const int32_t* __restrict__ selc, const int32_t* __restrict__ selb,
                                                   uint32_t* __restrict__ pmask, int HQ, int N, int r, int k2e, int NBm,
                                                   int W) {
  size_t t = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (t >= (size_t)HQ * N * r) return;
  const int slot = (int)(t % r);
  const size_t q = t / r;
  const size_t hq = q / N, n = q % N;
  const int j = selc[q * r + slot];
  if (j < 0) return;
  for (int u = 0; u < k2e; ++u) {
    const int bp = selb[(q * r + slot) * k2e + u];
    if (bp >= 0) atomicOr(&pmask[((hq * NBm + bp) * W + (j >> 5)) * N + n], 1u << (j & 31));
  }
}

// Pass 1 (FILL = false) counts the hits of every pair, k_pair_scan turns counts into offsets, pass 2
// (FILL = true) writes the lists in order.  One wave per (key block b', tile of 32 clusters).
template <bool FILL>
__global__ void __launch_bounds__(64) k_pair_hits(const uint32_t* __restrict__ pmask, const int32_t* __restrict__ selc,
                                                   const int32_t* __restrict__ selb, int32_t* __restrict__ pair_cnt,
                                                   const int32_t* __restrict__ pair_off, uint2* __restrict__ hits,
                                                   size_t hit_cap, int N, int Bs, int nb, int Ck, int r, int k2e, int Hq,
                                                   int Hkv) {
  __shared__ int cur[32];
  const int jt = blockIdx.x, bp = blockIdx.y, hk = blockIdx.z, NBm = nb - 1;
  const int G_ = Hq / Hkv, W = (Ck + 31) / 32;
  const size_t hqbase = (size_t)(hk / Hkv) * Hq + (size_t)(hk % Hkv) * G_;
  const int lane = threadIdx.x;
  const size_t pbase = (size_t)hk * ((size_t)NBm * Ck + 1) + (size_t)bp * Ck + jt * 32;
  if (lane < 32) cur[lane] = (FILL && jt * 32 + lane < Ck) ? pair_off[pbase + lane] : 0;
  __syncthreads();
  for (int g = 0; g < G_; ++g) {
    const size_t hq = hqbase + g;
    const uint32_t* colw = pmask + ((hq * NBm + bp) * W + jt) * N;
    for (int n0 = (bp + 1) * Bs; n0 < N; n0 += 64) {
      const int n = n0 + lane;
      const uint32_t word = n < N ? colw[n] : 0u;
      if (!__ballot(word != 0u)) continue;
      for (int jl = 0; jl < 32; ++jl) {
        const bool has = (word >> jl) & 1u;
        const unsigned long long bal = __ballot(has);
        if (!bal) continue;
        const int base = cur[jl];
        if (FILL && has) {
          const int rank = __popcll(bal & ((1ull << lane) - 1ull));
          // y holds the pair for now; k_hit_slots replaces it with the query's slot index
          hits[(size_t)hk * hit_cap + base + rank] =
              make_uint2((uint32_t)n | ((uint32_t)g << 22), (uint32_t)(bp * Ck + jt * 32 + jl));
        }
        __syncthreads();
        if (lane == 0) cur[jl] = base + __popcll(bal);
        __syncthreads();
      }
    }
  }
  if (!FILL && lane < 32 && jt * 32 + lane < Ck) pair_cnt[pbase + lane] = cur[lane];
}

// hits[].y: pair id -> slot*k2e + u of that pair in the query's exported selections (one thread per hit)
__global__ void __launch_bounds__(256) k_hit_slots(const int32_t* __restrict__ selc, const int32_t* __restrict__ selb,
                                                    const int32_t* __restrict__ pair_off, uint2* __restrict__ hits,
                                                    size_t hit_cap, int npair, int N, int Ck, int r, int k2e, int Hq,
                                                    int Hkv) {
  const int hk = blockIdx.y;
  const int total = pair_off[(size_t)hk * (npair + 1) + npair];
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= total) return;
  const int G_ = Hq / Hkv;
  const size_t hqbase = (size_t)(hk / Hkv) * Hq + (size_t)(hk % Hkv) * G_;
  uint2 h = hits[(size_t)hk * hit_cap + i];
  const size_t qn = (hqbase + (h.x >> 22)) * N + (h.x & 0x3fffffu);
  const int bp = (int)h.y / Ck, j = (int)h.y % Ck;
  int su = 0;
  for (int t = 0; t < r; ++t)
    if (selc[qn * r + t] == j)
      for (int u = 0; u < k2e; ++u)
        if (selb[(qn * r + t) * k2e + u] == bp) su = t * k2e + u;
  hits[(size_t)hk * hit_cap + i].y = (uint32_t)su;
}

// exclusive prefix of n counts per kv head, off[n] = total
__global__ void __launch_bounds__(1024) k_pair_scan(const int32_t* __restrict__ cnt, int32_t* __restrict__ off, int n) {
  __shared__ int wsum[16];
  const int hk = blockIdx.x, lane = threadIdx.x % 64, wave = threadIdx.x / 64;
  const int32_t* c = cnt + (size_t)hk * (n + 1);
  int32_t* o = off + (size_t)hk * (n + 1);
  const int per = (n + 1023) / 1024;
  int mine = 0;
  for (int u = 0; u < per; ++u) {
    int i = threadIdx.x * per + u;
    if (i < n) mine += c[i];
  }
  int incl = mine;
  for (int d = 1; d < 64; d <<= 1) {
    int v = __shfl_up(incl, d, 64);
    if (lane >= d) incl += v;
  }
  if (lane == 63) wsum[wave] = incl;
  __syncthreads();
  int base = 0;
  for (int w = 0; w < wave; ++w) base += wsum[w];
  int run = base + incl - mine;
  for (int u = 0; u < per; ++u) {
    int i = threadIdx.x * per + u;
    if (i < n) { o[i] = run; run += c[i]; }
  }
  if (threadIdx.x == 1023) o[n] = run;
}

// far-field state of every query  <-  state (+) partial states of its retrieved pairs.
// D/4 lanes per query, each owning 4 dims; part rows are [acc D | max | sum | pad2].
__global__ void __launch_bounds__(256) k_merge_ret(const int32_t* __restrict__ selb, const float* __restrict__ part,
                                                    float* __restrict__ ff_acc, float* __restrict__ ff_ml, size_t nq,
                                                    int N, int Bs, int D, int R2) {
  const int LPQ = D / 4;
  size_t t = (size_t)blockIdx.x * 256 + threadIdx.x;
  size_t q = t / LPQ;
  const int c = (int)(t % LPQ);
  if (q >= nq) return;
  if ((int)(q % N) < Bs) return;  // first block: no far field
  float m = ff_ml[q * 2], l = ff_ml[q * 2 + 1];
  float4 a = *reinterpret_cast<float4*>(ff_acc + q * D + 4 * c);
  if (!(l > 0.f)) { m = MUSE_NEG_INF; l = 0.f; a = make_float4(0.f, 0.f, 0.f, 0.f); }
  for (int su = 0; su < R2; ++su) {
    if (selb[q * R2 + su] < 0) continue;
    const float* pr = part + (q * R2 + su) * (size_t)(D + 4);
    const float pm = pr[D], pl = pr[D + 1];
    if (!(pl > 0.f)) continue;
    const float4 pa = *reinterpret_cast<const float4*>(pr + 4 * c);
    const float mn = fmaxf(m, pm);
    const float ca = __expf(m - mn), cb = __expf(pm - mn);
    l = l * ca + pl * cb;
    a.x = a.x * ca + pa.x * cb; a.y = a.y * ca + pa.y * cb;
    a.z = a.z * ca + pa.z * cb; a.w = a.w * ca + pa.w * cb;
    m = mn;
  }
  *reinterpret_cast<float4*>(ff_acc + q * D + 4 * c) = a;
  if (c == 0) { ff_ml[q * 2] = m; ff_ml[q * 2 + 1] = l; }
}

}  // namespace

int muse_ff_build_inverse_index(const MuseDims& d, const int32_t* selc, const int32_t* selb, FFWorkspace& w,
                                bool with_hits, hipStream_t st) {
  const int HQ = d.B * d.Hq, HK = d.B * d.Hkv, N = d.N, NBm = d.nb - 1, W = (d.Ck + 31) / 32;
  const size_t nq = (size_t)HQ * N;
  int rc;
  if ((rc = muse_launch_fill_i32((int32_t*)w.pairmask, nq * NBm * W, 0, st))) return rc;
  { MuseProf prof_("k_pairmask", st); hipLaunchKernelGGL(k_pairmask, dim3((unsigned)((nq * d.r + 255) / 256)), dim3(256), 0, st, selc, selb, w.pairmask, HQ, N, d.r, d.k2e, NBm, W); }
  MUSE_LAUNCH_CHECK();
  if (!with_hits) return MUSE_OK;
  dim3 g(W, NBm, HK);
  { MuseProf prof_("k_pair_hits", st); hipLaunchKernelGGL(k_pair_hits<false>, g, dim3(64), 0, st, w.pairmask, selc, selb, w.pair_cnt, w.pair_off, w.hits, w.hit_cap, N, d.Bs, d.nb, d.Ck, d.r, d.k2e, d.Hq, d.Hkv); }
  { MuseProf prof_("k_pair_scan", st); hipLaunchKernelGGL(k_pair_scan, dim3(HK), dim3(1024), 0, st, w.pair_cnt, w.pair_off, NBm * d.Ck); }
  { MuseProf prof_("k_pair_hits", st); hipLaunchKernelGGL(k_pair_hits<true>, g, dim3(64), 0, st, w.pairmask, selc, selb, w.pair_cnt, w.pair_off, w.hits, w.hit_cap, N, d.Bs, d.nb, d.Ck, d.r, d.k2e, d.Hq, d.Hkv); }
  {
    dim3 gh((unsigned)((w.hit_cap + 255) / 256), HK);
    { MuseProf prof_("k_hit_slots", st); hipLaunchKernelGGL(k_hit_slots, gh, dim3(256), 0, st, selc, selb, w.pair_off, w.hits, w.hit_cap, NBm * d.Ck, N, d.Ck, d.r, d.k2e, d.Hq, d.Hkv); }
  }
  MUSE_LAUNCH_CHECK();
  return MUSE_OK;
}

int muse_launch_merge_ret(const MuseDims& d, const int32_t* selb, const float* part, float* ff_acc, float* ff_ml,
                          hipStream_t st) {
  const size_t nq = (size_t)d.B * d.Hq * d.N;
  const size_t threads = nq * (d.D / 4);
  { MuseProf prof_("k_merge_ret", st); hipLaunchKernelGGL(k_merge_ret, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, st, selb, part, ff_acc, ff_ml, nq, d.N, d.Bs, d.D, d.r * d.k2e); }
  MUSE_LAUNCH_CHECK();
  return MUSE_OK;
}
