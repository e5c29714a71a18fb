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

// Pass 1 (FILL = false) counts the hits of every (pair, head of the group, slice of the query range),
// k_pair_scan turns the counts into offsets (pair-major, then head, then slice: the order of the lists),
// pass 2 (FILL = true) writes the lists.  One wave per (key block b', tile of 32 clusters, head, slice);
// lane jl keeps the running offset of cluster 32 jt + jl in a register.
template <bool FILL>
__global__ void __launch_bounds__(64) k_pair_hits(const uint32_t* __restrict__ pmask, int32_t* __restrict__ seg_cnt,
                                                   const int32_t* __restrict__ seg_off, uint2* __restrict__ hits,
                                                   size_t hit_cap, int N, int Bs, int nb, int Ck, int Hq, int Hkv) {
  const int jt = blockIdx.x, bp = blockIdx.y, NBm = nb - 1;
  const int G_ = Hq / Hkv, W = (Ck + 31) / 32, SEGT = G_ * kHitSeg;
  const int hk = blockIdx.z / SEGT, gs = blockIdx.z % SEGT, g = gs / kHitSeg, sg = gs % kHitSeg;
  const size_t hq = (size_t)(hk / Hkv) * Hq + (size_t)(hk % Hkv) * G_ + g;
  const int lane = threadIdx.x;
  const int nlo = (bp + 1) * Bs;
  const int per = ((N - nlo + kHitSeg * 64 - 1) / (kHitSeg * 64)) * 64;  // queries per slice, a multiple of 64
  const int nbeg = nlo + sg * per, nend = nbeg + per < N ? nbeg + per : N;
  const size_t sbase = (size_t)hk * ((size_t)NBm * Ck * SEGT + 1);
  const int jmine = jt * 32 + (lane & 31);
  const size_t sidx = sbase + ((size_t)bp * Ck + jmine) * SEGT + gs;
  int curv = (FILL && lane < 32 && jmine < Ck) ? seg_off[sidx] : 0;
  const uint32_t* colw = pmask + ((hq * NBm + bp) * W + jt) * N;
  for (int n0 = nbeg; n0 < nend; n0 += 256) {
    uint32_t words[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int n = n0 + 64 * u + lane;
      words[u] = n < nend ? colw[n] : 0u;
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const uint32_t word = words[u];
      unsigned long long nz = __ballot(word != 0u);
      uint32_t U = 0;  // clusters present in this chunk
      while (nz) {
        const int src = __ffsll((long long)nz) - 1;
        nz &= nz - 1;
        U |= (uint32_t)__builtin_amdgcn_readlane((int)word, src);
      }
      while (U) {
        const int jl = __ffs((int)U) - 1;
        U &= U - 1;
        const bool has = (word >> jl) & 1u;
        const unsigned long long bal = __ballot(has);
        const int base = __shfl(curv, jl, 64);
        if (FILL && has) {
          const int rank = __popcll(bal & ((1ull << lane) - 1ull));
          // y holds the pair for now; k_hit_slots replaces it with the query's slot index
          hits[(size_t)hk * hit_cap + base + rank] =
              make_uint2((uint32_t)(n0 + 64 * u + lane) | ((uint32_t)g << 22), (uint32_t)(bp * Ck + jt * 32 + jl));
        }
        if (lane == jl) curv += __popcll(bal);
      }
    }
  }
  if (!FILL && lane < 32 && jmine < Ck) seg_cnt[sidx] = curv;
}

// pair_off[hk][p] = seg_off[hk][p * SEGT]: where the list of pair p starts (p = npair: the total)
__global__ void __launch_bounds__(256) k_pair_offsets(const int32_t* __restrict__ seg_off, int32_t* __restrict__ pair_off,
                                                       int npair, int SEGT) {
  const int hk = blockIdx.y, p = blockIdx.x * 256 + threadIdx.x;
  if (p > npair) return;
  pair_off[(size_t)hk * (npair + 1) + p] = seg_off[(size_t)hk * ((size_t)npair * SEGT + 1) + (size_t)p * SEGT];
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
  const int SEGT = (d.Hq / d.Hkv) * kHitSeg, npair = NBm * d.Ck;
  dim3 g(W, NBm, HK * SEGT);
  { MuseProf prof_("k_pair_hits", st); hipLaunchKernelGGL(k_pair_hits<false>, g, dim3(64), 0, st, w.pairmask, w.seg_cnt, w.seg_off, w.hits, w.hit_cap, N, d.Bs, d.nb, d.Ck, d.Hq, d.Hkv); }
  { MuseProf prof_("k_pair_scan", st); hipLaunchKernelGGL(k_pair_scan, dim3(HK), dim3(1024), 0, st, w.seg_cnt, w.seg_off, npair * SEGT); }
  { MuseProf prof_("k_pair_offsets", st); hipLaunchKernelGGL(k_pair_offsets, dim3((npair + 256) / 256, HK), dim3(256), 0, st, w.seg_off, w.pair_off, npair, SEGT); }
  { MuseProf prof_("k_pair_hits", st); hipLaunchKernelGGL(k_pair_hits<true>, g, dim3(64), 0, st, w.pairmask, w.seg_cnt, w.seg_off, w.hits, w.hit_cap, N, d.Bs, d.nb, d.Ck, d.Hq, d.Hkv); }
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
