// Exact retrieval (Sec. 3.3): the inverse index "retrieved (key cluster, key block) pair -> queries" and
// the merge of the per-pair forward partial states into the far-field state of every query.
//
//   pairmask[hq][b'][j/32][n]  bit j%32 set iff query n of head hq retrieved the pair (j, b')
//   hits[hk][pair_off[hk][b'*Ck + j] ...]  the queries of all heads of the KV group that retrieved the
//                                           pair, ascending (head, position): x = n | g << 22, y = slot*k2e + u
// Ordered lists (ballot ranks, no atomics on the order) keep every later sum reproducible.  The bit matrix is
// built for fp32 inputs only (their key/value gradient kernel walks it); bf16 inputs build the lists directly.
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

// The hit lists are built by a counting sort whose order is fixed by construction.  The queries with a far field
// (positions Bs .. N-1) of every query head are cut into SEG slices of whole 64-query chunks; one workgroup owns a
// (slice, head), walks its chunks in order and keeps one counter per pair in LDS.  Each of its kHitWaves waves
// takes the pairs of one residue class (pair % kHitWaves), so a counter has one owner and the waves never wait
// for each other.  For a chunk and a selection slot, the lanes that name the same pair are found by ballots (one
// round per distinct pair of the wave's class among the 64 lanes) and ranked by lane, so a list is ascending in
// (head of the group, position) without any atomic deciding an order.  Pass 1 (FILL = false) leaves the counts per (kv head, head of the group x slice, pair); k_pair_totals,
// k_pair_scan and k_seg_offsets turn them into list starts (pair-major, then head of the group, then slice);
// pass 2 (FILL = true) starts from those and writes the hits, with the slot index the pair has in the query's
// exported selections.
constexpr int kHitWaves = 8;
template <bool FILL>
__global__ void __launch_bounds__(64 * kHitWaves) k_hit_lists(const int32_t* __restrict__ selc, const int32_t* __restrict__ selb,
                                                   int32_t* __restrict__ seg_cnt, const int32_t* __restrict__ seg_off,
                                                   uint2* __restrict__ hits, size_t hit_cap, int N, int Bs, int Ck,
                                                   int r, int k2e, int Hq, int Hkv, int npair, int SEG, int cps) {
  extern __shared__ int cur[];  // per pair: hits counted so far (pass 1) / next list position (pass 2)
  const int s = blockIdx.x, hq = blockIdx.y, lane = threadIdx.x % 64, wave = threadIdx.x / 64;
  const int G_ = Hq / Hkv, g = (hq % Hq) % G_;
  const int hk = (hq / Hq) * Hkv + (hq % Hq) / G_;
  const size_t sbase = ((size_t)hk * G_ * SEG + (size_t)g * SEG + s) * npair;
  for (int p = threadIdx.x; p < npair; p += 64 * kHitWaves) cur[p] = FILL ? seg_off[sbase + p] : 0;
  __syncthreads();
  const int chunks = (N - Bs + 63) / 64;
  const int c1 = (s + 1) * cps < chunks ? (s + 1) * cps : chunks;
  const unsigned long long below = (1ull << lane) - 1ull;
  for (int c = s * cps; c < c1; ++c) {
    const int n = Bs + 64 * c + lane;
    const bool valid = n < N;
    const size_t qn = (size_t)hq * N + (valid ? n : N - 1);
    for (int t = 0; t < r; ++t) {
      const int j = valid ? selc[qn * r + t] : -1;
      for (int u = 0; u < k2e; ++u) {
        const int bp = j >= 0 ? selb[(qn * r + t) * k2e + u] : -1;
        // (selections are trusted inputs; one outside the table is dropped rather than indexed)
        const int pair = (bp >= 0 && j < Ck && bp * Ck + j < npair) ? bp * Ck + j : -1;
        unsigned long long act = __ballot(pair >= 0 && pair % kHitWaves == wave);
        while (act) {
          const int src = __ffsll((long long)act) - 1;
          const int pv = __builtin_amdgcn_readlane(pair, src);
          const unsigned long long same = __ballot(pair == pv);
          const int base = cur[pv];
          if (FILL && pair == pv)
            hits[(size_t)hk * hit_cap + base + __popcll(same & below)] =
                make_uint2((uint32_t)n | ((uint32_t)g << 22), (uint32_t)(t * k2e + u));
          if (lane == src) cur[pv] = base + __popcll(same);
          act &= ~same;
        }
      }
    }
  }
  if (!FILL) {
    __syncthreads();
    for (int p = threadIdx.x; p < npair; p += 64 * kHitWaves) seg_cnt[sbase + p] = cur[p];
  }
}

// pair_cnt[hk][p] = hits of pair p over all (head of the group, slice) segments
__global__ void __launch_bounds__(256) k_pair_totals(const int32_t* __restrict__ seg_cnt, int32_t* __restrict__ pair_cnt,
                                                      int npair, int SEGT) {
  const int hk = blockIdx.y, p = blockIdx.x * 256 + threadIdx.x;
  if (p >= npair) return;
  const int32_t* c = seg_cnt + (size_t)hk * SEGT * npair + p;
  int tot = 0;
  for (int gs = 0; gs < SEGT; ++gs) tot += c[(size_t)gs * npair];
  pair_cnt[(size_t)hk * (npair + 1) + p] = tot;
}

// seg_off[hk][gs][p] = pair_off[hk][p] + hits of pair p in the segments before gs
__global__ void __launch_bounds__(256) k_seg_offsets(const int32_t* __restrict__ seg_cnt, const int32_t* __restrict__ pair_off,
                                                      int32_t* __restrict__ seg_off, int npair, int SEGT) {
  const int hk = blockIdx.y, p = blockIdx.x * 256 + threadIdx.x;
  if (p >= npair) return;
  const size_t base = (size_t)hk * SEGT * npair + p;
  int run = pair_off[(size_t)hk * (npair + 1) + p];
  for (int gs = 0; gs < SEGT; ++gs) {
    seg_off[base + (size_t)gs * npair] = run;
    run += seg_cnt[base + (size_t)gs * npair];
  }
}

// Work items of the per-pair retrieval kernels: a pair's hit tiles (32 hits each) are cut into runs of kRunTiles, so
// a heavy pair becomes many equal items and a light one a single item (no empty slices, no tails).
//   run_cnt[hk][p] = runs of pair p;  run_map[hk][run_off[hk][p] + u] = (p, first hit of run u, end of the run)
__global__ void __launch_bounds__(256) k_run_counts(const int32_t* __restrict__ pair_off, int32_t* __restrict__ run_cnt, int npair) {
  const int hk = blockIdx.y, p = blockIdx.x * 256 + threadIdx.x;
  if (p >= npair) return;
  const int32_t* po = pair_off + (size_t)hk * (npair + 1);
  const int tiles = (po[p + 1] - po[p] + 31) / 32;
  run_cnt[(size_t)hk * (npair + 1) + p] = (tiles + kRunTiles - 1) / kRunTiles;
}
__global__ void __launch_bounds__(256) k_run_fill(const int32_t* __restrict__ pair_off, const int32_t* __restrict__ run_off,
                                                   int4* __restrict__ run_map, int npair, size_t run_cap) {
  const int hk = blockIdx.y, p = blockIdx.x * 256 + threadIdx.x;
  if (p >= npair) return;
  const int32_t* po = pair_off + (size_t)hk * (npair + 1);
  const int32_t* ro = run_off + (size_t)hk * (npair + 1);
  const int lo = po[p], hi = po[p + 1];
  int4* out = run_map + (size_t)hk * run_cap + ro[p];
  for (int u = 0, h = lo; h < hi; ++u, h += 32 * kRunTiles)
    out[u] = make_int4(p, h, h + 32 * kRunTiles < hi ? h + 32 * kRunTiles : hi, 0);
}

// The same for the key/value gradient kernel: its items are (pair, hit slice), c3_slices of them per pair that has hits.
__global__ void __launch_bounds__(256) k_c3_counts(const int32_t* __restrict__ pair_off, int32_t* __restrict__ cnt, int npair) {
  const int hk = blockIdx.y, p = blockIdx.x * 256 + threadIdx.x;
  if (p >= npair) return;
  const int32_t* po = pair_off + (size_t)hk * (npair + 1);
  const int h = po[p + 1] - po[p];
  cnt[(size_t)hk * (npair + 1) + p] = h > 0 ? c3_slices(h) : 0;
}
__global__ void __launch_bounds__(256) k_c3_fill(const int32_t* __restrict__ pair_off, const int32_t* __restrict__ c3_off,
                                                  int2* __restrict__ c3_map, int npair, size_t run_cap) {
  const int hk = blockIdx.y, p = blockIdx.x * 256 + threadIdx.x;
  if (p >= npair) return;
  const int32_t* po = pair_off + (size_t)hk * (npair + 1);
  const int h = po[p + 1] - po[p];
  const int S = h > 0 ? c3_slices(h) : 0;
  int2* out = c3_map + (size_t)hk * run_cap + c3_off[(size_t)hk * (npair + 1) + p];
  for (int u = 0; u < S; ++u) out[u] = make_int2(p, u);
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
  auto fold = [&](float pm, float pl, const float4 pa) {
    const float mn = fmaxf(m, pm);
    const float ca = __expf(m - mn), cb = __expf(pm - mn);
    l = l * ca + pl * cb;
    a.x = a.x * ca + pa.x * cb; a.y = a.y * ca + pa.y * cb;
    a.z = a.z * ca + pa.z * cb; a.w = a.w * ca + pa.w * cb;
    m = mn;
  };
  if (R2 <= 8) {
    // the usual shape: all the query's partial states are requested together and folded in slot order
    float2 ml[8];
    float4 pa[8];
#pragma unroll
    for (int su = 0; su < 8; ++su) {
      const bool ok = su < R2 && selb[q * R2 + (su < R2 ? su : 0)] >= 0;
      const float* pr = part + (q * R2 + (su < R2 ? su : 0)) * (size_t)(D + 4);
      ml[su] = ok ? *reinterpret_cast<const float2*>(pr + D) : make_float2(0.f, 0.f);
      pa[su] = ok ? *reinterpret_cast<const float4*>(pr + 4 * c) : make_float4(0.f, 0.f, 0.f, 0.f);
    }
#pragma unroll
    for (int su = 0; su < 8; ++su)
      if (ml[su].y > 0.f) fold(ml[su].x, ml[su].y, pa[su]);
  } else {
    for (int su = 0; su < R2; ++su) {
      if (selb[q * R2 + su] < 0) continue;
      const float* pr = part + (q * R2 + su) * (size_t)(D + 4);
      const float pm = pr[D], pl = pr[D + 1];
      if (!(pl > 0.f)) continue;
      fold(pm, pl, *reinterpret_cast<const float4*>(pr + 4 * c));
    }
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
  if (!with_hits) {
    if ((rc = muse_launch_fill_i32((int32_t*)w.pairmask, nq * NBm * W, 0, st))) return rc;
    { MuseProf prof_("k_pairmask", st); hipLaunchKernelGGL(k_pairmask, dim3((unsigned)((nq * d.r + 255) / 256)), dim3(256), 0, st, selc, selb, w.pairmask, HQ, N, d.r, d.k2e, NBm, W); }
    MUSE_LAUNCH_CHECK();
    return MUSE_OK;
  }
  const int SEG = ff_hit_segments(d), SEGT = (d.Hq / d.Hkv) * SEG, npair = NBm * d.Ck;
  const int chunks = (N - d.Bs + 63) / 64, cps = (chunks + SEG - 1) / SEG;
  const size_t lds = (size_t)npair * sizeof(int);
  static_assert((size_t)15 * MUSE_MAX_CLUSTERS * sizeof(int) <= 128 * 1024, "the pair counters of the largest accepted shape fit the LDS");
  static bool attr_set = false;
  if (!attr_set) {
    MUSE_HIP_CHECK(hipFuncSetAttribute((const void*)k_hit_lists<false>, hipFuncAttributeMaxDynamicSharedMemorySize, 128 * 1024));
    MUSE_HIP_CHECK(hipFuncSetAttribute((const void*)k_hit_lists<true>, hipFuncAttributeMaxDynamicSharedMemorySize, 128 * 1024));
    attr_set = true;
  }
  const dim3 g(SEG, HQ), gp((npair + 255) / 256, HK);
  { MuseProf prof_("k_hit_lists", st); hipLaunchKernelGGL(k_hit_lists<false>, g, dim3(64 * kHitWaves), lds, st, selc, selb, w.seg_cnt, w.seg_off, w.hits, w.hit_cap, N, d.Bs, d.Ck, d.r, d.k2e, d.Hq, d.Hkv, npair, SEG, cps); }
  { MuseProf prof_("k_pair_totals", st); hipLaunchKernelGGL(k_pair_totals, gp, dim3(256), 0, st, w.seg_cnt, w.pair_cnt, npair, SEGT); }
  { MuseProf prof_("k_pair_scan", st); hipLaunchKernelGGL(k_pair_scan, dim3(HK), dim3(1024), 0, st, w.pair_cnt, w.pair_off, npair); }
  { MuseProf prof_("k_seg_offsets", st); hipLaunchKernelGGL(k_seg_offsets, gp, dim3(256), 0, st, w.seg_cnt, w.pair_off, w.seg_off, npair, SEGT); }
  { MuseProf prof_("k_hit_lists", st); hipLaunchKernelGGL(k_hit_lists<true>, g, dim3(64 * kHitWaves), lds, st, selc, selb, w.seg_cnt, w.seg_off, w.hits, w.hit_cap, N, d.Bs, d.Ck, d.r, d.k2e, d.Hq, d.Hkv, npair, SEG, cps); }
  // the pair kernels' work items (pair_cnt is free again: it holds the runs per pair now)
  { MuseProf prof_("k_run_counts", st); hipLaunchKernelGGL(k_run_counts, gp, dim3(256), 0, st, w.pair_off, w.pair_cnt, npair); }
  { MuseProf prof_("k_pair_scan", st); hipLaunchKernelGGL(k_pair_scan, dim3(HK), dim3(1024), 0, st, w.pair_cnt, w.run_off, npair); }
  { MuseProf prof_("k_run_fill", st); hipLaunchKernelGGL(k_run_fill, gp, dim3(256), 0, st, w.pair_off, w.run_off, w.run_map, npair, w.run_cap); }
  { MuseProf prof_("k_c3_counts", st); hipLaunchKernelGGL(k_c3_counts, gp, dim3(256), 0, st, w.pair_off, w.pair_cnt, npair); }
  { MuseProf prof_("k_pair_scan", st); hipLaunchKernelGGL(k_pair_scan, dim3(HK), dim3(1024), 0, st, w.pair_cnt, w.c3_off, npair); }
  { MuseProf prof_("k_c3_fill", st); hipLaunchKernelGGL(k_c3_fill, gp, dim3(256), 0, st, w.pair_off, w.c3_off, w.c3_map, npair, w.run_cap); }
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
