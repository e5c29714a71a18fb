// Far-field stages (Sec. 3.1-3.3): workspace layout and fp32-MFMA helpers shared by the forward and
// backward translation units.
//
// fp32 MFMA (v_mfma_f32_32x32x2_f32) conventions used throughout:
//   - accumulator element e = 4g+t of lane l is row 8g + 4(l/32) + t, column l%32;
//   - an operand lane supplies one value per instruction: its k-slot is l/32.
//   "Row pattern": operand X[row = l%32][c], contraction over the contiguous index c.  A lane loads
//   float4 groups X[row][8u + 4(l/32) .. +3]; instruction (u,t) uses element t, i.e. half h
//   contributes c = 8u + 4h + t.  Two row-pattern operands pair up consistently.
//   "Column pattern": A[m][k] = X[k][m] read as X[k0 + 8g + 4(l/32) + t][m0 + l%32] (coalesced over
//   lanes), pairing with a B operand taken straight from an accumulator (its rows are 8g+4h+t).
#pragma once
#include "common.h"

__device__ __forceinline__ f32x16_t mfma32(float a, float b, f32x16_t c) {
  return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ f32x16_t zero16() {
  f32x16_t z;
#pragma unroll
  for (int e = 0; e < 16; ++e) z[e] = 0.f;
  return z;
}

// acc += X[row][.] (row pattern, `row` already offset by 4*(l/32)) times the row-pattern operand b
template <int D>
__device__ __forceinline__ f32x16_t mfma_rows(f32x16_t acc, const float* __restrict__ row, const float (&b)[D / 8][4]) {
#pragma unroll
  for (int u = 0; u < D / 8; ++u) {
    float4 a = *reinterpret_cast<const float4*>(row + 8 * u);
    acc = mfma32(a.x, b[u][0], acc);
    acc = mfma32(a.y, b[u][1], acc);
    acc = mfma32(a.z, b[u][2], acc);
    acc = mfma32(a.w, b[u][3], acc);
  }
  return acc;
}

// One tile of 32 accumulated key summaries as the score MFMAs consume it: the lane's row-pattern groups
// of k-bar and its 16 mu-bar values.  Loading is separate from use so that every load of a tile is in
// flight before the first MFMA waits on one.
template <int D>
struct KTile {
  float4 a[D / 8];
  float mu[16];
};

template <int D>
__device__ __forceinline__ void load_ktile(KTile<D>& kt, const float* __restrict__ Amu, const float* __restrict__ Ak,
                                           int j0, int Ck, int col, int half) {
  int c = j0 + col;
  c = c < Ck ? c : Ck - 1;
  const float* row = Ak + (size_t)c * D + 4 * half;
#pragma unroll
  for (int u = 0; u < D / 8; ++u) kt.a[u] = *reinterpret_cast<const float4*>(row + 8 * u);
  if ((Ck & 3) == 0) {  // rows 8g + 4 half + t, t = 0..3, are one aligned float4
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      int base = j0 + 8 * g + 4 * half;
      base = base < Ck ? base : Ck - 4;
      const float4 m4 = *reinterpret_cast<const float4*>(Amu + base);
      kt.mu[4 * g] = m4.x; kt.mu[4 * g + 1] = m4.y; kt.mu[4 * g + 2] = m4.z; kt.mu[4 * g + 3] = m4.w;
    }
  } else {
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      int jr = j0 + 8 * (e / 4) + 4 * half + (e % 4);
      kt.mu[e] = Amu[jr < Ck ? jr : Ck - 1];
    }
  }
}

// scores^T of 32 key clusters (rows) x 32 queries (columns) against accumulated summaries, Eq. 7:
// accumulator preloaded with mu-bar, then += k-bar . q~
template <int D>
__device__ __forceinline__ f32x16_t score_ktile(const KTile<D>& kt, int j0, int Ck, const float (&qt)[D / 8][4], int half) {
  f32x16_t acc;
#pragma unroll
  for (int e = 0; e < 16; ++e) {
    const int jr = j0 + 8 * (e / 4) + 4 * half + (e % 4);
    acc[e] = jr < Ck ? kt.mu[e] : MUSE_NEG_INF;
  }
#pragma unroll
  for (int u = 0; u < D / 8; ++u) {
    acc = mfma32(kt.a[u].x, qt[u][0], acc);
    acc = mfma32(kt.a[u].y, qt[u][1], acc);
    acc = mfma32(kt.a[u].z, qt[u][2], acc);
    acc = mfma32(kt.a[u].w, qt[u][3], acc);
  }
  return acc;
}

template <int D>
__device__ __forceinline__ f32x16_t score_tile(const float* __restrict__ Amu, const float* __restrict__ Ak, int j0,
                                               int Ck, const float (&qt)[D / 8][4], int col, int half) {
  KTile<D> kt;
  load_ktile<D>(kt, Amu, Ak, j0, Ck, col, half);
  return score_ktile<D>(kt, j0, Ck, qt, half);
}

// The same tile for bf16 inputs, where the scores run on the 16-bit matrix cores without losing the precision
// that decides selections: k-bar is stored as a bf16 plane plus an fp16 plane of the remainder (together 19
// significant bits or more), the query operand is the bf16 query itself (exact, also as fp16), and the query
// centroid's share of q~ . k-bar is a per-cell scalar c = scale * qc_i . k-bar, the weighted mean of the tilt
// logits that the kernel which wrote the planes has at hand:  score = scale * q . (hi + mid) + (mu-bar - c).
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8_t;
template <int D>
struct KTileH {
  uint4 h[D / 16], m[D / 16];
  float mu[16];
};

template <int D>
__device__ __forceinline__ void load_ktile_h(KTileH<D>& kt, const float* __restrict__ Amuq,
                                             const bf16_t* __restrict__ Akb, const uint16_t* __restrict__ Akm, int j0,
                                             int Ck, int col, int half) {
  int c = j0 + col;
  c = c < Ck ? c : Ck - 1;
  const bf16_t* rh = Akb + (size_t)c * D + 8 * half;
  const uint16_t* rm = Akm + (size_t)c * D + 8 * half;
#pragma unroll
  for (int ks = 0; ks < D / 16; ++ks) {
    kt.h[ks] = *reinterpret_cast<const uint4*>(rh + 16 * ks);
    kt.m[ks] = *reinterpret_cast<const uint4*>(rm + 16 * ks);
  }
  if ((Ck & 3) == 0) {
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      int base = j0 + 8 * g + 4 * half;
      base = base < Ck ? base : Ck - 4;
      const float4 m4 = *reinterpret_cast<const float4*>(Amuq + base);
      kt.mu[4 * g] = m4.x; kt.mu[4 * g + 1] = m4.y; kt.mu[4 * g + 2] = m4.z; kt.mu[4 * g + 3] = m4.w;
    }
  } else {
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      int jr = j0 + 8 * (e / 4) + 4 * half + (e % 4);
      kt.mu[e] = Amuq[jr < Ck ? jr : Ck - 1];
    }
  }
}

// qb / qh: the lane's query (column) dims 16 ks + 8 half .. + 7 as bf16 and as fp16
template <int D>
__device__ __forceinline__ f32x16_t score_ktile_h(const KTileH<D>& kt, int j0, int Ck, const bf16x8_t (&qb)[D / 16],
                                                  const f16x8_t (&qh)[D / 16], float scale, int half) {
  f32x16_t acc;
#pragma unroll
  for (int e = 0; e < 16; ++e) acc[e] = 0.f;
#pragma unroll
  for (int ks = 0; ks < D / 16; ++ks) {
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, kt.h[ks]), qb[ks], acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8_t, kt.m[ks]), qh[ks], acc, 0, 0, 0);
  }
#pragma unroll
  for (int e = 0; e < 16; ++e) {
    const int jr = j0 + 8 * (e / 4) + 4 * half + (e % 4);
    acc[e] = jr < Ck ? fmaf(scale, acc[e], kt.mu[e]) : MUSE_NEG_INF;
  }
  return acc;
}

// The bf16 plane alone: an approximate score, off by at most scale * 2^-8 * |q| . |k-bar| (the plane is k-bar rounded
// to nearest), for the passes that only need to know which clusters can be among the r best.
template <int D>
struct KTileB {
  uint4 h[D / 16];
  float mu[16];
};
template <int D>
__device__ __forceinline__ void load_ktile_b(KTileB<D>& kt, const float* __restrict__ Amuq,
                                             const bf16_t* __restrict__ Akb, int j0, int Ck, int col, int half) {
  int c = j0 + col;
  c = c < Ck ? c : Ck - 1;
  const bf16_t* rh = Akb + (size_t)c * D + 8 * half;
#pragma unroll
  for (int ks = 0; ks < D / 16; ++ks) kt.h[ks] = *reinterpret_cast<const uint4*>(rh + 16 * ks);
  if ((Ck & 3) == 0) {
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      int base = j0 + 8 * g + 4 * half;
      base = base < Ck ? base : Ck - 4;
      const float4 m4 = *reinterpret_cast<const float4*>(Amuq + base);
      kt.mu[4 * g] = m4.x; kt.mu[4 * g + 1] = m4.y; kt.mu[4 * g + 2] = m4.z; kt.mu[4 * g + 3] = m4.w;
    }
  } else {
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      int jr = j0 + 8 * (e / 4) + 4 * half + (e % 4);
      kt.mu[e] = Amuq[jr < Ck ? jr : Ck - 1];
    }
  }
}
template <int D>
__device__ __forceinline__ f32x16_t score_ktile_b(const KTileB<D>& kt, int j0, int Ck, const bf16x8_t (&qb)[D / 16],
                                                  float scale, int half) {
  f32x16_t acc;
#pragma unroll
  for (int e = 0; e < 16; ++e) acc[e] = 0.f;
#pragma unroll
  for (int ks = 0; ks < D / 16; ++ks)
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, kt.h[ks]), qb[ks], acc, 0, 0, 0);
#pragma unroll
  for (int e = 0; e < 16; ++e) {
    const int jr = j0 + 8 * (e / 4) + 4 * half + (e % 4);
    acc[e] = jr < Ck ? fmaf(scale, acc[e], kt.mu[e]) : MUSE_NEG_INF;
  }
  return acc;
}

// bf16 MFMA (v_mfma_f32_32x32x16_bf16) helpers.  pack8: accumulator rows 4*g0..+3 and 4*g1..+3 of a lane
// become the 8 k-slots of a B (or A) operand; the matching other operand must use the same row order.
__device__ __forceinline__ bf16x8_t pack8(const f32x16_t& s, int g0, int g1) {
  bf16x8_t r;
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    r[t] = (__bf16)s[4 * g0 + t];
    r[4 + t] = (__bf16)s[4 * g1 + t];
  }
  return r;
}

// A operand for the second contraction from a transposed LDS tile `row` ([..][BN+8]): the 8 k-slots
// of lane half `half` over the 16 rows starting at r0
__device__ __forceinline__ bf16x8_t ld_tr8(const bf16_t* row, int r0, int half) {
  uint2 a = *reinterpret_cast<const uint2*>(row + r0 + 4 * half);
  uint2 b = *reinterpret_cast<const uint2*>(row + r0 + 8 + 4 * half);
  uint4 v = make_uint4(a.x, a.y, b.x, b.y);
  return *reinterpret_cast<bf16x8_t*>(&v);
}

__device__ __forceinline__ __bf16 bits_to_bf16(bf16_t b) { return __builtin_bit_cast(__bf16, b); }

__device__ __forceinline__ bf16x8_t cvt8(const float* __restrict__ p) {
  float4 a = *reinterpret_cast<const float4*>(p), b = *reinterpret_cast<const float4*>(p + 4);
  bf16x8_t r;
  r[0] = (__bf16)a.x; r[1] = (__bf16)a.y; r[2] = (__bf16)a.z; r[3] = (__bf16)a.w;
  r[4] = (__bf16)b.x; r[5] = (__bf16)b.y; r[6] = (__bf16)b.z; r[7] = (__bf16)b.w;
  return r;
}


constexpr int kMaxCk = 2304;  // key clusters a kernel can index in LDS
static_assert(kMaxCk >= MUSE_MAX_CLUSTERS, "the host accepts more clusters than the kernels index");
constexpr int kRunTiles = 4;  // hit tiles (of 32) per work item of the retrieval forward / dq pair kernels
constexpr int kC3Slices = 8;  // most waves that share the hits of one retrieved pair in the key/value gradients
constexpr int kC3TilesPerSlice = 4;  // a pair gets one slice per so many tiles of 32 hits
// hit slices of a pair in the key/value gradient kernel of the retrieval (depends on its hit count only)
__host__ __device__ inline int c3_slices(int nhits) {
  const int nt = (nhits + 31) / 32;
  const int s = nt / kC3TilesPerSlice;
  return s < 1 ? 1 : (s > kC3Slices ? kC3Slices : s);
}

struct FFWorkspace {
  // all heads
  int32_t *perm_k, *off_k, *perm_q, *off_q, *tile_off;
  void *Ks, *Vs;      // keys / values in bucketed order, input dtype
  float *ff_acc, *ff_ml;  // contiguous: [HQ,N,D] then [HQ,N,2]
  // backward only, all heads
  float* delta;
  uint32_t* selmask;   // [HQ][W][N] by bucketed query position
  int32_t* slotinfo;   // [HQ][N][r] by bucketed query position: cluster | retrieved-block mask << 16
  uint32_t* pairmask;  // [HQ][nb-1][W][N], fp32 inputs only
  int32_t* pair_off;             // inverse index of the retrieval: (kv head, key block, key cluster) -> hits
  int32_t* pair_cnt;             // hits per pair (later: runs per pair), [HK][pairs + 1]
  int32_t* run_off;              // [HK][pairs + 1]: first work item of every pair, [pairs] = their number
  int4* run_map;                 // [HK][run_cap]: (pair, first hit, end) of a work item
  int32_t* c3_off;               // [HK][pairs + 1]: first (pair, hit slice) item of every pair, [pairs] = their number
  int2* c3_map;                  // [HK][run_cap]: (pair, slice) items of the key/value gradient kernel
  size_t run_cap;                // work items per kv head the map can hold
  int32_t *seg_cnt, *seg_off;    // its construction: counts / list starts [HK][head of the group x query slice][pair]
  uint2* hits;                   // x = n | g << 22 (query position, head inside the KV group), y = slot*k2e + u
  size_t hit_cap;                // hits per kv head
  float* ret_part;               // per (query, slot, u): forward partial state [acc D | max | sum | pad2], or dq partial [D]
  float* knorm;                  // [HK]: largest Euclidean norm of a key row of the kv head (bf16 inputs); then [HK][64] partial maxima
  int32_t* ff_flag;              // [HQ][nb-1][ff_tile_grid_x]: tiles the one-plane forward kernel leaves to the two-plane one
  float *dKs, *dVs;            // fp32 gradients in bucketed key order
  float* c3_part;              // bf16 inputs, r > 0: [kC3Slices - 1][HK][N][2][D] partial dK | dV rows of the later hit slices of a pair
  float *dQacc, *dKacc, *dVacc;  // fp32 gradients in sequence order (alias the outputs when they are fp32)
  float* dQff;                   // far-field part of dQ, added to dQacc once the block-diagonal backward has finished
  void* qcT;                     // bf16 [hc][D][Cq padded to 32]: scaled query centroids of a head chunk, transposed
  // per chunk of `hc` query heads
  float* L;
  uint32_t* chainmask;  // [hc][Cq][ceil(Ck/32)]: key clusters retrieved by some query of the query cluster
  uint32_t* chainmaskT;  // [hc][Ck][ceil(Cq/32)]: the same bits, key-cluster-major
  // Value summaries and every cell gradient are stored in the input type.  The accumulated k-bar decides
  // selections: fp32 inputs keep it in fp32 (A_k); bf16 inputs keep a bf16 plane A_kb (also the operand of the
  // gradient contractions), an fp16 plane A_km of the remainder and the scalar A_c = mu-bar - scale * qc_i . k-bar
  // per cell.
  float *s_mu, *s_k, *A_mu, *A_k, *A_c;
  void *s_v, *A_v, *A_kb, *A_km;
  float *g_s_c, *g_A_c;
  void *g_s_k, *g_s_v, *g_A_k, *g_A_v;
  // dipole correction (MUSE_FLAG_DIPOLE): untilted covariances [HK][nb-1][Ck][D][D] (all heads) and the merged
  // matrices [hc][nb-1][Cq][D][D] of a head chunk
  float *dip_cov, *dip_cbar;
  int hc;
};

static inline size_t ff_al(size_t x) { return (x + 255) & ~(size_t)255; }

// query-range slices per head when the hit lists of the retrieval are built: enough (slice, head) waves to fill
// the device, every slice a whole number of 64-query chunks
static inline int ff_hit_segments(const MuseDims& d) {
  const int HQ = d.B * d.Hq, chunks = (d.N - d.Bs + 63) / 64;
  int seg = (2048 + HQ - 1) / HQ;
  seg = seg > chunks ? chunks : seg;
  return seg < 1 ? 1 : seg;
}
// bytes of the bit matrix (fp32 inputs) and of the segment counters (bf16 inputs) of the inverse index
static inline size_t ff_pairmask_bytes(const MuseDims& d) {
  size_t HQ = (size_t)d.B * d.Hq, W = (d.Ck + 31) / 32, NBm = d.nb > 1 ? d.nb - 1 : 1;
  return d.dtype == MUSE_DTYPE_BF16 ? 0 : HQ * d.N * W * 4 * NBm;
}
// most work items (runs of kRunTiles hit tiles inside one pair) a kv head can have
static inline size_t ff_run_cap(const MuseDims& d) {
  size_t NBm = d.nb > 1 ? d.nb - 1 : 1, R2 = (size_t)(d.r > 0 ? d.r : 1) * d.k2e;
  size_t npair = NBm * d.Ck, hits = (size_t)(d.Hq / d.Hkv) * d.N * R2;
  return (hits / 32 + npair) / kRunTiles + npair + 1;
}
static inline size_t ff_segcnt_bytes(const MuseDims& d) {
  size_t HK = (size_t)d.B * d.Hkv, NBm = d.nb > 1 ? d.nb - 1 : 1;
  return d.dtype == MUSE_DTYPE_BF16 ? HK * (d.Hq / d.Hkv) * ff_hit_segments(d) * NBm * d.Ck * 4 : 0;
}

// bytes of the all-heads part / of one query head of the chunked part
// x extent of the forward tile kernels' grid: the tiles of a (head, block) pair, rounded up to the 8 XCDs
static inline size_t ff_tile_grid_x(const MuseDims& d) { return (size_t)(d.Bs / 32 + d.Cq + 1 + 7) / 8 * 8; }
static inline size_t ff_flag_bytes(const MuseDims& d) {
  return (size_t)d.B * d.Hq * (d.nb > 1 ? d.nb - 1 : 1) * ff_tile_grid_x(d) * 4;
}
static inline size_t ff_fixed_bytes(const MuseDims& d, bool bwd) {
  size_t HQ = (size_t)d.B * d.Hq, HK = (size_t)d.B * d.Hkv, N = d.N, D = d.D;
  size_t es = d.dtype == MUSE_DTYPE_BF16 ? 2 : 4;
  size_t W = (d.Ck + 31) / 32, NBm = d.nb > 1 ? d.nb - 1 : 1, R2 = (size_t)(d.r > 0 ? d.r : 1) * d.k2e;
  size_t b = ff_al(HK * N * 4) + ff_al(HK * ((size_t)d.nb * d.Ck + 1) * 4) + ff_al(HQ * N * 4) +
             ff_al(HQ * ((size_t)d.nb * d.Cq + 1) * 4) + ff_al(HQ * d.nb * ((size_t)d.Cq + 1) * 4) +
             2 * ff_al(HK * N * D * es) + ff_al(HQ * N * (D + 2) * 4);
  // inverse index of the retrieval and its per-(query, slot) partial results
  b += ff_al(ff_pairmask_bytes(d)) + 4 * ff_al(HK * ((size_t)d.nb * d.Ck + 1) * 4) + 2 * ff_al(ff_segcnt_bytes(d)) +
       ff_al(HK * ff_run_cap(d) * 16) + ff_al(HK * ff_run_cap(d) * 8) +
       ff_al(HQ * N * R2 * 8) +
       ff_al(HQ * N * R2 * (D + 4) * 4);
  b += ff_al(HK * 65 * 4) + ff_al(ff_flag_bytes(d));
  if (bwd) {
    b += ff_al(HQ * N * 4) + ff_al(HQ * N * W * 4) + ff_al(HQ * N * (size_t)(d.r > 0 ? d.r : 1) * 4) + 2 * ff_al(HK * N * D * 4) +
         ff_al(HQ * N * D * 4) + ff_al(HQ * D * (size_t)((d.Cq + 31) / 32 * 32) * 2);
    if (d.grad_dtype != MUSE_DTYPE_FP32) b += ff_al(HQ * N * D * 4) + 2 * ff_al(HK * N * D * 4);
    if (es == 2 && d.r > 0 && d.nb > 1) b += ff_al((size_t)(kC3Slices - 1) * HK * N * 2 * D * 4);
  }
  if (d.dipole) b += ff_al(HK * NBm * d.Ck * D * D * 4);
  return b;
}

static inline size_t ff_head_bytes(const MuseDims& d, bool bwd) {
  size_t cells = (size_t)(d.nb > 1 ? d.nb - 1 : 1) * d.Cq * d.Ck, D = d.D;
  size_t es = d.dtype == MUSE_DTYPE_BF16 ? 2 : 4;
  size_t b = ff_al((size_t)d.Cq * d.N * 4) + ff_al((size_t)d.Cq * ((d.Ck + 31) / 32) * 4) + ff_al((size_t)d.Ck * ((d.Cq + 31) / 32) * 4) + 2 * ff_al(cells * 4) + ff_al(cells * D * 4) + 2 * ff_al(cells * D * es);
  b += es == 2 ? 2 * ff_al(cells * D * 2) + ff_al(cells * 4) : ff_al(cells * D * 4);
  if (bwd) b += 2 * ff_al(cells * 4) + 4 * ff_al(cells * D * es);
  if (d.dipole) b += ff_al((size_t)(d.nb > 1 ? d.nb - 1 : 1) * d.Cq * D * D * 4);
  return b;
}

// farfield.hip
int muse_ff_carve(const MuseDims& d, bool bwd, void* ws, size_t ws_bytes, FFWorkspace* w, void* dQ, void* dK, void* dV);
template <typename T>
int muse_ff_prepare(const MuseDims& d, const T* K, const T* V, const int32_t* aq, const int32_t* ak, FFWorkspace& w,
                    hipStream_t st);
template <typename T>
int muse_ff_summaries(const MuseDims& d, const float* qc, FFWorkspace& w, int h0, int hn, hipStream_t st);
template <typename T>
int muse_ff_block_summaries(const MuseDims& d, const int32_t* selc, const int32_t* aq, FFWorkspace& w, int h0, int hn,
                            hipStream_t st);

// attn_mfma.hip
int muse_launch_c3_pairs(const MuseDims& d, const void* Q, const void* dO, const void* Ks, const void* Vs,
                         const float* LSE, const float* delta, const int32_t* off_k, const int32_t* pair_off,
                         const int32_t* c3_off, const int2* c3_map, size_t run_cap, const uint2* hits, size_t hit_cap,
                         float* dKs, float* dVs, float* part, hipStream_t st);
int muse_launch_ret_fwd_pairs(const MuseDims& d, const void* Q, const void* Ks, const void* Vs, const int32_t* off_k,
                              const int32_t* run_off, const int4* run_map, size_t run_cap, const uint2* hits,
                              size_t hit_cap, float* part, hipStream_t st);
int muse_launch_ret_bwd_dq_pairs(const MuseDims& d, const void* Q, const void* dO, const void* Ks, const void* Vs,
                                 const float* LSE, const float* delta, const int32_t* off_k, const int32_t* run_off,
                                 const int4* run_map, size_t run_cap, const uint2* hits, size_t hit_cap, float* dqpart,
                                 hipStream_t st);
int muse_launch_ff_bwd_cells_mx(const MuseDims& d, const void* Q, const void* dO, const float* qc, const float* A_mu,
                                const void* A_kb, const void* A_v, const int32_t* perm_q, const int32_t* off_q,
                                const float* LSE, const float* delta, const uint32_t* selmask, float* g_A_c,
                                void* g_A_k, void* g_A_v, int h0, int hn, hipStream_t st);
int muse_launch_cells_to_keys_mx(const MuseDims& d, const void* Ks, const void* Vs, const float* qc, void* qcT,
                                 const float* L, const float* s_mu, const float* G_c, const void* G_k, const void* G_v,
                                 const int32_t* off_k, float* dKs, float* dVs, int h0, int hn, hipStream_t st);
// dipole.hip: dipole correction of the monopole-only mode (App. B), forward
template <typename T>
int muse_dipole_covariances(const MuseDims& d, FFWorkspace& w, hipStream_t st);
template <typename T>
int muse_dipole_apply(const MuseDims& d, const T* Q, const float* qc, const int32_t* aq, FFWorkspace& w, int h0, int hn,
                      hipStream_t st);
// retrieval.hip: pair bitmask + ordered hit lists from the exported selections; merge of the forward partials
int muse_ff_build_inverse_index(const MuseDims& d, const int32_t* selc, const int32_t* selb, FFWorkspace& w,
                                bool with_hits, hipStream_t st);
int muse_launch_merge_ret(const MuseDims& d, const int32_t* selb, const float* part, float* ff_acc, float* ff_ml,
                          hipStream_t st);
