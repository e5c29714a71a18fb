// Far-field forward (Sec. 3.1-3.3, Alg. 1): tilt logits q-bar.k, per-block tilted summaries
// (Eq. 4-6) fused with the exclusive causal accumulation, and per query tile: cluster scores
// (Eq. 7) with top-r selection, monopole attention over the non-retrieved clusters, spatial block
// selection, approximate attention over non-retrieved blocks, exact attention over the retrieved
// (cluster, block) pairs.  The result is a partial softmax state (max, sum, acc) per query that the
// block-diagonal attention kernel merges with the local part (Sec. 3.3 "Output merging").
//
// Summary arithmetic is fp32, and every score that decides a selection keeps fp32-like precision, so the
// discrete choices agree with an fp64 evaluation at a 1e-5 margin: fp32 inputs score on fp32 MFMA; bf16 inputs
// score the exact bf16 query against the accumulated key summary split into a bf16 plane plus an fp16 plane of
// the remainder (>= 19 significant bits, exact products, fp32 accumulation) on the 16-bit matrix cores, and the
// block selection scores stay fp32.
#include "ff_common.h"

#include <type_traits>

namespace {

// ------------------------------------------------------------------------------------------
// bucketed copies of K and V: Xs[p] = X[perm[p]]
// ------------------------------------------------------------------------------------------
template <typename T>
__global__ void __launch_bounds__(256) k_gather_rows(const T* __restrict__ X, const int32_t* __restrict__ perm,
                                                      T* __restrict__ Xs, int N, int D) {
  const int CPR = D * (int)sizeof(T) / 16;
  size_t h = blockIdx.y;
  size_t c = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (c >= (size_t)N * CPR) return;
  int p = (int)(c / CPR), cc = (int)(c % CPR);
  int src = perm[h * N + p];
  const uint4* s = reinterpret_cast<const uint4*>(X + (h * N + src) * D) + cc;
  uint4* dst = reinterpret_cast<uint4*>(Xs + (h * N + p) * D) + cc;
  *dst = *s;
}

// ------------------------------------------------------------------------------------------
// tile schedule: tile_off[hq][b][i] = number of 32-query tiles of clusters < i in block b
// ------------------------------------------------------------------------------------------
__global__ void k_tile_schedule(const int32_t* __restrict__ off_q, int32_t* __restrict__ tile_off, int HQ, int nb,
                                int Cq) {
  int t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= HQ * nb) return;
  int hq = t / nb, b = t % nb;
  const int32_t* o = off_q + (size_t)hq * ((size_t)nb * Cq + 1) + (size_t)b * Cq;
  int32_t* to = tile_off + (size_t)t * (Cq + 1);
  int run = 0;
  for (int i = 0; i < Cq; ++i) {
    to[i] = run;
    run += (o[i + 1] - o[i] + 31) / 32;
  }
  to[Cq] = run;
}

// ------------------------------------------------------------------------------------------
// tilt logits L[hl][i][p] = (scale * qc_i) . Ks[p]   (keys in bucketed order)
// ------------------------------------------------------------------------------------------
// The same for bf16 keys on the matrix cores: the fp32 operand scale * qc is split into three bf16 terms
// (hi + mid + lo carry its 24 significant bits, each remainder is exact in fp32), the products with the bf16 keys
// are exact and the sums fp32, so L keeps fp32 accuracy; one wave per 32 keys, rows = query clusters.
template <int D>
__global__ void __launch_bounds__(256) k_tilt_logits_mx(const bf16_t* __restrict__ Ks, const float* __restrict__ qc,
                                                         float* __restrict__ L, int h0, int N, int Cq, int Hq, int Hkv,
                                                         float scale) {
  constexpr int KS = D / 16;
  const int hl = blockIdx.y, hq = h0 + hl;
  const int hk = (hq / Hq) * Hkv + (hq % Hq) / (Hq / Hkv);
  const int wave = threadIdx.x / 64, lane = threadIdx.x % 64, col = lane % 32, half = lane / 32;
  const int p0 = (blockIdx.x * 4 + wave) * 32;
  if (p0 >= N) return;
  const int p = p0 + col < N ? p0 + col : N - 1;
  bf16x8_t kb[KS];
#pragma unroll
  for (int x = 0; x < KS; ++x)
    kb[x] = *reinterpret_cast<const bf16x8_t*>(Ks + ((size_t)hk * N + p) * D + 16 * x + 8 * half);
  for (int i0 = 0; i0 < Cq; i0 += 32) {
    const int ic = i0 + col < Cq ? i0 + col : Cq - 1;
    const float* qr = qc + ((size_t)hq * Cq + ic) * D + 8 * half;
    f32x16_t acc = zero16();
#pragma unroll
    for (int x = 0; x < KS; ++x) {
      const float4 a = *reinterpret_cast<const float4*>(qr + 16 * x), b = *reinterpret_cast<const float4*>(qr + 16 * x + 4);
      const float v[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
      bf16x8_t hi, mid, lo;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float s0 = scale * v[e];
        hi[e] = (__bf16)s0;
        const float r1 = s0 - (float)hi[e];
        mid[e] = (__bf16)r1;
        lo[e] = (__bf16)(r1 - (float)mid[e]);
      }
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(hi, kb[x], acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(mid, kb[x], acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lo, kb[x], acc, 0, 0, 0);
    }
    if (p0 + col < N) {
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int i = i0 + 8 * (e / 4) + 4 * half + (e % 4);
        if (i < Cq) L[((size_t)hl * Cq + i) * N + p0 + col] = acc[e];
      }
    }
  }
}

template <typename T, int D>
__global__ void __launch_bounds__(256) k_tilt_logits(const T* __restrict__ Ks, const float* __restrict__ qc,
                                                      float* __restrict__ L, int h0, int N, int Cq, int Hq, int Hkv,
                                                      float scale) {
  __shared__ float qs[32][D];
  const int hl = blockIdx.y, hq = h0 + hl;
  const int hk = (hq / Hq) * Hkv + (hq % Hq) / (Hq / Hkv);
  const int p = blockIdx.x * 256 + threadIdx.x;
  const bool live = p < N;
  float k[D];
  {
    const T* row = Ks + ((size_t)hk * N + (live ? p : 0)) * D;
#pragma unroll
    for (int d = 0; d < D; d += 4) ld4(row, d, &k[d]);
  }
  for (int i0 = 0; i0 < Cq; i0 += 32) {
    __syncthreads();
    for (int t = threadIdx.x; t < 32 * D; t += 256) {
      int ii = t / D, d = t % D;
      qs[ii][d] = (i0 + ii < Cq) ? scale * qc[((size_t)hq * Cq + i0 + ii) * D + d] : 0.f;
    }
    __syncthreads();
    for (int ii = 0; ii < 32 && i0 + ii < Cq; ++ii) {
      float s = 0.f;
#pragma unroll
      for (int d = 0; d < D; ++d) s = fmaf(qs[ii][d], k[d], s);
      if (live) L[((size_t)hl * Cq + i0 + ii) * N + p] = s;
    }
  }
}

// ------------------------------------------------------------------------------------------
// exclusive accumulation of the per-block summaries (Eq. 4-6) on fp32 MFMA.  One wave per (key cluster j,
// tile of 32 query clusters, 64-wide slice of the head dim); it walks the key blocks in order and
// keeps the running accumulation in registers.  For a segment (j, b):
//   E^T[key, i] = exp(L[i, key] - max_i)         (B operand, row pattern over the keys)
//   Ksum^T[d, i] += K^T[d, key] E^T[key, i]      (A operand = bucketed K rows, column pattern)
// A_*[b] is the accumulation of blocks 0..b (what query block b+1 sees), b = 0..nb-2; of the summary of
// key block b alone only mu-bar (s_mu) is written here.
// ------------------------------------------------------------------------------------------
template <typename T, int D>
__global__ void __launch_bounds__(64) __attribute__((amdgpu_waves_per_eu(2, 4))) k_summaries(const T* __restrict__ Ks, const T* __restrict__ Vs,
                                                   const float* __restrict__ L, const int32_t* __restrict__ off_k,
                                                   float* __restrict__ s_mu, float* __restrict__ A_mu,
                                                   float* __restrict__ A_k, T* __restrict__ A_v,
                                                   bf16_t* __restrict__ A_kb, uint16_t* __restrict__ A_km,
                                                   float* __restrict__ A_muq, int h0, int N, int nb, int Cq, int Ck,
                                                   int Hq, int Hkv) {
  constexpr int DS = D / 64;  // slices of the head dim
  constexpr int KCH = 8;  // keys per chunk
  __shared__ float tr[32][68];
  // x % 8 is the XCD a workgroup lands on (the grid's x extent is a multiple of 8): each XCD takes a run of
  // consecutive key clusters, whose per-cell scalars share 32-byte sectors, so a sector is merged in one L2
  const int j = (blockIdx.x % 8) * (gridDim.x / 8) + blockIdx.x / 8;
  if (j >= Ck) return;
  const int hl = blockIdx.z, hq = h0 + hl;
  const int hk = (hq / Hq) * Hkv + (hq % Hq) / (Hq / Hkv);
  const int it = blockIdx.y / DS, d0 = (blockIdx.y % DS) * 64;
  const int lane = threadIdx.x, col = lane % 32, half = lane / 32;
  const int i = it * 32 + col;
  const bool iv = i < Cq;
  const int ic = iv ? i : Cq - 1;
  const int NBm = nb - 1;
  const int32_t* ok = off_k + (size_t)hk * ((size_t)nb * Ck + 1);
  const float* Li = L + ((size_t)hl * Cq + ic) * N;
  // accumulator tile x, row m holds head dim d0 + 2 m + x: one paired load feeds both tiles
  const T* Kh = Ks + (size_t)hk * N * D + d0 + 2 * col;
  const T* Vh = Vs + (size_t)hk * N * D + d0 + 2 * col;

  // output rows of the lane after the LDS transpose: rows 4 ps + lane/16 of the tile, 4 head dims from 4 (lane%16)
  const int lrow = lane / 16, nrow = Cq - it * 32 < 32 ? Cq - it * 32 : 32;
  const uint32_t loff = (uint32_t)lrow * Ck * D + d0 + 4 * (lane % 16), pstr = 4u * Ck * D;
  // One chunk of keys as the lane consumes it; the loads of the next chunk (of this block or of the next
  // non-empty one) are issued before the current chunk is used.
  struct Chunk {
    float lg[KCH / 8][4];
    typename Pair<T>::raw kk[KCH / 8][4], vv[KCH / 8][4];
  };
  auto load_chunk = [&](Chunk& c, int c0, int hi) {
#pragma unroll
    for (int u = 0; u < KCH / 8; ++u)
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        const int p = c0 + 8 * u + 4 * half + t;
        const int pc = p < hi ? p : hi - 1;
        c.lg[u][t] = Li[pc];
        c.kk[u][t] = Pair<T>::ld(Kh, (size_t)pc * D);
        c.vv[u][t] = Pair<T>::ld(Vh, (size_t)pc * D);
      }
  };
  // position of the chunk in flight: block nb_, first key nc0, end of its cell nhi (nb_ == NBm: none)
  int nb_ = 0, nc0 = 0, nhi = 0;
  Chunk nxt;
  auto seek = [&]() {  // first non-empty cell at or after block nb_
    while (nb_ < NBm) {
      nc0 = ok[nb_ * Ck + j];
      nhi = ok[nb_ * Ck + j + 1];
      if (nc0 < nhi) break;
      ++nb_;
    }
    if (nb_ < NBm) load_chunk(nxt, nc0, nhi);
  };
  seek();

  // The accumulation runs directly in the accumulated summaries' registers, relative to the running maximum
  // Amx of all blocks so far; the block's own log-sum-exp (mu-bar of the block) is kept beside it as scalars.
  // AL: the weights' sum of the logits themselves, L = scale * qc_i . k, so AL / AS = scale * qc_i . k-bar
  float Amx = MUSE_NEG_INF, AS = 0.f, AL = 0.f;
  f32x16_t Aak[2], Aav[2];
  Aak[0] = zero16(); Aak[1] = zero16(); Aav[0] = zero16(); Aav[1] = zero16();
  for (int b = 0; b < NBm; ++b) {
    float mx = MUSE_NEG_INF, S = 0.f;
    bool empty = true;
    while (nb_ == b) {
      empty = false;
      // The prefetched chunk is first touched HERE: without this fence the compiler hoists the copy below (and
      // with it the wait for the loads) above the previous block's stores, into the iteration that issued them.
#pragma unroll
      for (int u = 0; u < KCH / 8; ++u)
#pragma unroll
        for (int t = 0; t < 4; ++t) asm volatile("" : "+v"(nxt.lg[u][t]), "+v"(nxt.kk[u][t]), "+v"(nxt.vv[u][t]) : : "memory");
      const Chunk cur = nxt;
      const int c0 = nc0, hi = nhi;
      nc0 += KCH;
      if (nc0 < nhi) load_chunk(nxt, nc0, nhi);
      else { ++nb_; seek(); }
      float lg[KCH / 8][4];
      float cm = MUSE_NEG_INF;
#pragma unroll
      for (int u = 0; u < KCH / 8; ++u)
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          lg[u][t] = c0 + 8 * u + 4 * half + t < hi ? cur.lg[u][t] : MUSE_NEG_INF;
          cm = fmaxf(cm, lg[u][t]);
        }
      cm = fmaxf(cm, __shfl_xor(cm, 32, 64));
      const float nmb = fmaxf(mx, cm);
      S *= __expf(mx - nmb);
      mx = nmb;
      const float nm = fmaxf(Amx, cm);
      const float resc = __expf(Amx - nm);
      Amx = nm;
      AS *= resc;
      AL *= resc;
#pragma unroll
      for (int x = 0; x < 2; ++x)
#pragma unroll
        for (int e = 0; e < 16; ++e) { Aak[x][e] *= resc; Aav[x][e] *= resc; }
#pragma unroll
      for (int u = 0; u < KCH / 8; ++u)
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          S += __expf(lg[u][t] - nmb);
          const float e = __expf(lg[u][t] - nm);
          AS += e;
          AL = fmaf(e, c0 + 8 * u + 4 * half + t < hi ? cur.lg[u][t] : 0.f, AL);
          Aak[0] = mfma32(Pair<T>::lo(cur.kk[u][t]), e, Aak[0]);
          Aak[1] = mfma32(Pair<T>::hi(cur.kk[u][t]), e, Aak[1]);
          Aav[0] = mfma32(Pair<T>::lo(cur.vv[u][t]), e, Aav[0]);
          Aav[1] = mfma32(Pair<T>::hi(cur.vv[u][t]), e, Aav[1]);
        }
    }
    S += __shfl_xor(S, 32, 64);
    const float ASt = AS + __shfl_xor(AS, 32, 64);
    const float ALt = AL + __shfl_xor(AL, 32, 64);
    const size_t cell = (((size_t)hl * NBm + b) * Cq + ic) * Ck + j;
    const bool aempty = ASt == 0.f;
    const float ainv = aempty ? 0.f : 1.f / ASt;
    if (iv && half == 0 && d0 == 0) {
      s_mu[cell] = empty ? MUSE_NEG_INF : mx + __logf(S);
      const float amu = aempty ? MUSE_NEG_INF : Amx + __logf(ASt);
      A_mu[cell] = amu;
      if (sizeof(T) == 2) A_muq[cell] = aempty ? MUSE_NEG_INF : amu - ALt * ainv;
    }
    // transpose each 64 x 32 accumulator slice through LDS so that a store instruction writes four whole
    // 256-byte row segments instead of 32 fragments of 32 bytes
    // Addresses: a uniform base per block plus 32-bit lane offsets that do not change over the blocks.
    const size_t rowbase = (((size_t)hl * NBm + b) * Cq + it * 32) * Ck + j;
    const size_t slab = rowbase * D;
    auto emit = [&](float* __restrict__ dstf, bf16_t* __restrict__ dsth, const f32x16_t(&a)[2], float sc) {
      float* pf = dstf ? dstf + slab : nullptr;
      bf16_t* ph = dsth ? dsth + slab : nullptr;
#pragma unroll
      for (int g = 0; g < 4; ++g)
#pragma unroll
        for (int t = 0; t < 4; ++t)
          *reinterpret_cast<float2*>(&tr[col][2 * (8 * g + 4 * half + t)]) = make_float2(a[0][4 * g + t] * sc, a[1][4 * g + t] * sc);
      wave_lds_fence();
#pragma unroll
      for (int ps = 0; ps < 8; ++ps) {
        if (4 * ps + lrow < nrow) {
          const float4 v = *reinterpret_cast<const float4*>(&tr[4 * ps + lrow][4 * (lane % 16)]);
          const uint32_t o = loff + ps * pstr;
          if (dstf) *reinterpret_cast<float4*>(pf + o) = v;
          if (dsth) { const unsigned long long pk = (unsigned long long)pack_bf16x2(v.x, v.y) | ((unsigned long long)pack_bf16x2(v.z, v.w) << 32); __builtin_nontemporal_store(pk, reinterpret_cast<unsigned long long*>(ph + o)); }
        }
      }
      wave_lds_fence();
    };
    // the accumulated k-bar of bf16 inputs as a bf16 plane and an fp16 plane of the remainder (what the 16-bit
    // score MFMAs of the tile kernel take)
    auto emit_planes = [&](const f32x16_t(&a)[2], float sc) {
      bf16_t* ph = A_kb + slab;
      uint16_t* pm = A_km + slab;
#pragma unroll
      for (int g = 0; g < 4; ++g)
#pragma unroll
        for (int t = 0; t < 4; ++t)
          *reinterpret_cast<float2*>(&tr[col][2 * (8 * g + 4 * half + t)]) = make_float2(a[0][4 * g + t] * sc, a[1][4 * g + t] * sc);
      wave_lds_fence();
#pragma unroll
      for (int ps = 0; ps < 8; ++ps) {
        if (4 * ps + lrow < nrow) {
          const float4 v = *reinterpret_cast<const float4*>(&tr[4 * ps + lrow][4 * (lane % 16)]);
          const uint32_t o = loff + ps * pstr;
          const uint32_t h01 = pack_bf16x2(v.x, v.y), h23 = pack_bf16x2(v.z, v.w);
          __builtin_nontemporal_store((unsigned long long)h01 | ((unsigned long long)h23 << 32), reinterpret_cast<unsigned long long*>(ph + o));
          const float r0 = v.x - __uint_as_float(h01 << 16), r1 = v.y - __uint_as_float(h01 & 0xffff0000u);
          const float r2 = v.z - __uint_as_float(h23 << 16), r3 = v.w - __uint_as_float(h23 & 0xffff0000u);
          auto hb = [](float x) { return (uint32_t)__builtin_bit_cast(unsigned short, (_Float16)x); };
          __builtin_nontemporal_store((unsigned long long)(hb(r0) | hb(r1) << 16) | ((unsigned long long)(hb(r2) | hb(r3) << 16) << 32), reinterpret_cast<unsigned long long*>(pm + o));
        }
      }
      wave_lds_fence();
    };
    // values go out in the input type; the accumulated k-bar in fp32 for fp32 inputs, as planes for bf16 inputs
    // The per-block rows s_k, s_v are read for retrieved (query cluster, key cluster) chains only, about one
    // chain in ten: they are written later, for those chains, by k_block_summaries; mu-bar is dense.
    constexpr bool kH = sizeof(T) == 2;
    if constexpr (kH) emit_planes(Aak, ainv);
    else emit(A_k, nullptr, Aak, ainv);
    emit(kH ? nullptr : reinterpret_cast<float*>(A_v), kH ? reinterpret_cast<bf16_t*>(A_v) : nullptr, Aav, ainv);
  }
}

// ------------------------------------------------------------------------------------------
// Per-block summaries (Eq. 4-6) of the retrieved chains.  chainmask[hl][i][j/32] has bit j%32 set when some
// query of cluster i (blocks >= 1) retrieved key cluster j; only those (i, j) chains are ever read at block
// granularity (block selection and component 2, forward and backward).
// ------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) k_chainmask(const int32_t* __restrict__ selc, const int32_t* __restrict__ aq,
                                                    uint32_t* __restrict__ chainmask, int h0, int N, int Bs, int r,
                                                    int Cq, int W) {
  const int hl = blockIdx.y;
  const size_t t = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (t >= (size_t)(N - Bs) * r) return;
  const size_t qn = (size_t)(h0 + hl) * N + Bs + t / r;
  const int j = selc[qn * r + t % r];
  if (j >= 0) atomicOr(&chainmask[((size_t)hl * Cq + aq[qn]) * W + (j >> 5)], 1u << (j & 31));
}

// the mask key-cluster-major: maskT[hl][j][i/32] bit i%32.  One wave per (32 query clusters, 32 key clusters): lane
// i holds the word of its row, a ballot per bit gives the 32 rows' bits of one column.
__global__ void __launch_bounds__(64) k_chainmask_t(const uint32_t* __restrict__ chainmask, uint32_t* __restrict__ maskT,
                                                     int Cq, int Ck, int W, int WT) {
  const int jt = blockIdx.x, itile = blockIdx.y, hl = blockIdx.z, lane = threadIdx.x;
  const int i = itile * 32 + lane;
  const uint32_t word = (lane < 32 && i < Cq) ? chainmask[((size_t)hl * Cq + i) * W + jt] : 0u;
  uint32_t mine = 0u;
#pragma unroll
  for (int jl = 0; jl < 32; ++jl) {
    const uint32_t colbits = (uint32_t)__ballot((word >> jl) & 1u);
    if (lane == jl) mine = colbits;
  }
  const int j = jt * 32 + lane;
  if (lane < 32 && j < Ck) maskT[((size_t)hl * Ck + j) * WT + itile] = mine;
}

// One wave per (query cluster i, tile of 32 key clusters).  A chain's blocks go to the wave's eight 8-lane
// groups (block b to group b % 8), each lane holding D/8 adjacent head dims.  With mu-bar known, the normalised
// weight of key p in cell (b, i, j) is exp(L[i][p] - mu-bar), so a row is one pass over the cell's keys.
template <typename T, int D>
__global__ void __launch_bounds__(64) k_block_summaries(const T* __restrict__ Ks, const T* __restrict__ Vs,
                                                         const float* __restrict__ L, const int32_t* __restrict__ off_k,
                                                         const uint32_t* __restrict__ chainmask,
                                                         const float* __restrict__ s_mu, float* __restrict__ s_k,
                                                         T* __restrict__ s_v, int h0, int N, int nb, int Cq, int Ck,
                                                         int Hq, int Hkv) {
  constexpr int DL = D / 8, NV = DL / 4, KB = 4;
  const int jt = blockIdx.x, i = blockIdx.y, hl = blockIdx.z, hq = h0 + hl;
  const int hk = (hq / Hq) * Hkv + (hq % Hq) / (Hq / Hkv);
  const int g = threadIdx.x >> 3, l8 = threadIdx.x & 7, NBm = nb - 1, W = (Ck + 31) / 32;
  uint32_t word = chainmask[((size_t)hl * Cq + i) * W + jt];
  const int32_t* ok = off_k + (size_t)hk * ((size_t)nb * Ck + 1);
  const float* Li = L + ((size_t)hl * Cq + i) * N;
  const T* Kh = Ks + (size_t)hk * N * D + DL * l8;
  const T* Vh = Vs + (size_t)hk * N * D + DL * l8;
  for (; word; word &= word - 1) {
    const int j = jt * 32 + __ffs((int)word) - 1;
    for (int b = g; b < NBm; b += 8) {
      const int lo = ok[b * Ck + j], hi = ok[b * Ck + j + 1];
      const size_t cell = (((size_t)hl * NBm + b) * Cq + i) * Ck + j;
      const float mu = s_mu[cell];
      float ak[DL], av[DL];
#pragma unroll
      for (int x = 0; x < DL; ++x) { ak[x] = 0.f; av[x] = 0.f; }
      for (int p0 = lo; p0 < hi; p0 += KB) {
        float lg[KB], kv[KB][DL], vv[KB][DL];
#pragma unroll
        for (int u = 0; u < KB; ++u) {  // all loads of the batch first
          const int p = p0 + u < hi ? p0 + u : hi - 1;
          lg[u] = Li[p];
#pragma unroll
          for (int x = 0; x < NV; ++x) {
            ld4(Kh, (size_t)p * D + 4 * x, &kv[u][4 * x]);
            ld4(Vh, (size_t)p * D + 4 * x, &vv[u][4 * x]);
          }
        }
#pragma unroll
        for (int u = 0; u < KB; ++u) {
          const float wgt = p0 + u < hi ? __expf(lg[u] - mu) : 0.f;
#pragma unroll
          for (int x = 0; x < DL; ++x) {
            ak[x] = fmaf(wgt, kv[u][x], ak[x]);
            av[x] = fmaf(wgt, vv[u][x], av[x]);
          }
        }
      }
#pragma unroll
      for (int x = 0; x < NV; ++x) {  // an empty cell gets zero rows
        st4(s_k, cell * D + DL * l8 + 4 * x, &ak[4 * x]);
        st4(s_v, cell * D + DL * l8 + 4 * x, &av[4 * x]);
      }
    }
  }
}

// The same rows on fp32 MFMA, key-cluster-major: one wave per (key cluster j, key block b), four blocks to a workgroup.  The query clusters
// whose chain (i, j) is retrieved are listed from the mask's column (ballot ranks, ascending i) and taken 32 at a
// time as the MFMA columns; the cell's keys are the contraction index, two per instruction, as in k_summaries:
//   E^T[key, i] = exp(L[i, key] - mu-bar[b, i, j]),   s_k^T[d, i] = sum_key K^T[d, key] E^T[key, i]
// A cell's keys are read once for all its chains instead of once per chain, and the sums leave through an LDS
// transpose as whole rows.
template <typename T, int D>
__global__ void __launch_bounds__(256) k_block_summaries_mx(const T* __restrict__ Ks, const T* __restrict__ Vs,
                                                            const float* __restrict__ L, const int32_t* __restrict__ off_k,
                                                            const uint32_t* __restrict__ maskT,
                                                            const float* __restrict__ s_mu, float* __restrict__ s_k,
                                                            T* __restrict__ s_v, int h0, int N, int nb, int Cq, int Ck,
                                                            int Hq, int Hkv) {
  constexpr int DS = D / 64;
  __shared__ float tr_all[4][32][68];
  __shared__ uint16_t list[MUSE_MAX_CLUSTERS];
  __shared__ int nflag_s;
  const int j = (blockIdx.x % 8) * (gridDim.x / 8) + blockIdx.x / 8;  // an XCD takes a run of consecutive clusters
  if (j >= Ck) return;
  // the four waves of a workgroup take four key blocks of the same cluster and share its list of chains
  const int wave = threadIdx.x / 64, b = 4 * blockIdx.y + wave, hl = blockIdx.z, hq = h0 + hl;
  const int hk = (hq / Hq) * Hkv + (hq % Hq) / (Hq / Hkv);
  const int lane = threadIdx.x % 64, col = lane % 32, half = lane / 32, NBm = nb - 1, WT = (Cq + 31) / 32;
  float (*tr)[68] = tr_all[wave];
  if (wave == 0) {
    int nf = 0;
    for (int i0 = 0; i0 < Cq; i0 += 64) {
      const int i = i0 + lane;
      const bool f = i < Cq && ((maskT[((size_t)hl * Ck + j) * WT + (i >> 5)] >> (i & 31)) & 1u);
      const unsigned long long bal = __ballot(f);
      if (f) list[nf + __popcll(bal & ((1ull << lane) - 1ull))] = (uint16_t)i;
      nf += __popcll(bal);
    }
    if (lane == 0) nflag_s = nf;
  }
  __syncthreads();
  const int nflag = nflag_s;
  if (nflag == 0 || b >= NBm) return;
  const int32_t* ok = off_k + (size_t)hk * ((size_t)nb * Ck + 1);
  const int lo = ok[b * Ck + j], hi = ok[b * Ck + j + 1];
  const int lrow = lane / 16;
  for (int it = 0; it * 32 < nflag; ++it) {
    const int nrow = nflag - 32 * it < 32 ? nflag - 32 * it : 32;
    const int il = list[32 * it + (col < nrow ? col : nrow - 1)];
    const size_t cell = (((size_t)hl * NBm + b) * Cq + il) * Ck + j;
    const float mu = s_mu[cell];
    const float* Li = L + ((size_t)hl * Cq + il) * N;
#pragma unroll
    for (int ds = 0; ds < DS; ++ds) {
      const int d0 = 64 * ds;
      // accumulator tile x, row m holds head dim d0 + 2 m + x: one paired load feeds both tiles
      const T* Kh = Ks + (size_t)hk * N * D + d0 + 2 * col;
      const T* Vh = Vs + (size_t)hk * N * D + d0 + 2 * col;
      f32x16_t ak[2], av[2];
      ak[0] = zero16(); ak[1] = zero16(); av[0] = zero16(); av[1] = zero16();
      for (int c0 = lo; c0 < hi; c0 += 8) {
        float lg[4];
        typename Pair<T>::raw kk[4], vv[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          const int p = c0 + 4 * half + t;
          const int pc = p < hi ? p : hi - 1;
          lg[t] = Li[pc];
          kk[t] = Pair<T>::ld(Kh, (size_t)pc * D);
          vv[t] = Pair<T>::ld(Vh, (size_t)pc * D);
        }
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          const float e = c0 + 4 * half + t < hi ? __expf(lg[t] - mu) : 0.f;
          ak[0] = mfma32(Pair<T>::lo(kk[t]), e, ak[0]);
          ak[1] = mfma32(Pair<T>::hi(kk[t]), e, ak[1]);
          av[0] = mfma32(Pair<T>::lo(vv[t]), e, av[0]);
          av[1] = mfma32(Pair<T>::hi(vv[t]), e, av[1]);
        }
      }
      // rows out through the LDS transpose: 16 lanes write one row's 64 dims (an empty cell gives zero rows)
      auto emit = [&](const f32x16_t(&a)[2], bool values) {
#pragma unroll
        for (int g = 0; g < 4; ++g)
#pragma unroll
          for (int t = 0; t < 4; ++t)
            *reinterpret_cast<float2*>(&tr[col][2 * (8 * g + 4 * half + t)]) = make_float2(a[0][4 * g + t], a[1][4 * g + t]);
        wave_lds_fence();
#pragma unroll
        for (int ps = 0; ps < 8; ++ps) {
          const int row = 4 * ps + lrow;
          if (row < nrow) {
            const float4 v = *reinterpret_cast<const float4*>(&tr[row][4 * (lane % 16)]);
            const size_t o = ((((size_t)hl * NBm + b) * Cq + list[32 * it + row]) * Ck + j) * D + d0 + 4 * (lane % 16);
            const float v4[4] = {v.x, v.y, v.z, v.w};
            if (values) st4_stream(s_v, o, v4);
            else st4_stream(s_k, o, v4);
          }
        }
        wave_lds_fence();
      };
      emit(ak, false);
      emit(av, true);
    }
  }
}

// ------------------------------------------------------------------------------------------
// the per-query-tile far-field kernel: one wave per tile of up to 32 queries of one
// (spatial block b >= 1, query cluster i): cluster scores (Eq. 7), the r retrieved clusters, and the
// monopole attention over all other clusters (component 1) as a partial softmax state
// ------------------------------------------------------------------------------------------
template <typename T, int D, int RCAP>
__global__ void __launch_bounds__(64) __attribute__((amdgpu_waves_per_eu(D == 64 ? 2 : 1, D == 64 ? 2 : 2))) k_farfield_fwd(
    const T* __restrict__ Q, const float* __restrict__ qc, const float* __restrict__ A_mu, const float* __restrict__ A_k,
    const bf16_t* __restrict__ A_kb, const uint16_t* __restrict__ A_km, const float* __restrict__ A_c,
    const T* __restrict__ A_v, const int32_t* __restrict__ perm_q, const int32_t* __restrict__ off_q,
    const int32_t* __restrict__ tile_off, float* __restrict__ ff_acc, float* __restrict__ ff_ml,
    int32_t* __restrict__ selc, int h0, int N, int nb, int Cq, int Ck, int r, float scale,
    const int32_t* __restrict__ only_flag) {
  constexpr int U = D / 8, DT = D / 32;
  // as the second launch behind the one-plane kernel: only the tiles that kernel flagged
  if (only_flag && only_flag[((size_t)blockIdx.z * (nb - 1) + blockIdx.y) * gridDim.x + blockIdx.x] == 0) return;
  // fp32 inputs: output tile x, row m holds head dim DT*m + x (a lane reads DT consecutive dims of a value row)
  using VF = Frag<T, DT>;
  constexpr bool kH = sizeof(T) == 2;  // bf16 inputs: P V on bf16 MFMA through a transposed value tile in LDS
  constexpr int CPR = D / 8, NIT = 32 * CPR / 64;
  __shared__ __attribute__((aligned(16))) bf16_t vt[kH ? D : 1][32 + 4];
  __shared__ float cs[64][RCAP];
  __shared__ int ci[64][RCAP];
  __shared__ int sel_s[32][RCAP];
  const int hl = blockIdx.z, hq = h0 + hl;
  const int b = blockIdx.y + 1, NBm = nb - 1;
  const int lane = threadIdx.x, col = lane % 32, half = lane / 32;

  const int32_t* to = tile_off + ((size_t)hq * nb + b) * (Cq + 1);
  // Workgroups go to the 8 XCDs round-robin by their linear id and the grid's x extent is a multiple of 8, so
  // x % 8 is the XCD: each XCD takes a contiguous run of the tiles, and the tiles of one (block, query cluster)
  // group, which stream the same cells at about the same time, share its L2.
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
  const int qlo = oq[b * Cq + i], qhi = oq[b * Cq + i + 1];
  int pos = qlo + 32 * tt + col;
  const bool valid = pos < qhi;
  pos = valid ? pos : qlo + 32 * tt;
  const int n = perm_q[(size_t)hq * N + pos];

  // fp32 inputs: q~ in the row pattern of the fp32 score MFMAs; bf16 inputs: the query itself as bf16 and fp16
  float qt[kH ? 1 : U][4];
  bf16x8_t qb[kH ? D / 16 : 1];
  f16x8_t qh[kH ? D / 16 : 1];
  {
    const T* qrow = Q + ((size_t)hq * N + n) * D;
    if constexpr (kH) {
#pragma unroll
      for (int ks = 0; ks < D / 16; ++ks) {
        qb[ks] = *reinterpret_cast<const bf16x8_t*>(qrow + 16 * ks + 8 * half);
#pragma unroll
        for (int e = 0; e < 8; ++e) qh[ks][e] = (_Float16)(float)qb[ks][e];
      }
    } else {
      const float* qci = qc + ((size_t)hq * Cq + i) * D;
#pragma unroll
      for (int u = 0; u < U; ++u) {
        float x[4];
        ld4(qrow, 8 * u + 4 * half, x);
        float4 c = *reinterpret_cast<const float4*>(qci + 8 * u + 4 * half);
        qt[u][0] = scale * (x[0] - c.x); qt[u][1] = scale * (x[1] - c.y);
        qt[u][2] = scale * (x[2] - c.z); qt[u][3] = scale * (x[3] - c.w);
      }
    }
  }
  const size_t acell = (((size_t)hl * NBm + (b - 1)) * Cq + i) * Ck;
  const float* Amu = A_mu + acell;
  const T* Av = A_v + acell * D;
  const int ntile = (Ck + 31) / 32;
  using KT = typename std::conditional<kH, KTileH<D>, KTile<D>>::type;
  auto load_kt = [&](KT& kt, int j0) {
    if constexpr (kH) load_ktile_h<D>(kt, A_c + acell, A_kb + acell * D, A_km + acell * D, j0, Ck, col, half);
    else load_ktile<D>(kt, Amu, A_k + acell * D, j0, Ck, col, half);
  };
  auto score_kt = [&](const KT& kt, int j0) {
    if constexpr (kH) return score_ktile_h<D>(kt, j0, Ck, qb, qh, scale, half);
    else return score_ktile<D>(kt, j0, Ck, qt, half);
  };

  // ---- pass 1: the r largest scores seen by this lane half (values only) ----
  float list[RCAP];
#pragma unroll
  for (int k = 0; k < RCAP; ++k) list[k] = MUSE_NEG_INF;
  {
    // insertion into the sorted list: new l_k = med3(x, l_{k-1}, l_k), new l_0 = max(x, l_0)
    auto insert = [&](const f32x16_t& acc) {
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const float x = acc[e];
#pragma unroll
        for (int k = RCAP - 1; k > 0; --k) list[k] = __builtin_amdgcn_fmed3f(x, list[k - 1], list[k]);
        list[0] = fmaxf(list[0], x);
      }
    };
    // two tile buffers: the loads of the next tile are in flight while this one is scored
    KT ka, kb;
    load_kt(ka, 0);
    for (int jt = 0; jt < ntile; jt += 2) {
      if (jt + 1 < ntile) load_kt(kb, (jt + 1) * 32);
      insert(score_kt(ka, jt * 32));
      if (jt + 1 < ntile) {
        if (jt + 2 < ntile) load_kt(ka, (jt + 2) * 32);
        insert(score_kt(kb, (jt + 1) * 32));
      }
    }
  }
  // ---- split the quota of r between the two halves of the query (ties: lower half first) ----
  int quota = 0;
  {
    float other[RCAP];
#pragma unroll
    for (int k = 0; k < RCAP; ++k) other[k] = __shfl_xor(list[k], 32, 64);
#pragma unroll
    for (int k = 0; k < RCAP; ++k) {
      int ahead = 0;
#pragma unroll
      for (int y = 0; y < RCAP; ++y) ahead += half == 0 ? (other[y] > list[k]) : (other[y] >= list[k]);
      quota += (k + ahead < r) && (list[k] > MUSE_NEG_INF);
    }
  }
  float thr = __builtin_huge_valf();
#pragma unroll
  for (int k = 0; k < RCAP; ++k)
    if (k == quota - 1) thr = list[k];
  int cgt = 0;
#pragma unroll
  for (int k = 0; k < RCAP; ++k) cgt += (k < quota) && (list[k] > thr);
  const int eqquota = quota - cgt;

  // ---- pass 2: same scores again; selected ones are recorded and masked, the rest is the
  //      monopole attention over accumulated value summaries (component 1) ----
  float m = MUSE_NEG_INF, l = 0.f;
  f32x16_t o[DT];
#pragma unroll
  for (int t = 0; t < DT; ++t) o[t] = zero16();
  int eqc = 0, ncand = 0;
  // a tile's operands: k-bar rows, mu-bar, and the value rows (bf16: this lane's chunks of the 32 x D tile;
  // fp32: the DT consecutive dims DT*col .. of its 16 rows), all loaded before the first use
  struct PTile {
    KT kt;
    typename VF::raw vv[kH ? 1 : 16];
    uint4 vch[kH ? NIT : 1];
  };
  auto load_ptile = [&](PTile& pt, int j0) {
    load_kt(pt.kt, j0);
    if constexpr (kH) {
#pragma unroll
      for (int it = 0; it < NIT; ++it) {
        const int c = lane + 64 * it, row = c % 32, cc = c / 32;  // lanes along the rows: conflict-free transposed stores
        const int jr = j0 + row < Ck ? j0 + row : Ck - 1;
        pt.vch[it] = *reinterpret_cast<const uint4*>(Av + (size_t)jr * D + cc * 8);
      }
    } else {
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        int jr = j0 + 8 * (e / 4) + 4 * half + (e % 4);
        jr = jr < Ck ? jr : Ck - 1;
        pt.vv[e] = VF::ld(Av, (size_t)jr * D + DT * col);
      }
    }
  };
  auto process = [&](const PTile& pt, int j0) {
    const KT& kt = pt.kt;
    const auto& vv = pt.vv;
    const auto& vch = pt.vch;
    f32x16_t acc = score_kt(kt, j0);
    float tmax = MUSE_NEG_INF;
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      float s = acc[e];
      bool eq = (s == thr) && (eqc < eqquota);
      bool take = (s > thr) || eq;
      eqc += eq;
      if (take) {
        cs[lane][ncand] = s;
        ci[lane][ncand] = j0 + 8 * (e / 4) + 4 * half + (e % 4);
        ++ncand;
        acc[e] = MUSE_NEG_INF;
      }
      tmax = fmaxf(tmax, acc[e]);
    }
    tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
    float mn = fmaxf(m, tmax);
    float mref = mn == MUSE_NEG_INF ? 0.f : mn;
    float alpha = __expf(m - mref);
    float psum = 0.f;
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      float p = __expf(acc[e] - mref);
      acc[e] = p;
      psum += p;
    }
    l = l * alpha + psum;
    m = mn;
#pragma unroll
    for (int t = 0; t < DT; ++t)
#pragma unroll
      for (int e = 0; e < 16; ++e) o[t][e] *= alpha;
    if constexpr (kH) {
      wave_lds_fence();
#pragma unroll
      for (int it = 0; it < NIT; ++it) {
        const int c = lane + 64 * it, row = c % 32, cc = c / 32;  // lanes along the rows: conflict-free transposed stores
        const bf16_t* pv = reinterpret_cast<const bf16_t*>(&vch[it]);
#pragma unroll
        for (int e = 0; e < 8; ++e) vt[cc * 8 + e][row] = pv[e];
      }
      wave_lds_fence();
#pragma unroll
      for (int G = 0; G < 2; ++G) {
        const bf16x8_t pf = pack8(acc, 2 * G, 2 * G + 1);
#pragma unroll
        for (int x = 0; x < DT; ++x)
          o[x] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ld_tr8(&vt[32 * x + col][0], 16 * G, half), pf, o[x], 0, 0, 0);
      }
    } else {
#pragma unroll
      for (int e = 0; e < 16; ++e) {
#pragma unroll
        for (int x = 0; x < DT; ++x) o[x] = mfma32(VF::get(vv[e], x), acc[e], o[x]);
      }
    }
  };
  // (two tile buffers, as in pass 1, need more registers than two waves per SIMD leave: measured slower)
  for (int jt = 0; jt < ntile; ++jt) {
    PTile pt;
    load_ptile(pt, jt * 32);
    process(pt, jt * 32);
  }
  // ---- order the selected clusters of each query by (score desc, index asc) ----
  for (int k = lane; k < 32 * RCAP; k += 64) (&sel_s[0][0])[k] = -1;
  __syncthreads();
  {
    const int nother = __shfl_xor(ncand, 32, 64);
    const int total = ncand + nother;
    for (int k = 0; k < ncand; ++k) {
      float sv = cs[lane][k];
      int iv = ci[lane][k];
      int rank = 0;
      for (int y = 0; y < ncand; ++y) rank += (cs[lane][y] > sv) || (cs[lane][y] == sv && ci[lane][y] < iv);
      for (int y = 0; y < nother; ++y)
        rank += (cs[lane ^ 32][y] > sv) || (cs[lane ^ 32][y] == sv && ci[lane ^ 32][y] < iv);
      sel_s[col][rank] = iv;
    }
    __syncthreads();
    if (valid && half == 0) {
      int32_t* out = selc + ((size_t)hq * N + n) * r;
      for (int k = 0; k < r; ++k) out[k] = k < total ? sel_s[col][k] : -1;
    }
  }
  l += __shfl_xor(l, 32, 64);
  if (!valid) return;
  float* fa = ff_acc + ((size_t)hq * N + n) * D;
#pragma unroll
  for (int g = 0; g < 4; ++g) {
    if (kH) {  // output tile x, row m holds head dim 32 x + m
#pragma unroll
      for (int x = 0; x < DT; ++x)
        *reinterpret_cast<float4*>(fa + 32 * x + 8 * g + 4 * half) =
            make_float4(o[x][4 * g], o[x][4 * g + 1], o[x][4 * g + 2], o[x][4 * g + 3]);
    } else if (DT == 2) {
#pragma unroll
      for (int tp = 0; tp < 2; ++tp)
        *reinterpret_cast<float4*>(fa + 2 * (8 * g + 4 * half + 2 * tp)) =
            make_float4(o[0][4 * g + 2 * tp], o[1][4 * g + 2 * tp], o[0][4 * g + 2 * tp + 1], o[1][4 * g + 2 * tp + 1]);
    } else {
#pragma unroll
      for (int t = 0; t < 4; ++t)
        *reinterpret_cast<float4*>(fa + 4 * (8 * g + 4 * half + t)) =
            make_float4(o[0][4 * g + t], o[1][4 * g + t], o[2 % DT][4 * g + t], o[3 % DT][4 * g + t]);
    }
  }
  if (half == 0) {
    ff_ml[((size_t)hq * N + n) * 2] = m;
    ff_ml[((size_t)hq * N + n) * 2 + 1] = l;
  }
}

// ------------------------------------------------------------------------------------------
// largest Euclidean norm of a key row per kv head: every k-bar is a convex combination of key rows, so this bounds
// |k-bar| for the error bound of the one-plane scores
// ------------------------------------------------------------------------------------------
constexpr int kNormParts = 64;  // workgroups per kv head in the first stage
template <int D>
__global__ void __launch_bounds__(256) k_key_norm_part(const bf16_t* __restrict__ K, float* __restrict__ part, int N) {
  __shared__ float red[4];
  const int hk = blockIdx.y;
  float best = 0.f;
  for (int n = blockIdx.x * 256 + threadIdx.x; n < N; n += 256 * kNormParts) {
    const bf16_t* row = K + ((size_t)hk * N + n) * D;
    float s = 0.f;
#pragma unroll
    for (int c = 0; c < D / 8; ++c) {
      const bf16x8_t v = *reinterpret_cast<const bf16x8_t*>(row + 8 * c);
#pragma unroll
      for (int e = 0; e < 8; ++e) s = fmaf((float)v[e], (float)v[e], s);
    }
    best = fmaxf(best, s);
  }
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) best = fmaxf(best, __shfl_xor(best, o, 64));
  if (threadIdx.x % 64 == 0) red[threadIdx.x / 64] = best;
  __syncthreads();
  if (threadIdx.x == 0) part[(size_t)hk * kNormParts + blockIdx.x] = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
}
__global__ void __launch_bounds__(64) k_key_norm_max(const float* __restrict__ part, float* __restrict__ knorm) {
  float best = part[(size_t)blockIdx.x * kNormParts + threadIdx.x];
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) best = fmaxf(best, __shfl_xor(best, o, 64));
  if (threadIdx.x == 0) knorm[blockIdx.x] = sqrtf(best);
}

// ------------------------------------------------------------------------------------------
// The per-query-tile far-field kernel for bf16 inputs whose first pass streams the bf16 plane of k-bar only.
// A score from the bf16 plane alone (Eq. 7 up to the plane's rounding) is off by at most
//   eps = scale * 2^-8 * |q| * max_n |k_n|     (plus the rounding of the fp32 accumulation),
// and r clusters reach the r-th largest approximate score, so the r-th largest exact score is at least that
// minus eps: the cut.
//   pass 1   approximate scores (bf16 plane and the per-cell scalar: 132 bytes per cell), the r largest per query;
//   pass 2   exact scores from both planes, as in the two-plane kernel; a cluster at or above the cut is a
//            candidate: listed and left out; the softmax over all others, and P V;
//   then     the r best candidates by (score, index) are the selection; the other candidates (a few per query)
//            re-enter the softmax state one by one.
// Against the two-plane kernel pass 1 reads 132 instead of 260 bytes per cell.  A lane's candidate list holds CAP
// entries; a tile where one overflows (many near-equal scores) is flagged and left to the two-plane kernel, which
// runs as a second launch over the flagged tiles only.
// ------------------------------------------------------------------------------------------
template <int D, int RCAP>
__global__ void __launch_bounds__(64) __attribute__((amdgpu_waves_per_eu(D == 64 ? 2 : 1, 2))) k_farfield_fwd_b(
    const bf16_t* __restrict__ Q, const bf16_t* __restrict__ A_kb, const uint16_t* __restrict__ A_km,
    const float* __restrict__ A_c, const bf16_t* __restrict__ A_v, const float* __restrict__ knorm,
    const int32_t* __restrict__ perm_q, const int32_t* __restrict__ off_q, const int32_t* __restrict__ tile_off,
    float* __restrict__ ff_acc, float* __restrict__ ff_ml, int32_t* __restrict__ selc, int32_t* __restrict__ flag,
    int h0, int N, int nb, int Cq, int Ck, int r, int Hq, int Hkv, float scale) {
  constexpr int DT = D / 32, KS = D / 16, CPR = D / 8, NIT = 32 * CPR / 64;
  constexpr int CAP = RCAP + 8;
  __shared__ __attribute__((aligned(16))) bf16_t vt[D][32 + 4];
  __shared__ float cs[64][CAP];   // scores of a lane's candidates
  __shared__ int ci[64][CAP];     // their clusters
  __shared__ int sel_s[32][RCAP];
  const int hl = blockIdx.z, hq = h0 + hl;
  const int hk = (hq / Hq) * Hkv + (hq % Hq) / (Hq / Hkv);
  const int b = blockIdx.y + 1, NBm = nb - 1;
  const int lane = threadIdx.x, col = lane % 32, half = lane / 32;

  const int32_t* to = tile_off + ((size_t)hq * nb + b) * (Cq + 1);
  const int ntl = to[Cq], run = (ntl + 7) / 8;
  const int tile = (blockIdx.x % 8) * run + blockIdx.x / 8;
  if ((int)blockIdx.x / 8 >= run || tile >= ntl) return;
  int32_t* myflag = flag + ((size_t)hl * NBm + (b - 1)) * gridDim.x + blockIdx.x;
  int lo_ = 0, hi_ = Cq;
  while (hi_ - lo_ > 1) {
    int mid = (lo_ + hi_) >> 1;
    if (to[mid] <= tile) lo_ = mid; else hi_ = mid;
  }
  const int i = lo_, tt = tile - to[lo_];
  const int32_t* oq = off_q + (size_t)hq * ((size_t)nb * Cq + 1);
  const int qlo = oq[b * Cq + i], qhi = oq[b * Cq + i + 1];
  int pos = qlo + 32 * tt + col;
  const bool valid = pos < qhi;
  pos = valid ? pos : qlo + 32 * tt;
  const int n = perm_q[(size_t)hq * N + pos];

  // the query itself as the bf16 operand (dims 16 ks + 8 half .. + 7), and its norm
  bf16x8_t qb[KS];
  f16x8_t qh[KS];
  float q2 = 0.f;
  {
    const bf16_t* qrow = Q + ((size_t)hq * N + n) * D;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      qb[ks] = *reinterpret_cast<const bf16x8_t*>(qrow + 16 * ks + 8 * half);
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        qh[ks][e] = (_Float16)(float)qb[ks][e];
        q2 = fmaf((float)qb[ks][e], (float)qb[ks][e], q2);
      }
    }
    q2 += __shfl_xor(q2, 32, 64);
  }
  // 2^-8: half an ulp of bf16; 1.01 and 1e-4 cover the rounding of the fp32 accumulation
  const float eps = 1.01f * scale * 0.00390625f * sqrtf(q2) * knorm[hk] + 1e-4f;
  const size_t acell = (((size_t)hl * NBm + (b - 1)) * Cq + i) * Ck;
  const bf16_t* Av = A_v + acell * D;
  const int ntile = (Ck + 31) / 32;
  using KT = KTileB<D>;
  auto load_kt = [&](KT& kt, int j0) { load_ktile_b<D>(kt, A_c + acell, A_kb + acell * D, j0, Ck, col, half); };
  auto score_kt = [&](const KT& kt, int j0) { return score_ktile_b<D>(kt, j0, Ck, qb, scale, half); };

  // ---- pass 1: the r largest approximate scores seen by this lane half ----
  float list[RCAP];
#pragma unroll
  for (int k = 0; k < RCAP; ++k) list[k] = MUSE_NEG_INF;
  {
    auto insert = [&](const f32x16_t& acc) {
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const float x = acc[e];
#pragma unroll
        for (int k = RCAP - 1; k > 0; --k) list[k] = __builtin_amdgcn_fmed3f(x, list[k - 1], list[k]);
        list[0] = fmaxf(list[0], x);
      }
    };
    KT ka, kb;
    load_kt(ka, 0);
    for (int jt = 0; jt < ntile; jt += 2) {
      if (jt + 1 < ntile) load_kt(kb, (jt + 1) * 32);
      insert(score_kt(ka, jt * 32));
      if (jt + 1 < ntile) {
        if (jt + 2 < ntile) load_kt(ka, (jt + 2) * 32);
        insert(score_kt(kb, (jt + 1) * 32));
      }
    }
  }
  // ---- the cut: the query's r-th largest approximate score, lowered by 2 eps ----
  float cut;
  {
    int quota = 0;
    float other[RCAP];
#pragma unroll
    for (int k = 0; k < RCAP; ++k) other[k] = __shfl_xor(list[k], 32, 64);
#pragma unroll
    for (int k = 0; k < RCAP; ++k) {
      int ahead = 0;
#pragma unroll
      for (int y = 0; y < RCAP; ++y) ahead += half == 0 ? (other[y] > list[k]) : (other[y] >= list[k]);
      quota += (k + ahead < r) && (list[k] > MUSE_NEG_INF);
    }
    float thr = __builtin_huge_valf();
#pragma unroll
    for (int k = 0; k < RCAP; ++k)
      if (k == quota - 1) thr = list[k];
    const int total = quota + __shfl_xor(quota, 32, 64);
    const float thrq = fminf(thr, __shfl_xor(thr, 32, 64));
    // fewer than r clusters with a finite score: every one of them is selected
    // r clusters have an approximate score of thrq or more, so an exact one of thrq - eps or more: the r-th
    // largest exact score is at least that
    cut = total < r ? -3.0e38f : thrq - eps;
  }

  // ---- pass 2: candidates listed and left out, the softmax over the rest, P V ----
  float m = MUSE_NEG_INF, l = 0.f;
  f32x16_t o[DT];
#pragma unroll
  for (int t = 0; t < DT; ++t) o[t] = zero16();
  int ncand = 0;
  bool over = false;
  struct PTile {
    KTileH<D> kt;
    uint4 vch[NIT];
  };
  auto load_ptile = [&](PTile& pt, int j0) {
    load_ktile_h<D>(pt.kt, A_c + acell, A_kb + acell * D, A_km + acell * D, j0, Ck, col, half);
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
      const int c = lane + 64 * it, row = c % 32, cc = c / 32;
      const int jr = j0 + row < Ck ? j0 + row : Ck - 1;
      pt.vch[it] = *reinterpret_cast<const uint4*>(Av + (size_t)jr * D + cc * 8);
    }
  };
  auto process = [&](const PTile& pt, int j0) {
    f32x16_t acc = score_ktile_h<D>(pt.kt, j0, Ck, qb, qh, scale, half);
    float tmax = MUSE_NEG_INF;
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      if (acc[e] >= cut) {
        if (ncand < CAP) {
          cs[lane][ncand] = acc[e];
          ci[lane][ncand] = j0 + 8 * (e / 4) + 4 * half + (e % 4);
          ++ncand;
        } else {
          over = true;
        }
        acc[e] = MUSE_NEG_INF;
      }
      tmax = fmaxf(tmax, acc[e]);
    }
    tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
    float mn = fmaxf(m, tmax);
    float mref = mn == MUSE_NEG_INF ? 0.f : mn;
    float alpha = __expf(m - mref);
    float psum = 0.f;
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      float p = __expf(acc[e] - mref);
      acc[e] = p;
      psum += p;
    }
    l = l * alpha + psum;
    m = mn;
#pragma unroll
    for (int t = 0; t < DT; ++t)
#pragma unroll
      for (int e = 0; e < 16; ++e) o[t][e] *= alpha;
    wave_lds_fence();
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
      const int c = lane + 64 * it, row = c % 32, cc = c / 32;
      const bf16_t* pv = reinterpret_cast<const bf16_t*>(&pt.vch[it]);
#pragma unroll
      for (int e = 0; e < 8; ++e) vt[cc * 8 + e][row] = pv[e];
    }
    wave_lds_fence();
#pragma unroll
    for (int G = 0; G < 2; ++G) {
      const bf16x8_t pf = pack8(acc, 2 * G, 2 * G + 1);
#pragma unroll
      for (int x = 0; x < DT; ++x)
        o[x] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ld_tr8(&vt[32 * x + col][0], 16 * G, half), pf, o[x], 0, 0, 0);
    }
  };
  for (int jt = 0; jt < ntile; ++jt) {
    PTile pt;
    load_ptile(pt, jt * 32);
    process(pt, jt * 32);
  }
  // a list overflowed somewhere in the tile: the two-plane kernel takes the whole tile
  const bool tile_over = __ballot(over) != 0ull;
  if (lane == 0) *myflag = tile_over ? 1 : 0;
  if (tile_over) return;

  for (int k = lane; k < 32 * RCAP; k += 64) (&sel_s[0][0])[k] = -1;
  __syncthreads();
  // ---- rank the query's candidates by (exact score desc, index asc); the r first are the selection ----
  // (the ranks go where the transposed value tile was: pass 2 is over)
  static_assert(sizeof(vt) >= 64 * CAP && 2 * CAP < 256, "the rank table (a byte per candidate) does not fit the value tile");
  unsigned char (*rk)[CAP] = reinterpret_cast<unsigned char (*)[CAP]>(&vt[0][0]);
  const int nother = __shfl_xor(ncand, 32, 64);
  {
    for (int k = 0; k < ncand; ++k) {
      const float sv = cs[lane][k];
      const int iv = ci[lane][k];
      int rank = 0;
      for (int y = 0; y < ncand; ++y) rank += (cs[lane][y] > sv) || (cs[lane][y] == sv && ci[lane][y] < iv);
      for (int y = 0; y < nother; ++y)
        rank += (cs[lane ^ 32][y] > sv) || (cs[lane ^ 32][y] == sv && ci[lane ^ 32][y] < iv);
      rk[lane][k] = (unsigned char)rank;
      if (rank < r) sel_s[col][rank] = iv;
    }
    __syncthreads();
    if (valid && half == 0) {
      const int total = ncand + nother;
      int32_t* out = selc + ((size_t)hq * N + n) * r;
      for (int k = 0; k < r; ++k) out[k] = k < total ? sel_s[col][k] : -1;
    }
  }
  // ---- the candidates that are not selected re-enter the softmax state (both halves of the query take each of
  //      them, in the same order: own list of the lower half first) ----
#pragma unroll
  for (int side = 0; side < 2; ++side) {
    const int src = side == 0 ? col : col + 32;  // the list of the lower half, then of the upper half
    const int cnt = src == lane ? ncand : nother;
    for (int k = 0; k < cnt; ++k) {
      if ((int)rk[src][k] < r) continue;
      const float s = cs[src][k];
      const int j = ci[src][k];
      const float mn = fmaxf(m, s);
      const float alpha = __expf(m - mn), pw = __expf(s - mn);
      l = l * alpha + (src == lane ? pw : 0.f);
      m = mn;
      const bf16_t* vr = Av + (size_t)j * D;
#pragma unroll
      for (int x = 0; x < DT; ++x)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          float v4[4];
          ld4(vr, 32 * x + 8 * g + 4 * half, v4);
#pragma unroll
          for (int u = 0; u < 4; ++u) o[x][4 * g + u] = fmaf(pw, v4[u], o[x][4 * g + u] * alpha);
        }
    }
  }
  l += __shfl_xor(l, 32, 64);
  if (!valid) return;
  float* fa = ff_acc + ((size_t)hq * N + n) * D;
#pragma unroll
  for (int g = 0; g < 4; ++g)
#pragma unroll
    for (int x = 0; x < DT; ++x)
      *reinterpret_cast<float4*>(fa + 32 * x + 8 * g + 4 * half) =
          make_float4(o[x][4 * g], o[x][4 * g + 1], o[x][4 * g + 2], o[x][4 * g + 3]);
  if (half == 0) {
    ff_ml[((size_t)hq * N + n) * 2] = m;
    ff_ml[((size_t)hq * N + n) * 2 + 1] = l;
  }
}

// ------------------------------------------------------------------------------------------
// Per query (blocks >= 1), over its r retrieved clusters: block selection on the per-block summaries
// (scores q~.k-bar + mu-bar of the preceding blocks, the k2 largest are retrieved, ties to the earlier
// block), then component 2 = monopole attention over the per-block summaries of the blocks NOT
// retrieved; fp32 inputs also take component 3 (exact attention over the retrieved pairs) here, bf16
// inputs take it on the matrix cores in the pair kernels.  The result is merged into the query's
// far-field state.  16 lanes per query, a lane owns the dims 64 x + 4 l16 + t; queries are visited in
// bucketed order so that neighbours share the summary rows.
// ------------------------------------------------------------------------------------------
template <typename T, int D, int NBC>
__global__ void __launch_bounds__(256) k_comp2_fwd(
    const T* __restrict__ Q, const float* __restrict__ qc, const T* __restrict__ Ks, const T* __restrict__ Vs,
    const float* __restrict__ L, const float* __restrict__ s_mu, const float* __restrict__ s_k,
    const T* __restrict__ s_v, const int32_t* __restrict__ perm_q, const int32_t* __restrict__ off_k,
    const int32_t* __restrict__ aq, const int32_t* __restrict__ selc, int32_t* __restrict__ selb,
    float* __restrict__ ff_acc, float* __restrict__ ff_ml, int h0, int N, int nb, int Bs, int Cq, int Ck, int r,
    int k2e, int Hq, int Hkv, float scale) {
  constexpr int NG = D / 64;
  const int hl = blockIdx.y, hq = h0 + hl;
  const int hk = (hq / Hq) * Hkv + (hq % Hq) / (Hq / Hkv);
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
  const int b = n / Bs, NBm = nb - 1;
  const int i = aq[qn];
  const int32_t* ok = off_k + (size_t)hk * ((size_t)nb * Ck + 1);
  float qt[NG][4];
#pragma unroll
  for (int x = 0; x < NG; ++x) {
    float q4[4];
    ld4(Q, qn * D + 64 * x + 4 * l16, q4);
    const float4 c4 = *reinterpret_cast<const float4*>(qc + ((size_t)hq * Cq + i) * D + 64 * x + 4 * l16);
    qt[x][0] = scale * (q4[0] - c4.x); qt[x][1] = scale * (q4[1] - c4.y);
    qt[x][2] = scale * (q4[2] - c4.z); qt[x][3] = scale * (q4[3] - c4.w);
  }
  // the four queries of a wave are neighbours in the block-major order: the largest b among them (wave-uniform)
  // bounds the block loops, so a wave of block-1 queries handles one summary row per cluster, not eight
  // (the bound is a template constant of the loop body below: one straight-line body per value, loads batched)
  int bwv = b;
  bwv = max(bwv, __shfl_xor(bwv, 16, 64));
  bwv = max(bwv, __shfl_xor(bwv, 32, 64));
  bwv = __builtin_amdgcn_readfirstlane(bwv);
  float m = MUSE_NEG_INF, l = 0.f, o[NG][4];
#pragma unroll
  for (int x = 0; x < NG; ++x)
#pragma unroll
    for (int t = 0; t < 4; ++t) o[x][t] = 0.f;
  auto add = [&](float lg, const float (&v)[NG][4]) {  // one more (logit, value row) into the running state
    const float mn = fmaxf(m, lg);
    const float a = __expf(m - mn), p = __expf(lg - mn);
    l = l * a + p;
    m = mn;
#pragma unroll
    for (int x = 0; x < NG; ++x)
#pragma unroll
      for (int t = 0; t < 4; ++t) o[x][t] = o[x][t] * a + p * v[x][t];
  };
  // the query's first eight retrieved clusters are read up front: a cluster's rows then wait for one round trip
  int sel8[8];
#pragma unroll
  for (int t = 0; t < 8; ++t) sel8[t] = t < r ? selc[qn * r + t] : -1;
  auto run = [&](auto bw_c) {
  constexpr int bw = decltype(bw_c)::value;
  for (int t = 0; t < r; ++t) {
    int j = -1;
#pragma unroll
    for (int u = 0; u < 8; ++u) j = t == u ? sel8[u] : j;
    if (t >= 8) j = selc[qn * r + t];
    if (j < 0) continue;
    // scores of the preceding blocks, 8 at a time: every load of a chunk is in flight together (with at
    // most 8 preceding blocks the value rows ride along, one round trip per retrieved cluster)
    float sc2[8 * NBC];
#pragma unroll
    for (int bp = 0; bp < 8 * NBC; ++bp) sc2[bp] = MUSE_NEG_INF;
    float vr[8][NG][4];
#pragma unroll
    for (int c0 = 0; c0 < 8 * NBC; c0 += 8) {
      if (c0 >= bw) break;
      float mu[8], part[8];
      float4 kr[8][NG];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        if (c0 + u >= bw) break;
        const int bp = c0 + u < b ? c0 + u : b - 1;
        const size_t cell = (((size_t)hl * NBm + bp) * Cq + i) * Ck + j;
        mu[u] = s_mu[cell];
#pragma unroll
        for (int x = 0; x < NG; ++x) {
          kr[u][x] = *reinterpret_cast<const float4*>(s_k + cell * D + 64 * x + 4 * l16);
          if (NBC == 1) ld4(s_v, cell * D + 64 * x + 4 * l16, vr[u][x]);
        }
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        if (c0 + u >= bw) break;
        float pa = 0.f;
#pragma unroll
        for (int x = 0; x < NG; ++x) {
          pa = fmaf(qt[x][0], kr[u][x].x, pa); pa = fmaf(qt[x][1], kr[u][x].y, pa);
          pa = fmaf(qt[x][2], kr[u][x].z, pa); pa = fmaf(qt[x][3], kr[u][x].w, pa);
        }
        part[u] = pa;
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        if (c0 + u >= bw) break;
        part[u] = group_sum<16>(part[u]);
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        if (c0 + u >= bw) break;
        if (c0 + u < b && mu[u] > MUSE_NEG_INF) sc2[c0 + u] = part[u] + mu[u];
      }
    }
    unsigned selbits = 0;
    for (int u = 0; u < k2e; ++u) {
      float best = MUSE_NEG_INF;
      int bi = -1;
#pragma unroll
      for (int bp = 0; bp < 8 * NBC; ++bp)
        if (!((selbits >> bp) & 1u) && sc2[bp] > best) { best = sc2[bp]; bi = bp; }
      if (bi >= 0) selbits |= 1u << bi;
      if (l16 == 0) selb[(qn * r + t) * k2e + u] = bi;
    }
    // component 2: value summaries of the blocks that are not retrieved
#pragma unroll
    for (int c0 = 0; c0 < 8 * NBC; c0 += 8) {
      if (c0 >= bw) break;
      if (NBC > 1) {
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          if (c0 + u >= bw) break;
          const int bp = c0 + u < b ? c0 + u : b - 1;
          const size_t cell = (((size_t)hl * NBm + bp) * Cq + i) * Ck + j;
#pragma unroll
          for (int x = 0; x < NG; ++x) ld4(s_v, cell * D + 64 * x + 4 * l16, vr[u][x]);
        }
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        if (c0 + u >= bw) break;
        if (!(sc2[c0 + u] > MUSE_NEG_INF) || ((selbits >> (c0 + u)) & 1u)) continue;
        add(sc2[c0 + u], vr[u]);
      }
    }
    if (sizeof(T) == 4) {  // component 3: the keys of the retrieved (cluster, block) pairs, with the full query
      for (int bp = 0; bp < b; ++bp) {
        if (!((selbits >> bp) & 1u)) continue;
        const int klo = ok[bp * Ck + j], khi = ok[bp * Ck + j + 1];
        for (int p_ = klo; p_ < khi; ++p_) {
          const size_t krow = ((size_t)hk * N + p_) * D;
          float pa = 0.f, v[NG][4];
#pragma unroll
          for (int x = 0; x < NG; ++x) {
            float k4[4];
            ld4(Ks, krow + 64 * x + 4 * l16, k4);
            ld4(Vs, krow + 64 * x + 4 * l16, v[x]);
            pa = fmaf(qt[x][0], k4[0], pa); pa = fmaf(qt[x][1], k4[1], pa);
            pa = fmaf(qt[x][2], k4[2], pa); pa = fmaf(qt[x][3], k4[3], pa);
          }
          pa = group_sum<16>(pa);
          add(pa + L[((size_t)hl * Cq + i) * N + p_], v);  // q.k = q~.k + q-bar.k
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
  if (!(l > 0.f)) return;
  // merge into the far-field state left by the tile kernel
  float fm = ff_ml[qn * 2], fl = ff_ml[qn * 2 + 1];
  float fa[NG][4];
#pragma unroll
  for (int x = 0; x < NG; ++x) {
    const float4 a4 = *reinterpret_cast<const float4*>(ff_acc + qn * D + 64 * x + 4 * l16);
    fa[x][0] = a4.x; fa[x][1] = a4.y; fa[x][2] = a4.z; fa[x][3] = a4.w;
  }
  if (!(fl > 0.f)) {
    fm = MUSE_NEG_INF; fl = 0.f;
#pragma unroll
    for (int x = 0; x < NG; ++x)
#pragma unroll
      for (int t = 0; t < 4; ++t) fa[x][t] = 0.f;
  }
  const float mn = fmaxf(fm, m);
  const float ca = __expf(fm - mn), cb = __expf(m - mn);
#pragma unroll
  for (int x = 0; x < NG; ++x)
    *reinterpret_cast<float4*>(ff_acc + qn * D + 64 * x + 4 * l16) =
        make_float4(fa[x][0] * ca + o[x][0] * cb, fa[x][1] * ca + o[x][1] * cb, fa[x][2] * ca + o[x][2] * cb,
                    fa[x][3] * ca + o[x][3] * cb);
  if (l16 == 0) {
    ff_ml[qn * 2] = mn;
    ff_ml[qn * 2 + 1] = fl * ca + l * cb;
  }
}

template <typename T>
int run_fwd_typed(const MuseDims& d, const T* Q, const T* K, const T* V, const float* qc, const int32_t* aq,
                  const int32_t* ak, void* O, float* LSE, int32_t* selc, int32_t* selb, FFWorkspace& w,
                  hipStream_t st);

}  // namespace

// carve the workspace; returns the number of heads per chunk (0 if too small)
int muse_ff_carve(const MuseDims& d, bool bwd, void* ws, size_t ws_bytes, FFWorkspace* w, void* dQ, void* dK,
                  void* dV) {
  size_t HQ = (size_t)d.B * d.Hq, HK = (size_t)d.B * d.Hkv, N = d.N, D = d.D;
  size_t es = d.dtype == MUSE_DTYPE_BF16 ? 2 : 4;
  size_t fixed = ff_fixed_bytes(d, bwd), per = ff_head_bytes(d, bwd);
  int G = d.Hq / d.Hkv;
  if (ws_bytes < fixed + per * G) return 0;
  size_t hc = (ws_bytes - fixed) / per;
  hc = hc > HQ ? HQ : hc;
  hc -= hc % G;
  char* p = (char*)ws;
  auto take = [&](size_t bytes) { char* r = p; p += ff_al(bytes); return r; };
  w->perm_k = (int32_t*)take(HK * N * 4);
  w->off_k = (int32_t*)take(HK * ((size_t)d.nb * d.Ck + 1) * 4);
  w->perm_q = (int32_t*)take(HQ * N * 4);
  w->off_q = (int32_t*)take(HQ * ((size_t)d.nb * d.Cq + 1) * 4);
  w->tile_off = (int32_t*)take(HQ * d.nb * ((size_t)d.Cq + 1) * 4);
  w->Ks = take(HK * N * D * es);
  w->Vs = take(HK * N * D * es);
  w->ff_acc = (float*)take(HQ * N * (D + 2) * 4);
  w->ff_ml = w->ff_acc + HQ * N * D;
  {
    size_t R2 = (size_t)(d.r > 0 ? d.r : 1) * d.k2e;
    w->pairmask = (uint32_t*)take(ff_pairmask_bytes(d));
    w->pair_off = (int32_t*)take(HK * ((size_t)d.nb * d.Ck + 1) * 4);
    w->pair_cnt = (int32_t*)take(HK * ((size_t)d.nb * d.Ck + 1) * 4);
    w->run_off = (int32_t*)take(HK * ((size_t)d.nb * d.Ck + 1) * 4);
    w->run_cap = ff_run_cap(d);
    w->run_map = (int4*)take(HK * w->run_cap * 16);
    w->c3_off = (int32_t*)take(HK * ((size_t)d.nb * d.Ck + 1) * 4);
    w->c3_map = (int2*)take(HK * w->run_cap * 8);
    w->seg_cnt = (int32_t*)take(ff_segcnt_bytes(d));
    w->seg_off = (int32_t*)take(ff_segcnt_bytes(d));
    w->hit_cap = (size_t)(d.Hq / d.Hkv) * N * R2;
    w->hits = (uint2*)take(HQ * N * R2 * 8);
    w->ret_part = (float*)take(HQ * N * R2 * (D + 4) * 4);
  }
  w->knorm = (float*)take(HK * 65 * 4);  // [HK] and the partial maxima [HK][64] behind them
  w->ff_flag = (int32_t*)take(ff_flag_bytes(d));
  if (bwd) {
    size_t W = (d.Ck + 31) / 32;
    w->delta = (float*)take(HQ * N * 4);
    w->selmask = (uint32_t*)take(HQ * N * W * 4);
    w->slotinfo = (int32_t*)take(HQ * N * (size_t)(d.r > 0 ? d.r : 1) * 4);
    w->dKs = (float*)take(HK * N * D * 4);
    w->dVs = (float*)take(HK * N * D * 4);
    w->dQff = (float*)take(HQ * N * D * 4);
    w->qcT = take(HQ * D * (size_t)((d.Cq + 31) / 32 * 32) * 2);
    w->c3_part = nullptr;
    if (es == 2 && d.r > 0 && d.nb > 1) w->c3_part = (float*)take((size_t)(kC3Slices - 1) * HK * N * 2 * D * 4);
    if (d.grad_dtype != MUSE_DTYPE_FP32) {
      w->dQacc = (float*)take(HQ * N * D * 4);
      w->dKacc = (float*)take(HK * N * D * 4);
      w->dVacc = (float*)take(HK * N * D * 4);
    } else {
      w->dQacc = (float*)dQ; w->dKacc = (float*)dK; w->dVacc = (float*)dV;
    }
  }
  w->dip_cov = nullptr; w->dip_cbar = nullptr;
  if (d.dipole) w->dip_cov = (float*)take(HK * (size_t)(d.nb > 1 ? d.nb - 1 : 1) * d.Ck * D * D * 4);
  size_t cells = (size_t)(d.nb > 1 ? d.nb - 1 : 1) * d.Cq * d.Ck;
  w->L = (float*)take(hc * d.Cq * N * 4);
  w->chainmask = (uint32_t*)take(hc * d.Cq * ((d.Ck + 31) / 32) * 4);
  w->chainmaskT = (uint32_t*)take(hc * d.Ck * ((d.Cq + 31) / 32) * 4);
  w->s_mu = (float*)take(hc * cells * 4);
  w->A_mu = (float*)take(hc * cells * 4);
  w->s_k = (float*)take(hc * cells * D * 4);
  w->s_v = take(hc * cells * D * es);
  w->A_v = take(hc * cells * D * es);
  w->A_k = nullptr; w->A_kb = nullptr; w->A_km = nullptr; w->A_c = nullptr;
  if (es == 2) {
    w->A_kb = take(hc * cells * D * 2);
    w->A_km = take(hc * cells * D * 2);
    w->A_c = (float*)take(hc * cells * 4);
  } else {
    w->A_k = (float*)take(hc * cells * D * 4);
  }
  if (bwd) {
    w->g_s_c = (float*)take(hc * cells * 4);
    w->g_A_c = (float*)take(hc * cells * 4);
    w->g_s_k = take(hc * cells * D * es);
    w->g_s_v = take(hc * cells * D * es);
    w->g_A_k = take(hc * cells * D * es);
    w->g_A_v = take(hc * cells * D * es);
  }
  if (d.dipole) w->dip_cbar = (float*)take(hc * (size_t)(d.nb > 1 ? d.nb - 1 : 1) * d.Cq * D * D * 4);
  w->hc = (int)hc;
  return (int)hc;
}

// stages shared by forward and backward: bucketing, bucketed copies, tile schedule
template <typename T>
int muse_ff_prepare(const MuseDims& d, const T* K, const T* V, const int32_t* aq, const int32_t* ak, FFWorkspace& w,
                    hipStream_t st) {
  const int HQ = d.B * d.Hq, HK = d.B * d.Hkv, N = d.N, D = d.D;
  int rc;
  if ((rc = muse_launch_bucket(ak, HK, N, d.Bs, d.Ck, w.perm_k, w.off_k, st))) return rc;
  if ((rc = muse_launch_bucket(aq, HQ, N, d.Bs, d.Cq, w.perm_q, w.off_q, st))) return rc;
  const int CPR = D * (int)sizeof(T) / 16;
  dim3 g((unsigned)(((size_t)N * CPR + 255) / 256), HK);
  { MuseProf prof_("k_gather_rows", st); hipLaunchKernelGGL(k_gather_rows<T>, g, dim3(256), 0, st, K, w.perm_k, (T*)w.Ks, N, D); }
  { MuseProf prof_("k_gather_rows", st); hipLaunchKernelGGL(k_gather_rows<T>, g, dim3(256), 0, st, V, w.perm_k, (T*)w.Vs, N, D); }
  { MuseProf prof_("k_tile_schedule", st); hipLaunchKernelGGL(k_tile_schedule, dim3((HQ * d.nb + 63) / 64), dim3(64), 0, st, w.off_q, w.tile_off, HQ, d.nb, d.Cq); }
  if constexpr (sizeof(T) == 2) {
    MuseProf prof_("k_key_norm_max", st);
    float* part = w.knorm + HK;  // [HK][kNormParts]
    if (D == 64) hipLaunchKernelGGL(k_key_norm_part<64>, dim3(kNormParts, HK), dim3(256), 0, st, (const bf16_t*)K, part, N);
    else hipLaunchKernelGGL(k_key_norm_part<128>, dim3(kNormParts, HK), dim3(256), 0, st, (const bf16_t*)K, part, N);
    hipLaunchKernelGGL(k_key_norm_max, dim3(HK), dim3(64), 0, st, (const float*)part, w.knorm);
  }
  MUSE_LAUNCH_CHECK();
  return MUSE_OK;
}

// summaries of the query heads [h0, h0+hn)
template <typename T>
int muse_ff_summaries(const MuseDims& d, const float* qc, FFWorkspace& w, int h0, int hn, hipStream_t st) {
  const int N = d.N;
  dim3 gl((N + 255) / 256, hn);
  dim3 gs((d.Ck + 7) / 8 * 8, ((d.Cq + 31) / 32) * (d.D / 64), hn);
  if (d.D == 64) {
    if constexpr (sizeof(T) == 2)
      { MuseProf prof_("k_tilt_logits", st); hipLaunchKernelGGL((k_tilt_logits_mx<64>), dim3((N + 127) / 128, hn), dim3(256), 0, st, (const bf16_t*)w.Ks, qc, w.L, h0, N, d.Cq, d.Hq, d.Hkv, d.scale); }
    else
      { MuseProf prof_("k_tilt_logits", st); hipLaunchKernelGGL((k_tilt_logits<T, 64>), gl, dim3(256), 0, st, (const T*)w.Ks, qc, w.L, h0, N, d.Cq, d.Hq, d.Hkv, d.scale); }
    { MuseProf prof_("k_summaries", st); hipLaunchKernelGGL((k_summaries<T, 64>), gs, dim3(64), 0, st, (const T*)w.Ks, (const T*)w.Vs, w.L, w.off_k, w.s_mu,
                       w.A_mu, w.A_k, (T*)w.A_v, (bf16_t*)w.A_kb, (uint16_t*)w.A_km, w.A_c, h0, N, d.nb, d.Cq, d.Ck, d.Hq, d.Hkv); }
  } else {
    if constexpr (sizeof(T) == 2)
      { MuseProf prof_("k_tilt_logits", st); hipLaunchKernelGGL((k_tilt_logits_mx<128>), dim3((N + 127) / 128, hn), dim3(256), 0, st, (const bf16_t*)w.Ks, qc, w.L, h0, N, d.Cq, d.Hq, d.Hkv, d.scale); }
    else
      { MuseProf prof_("k_tilt_logits", st); hipLaunchKernelGGL((k_tilt_logits<T, 128>), gl, dim3(256), 0, st, (const T*)w.Ks, qc, w.L, h0, N, d.Cq, d.Hq, d.Hkv, d.scale); }
    { MuseProf prof_("k_summaries", st); hipLaunchKernelGGL((k_summaries<T, 128>), gs, dim3(64), 0, st, (const T*)w.Ks, (const T*)w.Vs, w.L, w.off_k, w.s_mu,
                       w.A_mu, w.A_k, (T*)w.A_v, (bf16_t*)w.A_kb, (uint16_t*)w.A_km, w.A_c, h0, N, d.nb, d.Cq, d.Ck, d.Hq, d.Hkv); }
  }
  MUSE_LAUNCH_CHECK();
  return MUSE_OK;
}

// per-block summaries of the retrieved chains of the query heads [h0, h0+hn): needs selc of these heads
template <typename T>
int muse_ff_block_summaries(const MuseDims& d, const int32_t* selc, const int32_t* aq, FFWorkspace& w, int h0, int hn,
                            hipStream_t st) {
  if (d.nb <= 1 || d.r <= 0) return MUSE_OK;
  const int W = (d.Ck + 31) / 32;
  int rc;
  if ((rc = muse_launch_fill_i32((int32_t*)w.chainmask, (size_t)hn * d.Cq * W, 0, st))) return rc;
  dim3 gm((unsigned)(((size_t)(d.N - d.Bs) * d.r + 255) / 256), hn);
  { MuseProf prof_("k_chainmask", st); hipLaunchKernelGGL(k_chainmask, gm, dim3(256), 0, st, selc, aq, w.chainmask, h0, d.N, d.Bs, d.r, d.Cq, W); }
  dim3 gs(W, d.Cq, hn);
  if (sizeof(T) == 2) {  // bf16 inputs: key-cluster-major on fp32 MFMA
    const int WT = (d.Cq + 31) / 32;
    { MuseProf prof_("k_chainmask_t", st); hipLaunchKernelGGL(k_chainmask_t, dim3(W, WT, hn), dim3(64), 0, st, w.chainmask, w.chainmaskT, d.Cq, d.Ck, W, WT); }
    dim3 gj((d.Ck + 7) / 8 * 8, (d.nb - 1 + 3) / 4, hn);
    if (d.D == 64)
      { MuseProf prof_("k_block_summaries", st); hipLaunchKernelGGL((k_block_summaries_mx<T, 64>), gj, dim3(256), 0, st, (const T*)w.Ks, (const T*)w.Vs, w.L, w.off_k,
                         w.chainmaskT, w.s_mu, w.s_k, (T*)w.s_v, h0, d.N, d.nb, d.Cq, d.Ck, d.Hq, d.Hkv); }
    else
      { MuseProf prof_("k_block_summaries", st); hipLaunchKernelGGL((k_block_summaries_mx<T, 128>), gj, dim3(256), 0, st, (const T*)w.Ks, (const T*)w.Vs, w.L, w.off_k,
                         w.chainmaskT, w.s_mu, w.s_k, (T*)w.s_v, h0, d.N, d.nb, d.Cq, d.Ck, d.Hq, d.Hkv); }
  } else if (d.D == 64)
    { MuseProf prof_("k_block_summaries", st); hipLaunchKernelGGL((k_block_summaries<T, 64>), gs, dim3(64), 0, st, (const T*)w.Ks, (const T*)w.Vs, w.L, w.off_k,
                       w.chainmask, w.s_mu, w.s_k, (T*)w.s_v, h0, d.N, d.nb, d.Cq, d.Ck, d.Hq, d.Hkv); }
  else
    { MuseProf prof_("k_block_summaries", st); hipLaunchKernelGGL((k_block_summaries<T, 128>), gs, dim3(64), 0, st, (const T*)w.Ks, (const T*)w.Vs, w.L, w.off_k,
                       w.chainmask, w.s_mu, w.s_k, (T*)w.s_v, h0, d.N, d.nb, d.Cq, d.Ck, d.Hq, d.Hkv); }
  MUSE_LAUNCH_CHECK();
  return MUSE_OK;
}
template int muse_ff_block_summaries<float>(const MuseDims&, const int32_t*, const int32_t*, FFWorkspace&, int, int, hipStream_t);
template int muse_ff_block_summaries<bf16_t>(const MuseDims&, const int32_t*, const int32_t*, FFWorkspace&, int, int, hipStream_t);

template int muse_ff_prepare<float>(const MuseDims&, const float*, const float*, const int32_t*, const int32_t*, FFWorkspace&, hipStream_t);
template int muse_ff_prepare<bf16_t>(const MuseDims&, const bf16_t*, const bf16_t*, const int32_t*, const int32_t*, FFWorkspace&, hipStream_t);
template int muse_ff_summaries<float>(const MuseDims&, const float*, FFWorkspace&, int, int, hipStream_t);
template int muse_ff_summaries<bf16_t>(const MuseDims&, const float*, FFWorkspace&, int, int, hipStream_t);

namespace {

template <typename T, int D, int RCAP>
void launch_ff_fwd(const MuseDims& d, const T* Q, const float* qc, FFWorkspace& w, int32_t* selc, int h0, int hn,
                   hipStream_t st) {
  dim3 g((unsigned)ff_tile_grid_x(d), d.nb - 1, hn);
  const int32_t* only_flag = nullptr;
  if constexpr (sizeof(T) == 2) {
    if (d.r > 0) {
      // bf16 inputs: the one-plane kernel first; the two-plane kernel below then takes the tiles it flagged
      { MuseProf prof_("k_farfield_fwd", st); hipLaunchKernelGGL((k_farfield_fwd_b<D, RCAP>), g, dim3(64), 0, st, (const bf16_t*)Q, (const bf16_t*)w.A_kb, (const uint16_t*)w.A_km,
                         w.A_c, (const bf16_t*)w.A_v, w.knorm, w.perm_q, w.off_q, w.tile_off, w.ff_acc, w.ff_ml, selc, w.ff_flag, h0,
                         d.N, d.nb, d.Cq, d.Ck, d.r, d.Hq, d.Hkv, d.scale); }
      only_flag = w.ff_flag;
    }
  }
  { MuseProf prof_(only_flag ? "k_farfield_fwd_rest" : "k_farfield_fwd", st); hipLaunchKernelGGL((k_farfield_fwd<T, D, RCAP>), g, dim3(64), 0, st, Q, qc, w.A_mu, w.A_k, (const bf16_t*)w.A_kb, (const uint16_t*)w.A_km, w.A_c,
                     (const T*)w.A_v, w.perm_q, w.off_q, w.tile_off, w.ff_acc, w.ff_ml, selc, h0, d.N, d.nb, d.Cq, d.Ck, d.r, d.scale, only_flag); }
}

template <typename T, int D>
void launch_ff_fwd_r(const MuseDims& d, const T* Q, const float* qc, const int32_t* aq, FFWorkspace& w, int32_t* selc,
                     int32_t* selb, int h0, int hn, hipStream_t st) {
  if (d.r <= 8) launch_ff_fwd<T, D, 8>(d, Q, qc, w, selc, h0, hn, st);
  else if (d.r <= 16) launch_ff_fwd<T, D, 16>(d, Q, qc, w, selc, h0, hn, st);
  else launch_ff_fwd<T, D, 32>(d, Q, qc, w, selc, h0, hn, st);
  if (d.r > 0) {
    (void)muse_ff_block_summaries<T>(d, selc, aq, w, h0, hn, st);
    dim3 g(((d.N - d.Bs + 15) / 16 + 255) / 256 * 256, hn);  // a multiple of 256 (see the kernel)
    if (d.nb <= 9)
      { MuseProf prof_("k_comp2_fwd", st); hipLaunchKernelGGL((k_comp2_fwd<T, D, 1>), g, dim3(256), 0, st, Q, qc, (const T*)w.Ks, (const T*)w.Vs, w.L, w.s_mu, w.s_k,
                         (const T*)w.s_v, w.perm_q, w.off_k, aq, selc, selb, w.ff_acc, w.ff_ml, h0, d.N, d.nb, d.Bs, d.Cq, d.Ck, d.r,
                         d.k2e, d.Hq, d.Hkv, d.scale); }
    else
      { MuseProf prof_("k_comp2_fwd", st); hipLaunchKernelGGL((k_comp2_fwd<T, D, 2>), g, dim3(256), 0, st, Q, qc, (const T*)w.Ks, (const T*)w.Vs, w.L, w.s_mu, w.s_k,
                         (const T*)w.s_v, w.perm_q, w.off_k, aq, selc, selb, w.ff_acc, w.ff_ml, h0, d.N, d.nb, d.Bs, d.Cq, d.Ck, d.r,
                         d.k2e, d.Hq, d.Hkv, d.scale); }
  }
}

template <typename T>
int run_fwd_typed(const MuseDims& d, const T* Q, const T* K, const T* V, const float* qc, const int32_t* aq,
                  const int32_t* ak, void* O, float* LSE, int32_t* selc, int32_t* selb, FFWorkspace& w,
                  hipStream_t st) {
  const int HQ = d.B * d.Hq;
  int rc;
  if ((rc = muse_ff_prepare<T>(d, K, V, aq, ak, w, st))) return rc;
  if ((rc = muse_launch_fill(w.ff_ml, (size_t)HQ * d.N * 2, 0.f, st))) return rc;
  if (d.nb > 1) {
    if (d.dipole && (rc = muse_dipole_covariances<T>(d, w, st))) return rc;
    for (int h0 = 0; h0 < HQ; h0 += w.hc) {
      int hn = HQ - h0 < w.hc ? HQ - h0 : w.hc;
      if ((rc = muse_ff_summaries<T>(d, qc, w, h0, hn, st))) return rc;
      if (d.D == 64) launch_ff_fwd_r<T, 64>(d, Q, qc, aq, w, selc, selb, h0, hn, st);
      else launch_ff_fwd_r<T, 128>(d, Q, qc, aq, w, selc, selb, h0, hn, st);
      MUSE_LAUNCH_CHECK();
      // App. B: the merged dipole matrices of this chunk's heads, applied to the far-field state of their queries
      if (d.dipole && (rc = muse_dipole_apply<T>(d, Q, qc, aq, w, h0, hn, st))) return rc;
    }
  }
  if (d.nb > 1 && d.r > 0 && sizeof(T) == 2) {
    // exact retrieval (Sec. 3.3): inverse index pair -> queries, one dense MFMA block per retrieved pair
    if ((rc = muse_ff_build_inverse_index(d, selc, selb, w, true, st))) return rc;
    if ((rc = muse_launch_ret_fwd_pairs(d, Q, w.Ks, w.Vs, w.off_k, w.run_off, w.run_map, w.run_cap, w.hits, w.hit_cap, w.ret_part, st))) return rc;
    if ((rc = muse_launch_merge_ret(d, selb, w.ret_part, w.ff_acc, w.ff_ml, st))) return rc;
  }
  return muse_launch_attn_fwd(d, d.Bs, Q, K, V, w.ff_acc, O, LSE, st);
}

}  // namespace

size_t muse_farfield_fixed_bytes(const MuseDims& d, bool bwd) { return ff_fixed_bytes(d, bwd); }
size_t muse_farfield_ws_bytes(const MuseDims& d, bool bwd, int heads) {
  int G = d.Hq / d.Hkv;
  int h = heads < G ? G : heads;
  return ff_head_bytes(d, bwd) * (size_t)h;
}

int muse_run_fwd(const MuseDims& d, const void* Q, const void* K, const void* V, const float* qc, const int32_t* aq,
                 const int32_t* ak, void* O, float* LSE, int32_t* selc, int32_t* selb, void* ws, size_t ws_bytes,
                 hipStream_t st) {
  FFWorkspace w;
  if (!muse_ff_carve(d, d.keep_state, ws, ws_bytes, &w, nullptr, nullptr, nullptr)) return MUSE_ERR_WORKSPACE_TOO_SMALL;
  if (d.keep_state && w.hc < d.B * d.Hq) return MUSE_ERR_WORKSPACE_TOO_SMALL;
  // block-0 queries and r = 0 leave the selection outputs untouched by the tile kernel: pad them
  if (d.r > 0) {
    size_t nq = (size_t)d.B * d.Hq * d.N;
    int rc;
    if ((rc = muse_launch_fill_i32(selc, nq * d.r, -1, st))) return rc;
    if ((rc = muse_launch_fill_i32(selb, nq * d.r * d.k2e, -1, st))) return rc;
  }
  if (d.dtype == MUSE_DTYPE_FP32)
    return run_fwd_typed<float>(d, (const float*)Q, (const float*)K, (const float*)V, qc, aq, ak, O, LSE, selc, selb, w, st);
  return run_fwd_typed<bf16_t>(d, (const bf16_t*)Q, (const bf16_t*)K, (const bf16_t*)V, qc, aq, ak, O, LSE, selc, selb, w, st);
}
