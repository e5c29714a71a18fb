// bf16 causal attention on MFMA (Sec. 3, Eq. 1-2; Sec. 3.3 "Local attention"): keys restricted to
// the query's own spatial block of size Bs (Bs = N gives exact attention).  Forward plus the two
// backward kernels (dQ per query tile, dK/dV per key tile; no atomics).
//
// Tiling for 64-wide waves and v_mfma_f32_32x32x16_bf16:
//   - a wave owns 32 queries (fwd, dQ) or 32 keys (dK/dV) as the N-columns of the MFMA, so every
//     per-row softmax quantity lives in one lane (two lanes: the two halves hold different K-rows);
//   - scores are produced transposed (S^T = K Q^T in fwd/dQ, S = Q K^T in dK/dV) so that their
//     accumulator layout IS the B-operand layout of the following contraction: probabilities go
//     from registers straight back into the matrix cores, never through LDS;
//   - accumulator element e of lane l is row 8*(e/4) + 4*(l/32) + e%4, column l%32; an operand
//     lane holds 8 consecutive k for k-slot-half l/32.  For the second contraction the 8 k-slots of
//     half h over 16 keys are keys {4h..4h+3} and {8+4h..8+4h+3}: a permutation applied to both
//     operands, which a contraction does not see.
#include "ff_common.h"

namespace {

constexpr int BN = 64;  // rows staged in LDS per step
constexpr int TPAD = 4;  // padding of a transposed tile's rows: 34 dwords apart, conflict-free 8-byte operand reads

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

constexpr float kLazyLog2 = 8.f;  // the softmax reference follows the running maximum in steps of more than 2^8

// acc + the sum of the 8 bf16 values of an operand (v_dot2c_f32_bf16 against a pair of ones: two values per
// instruction, where adding the fp32 values takes one each)
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
__device__ __forceinline__ float sum8(const bf16x8_t& v, float acc) {
  const bf16x2_t ones = {(__bf16)1.0f, (__bf16)1.0f};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const bf16x2_t p = {v[2 * i], v[2 * i + 1]};
    acc = __builtin_amdgcn_fdot2_f32_bf16(p, ones, acc, false);
  }
  return acc;
}

// Numbering of the flash kernels' workgroups.  The tiles of 128 rows of one (batch, head, spatial block) group
// stream the same keys and values (forward, dQ) or queries (dK/dV); workgroups go to the 8 XCDs round-robin by
// their linear id, so with a grid of (8 tpg, ceil(groups / 8)) the workgroup (x, y) is on XCD x % 8 and takes
// tile x / 8 of group 8 y + x % 8: a group's tiles run on one XCD, one after the other, and its operand rows
// stay in that XCD's L2 instead of being fetched by all eight.  tpg = tiles per group (a block, or the whole
// sequence when the block size is not a multiple of 128).
struct FlashTile {
  int t, blk, tpg, h, b;  // tile inside the group, block of the group, tiles per group, head, batch
  bool ok;
};
template <int TR = 128>  // rows of a workgroup's tile
__device__ __forceinline__ FlashTile flash_tile(int N, int Bs, int H, int nbatch) {
  FlashTile r;
  const bool al = (Bs % TR) == 0;
  r.tpg = al ? Bs / TR : (N + TR - 1) / TR;
  const int nblk = al ? N / Bs : 1;
  const int g = blockIdx.y * 8 + blockIdx.x % 8;
  r.t = blockIdx.x / 8;
  r.ok = g < nbatch * H * nblk;
  r.blk = g % nblk;
  r.h = (g / nblk) % H;
  r.b = g / nblk / H;
  return r;
}
static dim3 flash_grid(int N, int Bs, int H, int nbatch, int TR = 128) {
  const bool al = (Bs % TR) == 0;
  const int tpg = al ? Bs / TR : (N + TR - 1) / TR, nblk = al ? N / Bs : 1;
  return dim3(8 * tpg, (nbatch * H * nblk + 7) / 8, 1);
}

// Staging of a tile through registers, so that the global loads of the next tile are in flight while the current one is
// consumed: fetch_tile into registers, commit_tile from registers into LDS.  The registers are named members,
// not an array: an array that is passed around and read through pointer casts ends up in memory (the compiler
// parks it in LDS), and the wait for its loads then comes right after they are issued.
struct TileRegs {
  uint4 a, b, c, d;
};
template <int D, int ROWS>
__device__ __forceinline__ uint4 fetch_chunk(const bf16_t* __restrict__ src, int r0, int N, int it) {
  const int c = threadIdx.x + 256 * it;
  int gr = r0 + c % ROWS;
  gr = gr < N ? gr : N - 1;
  return *reinterpret_cast<const uint4*>(src + (size_t)gr * D + (c / ROWS) * 8);
}
template <int D, int ROWS>
__device__ __forceinline__ void fetch_tile(const bf16_t* __restrict__ src, int r0, int N, TileRegs& r) {
  constexpr int NCH = ROWS * (D / 8) / 256;
  static_assert(NCH >= 1 && NCH <= 4, "tile does not fit four chunks per thread");
  r.a = fetch_chunk<D, ROWS>(src, r0, N, 0);
  if constexpr (NCH > 1) r.b = fetch_chunk<D, ROWS>(src, r0, N, 1);
  if constexpr (NCH > 2) r.c = fetch_chunk<D, ROWS>(src, r0, N, 2);
  if constexpr (NCH > 3) r.d = fetch_chunk<D, ROWS>(src, r0, N, 3);
}
template <int D, int ROWS, bool ROWM, bool TRANS>
__device__ __forceinline__ void commit_chunk(const uint4 v, int it, bf16_t (*rm)[D + 8], bf16_t (*tr)[ROWS + TPAD]) {
  const int c = threadIdx.x + 256 * it, row = c % ROWS, cc = c / ROWS;
  if (ROWM) *reinterpret_cast<uint4*>(&rm[row][cc * 8]) = v;
  if (TRANS) {
    tr[cc * 8 + 0][row] = (bf16_t)(v.x & 0xffffu); tr[cc * 8 + 1][row] = (bf16_t)(v.x >> 16);
    tr[cc * 8 + 2][row] = (bf16_t)(v.y & 0xffffu); tr[cc * 8 + 3][row] = (bf16_t)(v.y >> 16);
    tr[cc * 8 + 4][row] = (bf16_t)(v.z & 0xffffu); tr[cc * 8 + 5][row] = (bf16_t)(v.z >> 16);
    tr[cc * 8 + 6][row] = (bf16_t)(v.w & 0xffffu); tr[cc * 8 + 7][row] = (bf16_t)(v.w >> 16);
  }
}
template <int D, int ROWS, bool ROWM, bool TRANS>
__device__ __forceinline__ void commit_tile(const TileRegs& r, bf16_t (*rm)[D + 8], bf16_t (*tr)[ROWS + TPAD]) {
  constexpr int NCH = ROWS * (D / 8) / 256;
  commit_chunk<D, ROWS, ROWM, TRANS>(r.a, 0, rm, tr);
  if constexpr (NCH > 1) commit_chunk<D, ROWS, ROWM, TRANS>(r.b, 1, rm, tr);
  if constexpr (NCH > 2) commit_chunk<D, ROWS, ROWM, TRANS>(r.c, 2, rm, tr);
  if constexpr (NCH > 3) commit_chunk<D, ROWS, ROWM, TRANS>(r.d, 3, rm, tr);
}

// Transposed tile in operand order.  The second contraction of the backward kernels takes, for lane half h and the
// 16 rows r0 .. r0+15 of the staged tile, the rows r0 + {4h .. 4h+3} and r0 + {8+4h .. 8+4h+3} as its 8 k-slots.
// Stored in that order (inside every group of 16 rows the bits 2 and 3 of the row index change places) an operand
// is one 16-byte read instead of two 8-byte ones; an LDS instruction costs about the same whatever its width, and
// LDS instructions, not bytes, are what these kernels run out of.  Rows are padded to a multiple of 16 bytes.
constexpr int TPAD16 = 8;
__device__ __forceinline__ int tr_pos(int row) { return (row & ~12) | ((row & 4) << 1) | ((row & 8) >> 1); }
// rows 2r and 2r+1 (chunk cc of each) into the row-major tile, and their 8 columns into the transposed tile as
// 4-byte stores of two neighbouring rows (they stay neighbours in operand order)
template <int D, int ROWS, bool ROWM = true>
__device__ __forceinline__ void commit_pair(const uint4 a, const uint4 b, int r, int cc, bf16_t (*rm)[D + 8],
                                            bf16_t (*tr)[ROWS + TPAD16]) {
  if constexpr (ROWM) {
    *reinterpret_cast<uint4*>(&rm[2 * r][cc * 8]) = a;
    *reinterpret_cast<uint4*>(&rm[2 * r + 1][cc * 8]) = b;
  }
  const uint32_t wa[4] = {a.x, a.y, a.z, a.w}, wb[4] = {b.x, b.y, b.z, b.w};
  const int pos = tr_pos(2 * r);
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    *reinterpret_cast<uint32_t*>(&tr[cc * 8 + 2 * i][pos]) = __builtin_amdgcn_perm(wb[i], wa[i], 0x05040100u);
    *reinterpret_cast<uint32_t*>(&tr[cc * 8 + 2 * i + 1][pos]) = __builtin_amdgcn_perm(wb[i], wa[i], 0x07060302u);
  }
}
// the operand of lane half `half` over the 16 rows starting at r0 (a multiple of 16)
template <int W>
__device__ __forceinline__ bf16x8_t ld_tr16(const bf16_t (*tr)[W], int d, int r0, int half) {
  return *reinterpret_cast<const bf16x8_t*>(&tr[d][r0 + 8 * half]);
}

// Which row pair and which 16-byte chunk the c-th of a tile's (ROWS / 2) x (D / 8) staging units is: consecutive
// lanes take consecutive pairs of one chunk.  The 4-byte transposed stores of 32 lanes then fall into 32 different
// banks; the 16-byte row stores (lanes 288 bytes apart) pay a two-way conflict, 14 % of their time in a
// microbenchmark, where a mapping that spares them doubles the time of the transposed stores.
template <int D, int ROWS>
__device__ __forceinline__ void pair_unit(int c, int& pr, int& pc) {
  pr = c % (ROWS / 2);
  pc = c / (ROWS / 2);
}
// a whole tile in row pairs, unit c = thread + 256 i, chunk c / (ROWS / 2) for c = thread + 256 i.  Values, not
// references into the register struct, go through the helpers (see TileRegs).
template <int D, int ROWS>
__device__ __forceinline__ uint4 fetch_pair_row(const bf16_t* __restrict__ src, int r0, int N, int i, int which) {
  int pr, pc;
  pair_unit<D, ROWS>(threadIdx.x + 256 * i, pr, pc);
  int row = r0 + 2 * pr + which;
  row = row < N ? row : N - 1;
  return *reinterpret_cast<const uint4*>(src + (size_t)row * D + 8 * pc);
}
template <int D, int ROWS>
__device__ __forceinline__ void fetch_pairs(const bf16_t* __restrict__ src, int r0, int N, TileRegs& r) {
  constexpr int NP = ROWS / 2 * (D / 8) / 256;
  static_assert(NP == 1 || NP == 2, "one or two row pairs per thread");
  r.a = fetch_pair_row<D, ROWS>(src, r0, N, 0, 0);
  r.b = fetch_pair_row<D, ROWS>(src, r0, N, 0, 1);
  if constexpr (NP > 1) {
    r.c = fetch_pair_row<D, ROWS>(src, r0, N, 1, 0);
    r.d = fetch_pair_row<D, ROWS>(src, r0, N, 1, 1);
  }
}
template <int D, int ROWS, bool TRANS, bool ROWM>
__device__ __forceinline__ void commit_pair_i(const uint4 lo, const uint4 hi, int i, bf16_t (*rm)[D + 8],
                                              bf16_t (*tr)[ROWS + TPAD16]) {
  int pr, pc;
  pair_unit<D, ROWS>(threadIdx.x + 256 * i, pr, pc);
  if constexpr (TRANS) {
    commit_pair<D, ROWS, ROWM>(lo, hi, pr, pc, rm, tr);
  } else {
    *reinterpret_cast<uint4*>(&rm[2 * pr][pc * 8]) = lo;
    *reinterpret_cast<uint4*>(&rm[2 * pr + 1][pc * 8]) = hi;
  }
}
template <int D, int ROWS, bool TRANS, bool ROWM = true>
__device__ __forceinline__ void commit_pairs(const TileRegs& r, bf16_t (*rm)[D + 8], bf16_t (*tr)[ROWS + TPAD16]) {
  constexpr int NP = ROWS / 2 * (D / 8) / 256;
  commit_pair_i<D, ROWS, TRANS, ROWM>(r.a, r.b, 0, rm, tr);
  if constexpr (NP > 1) commit_pair_i<D, ROWS, TRANS, ROWM>(r.c, r.d, 1, rm, tr);
}

template <int D>
__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(D == 64 ? 3 : 2, D == 64 ? 3 : 2))) k_flash_fwd(const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K,
                                                    const bf16_t* __restrict__ V, const float* __restrict__ ff,
                                                    bf16_t* __restrict__ O, float* __restrict__ LSE, int N, int Bs,
                                                    int Hq, int Hkv, int nbatch, float scale_log2e) {
  constexpr int KS = D / 16, DT = D / 32;
  __shared__ __attribute__((aligned(16))) bf16_t ks[BN][D + 8];
  __shared__ __attribute__((aligned(16))) bf16_t vt[D][BN + TPAD16];
  const FlashTile ft = flash_tile(N, Bs, Hq, nbatch);
  if (!ft.ok) return;
  const int hq = ft.h, b = ft.b, hk = hq / (Hq / Hkv);
  const size_t qh = ((size_t)b * Hq + hq) * N, kh = ((size_t)b * Hkv + hk) * N;
  const int q0 = (ft.blk * ft.tpg + ft.tpg - 1 - ft.t) * 128;  // long rows first
  const int wave = threadIdx.x / 64, lane = threadIdx.x % 64, col = lane % 32, half = lane / 32;
  const int nq = q0 + 32 * wave + col;
  const int nqc = nq < N ? nq : N - 1;
  const int myb = (nqc / Bs) * Bs;
  const bool unaligned = (Bs % 128) != 0;

  bf16x8_t qf[KS];
#pragma unroll
  for (int s = 0; s < KS; ++s)
    qf[s] = *reinterpret_cast<const bf16x8_t*>(Q + (qh + nqc) * D + 16 * s + 8 * half);
  f32x16_t o[DT];
#pragma unroll
  for (int t = 0; t < DT; ++t)
#pragma unroll
    for (int e = 0; e < 16; ++e) o[t][e] = 0.f;
  float m = MUSE_NEG_INF, mref = 0.f, l = 0.f;

  const int kbeg = (q0 / Bs) * Bs, kend = min(q0 + 128, N);
  TileRegs kreg, vreg;
  fetch_tile<D, BN>(K + kh * D, kbeg, N, kreg);
  fetch_pairs<D, BN>(V + kh * D, kbeg, N, vreg);
  for (int k0 = kbeg; k0 < kend; k0 += BN) {
    __syncthreads();
    commit_tile<D, BN, true, false>(kreg, ks, nullptr);
    commit_pairs<D, BN, true, false>(vreg, nullptr, vt);
    __syncthreads();
    if (k0 + BN < kend) {  // in flight while this tile is consumed
      fetch_tile<D, BN>(K + kh * D, k0 + BN, N, kreg);
      fetch_pairs<D, BN>(V + kh * D, k0 + BN, N, vreg);
    }
    if (k0 > q0 + 32 * wave + 31) continue;  // every key of the tile is in this wave's future
    f32x16_t s[2];
#pragma unroll
    for (int kt = 0; kt < 2; ++kt) {
#pragma unroll
      for (int e = 0; e < 16; ++e) s[kt][e] = 0.f;
#pragma unroll
      for (int x = 0; x < KS; ++x) {
        bf16x8_t a = *reinterpret_cast<const bf16x8_t*>(&ks[32 * kt + col][16 * x + 8 * half]);
        s[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[x], s[kt], 0, 0, 0);
      }
    }
    if (unaligned || k0 + BN - 1 > q0 + 32 * wave || k0 + BN > N) {
#pragma unroll
      for (int kt = 0; kt < 2; ++kt)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          int kg = k0 + 32 * kt + 8 * (e / 4) + 4 * half + (e % 4);
          if (kg > nq || kg < myb) s[kt][e] = MUSE_NEG_INF;
        }
    }
    float tmax = MUSE_NEG_INF;
#pragma unroll
    for (int kt = 0; kt < 2; ++kt)
#pragma unroll
      for (int e = 0; e < 16; ++e) tmax = fmaxf(tmax, s[kt][e]);
    tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
    // The reference m of the running softmax only moves when a tile's maximum exceeds it by more than 2^8:
    // probabilities then stay below 256 (exact in bf16's range, sums in fp32), and the rescaling of the
    // accumulators, a multiply per output element, is skipped on all other tiles (wave-uniform branch).
    // O = o / l and LSE = m + log2 l hold for any reference as long as o, l and p use the same one.
    const float ts = tmax * scale_log2e;
    const bool up = ts > m + kLazyLog2;  // m = -inf: any finite maximum
    if (__builtin_amdgcn_ballot_w64(up) != 0) {
      const float mn = up ? ts : m;
      mref = mn == MUSE_NEG_INF ? 0.f : mn;
      const float alpha = fast_exp2(m - mref);
      l *= alpha;
      m = mn;
#pragma unroll
      for (int t = 0; t < DT; ++t)
#pragma unroll
        for (int e = 0; e < 16; ++e) o[t][e] *= alpha;
    }
    float psum = 0.f;
#pragma unroll
    for (int kt = 0; kt < 2; ++kt)
#pragma unroll
      for (int e = 0; e < 16; ++e) s[kt][e] = fast_exp2(fmaf(s[kt][e], scale_log2e, -mref));
#pragma unroll
    for (int kt = 0; kt < 2; ++kt)
#pragma unroll
      for (int G = 0; G < 2; ++G) {
        bf16x8_t pf = pack8(s[kt], 2 * G, 2 * G + 1);
        psum = sum8(pf, psum);  // the normaliser sums the probabilities as the matrix cores see them
#pragma unroll
        for (int t = 0; t < DT; ++t) {
          bf16x8_t a = ld_tr16(vt, 32 * t + col, 32 * kt + 16 * G, half);
          o[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf, o[t], 0, 0, 0);
        }
      }
    l += psum;
  }
  l += __shfl_xor(l, 32, 64);
  if (nq >= N) return;
  float mnat = m * 0.6931471805599453f;  // natural-log units
  float cl = 1.f;                        // weight of the local part after the merge
  float cf = 0.f, lf = 0.f;
  const float* fa = nullptr;
  if (ff) {
    const float* fm = ff + (size_t)nbatch * Hq * N * D + (qh + nq) * 2;  // [acc | (max,sum)] planes
    float mf = fm[0];
    lf = fm[1];
    if (lf > 0.f) {
      float mx = fmaxf(mnat, mf);
      cl = __expf(mnat - mx);
      cf = __expf(mf - mx);
      mnat = mx;
      fa = ff + (qh + nq) * D;
    }
  }
  float lt = l * cl + lf * cf;
  float inv = 1.f / lt;
#pragma unroll
  for (int t = 0; t < DT; ++t)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      int d = 32 * t + 8 * g + 4 * half;
      float v[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) v[u] = o[t][4 * g + u] * cl;
      if (fa) {
        float4 f = *reinterpret_cast<const float4*>(fa + d);
        v[0] += cf * f.x; v[1] += cf * f.y; v[2] += cf * f.z; v[3] += cf * f.w;
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) v[u] *= inv;
      st4(O, (qh + nq) * D + d, v);
    }
  if (half == 0) LSE[qh + nq] = mnat + __logf(lt);
}

// The forward for D = 64 with TWO query tiles per wave (a workgroup covers 256 queries): every key / value
// operand read from LDS feeds two MFMAs, and a barrier pair covers twice the matrix work.  At D = 64 the
// forward has only 4 D = 256 flop per score against a fixed cost per score in the vector unit, so what is
// spent per score on LDS reads and barriers decides how close the matrix cores get to their peak.
__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) k_flash_fwd2(
    const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K, const bf16_t* __restrict__ V, const float* __restrict__ ff,
    bf16_t* __restrict__ O, float* __restrict__ LSE, int N, int Bs, int Hq, int Hkv, int nbatch, float scale_log2e) {
  constexpr int D = 64, KS = D / 16, DT = D / 32, TR = 256;
  __shared__ __attribute__((aligned(16))) bf16_t ks[BN][D + 8];
  __shared__ __attribute__((aligned(16))) bf16_t vt[D][BN + TPAD16];
  const FlashTile ft = flash_tile<TR>(N, Bs, Hq, nbatch);
  if (!ft.ok) return;
  const int hq = ft.h, b = ft.b, hk = hq / (Hq / Hkv);
  const size_t qh = ((size_t)b * Hq + hq) * N, kh = ((size_t)b * Hkv + hk) * N;
  const int q0 = (ft.blk * ft.tpg + ft.tpg - 1 - ft.t) * TR;  // long rows first
  const int wave = threadIdx.x / 64, lane = threadIdx.x % 64, col = lane % 32, half = lane / 32;
  const int w0 = q0 + 64 * wave;  // first query of this wave; tile a = 0, 1 holds queries w0 + 32 a + col
  const bool unaligned = (Bs % TR) != 0;

  bf16x8_t qf[2][KS];
  int nq[2], myb[2];
#pragma unroll
  for (int a = 0; a < 2; ++a) {
    nq[a] = w0 + 32 * a + col;
    const int nqc = nq[a] < N ? nq[a] : N - 1;
    myb[a] = (nqc / Bs) * Bs;
#pragma unroll
    for (int x = 0; x < KS; ++x)
      qf[a][x] = *reinterpret_cast<const bf16x8_t*>(Q + (qh + nqc) * D + 16 * x + 8 * half);
  }
  f32x16_t o[2][DT];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int t = 0; t < DT; ++t)
#pragma unroll
      for (int e = 0; e < 16; ++e) o[a][t][e] = 0.f;
  float m[2] = {MUSE_NEG_INF, MUSE_NEG_INF}, mref[2] = {0.f, 0.f}, l[2] = {0.f, 0.f};

  const int kbeg = (q0 / Bs) * Bs, kend = min(q0 + TR, N);
  TileRegs kreg, vreg;
  fetch_tile<D, BN>(K + kh * D, kbeg, N, kreg);
  fetch_pairs<D, BN>(V + kh * D, kbeg, N, vreg);
  for (int k0 = kbeg; k0 < kend; k0 += BN) {
    __syncthreads();
    commit_tile<D, BN, true, false>(kreg, ks, nullptr);
    commit_pairs<D, BN, true, false>(vreg, nullptr, vt);
    __syncthreads();
    if (k0 + BN < kend) {  // in flight while this tile is consumed
      fetch_tile<D, BN>(K + kh * D, k0 + BN, N, kreg);
      fetch_pairs<D, BN>(V + kh * D, k0 + BN, N, vreg);
    }
    if (k0 > w0 + 63) continue;  // every key of the tile is in this wave's future
    f32x16_t s[2][2];            // [query tile][key half]
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
      for (int kt = 0; kt < 2; ++kt)
#pragma unroll
        for (int e = 0; e < 16; ++e) s[a][kt][e] = 0.f;
#pragma unroll
    for (int kt = 0; kt < 2; ++kt)
#pragma unroll
      for (int x = 0; x < KS; ++x) {
        const bf16x8_t kf = *reinterpret_cast<const bf16x8_t*>(&ks[32 * kt + col][16 * x + 8 * half]);
        s[0][kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[0][x], s[0][kt], 0, 0, 0);
        s[1][kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[1][x], s[1][kt], 0, 0, 0);
      }
    bf16x8_t pf[2][2][2];  // [query tile][key half][16-key group]
#pragma unroll
    for (int a = 0; a < 2; ++a) {
      if (unaligned || k0 + BN - 1 > w0 + 32 * a || k0 + BN > N) {  // wave-uniform
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
          for (int e = 0; e < 16; ++e) {
            const int kg = k0 + 32 * kt + 8 * (e / 4) + 4 * half + (e % 4);
            if (kg > nq[a] || kg < myb[a]) s[a][kt][e] = MUSE_NEG_INF;
          }
      }
      float tmax = MUSE_NEG_INF;
#pragma unroll
      for (int kt = 0; kt < 2; ++kt)
#pragma unroll
        for (int e = 0; e < 16; ++e) tmax = fmaxf(tmax, s[a][kt][e]);
      tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
      // lazy reference of the running softmax, as in k_flash_fwd
      const float ts = tmax * scale_log2e;
      const bool up = ts > m[a] + kLazyLog2;
      if (__builtin_amdgcn_ballot_w64(up) != 0) {
        const float mn = up ? ts : m[a];
        mref[a] = mn == MUSE_NEG_INF ? 0.f : mn;
        const float alpha = fast_exp2(m[a] - mref[a]);
        l[a] *= alpha;
        m[a] = mn;
#pragma unroll
        for (int t = 0; t < DT; ++t)
#pragma unroll
          for (int e = 0; e < 16; ++e) o[a][t][e] *= alpha;
      }
      float psum = 0.f;
#pragma unroll
      for (int kt = 0; kt < 2; ++kt) {
#pragma unroll
        for (int e = 0; e < 16; ++e) s[a][kt][e] = fast_exp2(fmaf(s[a][kt][e], scale_log2e, -mref[a]));
#pragma unroll
        for (int G = 0; G < 2; ++G) {
          pf[a][kt][G] = pack8(s[a][kt], 2 * G, 2 * G + 1);
          psum = sum8(pf[a][kt][G], psum);  // the normaliser sums the probabilities as the matrix cores see them
        }
      }
      l[a] += psum;
    }
#pragma unroll
    for (int kt = 0; kt < 2; ++kt)
#pragma unroll
      for (int G = 0; G < 2; ++G)
#pragma unroll
        for (int t = 0; t < DT; ++t) {
          const bf16x8_t vf = ld_tr16(vt, 32 * t + col, 32 * kt + 16 * G, half);
          o[0][t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[0][kt][G], o[0][t], 0, 0, 0);
          o[1][t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[1][kt][G], o[1][t], 0, 0, 0);
        }
  }
#pragma unroll
  for (int a = 0; a < 2; ++a) {
    const float lt0 = l[a] + __shfl_xor(l[a], 32, 64);
    if (nq[a] >= N) continue;
    const int n = nq[a];
    float mnat = m[a] * 0.6931471805599453f;  // natural-log units
    float cl = 1.f, cf = 0.f, lf = 0.f;       // weights of the local and the far-field part after the merge
    const float* fa = nullptr;
    if (ff) {
      const float* fm = ff + (size_t)nbatch * Hq * N * D + (qh + n) * 2;  // [acc | (max,sum)] planes
      const float mf = fm[0];
      lf = fm[1];
      if (lf > 0.f) {
        const float mx = fmaxf(mnat, mf);
        cl = __expf(mnat - mx);
        cf = __expf(mf - mx);
        mnat = mx;
        fa = ff + (qh + n) * D;
      }
    }
    const float lt = lt0 * cl + lf * cf;
    const float inv = 1.f / lt;
#pragma unroll
    for (int t = 0; t < DT; ++t)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int d = 32 * t + 8 * g + 4 * half;
        float v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u] = o[a][t][4 * g + u] * cl;
        if (fa) {
          const float4 f = *reinterpret_cast<const float4*>(fa + d);
          v[0] += cf * f.x; v[1] += cf * f.y; v[2] += cf * f.z; v[3] += cf * f.w;
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u] *= inv;
        st4(O, (qh + n) * D + d, v);
      }
    if (half == 0) LSE[qh + n] = mnat + __logf(lt);
  }
}

template <int D>
__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(D == 64 ? 3 : 2, D == 64 ? 3 : 2))) k_flash_bwd_dq(const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K,
                                                       const bf16_t* __restrict__ V, const bf16_t* __restrict__ dO,
                                                       const float* __restrict__ LSE, const float* __restrict__ delta,
                                                       float* __restrict__ dQ, int N, int Bs, int Hq, int Hkv,
                                                       int nbatch, float scale, float scale_log2e) {
  constexpr int KS = D / 16, DT = D / 32;
  __shared__ __attribute__((aligned(16))) bf16_t ks[BN][D + 8];
  __shared__ __attribute__((aligned(16))) bf16_t vs[BN][D + 8];
  __shared__ __attribute__((aligned(16))) bf16_t kt_[D][BN + TPAD16];
  const FlashTile ft = flash_tile(N, Bs, Hq, nbatch);
  if (!ft.ok) return;
  const int hq = ft.h, b = ft.b, hk = hq / (Hq / Hkv);
  const size_t qh = ((size_t)b * Hq + hq) * N, kh = ((size_t)b * Hkv + hk) * N;
  const int q0 = (ft.blk * ft.tpg + ft.tpg - 1 - ft.t) * 128;
  const int wave = threadIdx.x / 64, lane = threadIdx.x % 64, col = lane % 32, half = lane / 32;
  const int nq = q0 + 32 * wave + col;
  const int nqc = nq < N ? nq : N - 1;
  const int myb = (nqc / Bs) * Bs;

  bf16x8_t qf[KS], gf[KS];
#pragma unroll
  for (int s = 0; s < KS; ++s) {
    qf[s] = *reinterpret_cast<const bf16x8_t*>(Q + (qh + nqc) * D + 16 * s + 8 * half);
    gf[s] = *reinterpret_cast<const bf16x8_t*>(dO + (qh + nqc) * D + 16 * s + 8 * half);
  }
  const float lse2 = LSE[qh + nqc] * 1.4426950408889634f, dl = delta[qh + nqc];
  const bool unaligned = (Bs % 128) != 0;
  f32x16_t dq[DT];
#pragma unroll
  for (int t = 0; t < DT; ++t)
#pragma unroll
    for (int e = 0; e < 16; ++e) dq[t][e] = 0.f;

  const int kbeg = (q0 / Bs) * Bs, kend = min(q0 + 128, N);
  TileRegs kreg, vreg;
  fetch_pairs<D, BN>(K + kh * D, kbeg, N, kreg);
  fetch_pairs<D, BN>(V + kh * D, kbeg, N, vreg);
  for (int k0 = kbeg; k0 < kend; k0 += BN) {
    __syncthreads();
    commit_pairs<D, BN, true>(kreg, ks, kt_);
    commit_pairs<D, BN, false>(vreg, vs, nullptr);
    __syncthreads();
    if (k0 + BN < kend) {  // in flight while this tile is consumed
      fetch_pairs<D, BN>(K + kh * D, k0 + BN, N, kreg);
      fetch_pairs<D, BN>(V + kh * D, k0 + BN, N, vreg);
    }
    if (k0 > q0 + 32 * wave + 31) continue;
    const bool edge = unaligned || k0 + BN - 1 > q0 + 32 * wave || k0 + BN > N;
#pragma unroll
    for (int kt = 0; kt < 2; ++kt) {
      f32x16_t s, dp;
#pragma unroll
      for (int e = 0; e < 16; ++e) { s[e] = 0.f; dp[e] = 0.f; }
#pragma unroll
      for (int x = 0; x < KS; ++x) {
        bf16x8_t a = *reinterpret_cast<const bf16x8_t*>(&ks[32 * kt + col][16 * x + 8 * half]);
        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[x], s, 0, 0, 0);
        bf16x8_t av = *reinterpret_cast<const bf16x8_t*>(&vs[32 * kt + col][16 * x + 8 * half]);
        dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, gf[x], dp, 0, 0, 0);
      }
      if (edge) {  // wave-uniform: only tiles on the diagonal or at the sequence end hold masked entries
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          int kg = k0 + 32 * kt + 8 * (e / 4) + 4 * half + (e % 4);
          if (kg > nq || kg < myb) s[e] = MUSE_NEG_INF;  // p = 0
        }
      }
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const float p = fast_exp2(fmaf(s[e], scale_log2e, -lse2));
        s[e] = p * (dp[e] - dl);
      }
#pragma unroll
      for (int G = 0; G < 2; ++G) {
        bf16x8_t df = pack8(s, 2 * G, 2 * G + 1);
#pragma unroll
        for (int t = 0; t < DT; ++t) {
          bf16x8_t a = ld_tr16(kt_, 32 * t + col, 32 * kt + 16 * G, half);
          dq[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, df, dq[t], 0, 0, 0);
        }
      }
    }
  }
  if (nq >= N) return;
#pragma unroll
  for (int t = 0; t < DT; ++t)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      // every query row belongs to exactly one tile: the row is written, not added to
      *reinterpret_cast<float4*>(dQ + (qh + nq) * D + 32 * t + 8 * g + 4 * half) =
          make_float4(scale * dq[t][4 * g + 0], scale * dq[t][4 * g + 1], scale * dq[t][4 * g + 2], scale * dq[t][4 * g + 3]);
    }
}

template <int D>
__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(D == 64 ? 2 : 1, D == 64 ? 2 : 1))) k_flash_bwd_dkv(const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K,
                                                        const bf16_t* __restrict__ V, const bf16_t* __restrict__ dO,
                                                        const float* __restrict__ LSE, const float* __restrict__ delta,
                                                        float* __restrict__ dK, float* __restrict__ dV, int N, int Bs,
                                                        int Hq, int Hkv, int nbatch, float scale, float scale_log2e) {
  constexpr int KS = D / 16, DT = D / 32;
  constexpr int BQ = D == 64 ? 64 : 32;  // queries staged per step (LDS budget)
  __shared__ __attribute__((aligned(16))) bf16_t qs[BQ][D + 8];
  __shared__ __attribute__((aligned(16))) bf16_t gs[BQ][D + 8];
  __shared__ __attribute__((aligned(16))) bf16_t qt_[D][BQ + TPAD16];
  __shared__ __attribute__((aligned(16))) bf16_t gt_[D][BQ + TPAD16];
  __shared__ __attribute__((aligned(16))) float lse_s[BQ];
  __shared__ __attribute__((aligned(16))) float dl_s[BQ];
  const FlashTile ft = flash_tile(N, Bs, Hkv, nbatch);
  if (!ft.ok) return;
  const int hk = ft.h, b = ft.b, G_ = Hq / Hkv;
  const size_t kh = ((size_t)b * Hkv + hk) * N;
  const int k0 = (ft.blk * ft.tpg + ft.t) * 128;  // the first key tiles of a block see the most queries
  const int wave = threadIdx.x / 64, lane = threadIdx.x % 64, col = lane % 32, half = lane / 32;
  const int mk = k0 + 32 * wave + col;
  const int mkc = mk < N ? mk : N - 1;
  const int myend = min((mkc / Bs + 1) * Bs, N);
  const int qend = min((min(k0 + 127, N - 1) / Bs + 1) * Bs, N);

  bf16x8_t kf[KS], vf[KS];
#pragma unroll
  for (int s = 0; s < KS; ++s) {
    kf[s] = *reinterpret_cast<const bf16x8_t*>(K + (kh + mkc) * D + 16 * s + 8 * half);
    vf[s] = *reinterpret_cast<const bf16x8_t*>(V + (kh + mkc) * D + 16 * s + 8 * half);
  }
  f32x16_t dk[DT], dv[DT];
#pragma unroll
  for (int t = 0; t < DT; ++t)
#pragma unroll
    for (int e = 0; e < 16; ++e) { dk[t][e] = 0.f; dv[t][e] = 0.f; }

  for (int g = 0; g < G_; ++g) {
    const size_t qh = ((size_t)b * Hq + (size_t)hk * G_ + g) * N;
    TileRegs qreg, greg;
    float lreg = 0.f, dreg = 0.f;
    auto fetch = [&](int q0) {
      fetch_pairs<D, BQ>(Q + qh * D, q0, N, qreg);
      fetch_pairs<D, BQ>(dO + qh * D, q0, N, greg);
      if (threadIdx.x < BQ) {
        int n = q0 + threadIdx.x;
        n = n < N ? n : N - 1;
        lreg = LSE[qh + n];
        dreg = delta[qh + n];
      }
    };
    if (k0 < qend) fetch(k0);
    for (int q0 = k0; q0 < qend; q0 += BQ) {
      __syncthreads();
      commit_pairs<D, BQ, true>(qreg, qs, qt_);
      commit_pairs<D, BQ, true>(greg, gs, gt_);
      if (threadIdx.x < BQ) {
        lse_s[threadIdx.x] = lreg * 1.4426950408889634f;
        dl_s[threadIdx.x] = dreg;
      }
      __syncthreads();
      if (q0 + BQ < qend) fetch(q0 + BQ);  // in flight while this tile is consumed
      if (q0 + BQ - 1 < k0 + 32 * wave) continue;  // every query of the tile precedes this wave's keys
#pragma unroll
      for (int qt = 0; qt < BQ / 32; ++qt) {
        f32x16_t s, dp;
#pragma unroll
        for (int e = 0; e < 16; ++e) { s[e] = 0.f; dp[e] = 0.f; }
#pragma unroll
        for (int x = 0; x < KS; ++x) {
          bf16x8_t a = *reinterpret_cast<const bf16x8_t*>(&qs[32 * qt + col][16 * x + 8 * half]);
          s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, kf[x], s, 0, 0, 0);
          bf16x8_t ag = *reinterpret_cast<const bf16x8_t*>(&gs[32 * qt + col][16 * x + 8 * half]);
          dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ag, vf[x], dp, 0, 0, 0);
        }
        f32x16_t pr;
#pragma unroll
        for (int gq = 0; gq < 4; ++gq) {
          float4 l4 = *reinterpret_cast<const float4*>(&lse_s[32 * qt + 8 * gq + 4 * half]);
          float4 d4 = *reinterpret_cast<const float4*>(&dl_s[32 * qt + 8 * gq + 4 * half]);
          float lv[4] = {l4.x, l4.y, l4.z, l4.w}, dv4[4] = {d4.x, d4.y, d4.z, d4.w};
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            int e = 4 * gq + u;
            float p = fast_exp2(fmaf(s[e], scale_log2e, -lv[u]));
            {
              int n = q0 + 32 * qt + 8 * gq + 4 * half + u;
              p = (n < mk || n >= myend) ? 0.f : p;
            }
            pr[e] = p;
            s[e] = p * (dp[e] - dv4[u]);
          }
        }
#pragma unroll
        for (int G = 0; G < 2; ++G) {
          bf16x8_t pf = pack8(pr, 2 * G, 2 * G + 1);
          bf16x8_t df = pack8(s, 2 * G, 2 * G + 1);
#pragma unroll
          for (int t = 0; t < DT; ++t) {
            bf16x8_t ag = ld_tr16(gt_, 32 * t + col, 32 * qt + 16 * G, half);
            dv[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ag, pf, dv[t], 0, 0, 0);
            bf16x8_t aq = ld_tr16(qt_, 32 * t + col, 32 * qt + 16 * G, half);
            dk[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(aq, df, dk[t], 0, 0, 0);
          }
        }
      }
    }
  }
  if (mk >= N) return;
#pragma unroll
  for (int t = 0; t < DT; ++t)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      // every key row belongs to exactly one tile (the query heads of the group are summed in registers)
      size_t o = (kh + mk) * D + 32 * t + 8 * g + 4 * half;
      *reinterpret_cast<float4*>(dK + o) =
          make_float4(scale * dk[t][4 * g + 0], scale * dk[t][4 * g + 1], scale * dk[t][4 * g + 2], scale * dk[t][4 * g + 3]);
      *reinterpret_cast<float4*>(dV + o) = make_float4(dv[t][4 * g + 0], dv[t][4 * g + 1], dv[t][4 * g + 2], dv[t][4 * g + 3]);
    }
}

// dK/dV of the block diagonal for D = 64, arranged in phases so that a wave never waits for LDS right before a
// matrix instruction, and with the fewest vector instructions per score.  For a tile of 32 queries:
//   A  8 MFMAs   S = Q K^T and dP = dO V^T.  Their accumulators start at -LSE / scale and -delta (read from LDS
//                straight into the accumulator registers), so the probability is exp2(c S) and dS = P dP with no
//                further subtraction;
//   B  vector    P, dS, conversion to bf16 operands; the causal mask only on the tiles the diagonal crosses;
//   C  8 MFMAs   dV += P^T dO, dK += dS^T Q.
// The transposed operands of C are requested before B, the accumulator seeds and row operands of the next tile
// during C, so each request is in flight across a whole phase.  Two staged tiles of 64 queries: while one is
// consumed the next is written into the other (in the middle of the tile, when its global loads have landed) and
// the one after that is requested from memory, so a tile costs one barrier.  With two waves per SIMD the vector
// phase of one wave runs beside the matrix phases of the other.
template <int D>
__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) k_flash_bwd_dkv_p(
    const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K, const bf16_t* __restrict__ V,
    const bf16_t* __restrict__ dO, const float* __restrict__ LSE, const float* __restrict__ delta,
    float* __restrict__ dK, float* __restrict__ dV, int N, int Bs, int Hq, int Hkv, int nbatch, float scale,
    float scale_log2e) {
  constexpr int KS = D / 16, DT = D / 32;
  constexpr int BQ = 64, NQT = BQ / 32;
  __shared__ __attribute__((aligned(16))) bf16_t qs[2][BQ][D + 8];
  __shared__ __attribute__((aligned(16))) bf16_t gs[2][BQ][D + 8];
  __shared__ __attribute__((aligned(16))) bf16_t qt_[2][D][BQ + TPAD16];
  __shared__ __attribute__((aligned(16))) bf16_t gt_[2][D][BQ + TPAD16];
  __shared__ __attribute__((aligned(16))) float lse_s[2][BQ];  // -LSE / scale
  __shared__ __attribute__((aligned(16))) float dl_s[2][BQ];   // -delta
  const FlashTile ft = flash_tile(N, Bs, Hkv, nbatch);
  if (!ft.ok) return;
  const int hk = ft.h, b = ft.b, G_ = Hq / Hkv;
  const size_t kh = ((size_t)b * Hkv + hk) * N;
  const int k0 = (ft.blk * ft.tpg + ft.t) * 128;
  const int wave = threadIdx.x / 64, lane = threadIdx.x % 64, col = lane % 32, half = lane / 32;
  const int mk = k0 + 32 * wave + col;
  const int mkc = mk < N ? mk : N - 1;
  const int myend = min((mkc / Bs + 1) * Bs, N);
  const int qend = min((min(k0 + 127, N - 1) / Bs + 1) * Bs, N);
  // a tile of 128 keys inside one block with every row in range: only the diagonal needs a mask
  const bool aligned = (Bs % 128) == 0 && k0 + 128 <= N;
  const float seed = -1.4426950408889634f / scale_log2e;
  static_assert(BQ / 2 * (D / 8) == 256, "one pair of rows and one 16-byte chunk per thread");
  int pr_, pc_;  // row pair and chunk this thread stages
  pair_unit<D, BQ>(threadIdx.x, pr_, pc_);

  bf16x8_t kf[KS], vf[KS];
#pragma unroll
  for (int s = 0; s < KS; ++s) {
    kf[s] = *reinterpret_cast<const bf16x8_t*>(K + (kh + mkc) * D + 16 * s + 8 * half);
    vf[s] = *reinterpret_cast<const bf16x8_t*>(V + (kh + mkc) * D + 16 * s + 8 * half);
  }
  f32x16_t dk[DT], dv[DT];
#pragma unroll
  for (int t = 0; t < DT; ++t)
#pragma unroll
    for (int e = 0; e < 16; ++e) { dk[t][e] = 0.f; dv[t][e] = 0.f; }

  int cur = 0;  // the staged tile being consumed; the other one is written meanwhile: one barrier per tile
  for (int g = 0; g < G_; ++g) {
    const size_t qh = ((size_t)b * Hq + (size_t)hk * G_ + g) * N;
    uint4 qa, qb, ga, gb;  // rows 2r and 2r+1 of a coming tile, chunk cc, of Q and dO
    float lreg = 0.f, dreg = 0.f;
    auto fetch = [&](int q0) {
      int r0 = q0 + 2 * pr_, r1 = r0 + 1;
      r0 = r0 < N ? r0 : N - 1;
      r1 = r1 < N ? r1 : N - 1;
      qa = *reinterpret_cast<const uint4*>(Q + (qh + r0) * D + 8 * pc_);
      qb = *reinterpret_cast<const uint4*>(Q + (qh + r1) * D + 8 * pc_);
      ga = *reinterpret_cast<const uint4*>(dO + (qh + r0) * D + 8 * pc_);
      gb = *reinterpret_cast<const uint4*>(dO + (qh + r1) * D + 8 * pc_);
      if (threadIdx.x < BQ) {
        int n = q0 + threadIdx.x;
        n = n < N ? n : N - 1;
        lreg = LSE[qh + n];
        dreg = delta[qh + n];
      }
    };
    auto commit = [&](int buf) {
      commit_pair<D, BQ>(qa, qb, pr_, pc_, qs[buf], qt_[buf]);
      commit_pair<D, BQ>(ga, gb, pr_, pc_, gs[buf], gt_[buf]);
      if (threadIdx.x < BQ) {
        lse_s[buf][threadIdx.x] = lreg * seed;
        dl_s[buf][threadIdx.x] = -dreg;
      }
    };
    if (k0 < qend) {
      fetch(k0);
      commit(cur);  // every wave is past the barrier that ended the last tile of the previous head
      __syncthreads();
      if (k0 + BQ < qend) fetch(k0 + BQ);
    }
    for (int q0 = k0; q0 < qend; q0 += BQ) {
      const bool skip = q0 + BQ - 1 < k0 + 32 * wave;  // every query of the tile precedes this wave's keys
      bf16_t (*qsc)[D + 8] = qs[cur];
      bf16_t (*gsc)[D + 8] = gs[cur];
      bf16_t (*qtc)[BQ + TPAD16] = qt_[cur];
      bf16_t (*gtc)[BQ + TPAD16] = gt_[cur];
      const float* lsc = lse_s[cur];
      const float* dlc = dl_s[cur];
      f32x16_t s, dp;
      bf16x8_t aq[KS], ag[KS];
      auto seed_acc = [&](int qt) {
#pragma unroll
        for (int gq = 0; gq < 4; ++gq) {
          const float4 l4 = *reinterpret_cast<const float4*>(&lsc[32 * qt + 8 * gq + 4 * half]);
          const float4 d4 = *reinterpret_cast<const float4*>(&dlc[32 * qt + 8 * gq + 4 * half]);
          s[4 * gq + 0] = l4.x; s[4 * gq + 1] = l4.y; s[4 * gq + 2] = l4.z; s[4 * gq + 3] = l4.w;
          dp[4 * gq + 0] = d4.x; dp[4 * gq + 1] = d4.y; dp[4 * gq + 2] = d4.z; dp[4 * gq + 3] = d4.w;
        }
      };
      auto load_rows = [&](int qt, int part) {  // half of the row operands of a tile
#pragma unroll
        for (int x = part * (KS / 2); x < (part + 1) * (KS / 2); ++x) {
          aq[x] = *reinterpret_cast<const bf16x8_t*>(&qsc[32 * qt + col][16 * x + 8 * half]);
          ag[x] = *reinterpret_cast<const bf16x8_t*>(&gsc[32 * qt + col][16 * x + 8 * half]);
        }
      };
      auto tile = [&](int qt) {
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int x = 0; x < KS; ++x) {
          s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(aq[x], kf[x], s, 0, 0, 0);
          dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ag[x], vf[x], dp, 0, 0, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
        bf16x8_t tq[2][DT], tg[2][DT];
#pragma unroll
        for (int G = 0; G < 2; ++G)
#pragma unroll
          for (int t = 0; t < DT; ++t) {
            tg[G][t] = ld_tr16(gtc, 32 * t + col, 32 * qt + 16 * G, half);
            tq[G][t] = ld_tr16(qtc, 32 * t + col, 32 * qt + 16 * G, half);
          }
        __builtin_amdgcn_sched_barrier(0);
        if (aligned && q0 + 32 * qt >= k0 + 32 * wave + 32) {
#pragma unroll
          for (int e = 0; e < 16; ++e) {
            const float p = fast_exp2(s[e] * scale_log2e);
            s[e] = p;
            dp[e] = p * dp[e];
          }
        } else {
#pragma unroll
          for (int e = 0; e < 16; ++e) {
            const int n = q0 + 32 * qt + 8 * (e / 4) + 4 * half + e % 4;
            float p = fast_exp2(s[e] * scale_log2e);
            p = (n < mk || n >= myend) ? 0.f : p;
            s[e] = p;
            dp[e] = p * dp[e];
          }
        }
        bf16x8_t pf[2], df[2];
#pragma unroll
        for (int G = 0; G < 2; ++G) {
          pf[G] = pack8(s, 2 * G, 2 * G + 1);
          df[G] = pack8(dp, 2 * G, 2 * G + 1);
        }
        if (qt + 1 < NQT) seed_acc(qt + 1);
#pragma unroll
        for (int G = 0; G < 2; ++G) {
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int t = 0; t < DT; ++t) {
            dv[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(tg[G][t], pf[G], dv[t], 0, 0, 0);
            dk[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(tq[G][t], df[G], dk[t], 0, 0, 0);
          }
          __builtin_amdgcn_sched_barrier(0);
          if (qt + 1 < NQT) load_rows(qt + 1, G);  // the operands just consumed leave room for these
        }
      };
      if (!skip) {
        seed_acc(0);
        load_rows(0, 0);
        load_rows(0, 1);
        tile(0);
      }
      if (q0 + BQ < qend) {  // the next tile into the other buffer, the one after it into the registers
        commit(cur ^ 1);
        if (q0 + 2 * BQ < qend) fetch(q0 + 2 * BQ);
      }
      if (!skip) tile(1);
      __syncthreads();
      cur ^= 1;
    }
  }
  if (mk >= N) return;
#pragma unroll
  for (int t = 0; t < DT; ++t)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      size_t o = (kh + mk) * D + 32 * t + 8 * g + 4 * half;
      *reinterpret_cast<float4*>(dK + o) =
          make_float4(scale * dk[t][4 * g + 0], scale * dk[t][4 * g + 1], scale * dk[t][4 * g + 2], scale * dk[t][4 * g + 3]);
      *reinterpret_cast<float4*>(dV + o) = make_float4(dv[t][4 * g + 0], dv[t][4 * g + 1], dv[t][4 * g + 2], dv[t][4 * g + 3]);
    }
}

// ------------------------------------------------------------------------------------------
// Retrieval backward (Sec. 3.3 "Exact retrieval", gradient w.r.t. keys and values): one wave per
// retrieved (key cluster, key block) pair.  `hits` lists the queries that retrieved the pair (the
// inverse index: pair -> queries); they are gathered 32 at a time into LDS and the pair is treated as a
// dense attention-backward block on the matrix cores, the keys of the pair being the MFMA columns.
//   hit = n | g << 22  (query position, query head inside the KV group)
// A pair with many hits (at the operating ratio of Sec. 3.3 a pair has some 500, with a heavy tail) is shared by
// up to kC3Slices waves: slice s of S takes the hit tiles s, s + S, ...; slice 0 adds to the bucketed-order gradient
// rows of the pair's keys, the others write partial rows, which k_c3_reduce adds in slice order (fixed order, no
// atomics).  S depends on the pair's hit count only.
// ------------------------------------------------------------------------------------------

template <int D>
__global__ void __launch_bounds__(64) __attribute__((amdgpu_waves_per_eu(D == 64 ? 2 : 1, D == 64 ? 2 : 1))) k_c3_pairs(const bf16_t* __restrict__ Q, const bf16_t* __restrict__ dO,
                                                  const bf16_t* __restrict__ Ks, const bf16_t* __restrict__ Vs,
                                                  const float* __restrict__ LSE, const float* __restrict__ delta,
                                                  const int32_t* __restrict__ off_k, const int32_t* __restrict__ pair_off,
                                                  const int32_t* __restrict__ c3_off, const int2* __restrict__ c3_map,
                                                  const uint2* __restrict__ hits, float* __restrict__ dKs,
                                                  float* __restrict__ dVs, float* __restrict__ part, size_t run_cap,
                                                  size_t hit_cap, int N, int nb, int Ck, int Hq, int Hkv, int HK,
                                                  float scale, float scale_log2e) {
  constexpr int KS = D / 16, DT = D / 32;
  __shared__ __attribute__((aligned(16))) bf16_t qt_[D][32 + TPAD];
  __shared__ __attribute__((aligned(16))) bf16_t gt_[D][32 + TPAD];
  __shared__ __attribute__((aligned(16))) float lse_s[32];
  __shared__ __attribute__((aligned(16))) float dl_s[32];
  // one wave per work item (pair, hit slice): only the slices a pair has are launched
  const int hk = blockIdx.y, NBm = nb - 1;
  if ((int)blockIdx.x >= c3_off[(size_t)hk * ((size_t)NBm * Ck + 1) + (size_t)NBm * Ck]) return;  // past the last item
  const int2 item = c3_map[(size_t)hk * run_cap + blockIdx.x];  // (pair, slice)
  const int sl = item.y;
  const int G_ = Hq / Hkv;
  const size_t hqbase = (size_t)(hk / Hkv) * Hq + (size_t)(hk % Hkv) * G_;
  const int lane = threadIdx.x, col = lane % 32, half = lane / 32;
  const int32_t* ok = off_k + (size_t)hk * ((size_t)nb * Ck + 1);
  const int klo = ok[item.x], khi = ok[item.x + 1];  // pair = b' Ck + j indexes the segment table directly
  const int32_t* po = pair_off + (size_t)hk * ((size_t)NBm * Ck + 1) + item.x;
  const int hlo = po[0], hhi = po[1];
  if (klo == khi || hlo == hhi) return;
  const int S = c3_slices(hhi - hlo);
  if (sl >= S) return;
  const int step = 32 * S, hfirst = hlo + 32 * sl;  // this slice's hit tiles start at hfirst, hfirst + step, ...
  if (hfirst >= hhi) return;
  const uint2* hh = hits + (size_t)hk * hit_cap;
  for (int k0 = klo; k0 < khi; k0 += 32) {
    const int mk = k0 + col;
    const bool kvalid = mk < khi;
    const size_t krow = ((size_t)hk * N + (kvalid ? mk : klo)) * D;
    bf16x8_t kf[KS], vf[KS];
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      kf[s] = *reinterpret_cast<const bf16x8_t*>(Ks + krow + 16 * s + 8 * half);
      vf[s] = *reinterpret_cast<const bf16x8_t*>(Vs + krow + 16 * s + 8 * half);
    }
    f32x16_t dk[DT], dv[DT];
#pragma unroll
    for (int t = 0; t < DT; ++t)
#pragma unroll
      for (int e = 0; e < 16; ++e) { dk[t][e] = 0.f; dv[t][e] = 0.f; }
    // A tile of 32 hits: the hit of row `col` (one coalesced load of the list), that query's q and dO rows as
    // this lane's half of every 16 dims (the A operands of the score contractions as they are, and the source
    // of the transposed LDS tiles), its LSE and delta.  The next tile is gathered while this one is used; a
    // tile index past the end repeats the last hit, the values stay raw until they are used.
    constexpr int NIT = KS;
    struct HT {
      uint4 q[NIT], g[NIT];
      float lse, dl;
    };
    auto gather = [&](HT& t, int h0) {
      const int hi = h0 + col < hhi ? h0 + col : hhi - 1;
      const uint32_t hit = hh[hi].x;
      const size_t qn = (hqbase + (hit >> 22)) * N + (hit & 0x3fffffu);
#pragma unroll
      for (int it = 0; it < NIT; ++it) {
        t.q[it] = *reinterpret_cast<const uint4*>(Q + qn * D + 16 * it + 8 * half);
        t.g[it] = *reinterpret_cast<const uint4*>(dO + qn * D + 16 * it + 8 * half);
      }
      t.lse = LSE[qn];
      t.dl = delta[qn];
    };
    auto use = [&](const HT& t, int h0) {
      wave_lds_fence();
#pragma unroll
      for (int it = 0; it < NIT; ++it) {  // lanes run along the rows: conflict-free transposed stores
        const uint32_t wq[4] = {t.q[it].x, t.q[it].y, t.q[it].z, t.q[it].w};
        const uint32_t wg[4] = {t.g[it].x, t.g[it].y, t.g[it].z, t.g[it].w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          qt_[16 * it + 8 * half + 2 * e][col] = (bf16_t)(wq[e] & 0xffffu);
          qt_[16 * it + 8 * half + 2 * e + 1][col] = (bf16_t)(wq[e] >> 16);
          gt_[16 * it + 8 * half + 2 * e][col] = (bf16_t)(wg[e] & 0xffffu);
          gt_[16 * it + 8 * half + 2 * e + 1][col] = (bf16_t)(wg[e] >> 16);
        }
      }
      if (half == 0) {
        lse_s[col] = h0 + col < hhi ? t.lse * 1.4426950408889634f : __builtin_huge_valf();  // +inf -> p = 0
        dl_s[col] = t.dl;
      }
      wave_lds_fence();
      f32x16_t s, dp;
#pragma unroll
      for (int e = 0; e < 16; ++e) { s[e] = 0.f; dp[e] = 0.f; }
#pragma unroll
      for (int x = 0; x < KS; ++x) {
        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, t.q[x]), kf[x], s, 0, 0, 0);
        dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, t.g[x]), vf[x], dp, 0, 0, 0);
      }
      f32x16_t pr;
#pragma unroll
      for (int gq = 0; gq < 4; ++gq) {
        float4 l4 = *reinterpret_cast<const float4*>(&lse_s[8 * gq + 4 * half]);
        float4 d4 = *reinterpret_cast<const float4*>(&dl_s[8 * gq + 4 * half]);
        float lv[4] = {l4.x, l4.y, l4.z, l4.w}, dv4[4] = {d4.x, d4.y, d4.z, d4.w};
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const int e = 4 * gq + u;
          float p = fast_exp2(fmaf(s[e], scale_log2e, -lv[u]));
          p = kvalid ? p : 0.f;
          pr[e] = p;
          s[e] = p * (dp[e] - dv4[u]);
        }
      }
#pragma unroll
      for (int G = 0; G < 2; ++G) {
        bf16x8_t pf = pack8(pr, 2 * G, 2 * G + 1);
        bf16x8_t df = pack8(s, 2 * G, 2 * G + 1);
#pragma unroll
        for (int t = 0; t < DT; ++t) {
          bf16x8_t ag = ld_tr8(&gt_[32 * t + col][0], 16 * G, half);
          dv[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ag, pf, dv[t], 0, 0, 0);
          bf16x8_t aq = ld_tr8(&qt_[32 * t + col][0], 16 * G, half);
          dk[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(aq, df, dk[t], 0, 0, 0);
        }
      }
    };
    if constexpr (D == 64) {
      HT ta, tb;
      gather(ta, hfirst);
      for (int h0 = hfirst; h0 < hhi; h0 += 2 * step) {
        gather(tb, h0 + step);
        use(ta, h0);
        if (h0 + step < hhi) {
          gather(ta, h0 + 2 * step);
          use(tb, h0 + step);
        }
      }
    } else {  // two buffers do not fit the registers at D = 128
      for (int h0 = hfirst; h0 < hhi; h0 += step) {
        HT ta;
        gather(ta, h0);
        use(ta, h0);
      }
    }
    if (kvalid) {
      // slice 0 owns the gradient rows; a later slice leaves its share in its own partial rows [dK | dV]
      float* pk = sl == 0 ? dKs + ((size_t)hk * N + mk) * D : part + ((((size_t)(sl - 1) * HK + hk) * N + mk) * 2) * D;
      float* pv = sl == 0 ? dVs + ((size_t)hk * N + mk) * D : pk + D;
#pragma unroll
      for (int t = 0; t < DT; ++t)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int o = 32 * t + 8 * g + 4 * half;
          float4 a = make_float4(0.f, 0.f, 0.f, 0.f), c = a;
          if (sl == 0) { a = *reinterpret_cast<float4*>(pk + o); c = *reinterpret_cast<float4*>(pv + o); }
          a.x += scale * dk[t][4 * g + 0]; a.y += scale * dk[t][4 * g + 1];
          a.z += scale * dk[t][4 * g + 2]; a.w += scale * dk[t][4 * g + 3];
          c.x += dv[t][4 * g + 0]; c.y += dv[t][4 * g + 1]; c.z += dv[t][4 * g + 2]; c.w += dv[t][4 * g + 3];
          *reinterpret_cast<float4*>(pk + o) = a;
          *reinterpret_cast<float4*>(pv + o) = c;
        }
    }
  }
}

// adds the partial rows of the hit slices 1 .. S-1 of every pair to the rows slice 0 owns, in slice order: one wave per
// (key cluster, key block, kv head), 16 lanes per key row
template <int D>
__global__ void __launch_bounds__(64) k_c3_reduce(const int32_t* __restrict__ off_k, const int32_t* __restrict__ pair_off,
                                                   const int32_t* __restrict__ c3_off, const int2* __restrict__ c3_map,
                                                   const float* __restrict__ part, float* __restrict__ dKs,
                                                   float* __restrict__ dVs, size_t run_cap, int N, int nb, int Ck, int HK) {
  // walks the same item list as k_c3_pairs: the item (pair, slice 1) exists exactly for the pairs with partial rows
  const int hk = blockIdx.y, NBm = nb - 1;
  if ((int)blockIdx.x >= c3_off[(size_t)hk * ((size_t)NBm * Ck + 1) + (size_t)NBm * Ck]) return;
  const int2 item = c3_map[(size_t)hk * run_cap + blockIdx.x];
  if (item.y != 1) return;
  const int32_t* po = pair_off + (size_t)hk * ((size_t)NBm * Ck + 1) + item.x;
  const int S = c3_slices(po[1] - po[0]);
  const int32_t* ok = off_k + (size_t)hk * ((size_t)nb * Ck + 1);
  const int klo = ok[item.x], khi = ok[item.x + 1];
  const int lane = threadIdx.x, sub = lane / 16, l16 = lane % 16;
  for (int m = klo + sub; m < khi; m += 4)
    for (int d = 4 * l16; d < 2 * D; d += 64) {  // the row pair [dK | dV] as 2 D floats
      float* dst = (d < D ? dKs : dVs - D) + ((size_t)hk * N + m) * D + d;
      float4 a = *reinterpret_cast<float4*>(dst);
      for (int s = 1; s < S; ++s) {
        // a slice that got no hit tile wrote nothing
        if (po[0] + 32 * s >= po[1]) break;
        const float4 x = *reinterpret_cast<const float4*>(part + ((((size_t)(s - 1) * HK + hk) * N + m) * 2) * D + d);
        a.x += x.x; a.y += x.y; a.z += x.z; a.w += x.w;
      }
      *reinterpret_cast<float4*>(dst) = a;
    }
}

// ------------------------------------------------------------------------------------------
// Retrieval forward (Sec. 3.3 "Exact retrieval"): one wave per work item, a run of up to kRunTiles hit tiles of one
// retrieved pair (a heavy pair is many items, a light one a single item); the queries that retrieved the pair are
// the MFMA columns (32 at a time, rows read straight from Q), its keys the rows.
// A pair rarely has more than 32 keys: its key fragments and transposed value tile are then loaded once
// and reused by every hit tile; the hit list of the next tile is fetched while this one is computed.
// Writes, per (query, slot), the partial softmax state over the keys of the pair:
//   part[(qn*R2 + su)][0..D) = sum_m exp(l_m - max) v_m,  [D] = max (natural log units),  [D+1] = sum.
// ------------------------------------------------------------------------------------------
template <int D>
__global__ void __launch_bounds__(64) __attribute__((amdgpu_waves_per_eu(D == 64 ? 3 : 2, 4))) k_ret_fwd_pairs(const bf16_t* __restrict__ Q, const bf16_t* __restrict__ Ks,
                                                       const bf16_t* __restrict__ Vs, const int32_t* __restrict__ off_k,
                                                       const int32_t* __restrict__ run_off, const int4* __restrict__ run_map,
                                                       const uint2* __restrict__ hits, float* __restrict__ part,
                                                       size_t run_cap, size_t hit_cap, int N, int nb, int Ck,
                                                       int Hq, int Hkv, int R2, float scale_log2e) {
  constexpr int KS = D / 16, DT = D / 32, CPR = D / 8, NIT = 32 * CPR / 64;
  __shared__ __attribute__((aligned(16))) bf16_t vt[D][32 + TPAD];
  const int hk = blockIdx.y, NBm = nb - 1;
  if ((int)blockIdx.x >= run_off[(size_t)hk * ((size_t)NBm * Ck + 1) + (size_t)NBm * Ck]) return;  // past the last work item
  const int4 item = run_map[(size_t)hk * run_cap + blockIdx.x];  // (pair, first hit, end)
  const int G_ = Hq / Hkv;
  const size_t hqbase = (size_t)(hk / Hkv) * Hq + (size_t)(hk % Hkv) * G_;
  const int lane = threadIdx.x, col = lane % 32, half = lane / 32;
  const int32_t* ok = off_k + (size_t)hk * ((size_t)nb * Ck + 1);
  const int klo = ok[item.x], khi = ok[item.x + 1];  // pair = b' Ck + j indexes the segment table directly
  const int hlo = item.y, hhi = item.z;
  if (klo == khi) return;
  const uint2* hh = hits + (size_t)hk * hit_cap;
  const bool single = khi - klo <= 32;
  bf16x8_t kf[KS];
  auto stage = [&](int k0) {  // key fragments of row `col` and the transposed value tile of keys k0 .. k0+31
    uint4 v[NIT];
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
      const int c = lane + 64 * it, row = c % 32, cc = c / 32;  // lanes along the rows: conflict-free transposed stores
      const int kr = k0 + row < khi ? k0 + row : khi - 1;
      v[it] = *reinterpret_cast<const uint4*>(Vs + ((size_t)hk * N + kr) * D + cc * 8);
    }
    const int kr = k0 + col < khi ? k0 + col : khi - 1;
#pragma unroll
    for (int x = 0; x < KS; ++x)
      kf[x] = *reinterpret_cast<const bf16x8_t*>(Ks + ((size_t)hk * N + kr) * D + 16 * x + 8 * half);
    wave_lds_fence();
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
      const int c = lane + 64 * it, row = c % 32, cc = c / 32;  // lanes along the rows: conflict-free transposed stores
      const bf16_t* pv = reinterpret_cast<const bf16_t*>(&v[it]);
#pragma unroll
      for (int e = 0; e < 8; ++e) vt[cc * 8 + e][row] = pv[e];
    }
    wave_lds_fence();
  };
  // the hits of all the item's tiles are requested at once, and the query rows of tile t + 1 while tile t is
  // computed: one memory round trip per item after the first tile, not two per tile
  uint2 hitv[kRunTiles];
#pragma unroll
  for (int t = 0; t < kRunTiles; ++t) {
    const int h = hlo + 32 * t + col;
    hitv[t] = hh[h < hhi ? h : hhi - 1];
  }
  if (single) stage(klo);
  auto qrow = [&](const uint2 h) { return (hqbase + (h.x >> 22)) * N + (h.x & 0x3fffffu); };
  bf16x8_t qnext[KS];
  {
    const size_t q0 = qrow(hitv[0]);
#pragma unroll
    for (int s = 0; s < KS; ++s) qnext[s] = *reinterpret_cast<const bf16x8_t*>(Q + q0 * D + 16 * s + 8 * half);
  }
#pragma unroll
  for (int ti = 0; ti < kRunTiles; ++ti) {
    const int h0 = hlo + 32 * ti;
    if (h0 >= hhi) break;
    const bool hvalid = h0 + col < hhi;
    const uint2 hcur = hitv[ti];
    const size_t qn = qrow(hcur);
    bf16x8_t qf[KS];
#pragma unroll
    for (int s = 0; s < KS; ++s) qf[s] = qnext[s];
    if (ti + 1 < kRunTiles && h0 + 32 < hhi) {
      const size_t q1 = qrow(hitv[ti + 1 < kRunTiles ? ti + 1 : ti]);
#pragma unroll
      for (int s = 0; s < KS; ++s) qnext[s] = *reinterpret_cast<const bf16x8_t*>(Q + q1 * D + 16 * s + 8 * half);
    }
    f32x16_t o[DT];
#pragma unroll
    for (int t = 0; t < DT; ++t)
#pragma unroll
      for (int e = 0; e < 16; ++e) o[t][e] = 0.f;
    float m = MUSE_NEG_INF, l = 0.f;
    for (int k0 = klo; k0 < khi; k0 += 32) {
      if (!single) stage(k0);
      f32x16_t s;
#pragma unroll
      for (int e = 0; e < 16; ++e) s[e] = 0.f;
#pragma unroll
      for (int x = 0; x < KS; ++x) s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[x], qf[x], s, 0, 0, 0);
      float tmax = MUSE_NEG_INF;
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int kg = k0 + 8 * (e / 4) + 4 * half + (e % 4);
        if (kg >= khi) s[e] = MUSE_NEG_INF;
        tmax = fmaxf(tmax, s[e]);
      }
      tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
      const float mn = fmaxf(m, tmax * scale_log2e);
      const float alpha = fast_exp2(m - mn);  // every tile holds at least one key, so mn is finite
      float psum = 0.f;
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const float p = fast_exp2(fmaf(s[e], scale_log2e, -mn));
        s[e] = p;
        psum += p;
      }
      l = l * alpha + psum;
      m = mn;
#pragma unroll
      for (int t = 0; t < DT; ++t)
#pragma unroll
        for (int e = 0; e < 16; ++e) o[t][e] *= alpha;
#pragma unroll
      for (int G = 0; G < 2; ++G) {
        bf16x8_t pf = pack8(s, 2 * G, 2 * G + 1);
#pragma unroll
        for (int t = 0; t < DT; ++t) {
          bf16x8_t a = ld_tr8(&vt[32 * t + col][0], 16 * G, half);
          o[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf, o[t], 0, 0, 0);
        }
      }
    }
    l += __shfl_xor(l, 32, 64);
    if (hvalid) {
      float* pr = part + (qn * R2 + hcur.y) * (size_t)(D + 4);
#pragma unroll
      for (int t = 0; t < DT; ++t)
#pragma unroll
        for (int g = 0; g < 4; ++g)
          *reinterpret_cast<float4*>(pr + 32 * t + 8 * g + 4 * half) =
              make_float4(o[t][4 * g], o[t][4 * g + 1], o[t][4 * g + 2], o[t][4 * g + 3]);
      if (half == 0) { pr[D] = m * 0.6931471805599453f; pr[D + 1] = l; }
    }
  }
}

// ------------------------------------------------------------------------------------------
// Retrieval backward, gradient w.r.t. the queries: same tiling as the forward pair kernel;
// dqpart[(qn*R2 + su)][0..D) = scale * sum_m dl_m k_m over the keys of the pair.
// ------------------------------------------------------------------------------------------
template <int D>
__global__ void __launch_bounds__(64) __attribute__((amdgpu_waves_per_eu(D == 64 ? 2 : 1, 3))) k_ret_bwd_dq_pairs(const bf16_t* __restrict__ Q, const bf16_t* __restrict__ dO,
                                                          const bf16_t* __restrict__ Ks, const bf16_t* __restrict__ Vs,
                                                          const float* __restrict__ LSE, const float* __restrict__ delta,
                                                          const int32_t* __restrict__ off_k,
                                                          const int32_t* __restrict__ run_off,
                                                          const int4* __restrict__ run_map,
                                                          const uint2* __restrict__ hits, float* __restrict__ dqpart,
                                                          size_t run_cap, size_t hit_cap, int N, int nb, int Ck, int Hq,
                                                          int Hkv, int R2, float scale, float scale_log2e) {
  constexpr int KS = D / 16, DT = D / 32, CPR = D / 8, NIT = 32 * CPR / 64;
  __shared__ __attribute__((aligned(16))) bf16_t kt_[D][32 + TPAD];
  const int hk = blockIdx.y, NBm = nb - 1;
  if ((int)blockIdx.x >= run_off[(size_t)hk * ((size_t)NBm * Ck + 1) + (size_t)NBm * Ck]) return;  // past the last work item
  const int4 item = run_map[(size_t)hk * run_cap + blockIdx.x];  // (pair, first hit, end)
  const int G_ = Hq / Hkv;
  const size_t hqbase = (size_t)(hk / Hkv) * Hq + (size_t)(hk % Hkv) * G_;
  const int lane = threadIdx.x, col = lane % 32, half = lane / 32;
  const int32_t* ok = off_k + (size_t)hk * ((size_t)nb * Ck + 1);
  const int klo = ok[item.x], khi = ok[item.x + 1];  // pair = b' Ck + j indexes the segment table directly
  const int hlo = item.y, hhi = item.z;
  if (klo == khi) return;
  const uint2* hh = hits + (size_t)hk * hit_cap;
  const bool single = khi - klo <= 32;
  bf16x8_t kf[KS], vf[KS];
  auto stage = [&](int k0) {  // key / value fragments of row `col` and the transposed key tile of keys k0 .. k0+31
    uint4 v[NIT];
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
      const int c = lane + 64 * it, row = c % 32, cc = c / 32;  // lanes along the rows: conflict-free transposed stores
      const int kr = k0 + row < khi ? k0 + row : khi - 1;
      v[it] = *reinterpret_cast<const uint4*>(Ks + ((size_t)hk * N + kr) * D + cc * 8);
    }
    const int kr = k0 + col < khi ? k0 + col : khi - 1;
#pragma unroll
    for (int x = 0; x < KS; ++x) {
      kf[x] = *reinterpret_cast<const bf16x8_t*>(Ks + ((size_t)hk * N + kr) * D + 16 * x + 8 * half);
      vf[x] = *reinterpret_cast<const bf16x8_t*>(Vs + ((size_t)hk * N + kr) * D + 16 * x + 8 * half);
    }
    wave_lds_fence();
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
      const int c = lane + 64 * it, row = c % 32, cc = c / 32;  // lanes along the rows: conflict-free transposed stores
      const bf16_t* pv = reinterpret_cast<const bf16_t*>(&v[it]);
#pragma unroll
      for (int e = 0; e < 8; ++e) kt_[cc * 8 + e][row] = pv[e];
    }
    wave_lds_fence();
  };
  // the hits of all the item's tiles are requested at once, and the rows of tile t + 1 while tile t is computed
  uint2 hitv[kRunTiles];
#pragma unroll
  for (int t = 0; t < kRunTiles; ++t) {
    const int h = hlo + 32 * t + col;
    hitv[t] = hh[h < hhi ? h : hhi - 1];
  }
  if (single) stage(klo);
  auto qrow = [&](const uint2 h) { return (hqbase + (h.x >> 22)) * N + (h.x & 0x3fffffu); };
  bf16x8_t qnext[KS], gnext[KS];
  float lnext, dnext;
  {
    const size_t q0 = qrow(hitv[0]);
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      qnext[s] = *reinterpret_cast<const bf16x8_t*>(Q + q0 * D + 16 * s + 8 * half);
      gnext[s] = *reinterpret_cast<const bf16x8_t*>(dO + q0 * D + 16 * s + 8 * half);
    }
    lnext = LSE[q0];
    dnext = delta[q0];
  }
#pragma unroll
  for (int ti = 0; ti < kRunTiles; ++ti) {
    const int h0 = hlo + 32 * ti;
    if (h0 >= hhi) break;
    const bool hvalid = h0 + col < hhi;
    const uint2 hcur = hitv[ti];
    const size_t qn = qrow(hcur);
    bf16x8_t qf[KS], gf[KS];
#pragma unroll
    for (int s = 0; s < KS; ++s) { qf[s] = qnext[s]; gf[s] = gnext[s]; }
    const float lse2 = lnext * 1.4426950408889634f, dl = dnext;
    if (ti + 1 < kRunTiles && h0 + 32 < hhi) {
      const size_t q1 = qrow(hitv[ti + 1 < kRunTiles ? ti + 1 : ti]);
#pragma unroll
      for (int s = 0; s < KS; ++s) {
        qnext[s] = *reinterpret_cast<const bf16x8_t*>(Q + q1 * D + 16 * s + 8 * half);
        gnext[s] = *reinterpret_cast<const bf16x8_t*>(dO + q1 * D + 16 * s + 8 * half);
      }
      lnext = LSE[q1];
      dnext = delta[q1];
    }
    f32x16_t dq[DT];
#pragma unroll
    for (int t = 0; t < DT; ++t)
#pragma unroll
      for (int e = 0; e < 16; ++e) dq[t][e] = 0.f;
    for (int k0 = klo; k0 < khi; k0 += 32) {
      if (!single) stage(k0);
      f32x16_t s, dp;
#pragma unroll
      for (int e = 0; e < 16; ++e) { s[e] = 0.f; dp[e] = 0.f; }
#pragma unroll
      for (int x = 0; x < KS; ++x) {
        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[x], qf[x], s, 0, 0, 0);
        dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[x], gf[x], dp, 0, 0, 0);
      }
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int kg = k0 + 8 * (e / 4) + 4 * half + (e % 4);
        float p = fast_exp2(fmaf(s[e], scale_log2e, -lse2));
        p = kg < khi ? p : 0.f;
        s[e] = p * (dp[e] - dl);
      }
#pragma unroll
      for (int G = 0; G < 2; ++G) {
        bf16x8_t df = pack8(s, 2 * G, 2 * G + 1);
#pragma unroll
        for (int t = 0; t < DT; ++t) {
          bf16x8_t a = ld_tr8(&kt_[32 * t + col][0], 16 * G, half);
          dq[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, df, dq[t], 0, 0, 0);
        }
      }
    }
    if (hvalid) {
      float* pr = dqpart + (qn * R2 + hcur.y) * (size_t)D;
#pragma unroll
      for (int t = 0; t < DT; ++t)
#pragma unroll
        for (int g = 0; g < 4; ++g)
          *reinterpret_cast<float4*>(pr + 32 * t + 8 * g + 4 * half) =
              make_float4(scale * dq[t][4 * g], scale * dq[t][4 * g + 1], scale * dq[t][4 * g + 2], scale * dq[t][4 * g + 3]);
    }
  }
}

// ------------------------------------------------------------------------------------------
// Gradients of the accumulated cells (component 1) for bf16 inputs: the (b, i) group's queries against
// a tile of 32 key clusters is a dense attention-backward block with the accumulated summaries in the
// role of keys and values.  One block per group: its queries (QT tiles of 32 at a time, nearly always
// all of them) are staged in LDS once, and every wave walks its share of the cluster tiles with the
// next tile's summaries already in flight.
//   g_A_k = sum dl q~,  g_A_v = sum p dO,  g_A_c = sum [dl (1 - q~.kbar) - p dO.vbar]
// Operands are rounded to bf16 for the matrix cores (gradients only; no selection depends on them).
// A group with more than 32 QT queries takes further passes that add to the rows of the first.
// ------------------------------------------------------------------------------------------
template <int D, int QT>
__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(D == 64 ? 2 : 1, 2))) k_ff_bwd_cells_mx(
    const bf16_t* __restrict__ Q, const bf16_t* __restrict__ dO, const float* __restrict__ qc,
    const float* __restrict__ A_mu, const bf16_t* __restrict__ A_kb, const bf16_t* __restrict__ A_v,
    const int32_t* __restrict__ perm_q, const int32_t* __restrict__ off_q, const float* __restrict__ LSE,
    const float* __restrict__ delta, const uint32_t* __restrict__ selmask, float* __restrict__ g_A_c,
    bf16_t* __restrict__ g_A_k, bf16_t* __restrict__ g_A_v, int h0, int N, int nb, int Cq, int Ck, float scale) {
  constexpr int KS = D / 16, DT = D / 32, CPR = D / 8, QR = 32 * QT;
  __shared__ __attribute__((aligned(16))) bf16_t qs[QR][D + 8];
  __shared__ __attribute__((aligned(16))) bf16_t gs[QR][D + 8];
  __shared__ __attribute__((aligned(16))) bf16_t qt_[D][QR + TPAD];
  __shared__ __attribute__((aligned(16))) bf16_t gt_[D][QR + TPAD];
  __shared__ __attribute__((aligned(16))) float ls[QR];
  __shared__ __attribute__((aligned(16))) float ds[QR];
  __shared__ uint32_t mws[4][QR];
  __shared__ __attribute__((aligned(16))) bf16_t tw[4][32][D + 8];
  const int hl = blockIdx.z, hq = h0 + hl;
  const int NBm = nb - 1, W = (Ck + 31) / 32;
  const int b = blockIdx.y / Cq + 1, i = blockIdx.y % Cq;
  const int wave = threadIdx.x / 64, lane = threadIdx.x % 64, col = lane % 32, half = lane / 32;
  const int32_t* oq = off_q + (size_t)hq * ((size_t)nb * Cq + 1);
  const int qlo = oq[b * Cq + i], qhi = oq[b * Cq + i + 1];
  const size_t acell = (((size_t)hl * NBm + (b - 1)) * Cq + i) * Ck;
  const float* qci = qc + ((size_t)hq * Cq + i) * D;
  struct CT {  // one tile of 32 accumulated summaries as this lane's operand fragments
    bf16x8_t kf[KS], vf[KS];
    float amu;  // raw: any arithmetic on a prefetched value would wait for the whole prefetch at once
    uint32_t mw[QT];  // word of the selection mask of staged query 32 qt + col for this cluster tile
  };
  auto load_ct = [&](int jt, int q0, int qhi, CT& c) {
    const int jc = jt * 32 + col;
    const int jcc = jc < Ck ? jc : Ck - 1;
#pragma unroll
    for (int x = 0; x < KS; ++x) {
      c.kf[x] = *reinterpret_cast<const bf16x8_t*>(A_kb + (acell + jcc) * D + 16 * x + 8 * half);
      c.vf[x] = *reinterpret_cast<const bf16x8_t*>(A_v + (acell + jcc) * D + 16 * x + 8 * half);
    }
    c.amu = A_mu[acell + jcc];
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {
      const int pq = q0 + 32 * qt + col;
      c.mw[qt] = selmask[((size_t)hq * W + jt) * N + (pq < qhi ? pq : q0)];
    }
  };
  for (int q0 = qlo; q0 < qhi || q0 == qlo; q0 += QR) {  // an empty group still writes its (zero) cells
    const bool first = q0 == qlo;
    __syncthreads();
    for (int c = threadIdx.x; c < (q0 < qhi ? QR * CPR : 0); c += 256) {
      const int row = c % QR, cc = c / QR;  // lanes along the rows: conflict-free transposed stores
      const int pos = q0 + row < qhi ? q0 + row : q0;
      const size_t qn = (size_t)hq * N + perm_q[(size_t)hq * N + pos];
      uint4 qv = *reinterpret_cast<const uint4*>(Q + qn * D + cc * 8);
      uint4 gvv = *reinterpret_cast<const uint4*>(dO + qn * D + cc * 8);
      const bf16_t* pq = reinterpret_cast<const bf16_t*>(&qv);
      const bf16_t* pg = reinterpret_cast<const bf16_t*>(&gvv);
      float4 c0 = *reinterpret_cast<const float4*>(qci + cc * 8), c1 = *reinterpret_cast<const float4*>(qci + cc * 8 + 4);
      const float cv[8] = {c0.x, c0.y, c0.z, c0.w, c1.x, c1.y, c1.z, c1.w};
      bf16_t qtl[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) qtl[e] = f32_to_bf16_bits(scale * (bf16_bits_to_f32(pq[e]) - cv[e]));
      *reinterpret_cast<uint4*>(&qs[row][cc * 8]) = *reinterpret_cast<const uint4*>(qtl);
      *reinterpret_cast<uint4*>(&gs[row][cc * 8]) = gvv;
#pragma unroll
      for (int e = 0; e < 8; ++e) { qt_[cc * 8 + e][row] = qtl[e]; gt_[cc * 8 + e][row] = pg[e]; }
    }
    if (threadIdx.x < QR && q0 < qhi) {
      const int row = threadIdx.x;
      const bool ok = q0 + row < qhi;
      const size_t qn = (size_t)hq * N + perm_q[(size_t)hq * N + (ok ? q0 + row : q0)];
      ls[row] = ok ? LSE[qn] * 1.4426950408889634f : __builtin_huge_valf();  // +inf -> p = 0 for padding rows
      ds[row] = delta[qn];
    }
    __syncthreads();
    const int ntl = (qhi - q0 + 31) / 32 < QT ? (qhi - q0 + 31) / 32 : QT;  // staged query tiles (0 for an empty group)
    CT cur, nxt;
    if (wave < W) load_ct(wave, q0 < qhi ? q0 : 0, qhi, cur);
    for (int jt = wave; jt < W; jt += 4) {
      // always issued (the last tile again at the end): with the same number of loads in flight on every path
      // the wait for this tile's operands can leave the next tile's loads outstanding
      load_ct(jt + 4 < W ? jt + 4 : jt, q0 < qhi ? q0 : 0, qhi, nxt);
      // this wave's words of the selection mask: one per staged query, for cluster tile jt
      if (half == 0) {
#pragma unroll
        for (int qt = 0; qt < QT; ++qt) mws[wave][32 * qt + col] = cur.mw[qt];
      }
      wave_lds_fence();
      const int jc = jt * 32 + col;
      const bool jvalid = jc < Ck;
      const float amu2 = jvalid ? cur.amu * 1.4426950408889634f : MUSE_NEG_INF;
      f32x16_t gk[DT], gv[DT];
#pragma unroll
      for (int t = 0; t < DT; ++t)
#pragma unroll
        for (int e = 0; e < 16; ++e) { gk[t][e] = 0.f; gv[t][e] = 0.f; }
      float csum = 0.f;
      for (int qt = 0; qt < ntl; ++qt) {
        f32x16_t s, dp;
#pragma unroll
        for (int e = 0; e < 16; ++e) { s[e] = 0.f; dp[e] = 0.f; }
#pragma unroll
        for (int x = 0; x < KS; ++x) {
          bf16x8_t a = *reinterpret_cast<const bf16x8_t*>(&qs[32 * qt + col][16 * x + 8 * half]);
          s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, cur.kf[x], s, 0, 0, 0);
          bf16x8_t ag = *reinterpret_cast<const bf16x8_t*>(&gs[32 * qt + col][16 * x + 8 * half]);
          dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ag, cur.vf[x], dp, 0, 0, 0);
        }
        f32x16_t pr;
#pragma unroll
        for (int gq = 0; gq < 4; ++gq) {
          float4 l4 = *reinterpret_cast<const float4*>(&ls[32 * qt + 8 * gq + 4 * half]);
          float4 d4 = *reinterpret_cast<const float4*>(&ds[32 * qt + 8 * gq + 4 * half]);
          const float lv[4] = {l4.x, l4.y, l4.z, l4.w}, dv4[4] = {d4.x, d4.y, d4.z, d4.w};
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            const int e = 4 * gq + u, row = 32 * qt + 8 * gq + 4 * half + u;
            float p = fast_exp2(fmaf(s[e], 1.4426950408889634f, amu2 - lv[u]));
            p = ((mws[wave][row] >> col) & 1u) ? 0.f : p;
            const float dlg = p * (dp[e] - dv4[u]);
            csum += p > 0.f ? dlg * (1.f - s[e]) - p * dp[e] : 0.f;
            pr[e] = p;
            s[e] = dlg;
          }
        }
#pragma unroll
        for (int G = 0; G < 2; ++G) {
          bf16x8_t pf = pack8(pr, 2 * G, 2 * G + 1);
          bf16x8_t df = pack8(s, 2 * G, 2 * G + 1);
#pragma unroll
          for (int t = 0; t < DT; ++t) {
            bf16x8_t ag = ld_tr8(&gt_[32 * t + col][0], 32 * qt + 16 * G, half);
            gv[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ag, pf, gv[t], 0, 0, 0);
            bf16x8_t aq = ld_tr8(&qt_[32 * t + col][0], 32 * qt + 16 * G, half);
            gk[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(aq, df, gk[t], 0, 0, 0);
          }
        }
      }
      wave_lds_fence();  // mws is rewritten for the next cluster tile
      csum += __shfl_xor(csum, 32, 64);
      // rows go out through a per-wave LDS tile: a store instruction then writes 64 / (D/8) whole rows of
      // consecutive clusters (contiguous memory) instead of 32 fragments of 8 bytes
#pragma unroll
      for (int arr = 0; arr < 2; ++arr) {
        wave_lds_fence();
#pragma unroll
        for (int t = 0; t < DT; ++t)
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            const f32x16_t& a = arr == 0 ? gk[t] : gv[t];
            *reinterpret_cast<uint2*>(&tw[wave][col][32 * t + 8 * g + 4 * half]) =
                make_uint2(pack_bf16x2(a[4 * g], a[4 * g + 1]), pack_bf16x2(a[4 * g + 2], a[4 * g + 3]));
          }
        wave_lds_fence();
        bf16_t* dst = arr == 0 ? g_A_k : g_A_v;
#pragma unroll
        for (int it = 0; it < 32 * CPR / 64; ++it) {
          const int row = it * (64 / CPR) + lane / CPR, cc = lane % CPR;
          if (jt * 32 + row < Ck) {
            uint4 v = *reinterpret_cast<const uint4*>(&tw[wave][row][cc * 8]);
            uint4* o = reinterpret_cast<uint4*>(dst + (acell + jt * 32 + row) * D + cc * 8);
            if (!first) {  // further pass of a large group: add to what the earlier passes wrote
              const uint4 old = *o;
              const uint32_t* pn = reinterpret_cast<const uint32_t*>(&v);
              const uint32_t* po = reinterpret_cast<const uint32_t*>(&old);
              uint32_t rr[4];
#pragma unroll
              for (int u = 0; u < 4; ++u)
                rr[u] = pack_bf16x2(__uint_as_float(pn[u] << 16) + __uint_as_float(po[u] << 16),
                                    __uint_as_float(pn[u] & 0xffff0000u) + __uint_as_float(po[u] & 0xffff0000u));
              v = make_uint4(rr[0], rr[1], rr[2], rr[3]);
            }
            typedef uint32_t u4_t __attribute__((ext_vector_type(4)));
            const u4_t vs = {v.x, v.y, v.z, v.w};
            __builtin_nontemporal_store(vs, reinterpret_cast<u4_t*>(o));  // written once, read by the next kernel much later
          }
        }
      }
      if (jvalid && half == 0) g_A_c[acell + jc] = first ? csum : g_A_c[acell + jc] + csum;
      cur = nxt;
    }
  }
}

// ------------------------------------------------------------------------------------------
// Summary gradients -> keys and values for bf16 inputs: one wave per (kv head, key block b', key
// cluster j); the keys of the segment are the MFMA columns, 32 query clusters at a time the rows.
//   W[i,m] = exp(L[i,m] - mu[i]),  T[i,m] = G_c[i] + G_k[i].k_m + G_v[i].v_m
//   dv_m += sum_i W G_v[i],  dk_m += sum_i W G_k[i] + (W T) qbar_i
// G and qbar are rounded to bf16 for the matrix cores (gradients only).  The gradient rows are read once, as
// the row operands of T; for the contractions over i they go through a transposed tile in LDS, and qbar comes
// from a transposed bf16 copy qcT[head][d][i] (scale folded in, i padded to a multiple of 32 with zeros).
// ------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) k_qc_transpose(const float* __restrict__ qc, bf16_t* __restrict__ qcT, int D,
                                                       int Cq, int CqP, float scale) {
  const int h = blockIdx.y;
  const int t = blockIdx.x * 256 + threadIdx.x;
  if (t >= D * CqP) return;
  const int d = t / CqP, i = t % CqP;
  qcT[(size_t)h * D * CqP + t] = f32_to_bf16_bits(i < Cq ? scale * qc[((size_t)h * Cq + i) * D + d] : 0.f);
}

template <int D>
__global__ void __launch_bounds__(64) k_cells_to_keys_mx(const bf16_t* __restrict__ Ks, const bf16_t* __restrict__ Vs,
                                                          const bf16_t* __restrict__ qcT, const float* __restrict__ L,
                                                          const float* __restrict__ s_mu, const float* __restrict__ G_c,
                                                          const bf16_t* __restrict__ G_k, const bf16_t* __restrict__ G_v,
                                                          const int32_t* __restrict__ off_k, float* __restrict__ dKs,
                                                          float* __restrict__ dVs, int h0, int N, int nb, int Cq, int CqP,
                                                          int Ck, int Hq, int Hkv, int frozen) {
  constexpr int KS = D / 16, DT = D / 32;
  __shared__ __attribute__((aligned(16))) bf16_t gkT[D][32 + TPAD];
  __shared__ __attribute__((aligned(16))) bf16_t gvT[D][32 + TPAD];
  __shared__ __attribute__((aligned(16))) float mus[32];
  __shared__ __attribute__((aligned(16))) float gcs[32];
  __shared__ uint4 kbs[KS][64], vbs[KS][64];
  const int G_ = Hq / Hkv;
  const int hkl = blockIdx.z;
  const int hq0 = h0 + hkl * G_;
  const int hk = (hq0 / Hq) * Hkv + (hq0 % Hq) / G_;
  // x % 8 is the XCD a workgroup lands on (the grid's x extent is a multiple of 8): each XCD takes a run of
  // consecutive key clusters, whose per-cell scalars share 32-byte sectors, so a sector is fetched by one L2
  const int run = gridDim.x / 8;
  const int bp = blockIdx.y, j = (blockIdx.x % 8) * run + blockIdx.x / 8, NBm = nb - 1;
  if (j >= Ck) return;
  const int lane = threadIdx.x, col = lane % 32, half = lane / 32;
  const int32_t* ok = off_k + (size_t)hk * ((size_t)nb * Ck + 1);
  const int klo = ok[bp * Ck + j], khi = ok[bp * Ck + j + 1];
  for (int m0 = klo; m0 < khi; m0 += 32) {
    const int pm = m0 + col;
    const bool mvalid = pm < khi;
    const int pmc = mvalid ? pm : m0;
    // the lane's key and value fragments wait in LDS (they are needed once per tile of query clusters)
    wave_lds_fence();
#pragma unroll
    for (int x = 0; x < KS; ++x) {
      kbs[x][lane] = *reinterpret_cast<const uint4*>(Ks + ((size_t)hk * N + pmc) * D + 16 * x + 8 * half);
      vbs[x][lane] = *reinterpret_cast<const uint4*>(Vs + ((size_t)hk * N + pmc) * D + 16 * x + 8 * half);
    }
    f32x16_t dk[DT], dv[DT];
#pragma unroll
    for (int t = 0; t < DT; ++t)
#pragma unroll
      for (int e = 0; e < 16; ++e) { dk[t][e] = 0.f; dv[t][e] = 0.f; }
    for (int g = 0; g < G_; ++g) {
      const int hl = hkl * G_ + g;
      const bf16_t* qT = qcT + (size_t)hl * D * CqP;
      const float* Lh = L + (size_t)hl * Cq * N + pmc;
      // a tile's loads: the lane's gradient row (query cluster i0 + col), its scalars, the logits of the lane's
      // key against the 16 query clusters of its accumulator rows, all issued before the first use
      struct GT {
        bf16x8_t gkr[KS], gvr[KS];
        float mu, gc, lg[16];
      };
      auto load_gt = [&](GT& gt, int i0) {
        const int ic = i0 + col < Cq ? i0 + col : Cq - 1;
        const size_t cellA = (((size_t)hl * NBm + bp) * Cq + ic) * Ck + j;
#pragma unroll
        for (int x = 0; x < KS; ++x) {
          gt.gkr[x] = *reinterpret_cast<const bf16x8_t*>(G_k + cellA * D + 16 * x + 8 * half);
          gt.gvr[x] = *reinterpret_cast<const bf16x8_t*>(G_v + cellA * D + 16 * x + 8 * half);
        }
        gt.mu = s_mu[cellA];
        gt.gc = G_c[cellA];
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          int ir = i0 + 8 * (e / 4) + 4 * half + (e % 4);
          ir = ir < Cq ? ir : Cq - 1;
          gt.lg[e] = Lh[(size_t)ir * N];
        }
      };
      for (int i0 = 0; i0 < Cq; i0 += 32) {
        GT cur;
        load_gt(cur, i0);
        const bf16x8_t(&gkr)[KS] = cur.gkr;
        const bf16x8_t(&gvr)[KS] = cur.gvr;
        const float mu_l = cur.mu, gc_l = cur.gc;
        const float(&lg)[16] = cur.lg;
        wave_lds_fence();  // the previous tile's operand reads are done
        if (half == 0) { mus[col] = mu_l; gcs[col] = gc_l; }
#pragma unroll
        for (int x = 0; x < KS; ++x) {
          const bf16_t* pk = reinterpret_cast<const bf16_t*>(&gkr[x]);
          const bf16_t* pv = reinterpret_cast<const bf16_t*>(&gvr[x]);
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            gkT[16 * x + 8 * half + e][col] = pk[e];
            gvT[16 * x + 8 * half + e][col] = pv[e];
          }
        }
        wave_lds_fence();
        f32x16_t tacc, wv;
#pragma unroll
        for (int gq = 0; gq < 4; ++gq) {
          const float4 m4 = *reinterpret_cast<const float4*>(&mus[8 * gq + 4 * half]);
          const float4 c4 = *reinterpret_cast<const float4*>(&gcs[8 * gq + 4 * half]);
          const float mv[4] = {m4.x, m4.y, m4.z, m4.w}, cv[4] = {c4.x, c4.y, c4.z, c4.w};
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            const int e = 4 * gq + u;
            const bool iv = i0 + 8 * gq + 4 * half + u < Cq;
            tacc[e] = cv[u];
            wv[e] = (iv && mvalid) ? __expf(lg[e] - mv[u]) : 0.f;
          }
        }
        // frozen aggregation weights: nothing flows through W (the T term and its contraction with qbar drop out)
        if (!frozen) {
#pragma unroll
          for (int x = 0; x < KS; ++x) {
            tacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(gkr[x], __builtin_bit_cast(bf16x8_t, kbs[x][lane]), tacc, 0, 0, 0);
            tacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(gvr[x], __builtin_bit_cast(bf16x8_t, vbs[x][lane]), tacc, 0, 0, 0);
          }
        }
#pragma unroll
        for (int e = 0; e < 16; ++e) tacc[e] = (wv[e] > 0.f && !frozen) ? wv[e] * tacc[e] : 0.f;
#pragma unroll
        for (int G = 0; G < 2; ++G) {
          bf16x8_t wf = pack8(wv, 2 * G, 2 * G + 1);
          bf16x8_t tf = pack8(tacc, 2 * G, 2 * G + 1);
#pragma unroll
          for (int t = 0; t < DT; ++t) {
            const bf16x8_t ak = ld_tr8(&gkT[32 * t + col][0], 16 * G, half);
            const bf16x8_t av = ld_tr8(&gvT[32 * t + col][0], 16 * G, half);
            const bf16x8_t aq = ld_tr8(qT + (size_t)(32 * t + col) * CqP + i0, 16 * G, half);
            dv[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, wf, dv[t], 0, 0, 0);
            dk[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ak, wf, dk[t], 0, 0, 0);
            if (!frozen) dk[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(aq, tf, dk[t], 0, 0, 0);
          }
        }
      }
    }
    if (mvalid) {
      float* ok_ = dKs + ((size_t)hk * N + pm) * D;
      float* ov_ = dVs + ((size_t)hk * N + pm) * D;
#pragma unroll
      for (int t = 0; t < DT; ++t)
#pragma unroll
        for (int gg = 0; gg < 4; ++gg) {
          const int d = 32 * t + 8 * gg + 4 * half;
          float4 a = *reinterpret_cast<float4*>(ok_ + d), c = *reinterpret_cast<float4*>(ov_ + d);
          a.x += dk[t][4 * gg]; a.y += dk[t][4 * gg + 1]; a.z += dk[t][4 * gg + 2]; a.w += dk[t][4 * gg + 3];
          c.x += dv[t][4 * gg]; c.y += dv[t][4 * gg + 1]; c.z += dv[t][4 * gg + 2]; c.w += dv[t][4 * gg + 3];
          *reinterpret_cast<float4*>(ok_ + d) = a;
          *reinterpret_cast<float4*>(ov_ + d) = c;
        }
    }
  }
}

}  // namespace

int muse_launch_cells_to_keys_mx(const MuseDims& d, const void* Ks, const void* Vs, const float* qc, void* qcT,
                                 const float* L, const float* s_mu, const float* G_c, const void* G_k, const void* G_v,
                                 const int32_t* off_k, float* dKs, float* dVs, int h0, int hn, hipStream_t st) {
  const int CqP = (d.Cq + 31) / 32 * 32;
  // qcT holds the transposed centroids of the chunk's heads [h0, h0 + hn)
  { MuseProf prof_("k_qc_transpose", st); hipLaunchKernelGGL(k_qc_transpose, dim3((d.D * CqP + 255) / 256, hn), dim3(256), 0, st, qc + (size_t)h0 * d.Cq * d.D, (bf16_t*)qcT, d.D, d.Cq, CqP, d.scale); }
  dim3 g((d.Ck + 7) / 8 * 8, d.nb - 1, hn / (d.Hq / d.Hkv));
  if (d.D == 64)
    { MuseProf prof_("k_cells_to_keys_mx", st); hipLaunchKernelGGL(k_cells_to_keys_mx<64>, g, dim3(64), 0, st, (const bf16_t*)Ks, (const bf16_t*)Vs, (const bf16_t*)qcT, L, s_mu, G_c, (const bf16_t*)G_k, (const bf16_t*)G_v, off_k, dKs, dVs, h0, d.N, d.nb, d.Cq, CqP, d.Ck, d.Hq, d.Hkv, d.frozen_weights ? 1 : 0); }
  else
    { MuseProf prof_("k_cells_to_keys_mx", st); hipLaunchKernelGGL(k_cells_to_keys_mx<128>, g, dim3(64), 0, st, (const bf16_t*)Ks, (const bf16_t*)Vs, (const bf16_t*)qcT, L, s_mu, G_c, (const bf16_t*)G_k, (const bf16_t*)G_v, off_k, dKs, dVs, h0, d.N, d.nb, d.Cq, CqP, d.Ck, d.Hq, d.Hkv, d.frozen_weights ? 1 : 0); }
  MUSE_LAUNCH_CHECK();
  return MUSE_OK;
}

int muse_launch_ff_bwd_cells_mx(const MuseDims& d, const void* Q, const void* dO, const float* qc, const float* A_mu,
                                const void* A_kb, const void* A_v, const int32_t* perm_q, const int32_t* off_q,
                                const float* LSE, const float* delta, const uint32_t* selmask, float* g_A_c,
                                void* g_A_k, void* g_A_v, int h0, int hn, hipStream_t st) {
  dim3 g(1, (d.nb - 1) * d.Cq, hn);
  if (d.D == 64)
    { MuseProf prof_("k_ff_bwd_cells_mx", st); hipLaunchKernelGGL((k_ff_bwd_cells_mx<64, 3>), g, dim3(256), 0, st, (const bf16_t*)Q, (const bf16_t*)dO, qc, A_mu, (const bf16_t*)A_kb, (const bf16_t*)A_v, perm_q, off_q, LSE, delta, selmask, g_A_c, (bf16_t*)g_A_k, (bf16_t*)g_A_v, h0, d.N, d.nb, d.Cq, d.Ck, d.scale); }
  else
    { MuseProf prof_("k_ff_bwd_cells_mx", st); hipLaunchKernelGGL((k_ff_bwd_cells_mx<128, 1>), g, dim3(256), 0, st, (const bf16_t*)Q, (const bf16_t*)dO, qc, A_mu, (const bf16_t*)A_kb, (const bf16_t*)A_v, perm_q, off_q, LSE, delta, selmask, g_A_c, (bf16_t*)g_A_k, (bf16_t*)g_A_v, h0, d.N, d.nb, d.Cq, d.Ck, d.scale); }
  MUSE_LAUNCH_CHECK();
  return MUSE_OK;
}

int muse_launch_ret_fwd_pairs(const MuseDims& d, const void* Q, const void* Ks, const void* Vs, const int32_t* off_k,
                              const int32_t* run_off, const int4* run_map, size_t run_cap, const uint2* hits,
                              size_t hit_cap, float* part, hipStream_t st) {
  // one wave per work item (a run of hit tiles inside one pair); the grid covers the most there can be
  dim3 g((unsigned)run_cap, d.B * d.Hkv);
  float sl = d.scale * 1.4426950408889634f;
  if (d.D == 64)
    { MuseProf prof_("k_ret_fwd_pairs", st); hipLaunchKernelGGL(k_ret_fwd_pairs<64>, g, dim3(64), 0, st, (const bf16_t*)Q, (const bf16_t*)Ks, (const bf16_t*)Vs, off_k, run_off, run_map, hits, part, run_cap, hit_cap, d.N, d.nb, d.Ck, d.Hq, d.Hkv, d.r * d.k2e, sl); }
  else
    { MuseProf prof_("k_ret_fwd_pairs", st); hipLaunchKernelGGL(k_ret_fwd_pairs<128>, g, dim3(64), 0, st, (const bf16_t*)Q, (const bf16_t*)Ks, (const bf16_t*)Vs, off_k, run_off, run_map, hits, part, run_cap, hit_cap, d.N, d.nb, d.Ck, d.Hq, d.Hkv, d.r * d.k2e, sl); }
  MUSE_LAUNCH_CHECK();
  return MUSE_OK;
}

int muse_launch_ret_bwd_dq_pairs(const MuseDims& d, const void* Q, const void* dO, const void* Ks, const void* Vs,
                                 const float* LSE, const float* delta, const int32_t* off_k, const int32_t* run_off,
                                 const int4* run_map, size_t run_cap, const uint2* hits, size_t hit_cap, float* dqpart,
                                 hipStream_t st) {
  dim3 g((unsigned)run_cap, d.B * d.Hkv);
  float sl = d.scale * 1.4426950408889634f;
  if (d.D == 64)
    { MuseProf prof_("k_ret_bwd_dq_pairs", st); hipLaunchKernelGGL(k_ret_bwd_dq_pairs<64>, g, dim3(64), 0, st, (const bf16_t*)Q, (const bf16_t*)dO, (const bf16_t*)Ks, (const bf16_t*)Vs, LSE, delta, off_k, run_off, run_map, hits, dqpart, run_cap, hit_cap, d.N, d.nb, d.Ck, d.Hq, d.Hkv, d.r * d.k2e, d.scale, sl); }
  else
    { MuseProf prof_("k_ret_bwd_dq_pairs", st); hipLaunchKernelGGL(k_ret_bwd_dq_pairs<128>, g, dim3(64), 0, st, (const bf16_t*)Q, (const bf16_t*)dO, (const bf16_t*)Ks, (const bf16_t*)Vs, LSE, delta, off_k, run_off, run_map, hits, dqpart, run_cap, hit_cap, d.N, d.nb, d.Ck, d.Hq, d.Hkv, d.r * d.k2e, d.scale, sl); }
  MUSE_LAUNCH_CHECK();
  return MUSE_OK;
}

int muse_launch_c3_pairs(const MuseDims& d, const void* Q, const void* dO, const void* Ks, const void* Vs,
                         const float* LSE, const float* delta, const int32_t* off_k, const int32_t* pair_off,
                         const int32_t* c3_off, const int2* c3_map, size_t run_cap, const uint2* hits, size_t hit_cap,
                         float* dKs, float* dVs, float* part, hipStream_t st) {
  const int HK = d.B * d.Hkv;
  dim3 g((unsigned)run_cap, HK), gr((unsigned)run_cap, HK);
  float sl = d.scale * 1.4426950408889634f;
  if (d.D == 64) {
    { MuseProf prof_("k_c3_pairs", st); hipLaunchKernelGGL(k_c3_pairs<64>, g, dim3(64), 0, st, (const bf16_t*)Q, (const bf16_t*)dO, (const bf16_t*)Ks,
                       (const bf16_t*)Vs, LSE, delta, off_k, pair_off, c3_off, c3_map, hits, dKs, dVs, part, run_cap, hit_cap, d.N, d.nb, d.Ck, d.Hq, d.Hkv, HK, d.scale, sl); }
    { MuseProf prof_("k_c3_reduce", st); hipLaunchKernelGGL(k_c3_reduce<64>, gr, dim3(64), 0, st, off_k, pair_off, c3_off, c3_map, part, dKs, dVs, run_cap, d.N, d.nb, d.Ck, HK); }
  } else {
    { MuseProf prof_("k_c3_pairs", st); hipLaunchKernelGGL(k_c3_pairs<128>, g, dim3(64), 0, st, (const bf16_t*)Q, (const bf16_t*)dO, (const bf16_t*)Ks,
                       (const bf16_t*)Vs, LSE, delta, off_k, pair_off, c3_off, c3_map, hits, dKs, dVs, part, run_cap, hit_cap, d.N, d.nb, d.Ck, d.Hq, d.Hkv, HK, d.scale, sl); }
    { MuseProf prof_("k_c3_reduce", st); hipLaunchKernelGGL(k_c3_reduce<128>, gr, dim3(64), 0, st, off_k, pair_off, c3_off, c3_map, part, dKs, dVs, run_cap, d.N, d.nb, d.Ck, HK); }
  }
  MUSE_LAUNCH_CHECK();
  return MUSE_OK;
}

int muse_launch_attn_fwd_mfma(const MuseDims& d, int Bs, const void* Q, const void* K, const void* V,
                              const float* ff, void* O, float* LSE, hipStream_t st) {
  const dim3 g = flash_grid(d.N, Bs, d.Hq, d.B);
  float sl = d.scale * 1.4426950408889634f;
  if (d.D == 64)
    // two query tiles per wave (256-query workgroups)
    { MuseProf prof_("k_flash_fwd", st); hipLaunchKernelGGL(k_flash_fwd2, flash_grid(d.N, Bs, d.Hq, d.B, 256), dim3(256), 0, st, (const bf16_t*)Q, (const bf16_t*)K, (const bf16_t*)V, ff,
                       (bf16_t*)O, LSE, d.N, Bs, d.Hq, d.Hkv, d.B, sl); }
  else
    { MuseProf prof_("k_flash_fwd", st); hipLaunchKernelGGL(k_flash_fwd<128>, g, dim3(256), 0, st, (const bf16_t*)Q, (const bf16_t*)K, (const bf16_t*)V, ff,
                       (bf16_t*)O, LSE, d.N, Bs, d.Hq, d.Hkv, d.B, sl); }
  MUSE_LAUNCH_CHECK();
  return MUSE_OK;
}

int muse_launch_attn_bwd_mfma(const MuseDims& d, int Bs, const void* Q, const void* K, const void* V,
                              const void* dO, const float* LSE, const float* delta, float* dQacc,
                              float* dKacc, float* dVacc, hipStream_t st) {
  const dim3 gq = flash_grid(d.N, Bs, d.Hq, d.B), gk = flash_grid(d.N, Bs, d.Hkv, d.B);
  float sl = d.scale * 1.4426950408889634f;
  const bf16_t *q = (const bf16_t*)Q, *k = (const bf16_t*)K, *v = (const bf16_t*)V, *g = (const bf16_t*)dO;
  if (d.D == 64) {
    { MuseProf prof_("k_flash_bwd_dq", st); hipLaunchKernelGGL(k_flash_bwd_dq<64>, gq, dim3(256), 0, st, q, k, v, g, LSE, delta, dQacc, d.N, Bs, d.Hq, d.Hkv, d.B, d.scale, sl); }
    { MuseProf prof_("k_flash_bwd_dkv", st); hipLaunchKernelGGL(k_flash_bwd_dkv_p<64>, gk, dim3(256), 0, st, q, k, v, g, LSE, delta, dKacc, dVacc, d.N, Bs, d.Hq, d.Hkv, d.B, d.scale, sl); }
  } else {
    { MuseProf prof_("k_flash_bwd_dq", st); hipLaunchKernelGGL(k_flash_bwd_dq<128>, gq, dim3(256), 0, st, q, k, v, g, LSE, delta, dQacc, d.N, Bs, d.Hq, d.Hkv, d.B, d.scale, sl); }
    { MuseProf prof_("k_flash_bwd_dkv", st); hipLaunchKernelGGL(k_flash_bwd_dkv<128>, gk, dim3(256), 0, st, q, k, v, g, LSE, delta, dKacc, dVacc, d.N, Bs, d.Hq, d.Hkv, d.B, d.scale, sl); }
  }
  MUSE_LAUNCH_CHECK();
  return MUSE_OK;
}
