// Shared device helpers for the MuSe kernels (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/muse.h"

typedef uint16_t bf16_t;  // raw bfloat16 bits

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;

#define MUSE_WAVE 64
#define MUSE_MAX_CLUSTERS 2048  // largest Cq / Ck the host accepts (LDS tables of the bucketing and chain kernels)
#define MUSE_NEG_INF (-__builtin_huge_valf())

__device__ __forceinline__ float bf16_bits_to_f32(bf16_t h) {
  return __uint_as_float(((uint32_t)h) << 16);
}

// round-to-nearest-even by the hardware conversion (v_cvt_pk_bf16_f32 takes two values per instruction; the same
// rounding written out in integer arithmetic costs about seven instructions per value)
__device__ __forceinline__ bf16_t f32_to_bf16_bits(float f) { return __builtin_bit_cast(bf16_t, (__bf16)f); }

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_raw_t;
  const bf16x2_raw_t v = {(__bf16)lo, (__bf16)hi};
  return __builtin_bit_cast(uint32_t, v);
}

template <typename T>
struct Elem;
template <>
struct Elem<float> {
  static constexpr int kBytes = 4;
  __device__ static __forceinline__ float ld(const float* p, size_t i) { return p[i]; }
  __device__ static __forceinline__ void st(float* p, size_t i, float v) { p[i] = v; }
};
template <>
struct Elem<bf16_t> {
  static constexpr int kBytes = 2;
  __device__ static __forceinline__ float ld(const bf16_t* p, size_t i) { return bf16_bits_to_f32(p[i]); }
  __device__ static __forceinline__ void st(bf16_t* p, size_t i, float v) { p[i] = f32_to_bf16_bits(v); }
};

// loads 4 consecutive elements (address must be aligned to 4 elements)
__device__ __forceinline__ void ld4(const float* p, size_t i, float out[4]) {
  float4 v = *reinterpret_cast<const float4*>(p + i);
  out[0] = v.x; out[1] = v.y; out[2] = v.z; out[3] = v.w;
}
__device__ __forceinline__ void ld4(const bf16_t* p, size_t i, float out[4]) {
  uint2 v = *reinterpret_cast<const uint2*>(p + i);
  out[0] = __uint_as_float(v.x << 16); out[1] = __uint_as_float(v.x & 0xffff0000u);
  out[2] = __uint_as_float(v.y << 16); out[3] = __uint_as_float(v.y & 0xffff0000u);
}
// a pair of consecutive elements, raw (address aligned to 2 elements), and its two halves as floats
template <typename T>
struct Pair;
template <>
struct Pair<float> {
  using raw = float2;
  __device__ static __forceinline__ raw ld(const float* p, size_t i) { return *reinterpret_cast<const float2*>(p + i); }
  __device__ static __forceinline__ float lo(raw v) { return v.x; }
  __device__ static __forceinline__ float hi(raw v) { return v.y; }
};
template <>
struct Pair<bf16_t> {
  using raw = uint32_t;
  __device__ static __forceinline__ raw ld(const bf16_t* p, size_t i) { return *reinterpret_cast<const uint32_t*>(p + i); }
  __device__ static __forceinline__ float lo(raw v) { return __uint_as_float(v << 16); }
  __device__ static __forceinline__ float hi(raw v) { return __uint_as_float(v & 0xffff0000u); }
};
// DT consecutive elements (DT = 2 or 4, address aligned to DT elements), raw, with compile-time element access
template <typename T, int DT>
struct Frag;
template <>
struct Frag<float, 2> {
  using raw = float2;
  __device__ static __forceinline__ raw ld(const float* p, size_t i) { return *reinterpret_cast<const float2*>(p + i); }
  __device__ static __forceinline__ float get(const raw& v, int x) { return x ? v.y : v.x; }
};
template <>
struct Frag<float, 4> {
  using raw = float4;
  __device__ static __forceinline__ raw ld(const float* p, size_t i) { return *reinterpret_cast<const float4*>(p + i); }
  __device__ static __forceinline__ float get(const raw& v, int x) { return x == 0 ? v.x : x == 1 ? v.y : x == 2 ? v.z : v.w; }
};
template <>
struct Frag<bf16_t, 2> {
  using raw = uint32_t;
  __device__ static __forceinline__ raw ld(const bf16_t* p, size_t i) { return *reinterpret_cast<const uint32_t*>(p + i); }
  __device__ static __forceinline__ float get(const raw& v, int x) { return __uint_as_float(x ? (v & 0xffff0000u) : (v << 16)); }
};
template <>
struct Frag<bf16_t, 4> {
  using raw = uint2;
  __device__ static __forceinline__ raw ld(const bf16_t* p, size_t i) { return *reinterpret_cast<const uint2*>(p + i); }
  __device__ static __forceinline__ float get(const raw& v, int x) {
    const uint32_t w = x < 2 ? v.x : v.y;
    return __uint_as_float((x & 1) ? (w & 0xffff0000u) : (w << 16));
  }
};
__device__ __forceinline__ void st4(float* p, size_t i, const float v[4]) {
  *reinterpret_cast<float4*>(p + i) = make_float4(v[0], v[1], v[2], v[3]);
}
__device__ __forceinline__ void st4(bf16_t* p, size_t i, const float v[4]) {
  *reinterpret_cast<uint2*>(p + i) = make_uint2(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]));
}

// the same as streaming stores: for rows that are written once and read much later (the summaries and the cell
// gradients are several GB per head chunk; nothing of them is still in a cache when it is read)
__device__ __forceinline__ void st4_stream(float* p, size_t i, const float v[4]) {
  typedef float f4_t __attribute__((ext_vector_type(4)));
  const f4_t x = {v[0], v[1], v[2], v[3]};
  __builtin_nontemporal_store(x, reinterpret_cast<f4_t*>(p + i));
}
__device__ __forceinline__ void st4_stream(bf16_t* p, size_t i, const float v[4]) {
  const unsigned long long x = (unsigned long long)pack_bf16x2(v[0], v[1]) | ((unsigned long long)pack_bf16x2(v[2], v[3]) << 32);
  __builtin_nontemporal_store(x, reinterpret_cast<unsigned long long*>(p + i));
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
// Sums over aligned groups of 4, 8 or 16 lanes, result in every lane of the group, by DPP moves inside a row
// of 16 lanes (quad swaps, half-row mirror, row mirror): pure VALU, where a shuffle goes through the LDS
// crossbar.  The lanes of a group must be active together.
template <int CTRL>
__device__ __forceinline__ float dpp_add(float v) {
  return v + __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, false));
}
template <int G>
__device__ __forceinline__ float group_sum(float v) {
  static_assert(G == 4 || G == 8 || G == 16, "group of 4, 8 or 16 lanes");
  v = dpp_add<0xB1>(v);                        // quad_perm [1,0,3,2]
  v = dpp_add<0x4E>(v);                        // quad_perm [2,3,0,1]
  if constexpr (G >= 8) v = dpp_add<0x141>(v);   // row_half_mirror
  if constexpr (G >= 16) v = dpp_add<0x140>(v);  // row_mirror
  return v;
}
// sum over the 64 lanes, in every lane: row sums by DPP, then the four rows through scalar registers
__device__ __forceinline__ float wave_sum_dpp(float v) {
  v = group_sum<16>(v);
  const float r0 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 0));
  const float r1 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 16));
  const float r2 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 32));
  const float r3 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 48));
  return (r0 + r1) + (r2 + r3);
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

// Orders LDS traffic between the lanes of ONE wave (a block of 64 threads): the LDS pipeline serves a
// wave's requests in issue order, so a compiler-level fence is all that is needed; unlike
// __syncthreads() it does not wait for outstanding global stores.
__device__ __forceinline__ void wave_lds_fence() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// host-side launch parameters shared by the translation units
struct MuseDims {
  int B, Hq, Hkv, N, D, Cq, Ck, r, k2, k2e, Bs, nb, T;
  int dtype, grad_dtype;
  float scale;
  bool keep_state;  // MUSE_FLAG_KEEP_FWD_STATE
  bool frozen_weights;  // MUSE_FLAG_FROZEN_WEIGHTS
  bool streaming;       // MUSE_FLAG_STREAMING_KMEANS
  bool balanced;        // MUSE_FLAG_BALANCED_ASSIGN
  bool dipole;          // MUSE_FLAG_DIPOLE
};

#define MUSE_HIP_CHECK(expr)                      \
  do {                                            \
    hipError_t e__ = (expr);                      \
    if (e__ != hipSuccess) return MUSE_ERR_HIP;   \
  } while (0)

#define MUSE_LAUNCH_CHECK()                                   \
  do {                                                        \
    if (hipGetLastError() != hipSuccess) return MUSE_ERR_HIP; \
  } while (0)

// A second stream per device for stages that are independent of each other until a later join (the two
// K-means problems; the block-diagonal backward beside the far field).  Created on first use, default
// priority, non-blocking w.r.t. the null stream; the streams meet through the two events.  state: 0 untried,
// 1 ready, -1 unavailable (everything then runs on the caller's stream).  Calls of one process that overlap
// in time on one device would share it: they must be issued from one host thread at a time.
struct MuseAux {
  hipStream_t s = nullptr;
  hipEvent_t fork = nullptr, join = nullptr, mid = nullptr;
  int state = 0;
};
MuseAux& muse_aux_stream();

// Optional per-kernel timing (diagnostics for the benchmark): when enabled through
// muse_profile_enable, every launch is bracketed by HIP events on its stream.
// While profiling is on, everything runs on the caller's stream so that durations do not overlap.
bool muse_profiling();
struct MuseProf {
  MuseProf(const char* name, hipStream_t st);
  ~MuseProf();
  const char* name_;
  hipStream_t st_;
  int slot_;
};

// ---- stage launchers (one per translation unit) ------------------------------------------
// kmeans.hip
size_t muse_cluster_ws_bytes(const MuseDims& d);
// d.streaming: the centroids come from the streaming pass (trace [heads,N], counts [heads,C]: optional outputs
// of that pass; assign may then be NULL to stop after it)
int muse_launch_cluster(const MuseDims& d, const void* X, int H, int C, const int32_t* init_idx,
                        float* cent, int32_t* assign, int32_t* trace, float* counts, void* ws, hipStream_t st);
// Stable bucketing of the N positions of every head by (spatial block, cluster):
// perm [heads, N] position lists, off [heads, nb*C + 1] segment offsets.
int muse_launch_bucket(const int32_t* assign, int heads, int N, int Bs, int C, int32_t* perm,
                       int32_t* off, hipStream_t st);

// attn_simple.hip / attn_mfma.hip: causal attention restricted to keys m with
// floor(n/Bs)*Bs <= m <= n  (Bs = N gives exact attention).  ff (may be NULL): per query
// (max, sum, acc[D]) fp32 partial softmax state in natural-log units merged into the result.
int muse_launch_attn_fwd(const MuseDims& d, int Bs, const void* Q, const void* K, const void* V,
                         const float* ff, void* O, float* LSE, hipStream_t st);
// delta [B,Hq,N] = dO . O
int muse_launch_delta(const MuseDims& d, const void* O, const void* dO, float* delta, hipStream_t st);
// dQacc [B,Hq,N,D], dKacc, dVacc [B,Hkv,N,D] fp32: overwritten with the gradients of this attention.
int muse_launch_attn_bwd(const MuseDims& d, int Bs, const void* Q, const void* K, const void* V,
                         const void* dO, const float* LSE, const float* delta, float* dQacc,
                         float* dKacc, float* dVacc, hipStream_t st);
// fp32 accumulators -> gradient tensors of grad dtype, multiplied by `mul`
int muse_launch_cast(const float* src, void* dst, size_t n, int dst_dtype, float mul, hipStream_t st);
int muse_launch_fill(float* dst, size_t n, float v, hipStream_t st);
int muse_launch_fill_i32(int32_t* dst, size_t n, int32_t v, hipStream_t st);
