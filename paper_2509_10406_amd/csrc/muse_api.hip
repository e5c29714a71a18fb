// C-ABI entry points of libmuse: argument validation on the host, workspace carving, stage order.
#include <cstdlib>
#include <math.h>

#include <stdio.h>
#include <string.h>

#include <map>
#include <string>
#include <vector>

#include "common.h"

// farfield.hip
size_t muse_farfield_ws_bytes(const MuseDims& d, bool bwd, int heads_at_once);
size_t muse_farfield_fixed_bytes(const MuseDims& d, bool bwd);
int muse_run_fwd(const MuseDims& d, const void* Q, const void* K, const void* V, const float* qc,
                 const int32_t* aq, const int32_t* ak, void* O, float* LSE, int32_t* selc, int32_t* selb,
                 void* ws, size_t ws_bytes, hipStream_t st);
int muse_run_bwd(const MuseDims& d, const void* Q, const void* K, const void* V, const void* O, const float* LSE,
                 const void* dO, const float* qc, const int32_t* aq, const int32_t* ak, const int32_t* selc,
                 const int32_t* selb, void* dQ, void* dK, void* dV, void* ws, size_t ws_bytes, hipStream_t st);

// ---- per-kernel timing (diagnostics) ---------------------------------------------------------
namespace {
struct ProfRec { const char* name; hipEvent_t a, b; };
bool g_prof_on = false;
}  // namespace
bool muse_profiling() { return g_prof_on; }

MuseAux& muse_aux_stream() {
  static MuseAux a[64];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) dev = 0;
  MuseAux& x = a[dev];
  if (x.state == 0) {
    const char* serial = getenv("MUSE_SERIAL_STREAMS");  // "1": everything on the caller's stream
    if (serial && serial[0] == '1') { x.state = -1; return x; }
    x.state = (hipStreamCreateWithFlags(&x.s, hipStreamNonBlocking) == hipSuccess &&
               hipEventCreateWithFlags(&x.fork, hipEventDisableTiming) == hipSuccess &&
               hipEventCreateWithFlags(&x.join, hipEventDisableTiming) == hipSuccess &&
               hipEventCreateWithFlags(&x.mid, hipEventDisableTiming) == hipSuccess)
                  ? 1 : -1;
  }
  return x;
}
namespace {
std::vector<ProfRec> g_prof;
}  // namespace

MuseProf::MuseProf(const char* name, hipStream_t st) : name_(name), st_(st), slot_(-1) {
  if (!g_prof_on) return;
  ProfRec r{name, nullptr, nullptr};
  if (hipEventCreate(&r.a) != hipSuccess || hipEventCreate(&r.b) != hipSuccess) return;
  (void)hipEventRecord(r.a, st);
  g_prof.push_back(r);
  slot_ = (int)g_prof.size() - 1;
}
MuseProf::~MuseProf() {
  if (slot_ >= 0) (void)hipEventRecord(g_prof[slot_].b, st_);
}

namespace {

size_t al(size_t x) { return (x + 255) & ~(size_t)255; }

// validates and derives; `full` = the clustering / MuSe fields matter too
int make_dims(const muse_params* p, bool full, MuseDims* d) {
  if (!p) return MUSE_ERR_INVALID_ARG;
  if (p->B < 1 || p->Hq < 1 || p->Hkv < 1 || p->N < 1 || p->Hq % p->Hkv) return MUSE_ERR_INVALID_ARG;
  if (p->dtype != MUSE_DTYPE_FP32 && p->dtype != MUSE_DTYPE_BF16) return MUSE_ERR_INVALID_ARG;
  if (p->grad_dtype != MUSE_DTYPE_FP32 && p->grad_dtype != p->dtype) return MUSE_ERR_INVALID_ARG;
  if (p->flags & ~(uint32_t)(MUSE_FLAG_KEEP_FWD_STATE | MUSE_FLAG_FROZEN_WEIGHTS | MUSE_FLAG_STREAMING_KMEANS | MUSE_FLAG_BALANCED_ASSIGN | MUSE_FLAG_DIPOLE)) return MUSE_ERR_INVALID_ARG;
  d->keep_state = (p->flags & MUSE_FLAG_KEEP_FWD_STATE) != 0;
  d->frozen_weights = (p->flags & MUSE_FLAG_FROZEN_WEIGHTS) != 0;
  d->streaming = (p->flags & MUSE_FLAG_STREAMING_KMEANS) != 0;
  d->balanced = (p->flags & MUSE_FLAG_BALANCED_ASSIGN) != 0;
  d->dipole = false;
  if (!(p->scale >= 0.f) || isinf(p->scale)) return MUSE_ERR_INVALID_ARG;
  if (p->causal != 1) return MUSE_ERR_UNSUPPORTED;
  if (p->D != 64 && p->D != 128) return MUSE_ERR_UNSUPPORTED;
  if (p->Hq / p->Hkv > 8 || p->N > (1 << 22)) return MUSE_ERR_UNSUPPORTED;
  d->B = p->B; d->Hq = p->Hq; d->Hkv = p->Hkv; d->N = p->N; d->D = p->D;
  d->dtype = p->dtype; d->grad_dtype = p->grad_dtype;
  d->scale = p->scale > 0.f ? p->scale : 1.0f / sqrtf((float)p->D);
  d->Cq = d->Ck = 1; d->r = 0; d->k2 = 1; d->k2e = 1; d->Bs = p->N; d->nb = 1; d->T = 0;
  if (!full) return MUSE_OK;
  int Bs = p->block > 0 ? p->block : p->N / 8;
  if (p->block < 0 || Bs < 1 || p->N % Bs) return MUSE_ERR_INVALID_ARG;
  if (p->Cq < 1 || p->Ck < 1 || p->Cq > p->N || p->Ck > p->N) return MUSE_ERR_INVALID_ARG;
  if (p->r < 0 || p->r > p->Ck || p->k2 < 0 || p->kmeans_iters < 0) return MUSE_ERR_INVALID_ARG;
  if (p->Cq > MUSE_MAX_CLUSTERS || p->Ck > MUSE_MAX_CLUSTERS || p->r > 32 || p->N / Bs > 16 || Bs > 16384) return MUSE_ERR_UNSUPPORTED;
  d->Bs = Bs; d->nb = p->N / Bs; d->Cq = p->Cq; d->Ck = p->Ck;
  d->r = p->r;
  d->k2 = p->k2; d->T = p->kmeans_iters;
  d->k2e = p->k2 > 0 ? p->k2 : (d->nb > 1 ? d->nb - 1 : 1);
  if (d->k2e > 16) return MUSE_ERR_UNSUPPORTED;
  d->dipole = (p->flags & MUSE_FLAG_DIPOLE) != 0;
  if (d->dipole && d->r > 0) return MUSE_ERR_UNSUPPORTED;  // App. B "Compatibility with Retrieval": not combined
  return MUSE_OK;
}

// ---- stamp at the head of every workspace (MUSE_FLAG_KEEP_FWD_STATE) -------------------------
// The first kTagBytes of a workspace belong to the stamp; every layout starts behind it.
constexpr size_t kTagBytes = 256;
constexpr uint64_t kTagMagic = 0x4d755365a7c3f10bull;

__global__ void k_stamp(uint64_t* tag, uint64_t a, uint64_t b, uint64_t c, uint64_t d) {
  if (threadIdx.x == 0) { tag[0] = a; tag[1] = b; tag[2] = c; tag[3] = d; }
}

// what muse_bwd must find: the params that shape the forward state (the flags that only the backward reads
// left out), folded FNV-1a style
uint64_t params_hash(const muse_params* p) {
  muse_params q = *p;
  q.flags &= ~(uint32_t)MUSE_FLAG_FROZEN_WEIGHTS;
  const int32_t f[] = {q.B, q.Hq, q.Hkv, q.N, q.D, q.Cq, q.Ck, q.r, q.k2, q.block, q.dtype, q.causal, (int32_t)q.flags};
  uint64_t h = 0xcbf29ce484222325ull;
  auto mix = [&](uint32_t v) { for (int i = 0; i < 4; ++i) { h ^= (v >> (8 * i)) & 0xffu; h *= 0x100000001b3ull; } };
  for (int32_t v : f) mix((uint32_t)v);
  uint32_t sc; memcpy(&sc, &q.scale, 4);
  mix(sc);
  return h;
}

int stamp_clear(void* ws, hipStream_t st) {
  hipLaunchKernelGGL(k_stamp, dim3(1), dim3(64), 0, st, (uint64_t*)ws, 0ull, 0ull, 0ull, 0ull);
  MUSE_LAUNCH_CHECK();
  return MUSE_OK;
}
int stamp_write(void* ws, size_t ws_bytes, const muse_params* p, hipStream_t st) {
  hipLaunchKernelGGL(k_stamp, dim3(1), dim3(64), 0, st, (uint64_t*)ws, kTagMagic, params_hash(p),
                     (uint64_t)(uintptr_t)ws, (uint64_t)ws_bytes);
  MUSE_LAUNCH_CHECK();
  return MUSE_OK;
}
// waits for the work queued on st so far (the stamp is the last thing muse_fwd enqueues)
int stamp_check(void* ws, size_t ws_bytes, const muse_params* p, hipStream_t st) {
  uint64_t got[4] = {0, 0, 0, 0};
  MUSE_HIP_CHECK(hipMemcpyAsync(got, ws, sizeof(got), hipMemcpyDeviceToHost, st));
  MUSE_HIP_CHECK(hipStreamSynchronize(st));
  // the workspace may be larger than at the forward call as long as it starts at the same address: the layout
  // of the kept state depends on the params only (all heads in one chunk)
  if (got[0] != kTagMagic || got[1] != params_hash(p) || got[2] != (uint64_t)(uintptr_t)ws || got[3] > (uint64_t)ws_bytes)
    return MUSE_ERR_STATE;
  return MUSE_OK;
}

// App. C "Balanced Assignment": cap = floor(4 block / C) rows of a block per cluster must exist and leave room
// for every row of the block
bool balanced_cap_ok(const MuseDims& d, int C) {
  const long long cap = (4LL * d.Bs) / C;
  return cap >= 1 && cap * C >= d.Bs;
}

size_t exact_bwd_bytes(const MuseDims& d) {
  size_t q = (size_t)d.B * d.Hq * d.N, k = (size_t)d.B * d.Hkv * d.N;
  size_t b = al(q * 4);  // delta
  if (d.grad_dtype != MUSE_DTYPE_FP32) b += al(q * d.D * 4) + 2 * al(k * d.D * 4);
  return b;
}

}  // namespace

extern "C" {

const char* muse_strerror(int code) {
  switch (code) {
    case MUSE_OK: return "ok";
    case MUSE_ERR_INVALID_ARG: return "invalid argument";
    case MUSE_ERR_UNSUPPORTED: return "unsupported configuration";
    case MUSE_ERR_WORKSPACE_TOO_SMALL: return "workspace too small";
    case MUSE_ERR_HIP: return "HIP runtime error";
    case MUSE_ERR_STATE: return "workspace does not hold the forward state of these params";
    case MUSE_ERR_SCRATCH_LIMIT: return "input needs more scratch than the no-allocation entry point holds";
    default: return "unknown error code";
  }
}

int muse_workspace_bytes(const muse_params* p, int which, size_t* min_bytes, size_t* preferred) {
  if (!min_bytes) return MUSE_ERR_INVALID_ARG;
  MuseDims d;
  bool full = which == MUSE_WS_CLUSTER || which == MUSE_WS_FWD || which == MUSE_WS_BWD;
  int rc = make_dims(p, full, &d);
  if (rc) return rc;
  size_t mn = 0, pref = 0;
  switch (which) {
    case MUSE_WS_CLUSTER: mn = pref = 2 * muse_cluster_ws_bytes(d); break;  // queries and keys side by side
    case MUSE_WS_EXACT_FWD: mn = pref = 0; break;  // unused: the stamp slot alone
    case MUSE_WS_EXACT_BWD: mn = pref = exact_bwd_bytes(d); break;
    case MUSE_WS_FWD:
    case MUSE_WS_BWD: {
      if (which == MUSE_WS_BWD && d.dipole) return MUSE_ERR_UNSUPPORTED;
      bool bwd = which == MUSE_WS_BWD || d.keep_state;
      pref = muse_farfield_fixed_bytes(d, bwd) + muse_farfield_ws_bytes(d, bwd, d.B * d.Hq);
      mn = d.keep_state ? pref : muse_farfield_fixed_bytes(d, bwd) + muse_farfield_ws_bytes(d, bwd, 1);
      break;
    }
    default: return MUSE_ERR_INVALID_ARG;
  }
  *min_bytes = mn + kTagBytes;
  if (preferred) *preferred = pref + kTagBytes;
  return MUSE_OK;
}

int muse_cluster(const muse_params* p, const void* Q, const void* K, const int32_t* q_init_idx,
                 const int32_t* k_init_idx, float* q_centroids, int32_t* q_assign, float* k_centroids,
                 int32_t* k_assign, void* ws, size_t ws_bytes, void* stream) {
  MuseDims d;
  int rc = make_dims(p, true, &d);
  if (rc) return rc;
  if (!Q && !K) return MUSE_ERR_INVALID_ARG;
  if (Q && (!q_centroids || !q_assign)) return MUSE_ERR_INVALID_ARG;
  if (K && (!k_centroids || !k_assign)) return MUSE_ERR_INVALID_ARG;
  if (!ws) return MUSE_ERR_INVALID_ARG;
  if (d.balanced) {  // the cap of App. C must leave room for every row of a block
    if (Q && !balanced_cap_ok(d, d.Cq)) return MUSE_ERR_UNSUPPORTED;
    if (K && !balanced_cap_ok(d, d.Ck)) return MUSE_ERR_UNSUPPORTED;
  }
  if (ws_bytes < kTagBytes + 2 * muse_cluster_ws_bytes(d)) return MUSE_ERR_WORKSPACE_TOO_SMALL;
  hipStream_t st = (hipStream_t)stream;
  if ((rc = stamp_clear(ws, st))) return rc;
  char* w0 = (char*)ws + kTagBytes;
  // the two problems are independent: the keys go to the second stream (own half of the workspace)
  MuseAux& ax = muse_aux_stream();
  const bool two = Q && K && ax.state == 1 && !muse_profiling();
  hipStream_t sk = two ? ax.s : st;
  if (two) {
    MUSE_HIP_CHECK(hipEventRecord(ax.fork, st));
    MUSE_HIP_CHECK(hipStreamWaitEvent(sk, ax.fork, 0));
  }
  int rck = MUSE_OK, rcq = MUSE_OK;
  if (K) rck = muse_launch_cluster(d, K, d.Hkv, d.Ck, k_init_idx, k_centroids, k_assign, nullptr, nullptr, w0 + muse_cluster_ws_bytes(d), sk);
  // whatever happened, the caller's stream waits for what the second stream was given
  if (two && (hipEventRecord(ax.join, sk) != hipSuccess || hipStreamWaitEvent(st, ax.join, 0) != hipSuccess)) return MUSE_ERR_HIP;
  if (rck) return rck;
  if (Q) rcq = muse_launch_cluster(d, Q, d.Hq, d.Cq, q_init_idx, q_centroids, q_assign, nullptr, nullptr, w0, st);
  return rcq;
}

int muse_kmeans_stream(const muse_params* p, int side, const void* X, const int32_t* init_idx, float* centroids,
                       int32_t* stream_assign, float* counts, void* ws, size_t ws_bytes, void* stream) {
  MuseDims d;
  int rc = make_dims(p, true, &d);
  if (rc) return rc;
  if ((side != 0 && side != 1) || !X || !centroids || !ws) return MUSE_ERR_INVALID_ARG;
  if (ws_bytes < kTagBytes + muse_cluster_ws_bytes(d)) return MUSE_ERR_WORKSPACE_TOO_SMALL;
  d.streaming = true;
  if ((rc = stamp_clear(ws, (hipStream_t)stream))) return rc;
  return muse_launch_cluster(d, X, side ? d.Hkv : d.Hq, side ? d.Ck : d.Cq, init_idx, centroids, nullptr, stream_assign,
                             counts, (char*)ws + kTagBytes, (hipStream_t)stream);
}

int muse_fwd(const muse_params* p, const void* Q, const void* K, const void* V, const float* q_centroids,
             const int32_t* q_assign, const int32_t* k_assign, void* O, float* LSE, int32_t* sel_clusters,
             int32_t* sel_blocks, void* ws, size_t ws_bytes, void* stream) {
  MuseDims d;
  int rc = make_dims(p, true, &d);
  if (rc) return rc;
  if (!Q || !K || !V || !q_centroids || !q_assign || !k_assign || !O || !LSE || !ws) return MUSE_ERR_INVALID_ARG;
  if (d.r > 0 && (!sel_clusters || !sel_blocks)) return MUSE_ERR_INVALID_ARG;
  size_t need = d.keep_state ? muse_farfield_fixed_bytes(d, true) + muse_farfield_ws_bytes(d, true, d.B * d.Hq)
                             : muse_farfield_fixed_bytes(d, false) + muse_farfield_ws_bytes(d, false, 1);
  if (ws_bytes < kTagBytes + need) return MUSE_ERR_WORKSPACE_TOO_SMALL;
  hipStream_t st = (hipStream_t)stream;
  if ((rc = stamp_clear(ws, st))) return rc;
  rc = muse_run_fwd(d, Q, K, V, q_centroids, q_assign, k_assign, O, LSE, sel_clusters, sel_blocks, (char*)ws + kTagBytes,
                    ws_bytes - kTagBytes, st);
  if (rc == MUSE_OK && d.keep_state) rc = stamp_write(ws, ws_bytes, p, st);
  return rc;
}

int muse_bwd(const muse_params* p, const void* Q, const void* K, const void* V, const void* O, const float* LSE,
             const void* dO, const float* q_centroids, const int32_t* q_assign, const int32_t* k_assign,
             const int32_t* sel_clusters, const int32_t* sel_blocks, void* dQ, void* dK, void* dV, void* ws,
             size_t ws_bytes, void* stream) {
  MuseDims d;
  int rc = make_dims(p, true, &d);
  if (rc) return rc;
  if (!Q || !K || !V || !O || !LSE || !dO || !q_centroids || !q_assign || !k_assign || !dQ || !dK || !dV || !ws)
    return MUSE_ERR_INVALID_ARG;
  if (d.r > 0 && (!sel_clusters || !sel_blocks)) return MUSE_ERR_INVALID_ARG;
  if (d.dipole) return MUSE_ERR_UNSUPPORTED;  // the dipole correction has a forward only
  size_t need = muse_farfield_fixed_bytes(d, true) + muse_farfield_ws_bytes(d, true, d.keep_state ? d.B * d.Hq : 1);
  if (ws_bytes < kTagBytes + need) return MUSE_ERR_WORKSPACE_TOO_SMALL;
  hipStream_t st = (hipStream_t)stream;
  if (d.keep_state) {
    if ((rc = stamp_check(ws, ws_bytes, p, st))) return rc;
  } else if ((rc = stamp_clear(ws, st))) {
    return rc;
  }
  return muse_run_bwd(d, Q, K, V, O, LSE, dO, q_centroids, q_assign, k_assign, sel_clusters, sel_blocks, dQ, dK, dV,
                      (char*)ws + kTagBytes, ws_bytes - kTagBytes, st);
}

int exact_attn_fwd(const muse_params* p, const void* Q, const void* K, const void* V, void* O, float* LSE,
                   void* ws, size_t ws_bytes, void* stream) {
  (void)ws; (void)ws_bytes;
  MuseDims d;
  int rc = make_dims(p, false, &d);
  if (rc) return rc;
  if (!Q || !K || !V || !O || !LSE) return MUSE_ERR_INVALID_ARG;
  return muse_launch_attn_fwd(d, d.N, Q, K, V, nullptr, O, LSE, (hipStream_t)stream);
}

int exact_attn_bwd(const muse_params* p, const void* Q, const void* K, const void* V, const void* O,
                   const float* LSE, const void* dO, void* dQ, void* dK, void* dV, void* ws, size_t ws_bytes,
                   void* stream) {
  MuseDims d;
  int rc = make_dims(p, false, &d);
  if (rc) return rc;
  if (!Q || !K || !V || !O || !LSE || !dO || !dQ || !dK || !dV || !ws) return MUSE_ERR_INVALID_ARG;
  if (ws_bytes < kTagBytes + exact_bwd_bytes(d)) return MUSE_ERR_WORKSPACE_TOO_SMALL;
  hipStream_t st = (hipStream_t)stream;
  if ((rc = stamp_clear(ws, st))) return rc;
  size_t q = (size_t)d.B * d.Hq * d.N, k = (size_t)d.B * d.Hkv * d.N;
  char* w = (char*)ws + kTagBytes;
  float* delta = (float*)w; w += al(q * 4);
  float *aq, *ak, *av;
  bool direct = d.grad_dtype == MUSE_DTYPE_FP32;
  if (direct) {
    aq = (float*)dQ; ak = (float*)dK; av = (float*)dV;
  } else {
    aq = (float*)w; w += al(q * d.D * 4);
    ak = (float*)w; w += al(k * d.D * 4);
    av = (float*)w;
  }
  if ((rc = muse_launch_delta(d, O, dO, delta, st))) return rc;
  if ((rc = muse_launch_attn_bwd(d, d.N, Q, K, V, dO, LSE, delta, aq, ak, av, st))) return rc;
  if (!direct) {
    if ((rc = muse_launch_cast(aq, dQ, q * d.D, d.grad_dtype, 1.f, st))) return rc;
    if ((rc = muse_launch_cast(ak, dK, k * d.D, d.grad_dtype, 1.f, st))) return rc;
    if ((rc = muse_launch_cast(av, dV, k * d.D, d.grad_dtype, 1.f, st))) return rc;
  }
  return MUSE_OK;
}

// ---- exact_attn_bwd for callers that cannot allocate ------------------------------------------
// The scratch of exact_attn_bwd (delta, and the fp32 accumulators when the gradients leave in bf16) lives in a
// file-scope device array instead of a caller workspace.  In host code the array's name is only a handle: its
// device address is looked up once per device and kept.
static __device__ __align__(256) unsigned char scratch[MUSE_STATIC_SCRATCH_BYTES];
namespace {
void* g_scratch_ptr[64];  // per device, NULL until the first call on it
}

int exact_attn_bwd_static(const muse_params* p, const void* Q, const void* K, const void* V, const void* O,
                          const float* LSE, const void* dO, void* dQ, void* dK, void* dV, void* stream) {
  MuseDims d;
  int rc = make_dims(p, false, &d);
  if (rc) return rc;
  if (!Q || !K || !V || !O || !LSE || !dO || !dQ || !dK || !dV) return MUSE_ERR_INVALID_ARG;
  if (kTagBytes + exact_bwd_bytes(d) > (size_t)MUSE_STATIC_SCRATCH_BYTES) return MUSE_ERR_SCRATCH_LIMIT;
  if (muse_profiling()) return MUSE_ERR_UNSUPPORTED;  // the per-kernel timing creates events
  int dev = 0;
  MUSE_HIP_CHECK(hipGetDevice(&dev));
  if (dev < 0 || dev >= 64) return MUSE_ERR_UNSUPPORTED;
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    MUSE_HIP_CHECK(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
    if (!ptr) return MUSE_ERR_HIP;
    g_scratch_ptr[dev] = ptr;
  }
  return exact_attn_bwd(p, Q, K, V, O, LSE, dO, dQ, dK, dV, g_scratch_ptr[dev], (size_t)MUSE_STATIC_SCRATCH_BYTES, stream);
}

int muse_profile_enable(int on) {
  for (auto& r : g_prof) { (void)hipEventDestroy(r.a); (void)hipEventDestroy(r.b); }
  g_prof.clear();
  g_prof_on = on != 0;
  return MUSE_OK;
}

int muse_profile_report(char* buf, size_t cap) {
  if (!buf || cap == 0) return MUSE_ERR_INVALID_ARG;
  std::map<std::string, std::pair<int, double>> agg;
  for (auto& r : g_prof) {
    if (hipEventSynchronize(r.b) != hipSuccess) return MUSE_ERR_HIP;
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, r.a, r.b) != hipSuccess) return MUSE_ERR_HIP;
    auto& e = agg[r.name];
    e.first += 1;
    e.second += ms;
  }
  size_t used = 0;
  buf[0] = 0;
  for (auto& kv : agg) {
    int n = snprintf(buf + used, cap - used, "%s %d %.6f\n", kv.first.c_str(), kv.second.first, kv.second.second);
    if (n < 0 || (size_t)n >= cap - used) return MUSE_ERR_INVALID_ARG;
    used += (size_t)n;
  }
  return MUSE_OK;
}

}  // extern "C"
