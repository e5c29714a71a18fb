/*
 * libmuse — Multipole Semantic Attention (MuSe), causal, training-time, on one
 * AMD MI355X (gfx950).  C ABI; no C++ or framework types cross this boundary.
 *
 * Problem statement (Alg. 1 header): queries Q, keys K, values V of length N per
 * head, a spatial block size, cluster counts, retrieval counts k1 (= r) and k2;
 * output O of length N.  The method is Sec. 3 (Eq. 1-7) with the clustering of
 * App. C; the backward pass freezes the discrete choices and treats the query
 * centroids as constants (App. C "Centroid Gradient Flow").
 *
 * Conventions for every entry point
 *   - All tensor pointers are DEVICE pointers on the current HIP device, owned by
 *     the caller; the library never allocates, frees or keeps them.  `ws` is a
 *     caller-owned device scratch buffer of `ws_bytes` bytes, 256-byte aligned;
 *     its required size comes from muse_workspace_bytes().  Its contents are
 *     undefined before and after a call (except under MUSE_FLAG_KEEP_FWD_STATE).
 *   - `p` is a HOST pointer.  `stream` is a hipStream_t passed as void* (NULL =
 *     default stream).  Work is enqueued on that stream; calls return without
 *     synchronising (one exception: muse_bwd under MUSE_FLAG_KEEP_FWD_STATE, see there).
 *   - Process state the library keeps: per device, one extra non-blocking stream and
 *     three events, created on first use (see "Streams" below); per process, which
 *     kernels have had their dynamic-LDS limit raised; the diagnostics of
 *     muse_profile_*.  Nothing else survives a call.  Because the extra stream is
 *     shared, ONE host thread at a time may issue calls on a device; calls that use
 *     different workspaces may be queued on different streams back to back.
 *   - Layout: Q, O, dO, dQ are [B, Hq, N, D]; K, V, dK, dV are [B, Hkv, N, D];
 *     row-major, contiguous, element type given by p->dtype (fp32 or bf16).
 *     Hq % Hkv == 0; query head h uses kv head h / (Hq / Hkv) (GQA, Sec. 6).
 *   - Index inputs are trusted: q_assign / k_assign entries must lie in [0, Cq) / [0, Ck),
 *     init_idx entries in [0, N), and sel_clusters / sel_blocks must be what muse_fwd wrote
 *     for the same inputs (entries < 0 are padding).  Other values are undefined behaviour.
 *   - Return value: MUSE_OK (0) or a negative MUSE_ERR_* code.  Every check that
 *     depends only on `p`, the pointers and ws_bytes is made on the host before
 *     anything is launched: INVALID_ARG, UNSUPPORTED and WORKSPACE_TOO_SMALL mean
 *     nothing was enqueued.  MUSE_ERR_HIP (a launch or runtime call failed) can
 *     come after earlier kernels of the call were enqueued; the library's extra
 *     stream has then still been joined to `stream`, so waiting for `stream`
 *     waits for everything the call started.
 */
#ifndef MUSE_H_
#define MUSE_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  MUSE_OK = 0,
  MUSE_ERR_INVALID_ARG = -1,        /* NULL pointer, non-positive size, N % block != 0, ... */
  MUSE_ERR_UNSUPPORTED = -2,        /* non-causal, D not in {64,128}, sizes beyond the kernels' limits */
  MUSE_ERR_WORKSPACE_TOO_SMALL = -3,
  MUSE_ERR_HIP = -4,                /* a HIP call or launch failed */
  MUSE_ERR_STATE = -5,              /* MUSE_FLAG_KEEP_FWD_STATE: the workspace does not hold the forward state
                                       of these params (another workspace, other params, or overwritten) */
  MUSE_ERR_SCRATCH_LIMIT = -6       /* exact_attn_bwd_static: the input needs more than MUSE_STATIC_SCRATCH_BYTES */
};

enum { MUSE_DTYPE_FP32 = 0, MUSE_DTYPE_BF16 = 1 };
/* MUSE_FLAG_KEEP_FWD_STATE: muse_fwd lays its workspace out as muse_bwd does and leaves the bucketing and
 * the summaries there; muse_bwd called with the same flag, the same params and the SAME, untouched
 * workspace reuses them instead of recomputing (the usual save-for-backward of a training step).  Needs a
 * workspace that holds all heads at once (the `preferred` size of MUSE_WS_BWD), else
 * MUSE_ERR_WORKSPACE_TOO_SMALL.  muse_fwd stamps the head of the workspace (a hash of the params, the
 * workspace address) after its last kernel; every other entry point that is handed a workspace clears the
 * stamp.  muse_bwd reads the stamp back before it launches anything -- this waits for the work queued on
 * `stream` so far, the one place where the library synchronises -- and returns MUSE_ERR_STATE if it does not
 * match.  The stamp cannot see a caller who overwrites the middle of the workspace. */
enum { MUSE_FLAG_KEEP_FWD_STATE = 1,
/* MUSE_FLAG_FROZEN_WEIGHTS (muse_bwd only; App. C "Aggregation Weight Gradient Flow", the non-differentiable
 * variant): the tilted aggregation weights e_m / S of every summary and its log-mass mu-bar are constants of
 * the backward, so a summarised key receives a gradient only through the aggregated key, dk_m = (e_m / S) g_kbar
 * (and dv_m = (e_m / S) g_vbar as before); dQ and dV are unchanged.  The default differentiates through the
 * weights. */
       MUSE_FLAG_FROZEN_WEIGHTS = 2,
/* MUSE_FLAG_STREAMING_KMEANS (muse_cluster only; App. C "Centroid Computation"): the centroids come from the
 * single streaming pass described at muse_kmeans_stream instead of Lloyd iterations (kmeans_iters is ignored);
 * the final nearest-centroid assignment is the same. */
       MUSE_FLAG_STREAMING_KMEANS = 4,
/* MUSE_FLAG_BALANCED_ASSIGN (muse_cluster only; App. C "Balanced Assignment"): in the final assignment a cluster
 * holds at most cap = floor(4 block / C) rows of a spatial block.  Of the rows of a block that name centroid j
 * as their nearest, the first cap in sequence order keep it; the others, one after the other in sequence order,
 * go to the nearest centroid that still has room in the block at that moment (lowest index on ties).
 * MUSE_ERR_UNSUPPORTED if cap < 1 or cap * C < block. */
       MUSE_FLAG_BALANCED_ASSIGN = 8,
/* MUSE_FLAG_DIPOLE (muse_fwd only, r must be 0; App. B "Dipole Correction" with the pre-merged matrix of Eq.
 * "premerge" and the shared covariances of "Untilted (Partially Specialized) Covariances"): in the monopole-only
 * mode every query of block b >= 1 and query cluster i gets  O_n += w_far(n) C-bar_ib q~_n,  where
 * C-bar_ib = sum_j p_ib(j) Cov_0jb(v,k), Cov_0jb the equal-weight covariance of the keys of cluster j in the blocks
 * before b, p_ib the softmax over j of the accumulated log-masses, and w_far the far field's share of the query's
 * softmax mass; scores and LSE are unchanged.  MUSE_ERR_UNSUPPORTED with r > 0 (the paper does not combine the
 * merged correction with retrieval) and in muse_bwd (no backward is defined for it).  The workspace grows by the
 * covariances, 4 D^2 bytes per (kv head, key block, key cluster). */
       MUSE_FLAG_DIPOLE = 16 };
enum { MUSE_WS_CLUSTER = 0, MUSE_WS_FWD = 1, MUSE_WS_BWD = 2, MUSE_WS_EXACT_FWD = 3, MUSE_WS_EXACT_BWD = 4 };

typedef struct {
  int32_t B, Hq, Hkv;   /* batch, query heads, key/value heads */
  int32_t N, D;         /* sequence length, head dimension (64 or 128) */
  int32_t Cq, Ck;       /* number of query / key clusters (Sec. 3 "Clustering"), 1 <= C <= 2048 */
  int32_t r;            /* k1: key clusters retrieved per query (Sec. 3.2), 0 <= r <= min(Ck, 32) */
  int32_t k2;           /* spatial blocks retrieved per retrieved cluster (Sec. 3.2);
                           0 = every preceding block of a retrieved cluster */
  int32_t block;        /* spatial block size (Sec. 3 "Spatial blocks"); 0 -> N/8.  N % block == 0,
                           N/block <= 16 */
  int32_t kmeans_iters; /* T: Lloyd iterations (assign + mean update) before the final assignment */
  int32_t dtype;        /* MUSE_DTYPE_*: element type of Q,K,V,O,dO */
  int32_t grad_dtype;   /* element type of dQ,dK,dV: MUSE_DTYPE_FP32 or the same as dtype */
  int32_t causal;       /* must be 1 (the paper defines the causal form only) */
  uint32_t flags;       /* MUSE_FLAG_* bits, others must be 0 */
  float scale;          /* logit scale applied to q (Eq. 1 has none written); 0 -> 1/sqrt(D) */
} muse_params;

/* Streams: every entry point is asynchronous on `stream` (a hipStream_t; NULL = the null stream).  muse_cluster
 * and muse_bwd run stages that do not depend on each other (the two K-means problems; the block-diagonal
 * backward beside the far field) on a second, library-owned, non-blocking stream of the current device,
 * created on first use; the two streams meet through events before the entry point's last kernels, so work
 * enqueued on `stream` afterwards sees every output.  One host thread at a time may issue calls on a
 * device.  If the second stream cannot be created, or the environment variable MUSE_SERIAL_STREAMS is "1" when
 * the library first runs on the device, everything runs on `stream`.
 *
 * Storage: for bf16 inputs the value summaries, the gradients of the summaries and the bf16 part of the
 * accumulated key summaries are kept in bf16 in the workspace.  Every quantity that decides a selection keeps
 * fp32 precision: the accumulated key summaries of bf16 inputs are a bf16 plane plus an fp16 plane of the
 * remainder, and their scores against the (exact) bf16 queries accumulate in fp32. */

/* Bytes of device scratch that entry point `which` (MUSE_WS_*) needs for `p`.  The far-field
 * stages keep the summaries tensor of Sec. 3 ([Cq, Ck, N/block] cells of 2D+1 floats) in the
 * workspace for as many heads at a time as fit: any size >= the returned minimum works, and
 * *preferred (may be NULL) is the size at which all heads are processed in one pass. */
int muse_workspace_bytes(const muse_params* p, int which, size_t* min_bytes, size_t* preferred);

/* Clustering (Sec. 3 "Clustering", App. C): per head, K-means of the query rows into Cq clusters and
 * of the key rows into Ck clusters (keys once per kv head).  Initial centroid j = row init_idx[j]
 * (App. C initialisation: the caller draws a seeded shuffle and takes every floor(N/C)-th index);
 * if an init_idx pointer is NULL the initial centroids are read from the centroid buffer instead.
 * Then T = kmeans_iters times { nearest-centroid assignment; centroid <- mean of its points (an empty
 * cluster keeps its centroid) } and one final assignment.  Nearest means smallest
 * ||c||^2 - 2<x,c> (App. C, the ||x||^2 term dropped), lowest index on ties; for bf16 inputs the
 * centroids are rounded to bf16 for this score, products are exact and sums are fp32.
 *   q_init_idx [B,Hq,Cq] / k_init_idx [B,Hkv,Ck]  int32 row indices in [0,N)       (in, may be NULL)
 *   q_centroids [B,Hq,Cq,D] / k_centroids [B,Hkv,Ck,D]  fp32, centroids of the raw rows   (in/out)
 *   q_assign [B,Hq,N] / k_assign [B,Hkv,N]  int32 cluster of every row                       (out)
 * Q or K may be NULL to skip that side (its other pointers are then ignored). */
int muse_cluster(const muse_params* p, const void* Q, const void* K,
                 const int32_t* q_init_idx, const int32_t* k_init_idx,
                 float* q_centroids, int32_t* q_assign,
                 float* k_centroids, int32_t* k_assign,
                 void* ws, size_t ws_bytes, void* stream);

/* The streaming centroid pass alone, for one side (App. C "Centroid Computation", step 2): per head, the rows
 * are visited once in sequence order in minibatches of 64.  All rows of a minibatch are assigned to their
 * nearest centroid as the centroids stand when the minibatch starts (smallest ||c^||^2 - 2 <x^, c^> on binary16
 * values x^ = fp16(x), c^ = fp16(t / c), fp32 sums, lowest index on ties); then, row by row, the total and count
 * of the row's centroid become t <- 0.9 t + x^, c <- 0.9 c + 1 (fp32, one fused multiply-add each).  Totals start
 * at the row init_idx[j] with count 1; the centroid is t / c.  Rows must lie in the binary16 range.
 *   side: 0 = query rows (B*Hq heads, Cq clusters), 1 = key rows (B*Hkv heads, Ck clusters)
 *   X [B,H,N,D] dtype (in); init_idx [B,H,C] int32 (in; NULL: start from `centroids`)
 *   centroids [B,H,C,D] fp32 (in/out)
 *   stream_assign [B,H,N] int32: the centroid each row went to when its minibatch was processed (out, may be NULL)
 *   counts [B,H,C] fp32: the decayed counts c (out, may be NULL)
 *   ws: at least half of MUSE_WS_CLUSTER.
 * Errors as muse_cluster. */
int muse_kmeans_stream(const muse_params* p, int side, const void* X, const int32_t* init_idx, float* centroids,
                       int32_t* stream_assign, float* counts, void* ws, size_t ws_bytes, void* stream);

/* Forward (Sec. 3.1-3.3, Alg. 1): per-block tilted summaries (Eq. 4-6), exclusive causal
 * accumulation, cluster selection by Eq. 7, spatial block selection, exact attention on the
 * retrieved (cluster, block) pairs with the full query, exact causal attention inside the
 * query's own block, all merged in one softmax.
 *   q_centroids, q_assign, k_assign: as produced by muse_cluster (any partition is valid)   (in)
 *   O [B,Hq,N,D] dtype; LSE [B,Hq,N] fp32 log of the merged softmax normaliser             (out)
 *   sel_clusters [B,Hq,N,r] int32: retrieved key clusters in descending score order, -1 padded;
 *   sel_blocks [B,Hq,N,r,k2e] int32, k2e = k2 or N/block-1 when k2 == 0: retrieved blocks of each,
 *   descending score, -1 padded.  Required when r > 0 (muse_bwd reads them)                 (out) */
int muse_fwd(const muse_params* p, const void* Q, const void* K, const void* V,
             const float* q_centroids, const int32_t* q_assign, const int32_t* k_assign,
             void* O, float* LSE, int32_t* sel_clusters, int32_t* sel_blocks,
             void* ws, size_t ws_bytes, void* stream);

/* Backward of muse_fwd: gradient of (Q,K,V) -> O contracted with dO, with the assignments, the
 * selections and the query centroids held fixed (App. C "Centroid Gradient Flow"); gradient does flow
 * into K and V through the tilted aggregation weights (the default of App. C "Aggregation Weight
 * Gradient Flow").  O, LSE, sel_* are the outputs of muse_fwd for the same inputs.
 *   dQ [B,Hq,N,D], dK, dV [B,Hkv,N,D] of grad_dtype (summed over the query heads of a group)   (out)
 * Every sum has a single owner and a fixed order (no floating-point atomics): repeated calls, and calls
 * whose workspace forces a different chunking of the heads, return identical bits. */
int muse_bwd(const muse_params* p, const void* Q, const void* K, const void* V,
             const void* O, const float* LSE, const void* dO,
             const float* q_centroids, const int32_t* q_assign, const int32_t* k_assign,
             const int32_t* sel_clusters, const int32_t* sel_blocks,
             void* dQ, void* dK, void* dV,
             void* ws, size_t ws_bytes, void* stream);

/* Exact causal softmax attention (Sec. 3, Eq. 1-2) with the same scale, and its gradient: the
 * in-house baseline the MuSe timings are compared with.  Uses N, D, B, Hq, Hkv, dtype, grad_dtype,
 * scale of p; the other fields are ignored. */
int exact_attn_fwd(const muse_params* p, const void* Q, const void* K, const void* V,
                   void* O, float* LSE, void* ws, size_t ws_bytes, void* stream);
int exact_attn_bwd(const muse_params* p, const void* Q, const void* K, const void* V,
                   const void* O, const float* LSE, const void* dO,
                   void* dQ, void* dK, void* dV, void* ws, size_t ws_bytes, void* stream);

/* exact_attn_bwd for callers that cannot allocate device memory or pass a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and same results,
 * bit for bit, as exact_attn_bwd; the scratch (one float per query row, plus fp32 accumulators of dQ, dK, dV when
 * grad_dtype is not fp32) is a device array of MUSE_STATIC_SCRATCH_BYTES inside the library, which every device
 * the library runs on holds until the process ends.  The call allocates nothing (no hipMalloc, no events):
 *   - MUSE_ERR_SCRATCH_LIMIT if 256 + 4 B Hq N (+ 4 D N B (Hq + 2 Hkv) for non-fp32 gradients, each part rounded
 *     up to 256) exceeds MUSE_STATIC_SCRATCH_BYTES; nothing is launched;
 *   - MUSE_ERR_UNSUPPORTED while muse_profile_enable(1) is in force (the timing creates events);
 *   - all calls on one device share the one array: two calls whose work overlaps in time on a device (different
 *     streams, or different threads) race; calls on one stream are ordered and safe.  What must start at zero is
 *     cleared by the call itself. */
#define MUSE_STATIC_SCRATCH_BYTES (64u << 20)
int exact_attn_bwd_static(const muse_params* p, const void* Q, const void* K, const void* V,
                          const void* O, const float* LSE, const void* dO,
                          void* dQ, void* dK, void* dV, void* stream);

/* Diagnostics for benchmarks (not part of the method; process-wide, not thread-safe, allocates HIP
 * events): after muse_profile_enable(1) every kernel the library launches is bracketed by HIP events on
 * its stream; muse_profile_report synchronises those events and writes one line per kernel name,
 * "<name> <launches> <total milliseconds>", into the HOST buffer buf of cap bytes (INVALID_ARG if it
 * does not fit).  muse_profile_enable(0 or 1) also discards what was recorded so far. */
int muse_profile_enable(int on);
int muse_profile_report(char* buf, size_t cap);

/* Measurement aid (not part of the method; synchronises `stream`, creates and destroys two HIP events): runs a
 * plain streaming copy of the first half of the DEVICE buffer buf (bytes >= 1 GiB, 256-byte aligned, contents
 * overwritten) into its second half, and a loop of independent bf16 MFMA 32x32x16 instructions on every SIMD, five
 * times each, and reports the best: *copy_gbps = bytes read plus bytes written per second / 1e9, *mfma_bf16_tflops =
 * 2 x 32 x 32 x 16 flop per instruction / 1e12 (HOST pointers).  These are what the device delivers to the simplest
 * kernel of each kind, to set beside the published peaks.  INVALID_ARG for null or misaligned pointers,
 * WORKSPACE_TOO_SMALL below 1 GiB. */
int muse_probe_peaks(void* buf, size_t bytes, double* copy_gbps, double* mfma_bf16_tflops, void* stream);

/* Static, NUL-terminated description of a return code. */
const char* muse_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* MUSE_H_ */
