/*
 * CPU oracle for Multipole Semantic Attention (MuSe), causal, one (batch, head) per call.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the plain, slow, fp64 statement of what
 * the method computes.  Only the tests, the smoke check and the benchmark's
 * cpu_baseline leg may call it; the GPU library never does and shares no code
 * with it.
 *
 * Everything is written step by step in the order and notation of the paper:
 *   - exact softmax attention                       : Sec. 3, Eq. 1-2
 *   - clustering (init rule, nearest centroid with
 *     the ||x||^2-free distance identity)           : App. C "Centroid Computation",
 *                                                     "Balanced Assignment" (cap off)
 *   - per-block tilted summaries  S, k-bar, v-bar, mu: Sec. 3.1, Eq. 4-6
 *   - exclusive causal accumulation (the (+) merge)  : Sec. 3.1 "Causal accumulation",
 *                                                     Alg. 1 "Causal accumulation"
 *   - cluster selection, score = q~ . k-bar + mu     : Sec. 3.2, Eq. 7
 *   - spatial block selection on pre-accumulation
 *     summaries, block-causal mask b_q > b_k         : Sec. 3.2 "Spatial block selection"
 *   - exact retrieval with the full query, local
 *     block-diagonal attention, 4-component merge    : Sec. 3.3
 *   - dipole correction of the monopole-only mode, per cell
 *     (tilted) and pre-merged with untilted covariances : App. B "Dipole Correction",
 *                                                     "Untilted (Partially Specialized) Covariances"
 *   - backward: discrete choices frozen, query
 *     centroid a constant                            : App. C "Centroid Gradient Flow";
 *     gradient flows into K,V through the tilted aggregation weights (the default,
 *     differentiable aggregation of App. C "Aggregation Weight Gradient Flow").
 *
 * Readings where the paper is silent (all listed in the design notes of the repo):
 *   - Lloyd iterations (assign + mean update) at a fixed count T followed by a
 *     final assignment are the default clustering; empty cluster keeps
 *     its centroid; ties go to the lowest index.  The streaming mini-batch pass of
 *     App. C is oracle_kmeans_stream (rows in sequence order, state in binary32,
 *     similarity on binary16 values; pinned by a closed form for one cluster, the
 *     running mean at beta = 1, a hand-worked minibatch and the decay weights
 *     recomputed from the returned assignment).
 *   - logit scale: q is multiplied by `scale` before anything else; centroids are
 *     centroids of the raw rows, so q-bar = scale * centroid.
 *   - empty cells have mu = -inf and are never candidates; fewer than r finite
 *     candidates -> fewer selections, slots padded with -1.
 *   - k2 == 0 means "retrieve every preceding block of a selected cluster".
 *
 * Parity pins (tests, CPU only): equals exact attention when every key is its own
 * cluster, when every query is its own cluster, when r covers all clusters with
 * k2 == 0, and when the block is the whole sequence; key-translation invariance;
 * closed form for C_q = 1, q-bar = 0; scan == summary of the union; an independent
 * N x N real-key formulation on tiny inputs; finite-difference gradients; exact
 * attention against a library routine.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
  int32_t N, D, Bs, Cq, Ck, r, k2;
  double scale;
  /* App. C "Aggregation Weight Gradient Flow", non-differentiable variant: the tilted aggregation
   * weights e_m / S and the log-mass mu-bar of every summary are constants of the backward. */
  int32_t frozen_weights;
  /* App. B "Dipole Correction" (forward only, monopole-only mode r = 0):
   *   0 none;
   *   1 per-cell tilted dipole, Eq. "dipole-shift": the value of the accumulated summary (i,j,b)
   *     becomes v-bar + Cov_ij(v,k) q~, Cov_ij the q-bar_i-tilted covariance of its keys;
   *   2 pre-merged untilted dipole, Eq. "premerge" with the shared covariances of "Untilted
   *     (Partially Specialized) Covariances": one matrix C-bar_ib = sum_j p_ib(j) Cov_0jb(v,k)
   *     per (query cluster, query block), applied once per query as C-bar q~.
   * Causal reading (the appendix has no blocks): the key set of cluster j seen from query block b
   * is its keys in the blocks before b, as for the accumulated summaries; p_ib(j) is the softmax
   * of the accumulated log-masses A-mu_ijb over j; and because the far field shares the one
   * softmax with the query's own block, the merged correction enters the output with the far
   * field's share of the softmax mass:  O_n += w_far(n) C-bar_ib q~_n. */
  int32_t dipole;
  /* Keys inside the tilted weights exp(q-bar . k) of Eq. 4-6 when they are to differ from the keys
   * that are aggregated (NULL: the same K).  Only the pins use it: with Kw held at K the forward is the
   * function whose derivative the frozen-weights backward is. */
  const double* Kw;
} omuse_params;

/* ------------------------------------------------------------------ */
/* storage-format rounding (IEEE binary32, and bfloat16 = top 16 bits  */
/* of binary32 with round-to-nearest-even)                             */
/* ------------------------------------------------------------------ */
static double round_f32(double x) { return (double)(float)x; }

static double round_bf16(double x) {
  float f = (float)x;
  uint32_t u;
  memcpy(&u, &f, 4);
  if ((u & 0x7f800000u) == 0x7f800000u) return (double)f; /* inf / nan */
  uint32_t lsb = (u >> 16) & 1u;
  u += 0x7fffu + lsb;
  u &= 0xffff0000u;
  memcpy(&f, &u, 4);
  return (double)f;
}

double oracle_round_bf16(double x) { return round_bf16(x); }

static double dot(const double* a, const double* b, int D) {
  double s = 0.0;
  for (int d = 0; d < D; ++d) s += a[d] * b[d];
  return s;
}

/* ------------------------------------------------------------------ */
/* Exact causal softmax attention, Eq. 1-2, logits scale * q.k, m <= n */
/* ------------------------------------------------------------------ */
void oracle_exact_fwd(int N, int D, double scale, const double* Q, const double* K,
                      const double* V, int nrows, const int32_t* rows, double* O,
                      double* LSE) {
  double* l = (double*)malloc(sizeof(double) * (size_t)N);
  int cnt = rows ? nrows : N;
  for (int t = 0; t < cnt; ++t) {
    int n = rows ? rows[t] : t;
    const double* q = Q + (size_t)n * D;
    double mx = -INFINITY;
    for (int m = 0; m <= n; ++m) {
      l[m] = scale * dot(q, K + (size_t)m * D, D);
      if (l[m] > mx) mx = l[m];
    }
    double Z = 0.0;
    for (int m = 0; m <= n; ++m) Z += exp(l[m] - mx);
    double* o = O + (size_t)n * D;
    for (int d = 0; d < D; ++d) o[d] = 0.0;
    for (int m = 0; m <= n; ++m) {
      double p = exp(l[m] - mx) / Z;
      const double* v = V + (size_t)m * D;
      for (int d = 0; d < D; ++d) o[d] += p * v[d];
    }
    LSE[n] = mx + log(Z);
  }
  free(l);
}

/* Gradient of the above, contracted with dO, summed over the listed rows.
 * p = exp(l - LSE), delta = dO.O, dl = p (dO.v - delta). */
void oracle_exact_bwd(int N, int D, double scale, const double* Q, const double* K,
                      const double* V, const double* O, const double* LSE,
                      const double* dO, int nrows, const int32_t* rows, double* dQ,
                      double* dK, double* dV) {
  memset(dQ, 0, sizeof(double) * (size_t)N * D);
  memset(dK, 0, sizeof(double) * (size_t)N * D);
  memset(dV, 0, sizeof(double) * (size_t)N * D);
  int cnt = rows ? nrows : N;
  for (int t = 0; t < cnt; ++t) {
    int n = rows ? rows[t] : t;
    const double* q = Q + (size_t)n * D;
    const double* g = dO + (size_t)n * D;
    double delta = dot(g, O + (size_t)n * D, D);
    for (int m = 0; m <= n; ++m) {
      const double* k = K + (size_t)m * D;
      const double* v = V + (size_t)m * D;
      double p = exp(scale * dot(q, k, D) - LSE[n]);
      double dl = p * (dot(g, v, D) - delta);
      for (int d = 0; d < D; ++d) {
        dQ[(size_t)n * D + d] += dl * scale * k[d];
        dK[(size_t)m * D + d] += dl * scale * q[d];
        dV[(size_t)m * D + d] += p * g[d];
      }
    }
  }
}

/* ------------------------------------------------------------------ */
/* Clustering: App. C.  Lloyd, T iterations + final assignment.        */
/* score(n,j) = ||c^_j||^2 - 2 <x_n, c^_j>  (||x||^2 dropped);         */
/* c^ = master centroid rounded to the storage type used for scoring   */
/* (round_mode 0: binary32, 1: bfloat16).  Master centroids are kept   */
/* as binary32 values.  init_idx == NULL -> start from `cent` as given.*/
/* ------------------------------------------------------------------ */
static void assign_points(int N, int D, int C, int round_mode, const double* X,
                          const double* cent, int32_t* assign, double* margin) {
  double* ch = (double*)malloc(sizeof(double) * (size_t)C * D);
  double* c2 = (double*)malloc(sizeof(double) * (size_t)C);
  for (int j = 0; j < C; ++j) {
    for (int d = 0; d < D; ++d) {
      double c = cent[(size_t)j * D + d];
      ch[(size_t)j * D + d] = round_mode == 1 ? round_bf16(c) : round_f32(c);
    }
    c2[j] = dot(ch + (size_t)j * D, ch + (size_t)j * D, D);
  }
  for (int n = 0; n < N; ++n) {
    double best = INFINITY, second = INFINITY;
    int bj = 0;
    for (int j = 0; j < C; ++j) {
      double s = c2[j] - 2.0 * dot(X + (size_t)n * D, ch + (size_t)j * D, D);
      if (s < best) {
        second = best;
        best = s;
        bj = j;
      } else if (s < second) {
        second = s;
      }
    }
    assign[n] = bj;
    if (margin) {
      double den = fmax(1.0, fmax(fabs(best), fabs(second)));
      margin[n] = isfinite(second) ? (second - best) / den : INFINITY;
    }
  }
  free(ch);
  free(c2);
}

void oracle_kmeans(int N, int D, int C, int T, int round_mode, const double* X,
                   const int32_t* init_idx, double* cent, int32_t* assign,
                   double* margin, int32_t* counts, double* objective) {
  if (init_idx)
    for (int j = 0; j < C; ++j)
      for (int d = 0; d < D; ++d)
        cent[(size_t)j * D + d] = round_f32(X[(size_t)init_idx[j] * D + d]);
  double* sum = (double*)malloc(sizeof(double) * (size_t)C * D);
  for (int t = 0; t < T; ++t) {
    assign_points(N, D, C, round_mode, X, cent, assign, NULL);
    if (objective) {
      double obj = 0.0;
      for (int n = 0; n < N; ++n)
        for (int d = 0; d < D; ++d) {
          double e = X[(size_t)n * D + d] - cent[(size_t)assign[n] * D + d];
          obj += e * e;
        }
      objective[t] = obj;
    }
    memset(sum, 0, sizeof(double) * (size_t)C * D);
    for (int j = 0; j < C; ++j) counts[j] = 0;
    for (int n = 0; n < N; ++n) {
      counts[assign[n]]++;
      for (int d = 0; d < D; ++d) sum[(size_t)assign[n] * D + d] += X[(size_t)n * D + d];
    }
    for (int j = 0; j < C; ++j)
      if (counts[j] > 0)
        for (int d = 0; d < D; ++d)
          cent[(size_t)j * D + d] = round_f32(sum[(size_t)j * D + d] / counts[j]);
  }
  assign_points(N, D, C, round_mode, X, cent, assign, margin);
  for (int j = 0; j < C; ++j) counts[j] = 0;
  for (int n = 0; n < N; ++n) counts[assign[n]]++;
  if (objective) {
    double obj = 0.0;
    for (int n = 0; n < N; ++n)
      for (int d = 0; d < D; ++d) {
        double e = X[(size_t)n * D + d] - cent[(size_t)assign[n] * D + d];
        obj += e * e;
      }
    objective[T] = obj;
  }
  free(sum);
}

/* ------------------------------------------------------------------ */
/* Balanced assignment: App. C "Balanced Assignment".                    */
/*                                                                     */
/* Inside every spatial block a cluster holds at most `cap` rows (the  */
/* paper: 4 B / K).  The paper does not say which rows give way; the   */
/* reading here has two phases, both in position order:                */
/*   A. every row names its nearest centroid (same score and ties as   */
/*      assign_points); of the rows of a block that name centroid j    */
/*      the first `cap` keep it;                                        */
/*   B. the others, one after the other in position order, go to the   */
/*      nearest centroid that still has room in the block at that      */
/*      moment (rows kept in phase A and rows placed earlier in phase  */
/*      B count), lowest index on ties.                                 */
/* With forced != NULL the pass is replayed along the given assignment */
/* and checked instead: a row whose forced cluster scores within `tol` */
/* (relative) of its nearest one names that cluster in phase A; any    */
/* other row names its nearest one and must be displaced; a displaced  */
/* row's forced cluster must have room when its turn comes and score   */
/* within `tol` of the best cluster with room.  report[0] = largest    */
/* relative regret of a phase B choice, report[1] = number of rows     */
/* that break a rule (kept beyond the cap, placed without room, placed */
/* although their nearest cluster had room for them).                   */
/* ------------------------------------------------------------------ */
void oracle_balanced_assign(int N, int D, int C, int Bs, int cap, int round_mode, const double* X,
                            const double* cent, const int32_t* forced, double tol, int32_t* assign,
                            double* report) {
  double* ch = (double*)malloc(sizeof(double) * (size_t)C * D);
  double* c2 = (double*)malloc(sizeof(double) * (size_t)C);
  double* sc = (double*)malloc(sizeof(double) * (size_t)C);
  int32_t* named = (int32_t*)malloc(sizeof(int32_t) * (size_t)N);
  char* moved = (char*)malloc((size_t)N);
  int32_t* count = (int32_t*)malloc(sizeof(int32_t) * (size_t)C);
  double worst = 0.0, broken = 0.0;
  for (int j = 0; j < C; ++j) {
    for (int d = 0; d < D; ++d) {
      double c = cent[(size_t)j * D + d];
      ch[(size_t)j * D + d] = round_mode == 1 ? round_bf16(c) : round_f32(c);
    }
    c2[j] = dot(ch + (size_t)j * D, ch + (size_t)j * D, D);
  }
  for (int b0 = 0; b0 < N; b0 += Bs) {
    int b1 = b0 + Bs < N ? b0 + Bs : N;
    /* phase A */
    for (int j = 0; j < C; ++j) count[j] = 0;
    for (int n = b0; n < b1; ++n) {
      double best = INFINITY;
      int bj = 0;
      for (int j = 0; j < C; ++j) {
        sc[j] = c2[j] - 2.0 * dot(X + (size_t)n * D, ch + (size_t)j * D, D);
        if (sc[j] < best) {
          best = sc[j];
          bj = j;
        }
      }
      int name = bj;
      if (forced) {
        double sf = sc[forced[n]];
        if ((sf - best) / fmax(1.0, fmax(fabs(best), fabs(sf))) <= tol) name = forced[n];
      }
      named[n] = name;
      moved[n] = count[name] >= cap;
      if (!moved[n]) count[name]++;
      if (forced && !moved[n] && forced[n] != name) broken += 1.0; /* had room in its nearest cluster */
      if (forced && moved[n] && forced[n] == name) broken += 1.0;  /* kept beyond the cap */
      if (!moved[n]) assign[n] = name;
    }
    /* phase B */
    for (int n = b0; n < b1; ++n) {
      if (!moved[n]) continue;
      double best = INFINITY;
      int bj = -1;
      for (int j = 0; j < C; ++j) {
        sc[j] = c2[j] - 2.0 * dot(X + (size_t)n * D, ch + (size_t)j * D, D);
        if (count[j] < cap && sc[j] < best) {
          best = sc[j];
          bj = j;
        }
      }
      int take = bj;
      if (forced) {
        take = forced[n];
        if (count[take] >= cap) {
          broken += 1.0;
        } else {
          double reg = (sc[take] - best) / fmax(1.0, fmax(fabs(best), fabs(sc[take])));
          if (reg > worst) worst = reg;
        }
      }
      assign[n] = take;
      if (take >= 0) count[take]++;
    }
  }
  if (report) {
    report[0] = worst;
    report[1] = broken;
  }
  free(ch); free(c2); free(sc); free(named); free(moved); free(count);
}

/* ------------------------------------------------------------------ */
/* Streaming centroid pass: App. C "Centroid Computation", step 2.      */
/*                                                                     */
/* One pass over the rows in sequence order, in minibatches of `mb`    */
/* rows (the paper: 64).  All rows of a minibatch are assigned to their */
/* nearest centroid as the centroids stand when the minibatch starts;  */
/* then, row by row in order, the total and the count of the row's     */
/* centroid decay and absorb the row: t <- beta t + x, c <- beta c + 1, */
/* and the centroid is t / c.  Totals start at the initial centroid    */
/* (the row init_idx[j]) with count 1.                                 */
/*                                                                     */
/* Precision (the paper fixes float16 for the clustering computations, */
/* and says no more): rows and centroids enter the similarity as       */
/* binary16 values (x^ = fp16(x), c^ = fp16(t / c)); the score         */
/* ||c^||^2 - 2 <x^, c^> is evaluated exactly here (fp64 of exact      */
/* products).  The state t, c is binary32, each update one fused       */
/* multiply-add, t / c one binary32 division: these decide the rounded */
/* centroid, so they are taken in that precision on purpose, not fp64. */
/* Ties go to the lowest index.                                        */
/*                                                                     */
/* forced != NULL: row v is assigned to forced[v] instead of the       */
/* nearest centroid, and regret[v] says how much worse that choice     */
/* scores than the best one (relative, 0 when it is a best one).       */
/* ------------------------------------------------------------------ */
static double round_fp16(double x) {
  if (x == 0.0 || !isfinite(x)) return x;
  double a = fabs(x);
  if (a >= 65520.0) return copysign(INFINITY, x); /* halfway to 2^16 rounds to even = overflow */
  int e;
  frexp(a, &e);             /* a = m 2^e, 0.5 <= m < 1 */
  int ex = e - 1;           /* floor(log2 a) */
  if (ex < -14) ex = -14;   /* subnormal range: fixed quantum 2^-24 */
  double q = ldexp(1.0, ex - 10);
  return copysign(nearbyint(a / q) * q, x); /* nearbyint: round to nearest, ties to even */
}

double oracle_round_fp16(double x) { return round_fp16(x); }

void oracle_kmeans_stream(int N, int D, int C, int mb, double beta, const double* X,
                          const int32_t* init_idx, const int32_t* forced, double* cent,
                          double* t_out, double* c_out, int32_t* assign, double* margin,
                          double* regret) {
  const float bf = (float)beta;
  double* xh = (double*)malloc(sizeof(double) * (size_t)N * D); /* x^ */
  for (size_t k = 0; k < (size_t)N * D; ++k) xh[k] = round_fp16(X[k]);
  float* t = (float*)malloc(sizeof(float) * (size_t)C * D);
  float* c = (float*)malloc(sizeof(float) * (size_t)C);
  double* ch = (double*)malloc(sizeof(double) * (size_t)C * D); /* c^ */
  double* c2 = (double*)malloc(sizeof(double) * (size_t)C);
  for (int j = 0; j < C; ++j) {
    for (int d = 0; d < D; ++d) t[(size_t)j * D + d] = (float)xh[(size_t)init_idx[j] * D + d];
    c[j] = 1.0f;
  }
  for (int v0 = 0; v0 < N; v0 += mb) {
    int v1 = v0 + mb < N ? v0 + mb : N;
    /* centroids as they stand now */
    for (int j = 0; j < C; ++j) {
      for (int d = 0; d < D; ++d) ch[(size_t)j * D + d] = round_fp16((double)(t[(size_t)j * D + d] / c[j]));
      c2[j] = dot(ch + (size_t)j * D, ch + (size_t)j * D, D);
    }
    /* nearest centroid of every row of the minibatch */
    for (int v = v0; v < v1; ++v) {
      double best = INFINITY, second = INFINITY;
      int bj = 0;
      for (int j = 0; j < C; ++j) {
        double s = c2[j] - 2.0 * dot(xh + (size_t)v * D, ch + (size_t)j * D, D);
        if (s < best) {
          second = best;
          best = s;
          bj = j;
        } else if (s < second) {
          second = s;
        }
      }
      if (margin) {
        double den = fmax(1.0, fmax(fabs(best), fabs(second)));
        margin[v] = isfinite(second) ? (second - best) / den : INFINITY;
      }
      if (forced) {
        int fj = forced[v];
        double sf = c2[fj] - 2.0 * dot(xh + (size_t)v * D, ch + (size_t)fj * D, D);
        if (regret) regret[v] = (sf - best) / fmax(1.0, fmax(fabs(best), fabs(sf)));
        bj = fj;
      } else if (regret) {
        regret[v] = 0.0;
      }
      assign[v] = bj;
    }
    /* the rows update their centroids one after the other */
    for (int v = v0; v < v1; ++v) {
      int j = assign[v];
      for (int d = 0; d < D; ++d)
        t[(size_t)j * D + d] = fmaf(bf, t[(size_t)j * D + d], (float)xh[(size_t)v * D + d]);
      c[j] = fmaf(bf, c[j], 1.0f);
    }
  }
  for (int j = 0; j < C; ++j) {
    for (int d = 0; d < D; ++d) {
      cent[(size_t)j * D + d] = (double)(t[(size_t)j * D + d] / c[j]);
      if (t_out) t_out[(size_t)j * D + d] = (double)t[(size_t)j * D + d];
    }
    if (c_out) c_out[j] = (double)c[j];
  }
  free(xh);
  free(t);
  free(c);
  free(ch);
  free(c2);
}

/* ------------------------------------------------------------------ */
/* Summaries                                                           */
/* ------------------------------------------------------------------ */
typedef struct {
  int nb, Cq, Ck, D;
  int32_t* seg_off; /* [nb*Ck+1]  keys of (block b, cluster j): seg_idx[seg_off[b*Ck+j] ..) */
  int32_t* seg_idx; /* [N] key positions, increasing inside a segment */
  /* per query cluster i (NULL when i is not needed): cell (j,b) at index j*nb+b */
  double **mu, **kb, **vb;    /* per-block (pre-accumulation) summaries, Eq. 4-6 */
  double **Amu, **Akb, **Avb; /* exclusive accumulation: blocks 0..b-1 */
  double* qbar;               /* [Cq,D] = scale * centroid */
} summ_t;

static void bucket_keys(const omuse_params* p, const int32_t* ak, summ_t* s) {
  int nb = p->N / p->Bs, Ck = p->Ck, N = p->N;
  s->seg_off = (int32_t*)calloc((size_t)nb * Ck + 1, sizeof(int32_t));
  s->seg_idx = (int32_t*)malloc(sizeof(int32_t) * (size_t)N);
  for (int m = 0; m < N; ++m) s->seg_off[(m / p->Bs) * Ck + ak[m] + 1]++;
  for (int t = 0; t < nb * Ck; ++t) s->seg_off[t + 1] += s->seg_off[t];
  int32_t* cur = (int32_t*)malloc(sizeof(int32_t) * (size_t)nb * Ck);
  memcpy(cur, s->seg_off, sizeof(int32_t) * (size_t)nb * Ck);
  for (int m = 0; m < N; ++m) s->seg_idx[cur[(m / p->Bs) * Ck + ak[m]]++] = m;
  free(cur);
}

/* (mu1,k1,v1) (+) (mu2,k2,v2): logaddexp on mu, convex combination on k, v.
 * The empty summary (mu = -inf) is the identity. */
static void oplus(int D, double mu1, const double* k1, const double* v1, double mu2,
                  const double* k2, const double* v2, double* mu, double* k, double* v) {
  if (mu1 == -INFINITY && mu2 == -INFINITY) {
    *mu = -INFINITY;
    for (int d = 0; d < D; ++d) k[d] = v[d] = 0.0;
    return;
  }
  double mx = mu1 > mu2 ? mu1 : mu2;
  double m = mx + log(exp(mu1 - mx) + exp(mu2 - mx));
  double w1 = exp(mu1 - m), w2 = exp(mu2 - m);
  for (int d = 0; d < D; ++d) {
    k[d] = w1 * k1[d] + w2 * k2[d];
    v[d] = w1 * v1[d] + w2 * v2[d];
  }
  *mu = m;
}

static void summaries_for_cluster(const omuse_params* p, const double* K, const double* V,
                                  summ_t* s, int i) {
  int nb = s->nb, Ck = s->Ck, D = s->D;
  size_t cells = (size_t)Ck * nb;
  s->mu[i] = (double*)malloc(sizeof(double) * cells);
  s->kb[i] = (double*)calloc(cells * D, sizeof(double));
  s->vb[i] = (double*)calloc(cells * D, sizeof(double));
  s->Amu[i] = (double*)malloc(sizeof(double) * cells);
  s->Akb[i] = (double*)calloc(cells * D, sizeof(double));
  s->Avb[i] = (double*)calloc(cells * D, sizeof(double));
  const double* qb = s->qbar + (size_t)i * D;
  const double* Kw = p->Kw ? p->Kw : K; /* the keys inside the weights */
  for (int j = 0; j < Ck; ++j) {
    for (int b = 0; b < nb; ++b) {
      size_t c = (size_t)j * nb + b;
      int lo = s->seg_off[b * Ck + j], hi = s->seg_off[b * Ck + j + 1];
      if (lo == hi) {
        s->mu[i][c] = -INFINITY;
        continue;
      }
      /* attention from the query centroid to the keys of (j, b): Eq. 4-6 */
      double mx = -INFINITY;
      for (int t = lo; t < hi; ++t) {
        double l = dot(qb, Kw + (size_t)s->seg_idx[t] * D, D);
        if (l > mx) mx = l;
      }
      double S = 0.0;
      for (int t = lo; t < hi; ++t) {
        int m = s->seg_idx[t];
        double e = exp(dot(qb, Kw + (size_t)m * D, D) - mx);
        S += e;
        for (int d = 0; d < D; ++d) {
          s->kb[i][c * D + d] += e * K[(size_t)m * D + d];
          s->vb[i][c * D + d] += e * V[(size_t)m * D + d];
        }
      }
      for (int d = 0; d < D; ++d) {
        s->kb[i][c * D + d] /= S;
        s->vb[i][c * D + d] /= S;
      }
      s->mu[i][c] = mx + log(S);
    }
    /* exclusive accumulation along the block axis, sequentially */
    size_t c0 = (size_t)j * nb;
    s->Amu[i][c0] = -INFINITY;
    for (int b = 1; b < nb; ++b) {
      size_t c = c0 + b;
      oplus(D, s->Amu[i][c - 1], s->Akb[i] + (c - 1) * D, s->Avb[i] + (c - 1) * D,
            s->mu[i][c - 1], s->kb[i] + (c - 1) * D, s->vb[i] + (c - 1) * D, &s->Amu[i][c],
            s->Akb[i] + c * D, s->Avb[i] + c * D);
    }
  }
}

static summ_t* summ_new(const omuse_params* p, const double* qc, const int32_t* ak) {
  summ_t* s = (summ_t*)calloc(1, sizeof(summ_t));
  s->nb = p->N / p->Bs;
  s->Cq = p->Cq;
  s->Ck = p->Ck;
  s->D = p->D;
  bucket_keys(p, ak, s);
  s->mu = (double**)calloc(p->Cq, sizeof(double*));
  s->kb = (double**)calloc(p->Cq, sizeof(double*));
  s->vb = (double**)calloc(p->Cq, sizeof(double*));
  s->Amu = (double**)calloc(p->Cq, sizeof(double*));
  s->Akb = (double**)calloc(p->Cq, sizeof(double*));
  s->Avb = (double**)calloc(p->Cq, sizeof(double*));
  s->qbar = (double*)malloc(sizeof(double) * (size_t)p->Cq * p->D);
  for (size_t t = 0; t < (size_t)p->Cq * p->D; ++t) s->qbar[t] = p->scale * qc[t];
  return s;
}

static void summ_free(summ_t* s) {
  for (int i = 0; i < s->Cq; ++i) {
    free(s->mu[i]); free(s->kb[i]); free(s->vb[i]);
    free(s->Amu[i]); free(s->Akb[i]); free(s->Avb[i]);
  }
  free(s->mu); free(s->kb); free(s->vb); free(s->Amu); free(s->Akb); free(s->Avb);
  free(s->seg_off); free(s->seg_idx); free(s->qbar);
  free(s);
}

/* Export of the summaries of one query cluster, for the pins.
 * Layout of every output: [Ck, nb] (x D for the vectors). */
void oracle_summaries(const omuse_params* p, const double* K, const double* V,
                      const double* qc, const int32_t* ak, int i, double* mu, double* kb,
                      double* vb, double* Amu, double* Akb, double* Avb) {
  summ_t* s = summ_new(p, qc, ak);
  summaries_for_cluster(p, K, V, s, i);
  size_t cells = (size_t)p->Ck * s->nb;
  memcpy(mu, s->mu[i], sizeof(double) * cells);
  memcpy(kb, s->kb[i], sizeof(double) * cells * p->D);
  memcpy(vb, s->vb[i], sizeof(double) * cells * p->D);
  memcpy(Amu, s->Amu[i], sizeof(double) * cells);
  memcpy(Akb, s->Akb[i], sizeof(double) * cells * p->D);
  memcpy(Avb, s->Avb[i], sizeof(double) * cells * p->D);
  summ_free(s);
}

/* ------------------------------------------------------------------ */
/* Per-query list of "virtual keys": every term of the one softmax     */
/* that the four components are merged into (Sec. 3.3 Output merging). */
/* ------------------------------------------------------------------ */
enum { VK_ACC = 1, VK_BLK = 2, VK_RET = 3, VK_LOC = 4 };
typedef struct {
  double logit;
  int type; /* component 1..4 */
  int j, b; /* summary cell (types 1, 2) */
  int m;    /* real key position (types 3, 4) */
} vkey_t;

/* top-`want` of cand[0..n) (values val[], ids id[]), descending value, ties to
 * the lower id; candidates are only finite values.  Returns how many were taken;
 * *gap = (value of the last taken) - (best value not taken), relative to
 * max(1,|a|,|b|), +inf when nothing is left out. */
static int top_select(int n, const double* val, const int* id, int want, int* out,
                      double* gap) {
  char* used = (char*)calloc((size_t)n + 1, 1);
  int got = 0;
  double last = INFINITY;
  while (got < want) {
    int best = -1;
    for (int t = 0; t < n; ++t) {
      if (used[t] || val[t] == -INFINITY) continue;
      if (best < 0 || val[t] > val[best] || (val[t] == val[best] && id[t] < id[best]))
        best = t;
    }
    if (best < 0) break;
    used[best] = 1;
    out[got++] = best;
    last = val[best];
  }
  double next = -INFINITY;
  for (int t = 0; t < n; ++t)
    if (!used[t] && val[t] != -INFINITY && val[t] > next) next = val[t];
  if (gap) {
    if (got == 0 || next == -INFINITY)
      *gap = INFINITY;
    else
      *gap = (last - next) / fmax(1.0, fmax(fabs(last), fabs(next)));
  }
  free(used);
  return got;
}

/* Slack of a GIVEN selection chosen[0..nslots) (entries < 0 are padding) among the candidates
 * val[0..n) (a candidate's id is its index; -inf = not a candidate): (lowest chosen value) -
 * (highest value left out), relative to max(1,|a|,|b|) as in top_select.  For the selection that
 * top_select takes it equals its gap (>= 0); a negative slack says a better candidate was left
 * out.  +inf when nothing is left out; -inf when the selection is malformed: an entry out of
 * range, not a candidate or chosen twice, or fewer entries than min(want, candidates). */
static double selection_slack(int n, const double* val, int want, const int32_t* chosen,
                              int nslots) {
  char* used = (char*)calloc((size_t)n + 1, 1);
  int got = 0, cand = 0, bad = 0;
  double low = INFINITY, next = -INFINITY;
  for (int t = 0; t < nslots; ++t) {
    int c = chosen[t];
    if (c < 0) continue;
    if (c >= n || used[c] || val[c] == -INFINITY) { bad = 1; break; }
    used[c] = 1;
    ++got;
    if (val[c] < low) low = val[c];
  }
  for (int t = 0; t < n; ++t) {
    if (val[t] == -INFINITY) continue;
    ++cand;
    if (!used[t] && val[t] > next) next = val[t];
  }
  free(used);
  if (bad || got != (want < cand ? want : cand)) return -INFINITY;
  if (got == 0 || next == -INFINITY) return INFINITY;
  return (low - next) / fmax(1.0, fmax(fabs(low), fabs(next)));
}

typedef struct {
  const omuse_params* p;
  const double *Q, *K, *V;
  const int32_t *aq, *ak;
  summ_t* s;
  int k2e; /* slots per selected cluster: k2, or nb-1 when k2 == 0 */
} ctx_t;

/* Covariance Cov(v,k)[a*D + c] = E[(v_a - E v_a)(k_c - E k_c)] of the keys of cluster j in the
 * blocks before b, under the weights exp(qb . k) (qb == NULL: equal weights, the untilted
 * covariance Cov_0j of App. B).  Zero for an empty set. */
static void cov_vk(const ctx_t* c, const double* qb, int j, int b, double* cov) {
  int D = c->p->D, Ck = c->p->Ck;
  for (int t = 0; t < D * D; ++t) cov[t] = 0.0;
  double mx = -INFINITY;
  for (int bp = 0; bp < b; ++bp)
    for (int u = c->s->seg_off[bp * Ck + j]; u < c->s->seg_off[bp * Ck + j + 1]; ++u) {
      double l = qb ? dot(qb, c->K + (size_t)c->s->seg_idx[u] * D, D) : 0.0;
      if (l > mx) mx = l;
    }
  if (mx == -INFINITY) return;
  double* km = (double*)calloc(2 * (size_t)D, sizeof(double));
  double* vm = km + D;
  double S = 0.0;
  for (int bp = 0; bp < b; ++bp)
    for (int u = c->s->seg_off[bp * Ck + j]; u < c->s->seg_off[bp * Ck + j + 1]; ++u) {
      int m = c->s->seg_idx[u];
      double w = exp((qb ? dot(qb, c->K + (size_t)m * D, D) : 0.0) - mx);
      S += w;
      for (int d = 0; d < D; ++d) {
        km[d] += w * c->K[(size_t)m * D + d];
        vm[d] += w * c->V[(size_t)m * D + d];
      }
    }
  for (int d = 0; d < D; ++d) { km[d] /= S; vm[d] /= S; }
  for (int bp = 0; bp < b; ++bp)
    for (int u = c->s->seg_off[bp * Ck + j]; u < c->s->seg_off[bp * Ck + j + 1]; ++u) {
      int m = c->s->seg_idx[u];
      double w = exp((qb ? dot(qb, c->K + (size_t)m * D, D) : 0.0) - mx) / S;
      for (int a = 0; a < D; ++a)
        for (int d = 0; d < D; ++d)
          cov[a * D + d] += w * (c->V[(size_t)m * D + a] - vm[a]) * (c->K[(size_t)m * D + d] - km[d]);
    }
  free(km);
}

/* Pre-merged dipole matrix of (query cluster i, query block b), App. B Eq. "premerge" with untilted
 * covariances:  C-bar = sum_j p(j) Cov_0jb(v,k),  p = softmax over j of the accumulated log-masses. */
static void merged_dipole(const ctx_t* c, int i, int b, double* cbar) {
  int D = c->p->D, Ck = c->p->Ck, nb = c->s->nb;
  for (int t = 0; t < D * D; ++t) cbar[t] = 0.0;
  const double* Amu = c->s->Amu[i];
  double mx = -INFINITY, Z = 0.0;
  for (int j = 0; j < Ck; ++j)
    if (Amu[(size_t)j * nb + b] > mx) mx = Amu[(size_t)j * nb + b];
  if (mx == -INFINITY) return;
  for (int j = 0; j < Ck; ++j) Z += exp(Amu[(size_t)j * nb + b] - mx);
  double* cov = (double*)malloc(sizeof(double) * (size_t)D * D);
  for (int j = 0; j < Ck; ++j) {
    double pj = exp(Amu[(size_t)j * nb + b] - mx) / Z;
    if (pj == 0.0) continue;
    cov_vk(c, NULL, j, b, cov);
    for (int t = 0; t < D * D; ++t) cbar[t] += pj * cov[t];
  }
  free(cov);
}

/* Builds the virtual keys of query n.  When sel_given, the selections in
 * selc[r] / selb[r*k2e] are used as they are (entries < 0 ignored); otherwise
 * they are computed (Eq. 7 and the block selection) and written there.
 * margin_c / margin_b (may be NULL): the gap of the cluster selection / the smallest gap of
 * the block selections (top_select); for given selections their slack (selection_slack). */
static int build_vkeys(const ctx_t* c, int n, int sel_given, int32_t* selc, int32_t* selb,
                       double* margin_c, double* margin_b, double* qs, double* qt,
                       vkey_t* vk, double* tmpv, int* tmpi, int* tmpo) {
  const omuse_params* p = c->p;
  int D = p->D, Ck = p->Ck, nb = c->s->nb, r = p->r, k2e = c->k2e;
  int b = n / p->Bs, i = c->aq[n];
  int nv = 0;
  for (int d = 0; d < D; ++d) {
    qs[d] = p->scale * c->Q[(size_t)n * D + d];
    qt[d] = qs[d] - c->s->qbar[(size_t)i * D + d];
  }
  if (margin_c) *margin_c = INFINITY;
  if (margin_b) *margin_b = INFINITY;
  if (!sel_given) {
    for (int t = 0; t < r; ++t) selc[t] = -1;
    for (int t = 0; t < r * k2e; ++t) selb[t] = -1;
  }
  if (b >= 1) {
    const double *Amu = c->s->Amu[i], *Akb = c->s->Akb[i];
    const double *mu = c->s->mu[i], *kb = c->s->kb[i];
    /* cluster selection: scores against the accumulated summaries, Eq. 7 */
    for (int j = 0; j < Ck; ++j) {
      size_t cell = (size_t)j * nb + b;
      tmpv[j] = Amu[cell] == -INFINITY ? -INFINITY : dot(qt, Akb + cell * D, D) + Amu[cell];
      tmpi[j] = j;
    }
    if (!sel_given) {
      int got = top_select(Ck, tmpv, tmpi, r, tmpo, margin_c);
      for (int t = 0; t < got; ++t) selc[t] = tmpo[t];
    } else if (margin_c) {
      *margin_c = selection_slack(Ck, tmpv, r, selc, r);
    }
    /* component 1: non-retrieved clusters, accumulated summaries */
    for (int j = 0; j < Ck; ++j) {
      if (tmpv[j] == -INFINITY) continue;
      int is_sel = 0;
      for (int t = 0; t < r; ++t) is_sel |= (selc[t] == j);
      if (is_sel) continue;
      vk[nv++] = (vkey_t){tmpv[j], VK_ACC, j, b, -1};
    }
    /* per selected cluster: block selection on the pre-accumulation summaries */
    for (int t = 0; t < r; ++t) {
      int j = selc[t];
      if (j < 0) continue;
      double* bv = tmpv + Ck; /* scores of blocks b' < b */
      int* bi = tmpi + Ck;
      for (int bp = 0; bp < b; ++bp) {
        size_t cell = (size_t)j * nb + bp;
        bv[bp] = mu[cell] == -INFINITY ? -INFINITY : dot(qt, kb + cell * D, D) + mu[cell];
        bi[bp] = bp;
      }
      if (!sel_given) {
        double gap;
        int want = p->k2 == 0 ? b : p->k2;
        int got = top_select(b, bv, bi, want, tmpo, &gap);
        for (int u = 0; u < got; ++u) selb[t * k2e + u] = tmpo[u];
        if (margin_b && gap < *margin_b) *margin_b = gap;
      } else if (margin_b) {
        double gap = selection_slack(b, bv, p->k2 == 0 ? b : p->k2, selb + t * k2e, k2e);
        if (gap < *margin_b) *margin_b = gap;
      }
      for (int bp = 0; bp < b; ++bp) {
        if (bv[bp] == -INFINITY) continue;
        int is_sel = 0;
        for (int u = 0; u < k2e; ++u) is_sel |= (selb[t * k2e + u] == bp);
        if (!is_sel) { /* component 2 */
          vk[nv++] = (vkey_t){bv[bp], VK_BLK, j, bp, -1};
        } else { /* component 3: exact, full query */
          int lo = c->s->seg_off[bp * Ck + j], hi = c->s->seg_off[bp * Ck + j + 1];
          for (int u = lo; u < hi; ++u) {
            int m = c->s->seg_idx[u];
            vk[nv++] = (vkey_t){dot(qs, c->K + (size_t)m * D, D), VK_RET, j, bp, m};
          }
        }
      }
    }
  }
  /* component 4: local block, causal */
  for (int m = b * p->Bs; m <= n; ++m)
    vk[nv++] = (vkey_t){dot(qs, c->K + (size_t)m * D, D), VK_LOC, -1, b, m};
  return nv;
}

static const double* vkey_value(const ctx_t* c, int i, const vkey_t* v) {
  int D = c->p->D, nb = c->s->nb;
  if (v->type == VK_ACC) return c->s->Avb[i] + ((size_t)v->j * nb + v->b) * D;
  if (v->type == VK_BLK) return c->s->vb[i] + ((size_t)v->j * nb + v->b) * D;
  return c->V + (size_t)v->m * D;
}

static void needed_clusters(const omuse_params* p, const double* K, const double* V,
                            const int32_t* aq, int nrows, const int32_t* rows, summ_t* s) {
  int cnt = rows ? nrows : p->N;
  for (int t = 0; t < cnt; ++t) {
    int n = rows ? rows[t] : t;
    int i = aq[n];
    if (!s->mu[i]) summaries_for_cluster(p, K, V, s, i);
  }
}

static size_t max_vkeys(const omuse_params* p) {
  size_t nb = (size_t)(p->N / p->Bs);
  return (size_t)p->Ck * (nb + 1) + 2 * (size_t)p->N + 16;
}

/* Forward.  Q,K,V [N,D]; qc [Cq,D] centroids of the raw query rows; aq, ak
 * assignments.  rows == NULL -> all queries.  Outputs for the listed rows:
 * O [N,D], LSE [N], selc [N,r], selb [N,r,k2e], margins [N] (may be NULL).
 * comp_mass [N,4] (may be NULL): softmax mass of each of the four components. */
int oracle_muse_fwd(const omuse_params* p, const double* Q, const double* K, const double* V,
                    const double* qc, const int32_t* aq, const int32_t* ak, int nrows,
                    const int32_t* rows, int sel_given, double* O, double* LSE,
                    int32_t* selc, int32_t* selb, double* margin_c, double* margin_b,
                    double* comp_mass) {
  if (p->N % p->Bs) return -1;
  if (p->dipole && p->r > 0) return -2; /* App. B "Compatibility with Retrieval": not combined */
  int D = p->D, nb = p->N / p->Bs;
  ctx_t c = {p, Q, K, V, aq, ak, summ_new(p, qc, ak), p->k2 == 0 ? (nb > 1 ? nb - 1 : 1) : p->k2};
  needed_clusters(p, K, V, aq, nrows, rows, c.s);
  /* dipole: per-cell covariance / merged matrices are built when first needed and kept */
  double** cbar = NULL; /* [Cq*nb] -> D*D, mode 2 */
  double* covt = NULL;  /* D*D scratch, mode 1 */
  double* dval = NULL;  /* D scratch */
  if (p->dipole) {
    cbar = (double**)calloc((size_t)p->Cq * nb, sizeof(double*));
    covt = (double*)malloc(sizeof(double) * (size_t)D * D);
    dval = (double*)malloc(sizeof(double) * (size_t)D);
  }
  vkey_t* vk = (vkey_t*)malloc(sizeof(vkey_t) * max_vkeys(p));
  double* tmpv = (double*)malloc(sizeof(double) * ((size_t)p->Ck + nb + 1));
  int* tmpi = (int*)malloc(sizeof(int) * ((size_t)p->Ck + nb + 1));
  int* tmpo = (int*)malloc(sizeof(int) * ((size_t)p->Ck + nb + 1));
  double* qs = (double*)malloc(sizeof(double) * 2 * D);
  int cnt = rows ? nrows : p->N;
  for (int t = 0; t < cnt; ++t) {
    int n = rows ? rows[t] : t;
    int nv = build_vkeys(&c, n, sel_given, selc + (size_t)n * p->r,
                         selb + (size_t)n * p->r * c.k2e, margin_c ? margin_c + n : NULL,
                         margin_b ? margin_b + n : NULL, qs, qs + D, vk, tmpv, tmpi, tmpo);
    /* one softmax over the union of the four components */
    double mx = -INFINITY;
    for (int u = 0; u < nv; ++u)
      if (vk[u].logit > mx) mx = vk[u].logit;
    double Z = 0.0;
    for (int u = 0; u < nv; ++u) Z += exp(vk[u].logit - mx);
    double* o = O + (size_t)n * D;
    for (int d = 0; d < D; ++d) o[d] = 0.0;
    if (comp_mass)
      for (int u = 0; u < 4; ++u) comp_mass[(size_t)n * 4 + u] = 0.0;
    double wfar = 0.0; /* share of the accumulated summaries (component 1) in the softmax */
    for (int u = 0; u < nv; ++u) {
      double w = exp(vk[u].logit - mx) / Z;
      const double* val = vkey_value(&c, aq[n], &vk[u]);
      if (p->dipole == 1 && vk[u].type == VK_ACC) {
        /* Eq. "dipole-shift": v-bar + Cov_ij(v,k) q~ with the tilted covariance of the cell */
        cov_vk(&c, c.s->qbar + (size_t)aq[n] * D, vk[u].j, vk[u].b, covt);
        for (int a = 0; a < D; ++a) dval[a] = val[a] + dot(covt + (size_t)a * D, qs + D, D);
        val = dval;
      }
      for (int d = 0; d < D; ++d) o[d] += w * val[d];
      if (vk[u].type == VK_ACC) wfar += w;
      if (comp_mass) comp_mass[(size_t)n * 4 + vk[u].type - 1] += w;
    }
    if (p->dipole == 2 && wfar > 0.0) {
      /* Eq. "premerge": one matrix per (query cluster, query block), applied to q~ */
      int b = n / p->Bs;
      size_t slot = (size_t)aq[n] * nb + b;
      if (!cbar[slot]) {
        cbar[slot] = (double*)malloc(sizeof(double) * (size_t)D * D);
        merged_dipole(&c, aq[n], b, cbar[slot]);
      }
      for (int a = 0; a < D; ++a) o[a] += wfar * dot(cbar[slot] + (size_t)a * D, qs + D, D);
    }
    LSE[n] = mx + log(Z);
  }
  if (p->dipole) {
    for (size_t t = 0; t < (size_t)p->Cq * nb; ++t) free(cbar[t]);
    free(cbar); free(covt); free(dval);
  }
  free(vk); free(tmpv); free(tmpi); free(tmpo); free(qs);
  summ_free(c.s);
  return 0;
}

/* Backward: derivative of (Q,K,V) -> O of oracle_muse_fwd with aq, ak, the
 * selections and q-bar held fixed, contracted with dO, summed over the listed
 * rows.  dQ, dK, dV [N,D] are overwritten. */
int oracle_muse_bwd(const omuse_params* p, const double* Q, const double* K, const double* V,
                    const double* qc, const int32_t* aq, const int32_t* ak, int nrows,
                    const int32_t* rows, const double* O, const double* LSE,
                    const double* dO, const int32_t* selc, const int32_t* selb, double* dQ,
                    double* dK, double* dV) {
  if (p->N % p->Bs) return -1;
  if (p->dipole) return -2; /* the dipole correction is defined for the forward only here */
  int D = p->D, nb = p->N / p->Bs, Ck = p->Ck, Cq = p->Cq, N = p->N;
  ctx_t c = {p, Q, K, V, aq, ak, summ_new(p, qc, ak), p->k2 == 0 ? (nb > 1 ? nb - 1 : 1) : p->k2};
  summ_t* s = c.s;
  needed_clusters(p, K, V, aq, nrows, rows, s);
  memset(dQ, 0, sizeof(double) * (size_t)N * D);
  memset(dK, 0, sizeof(double) * (size_t)N * D);
  memset(dV, 0, sizeof(double) * (size_t)N * D);
  size_t cells = (size_t)Ck * nb;
  /* gradients w.r.t. the normalised summaries (mu, k-bar, v-bar) of every cell */
  double** gmu = (double**)calloc(Cq, sizeof(double*));
  double** gkb = (double**)calloc(Cq, sizeof(double*));
  double** gvb = (double**)calloc(Cq, sizeof(double*));
  double** gAmu = (double**)calloc(Cq, sizeof(double*));
  double** gAkb = (double**)calloc(Cq, sizeof(double*));
  double** gAvb = (double**)calloc(Cq, sizeof(double*));
  for (int i = 0; i < Cq; ++i) {
    if (!s->mu[i]) continue;
    gmu[i] = (double*)calloc(cells, sizeof(double));
    gkb[i] = (double*)calloc(cells * D, sizeof(double));
    gvb[i] = (double*)calloc(cells * D, sizeof(double));
    gAmu[i] = (double*)calloc(cells, sizeof(double));
    gAkb[i] = (double*)calloc(cells * D, sizeof(double));
    gAvb[i] = (double*)calloc(cells * D, sizeof(double));
  }
  vkey_t* vk = (vkey_t*)malloc(sizeof(vkey_t) * max_vkeys(p));
  double* tmpv = (double*)malloc(sizeof(double) * ((size_t)Ck + nb + 1));
  int* tmpi = (int*)malloc(sizeof(int) * ((size_t)Ck + nb + 1));
  int* tmpo = (int*)malloc(sizeof(int) * ((size_t)Ck + nb + 1));
  double* qs = (double*)malloc(sizeof(double) * 2 * D);
  double* qt = qs + D;
  int32_t* sc_tmp = (int32_t*)malloc(sizeof(int32_t) * (size_t)(p->r > 0 ? p->r : 1));
  int32_t* sb_tmp = (int32_t*)malloc(sizeof(int32_t) * (size_t)(p->r > 0 ? p->r : 1) * c.k2e);
  int cnt = rows ? nrows : N;

  /* step 1: through the softmax of every query */
  for (int t = 0; t < cnt; ++t) {
    int n = rows ? rows[t] : t;
    int i = aq[n];
    memcpy(sc_tmp, selc + (size_t)n * p->r, sizeof(int32_t) * p->r);
    memcpy(sb_tmp, selb + (size_t)n * p->r * c.k2e, sizeof(int32_t) * p->r * c.k2e);
    int nv = build_vkeys(&c, n, 1, sc_tmp, sb_tmp, NULL, NULL, qs, qt, vk, tmpv, tmpi, tmpo);
    const double* g = dO + (size_t)n * D;
    double delta = dot(g, O + (size_t)n * D, D);
    for (int u = 0; u < nv; ++u) {
      const double* val = vkey_value(&c, i, &vk[u]);
      double pw = exp(vk[u].logit - LSE[n]);
      double dl = pw * (dot(g, val, D) - delta);
      if (vk[u].type >= VK_RET) { /* real key: logit = scale * q.k */
        int m = vk[u].m;
        for (int d = 0; d < D; ++d) {
          dQ[(size_t)n * D + d] += dl * p->scale * K[(size_t)m * D + d];
          dK[(size_t)m * D + d] += dl * qs[d];
          dV[(size_t)m * D + d] += pw * g[d];
        }
      } else { /* summary cell: logit = q~ . kappa + mu, value = v-bar */
        size_t cell = (size_t)vk[u].j * nb + vk[u].b;
        const double* kap = (vk[u].type == VK_ACC ? s->Akb[i] : s->kb[i]) + cell * D;
        double* gk = (vk[u].type == VK_ACC ? gAkb[i] : gkb[i]) + cell * D;
        double* gv = (vk[u].type == VK_ACC ? gAvb[i] : gvb[i]) + cell * D;
        double* gm = (vk[u].type == VK_ACC ? gAmu[i] : gmu[i]) + cell;
        *gm += dl;
        for (int d = 0; d < D; ++d) {
          /* q~ = scale*q - q-bar with q-bar constant */
          dQ[(size_t)n * D + d] += dl * p->scale * kap[d];
          gk[d] += dl * qt[d];
          gv[d] += pw * g[d];
        }
      }
    }
  }

  /* step 2: through the summaries, in unnormalised form.
   * cell: S = sum e_m, Ksum = sum e_m k_m, Vsum = sum e_m v_m, e_m = exp(q-bar.k_m),
   *       mu = log S, k-bar = Ksum/S, v-bar = Vsum/S
   *   =>  dKsum = g_k/S, dVsum = g_v/S, dS = (g_mu - g_k.k-bar - g_v.v-bar)/S.
   * accumulated cell b = plain sums of (S,Ksum,Vsum) over b' < b, so each
   * per-block cell also receives the gradients of all later accumulated cells. */
  double* dKsum = (double*)malloc(sizeof(double) * D);
  double* dVsum = (double*)malloc(sizeof(double) * D);
  for (int i = 0; i < Cq; ++i) {
    if (!s->mu[i]) continue;
    const double* qb = s->qbar + (size_t)i * D;
    for (int j = 0; j < Ck; ++j) {
      for (int bp = 0; bp < nb; ++bp) {
        size_t cell = (size_t)j * nb + bp;
        if (s->mu[i][cell] == -INFINITY) continue;
        double S = exp(s->mu[i][cell]);
        double dS = (gmu[i][cell] - dot(gkb[i] + cell * D, s->kb[i] + cell * D, D) -
                     dot(gvb[i] + cell * D, s->vb[i] + cell * D, D)) / S;
        for (int d = 0; d < D; ++d) {
          dKsum[d] = gkb[i][cell * D + d] / S;
          dVsum[d] = gvb[i][cell * D + d] / S;
        }
        for (int b = bp + 1; b < nb; ++b) {
          size_t ac = (size_t)j * nb + b;
          double AS = exp(s->Amu[i][ac]);
          dS += (gAmu[i][ac] - dot(gAkb[i] + ac * D, s->Akb[i] + ac * D, D) -
                 dot(gAvb[i] + ac * D, s->Avb[i] + ac * D, D)) / AS;
          for (int d = 0; d < D; ++d) {
            dKsum[d] += gAkb[i][ac * D + d] / AS;
            dVsum[d] += gAvb[i][ac * D + d] / AS;
          }
        }
        /* through the tilted weights to the keys and values of the cell;
         * nothing goes to q-bar.  With frozen weights e_m and S are constants: only the aggregated
         * keys and values receive a gradient (coef = 0). */
        int lo = s->seg_off[bp * Ck + j], hi = s->seg_off[bp * Ck + j + 1];
        for (int u = lo; u < hi; ++u) {
          int m = s->seg_idx[u];
          const double* k = K + (size_t)m * D;
          const double* v = V + (size_t)m * D;
          double e = exp(dot(qb, k, D));
          double coef = p->frozen_weights ? 0.0 : e * (dS + dot(dKsum, k, D) + dot(dVsum, v, D));
          for (int d = 0; d < D; ++d) {
            dV[(size_t)m * D + d] += e * dVsum[d];
            dK[(size_t)m * D + d] += e * dKsum[d] + coef * qb[d];
          }
        }
      }
    }
  }
  free(dKsum); free(dVsum);
  for (int i = 0; i < Cq; ++i) {
    free(gmu[i]); free(gkb[i]); free(gvb[i]); free(gAmu[i]); free(gAkb[i]); free(gAvb[i]);
  }
  free(gmu); free(gkb); free(gvb); free(gAmu); free(gAkb); free(gAvb);
  free(vk); free(tmpv); free(tmpi); free(tmpo); free(qs); free(sc_tmp); free(sb_tmp);
  summ_free(c.s);
  return 0;
}
