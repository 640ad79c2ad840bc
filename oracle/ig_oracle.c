/*
 * CPU oracle for the InfiniGen attention rehearsal and the sparse decode attention it drives.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain restatement of what the method
 * computes, written from the paper; it shares no code with the HIP library and is imported only
 * by the tests, by the smoke check and by the benchmark's CPU-baseline leg.
 *
 * Conventions: row-major arrays; projections are y = x W with W [in, out] (Section 2.1).
 * All arrays are float32; every sum is accumulated in double and rounded to float once, so a
 * result does not depend on summation order.  Decisions (the threshold test) are taken on the
 * rounded float32 scores, the precision the GPU path also decides in.
 *
 * Pins (tests/test_oracle_*.py): skew invariance and SVD structure (Section 4.2, Eq. 2 and Eq. 3),
 * brute-force column ranking, dense-attention equivalence, brute-force threshold enumeration,
 * the exp(-alpha) weight bound of Section 4.3, singular values against LAPACK; the head-equalised
 * selection against rank counting, its reduction to the threshold lists when all heads agree,
 * and the 20 % cap against the token budget the paper prints (Section 5.3: 409 of 2048);
 * the pool counters against hand-worked cases and an array formulation.
 * Unpinned: how well the speculated set recalls the true one (the paper gives model-level
 * accuracy only) -- "parity unpinned" for approximation quality; it is reported, never asserted.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define IGO_OK 0
#define IGO_EINVAL 1
#define IGO_ENOCONV 2
#define IGO_ENOMEM 3

/* ------------------------------------------------------------------------------------------
 * Offline skewing (Section 4.2 "Skewed Partial Weight", Eq. 2 and Eq. 3; Section 4.3
 * "Prefetching Scheme").  For every head h the n_cal x d block Q_h of the calibration query
 * matrix is factored Q_h = U S V^T and A_h = V, so that Q_h A_h = U S.  The query / key
 * weights of that head are multiplied by A_h from the right.  Reading: A is block diagonal,
 * one d x d block per head, because the identity of Eq. 2 is per head.
 *
 * The SVD is a one-sided Jacobi (Hestenes) iteration in double: columns of a working copy G
 * of Q_h are rotated pairwise until mutually orthogonal, the same rotations accumulated in V.
 * Then G = U S column-wise, |G_j| = sigma_j.  Columns are sorted by descending sigma, and each
 * column of V has its sign chosen so that its largest-magnitude entry is positive.
 * ------------------------------------------------------------------------------------------ */
static int jacobi_svd_v(int n, int d, const double *Q /*[n,d]*/, double *V /*[d,d]*/,
                        double *sigma /*[d]*/) {
  double *G = (double *)malloc(sizeof(double) * (size_t)n * d);
  if (!G) return IGO_ENOMEM;
  memcpy(G, Q, sizeof(double) * (size_t)n * d);
  for (int i = 0; i < d; ++i)
    for (int j = 0; j < d; ++j) V[i * d + j] = (i == j) ? 1.0 : 0.0;
  const double eps = 1e-15;
  int converged = 0;
  for (int sweep = 0; sweep < 60 && !converged; ++sweep) {
    converged = 1;
    for (int p = 0; p < d - 1; ++p) {
      for (int q = p + 1; q < d; ++q) {
        double a = 0, b = 0, g = 0;
        for (int i = 0; i < n; ++i) {
          double gp = G[i * d + p], gq = G[i * d + q];
          a += gp * gp;
          b += gq * gq;
          g += gp * gq;
        }
        if (fabs(g) <= eps * sqrt(a * b) || g == 0.0) continue;
        converged = 0;
        double zeta = (b - a) / (2.0 * g);
        double t = (zeta >= 0 ? 1.0 : -1.0) / (fabs(zeta) + sqrt(1.0 + zeta * zeta));
        double c = 1.0 / sqrt(1.0 + t * t), s = c * t;
        for (int i = 0; i < n; ++i) {
          double gp = G[i * d + p], gq = G[i * d + q];
          G[i * d + p] = c * gp - s * gq;
          G[i * d + q] = s * gp + c * gq;
        }
        for (int i = 0; i < d; ++i) {
          double vp = V[i * d + p], vq = V[i * d + q];
          V[i * d + p] = c * vp - s * vq;
          V[i * d + q] = s * vp + c * vq;
        }
      }
    }
  }
  for (int j = 0; j < d; ++j) {
    double a = 0;
    for (int i = 0; i < n; ++i) a += G[i * d + j] * G[i * d + j];
    sigma[j] = sqrt(a);
  }
  free(G);
  /* sort columns by descending sigma (selection sort; d is small) */
  for (int j = 0; j < d - 1; ++j) {
    int best = j;
    for (int k = j + 1; k < d; ++k)
      if (sigma[k] > sigma[best]) best = k;
    if (best != j) {
      double ts = sigma[j];
      sigma[j] = sigma[best];
      sigma[best] = ts;
      for (int i = 0; i < d; ++i) {
        double tv = V[i * d + j];
        V[i * d + j] = V[i * d + best];
        V[i * d + best] = tv;
      }
    }
  }
  /* sign convention: largest-magnitude entry of every column positive */
  for (int j = 0; j < d; ++j) {
    int arg = 0;
    for (int i = 1; i < d; ++i)
      if (fabs(V[i * d + j]) > fabs(V[arg * d + j])) arg = i;
    if (V[arg * d + j] < 0)
      for (int i = 0; i < d; ++i) V[i * d + j] = -V[i * d + j];
  }
  return converged ? IGO_OK : IGO_ENOCONV;
}

/* out[:, head h] = W[:, head h] * A_h for a [rows, D] matrix W (rows = D for weights, 1 for a bias). */
static void right_multiply_heads(int rows, int D, int H, const float *W, const float *A, float *out) {
  int d = D / H;
  for (int i = 0; i < rows; ++i)
    for (int h = 0; h < H; ++h)
      for (int j = 0; j < d; ++j) {
        double acc = 0;
        for (int k = 0; k < d; ++k)
          acc += (double)W[(size_t)i * D + h * d + k] * (double)A[((size_t)h * d + k) * d + j];
        out[(size_t)i * D + h * d + j] = (float)acc;
      }
}

int igo_skew(int D, int H, int n_cal, const float *Wq, const float *Wk, const float *bq,
             const float *bk, const float *Qcal /*[n_cal,D]*/, float *A /*[H,d,d]*/,
             float *sigma_out /*[H,d] or NULL*/, float *Wq_s, float *Wk_s, float *bq_s,
             float *bk_s) {
  if (D <= 0 || H <= 0 || D % H || n_cal <= 0 || !Qcal || !A) return IGO_EINVAL;
  int d = D / H;
  double *Qh = (double *)malloc(sizeof(double) * (size_t)n_cal * d);
  double *V = (double *)malloc(sizeof(double) * (size_t)d * d);
  double *sg = (double *)malloc(sizeof(double) * d);
  if (!Qh || !V || !sg) return IGO_ENOMEM;
  int rc = IGO_OK;
  for (int h = 0; h < H; ++h) {
    for (int i = 0; i < n_cal; ++i)
      for (int j = 0; j < d; ++j) Qh[(size_t)i * d + j] = Qcal[(size_t)i * D + h * d + j];
    int r = jacobi_svd_v(n_cal, d, Qh, V, sg);
    if (r != IGO_OK) rc = r;
    for (int i = 0; i < d * d; ++i) A[(size_t)h * d * d + i] = (float)V[i];
    if (sigma_out)
      for (int j = 0; j < d; ++j) sigma_out[h * d + j] = (float)sg[j];
  }
  free(Qh);
  free(V);
  free(sg);
  if (Wq && Wq_s) right_multiply_heads(D, D, H, Wq, A, Wq_s);
  if (Wk && Wk_s) right_multiply_heads(D, D, H, Wk, A, Wk_s);
  if (bq && bq_s) right_multiply_heads(1, D, H, bq, A, bq_s);
  if (bk && bk_s) right_multiply_heads(1, D, H, bk, A, bk_s);
  return rc;
}

/* Apply per-head skewing matrices to row vectors: Y[row, head h] = X[row, head h] * A_h.
 * (Q~ = Q A, K~ = K A of Eq. 2.)  X, Y are [rows, H*d]. */
int igo_apply_skew(int rows, int H, int d, const float *X, const float *A, float *Y) {
  if (rows < 0 || H <= 0 || d <= 0) return IGO_EINVAL;
  right_multiply_heads(rows, H * d, H, X, A, Y);
  return IGO_OK;
}

/* ------------------------------------------------------------------------------------------
 * Rotary position embedding, rotate-half pairing (j, j + d/2), angle pos * theta^(-2j/d).
 * The paper evaluates Llama-2 but does not state how skewing composes with it; the workload
 * definition fixes "rotary embedding applied to q / k before skewing".  X is [rows, H, d],
 * pos is [rows]; in place allowed.
 * ------------------------------------------------------------------------------------------ */
int igo_rope(int rows, int H, int d, const int32_t *pos, double theta, const float *X, float *Y) {
  if (d % 2) return IGO_EINVAL;
  int half = d / 2;
  for (int i = 0; i < rows; ++i)
    for (int h = 0; h < H; ++h) {
      const float *x = X + ((size_t)i * H + h) * d;
      float *y = Y + ((size_t)i * H + h) * d;
      for (int j = 0; j < half; ++j) {
        double ang = (double)pos[i] * pow(theta, -2.0 * j / d);
        double c = cos(ang), s = sin(ang);
        double a = x[j], b = x[j + half];
        y[j] = (float)(a * c - b * s);
        y[j + half] = (float)(b * c + a * s);
      }
    }
  return IGO_OK;
}

/* ------------------------------------------------------------------------------------------
 * Partial weight index generation (Section 4.3 "Prefill Stage").  Element-wise absolute values
 * of the skewed query and key matrices are added, every column is summed over the rows, and the
 * top-k columns are kept; k = floor(ratio * d) per head (30 % in the paper).  Ks == NULL ranks
 * by the query term alone.  Ties go to the lower column; indices are returned ascending.
 * Qs, Ks are [n, H*d]; idx is [H, r].
 * ------------------------------------------------------------------------------------------ */
int igo_partial_index(int H, int d, int n, const float *Qs, const float *Ks, double ratio,
                      int32_t *idx, int32_t *r_out) {
  if (H <= 0 || d <= 0 || n <= 0 || !Qs || !(ratio > 0.0) || ratio > 1.0) return IGO_EINVAL;
  int r = (int)floor(ratio * (double)d);
  if (r < 1) return IGO_EINVAL;
  if (r_out) *r_out = r;
  if (!idx) return IGO_OK;
  int D = H * d;
  double *c = (double *)malloc(sizeof(double) * d);
  char *taken = (char *)malloc(d);
  if (!c || !taken) return IGO_ENOMEM;
  for (int h = 0; h < H; ++h) {
    for (int j = 0; j < d; ++j) {
      double acc = 0;
      for (int i = 0; i < n; ++i) {
        acc += fabs((double)Qs[(size_t)i * D + h * d + j]);
        if (Ks) acc += fabs((double)Ks[(size_t)i * D + h * d + j]);
      }
      c[j] = acc;
    }
    memset(taken, 0, d);
    for (int k = 0; k < r; ++k) {
      int best = -1;
      for (int j = 0; j < d; ++j)
        if (!taken[j] && (best < 0 || c[j] > c[best])) best = j;
      taken[best] = 1;
    }
    int k = 0;
    for (int j = 0; j < d; ++j)
      if (taken[j]) idx[h * r + k++] = j;
  }
  free(c);
  free(taken);
  return IGO_OK;
}

/* ------------------------------------------------------------------------------------------
 * Partial query projection (Section 4.3 "Decoding Stage"): the attention input of the previous
 * layer times the partial (column-sliced) skewed query weight.
 *   q_p[b,h,k] = sum_i x[b,i] * Wq_s[i, h*d + idx[h,k]]  (+ bq_s[h*d + idx[h,k]])
 * x [B,D], Wq_s [D,D], q_p [B,H,r].
 * ------------------------------------------------------------------------------------------ */
int igo_project(int B, int H, int d, int r, const float *x, const float *Wq_s, const float *bq_s,
                const int32_t *idx, float *q_p) {
  int D = H * d;
  for (int b = 0; b < B; ++b)
    for (int h = 0; h < H; ++h)
      for (int k = 0; k < r; ++k) {
        int col = h * d + idx[h * r + k];
        double acc = bq_s ? (double)bq_s[col] : 0.0;
        for (int i = 0; i < D; ++i) acc += (double)x[(size_t)b * D + i] * (double)Wq_s[(size_t)i * D + col];
        q_p[((size_t)b * H + h) * r + k] = (float)acc;
      }
  return IGO_OK;
}

/* Same step for a model with rotary embedding between projection and skewing: the full query
 * q = x Wq (+ bq) is rotated at the sequence's current position, then multiplied by the kept
 * columns of the head's skewing matrix: q_p[b,h,k] = sum_j rot(q)[b,h,j] * A_h[j, idx[h,k]]. */
int igo_project_rope(int B, int H, int d, int r, const float *x, const float *Wq, const float *bq,
                     const int32_t *pos, double theta, const float *A, const int32_t *idx,
                     float *q_p) {
  int D = H * d, half = d / 2;
  if (d % 2) return IGO_EINVAL;
  double *q = (double *)malloc(sizeof(double) * D);
  double *qr = (double *)malloc(sizeof(double) * D);
  if (!q || !qr) return IGO_ENOMEM;
  for (int b = 0; b < B; ++b) {
    for (int c = 0; c < D; ++c) {
      double acc = bq ? (double)bq[c] : 0.0;
      for (int i = 0; i < D; ++i) acc += (double)x[(size_t)b * D + i] * (double)Wq[(size_t)i * D + c];
      q[c] = acc;
    }
    for (int h = 0; h < H; ++h)
      for (int j = 0; j < half; ++j) {
        double ang = (double)pos[b] * pow(theta, -2.0 * j / d);
        double cs = cos(ang), sn = sin(ang);
        double a = q[h * d + j], bb = q[h * d + j + half];
        qr[h * d + j] = a * cs - bb * sn;
        qr[h * d + j + half] = bb * cs + a * sn;
      }
    for (int h = 0; h < H; ++h)
      for (int k = 0; k < r; ++k) {
        double acc = 0;
        for (int j = 0; j < d; ++j)
          acc += qr[h * d + j] * (double)A[((size_t)h * d + j) * d + idx[h * r + k]];
        q_p[((size_t)b * H + h) * r + k] = (float)acc;
      }
  }
  free(q);
  free(qr);
  return IGO_OK;
}

/* ------------------------------------------------------------------------------------------
 * Speculated attention score (Section 4.3 "Decoding Stage", Fig. 10): partial query times the
 * partial key cache, i.e. the kept columns of the skewed keys of all N cached tokens.
 *   s[b,h,t] = scale * sum_k q_p[b,h,k] * Kt[b,h,t, idx[h,k]]
 * Kt [B,H,N_cap,d] (only t < N read), s [B,H,N].  Reading: "score" is the softmax logit, so
 * the same scale as in the attention itself applies (the alpha example of Section 4.3 divides
 * weights by e^alpha, which needs the score to be the logit).
 * ------------------------------------------------------------------------------------------ */
int igo_scan(int B, int H, int N, int N_cap, int d, int r, float scale, const float *q_p,
             const float *Kt, const int32_t *idx, float *s) {
  for (int b = 0; b < B; ++b)
    for (int h = 0; h < H; ++h) {
      const float *qp = q_p + ((size_t)b * H + h) * r;
      for (int t = 0; t < N; ++t) {
        const float *k = Kt + (((size_t)b * H + h) * N_cap + t) * d;
        double acc = 0;
        for (int j = 0; j < r; ++j) acc += (double)qp[j] * (double)k[idx[h * r + j]];
        s[((size_t)b * H + h) * N + t] = (float)((double)scale * acc);
      }
    }
  return IGO_OK;
}

/* ------------------------------------------------------------------------------------------
 * Token selection (Section 4.3 "Decoding Stage"): per head, keep the tokens whose speculated
 * score reaches the maximum score minus alpha.  Reading: "at least" (>=); the argmax is always
 * kept.  Lists are ascending in t.  alpha = +inf keeps every token.  sel_idx [B*H, stride],
 * sel_cnt [B*H]; a list longer than stride is an error here (the oracle never truncates).
 * ------------------------------------------------------------------------------------------ */
int igo_select(int B, int H, int N, const float *s, float alpha, int32_t *sel_idx, int32_t stride,
               int32_t *sel_cnt) {
  if (!(alpha >= 0.0f)) return IGO_EINVAL;
  for (int bh = 0; bh < B * H; ++bh) {
    const float *sc = s + (size_t)bh * N;
    float m = -INFINITY;
    for (int t = 0; t < N; ++t)
      if (sc[t] > m) m = sc[t];
    float thr = m - alpha;
    int n = 0;
    for (int t = 0; t < N; ++t)
      if (sc[t] >= thr) {
        if (n >= stride) return IGO_EINVAL;
        sel_idx[(size_t)bh * stride + n++] = t;
      }
    sel_cnt[bh] = n;
  }
  return IGO_OK;
}

/* ------------------------------------------------------------------------------------------
 * Head-equalised selection (Section 4.3 "Decoding Stage", last sentences; Section 5.1 "Key
 * Metric"): heads of a layer are computed in parallel, so every head fetches the same number of
 * tokens, the average over the heads of the number of tokens between the maximum score and the
 * threshold; a layer sends at most max_frac (20 %) of the cache.
 * Readings: the average is taken per sequence, over its H heads, and truncated:
 *   c[b,h] = #{ t : s[b,h,t] >= max_t s[b,h,t] - alpha },  n_b = floor(sum_h c[b,h] / H),
 *   n_b <- min(n_b, floor(max_frac * N)),  n_b <- max(n_b, 1);
 * head (b,h) then keeps its n_b highest-scoring tokens (equal scores: the earlier token first),
 * listed in ascending t.  n_eq [B] receives n_b; sel_cnt [B*H] = n_b for every head of b.
 * The order "score descending, then t ascending" is produced by a plain sort of (score, t) pairs.
 * ------------------------------------------------------------------------------------------ */
typedef struct {
  float s;
  int32_t t;
} igo_scored;

static int igo_by_score_then_token(const void *a, const void *b) {
  const igo_scored *x = (const igo_scored *)a, *y = (const igo_scored *)b;
  if (x->s > y->s) return -1;
  if (x->s < y->s) return 1;
  return (x->t > y->t) - (x->t < y->t);
}

static int igo_by_token(const void *a, const void *b) {
  const int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
  return (x > y) - (x < y);
}

int igo_select_equalized(int B, int H, int N, const float *s, float alpha, double max_frac,
                         int32_t *sel_idx, int32_t stride, int32_t *sel_cnt, int32_t *n_eq) {
  if (!(alpha >= 0.0f) || !(max_frac > 0.0) || max_frac > 1.0) return IGO_EINVAL;
  igo_scored *v = (igo_scored *)malloc(sizeof(igo_scored) * (size_t)N);
  if (!v) return IGO_ENOMEM;
  int cap = (int)floor(max_frac * (double)N);
  if (cap < 1) cap = 1;
  for (int b = 0; b < B; ++b) {
    long total = 0;
    for (int h = 0; h < H; ++h) {
      const float *sc = s + ((size_t)b * H + h) * N;
      float m = -INFINITY;
      for (int t = 0; t < N; ++t)
        if (sc[t] > m) m = sc[t];
      const float thr = m - alpha;
      for (int t = 0; t < N; ++t)
        if (sc[t] >= thr) ++total;
    }
    int n = (int)(total / H);
    if (n > cap) n = cap;
    if (n < 1) n = 1;
    if (n > stride) {
      free(v);
      return IGO_EINVAL;
    }
    if (n_eq) n_eq[b] = n;
    for (int h = 0; h < H; ++h) {
      const size_t bh = (size_t)b * H + h;
      for (int t = 0; t < N; ++t) {
        v[t].s = s[bh * N + t];
        v[t].t = t;
      }
      qsort(v, (size_t)N, sizeof(igo_scored), igo_by_score_then_token);
      for (int j = 0; j < n; ++j) sel_idx[bh * stride + j] = v[j].t;
      qsort(sel_idx + bh * stride, (size_t)n, sizeof(int32_t), igo_by_token);
      sel_cnt[bh] = n;
    }
  }
  free(v);
  return IGO_OK;
}

/* ------------------------------------------------------------------------------------------
 * KV cache pool management, counter-based policy (Section 4.4): the pool manager increments a
 * counter for each prefetched KV entry; the victim is the entry with the smallest count; if any
 * counter becomes saturated, all counter values are reduced by half.  The victim is overwritten
 * by the newly generated key and value (the order of entries in the pool is arbitrary).
 * Readings: one counter per pool slot of every (sequence, head) pool, counters [B*H, N_cap];
 * a counter is saturated when it reaches counter_max; the halving (integer division by two) is
 * applied to the pool of that (sequence, head) after all increments of the step; equal smallest
 * counts: the lowest slot; an overwritten slot restarts at zero (done by the caller here: the
 * oracle only names the victim).
 * ------------------------------------------------------------------------------------------ */
int igo_pool_touch(int BH, int N, int N_cap, const int32_t *sel_idx, int32_t stride,
                   const int32_t *sel_cnt, int32_t *counters, int32_t counter_max) {
  if (counter_max < 1) return IGO_EINVAL;
  for (int bh = 0; bh < BH; ++bh) {
    int32_t *c = counters + (size_t)bh * N_cap;
    int saturated = 0;
    for (int j = 0; j < sel_cnt[bh]; ++j) {
      int t = sel_idx[(size_t)bh * stride + j];
      if (t < 0 || t >= N) return IGO_EINVAL;
      if (c[t] < counter_max) c[t] += 1;
      if (c[t] >= counter_max) saturated = 1;
    }
    if (saturated)
      for (int t = 0; t < N; ++t) c[t] /= 2;
  }
  return IGO_OK;
}

int igo_pool_victim(int BH, int N, int N_cap, const int32_t *counters, int32_t *victim) {
  if (N < 1) return IGO_EINVAL;
  for (int bh = 0; bh < BH; ++bh) {
    const int32_t *c = counters + (size_t)bh * N_cap;
    int best = 0;
    for (int t = 1; t < N; ++t)
      if (c[t] < c[best]) best = t;
    victim[bh] = best;
  }
  return IGO_OK;
}

/* ------------------------------------------------------------------------------------------
 * The two comparison policies of Section 4.4 (Table 2): FIFO evicts the oldest residing entry
 * regardless of its use; LRU evicts the entry whose last use lies furthest back (the paper names
 * the usual doubly linked list that promotes accessed entries to the head; the victim such a list
 * yields is the entry with the oldest last-use time, which is what is written out here).
 * Readings: time is a step number the caller supplies (any non-decreasing int32); every pool slot
 * carries one stamp, stamps [B*H, N_cap]: FIFO -- the step its entry was written (prefill entries:
 * their token position, so that the prompt's first token is the oldest); LRU -- the step its entry
 * was last prefetched or written.  "Use" is being prefetched, as for the counter policy.  Equal
 * stamps: the lowest slot.  The overwritten slot gets the current step (done by the caller here).
 * ------------------------------------------------------------------------------------------ */
int igo_pool_touch_lru(int BH, int N, int N_cap, const int32_t *sel_idx, int32_t stride,
                       const int32_t *sel_cnt, int32_t *stamps, int32_t now) {
  for (int bh = 0; bh < BH; ++bh)
    for (int j = 0; j < sel_cnt[bh]; ++j) {
      int t = sel_idx[(size_t)bh * stride + j];
      if (t < 0 || t >= N) return IGO_EINVAL;
      stamps[(size_t)bh * N_cap + t] = now;
    }
  return IGO_OK;
}

/* oldest stamp among the first N slots of every pool: the FIFO victim when the stamps are
 * insertion steps, the LRU victim when they are last-use steps */
int igo_pool_victim_oldest(int BH, int N, int N_cap, const int32_t *stamps, int32_t *victim) {
  if (N < 1) return IGO_EINVAL;
  for (int bh = 0; bh < BH; ++bh) {
    const int32_t *s = stamps + (size_t)bh * N_cap;
    int oldest = 0;
    for (int t = 1; t < N; ++t)
      if (s[t] < s[oldest]) oldest = t;
    victim[bh] = oldest;
  }
  return IGO_OK;
}

/* ------------------------------------------------------------------------------------------
 * Prefetch of the selected rows (Section 4.1, Section 4.3): plain row copies out of the pool.
 * pool [B*H, N_cap, d] -> out [B*H, stride, d]; rows j >= sel_cnt are left untouched.
 * ------------------------------------------------------------------------------------------ */
int igo_gather(int BH, int N_cap, int d, const float *pool, const int32_t *sel_idx, int32_t stride,
               const int32_t *sel_cnt, float *out) {
  for (int bh = 0; bh < BH; ++bh)
    for (int j = 0; j < sel_cnt[bh]; ++j) {
      int t = sel_idx[(size_t)bh * stride + j];
      if (t < 0 || t >= N_cap) return IGO_EINVAL;
      memcpy(out + ((size_t)bh * stride + j) * d, pool + ((size_t)bh * N_cap + t) * d,
             sizeof(float) * d);
    }
  return IGO_OK;
}

/* ------------------------------------------------------------------------------------------
 * Decode attention over the fetched rows only (Section 2.1: softmax(Q K^T) V per head; Section
 * 4.1: computed with the few important tokens).  One query row per (b,h):
 *   l_j = scale * q . K_sel[j],  p = softmax(l),  out = sum_j p_j V_sel[j]
 * An optional extra row (k_new, v_new: the token being decoded, whose key did not exist when
 * the selection was speculated) is always attended.  q, out, k_new, v_new [B*H, d];
 * K_sel, V_sel [B*H, stride, d].
 * ------------------------------------------------------------------------------------------ */
int igo_attend(int BH, int d, int32_t stride, float scale, const float *q, const float *K_sel,
               const float *V_sel, const int32_t *sel_cnt, const float *k_new, const float *v_new,
               float *out) {
  for (int bh = 0; bh < BH; ++bh) {
    int n = sel_cnt[bh];
    int rows = n + (k_new ? 1 : 0);
    const float *qv = q + (size_t)bh * d;
    double *l = (double *)malloc(sizeof(double) * (rows > 0 ? rows : 1));
    if (!l) return IGO_ENOMEM;
    double m = -INFINITY;
    for (int j = 0; j < rows; ++j) {
      const float *k = (j < n) ? K_sel + ((size_t)bh * stride + j) * d : k_new + (size_t)bh * d;
      double acc = 0;
      for (int c = 0; c < d; ++c) acc += (double)qv[c] * (double)k[c];
      l[j] = (double)scale * acc;
      if (l[j] > m) m = l[j];
    }
    double z = 0;
    for (int j = 0; j < rows; ++j) {
      l[j] = exp(l[j] - m);
      z += l[j];
    }
    for (int c = 0; c < d; ++c) {
      double acc = 0;
      for (int j = 0; j < rows; ++j) {
        const float *v = (j < n) ? V_sel + ((size_t)bh * stride + j) * d : v_new + (size_t)bh * d;
        acc += l[j] * (double)v[c];
      }
      out[(size_t)bh * d + c] = rows > 0 ? (float)(acc / z) : 0.0f;
    }
    free(l);
  }
  return IGO_OK;
}
