// Host-side, offline parts of the library: weight skewing and partial weight index generation.
// Plain C++ (no GPU calls); float32 data, double arithmetic.
#include <math.h>
#include <stdint.h>
#include <string.h>

#include <algorithm>
#include <numeric>
#include <vector>

#include "../../include/infinigen.h"

struct ig_ctx;
int ig_fail(ig_ctx *ctx, int code, const char *fmt, ...);

namespace {

// Eigen-decomposition of a symmetric d x d matrix by cyclic two-sided Jacobi rotations.
// On return G's diagonal holds the eigenvalues and the columns of V the eigenvectors.
bool jacobi_eigen(int d, std::vector<double> &G, std::vector<double> &V) {
  V.assign((size_t)d * d, 0.0);
  for (int i = 0; i < d; ++i) V[(size_t)i * d + i] = 1.0;
  for (int sweep = 0; sweep < 80; ++sweep) {
    bool rotated = false;
    for (int p = 0; p < d - 1; ++p)
      for (int q = p + 1; q < d; ++q) {
        double gpq = G[(size_t)p * d + q];
        double gpp = G[(size_t)p * d + p], gqq = G[(size_t)q * d + q];
        if (gpq == 0.0 || fabs(gpq) <= 1e-17 * sqrt(fabs(gpp * gqq))) continue;
        rotated = true;
        double theta = (gqq - gpp) / (2.0 * gpq);
        double t = (theta >= 0 ? 1.0 : -1.0) / (fabs(theta) + sqrt(theta * theta + 1.0));
        double c = 1.0 / sqrt(t * t + 1.0), s = t * c;
        for (int k = 0; k < d; ++k) {   // columns p, q
          double a = G[(size_t)k * d + p], b = G[(size_t)k * d + q];
          G[(size_t)k * d + p] = c * a - s * b;
          G[(size_t)k * d + q] = s * a + c * b;
        }
        for (int k = 0; k < d; ++k) {   // rows p, q
          double a = G[(size_t)p * d + k], b = G[(size_t)q * d + k];
          G[(size_t)p * d + k] = c * a - s * b;
          G[(size_t)q * d + k] = s * a + c * b;
        }
        for (int k = 0; k < d; ++k) {
          double a = V[(size_t)k * d + p], b = V[(size_t)k * d + q];
          V[(size_t)k * d + p] = c * a - s * b;
          V[(size_t)k * d + q] = s * a + c * b;
        }
      }
    if (!rotated) return true;
  }
  return false;
}

// out[:, head h] = W[:, head h] * A_h, rows of W processed one at a time.
void skew_rows(int rows, int D, int H, const float *W, const float *A, float *out) {
  const int d = D / H;
  std::vector<double> acc(d);
  for (int i = 0; i < rows; ++i)
    for (int h = 0; h < H; ++h) {
      std::fill(acc.begin(), acc.end(), 0.0);
      const float *w = W + (size_t)i * D + (size_t)h * d;
      const float *a = A + (size_t)h * d * d;
      for (int k = 0; k < d; ++k) {
        const double wk = w[k];
        const float *ak = a + (size_t)k * d;
        for (int j = 0; j < d; ++j) acc[j] += wk * (double)ak[j];
      }
      float *o = out + (size_t)i * D + (size_t)h * d;
      for (int j = 0; j < d; ++j) o[j] = (float)acc[j];
    }
}

}  // namespace

extern "C" int ig_skew_offline(ig_ctx *ctx, int D, int H, int n_cal, const float *Wq, const float *Wk,
                               const float *bq, const float *bk, const float *Qcal, float *A,
                               float *sigma, float *Wq_s, float *Wk_s, float *bq_s, float *bk_s) {
  if (D < 1 || H < 1 || D % H || n_cal < 1) return ig_fail(ctx, IG_ESHAPE, "ig_skew_offline: bad shape");
  if (!Qcal || !A) return ig_fail(ctx, IG_EINVAL, "ig_skew_offline: Qcal or A is NULL");
  const int d = D / H;
  int rc = IG_OK;
  std::vector<double> G((size_t)d * d), V, qrow(d);
  std::vector<int> order(d);
  for (int h = 0; h < H; ++h) {
    // Gram matrix of the head's calibration queries: Q_h^T Q_h = V S^2 V^T, so its eigenvectors
    // are the right singular vectors of Q_h and its eigenvalues the squared singular values.
    std::fill(G.begin(), G.end(), 0.0);
    for (int i = 0; i < n_cal; ++i) {
      const float *row = Qcal + (size_t)i * D + (size_t)h * d;
      for (int a = 0; a < d; ++a) qrow[a] = row[a];
      for (int a = 0; a < d; ++a) {
        const double qa = qrow[a];
        double *g = &G[(size_t)a * d];
        for (int b = a; b < d; ++b) g[b] += qa * qrow[b];
      }
    }
    for (int a = 0; a < d; ++a)
      for (int b = 0; b < a; ++b) G[(size_t)a * d + b] = G[(size_t)b * d + a];
    if (!jacobi_eigen(d, G, V)) rc = IG_ENOCONV;
    std::iota(order.begin(), order.end(), 0);
    std::stable_sort(order.begin(), order.end(), [&](int x, int y) {
      return G[(size_t)x * d + x] > G[(size_t)y * d + y];
    });
    float *Ah = A + (size_t)h * d * d;
    for (int j = 0; j < d; ++j) {
      const int src = order[j];
      int arg = 0;
      for (int i = 1; i < d; ++i)
        if (fabs(V[(size_t)i * d + src]) > fabs(V[(size_t)arg * d + src])) arg = i;
      const double sgn = V[(size_t)arg * d + src] < 0 ? -1.0 : 1.0;
      for (int i = 0; i < d; ++i) Ah[(size_t)i * d + j] = (float)(sgn * V[(size_t)i * d + src]);
      if (sigma) sigma[(size_t)h * d + j] = (float)sqrt(std::max(0.0, G[(size_t)src * d + src]));
    }
  }
  if (Wq && Wq_s) skew_rows(D, D, H, Wq, A, Wq_s);
  if (Wk && Wk_s) skew_rows(D, D, H, Wk, A, Wk_s);
  if (bq && bq_s) skew_rows(1, D, H, bq, A, bq_s);
  if (bk && bk_s) skew_rows(1, D, H, bk, A, bk_s);
  if (rc == IG_ENOCONV) return ig_fail(ctx, rc, "ig_skew_offline: Jacobi sweeps exceeded their cap");
  return rc;
}

extern "C" int ig_partial_index(ig_ctx *ctx, int H, int d, int n, const float *Qs, const float *Ks,
                                double ratio, int32_t *idx, int32_t *r_out) {
  if (H < 1 || d < 1 || n < 1) return ig_fail(ctx, IG_ESHAPE, "ig_partial_index: bad shape");
  if (!Qs) return ig_fail(ctx, IG_EINVAL, "ig_partial_index: Qs is NULL");
  if (!(ratio > 0.0) || ratio > 1.0) return ig_fail(ctx, IG_EINVAL, "ig_partial_index: ratio must be in (0, 1]");
  const int r = (int)floor(ratio * (double)d);
  if (r < 1) return ig_fail(ctx, IG_ESHAPE, "ig_partial_index: ratio * d < 1");
  if (r_out) *r_out = r;
  if (!idx) return IG_OK;
  const size_t D = (size_t)H * d;
  std::vector<double> colsum(D, 0.0);
  for (int i = 0; i < n; ++i) {
    const float *qrow = Qs + (size_t)i * D;
    for (size_t c = 0; c < D; ++c) colsum[c] += fabs((double)qrow[c]);
    if (Ks) {
      const float *krow = Ks + (size_t)i * D;
      for (size_t c = 0; c < D; ++c) colsum[c] += fabs((double)krow[c]);
    }
  }
  std::vector<int> order(d);
  for (int h = 0; h < H; ++h) {
    const double *c = &colsum[(size_t)h * d];
    std::iota(order.begin(), order.end(), 0);
    std::stable_sort(order.begin(), order.end(), [&](int x, int y) { return c[x] > c[y]; });
    std::vector<int> keep(order.begin(), order.begin() + r);
    std::sort(keep.begin(), keep.end());
    for (int k = 0; k < r; ++k) idx[(size_t)h * r + k] = keep[k];
  }
  return IG_OK;
}

// Y[:, head h] = X[:, head h] * A_h for every row of X (Eq. 2: the skewed query / key matrix of a
// set of rows, e.g. the prompt's queries that ig_partial_index ranks).  In place when Y == X.
extern "C" int ig_apply_skew(ig_ctx *ctx, int H, int d, int n, const float *X, const float *A, float *Y) {
  if (H < 1 || d < 1 || n < 1) return ig_fail(ctx, IG_ESHAPE, "ig_apply_skew: bad shape");
  if (!X || !A || !Y) return ig_fail(ctx, IG_EINVAL, "ig_apply_skew: NULL argument");
  skew_rows(n, H * d, H, X, A, Y);   // a row's head block is read in full before it is written
  return IG_OK;
}

// Rotary embedding of rows [n, H, d] in place, row i at position pos[i]: pairs (c, c + d/2) are
// rotated by pos * theta^(-2c/d) (the convention of the rehearsal's own rotation, so that queries a
// caller prepares on the host -- calibration queries, a layer's real query -- match the keys).
extern "C" int ig_rope_rows(ig_ctx *ctx, int n, int H, int d, const int32_t *pos, double theta, float *q) {
  if (n < 1 || H < 1 || d < 2 || d % 2) return ig_fail(ctx, IG_ESHAPE, "ig_rope_rows: bad shape (d must be even)");
  if (!pos || !q) return ig_fail(ctx, IG_EINVAL, "ig_rope_rows: NULL argument");
  if (!(theta > 0.0)) return ig_fail(ctx, IG_EINVAL, "ig_rope_rows: theta must be positive");
  const int half = d / 2;
  std::vector<double> freq(half);
  for (int c = 0; c < half; ++c) freq[c] = pow(theta, -2.0 * (double)c / (double)d);
  for (int i = 0; i < n; ++i)
    for (int c = 0; c < half; ++c) {
      const double ang = (double)pos[i] * freq[c], cs = cos(ang), sn = sin(ang);
      for (int h = 0; h < H; ++h) {
        float *row = q + ((size_t)i * H + h) * d;
        const double a = row[c], b = row[c + half];
        row[c] = (float)(a * cs - b * sn);
        row[c + half] = (float)(b * cs + a * sn);
      }
    }
  return IG_OK;
}

// ---- speculation on the CPU with the partial key cache in host memory ---------------------------
// Section 6.2 "Memory Consumption" names this as a way to take the partial key cache off the GPU:
// the partial query is computed on the GPU as usual and fetched; scan, maximum, threshold and the
// index lists are worked out on the host, over a host copy of the partial key cache in the same
// tiled channel-plane layout the GPU scan reads (a slab built by ig_slab_build and copied to host
// memory is valid input).  The arithmetic is that of the GPU scan, in the same order: the query
// entry is scaled first, a token's score is accumulated channel by channel with fused
// multiply-adds in float32, so for the same partial query the scores and the lists are the same
// bit for bit.  (sequence, head) pairs are spread over host threads.
#include <thread>

namespace {

inline float half_bits_to_float(uint16_t h) {
  const uint32_t sign = (uint32_t)(h & 0x8000u) << 16;
  uint32_t exp = (h >> 10) & 0x1fu, man = h & 0x3ffu;
  uint32_t bits;
  if (exp == 0) {
    if (man == 0) {
      bits = sign;
    } else {                                  // subnormal half: normalise
      int e = -1;
      do { ++e; man <<= 1; } while (!(man & 0x400u));
      bits = sign | ((uint32_t)(127 - 15 - e) << 23) | ((man & 0x3ffu) << 13);
    }
  } else if (exp == 31) {
    bits = sign | 0x7f800000u | (man << 13);
  } else {
    bits = sign | ((exp + 127 - 15) << 23) | (man << 13);
  }
  float f;
  memcpy(&f, &bits, 4);
  return f;
}

// scores of tokens [t0, t1) of one (b,h): s[t] = sum_j float(K[t, j]) * (q_p[j] * scale), in channel
// order with fused multiply-adds
template <typename E>
void scan_range(const E *pair, int t0, int t1, int tile, int r, const float *qs, float *s) {
  for (int t = t0; t < t1; ++t) {
    const E *col = pair + (size_t)(t / tile) * r * tile + t % tile;
    float acc = 0.f;
    for (int j = 0; j < r; ++j) {
      float k;
      if (sizeof(E) == 2) k = half_bits_to_float((uint16_t)col[(size_t)j * tile]);
      else memcpy(&k, &col[(size_t)j * tile], 4);
      acc = fmaf(k, qs[j], acc);
    }
    s[t] = acc;
  }
}

#if defined(__x86_64__)
#include <immintrin.h>
// the same sums for n64 whole groups of 64 tokens (F16C conversion, FMA; 64 tokens stay in 8
// registers over all channels): identical results, lane by lane
__attribute__((target("avx2,f16c,fma")))
void scan_groups_f16_avx2(const uint16_t *pair, int n64, int tile, int r, const float *qs, float *s) {
  for (int g = 0; g < n64; ++g) {
    const int t0 = g * 64;
    const uint16_t *base = pair + (size_t)(t0 / tile) * r * tile + t0 % tile;
    __m256 acc[8];
    for (int u = 0; u < 8; ++u) acc[u] = _mm256_setzero_ps();
    for (int j = 0; j < r; ++j) {
      const uint16_t *p = base + (size_t)j * tile;
      const __m256 q = _mm256_set1_ps(qs[j]);
      for (int u = 0; u < 8; ++u)
        acc[u] = _mm256_fmadd_ps(_mm256_cvtph_ps(_mm_loadu_si128((const __m128i *)(p + 8 * u))), q, acc[u]);
    }
    for (int u = 0; u < 8; ++u) _mm256_storeu_ps(s + t0 + 8 * u, acc[u]);
  }
}
#endif

}  // namespace

extern "C" int ig_speculate_host(ig_ctx *ctx, const ig_desc *d, const float *q_p, const void *slab_host,
                                 int32_t *sel_idx, int32_t sel_stride, int32_t *sel_cnt,
                                 float *scores_opt, int threads) {
  if (!d) return ig_fail(ctx, IG_EINVAL, "descriptor is NULL");
  if (d->dtype != IG_F32 && d->dtype != IG_F16) return ig_fail(ctx, IG_EDTYPE, "unknown dtype %d", d->dtype);
  if (d->B < 1 || d->H < 1 || d->r < 1 || d->N < 1 || d->N_cap < d->N)
    return ig_fail(ctx, IG_ESHAPE, "ig_speculate_host: bad shape");
  if (!(d->alpha >= 0.0f)) return ig_fail(ctx, IG_EINVAL, "alpha must be >= 0");
  if (!q_p || !slab_host || !sel_idx || !sel_cnt) return ig_fail(ctx, IG_EINVAL, "ig_speculate_host: NULL argument");
  if (sel_stride < 1) return ig_fail(ctx, IG_ESHAPE, "sel_stride = %d", sel_stride);
  const int tile = d->dtype == IG_F16 ? 512 : 256;
  const int nTiles = (d->N_cap + tile - 1) / tile;
  const int BH = d->B * d->H, r = d->r, N = d->N;
  int nthreads = threads > 0 ? threads : (int)std::thread::hardware_concurrency();
  nthreads = std::max(1, std::min(nthreads, std::min(BH, 64)));
#if defined(__x86_64__)
  const bool simd = d->dtype == IG_F16 && __builtin_cpu_supports("avx2") && __builtin_cpu_supports("f16c") &&
                    __builtin_cpu_supports("fma");
#else
  const bool simd = false;
#endif
  std::vector<int> clamped(nthreads, 0);
  auto work = [&](int tid) {
    std::vector<float> s((size_t)N), qs(r);
    for (int bh = tid; bh < BH; bh += nthreads) {
      for (int j = 0; j < r; ++j) qs[j] = q_p[(size_t)bh * r + j] * d->scale;
      const size_t pair_off = (size_t)bh * nTiles * r * tile;
      if (d->dtype == IG_F16) {
        const uint16_t *pair = static_cast<const uint16_t *>(slab_host) + pair_off;
        int done = 0;                          // whole groups of 64 tokens go through the vector loop
#if defined(__x86_64__)
        if (simd) {
          scan_groups_f16_avx2(pair, N / 64, tile, r, qs.data(), s.data());
          done = N / 64 * 64;
        }
#endif
        scan_range<uint16_t>(pair, done, N, tile, r, qs.data(), s.data());
      } else {
        scan_range<uint32_t>(static_cast<const uint32_t *>(slab_host) + pair_off, 0, N, tile, r, qs.data(), s.data());
      }
      if (scores_opt) memcpy(scores_opt + (size_t)bh * N, s.data(), sizeof(float) * N);
      float m = -INFINITY;
      for (int t = 0; t < N; ++t) m = s[t] > m ? s[t] : m;
      const float thr = m - d->alpha;
      int n = 0;
      int32_t *list = sel_idx + (size_t)bh * sel_stride;
      for (int t = 0; t < N; ++t)
        if (s[t] >= thr) {
          if (n < sel_stride) list[n] = t;
          ++n;
        }
      if (n > sel_stride) clamped[tid] = 1;
      sel_cnt[bh] = std::min(n, (int)sel_stride);
    }
  };
  std::vector<std::thread> pool;
  for (int t = 1; t < nthreads; ++t) pool.emplace_back(work, t);
  work(0);
  for (auto &t : pool) t.join();
  for (int c : clamped)
    if (c) return ig_fail(ctx, IG_ECAPACITY, "a selected-token list was longer than sel_stride and was clamped");
  return IG_OK;
}
