// Offline skewing on the GPU (Section 4.2 "Skewed Partial Weight", Eq. 2 and Eq. 3; Section 4.3
// "Prefetching Scheme"): per head, A_h = V of the SVD Q_h = U S V^T of the calibration queries.
//
// As in the host version, V is obtained from the Gram matrix: Q_h^T Q_h = V S^2 V^T.
//   gram_heads     G_h = Q_h^T Q_h in double, one thread per entry of the upper triangle
//   jacobi_heads   one workgroup per head: cyclic two-sided Jacobi with a round-robin (tournament)
//                  ordering, so that the d/2 rotations of a round act on disjoint index pairs and
//                  run in parallel: rotations are computed from the current G, then applied to
//                  the columns of G and V, then to the rows of G, with a barrier after each phase.
//                  The number of sweeps is fixed (no data-dependent loop); what is left off the
//                  diagonal afterwards is checked and flagged.  Eigenvalues are then ranked in
//                  descending order (the earlier column first on ties), each eigenvector's sign is
//                  chosen so that its largest-magnitude entry is positive, and A_h (float32) and
//                  the singular values sqrt(lambda) are written.
// G and V live in a double-precision workspace in device memory (128 KiB each per head at d = 128:
// they stay in L2); all arithmetic is double.
#include "ig_internal.h"

namespace {

constexpr int JACOBI_SWEEPS = 16;

__global__ __launch_bounds__(256) void gram_heads(const float *__restrict__ Qcal, double *__restrict__ G,
                                                  int n, int D, int d) {
  const int h = blockIdx.y;
  const int e = blockIdx.x * 256 + threadIdx.x;
  if (e >= d * d) return;
  const int a = e / d, b = e % d;
  if (b < a) return;
  const float *col = Qcal + (long)h * d;
  double acc = 0.0;
  for (int i = 0; i < n; ++i) acc += (double)col[(long)i * D + a] * (double)col[(long)i * D + b];
  G[((long)h * d + a) * d + b] = acc;
  G[((long)h * d + b) * d + a] = acc;
}

__global__ __launch_bounds__(256) void jacobi_heads(double *__restrict__ Gall, double *__restrict__ Vall,
                                                    float *__restrict__ A, float *__restrict__ sigma,
                                                    int32_t *status, int d) {
  extern __shared__ double rot[];            // c[half], s[half], then int p[half], q[half]
  __shared__ double lam[256];
  __shared__ double s_off, s_diag;
  const int h = blockIdx.x, tid = threadIdx.x;
  const int half = d / 2, m = d - 1;
  double *cc = rot, *ss = rot + half;
  int *pp = reinterpret_cast<int *>(rot + 2 * half), *qq = pp + half;
  double *G = Gall + (long)h * d * d, *V = Vall + (long)h * d * d;
  for (int e = tid; e < d * d; e += 256) V[e] = (e / d == e % d) ? 1.0 : 0.0;
  __syncthreads();
  for (int sweep = 0; sweep < JACOBI_SWEEPS; ++sweep) {
    for (int r = 0; r < m; ++r) {
      // round r of the tournament: pair 0 is (r, d-1), pair k is ((r+k) mod m, (r-k) mod m)
      for (int k = tid; k < half; k += 256) {
        int p = k == 0 ? r : (r + k) % m;
        int q = k == 0 ? d - 1 : (r - k + m) % m;
        if (p > q) { const int t = p; p = q; q = t; }
        const double gpq = G[(long)p * d + q], gpp = G[(long)p * d + p], gqq = G[(long)q * d + q];
        double c = 1.0, s = 0.0;
        if (gpq != 0.0 && fabs(gpq) > 1e-17 * sqrt(fabs(gpp * gqq))) {
          const double theta = (gqq - gpp) / (2.0 * gpq);
          const double t = (theta >= 0 ? 1.0 : -1.0) / (fabs(theta) + sqrt(theta * theta + 1.0));
          c = 1.0 / sqrt(t * t + 1.0);
          s = t * c;
        }
        cc[k] = c; ss[k] = s; pp[k] = p; qq[k] = q;
      }
      __syncthreads();
      // columns p, q of G and V (consecutive threads: the pairs of one row)
      for (int item = tid; item < half * d; item += 256) {
        const int i = item / half, k = item % half;
        const int p = pp[k], q = qq[k];
        const double c = cc[k], s = ss[k];
        double a = G[(long)i * d + p], b = G[(long)i * d + q];
        G[(long)i * d + p] = c * a - s * b;
        G[(long)i * d + q] = s * a + c * b;
        a = V[(long)i * d + p]; b = V[(long)i * d + q];
        V[(long)i * d + p] = c * a - s * b;
        V[(long)i * d + q] = s * a + c * b;
      }
      __syncthreads();
      // rows p, q of G (consecutive threads: consecutive columns)
      for (int item = tid; item < half * d; item += 256) {
        const int k = item / d, j = item % d;
        const int p = pp[k], q = qq[k];
        const double c = cc[k], s = ss[k];
        const double a = G[(long)p * d + j], b = G[(long)q * d + j];
        G[(long)p * d + j] = c * a - s * b;
        G[(long)q * d + j] = s * a + c * b;
      }
      __syncthreads();
    }
  }
  // what is left off the diagonal, against the largest eigenvalue
  if (tid == 0) { s_off = 0.0; s_diag = 0.0; }
  __syncthreads();
  {
    double off = 0.0, dg = 0.0;
    for (int e = tid; e < d * d; e += 256) {
      const double v = fabs(G[e]);
      if (e / d == e % d) dg = fmax(dg, v); else off = fmax(off, v);
    }
    // maxima of non-negative doubles: their bit patterns order like unsigned integers
    atomicMax(reinterpret_cast<unsigned long long *>(&s_off), (unsigned long long)__double_as_longlong(off));
    atomicMax(reinterpret_cast<unsigned long long *>(&s_diag), (unsigned long long)__double_as_longlong(dg));
  }
  __syncthreads();
  if (tid == 0 && s_off > 1e-9 * s_diag) atomicOr(status, IG_STATUS_NOCONV);
  // rank the eigenvalues (descending, the earlier column first on ties), fix signs, write out
  if (tid < d) lam[tid] = G[(long)tid * d + tid];
  __syncthreads();
  for (int j = tid; j < d; j += 256) {
    const double lj = lam[j];
    int rank = 0;
    for (int i = 0; i < d; ++i) rank += (lam[i] > lj) || (lam[i] == lj && i < j);
    int arg = 0;
    for (int i = 1; i < d; ++i)
      if (fabs(V[(long)i * d + j]) > fabs(V[(long)arg * d + j])) arg = i;
    const double sgn = V[(long)arg * d + j] < 0 ? -1.0 : 1.0;
    float *Ah = A + (long)h * d * d;
    for (int i = 0; i < d; ++i) Ah[(long)i * d + rank] = (float)(sgn * V[(long)i * d + j]);
    if (sigma) sigma[(long)h * d + rank] = (float)sqrt(fmax(0.0, lj));
  }
}

}  // namespace

size_t ig_skew_workspace(int H, int d) { return (size_t)2 * H * d * d * sizeof(double); }

int ig_launch_skew(ig_ctx *ctx, int D, int H, int n_cal, const float *Qcal, double *ws, float *A,
                   float *sigma, hipStream_t s) {
  const int d = D / H;
  double *G = ws, *V = ws + (size_t)H * d * d;
  auto k1 = gram_heads;
  IG_LAUNCH(ctx, IG_K_BUILD, k1, dim3((d * d + 255) / 256, H), dim3(256), s, Qcal, G, n_cal, D, d);
  auto k2 = jacobi_heads;
  const size_t lds = (size_t)(d / 2) * (2 * sizeof(double) + 2 * sizeof(int));
  if (ctx->profiling) {
    hipEvent_t e0, e1;
    ig_prof_events(ctx, IG_K_BUILD, &e0, &e1);
    hipExtLaunchKernelGGL(k2, dim3(H), dim3(256), (unsigned)lds, s, e0, e1, 0, G, V, A, sigma, ctx->status, d);
  } else {
    hipLaunchKernelGGL(k2, dim3(H), dim3(256), (unsigned)lds, s, G, V, A, sigma, ctx->status, d);
  }
  hipError_t le = hipGetLastError();
  if (le != hipSuccess) return ig_hip_fail(ctx, le, "jacobi_heads");
  return IG_OK;
}
