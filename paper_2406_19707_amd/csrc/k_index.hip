// Partial weight index generation on the GPU (Section 4.3 "Prefill Stage"): per head, the
// r = floor(ratio*d) columns with the largest sum over the prompt's rows of |Q~| + |K~|.
//
// Two kernels, both with a fixed summation order (no floating-point atomics, so a run repeats
// bit for bit):
//   column_abs_sums   a workgroup takes 256 consecutive columns and one of ROW_CHUNKS row ranges;
//                     thread c walks its column down the range (a wave reads 64 consecutive
//                     elements of a row: coalesced) and writes one partial sum
//   top_columns       one workgroup per head: adds the ROW_CHUNKS partial sums of each column in
//                     order, ranks the d columns (column j beats c when its sum is larger, or
//                     equal with j < c), keeps ranks < r and writes them in ascending order
#include "ig_internal.h"

namespace {

constexpr int ROW_CHUNKS = 32;

template <typename T>
__global__ __launch_bounds__(256) void column_abs_sums(const T *__restrict__ Qs, const T *__restrict__ Ks,
                                                       float *__restrict__ part, int n, int D) {
  const int c = blockIdx.x * 256 + threadIdx.x;
  const int chunk = blockIdx.y;
  const int rows_per = (n + ROW_CHUNKS - 1) / ROW_CHUNKS;
  const int i0 = chunk * rows_per, i1 = min(n, i0 + rows_per);
  if (c >= D) return;
  float acc = 0.f;
  for (int i = i0; i < i1; ++i) {
    acc += fabsf((float)Qs[(long)i * D + c]);
    if (Ks) acc += fabsf((float)Ks[(long)i * D + c]);
  }
  part[(long)chunk * D + c] = acc;
}

__global__ __launch_bounds__(256) void top_columns(const float *__restrict__ part, int32_t *__restrict__ idx,
                                                   int d, int D, int r) {
  __shared__ float sum[256];
  __shared__ int keep[256];
  __shared__ int wave_tot[4];
  const int h = blockIdx.x, c = threadIdx.x, lane = c & 63, w = c >> 6;
  float v = -1.f;                       // sums are >= 0: unused lanes never win
  if (c < d) {
    v = 0.f;
    for (int k = 0; k < ROW_CHUNKS; ++k) v += part[(long)k * D + h * d + c];
  }
  sum[c] = v;
  __syncthreads();
  int rank = 0;
  if (c < d)
    for (int j = 0; j < d; ++j) rank += (sum[j] > v) || (sum[j] == v && j < c);
  const bool kept = c < d && rank < r;
  keep[c] = kept;
  const unsigned long long bal = __ballot(kept);
  if (lane == 0) wave_tot[w] = __popcll(bal);
  __syncthreads();
  int pos = lanes_below(bal);
  for (int k = 0; k < w; ++k) pos += wave_tot[k];
  if (kept) idx[h * r + pos] = c;
}

}  // namespace

int ig_launch_partial_index(ig_ctx *ctx, int dtype, int H, int d, int n, const void *Qs, const void *Ks,
                            int r, float *part, int32_t *idx, hipStream_t s) {
  const int D = H * d;
  dim3 grid((D + 255) / 256, ROW_CHUNKS), block(256);
  if (dtype == IG_F16) {
    auto k = column_abs_sums<half_t>;
    IG_LAUNCH(ctx, IG_K_BUILD, k, grid, block, s, (const half_t *)Qs, (const half_t *)Ks, part, n, D);
  } else {
    auto k = column_abs_sums<float>;
    IG_LAUNCH(ctx, IG_K_BUILD, k, grid, block, s, (const float *)Qs, (const float *)Ks, part, n, D);
  }
  auto k2 = top_columns;
  IG_LAUNCH(ctx, IG_K_BUILD, k2, dim3(H), dim3(256), s, (const float *)part, idx, d, D, r);
  return IG_OK;
}

size_t ig_partial_index_workspace(int H, int d) { return (size_t)ROW_CHUNKS * H * d * sizeof(float); }
