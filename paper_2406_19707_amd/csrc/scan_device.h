// Device side of the partial key cache scan: argument block, the per-wave tile scan, the partial
// query (split-K sums), ordered compaction, and the body of the one-workgroup-per-(b,h) kernel.
// Shared by the scan kernels and by the kernel that runs a layer's scan next to the previous
// layer's attention in one launch.
#ifndef IG_SCAN_DEVICE_H
#define IG_SCAN_DEVICE_H
#include "ig_internal.h"

struct ScanArgs {
  const void *slab;
  const float *qsrc;
  const float *bias;
  int32_t *sel_idx;
  int32_t *sel_cnt;
  float *scores_out;   // optional dump (fused) / score buffer (tiled)
  float *tmax;         // tiled path: per-tile maxima
  int32_t *status;
  long ks_stride;
  long b_stride;
  int ks;
  int H, r, N;
  int nTiles;   // tiles allocated per (b,h): the slab's stride (from N_cap)
  int nValid;   // tiles that hold valid tokens (from N): the only ones read
  int sel_stride;
  float scale, alpha;
};

namespace {


// Partial query of (b,h), kept in registers: lane l of every scanning wave holds q[l + 64*k], k < 4
// (r <= 256), scaled.  value(j) = scale * (bias[h*r+j] + sum_s qsrc[s*ks_stride + b*b_stride + h*r + j]).
// The loads are issued by query_issue() BEFORE the wave's slab loads, so they sit at the head of
// the memory queue and return early; query_finish() adds them in a fixed order.  During the scan a
// channel's query entry is broadcast with v_readlane, so the inner loop touches neither LDS nor a
// barrier.
struct QueryLoads {
  float part[IG_KS_MAX];   // split-K partial sums of channel `lane` (r <= 64 needs only these)
  float bias;
  bool live;               // the lane's channel exists (lane + 64*k < r)
};
__device__ __forceinline__ void query_issue(const ScanArgs &a, int b, int h, int lane, int k, QueryLoads &ql) {
  // straight-line code, every load unconditional (channel and split clamped, surplus values dropped
  // in query_finish): the compiler then keeps exact counts of the loads outstanding, where a branch
  // around a load makes it wait for everything issued so far
  const int j = min(lane + 64 * k, a.r - 1);
  const float *p = a.qsrc + (long)b * a.b_stride + (long)h * a.r + j;
#pragma unroll
  for (int s = 0; s < IG_KS_MAX; ++s) ql.part[s] = p[(long)min(s, a.ks - 1) * a.ks_stride];
  ql.bias = a.bias ? a.bias[h * a.r + j] : 0.f;
  ql.live = lane + 64 * k < a.r;
}
__device__ __forceinline__ float query_finish(const ScanArgs &a, const QueryLoads &ql) {
  float acc = ql.bias;
#pragma unroll
  for (int s = 0; s < IG_KS_MAX; ++s) acc += s < a.ks ? ql.part[s] : 0.f;
  return ql.live ? acc * a.scale : 0.f;
}
// lane l (< CH) gets q[j0 + l] out of the four per-lane registers
__device__ __forceinline__ float query_block(const float (&qv)[4], int j0, int lane) {
  const int j = j0 + lane;
  const int src = j & 63, k = (j >> 6) & 3;
  const float t0 = __shfl(qv[0], src, 64), t1 = __shfl(qv[1], src, 64);
  const float t2 = __shfl(qv[2], src, 64), t3 = __shfl(qv[3], src, 64);
  const float t = k == 0 ? t0 : (k == 1 ? t1 : (k == 2 ? t2 : t3));
  return j < 256 ? t : 0.f;
}

template <typename T, int CH>
__device__ __forceinline__ void load_block(const T *tile, int r, int j0, int lane,
                                           typename SlabElem<T>::vec (&v)[CH]) {
  constexpr int TPL = SlabElem<T>::TPL;
  constexpr int TILE = IG_WAVE * TPL;
  const char *base = reinterpret_cast<const char *>(tile);
  const unsigned lane_off = (unsigned)lane * (unsigned)(TPL * sizeof(T));
#pragma unroll
  for (int j = 0; j < CH; ++j) {
    const int jj = min(j0 + j, r - 1);   // channels past r re-read the last plane; their query entry is 0
    const char *plane = base + (size_t)jj * (TILE * sizeof(T));
    v[j] = *reinterpret_cast<const typename SlabElem<T>::vec *>(plane + lane_off);
  }
}

// qblk: lane l holds the query entry of channel j0 + l (0 past r)
template <typename T, int CH>
__device__ __forceinline__ void fma_block(const typename SlabElem<T>::vec (&v)[CH], float qblk,
                                          float (&acc)[SlabElem<T>::TPL]) {
  constexpr int TPL = SlabElem<T>::TPL;
  const int qbits = __float_as_int(qblk);
#pragma unroll
  for (int j = 0; j < CH; ++j) {
    const float qj = __int_as_float(__builtin_amdgcn_readlane(qbits, j));
#pragma unroll
    for (int e = 0; e < TPL; ++e) acc[e] = fmaf((float)v[j][e], qj, acc[e]);
  }
}

// All channels of one tile for one wave: query loads, slab loads, then FMAs as the data arrives.
template <typename T, int CH>
__device__ __forceinline__ void scan_tile(const ScanArgs &a, const T *tile, int b, int h, int lane,
                                          float (&acc)[SlabElem<T>::TPL]) {
  constexpr int TPL = SlabElem<T>::TPL;
  typename SlabElem<T>::vec v[CH];
#pragma unroll
  for (int e = 0; e < TPL; ++e) acc[e] = 0.f;
  QueryLoads ql;
  query_issue(a, b, h, lane, 0, ql);
  load_block<T, CH>(tile, a.r, 0, lane, v);
  float qv[4];
  qv[0] = query_finish(a, ql);
  qv[1] = qv[2] = qv[3] = 0.f;
  if (a.r <= CH) {           // the usual case: one block, lane l already holds channel l
    fma_block<T, CH>(v, qv[0], acc);
    return;
  }
  if (a.r > 64) {            // wide heads: three more registers per lane
    for (int k = 1; k < 4; ++k) {
      query_issue(a, b, h, lane, k, ql);
      qv[k] = query_finish(a, ql);
    }
  }
  fma_block<T, CH>(v, query_block(qv, 0, lane), acc);
  for (int j0 = CH; j0 < a.r; j0 += CH) {
    load_block<T, CH>(tile, a.r, j0, lane, v);
    fma_block<T, CH>(v, query_block(qv, j0, lane), acc);
  }
}

// The same with the query already in registers (qv[k]: scaled entry of channel lane + 64*k) and
// the first channel block already loaded into v.
template <typename T, int CH>
__device__ __forceinline__ void scan_tile_given_q(const ScanArgs &a, const T *tile, int lane,
                                                  typename SlabElem<T>::vec (&v)[CH], const float (&qv)[4],
                                                  float (&acc)[SlabElem<T>::TPL]) {
  if (a.r <= CH) {
    fma_block<T, CH>(v, qv[0], acc);
    return;
  }
  fma_block<T, CH>(v, query_block(qv, 0, lane), acc);
  for (int j0 = CH; j0 < a.r; j0 += CH) {
    load_block<T, CH>(tile, a.r, j0, lane, v);
    fma_block<T, CH>(v, query_block(qv, j0, lane), acc);
  }
}

// A lane's TPL consecutive scores go out as 16-byte stores when the run is whole and aligned.
template <int TPL>
__device__ __forceinline__ void store_scores(float *dst /* score of token 0 of the head */, long head_off,
                                             int t, int N, const float (&acc)[TPL]) {
  float *p = dst + head_off + t;
  if (t + TPL <= N && ((head_off + t) & 3) == 0) {
#pragma unroll
    for (int e = 0; e < TPL; e += 4) {
      floatx4 v = {acc[e], acc[e + 1], acc[e + 2], acc[e + 3]};
      *reinterpret_cast<floatx4 *>(p + e) = v;
    }
  } else {
#pragma unroll
    for (int e = 0; e < TPL; ++e)
      if (t + e < N) p[e] = acc[e];
  }
}

// Threshold + ordered compaction of the scores a block holds in registers.  Wave w (< NW) holds
// the scores of tokens t0 + lane*TPL + e (e < TPL); waves are in ascending token order; waves
// with w >= NW hold nothing.  `base` is the number of tokens already emitted for this (b,h).
// The slot of (lane, e) is the number of kept tokens in lower lanes -- one ballot and one
// masked bit count per e -- plus the kept tokens of the lane's own lower e.  Returns the block's total.
template <int TPL, int NW>
__device__ __forceinline__ int compact_block(const float (&sc)[TPL], int t0, int N, float thr,
                                             int base, int32_t *list, int sel_stride, int *lds_cnt,
                                             int w, int lane) {
  unsigned mask = 0;
  int below = 0, total = 0;
#pragma unroll
  for (int e = 0; e < TPL; ++e) {
    const int t = t0 + lane * TPL + e;
    const bool keep = w < NW && t < N && sc[e] >= thr;
    const unsigned long long bal = __ballot(keep);
    below += lanes_below(bal);
    total += __popcll(bal);
    mask |= (keep ? 1u : 0u) << e;
  }
  if (lane == 0 && w < NW) lds_cnt[w] = total;
  __syncthreads();
  int before = 0, all = 0;
#pragma unroll
  for (int k = 0; k < NW; ++k) {
    int c = lds_cnt[k];
    before += (k < w) ? c : 0;
    all += c;
  }
  int pos = base + before + below;
#pragma unroll
  for (int e = 0; e < TPL; ++e) {
    if (mask & (1u << e)) {
      if (pos < sel_stride) list[pos] = t0 + lane * TPL + e;
      ++pos;
    }
  }
  __syncthreads();   // lds_cnt may be reused by the caller
  return all;
}

// One workgroup per (b,h); wave w scans tile w (nValid <= NW) and keeps its scores in registers.
template <typename T, int CH, int NW>
__device__ __forceinline__ void scan_select_fused_body(const ScanArgs &a, const int bh) {
  constexpr int TPL = SlabElem<T>::TPL;
  constexpr int TILE = IG_WAVE * TPL;
  __shared__ float lds_max[NW];
  __shared__ int lds_cnt[NW];
  const int b = bh / a.H, h = bh % a.H;
  // the wave index is made a scalar so that tile addresses stay in scalar registers
  const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const bool active = w < a.nValid;
  const T *tile = static_cast<const T *>(a.slab) + ((long)bh * a.nTiles + (active ? w : 0)) * a.r * TILE;
  float acc[TPL];
#pragma unroll
  for (int e = 0; e < TPL; ++e) acc[e] = 0.f;
  if (active) scan_tile<T, CH>(a, tile, b, h, lane, acc);
  const int t0 = w * TILE;
  float m = -INFINITY;
#pragma unroll
  for (int e = 0; e < TPL; ++e) {
    int t = t0 + lane * TPL + e;
    if (!active || t >= a.N) acc[e] = -INFINITY;
    m = fmaxf(m, acc[e]);
  }
  if (a.scores_out && active) store_scores<TPL>(a.scores_out, (long)bh * a.N, t0 + lane * TPL, a.N, acc);
  m = wave_max(m);
  if (lane == 0) lds_max[w] = m;
  __syncthreads();
  float mm = lds_max[0];
#pragma unroll
  for (int k = 1; k < NW; ++k) mm = fmaxf(mm, lds_max[k]);
  const float thr = mm - a.alpha;
  int all = compact_block<TPL, NW>(acc, t0, a.N, thr, 0, a.sel_idx + (long)bh * a.sel_stride,
                                   a.sel_stride, lds_cnt, w, lane);
  if (threadIdx.x == 0) {
    a.sel_cnt[bh] = min(all, a.sel_stride);
    if (all > a.sel_stride) atomicOr(a.status, IG_STATUS_CAPACITY);
  }
}

}  // namespace

// fills the argument block from the descriptor and the query source (validates shapes)
int ig_scan_args(ig_ctx *ctx, const ig_desc *d, const QSource &q, const void *slab, int32_t *sel_idx,
                 int32_t sel_stride, int32_t *sel_cnt, float *scores_opt, ScanArgs *a);
int ig_pick_ch(int r, int cap);

#endif
