// Partial key cache scan, per-head maximum, (max - alpha) threshold and compaction
// (Section 4.3 "Decoding Stage": speculated score = partial query x partial key cache; tokens whose
// score reaches the maximum minus alpha are kept).
//
// Layout the scan relies on (written by ig_slab_build): per (sequence, head) the tokens are cut
// into tiles of 64 x TPL tokens (TPL = 8 halves or 4 floats = 16 bytes per lane); inside a tile the
// r kept channels are planes of TILE contiguous tokens.  A wave owns one tile: for every channel it
// issues one fully coalesced 1 KiB load (lane l gets tokens l*TPL .. l*TPL+TPL-1 of that channel)
// and multiplies by the wave-uniform partial query entry, so a token's score is accumulated in
// one lane without any cross-lane reduction.  The kernel is HBM-bound (1 FMA per 2 bytes).
//
// The partial query comes from the projection's split-K partial sums, added here in a fixed order
// (no separate reduction kernel); for rotary models on the fused path the workgroup also applies
// the rotation and the partial skew itself (rope_query) while its first slab loads are in flight.
#include "scan_device.h"

namespace {

// One workgroup per (b,h); wave w scans tile w (nValid <= NW) and keeps its scores in registers.
template <typename T, int CH, int NW, bool ROPE>
__global__ __launch_bounds__(NW * 64) void scan_select_fused(ScanArgs a) {
  scan_select_fused_body<T, CH, NW, ROPE>(a, blockIdx.x);
}

// Sequences of up to LDS_SCORES tokens that do not fit 16 waves at once: still one workgroup of
// 16 waves per (b,h); wave w scans tiles w, w + 16, ... and parks the scores in LDS (4 B/token,
// 128 KiB), so that the threshold pass needs neither a score buffer in memory nor further
// kernels.  The waves run through their tiles without meeting; they meet once for the maximum.
constexpr int LDS_SCORES = 32768;

template <typename T, int CH, bool ROPE>
__global__ __launch_bounds__(1024) void scan_select_lds(ScanArgs a) {
  constexpr int TPL = SlabElem<T>::TPL;
  constexpr int TILE = IG_WAVE * TPL;
  constexpr int NW = 16;
  __shared__ float lds_s[LDS_SCORES];
  __shared__ float lds_max[NW];
  __shared__ int lds_cnt[NW];
  const int bh = blockIdx.x, b = bh / a.H, h = bh % a.H;
  const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const T *head = static_cast<const T *>(a.slab) + (long)bh * a.nTiles * a.r * TILE;
  typename SlabElem<T>::vec v[CH];
  // first channel block of the wave's first tile in flight while the partial query is worked out
  if (w < a.nValid) load_block<T, CH>(head + (long)w * a.r * TILE, a.r, 0, lane, v);
  float qv[4];
  if constexpr (ROPE) {
    __shared__ float q_lds[512], qr_lds[512], psum[NW * 64], qp_lds[256];
    rope_query<NW * 64>(a, b, h, q_lds, qr_lds, psum, qp_lds);
#pragma unroll
    for (int k = 0; k < 4; ++k) qv[k] = (lane + 64 * k < a.r) ? qp_lds[lane + 64 * k] * a.scale : 0.f;
  } else {
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      qv[k] = 0.f;
      if (64 * k < a.r) {
        QueryLoads ql;
        query_issue(a, b, h, lane, k, ql);
        qv[k] = query_finish(a, ql);
      }
    }
  }
  float m = -INFINITY;
  for (int ti = w; ti < a.nValid; ti += NW) {
    const T *tile = head + (long)ti * a.r * TILE;
    if (ti != w) load_block<T, CH>(tile, a.r, 0, lane, v);
    float acc[TPL];
#pragma unroll
    for (int e = 0; e < TPL; ++e) acc[e] = 0.f;
    scan_tile_given_q<T, CH>(a, tile, lane, v, qv, acc);
    const int t0 = ti * TILE;
    if (a.scores_out) store_scores<TPL>(a.scores_out, (long)bh * a.N, t0 + lane * TPL, a.N, acc);
#pragma unroll
    for (int e = 0; e < TPL; ++e) {
      if (t0 + lane * TPL + e >= a.N) acc[e] = -INFINITY;
      m = fmaxf(m, acc[e]);
    }
#pragma unroll
    for (int e = 0; e < TPL; e += 4) {
      const floatx4 o = {acc[e], acc[e + 1], acc[e + 2], acc[e + 3]};
      *reinterpret_cast<floatx4 *>(lds_s + t0 + lane * TPL + e) = o;
    }
  }
  m = wave_max(m);
  if (lane == 0) lds_max[w] = m;
  __syncthreads();
  float mm = lds_max[0];
#pragma unroll
  for (int k = 1; k < NW; ++k) mm = fmaxf(mm, lds_max[k]);
  const float thr = mm - a.alpha;
  int base = 0;
  for (int t0w = 0; t0w < a.nValid; t0w += NW) {       // 16 tiles per pass, in token order
    const int ti = t0w + w;
    float acc[TPL];
#pragma unroll
    for (int e = 0; e < TPL; e += 4) {
      floatx4 o = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
      if (ti < a.nValid) o = *reinterpret_cast<const floatx4 *>(lds_s + ti * TILE + lane * TPL + e);
#pragma unroll
      for (int k = 0; k < 4; ++k) acc[e + k] = o[k];
    }
    base += compact_block<TPL, NW>(acc, ti * TILE, a.N, thr, base, a.sel_idx + (long)bh * a.sel_stride,
                                   a.sel_stride, lds_cnt, w, lane);
  }
  if (threadIdx.x == 0) {
    a.sel_cnt[bh] = min(base, a.sel_stride);
    if (base > a.sel_stride) atomicOr(a.status, IG_STATUS_CAPACITY);
  }
}

// Long sequences / few heads: one wave per tile, 4 tiles per workgroup; scores and per-tile maxima
// go to a buffer, and select_count / select_write do the threshold pass.
template <typename T, int CH>
__global__ __launch_bounds__(256) void scan_tiles(ScanArgs a) {
  constexpr int TPL = SlabElem<T>::TPL;
  constexpr int TILE = IG_WAVE * TPL;
  const int bh = blockIdx.y, b = bh / a.H, h = bh % a.H;
  const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int tileno = blockIdx.x * 4 + w;
  if (tileno >= a.nValid) return;
  const T *tile = static_cast<const T *>(a.slab) + ((long)bh * a.nTiles + tileno) * a.r * TILE;
  float acc[TPL];
  scan_tile<T, CH>(a, tile, b, h, lane, acc);
  const int t0 = tileno * TILE;
  store_scores<TPL>(a.scores_out, (long)bh * a.N, t0 + lane * TPL, a.N, acc);
  float m = -INFINITY;
#pragma unroll
  for (int e = 0; e < TPL; ++e)
    if (t0 + lane * TPL + e < a.N) m = fmaxf(m, acc[e]);
  m = wave_max(m);
  if (lane == 0) a.tmax[(long)bh * a.nTiles + tileno] = m;
}

// Threshold + compaction from the score buffer, for sequences too long for one workgroup.  The
// tokens of a (b,h) are cut into parts of SELECT_PART tokens, one workgroup of 16 waves each, so
// that a long sequence is spread over many compute units.  select_count computes the threshold
// from the per-tile maxima and counts the kept tokens of each part; select_write adds up the
// counts of the preceding parts (a handful of values) and writes its part of the ascending list.
constexpr int SELECT_PART = 4096;   // 1024 threads x 4 tokens

__device__ __forceinline__ float select_threshold(const ScanArgs &a, int bh, float *lds_max, int w, int lane) {
  float m = -INFINITY;
  for (int k = threadIdx.x; k < a.nValid; k += 1024) m = fmaxf(m, a.tmax[(long)bh * a.nTiles + k]);
  m = wave_max(m);
  if (lane == 0) lds_max[w] = m;
  __syncthreads();
  float mm = lds_max[0];
#pragma unroll
  for (int k = 1; k < 16; ++k) mm = fmaxf(mm, lds_max[k]);
  return mm - a.alpha;
}

__device__ __forceinline__ void select_load(const ScanArgs &a, int bh, int t0, int lane, float (&sc)[4]) {
  const float *s = a.scores_out + (long)bh * a.N;
  const int t = t0 + lane * 4;
  if (t + 3 < a.N && (((long)bh * a.N + t) & 3) == 0) {
    const floatx4 v = *reinterpret_cast<const floatx4 *>(s + t);
#pragma unroll
    for (int e = 0; e < 4; ++e) sc[e] = v[e];
  } else {
#pragma unroll
    for (int e = 0; e < 4; ++e) sc[e] = (t + e < a.N) ? s[t + e] : -INFINITY;
  }
}

__global__ __launch_bounds__(1024) void select_count(ScanArgs a, int32_t *pcount, int nParts) {
  __shared__ float lds_max[16];
  __shared__ int lds_cnt[16];
  const int part = blockIdx.x, bh = blockIdx.y;
  const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int t0 = part * SELECT_PART + w * 256;
  float sc[4];
  select_load(a, bh, t0, lane, sc);
  const float thr = select_threshold(a, bh, lds_max, w, lane);
  int total = 0;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const int t = t0 + lane * 4 + e;
    total += __popcll(__ballot(t < a.N && sc[e] >= thr));
  }
  if (lane == 0) lds_cnt[w] = total;
  __syncthreads();
  if (threadIdx.x == 0) {
    int all = 0;
#pragma unroll
    for (int k = 0; k < 16; ++k) all += lds_cnt[k];
    pcount[(long)bh * nParts + part] = all;
  }
}

__global__ __launch_bounds__(1024) void select_write(ScanArgs a, const int32_t *pcount, int nParts) {
  __shared__ float lds_max[16];
  __shared__ int lds_cnt[16];
  const int part = blockIdx.x, bh = blockIdx.y;
  const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int t0 = part * SELECT_PART + w * 256;
  float sc[4];
  select_load(a, bh, t0, lane, sc);
  int base = 0;
  for (int p = lane; p < part; p += 64) base += pcount[(long)bh * nParts + p];
  base = wave_sum(base);
  const float thr = select_threshold(a, bh, lds_max, w, lane);
  const int mine = compact_block<4, 16>(sc, t0, a.N, thr, base, a.sel_idx + (long)bh * a.sel_stride,
                                        a.sel_stride, lds_cnt, w, lane);
  if (part == nParts - 1 && threadIdx.x == 0) {
    const int all = base + mine;
    a.sel_cnt[bh] = min(all, a.sel_stride);
    if (all > a.sel_stride) atomicOr(a.status, IG_STATUS_CAPACITY);
  }
}

// channel block size: the smallest multiple of 4 (<= 40) whose multiples cover r with least waste
int pick_ch(int r, int cap) {
  return ig_pick_ch(r, cap);
}

}  // namespace

int ig_pick_ch(int r, int cap) {
  int best = 4, best_waste = 1 << 30;
  for (int ch = cap; ch >= 4; ch -= 4) {
    int blocks = (r + ch - 1) / ch;
    int waste = blocks * ch - r + (blocks - 1) * 2;   // prefer fewer blocks on ties
    if (waste < best_waste) { best_waste = waste; best = ch; }
  }
  return best;
}

namespace {

template <typename T, int NW>
int launch_fused(ig_ctx *ctx, const ScanArgs &a, int BH, int ch, hipStream_t s) {
  dim3 grid(BH), block(NW * 64);
#define CASE(CHV)                                                              \
  case CHV: {                                                                  \
    if (a.A_p) {                                                               \
      auto k = scan_select_fused<T, CHV, NW, true>;                            \
      IG_LAUNCH(ctx, IG_K_SCAN, k, grid, block, s, a);                         \
    } else {                                                                   \
      auto k = scan_select_fused<T, CHV, NW, false>;                           \
      IG_LAUNCH(ctx, IG_K_SCAN, k, grid, block, s, a);                         \
    }                                                                          \
    return IG_OK;                                                              \
  }
  // registers per wave shrink as the workgroup grows: 4 waves allow 40 loads in flight, 8 waves 24,
  // 16 waves 12
  switch (ch) {
    CASE(4) CASE(8) CASE(12)
    default: break;
  }
  if constexpr (NW <= 8) {
    switch (ch) {
      CASE(16) CASE(20) CASE(24)
      default: break;
    }
  }
  if constexpr (NW <= 4) {
    switch (ch) {
      CASE(28) CASE(32) CASE(36) CASE(40)
      default: break;
    }
  }
#undef CASE
  return ig_fail(ctx, IG_ESHAPE, "scan: unsupported channel block %d", ch);
}

template <typename T>
int launch_lds(ig_ctx *ctx, const ScanArgs &a, int BH, int ch, hipStream_t s) {
  dim3 grid(BH), block(1024);
#define CASE(CHV)                                                              \
  case CHV: {                                                                  \
    if (a.A_p) {                                                               \
      auto k = scan_select_lds<T, CHV, true>;                                  \
      IG_LAUNCH(ctx, IG_K_SCAN, k, grid, block, s, a);                         \
    } else {                                                                   \
      auto k = scan_select_lds<T, CHV, false>;                                 \
      IG_LAUNCH(ctx, IG_K_SCAN, k, grid, block, s, a);                         \
    }                                                                          \
    return IG_OK;                                                              \
  }
  switch (ch) {
    CASE(4) CASE(8)
    default: break;
  }
#undef CASE
  return ig_fail(ctx, IG_ESHAPE, "scan: unsupported channel block %d", ch);
}

template <typename T>
int launch_tiles(ig_ctx *ctx, const ScanArgs &a, int BH, int ch, hipStream_t s) {
  dim3 grid((a.nValid + 3) / 4, BH), block(256);
#define CASE(CHV)                                                              \
  case CHV: {                                                                  \
    auto k = scan_tiles<T, CHV>;                                               \
    IG_LAUNCH(ctx, IG_K_SCAN, k, grid, block, s, a);                           \
    break;                                                                     \
  }
  switch (ch) {
    CASE(4) CASE(8) CASE(12) CASE(16) CASE(20) CASE(24) CASE(28) CASE(32) CASE(36) CASE(40)
    default: return ig_fail(ctx, IG_ESHAPE, "scan: unsupported channel block %d", ch);
  }
#undef CASE
  const int nParts = (a.N + SELECT_PART - 1) / SELECT_PART;
  int rc = ig_ensure(ctx, (void **)&ctx->pcount, &ctx->pcount_bytes, (size_t)BH * nParts * sizeof(int32_t));
  if (rc) return rc;
  auto k2 = select_count;
  IG_LAUNCH(ctx, IG_K_SELECT, k2, dim3(nParts, BH), dim3(1024), s, a, ctx->pcount, nParts);
  auto k3 = select_write;
  IG_LAUNCH(ctx, IG_K_SELECT, k3, dim3(nParts, BH), dim3(1024), s, a, (const int32_t *)ctx->pcount, nParts);
  return IG_OK;
}

template <typename T>
int launch_scan(ig_ctx *ctx, const ig_desc *d, ScanArgs &a, hipStream_t s) {
  const int BH = d->B * d->H;
  const int nTiles = a.nValid;     // the work, not the capacity, picks the kernel
  // One workgroup per (b,h) when it fits and there are enough (b,h) pairs to fill the chip;
  // otherwise one wave per tile so that long sequences spread over all compute units.
  const bool fused = ig_scan_is_fused(d);
  if (fused) {
    // When all workgroups fit on the chip at once (one round) a wave should have all its channels
    // in flight; with several rounds, smaller blocks leave room for more resident workgroups whose
    // load and select phases then overlap (measured: 60 % -> 71 % of HBM peak at 1120 workgroups).
    if (nTiles <= 4) return launch_fused<T, 4>(ctx, a, BH, pick_ch(d->r, BH > 512 ? 20 : 40), s);
    if (nTiles <= 8) return launch_fused<T, 8>(ctx, a, BH, pick_ch(d->r, 16), s);
    if (nTiles <= 16) return launch_fused<T, 16>(ctx, a, BH, pick_ch(d->r, 12), s);
    // 16 waves already keep a compute unit's memory queue full: 8 loads per wave in flight are
    // enough (4, 8 and 12 measured the same), and 12 would spill registers
    return launch_lds<T>(ctx, a, BH, pick_ch(d->r, 8), s);
  }
  size_t need_s = (size_t)BH * d->N * sizeof(float), need_m = (size_t)BH * a.nTiles * sizeof(float);
  float *user_scores = a.scores_out;
  if (!user_scores) {
    int rc = ig_ensure(ctx, (void **)&ctx->scores, &ctx->scores_bytes, need_s);
    if (rc) return rc;
    a.scores_out = ctx->scores;
  }
  int rc = ig_ensure(ctx, (void **)&ctx->tmax, &ctx->tmax_bytes, need_m);
  if (rc) return rc;
  a.tmax = ctx->tmax;
  // at most 28 channel loads in flight: 32 and more leave one wave per SIMD (measured with r = 38:
  // 30.8 us against 35.5 us at 80 pairs of 32768 tokens)
  return launch_tiles<T>(ctx, a, BH, pick_ch(d->r, 28), s);
}

}  // namespace

// One workgroup per (b,h) and a single kernel when a pair fits 16 waves (scores stay in registers)
// or 32768 tokens (scores parked in LDS) and there are enough pairs to fill the chip; otherwise
// one wave per tile and the threshold pass in two further kernels.
bool ig_scan_is_fused(const ig_desc *d) {
  const int tile = ig_tile_tokens(d->dtype);
  const int nTiles = (d->N + tile - 1) / tile;        // tiles with valid tokens
  const int BH = d->B * d->H;
  if (nTiles > 16) return nTiles * tile <= 32768 && BH >= 64;     // scores parked in LDS, one workgroup per pair
  return BH >= 128 || nTiles <= 4;
}

int ig_scan_args(ig_ctx *ctx, const ig_desc *d, const QSource &q, const void *slab, int32_t *sel_idx,
                 int32_t sel_stride, int32_t *sel_cnt, float *scores_opt, ScanArgs *out) {
  ScanArgs &a = *out;
  a.slab = slab;
  a.qsrc = q.qsrc;
  a.bias = q.bias;
  a.sel_idx = sel_idx;
  a.sel_cnt = sel_cnt;
  a.scores_out = scores_opt;
  a.tmax = nullptr;
  a.status = ctx->status;
  a.ks_stride = q.ks_stride;
  a.b_stride = q.b_stride;
  a.ks = q.ks;
  a.H = d->H;
  a.r = d->r;
  a.N = d->N;
  const int tile = ig_tile_tokens(d->dtype);
  a.nTiles = (d->N_cap + tile - 1) / tile;
  a.nValid = (d->N + tile - 1) / tile;
  a.sel_stride = sel_stride;
  a.scale = d->scale;
  a.alpha = d->alpha;
  a.A_p = q.A_p;
  a.pos = q.pos;
  a.d = d->d;
  a.theta = d->rope_theta;
  if (q.A_p && !ig_scan_is_fused(d)) return ig_fail(ctx, IG_EINVAL, "scan: rotary query source needs the fused path");
  if (q.A_p && d->d > 512) return ig_fail(ctx, IG_ESHAPE, "rope: d = %d exceeds 512", d->d);
  if (d->r > 256) return ig_fail(ctx, IG_ESHAPE, "r = %d exceeds 256", d->r);
  if (q.ks < 1 || q.ks > IG_KS_MAX) return ig_fail(ctx, IG_ESHAPE, "split-K %d out of range", q.ks);
  return IG_OK;
}

int ig_launch_scan_select(ig_ctx *ctx, const ig_desc *d, const QSource &q, const void *slab,
                          int32_t *sel_idx, int32_t sel_stride, int32_t *sel_cnt,
                          float *scores_opt, hipStream_t s) {
  ScanArgs a;
  int rc = ig_scan_args(ctx, d, q, slab, sel_idx, sel_stride, sel_cnt, scores_opt, &a);
  if (rc) return rc;
  return d->dtype == IG_F16 ? launch_scan<half_t>(ctx, d, a, s) : launch_scan<float>(ctx, d, a, s);
}
