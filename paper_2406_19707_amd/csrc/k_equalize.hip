// Head-equalised selection (Section 4.3 "Decoding Stage", closing sentences: every head of a
// layer fetches the same number of tokens, the average over the heads of the tokens between the
// maximum score and the threshold; Section 5.1 "Key Metric": at most 20 % of the cache per layer).
//
// Input: the speculated scores s [B,H,N] and the per-head threshold counts of ig_speculate.
// One workgroup per (sequence, head):
//   n      = clamp(floor(sum_h count[b,h] / H), 1, cap)
//   T      = the n-th largest score of the head, found exactly by a most-significant-digit radix
//            select on an order-preserving integer image of the float (4 passes of 8 bits, one
//            256-bin LDS histogram each).  The keys of a head stay in registers (KPT per thread)
//            when they fit; longer sequences re-read the scores from L2 in every pass.
//   list   = tokens with score > T, plus the earliest tokens with score == T until n are kept,
//            written in ascending token order with ballot / bit-count prefix ranks.
// Integer work after the scores: the result is exact for the scores given.
#include "ig_internal.h"

namespace {

// order-preserving image of a float: larger float <-> larger unsigned; -0 is folded onto +0
__device__ __forceinline__ unsigned score_key(float s) {
  const unsigned b = __float_as_uint(s + 0.0f);
  return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

template <int THREADS, int KPT>
__global__ __launch_bounds__(THREADS) void equalize_select(const float *__restrict__ scores,
                                                           const int32_t *__restrict__ thr_cnt,
                                                           int32_t *__restrict__ sel_idx,
                                                           int32_t *__restrict__ sel_cnt,
                                                           int32_t *status, int H, int N, int cap,
                                                           int stride) {
  constexpr int NW = THREADS / 64;
  __shared__ unsigned hist[256];
  __shared__ unsigned wave_sum_lds[4];
  __shared__ unsigned s_prefix;
  __shared__ int s_need, s_total;
  __shared__ int w_eq[NW], w_keep[NW];
  const int bh = blockIdx.x, b = bh / H;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const float *s = scores + (long)bh * N;

  // ---- n: truncated mean of the sequence's threshold counts, capped ----
  if (tid == 0) s_total = 0;
  __syncthreads();
  {
    int part = 0;
    for (int h = tid; h < H; h += THREADS) part += thr_cnt[b * H + h];
    part = wave_sum(part);
    if (lane == 0 && part) atomicAdd(&s_total, part);
  }
  __syncthreads();
  const int n = max(1, min(min(s_total / H, cap), N));

  // keys of tokens tid, tid + THREADS, ... (KPT of them) in registers; KPT == 0: re-read each pass
  unsigned keys[KPT > 0 ? KPT : 1];
  if (KPT > 0) {
#pragma unroll
    for (int i = 0; i < KPT; ++i) {
      const int t = i * THREADS + tid;
      keys[i] = t < N ? score_key(s[t]) : 0u;
    }
  }

  // ---- radix select of the n-th largest key ----
  unsigned prefix = 0;
  int need = n;
  for (int pass = 0; pass < 4; ++pass) {
    const int shift = 24 - 8 * pass;
    const unsigned hi_mask = pass == 0 ? 0u : (0xFFFFFFFFu << (shift + 8));
    if (tid < 256) hist[tid] = 0;
    __syncthreads();
    if (KPT > 0) {
#pragma unroll
      for (int i = 0; i < KPT; ++i) {
        const unsigned k = keys[i];
        if (i * THREADS + tid < N && (k & hi_mask) == prefix) atomicAdd(&hist[(k >> shift) & 255u], 1u);
      }
    } else {
      for (int t = tid; t < N; t += THREADS) {
        const unsigned k = score_key(s[t]);
        if ((k & hi_mask) == prefix) atomicAdd(&hist[(k >> shift) & 255u], 1u);
      }
    }
    __syncthreads();
    // bin d holds the target when (#keys in bins above d) < need <= (#keys in bins >= d)
    unsigned mine = 0, incl = 0;
    if (tid < 256) {
      mine = hist[tid];
      incl = mine;                             // suffix sum inside the wave: bins tid..(wave end)
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) {
        const unsigned u = __shfl_down(incl, o, 64);
        if (lane + o < 64) incl += u;
      }
      if (lane == 0) wave_sum_lds[w] = incl;   // total of this wave's 64 bins
    }
    __syncthreads();                           // every wave of the workgroup takes part
    if (tid < 256) {
      unsigned above = incl - mine;
      for (int k = w + 1; k < 4; ++k) above += wave_sum_lds[k];
      if ((int)above < need && need <= (int)(above + mine)) {
        s_prefix = prefix | ((unsigned)tid << shift);
        s_need = need - (int)above;
      }
    }
    __syncthreads();
    prefix = s_prefix;
    need = s_need;
    __syncthreads();
  }
  const unsigned T = prefix;       // key of the n-th largest score; `need` tokens equal to it are kept

  // ---- ordered compaction ----
  int base_out = 0, base_eq = 0;
  int32_t *list = sel_idx + (long)bh * stride;
  auto step = [&](int t0, unsigned k) {      // tokens t0 .. t0 + THREADS - 1, one per thread
    const int t = t0 + tid;
    const bool gt = t < N && k > T, eq = t < N && k == T;
    const unsigned long long be = __ballot(eq);
    if (lane == 0) w_eq[w] = __popcll(be);
    __syncthreads();
    int eq_rank = base_eq + lanes_below(be), eq_all = 0;
#pragma unroll
    for (int i = 0; i < NW; ++i) {
      const int c = w_eq[i];
      eq_rank += i < w ? c : 0;
      eq_all += c;
    }
    const bool keep = gt || (eq && eq_rank < need);
    const unsigned long long bk = __ballot(keep);
    if (lane == 0) w_keep[w] = __popcll(bk);
    __syncthreads();
    int pos = base_out + lanes_below(bk), keep_all = 0;
#pragma unroll
    for (int i = 0; i < NW; ++i) {
      const int c = w_keep[i];
      pos += i < w ? c : 0;
      keep_all += c;
    }
    if (keep && pos < stride) list[pos] = t;
    base_out += keep_all;
    base_eq += eq_all;
  };
  if constexpr (KPT > 0) {
#pragma unroll
    for (int it = 0; it < KPT; ++it)
      if (it * THREADS < N) step(it * THREADS, keys[it]);     // wave-uniform condition
  } else {
    for (int t0 = 0; t0 < N; t0 += THREADS) step(t0, t0 + tid < N ? score_key(s[t0 + tid]) : 0u);
  }
  if (tid == 0) {
    sel_cnt[bh] = min(base_out, stride);
    if (base_out > stride) atomicOr(status, IG_STATUS_CAPACITY);
  }
}

}  // namespace

int ig_launch_equalize(ig_ctx *ctx, const ig_desc *d, const float *scores, const int32_t *thr_cnt,
                       int cap, int32_t *sel_idx, int32_t sel_stride, int32_t *sel_cnt,
                       hipStream_t s) {
  const int BH = d->B * d->H;
#define EQ_CASE(THREADS, KPT)                                                                      \
  {                                                                                                \
    auto k = equalize_select<THREADS, KPT>;                                                        \
    IG_LAUNCH(ctx, IG_K_SELECT, k, dim3(BH), dim3(THREADS), s, scores, thr_cnt, sel_idx, sel_cnt,  \
              ctx->status, (int)d->H, (int)d->N, cap, (int)sel_stride);                            \
    return IG_OK;                                                                                  \
  }
  if (d->N <= 256 * 8) EQ_CASE(256, 8)
  if (d->N <= 256 * 16) EQ_CASE(256, 16)
  if (d->N <= 1024 * 16) EQ_CASE(1024, 16)
  if (d->N <= 1024 * 32) EQ_CASE(1024, 32)
  EQ_CASE(1024, 0)
#undef EQ_CASE
}
