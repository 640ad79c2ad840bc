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
// (no separate reduction kernel), or, for rotary models, finished from the finalisation kernel
// that applies the rotation and the partial skew between projection and scan.
#include "scan_device.h"

namespace {

// One workgroup per (b,h); wave w scans tile w (nValid <= NW) and keeps its scores in registers.
template <typename T, int CH, int NW>
__global__ __launch_bounds__(NW * 64) void scan_select_fused(ScanArgs a) {
  scan_select_fused_body<T, CH, NW>(a, blockIdx.x);
}

// Sequences of up to LDS_SCORES tokens that do not fit 16 waves at once: still one workgroup of
// 16 waves per (b,h); wave w scans tiles w, w + 16, ... and parks the scores in LDS (4 B/token,
// 128 KiB), so that the threshold pass needs neither a score buffer in memory nor further
// kernels.  The waves run through their tiles without meeting; they meet once for the maximum.
constexpr int LDS_SCORES = 32768;

template <typename T, int CH>
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
  // first channel block of the wave's first tile in flight while the partial query arrives
  if (w < a.nValid) load_block<T, CH>(head + (long)w * a.r * TILE, a.r, 0, lane, v);
  float qv[4];
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    qv[k] = 0.f;
    if (64 * k < a.r) {
      QueryLoads ql;
      query_issue(a, b, h, lane, k, ql);
      qv[k] = query_finish(a, ql);
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

// ---- streaming form: rolling load window, pairs optionally split over several workgroups ---------
// For the kept-channel counts the workloads use (R is a template parameter) a wave's tiles are one
// contiguous run of TPW*R KiB, read as a flat stream through a window of WIN 1 KiB loads: every
// load is consumed in issue order and its register is refilled at once with the load WIN places
// ahead, so a wave keeps WIN KiB in flight from its first instruction to its last, across tile
// boundaries, with no clamped re-reads and no per-block drain.  A workgroup of NW waves covers
// NW*TPW consecutive tiles of one (b,h); the scores stay in registers.
//
// A pair with more tiles than that is split over S workgroups whose ids lie within 8*S of each
// other (so that long sequences with few (b,h) pairs still put every compute unit to work).  The splits meet twice through a
// small per-pair record in device memory: once for the pair's maximum, once for the kept-token
// counts that give each split its offset in the ascending list.  Every split publishes one
// self-validating 8-byte word per meeting (relaxed agent-scope atomic store) and polls its
// partners' words (relaxed agent-scope atomic loads); both waits are bounded.  A workgroup whose wait runs out (its partners were not scheduled in time) takes
// the slow, self-sufficient route: it rescans the whole pair on its own and writes the whole list.
// Every store on either route is the exact final value, so the routes can mix freely within a
// pair; the last workgroup of a pair to finish zeroes the record for the next call.
struct PairSync {
  int done;            // splits that have finished with the record
  int pad[3];
  unsigned long long smax[IG_SPLIT_MAX];   // per split: bit 63 = published, low word = image of its maximum
  unsigned long long scnt[IG_SPLIT_MAX];   // per split: bit 63 = published, low word = its kept-token count
  int tail[12];
};
static_assert(sizeof(PairSync) == IG_PAIR_SYNC_BYTES, "PairSync size");
constexpr unsigned long long PUBLISHED = 1ull << 63;

__device__ __forceinline__ unsigned order_bits(float v) {
  const unsigned u = __float_as_uint(v);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float order_float(unsigned k) {
  return __uint_as_float((k & 0x80000000u) ? (k & 0x7fffffffu) : ~k);
}

// Wave 0 only.  Lane j < S polls slot j until every split has published; each slot carries its
// own "published" bit, so nothing has to be ordered against anything else and plain (relaxed)
// agent-scope atomics suffice -- no cache write-back or invalidation.  Returns false when `limit`
// ticks of the 100 MHz clock pass first (limit < 0: gives up without looking, which forces the
// slow route); *val is the lane's slot value (lanes >= S: just the bit).
__device__ __forceinline__ bool poll_slots(const unsigned long long *slots, int S, int lane, long limit,
                                           unsigned long long *val) {
  *val = PUBLISHED;
  if (limit < 0) return false;
  const long t0 = wall_clock64();
  while (true) {
    unsigned long long v = PUBLISHED;
    if (lane < S) v = __hip_atomic_load(slots + lane, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (__ballot((v & PUBLISHED) != 0) == ~0ull) {
      *val = v;
      return true;
    }
    if (wall_clock64() - t0 > limit) return false;
    __builtin_amdgcn_s_sleep(2);
  }
}

// Threshold + ordered compaction for a workgroup whose wave w holds, in registers, the scores of
// tiles w*TPW + i (i < TPW) counted from token t_first; token order is (w, i, lane, e).
// count_only: returns the workgroup's number of kept tokens and writes nothing.  Otherwise every
// wave first packs its kept token ids into its own LDS row (stage, TPW*TILE entries per wave) and
// then copies the row out with whole-wave stores: a handful of coalesced store instructions per
// wave instead of one scattered store per score register, which matters because every memory
// instruction of the epilogue queues behind the other workgroups' streaming loads.
// The three steps are separate so that a split pair can publish its count right after the first
// and pack (LDS only) while the partners' counts are on their way:
//   compact_rank  -> which scores are kept (bit masks), each lane's rank inside its wave, the
//                    wave's total, and across the workgroup: kept tokens in earlier waves / in all
//   compact_pack  -> the wave's kept token ids into its LDS row, in token order
//   compact_store -> the row to list[base + before ...]
template <int TPW>
struct Kept {
  unsigned mask[TPW];
  int rank[TPW];
  int mine, before, all;
};
template <int TPL, int NW, int TPW>
__device__ __forceinline__ void compact_rank(const float (&sc)[TPW][TPL], float thr, int N, int t_first,
                                             int *lds_cnt /* [NW] */, int w, int lane, Kept<TPW> &k) {
  constexpr int TILE = IG_WAVE * TPL;
  k.mine = 0;
#pragma unroll
  for (int i = 0; i < TPW; ++i) {
    const int t0 = t_first + (w * TPW + i) * TILE + lane * TPL;
    k.mask[i] = 0;
    int below = 0, total = 0;
#pragma unroll
    for (int e = 0; e < TPL; ++e) {
      const bool keep = t0 + e < N && sc[i][e] >= thr;
      const unsigned long long bal = __ballot(keep);
      below += lanes_below(bal);
      total += __popcll(bal);
      k.mask[i] |= (keep ? 1u : 0u) << e;
    }
    k.rank[i] = k.mine + below;
    k.mine += total;
  }
  if (lane == 0) lds_cnt[w] = k.mine;
  __syncthreads();
  k.before = 0;
  k.all = 0;
#pragma unroll
  for (int j = 0; j < NW; ++j) {
    const int c = lds_cnt[j];
    k.before += (j < w) ? c : 0;
    k.all += c;
  }
  __syncthreads();   // lds_cnt is reused
}
template <int TPL, int NW, int TPW>
__device__ __forceinline__ void compact_pack(const Kept<TPW> &k, int t_first, int32_t *stage, int w, int lane) {
  constexpr int TILE = IG_WAVE * TPL;
  int32_t *row = stage + w * (TPW * TILE);
#pragma unroll
  for (int i = 0; i < TPW; ++i) {
    const int t0 = t_first + (w * TPW + i) * TILE + lane * TPL;
    int p = k.rank[i];
#pragma unroll
    for (int e = 0; e < TPL; ++e) {
      if (k.mask[i] & (1u << e)) row[p++] = t0 + e;
    }
  }
}
template <int TPL, int TPW>
__device__ __forceinline__ void compact_store(const Kept<TPW> &k, int base, int32_t *list, int sel_stride,
                                              const int32_t *stage, int w, int lane) {
  constexpr int TILE = IG_WAVE * TPL;
  const int32_t *row = stage + w * (TPW * TILE);
  const int out0 = base + k.before;
  for (int j = lane; j < k.mine; j += IG_WAVE)
    if (out0 + j < sel_stride) list[out0 + j] = row[j];
}
template <int TPL, int NW, int TPW>
__device__ __forceinline__ int compact_tiles(const float (&sc)[TPW][TPL], float thr, int N, int base,
                                             int32_t *list, int sel_stride, int t_first, int *lds_cnt /* [NW] */,
                                             int32_t *stage, int w, int lane, bool count_only) {
  Kept<TPW> k;
  compact_rank<TPL, NW, TPW>(sc, thr, N, t_first, lds_cnt, w, lane, k);
  if (count_only) return k.all;
  compact_pack<TPL, NW, TPW>(k, t_first, stage, w, lane);
  compact_store<TPL, TPW>(k, base, list, sel_stride, stage, w, lane);
  return k.all;
}

// ---- head-equalised selection inside the streaming kernel ----------------------------------------
// Section 4.3 "Decoding Stage", closing sentences: every head of a sequence keeps the same number
// of tokens, the (truncated) mean over the heads of the per-head threshold counts, at most `cap`
// (Section 5.1 "Key Metric"); a head keeps its n highest scores, the earlier token on equal scores.
// The workgroups of a sequence's heads exchange their threshold counts through a small record in
// device memory, the way the splits of a pair exchange maxima: one self-validating word per head,
// a bounded wait, and a self-sufficient route for a workgroup whose wait runs out (it works out the
// other heads' counts alone).  The scores never leave the registers.
struct EqArgs {
  unsigned long long *seq;   // [B][H + 1]: per head "published | threshold count"; then the arrivals counter
  int32_t *thr_cnt;          // optional: the per-head threshold counts [B*H]
  int cap;                   // floor(max_frac * N), at least 1
};

// order-preserving image of a score (larger score <-> larger key; -0 folded onto +0): the key the
// stand-alone equalisation kernel selects on, so both give the same lists
__device__ __forceinline__ unsigned eq_key(float s) {
  const unsigned b = __float_as_uint(s + 0.0f);
  return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

// Wave 0 only: waits until all H heads of the sequence have published, returns their sum.
__device__ __forceinline__ bool poll_heads(const unsigned long long *slots, int H, int lane, long limit, int *total) {
  *total = 0;
  if (limit < 0) return false;
  const long t0 = wall_clock64();
  while (true) {
    int sum = 0;
    bool all = true;
    for (int c = 0; c < H; c += IG_WAVE) {
      unsigned long long v = PUBLISHED;
      if (c + lane < H) v = __hip_atomic_load(slots + c + lane, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      all = all && __ballot((v & PUBLISHED) != 0) == ~0ull;
      sum += (c + lane < H) ? (int)(unsigned)v : 0;
    }
    if (all) {
      *total = wave_sum(sum);
      return true;
    }
    if (wall_clock64() - t0 > limit) return false;
    __builtin_amdgcn_s_sleep(2);
  }
}

// Key of the n-th largest valid score of the workgroup's tokens (4 waves; wave w holds tiles
// w*TPW + i): most-significant-digit radix select, 4 passes of 8 bits, one 256-bin LDS histogram
// each.  *need_out = how many tokens equal to that key are to be kept.
template <int TPL, int TPW>
__device__ __forceinline__ unsigned nth_largest_key(const float (&sc)[TPW][TPL], const unsigned (&valid)[TPW], int n,
                                                    unsigned *hist /*[256]*/, unsigned *wsum /*[4]*/,
                                                    unsigned *s_prefix, int *s_need, int *need_out) {
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  unsigned prefix = 0;
  int need = n;
  for (int pass = 0; pass < 4; ++pass) {
    const int shift = 24 - 8 * pass;
    const unsigned hi_mask = pass == 0 ? 0u : (0xFFFFFFFFu << (shift + 8));
    hist[tid] = 0;
    __syncthreads();
#pragma unroll
    for (int i = 0; i < TPW; ++i)
#pragma unroll
      for (int e = 0; e < TPL; ++e) {
        const unsigned k = eq_key(sc[i][e]);
        if (((valid[i] >> e) & 1u) && (k & hi_mask) == prefix) atomicAdd(&hist[(k >> shift) & 255u], 1u);
      }
    __syncthreads();
    // bin d holds the target when (#keys in bins above d) < need <= (#keys in bins >= d)
    const unsigned mine = hist[tid];
    unsigned incl = mine;                     // suffix sum inside the wave: bins tid .. (wave end)
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const unsigned u = __shfl_down(incl, o, 64);
      if (lane + o < 64) incl += u;
    }
    if (lane == 0) wsum[w] = incl;
    __syncthreads();
    unsigned above = incl - mine;
    for (int k = w + 1; k < 4; ++k) above += wsum[k];
    if ((int)above < need && need <= (int)(above + mine)) {
      *s_prefix = prefix | ((unsigned)tid << shift);
      *s_need = need - (int)above;
    }
    __syncthreads();
    prefix = *s_prefix;
    need = *s_need;
    __syncthreads();
  }
  *need_out = need;
  return prefix;
}

// Ordered compaction of the tokens whose key exceeds T plus the first `need` tokens (in token
// order) whose key equals T; otherwise as compact_tiles.  Returns the number of tokens kept.
template <int TPL, int NW, int TPW>
__device__ __forceinline__ int compact_tiles_topn(const float (&sc)[TPW][TPL], const unsigned (&valid)[TPW], unsigned T,
                                                  int need, int32_t *list, int sel_stride, int *lds_cnt /*[NW]*/,
                                                  int32_t *stage, int w, int lane) {
  constexpr int TILE = IG_WAVE * TPL;
  unsigned eqm[TPW], keep[TPW];
  int eq_rank[TPW], eq_mine = 0;
#pragma unroll
  for (int i = 0; i < TPW; ++i) {
    eqm[i] = 0;
    keep[i] = 0;
    int below = 0, total = 0;
#pragma unroll
    for (int e = 0; e < TPL; ++e) {
      const unsigned k = eq_key(sc[i][e]);
      const bool ok = (valid[i] >> e) & 1u;
      const bool eq = ok && k == T;
      const unsigned long long bal = __ballot(eq);
      below += lanes_below(bal);
      total += __popcll(bal);
      eqm[i] |= (eq ? 1u : 0u) << e;
      keep[i] |= ((ok && k > T) ? 1u : 0u) << e;
    }
    eq_rank[i] = eq_mine + below;
    eq_mine += total;
  }
  if (lane == 0) lds_cnt[w] = eq_mine;
  __syncthreads();
  int eq_before = 0;
#pragma unroll
  for (int k = 0; k < NW; ++k) eq_before += (k < w) ? lds_cnt[k] : 0;
  __syncthreads();   // lds_cnt is reused
  int rank[TPW], mine = 0;
#pragma unroll
  for (int i = 0; i < TPW; ++i) {
    int p = eq_before + eq_rank[i];
    int below = 0, total = 0;
#pragma unroll
    for (int e = 0; e < TPL; ++e) {
      if ((eqm[i] >> e) & 1u) {
        if (p < need) keep[i] |= 1u << e;
        ++p;
      }
      const unsigned long long bal = __ballot((keep[i] >> e) & 1u);
      below += lanes_below(bal);
      total += __popcll(bal);
    }
    rank[i] = mine + below;
    mine += total;
  }
  if (lane == 0) lds_cnt[w] = mine;
  __syncthreads();
  int before = 0, all = 0;
#pragma unroll
  for (int k = 0; k < NW; ++k) {
    const int c = lds_cnt[k];
    before += (k < w) ? c : 0;
    all += c;
  }
  __syncthreads();
  int32_t *row = stage + w * (TPW * TILE);
#pragma unroll
  for (int i = 0; i < TPW; ++i) {
    const int t0 = (w * TPW + i) * TILE + lane * TPL;
    int p = rank[i];
#pragma unroll
    for (int e = 0; e < TPL; ++e)
      if ((keep[i] >> e) & 1u) row[p++] = t0 + e;
  }
  for (int j = lane; j < mine; j += IG_WAVE)
    if (before + j < sel_stride) list[before + j] = row[j];
  return all;
}

// The slow route, step by step: 16-byte loads in blocks of 8 channels, NW tiles per round in token
// order, by this workgroup alone.  pair_max: the pair's maximum; rescan_pair: scores again, then
// threshold and the whole ascending list and its count.
template <typename T, int NW>
__device__ __forceinline__ float pair_max(const ScanArgs &a, int bh, float q_lane, float *lds_max) {
  constexpr int TPL = SlabElem<T>::TPL;
  constexpr int TILE = IG_WAVE * TPL;
  const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const T *head = static_cast<const T *>(a.slab) + (long)bh * a.nTiles * a.r * TILE;
  const float qv[4] = {q_lane, 0.f, 0.f, 0.f};
  typename SlabElem<T>::vec v[8];
  float m = -INFINITY;
  for (int ti = w; ti < a.nValid; ti += NW) {
    const T *tile = head + (long)ti * a.r * TILE;
    float acc[TPL];
#pragma unroll
    for (int e = 0; e < TPL; ++e) acc[e] = 0.f;
    load_block<T, 8>(tile, a.r, 0, lane, v);
    scan_tile_given_q<T, 8>(a, tile, lane, v, qv, acc);
#pragma unroll
    for (int e = 0; e < TPL; ++e)
      if (ti * TILE + lane * TPL + e < a.N) m = fmaxf(m, acc[e]);
  }
  m = wave_max(m);
  __syncthreads();
  if (lane == 0) lds_max[w] = m;
  __syncthreads();
  float mm = lds_max[0];
#pragma unroll
  for (int k = 1; k < NW; ++k) mm = fmaxf(mm, lds_max[k]);
  return mm;
}

template <typename T, int NW>
__device__ __forceinline__ void rescan_pair(const ScanArgs &a, int bh, float q_lane, float thr, int *lds_cnt) {
  constexpr int TPL = SlabElem<T>::TPL;
  constexpr int TILE = IG_WAVE * TPL;
  const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const T *head = static_cast<const T *>(a.slab) + (long)bh * a.nTiles * a.r * TILE;
  const float qv[4] = {q_lane, 0.f, 0.f, 0.f};
  typename SlabElem<T>::vec v[8];
  int base = 0;
  for (int t0w = 0; t0w < a.nValid; t0w += NW) {
    const int ti = t0w + w;
    float acc[TPL];
#pragma unroll
    for (int e = 0; e < TPL; ++e) acc[e] = 0.f;
    if (ti < a.nValid) {
      const T *tile = head + (long)ti * a.r * TILE;
      load_block<T, 8>(tile, a.r, 0, lane, v);
      scan_tile_given_q<T, 8>(a, tile, lane, v, qv, acc);
    }
    base += compact_block<TPL, NW>(acc, ti * TILE, a.N, thr, base, a.sel_idx + (long)bh * a.sel_stride,
                                   a.sel_stride, lds_cnt, w, lane);
  }
  if (threadIdx.x == 0) {
    a.sel_cnt[bh] = min(base, a.sel_stride);
    if (base > a.sel_stride) atomicOr(a.status, IG_STATUS_CAPACITY);
  }
}

// Slow route of the head-equalised form: the threshold count of another head of the sequence,
// worked out by this workgroup alone (q_lane: that head's partial query).
template <typename T, int NW>
__device__ __forceinline__ int count_pair(const ScanArgs &a, int bh, float q_lane, float thr, int *lds_cnt) {
  constexpr int TPL = SlabElem<T>::TPL;
  constexpr int TILE = IG_WAVE * TPL;
  const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const T *head = static_cast<const T *>(a.slab) + (long)bh * a.nTiles * a.r * TILE;
  const float qv[4] = {q_lane, 0.f, 0.f, 0.f};
  typename SlabElem<T>::vec v[8];
  int n = 0;
  for (int ti = w; ti < a.nValid; ti += NW) {
    const T *tile = head + (long)ti * a.r * TILE;
    float acc[TPL];
#pragma unroll
    for (int e = 0; e < TPL; ++e) acc[e] = 0.f;
    load_block<T, 8>(tile, a.r, 0, lane, v);
    scan_tile_given_q<T, 8>(a, tile, lane, v, qv, acc);
#pragma unroll
    for (int e = 0; e < TPL; ++e) n += (ti * TILE + lane * TPL + e < a.N && acc[e] >= thr) ? 1 : 0;
  }
  n = wave_sum(n);
  __syncthreads();
  if (lane == 0) lds_cnt[w] = n;
  __syncthreads();
  int all = 0;
#pragma unroll
  for (int k = 0; k < NW; ++k) all += lds_cnt[k];
  __syncthreads();
  return all;
}

// Partial query of a rotary model inside the streaming kernel (Section 4.3 "Decoding Stage" for
// models whose skew cannot be folded into W_Q): qsrc holds the split-K partial sums of the FULL
// projection x W_Q ([ks][b][D] columns) and the workgroup finishes its head itself --
//   q[c]   = bias[h*d+c] + sum_s part[s][b][h*d+c]            (split-K sums in a fixed order)
//   rotate pairs (c, c+d/2) by pos[b]*theta^(-2c/d)            (angle in double)
//   q_p[k] = sum_c q_rot[c] * A_p[h][c][k]                     (rows split over thread groups, added in order)
// -- the arithmetic of the stand-alone finalisation kernel.  Loads return to a wave in the order
// it issued them, so everything the prologue reads (partial sums, position, the thread's rows of
// A_p) is issued by rope_issue BEFORE the wave's slab window; rope_finish then runs while the window
// is still travelling.  Heads of up to 256 columns; a thread prefetches rope_pf(r) rows of A_p, the
// share of a 128-column head when 256 threads are split into groups of r.
constexpr int rope_pf(int r) { return (128 + 256 / r - 1) / (256 / r); }
struct RopeArgs {
  const float *A_p;     // [H, d, r]
  const int32_t *pos;   // [B]
  int d;
  double freq_step;     // -(2/d) log2(theta)
};
template <int PF>
struct RopeLoads {
  float part[IG_KS_MAX];
  float bias;
  float apf[PF];
  int position;
};
template <int THREADS, int PF>
__device__ __forceinline__ void rope_issue(const ScanArgs &a, const RopeArgs &ra, int b, int h, RopeLoads<PF> &L) {
  // straight-line code, every load unconditional (addresses clamped, surplus values discarded
  // later): the compiler can then count exactly how many loads may still be outstanding at each
  // use, instead of waiting for all of them -- the slab window included -- after a branch
  const int t = threadIdx.x, d = ra.d, r = a.r;
  const float *p = a.qsrc + (long)b * a.b_stride + (long)h * d + min(t, d - 1);
#pragma unroll
  for (int s = 0; s < IG_KS_MAX; ++s) L.part[s] = p[(long)min(s, a.ks - 1) * a.ks_stride];
  L.bias = a.bias ? a.bias[h * d + min(t, d - 1)] : 0.f;
  L.position = ra.pos[b];
  const int G = THREADS / r, k = t % r, g = min(t / r, G - 1);
  const int per = (d + G - 1) / G;
  const int c0 = min(d, g * per);
  const float *ap = ra.A_p + (long)h * d * r + k;
#pragma unroll
  for (int i = 0; i < PF; ++i) L.apf[i] = ap[(long)min(c0 + i, d - 1) * r];
}
template <int THREADS, int PF>
__device__ __forceinline__ void rope_finish(const ScanArgs &a, const RopeArgs &ra, const RopeLoads<PF> &L,
                                            float *q_lds, float *qr_lds, float *psum, float *qp_lds) {
  const int t = threadIdx.x, d = ra.d, r = a.r;
  {
    float acc = L.bias;
#pragma unroll
    for (int s = 0; s < IG_KS_MAX; ++s) acc += s < a.ks ? L.part[s] : 0.f;
    if (t < d) q_lds[t] = acc;
  }
  __syncthreads();
  const int half = d / 2;
  if (t < half) {
    double sn, cs;
    rope_sincos((double)L.position * exp2((double)t * ra.freq_step), &sn, &cs);
    const float x0 = q_lds[t], x1 = q_lds[t + half];
    qr_lds[t] = (float)((double)x0 * cs - (double)x1 * sn);
    qr_lds[t + half] = (float)((double)x1 * cs + (double)x0 * sn);
  }
  __syncthreads();
  const int G = THREADS / r, g = t / r;
  const int per = (d + G - 1) / G;
  const int c0 = g < G ? min(d, g * per) : d, c1 = g < G ? min(d, (g + 1) * per) : d;
  float acc = 0.f;
#pragma unroll
  for (int i = 0; i < PF; ++i)
    if (c0 + i < c1) acc = fmaf(qr_lds[c0 + i], L.apf[i], acc);
  psum[t] = acc;
  __syncthreads();
  if (t < r) {
    float tot = 0.f;
    for (int gg = 0; gg < G; ++gg) tot += psum[gg * r + t];
    qp_lds[t] = tot;
  }
  __syncthreads();
}
// shapes the in-kernel prologue takes: one column per thread, every thread's rows of A_p prefetched
static inline bool rope_prologue_fits(int threads, int d, int r) {
  if (d > threads || d > 256 || r > threads) return false;
  const int G = threads / r;
  return (d + G - 1) / G <= rope_pf(r);
}

template <typename T, int R, int NW, int TPW, int WIN, int MINW, bool ROPE, bool EQ>
__global__ __launch_bounds__(NW * 64, MINW) void scan_select_stream(ScanArgs a, RopeArgs ra, EqArgs eq, int S, int BH, PairSync *sync, long spin_limit) {
  constexpr int TPL = SlabElem<T>::TPL;
  constexpr int TILE = IG_WAVE * TPL;
  constexpr int NLOAD = TPW * R;              // 1 KiB loads of a wave with all its tiles valid
  typedef typename SlabElem<T>::vec vec;
  __shared__ float lds_max[NW];
  __shared__ int lds_cnt[NW];
  __shared__ int lds_flag[2];
  __shared__ int32_t stage[NW * TPW * TILE];
  __shared__ float lds_gmax;
  // Workgroup -> (pair, split): groups of 8 pairs take 8*S consecutive ids, split-major inside the
  // group (id = group*8*S + split*8 + pair%8).  Workgroups are handed to the 8 XCDs round-robin by
  // id, so the S workgroups of a pair land on one XCD and what they all read besides the slab (the
  // projection's partial sums; for rotary models the head's columns of the skewing matrix) is
  // fetched into that XCD's L2 once instead of S times, while a pair's workgroups still start
  // within 8*S ids of each other.  (Only where bytes are fetched from changes with the hardware's
  // dispatch order, not the result.)
  const int grp = blockIdx.x / (8 * S), rem = blockIdx.x - grp * 8 * S;
  const int s = rem >> 3, bh = grp * 8 + (rem & 7);
  if (bh >= BH) return;                                   // the grid is rounded up to whole groups
  const int b = bh / a.H, h = bh - b * a.H;
  const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int tile0 = s * (NW * TPW);                       // first tile of this workgroup
  const int my0 = tile0 + w * TPW;                        // first tile of this wave
  const int nact = max(0, min(TPW, a.nValid - my0));      // valid tiles of this wave (wave-uniform)
  // a wave with fewer valid tiles re-reads its last valid one in their place (masked below), and a
  // wave with none the pair's last valid tile, so the load sequence is the same for every wave
  const char *tbase[TPW];
#pragma unroll
  for (int i = 0; i < TPW; ++i)
    tbase[i] = reinterpret_cast<const char *>(static_cast<const T *>(a.slab) +
                                              ((long)bh * a.nTiles + min(my0 + max(0, min(i, nact - 1)), a.nValid - 1)) * R * TILE);
  const int lane_off = lane * (int)sizeof(vec);
  constexpr int PLANE = TILE * (int)sizeof(T);            // bytes of one channel plane (1 KiB)
  vec v[WIN];
  // the query's own loads go out first, so that they head the wave's memory queue
  QueryLoads ql;
  RopeLoads<rope_pf(R)> rl;
  if constexpr (ROPE) rope_issue<NW * 64, rope_pf(R)>(a, ra, b, h, rl);
  else query_issue(a, b, h, lane, 0, ql);
  __builtin_amdgcn_sched_barrier(0);
  // (unconditional, like the query's loads: a branch here would make the compiler wait for the
  // whole window wherever the query is first used)
#pragma unroll
  for (int k = 0; k < WIN && k < NLOAD; ++k)
    v[k] = *reinterpret_cast<const vec *>(tbase[k / R] + (k % R) * PLANE + lane_off);
  __builtin_amdgcn_sched_barrier(0);
  float q_lane;
  __shared__ float q_lds[ROPE ? 256 : 1], qr_lds[ROPE ? 256 : 1], psum[ROPE ? NW * 64 : 1], qp_lds[ROPE ? 64 : 1];
  if constexpr (ROPE) {
    rope_finish<NW * 64, rope_pf(R)>(a, ra, rl, q_lds, qr_lds, psum, qp_lds);
    q_lane = lane < R ? qp_lds[lane] * a.scale : 0.f;
  } else {
    q_lane = query_finish(a, ql);
  }
  float sc[TPW][TPL];
#pragma unroll
  for (int i = 0; i < TPW; ++i)
#pragma unroll
    for (int e = 0; e < TPL; ++e) sc[i][e] = 0.f;
  if (nact > 0) {
    const int qbits = __float_as_int(q_lane);
#pragma unroll
    for (int k = 0; k < NLOAD; ++k) {
      const int i = k / R, j = k % R;
      const float qj = __int_as_float(__builtin_amdgcn_readlane(qbits, j));
#pragma unroll
      for (int e = 0; e < TPL; ++e) sc[i][e] = fmaf((float)v[k % WIN][e], qj, sc[i][e]);
      if (k + WIN < NLOAD)
        v[k % WIN] = *reinterpret_cast<const vec *>(tbase[(k + WIN) / R] + ((k + WIN) % R) * PLANE + lane_off);
      __builtin_amdgcn_sched_barrier(0);     // keeps issue order = consumption order: WIN - 1 loads stay in flight
    }
  }
  // mask, optional dump, workgroup maximum
  float m = -INFINITY;
#pragma unroll
  for (int i = 0; i < TPW; ++i) {
    const int t0 = (my0 + i) * TILE + lane * TPL;
    if (a.scores_out && i < nact) store_scores<TPL>(a.scores_out, (long)bh * a.N, t0, a.N, sc[i]);
#pragma unroll
    for (int e = 0; e < TPL; ++e) {
      if (i >= nact || t0 + e >= a.N) sc[i][e] = -INFINITY;
      m = fmaxf(m, sc[i][e]);
    }
  }
  m = wave_max(m);
  if (lane == 0) lds_max[w] = m;
  __syncthreads();
  float mm = lds_max[0];
#pragma unroll
  for (int k = 1; k < NW; ++k) mm = fmaxf(mm, lds_max[k]);
  int32_t *list = a.sel_idx + (long)bh * a.sel_stride;
  if constexpr (EQ) {
    // ---- head-equalised lists (one workgroup per pair: S == 1) ----
    static_assert(NW == 4, "the radix select's histogram scan is written for 4 waves");
    __shared__ unsigned eq_hist[256], eq_wsum[4], eq_prefix;
    __shared__ int eq_need;
    const int cnt = compact_tiles<TPL, NW, TPW>(sc, mm - a.alpha, a.N, 0, list, a.sel_stride, 0, lds_cnt, stage, w, lane, true);
    if (eq.thr_cnt && threadIdx.x == 0) eq.thr_cnt[bh] = cnt;
    unsigned long long *rec = eq.seq + (long)b * (a.H + 1);
    if (w == 0) {
      if (lane == 0)
        __hip_atomic_store(&rec[h], PUBLISHED | (unsigned long long)(unsigned)cnt, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      int total = 0;
      const bool ok = poll_heads(rec, a.H, lane, spin_limit, &total);
      if (lane == 0) {
        lds_flag[0] = ok;
        lds_flag[1] = total;
      }
      if (!ok) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // own slot has landed before "done"
    }
    __syncthreads();
    // the record has been read for the last time: report it now, the answer is looked at at the end
    unsigned long long prev_done = 0;
    if (w == 0 && lane == 0)
      prev_done = __hip_atomic_fetch_add(&rec[a.H], 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    int total = lds_flag[1];
    if (lds_flag[0] == 0) {
      // the other heads' counts did not arrive in time: work them out alone, head by head
      total = 0;
      for (int h2 = 0; h2 < a.H; ++h2) {
        if (h2 == h) {
          total += cnt;
          continue;
        }
        float q2;
        if constexpr (ROPE) {
          RopeLoads<rope_pf(R)> rl2;
          rope_issue<NW * 64, rope_pf(R)>(a, ra, b, h2, rl2);
          __syncthreads();
          rope_finish<NW * 64, rope_pf(R)>(a, ra, rl2, q_lds, qr_lds, psum, qp_lds);
          q2 = lane < R ? qp_lds[lane] * a.scale : 0.f;
        } else {
          QueryLoads ql2;
          query_issue(a, b, h2, lane, 0, ql2);
          q2 = query_finish(a, ql2);
        }
        const float m2 = pair_max<T, NW>(a, b * a.H + h2, q2, lds_max);
        total += count_pair<T, NW>(a, b * a.H + h2, q2, m2 - a.alpha, lds_cnt);
      }
    }
    const int n = max(1, min(min(total / a.H, eq.cap), a.N));
    unsigned valid[TPW];
#pragma unroll
    for (int i = 0; i < TPW; ++i) {
      const int t0 = (my0 + i) * TILE + lane * TPL;
      valid[i] = 0;
#pragma unroll
      for (int e = 0; e < TPL; ++e) valid[i] |= ((i < nact && t0 + e < a.N) ? 1u : 0u) << e;
    }
    int need = 0;
    const unsigned Tkey = nth_largest_key<TPL, TPW>(sc, valid, n, eq_hist, eq_wsum, &eq_prefix, &eq_need, &need);
    const int all = compact_tiles_topn<TPL, NW, TPW>(sc, valid, Tkey, need, list, a.sel_stride, lds_cnt, stage, w, lane);
    if (threadIdx.x == 0) {
      a.sel_cnt[bh] = min(all, a.sel_stride);
      if (all > a.sel_stride) atomicOr(a.status, IG_STATUS_CAPACITY);
    }
    // the last head to have reported clears the sequence's record for the next call
    if (w == 0) {
      const int prev_lo = __builtin_amdgcn_readfirstlane((int)prev_done);
      if (prev_lo == a.H - 1) {
        for (int c = lane; c <= a.H; c += IG_WAVE)
          __hip_atomic_store(&rec[c], 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
    }
    return;
  }
  if (S == 1) {
    const int all = compact_tiles<TPL, NW, TPW>(sc, mm - a.alpha, a.N, 0, list, a.sel_stride, 0, lds_cnt, stage, w, lane, false);
    if (threadIdx.x == 0) {
      a.sel_cnt[bh] = min(all, a.sel_stride);
      if (all > a.sel_stride) atomicOr(a.status, IG_STATUS_CAPACITY);
    }
    return;
  }
  // ---- the pair's splits meet: maximum ----
  PairSync *ps = sync + bh;
  if (w == 0) {
    if (lane == 0)
      __hip_atomic_store(&ps->smax[s], PUBLISHED | order_bits(mm), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    unsigned long long v;
    const bool ok = poll_slots(ps->smax, S, lane, spin_limit, &v);
    const float g = wave_max((ok && lane < S) ? order_float((unsigned)v) : -INFINITY);
    if (lane == 0) {
      lds_flag[0] = ok;
      lds_gmax = g;
    }
  }
  __syncthreads();
  const bool slow = lds_flag[0] == 0;
  // the partners' maxima did not arrive in time: find the pair's maximum alone (this split's
  // count can then be published all the same, so that partners which are only late are not held up)
  const float gmax = slow ? pair_max<T, NW>(a, bh, q_lane, lds_max) : lds_gmax;
  const float thr = gmax - a.alpha;
  // ---- the pair's splits meet: counts ----
  // (ranks first, then the count goes out; the kept ids are packed into LDS while the partners'
  // counts are on their way, and only the stores wait for this split's offset)
  Kept<TPW> kept;
  compact_rank<TPL, NW, TPW>(sc, thr, a.N, tile0 * TILE, lds_cnt, w, lane, kept);
  const int mine = kept.all;
  if (w == 0 && lane == 0)
    __hip_atomic_store(&ps->scnt[s], PUBLISHED | (unsigned)mine, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  compact_pack<TPL, NW, TPW>(kept, tile0 * TILE, stage, w, lane);
  if (w == 0) {
    unsigned long long v = 0;
    const bool ok = !slow && poll_slots(ps->scnt, S, lane, spin_limit, &v);
    const int c = (ok && lane < S) ? (int)(unsigned)v : 0;
    const int all = wave_sum(c), base = wave_sum(lane < s ? c : 0);
    if (lane == 0) {
      lds_flag[1] = ok;
      lds_cnt[0] = base;
      lds_flag[0] = all;
    }
    // a split that goes on alone makes sure its own slots have landed before it reports "done"
    if (!ok) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  }
  __syncthreads();
  // This split has read the record for the last time: its "done" goes out now, so that the trip to
  // the counter runs under the list stores; the last split to get there clears the record for the
  // next call (below, once the counter's answer is back).
  int prev_done = 0;
  if (w == 0 && lane == 0) prev_done = __hip_atomic_fetch_add(&ps->done, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  if (lds_flag[1]) {
    const int base = lds_cnt[0], all = lds_flag[0];
    compact_store<TPL, TPW>(kept, base, list, a.sel_stride, stage, w, lane);
    if (s == S - 1 && threadIdx.x == 0) {
      a.sel_cnt[bh] = min(all, a.sel_stride);
      if (all > a.sel_stride) atomicOr(a.status, IG_STATUS_CAPACITY);
    }
  } else {
    rescan_pair<T, NW>(a, bh, q_lane, thr, lds_cnt);
  }
  // ---- the last split to have reported "done" clears the record for the next call ----
  if (w == 0) {
    const int prev = __builtin_amdgcn_readfirstlane(prev_done);
    if (prev == S - 1) {
      if (lane < S) {
        __hip_atomic_store(&ps->smax[lane], 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(&ps->scnt[lane], 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
      if (lane == 0) __hip_atomic_store(&ps->done, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
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
    auto k = scan_select_fused<T, CHV, NW>;                                    \
    IG_LAUNCH(ctx, IG_K_SCAN, k, grid, block, s, a);                           \
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

// streaming form: the (kept channels, tiles per wave) combinations that are built; 4 waves per
// workgroup, 8 loads of 1 KiB in flight per wave (deeper windows measured the same), registers held
// to 96 so that five workgroups share a compute unit (one tile or two per wave) or to 128 (four)
template <typename T, int R, int NW, int TPW, int WIN, int MINW>
int launch_stream_one(ig_ctx *ctx, const ScanArgs &a, const RopeArgs *ra, const EqArgs *eq, int BH, int S, hipStream_t s) {
  dim3 grid((unsigned)((BH + 7) / 8 * 8 * S)), block(NW * 64);
  PairSync *sync = static_cast<PairSync *>(ctx->pair_sync);
  if (eq) {
    if constexpr (TPW <= 2) {      // head-equalised lists: the forms with one workgroup per pair
      if (S != 1) return ig_fail(ctx, IG_ESHAPE, "scan: head-equalised lists need one workgroup per pair");
      if (ra) {
        auto k = scan_select_stream<T, R, NW, TPW, WIN, 3, true, true>;    // (few workgroups per compute unit here)
        IG_LAUNCH(ctx, IG_K_SCAN, k, grid, block, s, a, *ra, *eq, S, BH, sync, ctx->spin_limit);
      } else {
        auto k = scan_select_stream<T, R, NW, TPW, WIN, 4, false, true>;
        IG_LAUNCH(ctx, IG_K_SCAN, k, grid, block, s, a, RopeArgs{}, *eq, S, BH, sync, ctx->spin_limit);
      }
      return IG_OK;
    }
    return ig_fail(ctx, IG_ESHAPE, "scan: head-equalised lists are not built for %d tiles per wave", TPW);
  }
  if (ra) {
    auto k = scan_select_stream<T, R, NW, TPW, WIN, MINW, true, false>;
    IG_LAUNCH(ctx, IG_K_SCAN, k, grid, block, s, a, *ra, EqArgs{}, S, BH, sync, ctx->spin_limit);
  } else {
    auto k = scan_select_stream<T, R, NW, TPW, WIN, MINW, false, false>;
    IG_LAUNCH(ctx, IG_K_SCAN, k, grid, block, s, a, RopeArgs{}, EqArgs{}, S, BH, sync, ctx->spin_limit);
  }
  return IG_OK;
}

template <typename T, int R>
int launch_stream_r(ig_ctx *ctx, const ScanArgs &a, const RopeArgs *ra, const EqArgs *eq, int BH, int TPW, int S, hipStream_t s) {
  if (TPW == 1) return launch_stream_one<T, R, 4, 1, 8, 5>(ctx, a, ra, eq, BH, S, s);
  if (TPW == 2) return launch_stream_one<T, R, 4, 2, 8, 5>(ctx, a, ra, eq, BH, S, s);
  if constexpr (R <= 32) {   // (with more channels the unrolled stream of 4 tiles no longer stays in registers)
    if (TPW == 4) return launch_stream_one<T, R, 4, 4, 8, 4>(ctx, a, ra, eq, BH, S, s);
  }
  return ig_fail(ctx, IG_ESHAPE, "scan: streaming form with %d tiles per wave is not built", TPW);
}

int launch_stream(ig_ctx *ctx, const ScanArgs &a, const RopeArgs *ra, const EqArgs *eq, int BH, int TPW, int S, hipStream_t s) {
  if (S < 1 || S > IG_SPLIT_MAX) return ig_fail(ctx, IG_ESHAPE, "scan: %d splits per pair", S);
  if (S > 1) {
    int rc = ig_ensure_zeroed(ctx, &ctx->pair_sync, &ctx->pair_sync_bytes, (size_t)BH * IG_PAIR_SYNC_BYTES);
    if (rc) return rc;
  }
  if (a.r == 38) return launch_stream_r<half_t, 38>(ctx, a, ra, eq, BH, TPW, S, s);
  if (a.r == 25) return launch_stream_r<half_t, 25>(ctx, a, ra, eq, BH, TPW, S, s);
  return ig_fail(ctx, IG_ESHAPE, "scan: streaming form is not built for r = %d", a.r);
}

template <typename T>
int launch_lds(ig_ctx *ctx, const ScanArgs &a, int BH, int ch, hipStream_t s) {
  dim3 grid(BH), block(1024);
#define CASE(CHV)                                                              \
  case CHV: {                                                                  \
    auto k = scan_select_lds<T, CHV>;                                          \
    IG_LAUNCH(ctx, IG_K_SCAN, k, grid, block, s, a);                           \
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
int launch_scan(ig_ctx *ctx, const ig_desc *d, ScanArgs &a, const QSource *rope, const EqArgs *eq, hipStream_t s) {
  const int BH = d->B * d->H;
  const int nTiles = a.nValid;     // the work, not the capacity, picks the kernel
  // One workgroup per (b,h) when it fits and there are enough (b,h) pairs to fill the chip;
  // otherwise one wave per tile so that long sequences spread over all compute units.
  int tpw = 0, S = 0;
  if (ig_scan_stream_form(d, &tpw, &S)) {
    if (!rope) return launch_stream(ctx, a, nullptr, eq, BH, tpw, S, s);
    RopeArgs ra{rope->A_p, rope->pos, d->d, -2.0 / (double)d->d * log2((double)d->rope_theta)};
    return launch_stream(ctx, a, &ra, eq, BH, tpw, S, s);
  }
  if (rope) return ig_fail(ctx, IG_EINVAL, "scan: a rotary query source needs the streaming form");
  if (eq) return ig_fail(ctx, IG_EINVAL, "scan: head-equalised lists need the streaming form");
  const bool fused = ig_scan_is_fused(d);
  if (fused) {
    // When all workgroups fit on the chip at once (one round) a wave should have all its channels
    // in flight; with several rounds, smaller blocks leave room for more resident workgroups whose
    // load and select phases then overlap (measured at 1120 workgroups of 2048 tokens: 36.5 us with
    // 40-channel blocks, 33.5-33.9 us = 64-65 % of the HBM peak with 20).
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

// The streaming form (rolling load window, one kernel, pairs split over workgroups when they are
// long) takes half-precision slabs with the kept-channel counts it is built for, where it measured
// faster than the forms below: sequences of up to 8 tiles with enough pairs to fill the chip (no
// split), and every sequence beyond 16 tiles (8 tiles per workgroup, 16 when that would need more
// than IG_SPLIT_MAX workgroups per pair and r <= 32; 4 when there are few pairs, to get more
// workgroups).
bool ig_scan_stream_form(const ig_desc *d, int *tpw, int *S) {
  if (d->dtype != IG_F16 || (d->r != 38 && d->r != 25)) return false;
  const int tile = ig_tile_tokens(d->dtype);
  const int nValid = (d->N + tile - 1) / tile;
  const int BH = d->B * d->H;
  if (nValid <= 4) {
    // one tile per wave: about a tenth faster than the block-loading form up to a few hundred
    // pairs (9.3 against 10.5 us on 256 pairs of 2048 tokens); with a thousand pairs and more the
    // block-loading form with its fewer resident workgroups is ahead (31.8 against 32.8 us)
    if (BH < 128 || BH > 512) return false;
    *tpw = 1;
    *S = 1;
    return true;
  }
  if (nValid <= 8) {
    if (BH < 128) return false;
    *tpw = 2;
    *S = 1;
    return true;
  }
  if (nValid <= 16) return false;
  int t = BH * ((nValid + 7) / 8) >= 512 ? 2 : 1;
  if ((nValid + 4 * t - 1) / (4 * t) > IG_SPLIT_MAX) t = 2;
  if ((nValid + 4 * t - 1) / (4 * t) > IG_SPLIT_MAX) t = 4;
  if ((nValid + 4 * t - 1) / (4 * t) > IG_SPLIT_MAX || (t == 4 && d->r > 32)) return false;
  *tpw = t;
  *S = (nValid + 4 * t - 1) / (4 * t);
  return true;
}

// Shapes whose scan finishes a rotary model's partial query itself (from the full projection's
// split-K sums) instead of reading it from the finalisation kernel: the streaming form with one
// workgroup per pair, heads that fit its prologue.  Where a pair is split over S workgroups every
// one of them would repeat the prologue (S times the work, and 2.5-3 us of latency at the start of
// each): there the query is finished once, by the finalisation kernel, and the scan starts with it
// (measured on 160 pairs of 32768 tokens, S = 8: scan 52.1 -> 49.7 us, the finalisation kernel adds
// 4.8 us including its launch, the projection + scan sequence 65.3 -> 66.7 us).
bool ig_scan_takes_rope(const ig_desc *d) {
  int tpw = 0, S = 0;
  return d->rope && ig_scan_stream_form(d, &tpw, &S) && S == 1 && rope_prologue_fits(256, d->d, d->r);
}

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
  const QSource *rope = q.A_p ? &q : nullptr;
  if (rope && !ig_scan_takes_rope(d)) return ig_fail(ctx, IG_EINVAL, "scan: this shape takes no rotary query source");
  return d->dtype == IG_F16 ? launch_scan<half_t>(ctx, d, a, rope, nullptr, s)
                            : launch_scan<float>(ctx, d, a, rope, nullptr, s);
}

// Shapes whose scan builds the head-equalised lists itself: the streaming form with one
// workgroup per pair (every head's workgroup of a sequence then runs at the same time).
bool ig_scan_equalizes(const ig_desc *d) {
  int tpw = 0, S = 0;
  return ig_scan_stream_form(d, &tpw, &S) && S == 1 && tpw <= 2 && (!d->rope || ig_scan_takes_rope(d));
}

int ig_launch_scan_equalized(ig_ctx *ctx, const ig_desc *d, const QSource &q, const void *slab, int cap,
                             int32_t *sel_idx, int32_t sel_stride, int32_t *sel_cnt, int32_t *thr_cnt_opt,
                             hipStream_t s) {
  if (!ig_scan_equalizes(d)) return ig_fail(ctx, IG_ESHAPE, "scan: this shape does not build equalised lists itself");
  ScanArgs a;
  int rc = ig_scan_args(ctx, d, q, slab, sel_idx, sel_stride, sel_cnt, nullptr, &a);
  if (rc) return rc;
  rc = ig_ensure_zeroed(ctx, &ctx->seq_sync, &ctx->seq_sync_bytes, (size_t)d->B * (d->H + 1) * sizeof(unsigned long long));
  if (rc) return rc;
  EqArgs eq{static_cast<unsigned long long *>(ctx->seq_sync), thr_cnt_opt, cap};
  const QSource *rope = q.A_p ? &q : nullptr;
  return launch_scan<half_t>(ctx, d, a, rope, &eq, s);
}
