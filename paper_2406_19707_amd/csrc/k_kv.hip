// Partial key cache construction (Section 4.3 "Prefill Stage"), prefetch of the selected K/V rows
// (Section 4.1, Section 4.3) and decode attention over the fetched rows (Section 2.1).
#include "ig_internal.h"

namespace {

typedef uint4 u128;

// Store for gathered rows.  Marked non-temporal: written with plain stores, the rows stay dirty in
// the last-level cache and their write-back lands in the next kernels (measured: the following
// partial key cache scan slows from 29 to 35 us on a 159 MB slab); streamed out, it does not.
__device__ __forceinline__ void store_stream(u128 *p, const u128 &v) {
  typedef unsigned int v4u __attribute__((ext_vector_type(4)));
  const v4u t = {v.x, v.y, v.z, v.w};
  __builtin_nontemporal_store(t, reinterpret_cast<v4u *>(p));
}

// ---- slab build ---------------------------------------------------------------------------------
// A workgroup takes 32 consecutive tokens of one (b,h): the full key rows are read coalesced
// (also when the pool is pinned host memory) into LDS, then the r kept channels are written to the
// tile's channel planes, consecutive threads writing consecutive tokens.
template <typename T>
__global__ __launch_bounds__(256) void slab_build(const T *__restrict__ Kpool,
                                                  const int32_t *__restrict__ idx,
                                                  T *__restrict__ slab, int H, int d, int r, int N,
                                                  int N_cap, int nTiles) {
  constexpr int TPL = Elem<T>::TPL;              // elements of a pool row per 16-byte unit
  constexpr int TILE = IG_WAVE * SlabElem<T>::TPL;
  constexpr int CHUNK = 32;
  __shared__ T rows[CHUNK * (256 + 8)];
  const int ldr = d + 8;
  const int bh = blockIdx.y, h = bh % H;
  const int t0 = blockIdx.x * CHUNK;
  const int upr = d / TPL;   // 16-byte units per row (d is a multiple of TPL)
  for (int u = threadIdx.x; u < CHUNK * upr; u += blockDim.x) {
    int tt = u / upr, c = (u % upr) * TPL;
    int t = t0 + tt;
    typename Elem<T>::vec v;
#pragma unroll
    for (int e = 0; e < TPL; ++e) v[e] = (T)0;
    if (t < N) v = *reinterpret_cast<const typename Elem<T>::vec *>(Kpool + ((long)bh * N_cap + t) * d + c);
#pragma unroll
    for (int e = 0; e < TPL; ++e) rows[tt * ldr + c + e] = v[e];
  }
  __syncthreads();
  for (int u = threadIdx.x; u < CHUNK * r; u += blockDim.x) {
    int j = u / CHUNK, tt = u % CHUNK;
    int t = t0 + tt;
    if (t >= nTiles * TILE) continue;
    int tile = t / TILE, tin = t % TILE;
    slab[((long)bh * nTiles + tile) * r * TILE + (long)j * TILE + tin] = rows[tt * ldr + idx[h * r + j]];
  }
}

// ---- append of the token just decoded (Section 2.1: the new key and value join the cache; Section
// 4.4: the matching partial key cache entry is updated with it) -------------------------------------
// One workgroup per (b,h): the K and V rows go to slot `slot` of the pools (16-byte units, device
// or mapped pinned host memory), the r kept channels of the key to the slab's channel planes.
template <typename T>
__global__ __launch_bounds__(64) void append_token(const T *__restrict__ k_new, const T *__restrict__ v_new,
                                                   const int32_t *__restrict__ idx, T *__restrict__ slab,
                                                   u128 *__restrict__ Kpool, u128 *__restrict__ Vpool,
                                                   int H, int d, int r, int N_cap, int nTiles, int slot_all,
                                                   const int32_t *__restrict__ slots,
                                                   int32_t *__restrict__ counters) {
  constexpr int TPL = Elem<T>::TPL;
  constexpr int TILE = IG_WAVE * SlabElem<T>::TPL;
  const int bh = blockIdx.x, h = bh % H;
  // one slot for every pool (append) or the pool's own victim slot (replacement); a slot outside
  // the pool is ignored
  const int slot = slots ? slots[bh] : slot_all;
  if (slot < 0 || slot >= N_cap) return;
  if (counters && threadIdx.x == 0) counters[(long)bh * N_cap + slot] = 0;
  const int U = d / TPL;
  const u128 *kn = reinterpret_cast<const u128 *>(k_new + (long)bh * d);
  const u128 *vn = reinterpret_cast<const u128 *>(v_new + (long)bh * d);
  for (int c = threadIdx.x; c < U; c += 64) {
    Kpool[((long)bh * N_cap + slot) * U + c] = kn[c];
    Vpool[((long)bh * N_cap + slot) * U + c] = vn[c];
  }
  const int tile = slot / TILE, tin = slot % TILE;
  for (int j = threadIdx.x; j < r; j += 64)
    slab[((long)bh * nTiles + tile) * r * TILE + (long)j * TILE + tin] = k_new[(long)bh * d + idx[h * r + j]];
}

// ---- pool counters (Section 4.4, counter-based victim selection) ------------------------------------
// One workgroup per (b,h) pool.  touch: +1 (saturating) on the counter of every prefetched slot; a
// list holds a slot once, so plain stores suffice; if a counter reached the saturation value, all
// counters of the pool are halved after the increments.  victim: the slot with the smallest count
// among the N valid ones, the lowest slot on ties (minimum over count * 2^32 + slot).
__global__ __launch_bounds__(256) void pool_touch(const int32_t *__restrict__ sel_idx,
                                                  const int32_t *__restrict__ sel_cnt,
                                                  int32_t *__restrict__ counters, int stride, int N,
                                                  int N_cap, int counter_max) {
  const int bh = blockIdx.x;
  int32_t *c = counters + (long)bh * N_cap;
  const int n = min(sel_cnt[bh], stride);
  int sat = 0;
  for (int j = threadIdx.x; j < n; j += 256) {
    const int t = sel_idx[(long)bh * stride + j];
    if (t >= 0 && t < N) {
      const int v = min(c[t] + 1, counter_max);
      c[t] = v;
      sat |= v >= counter_max;
    }
  }
  if (__syncthreads_or(sat))
    for (int t = threadIdx.x; t < N; t += 256) c[t] >>= 1;
}

__global__ __launch_bounds__(256) void pool_victim(const int32_t *__restrict__ counters,
                                                   int32_t *__restrict__ victim, int N, int N_cap) {
  __shared__ unsigned long long best[4];
  const int bh = blockIdx.x, lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int32_t *c = counters + (long)bh * N_cap;
  unsigned long long m = ~0ull;
  for (int t = threadIdx.x; t < N; t += 256) {
    const unsigned long long key = ((unsigned long long)(unsigned)c[t] << 32) | (unsigned)t;
    m = key < m ? key : m;
  }
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) {
    const unsigned long long u = __shfl_xor(m, o, 64);
    m = u < m ? u : m;
  }
  if (lane == 0) best[w] = m;
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int k = 1; k < 4; ++k) m = best[k] < m ? best[k] : m;
    victim[bh] = (int32_t)(m & 0xFFFFFFFFull);
  }
}

// ---- work split shared by gather and attention --------------------------------------------------
// Selected-token lists are very uneven (a few heads keep a thousand rows, most a few dozen), and
// one compute unit moves well under 100 GB/s, so a list is cut into up to SLICE_MAX slices of at
// most SLICE_ROWS rows where possible: slices = min(SLICE_MAX, ceil(rows / SLICE_ROWS)), slice s
// covering rows [rows*s/slices, rows*(s+1)/slices).  Every workgroup derives this from the
// device-side count, so the host never reads the counts; surplus workgroups leave at once.
//
// Workgroups are handed to the 8 XCDs round-robin by linear id, and an XCD reaches only about an
// eighth of the HBM bandwidth, so the work has to be even per XCD, not just per compute unit:
// heavy lists cluster by head (and H is normally a multiple of 8), so mapping (b,h) -> id = b*H+h
// would send every slice of the heavy heads to the same XCD.  work_item() therefore decodes the
// linear id as slice = id / BH, t = id % BH, b = t / H, h = (t % H - b - 5*slice) mod H, which puts
// (b, h, slice) on XCD (h + b + 5*slice) % 8: the slices of one list, the sequences of one head and
// the heads of one sequence are each spread over all XCDs.
constexpr int SLICE_ROWS = 128;
constexpr int SLICE_MAX = IG_SLICE_MAX;
__device__ __forceinline__ void work_item(int H, int BH, int *bh, int *slice) {
  const int id = blockIdx.x;
  const int s = id / BH, t = id - s * BH;
  const int b = t / H;
  int h = (t - b * H - b - 5 * s) % H;
  if (h < 0) h += H;
  *bh = b * H + h;
  *slice = s;
}
__device__ __forceinline__ bool slice_range(int rows, int s, int max_slices, int *row0, int *row1, int *slices) {
  int n = (rows + SLICE_ROWS - 1) / SLICE_ROWS;
  n = max(1, min(n, max_slices));
  *slices = n;
  if (s >= n) return false;
  *row0 = (int)((long)rows * s / n);
  *row1 = (int)((long)rows * (s + 1) / n);
  return true;
}

// ---- gather, device-resident pool ---------------------------------------------------------------
// Row copies in 16-byte units, U units per row; grid B*H*SLICE_MAX (see work_item).  A thread's copies are
// issued in batches of GATHER_BATCH, so that index loads, then K and V row loads, are in flight
// together.
constexpr int GATHER_BATCH = 8;
__global__ __launch_bounds__(256) void gather_rows_sliced(
    const u128 *__restrict__ Kpool, const u128 *__restrict__ Vpool, const int32_t *__restrict__ sel_idx,
    const int32_t *__restrict__ sel_cnt, u128 *__restrict__ K_sel, u128 *__restrict__ V_sel, int N_cap,
    int stride, int U, int H, int BH) {
  int bh, slice;
  work_item(H, BH, &bh, &slice);
  const int cnt = min(sel_cnt[bh], stride);
  int row0, row1, slices;
  if (!slice_range(cnt, slice, SLICE_MAX, &row0, &row1, &slices) || row1 <= row0) return;
  const int32_t *list = sel_idx + (long)bh * stride + row0;
  const long src0 = (long)bh * N_cap * U, dst0 = ((long)bh * stride + row0) * U;
  const int total = (row1 - row0) * U;
  // Branch-free batches (so that all loads of a batch are issued before the first store): a unit
  // past the end is clamped to the last unit, which is then copied more than once with identical
  // bytes.
  for (int u0 = threadIdx.x; u0 < total; u0 += 256 * GATHER_BATCH) {
    u128 kv[GATHER_BATCH], vv[GATHER_BATCH];
    long src[GATHER_BATCH];
#pragma unroll
    for (int i = 0; i < GATHER_BATCH; ++i) {
      const int u = min(u0 + 256 * i, total - 1);
      const int rr = u / U, c = u - rr * U;
      src[i] = src0 + (long)list[rr] * U + c;
    }
#pragma unroll
    for (int i = 0; i < GATHER_BATCH; ++i) {
      kv[i] = Kpool[src[i]];
      vv[i] = Vpool[src[i]];
    }
#pragma unroll
    for (int i = 0; i < GATHER_BATCH; ++i) {
      const int u = min(u0 + 256 * i, total - 1);
      store_stream(K_sel + dst0 + u, kv[i]);
      store_stream(V_sel + dst0 + u, vv[i]);
    }
  }
}

// ---- gather, pinned-host pool --------------------------------------------------------------------
// The rows of all lists are treated as one flat sequence and cut into equal ranges, one per
// workgroup: every workgroup reads the B*H counts (one coalesced read), builds their prefix sum in
// LDS, takes rows [T*g/G, T*(g+1)/G) of the T selected rows and finds the list of each row by
// binary search in the prefix array.  The split is therefore even whatever the skew of the list
// lengths, consecutive workgroups (which go to different XCDs) take consecutive ranges, the grid
// is fixed, and the host never reads a count.  Row copies are in 16-byte units, U units per row;
// a thread's copies are issued in branch-free batches of GATHER_BATCH (index loads, then K and V
// row loads, all in flight before the first store).  For a pinned-host pool the grid is kept
// small: a hundred workgroups keep more than enough PCIe reads outstanding, and the compute units
// stay free for the kernels of the other stream, which stalled rows would otherwise block.
constexpr int GATHER_MIN_ROWS = 32;   // a workgroup takes at least this many rows (when there are that many)
template <int THREADS, int BATCH>
__global__ __launch_bounds__(THREADS) void gather_rows_flat(
    const u128 *__restrict__ Kpool, const u128 *__restrict__ Vpool, const int32_t *__restrict__ sel_idx,
    const int32_t *__restrict__ sel_cnt, u128 *__restrict__ K_sel, u128 *__restrict__ V_sel, int N_cap,
    int stride, int U, int BH) {
  extern __shared__ int pre[];          // pre[i] = rows of lists 0..i-1, i <= BH
  constexpr int WAVES = THREADS / 64;
  __shared__ int wave_tot[WAVES];
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  // inclusive prefix sum of the clamped counts: each thread owns a run of consecutive lists
  const int per = (BH + THREADS - 1) / THREADS;
  const int i0 = tid * per;
  int run = 0;
  for (int i = i0; i < min(BH, i0 + per); ++i) {
    run += min(sel_cnt[i], stride);
    pre[i + 1] = run;                    // local to the thread's run for now
  }
  int incl = wave_incl_scan(run, lane);
  if (lane == 63) wave_tot[w] = incl;
  __syncthreads();
  int offset = incl - run;
  for (int k = 0; k < w; ++k) offset += wave_tot[k];
  for (int i = i0; i < min(BH, i0 + per); ++i) pre[i + 1] += offset;
  if (tid == 0) pre[0] = 0;
  __syncthreads();
  const long T = pre[BH];
  const int G = gridDim.x, g = blockIdx.x;
  long per_wg = (T + G - 1) / G;
  if (per_wg < GATHER_MIN_ROWS) per_wg = GATHER_MIN_ROWS;
  const long r0 = (long)g * per_wg, r1 = min(T, r0 + per_wg);
  if (r0 >= r1) return;
  const long total = (r1 - r0) * U;
  int top = 1;
  while (top * 2 < BH) top *= 2;
  for (long u0 = tid; u0 < total; u0 += THREADS * BATCH) {
    u128 kv[BATCH], vv[BATCH];
    long src[BATCH], dst[BATCH];
#pragma unroll
    for (int i = 0; i < BATCH; ++i) {
      const long u = min(u0 + THREADS * i, total - 1);   // past the end: the last unit again (same bytes)
      const int row = (int)(r0 + u / U), c = (int)(u % U);
      // list of this row: the last bh with pre[bh] <= row (fixed trip count, so the searches of a
      // batch interleave)
      int lo = 0;
      for (int step = top; step >= 1; step >>= 1) {
        const int cand = lo + step;
        if (cand < BH && pre[cand] <= row) lo = cand;
      }
      const int j = row - pre[lo];
      const long t = sel_idx[(long)lo * stride + j];
      src[i] = ((long)lo * N_cap + t) * U + c;
      dst[i] = ((long)lo * stride + j) * U + c;
    }
#pragma unroll
    for (int i = 0; i < BATCH; ++i) {
      kv[i] = Kpool[src[i]];
      vv[i] = Vpool[src[i]];
    }
#pragma unroll
    for (int i = 0; i < BATCH; ++i) {
      K_sel[dst[i]] = kv[i];             // plain stores: with a pinned-host pool the streamed form
      V_sel[dst[i]] = vv[i];             // measured slower (pipelined step 1107 vs 1083 us per layer)
    }
  }
}

// ---- attention ----------------------------------------------------------------------------------
// grid B*H*SLICE_MAX (see work_item), 4 waves per workgroup, one slice of the (b,h) list each.  A row of d
// elements is covered by LPR = d*sizeof(T)/16 lanes, 16 bytes each, so a wave step covers 64/LPR
// rows; waves interleave over the rows, and steps are issued in batches of ATT_BATCH so that a
// batch's K and V loads are all in flight before the first is used.  Every lane group keeps an
// online-softmax state (running max, normaliser, weighted sum for its 16-byte slice of V); states
// are merged across lane groups with shuffles and across waves through LDS, in a fixed order.
//
// A list with one slice writes its output directly.  With several slices each workgroup publishes
// its state (max, normaliser, d sums) with device-coherent stores and bumps a per-(b,h) counter;
// the workgroup that arrives last reads all states with device-coherent loads and merges them in
// slice order, so the result does not depend on arrival order.  Coherent stores and loads are used
// instead of a device-wide fence, which would write back and invalidate the whole L2 per
// workgroup.  The counter is left at zero for the next call.
constexpr int ATT_BATCH = 8;

template <typename T> __device__ __forceinline__ void to_float(const u128 &raw, float (&f)[Elem<T>::TPL]);
template <> __device__ __forceinline__ void to_float<half_t>(const u128 &raw, float (&f)[8]) {
  const half8 h = *reinterpret_cast<const half8 *>(&raw);
#pragma unroll
  for (int e = 0; e < 8; ++e) f[e] = (float)h[e];
}
template <> __device__ __forceinline__ void to_float<float>(const u128 &raw, float (&f)[4]) {
  const floatx4 v = *reinterpret_cast<const floatx4 *>(&raw);
#pragma unroll
  for (int e = 0; e < 4; ++e) f[e] = v[e];
}

__device__ __forceinline__ float exp_or_zero(float m, float M) { return (m == -INFINITY) ? 0.f : __expf(m - M); }
__device__ __forceinline__ void coherent_store(float *p, float v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float coherent_load(const float *p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

template <typename T, bool INDEXED>
__global__ __launch_bounds__(256) void sparse_attention(
    const T *__restrict__ q, const u128 *__restrict__ K, const u128 *__restrict__ V,
    const int32_t *__restrict__ sel_idx, const int32_t *__restrict__ sel_cnt, int stride, int kv_rows,
    int LPR, const T *__restrict__ k_new, const T *__restrict__ v_new, T *__restrict__ out, float scale,
    int d, float *part, int32_t *counters, int H, int BH, u128 *__restrict__ K_out,
    u128 *__restrict__ V_out) {
  constexpr int TPL = Elem<T>::TPL;
  __shared__ float sm[4], sz[4];
  __shared__ float sacc[4][512];
  __shared__ int s_last;
  constexpr int max_slices = SLICE_MAX;
  int bh, slice;
  work_item(H, BH, &bh, &slice);
  const int n = min(sel_cnt[bh], stride);
  const int rows = n + (k_new ? 1 : 0);
  int row0 = 0, row1 = 0, slices = 1;
  if (!slice_range(rows, slice, max_slices, &row0, &row1, &slices)) return;
  const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int RPW = 64 / LPR;            // rows per wave step
  const int sub = lane / LPR, li = lane % LPR;
  float qf[TPL];
  {
    u128 raw = *reinterpret_cast<const u128 *>(q + (long)bh * d + li * TPL);
    to_float<T>(raw, qf);
#pragma unroll
    for (int e = 0; e < TPL; ++e) qf[e] *= scale;
  }
  float m = -INFINITY, z = 0.f, acc[TPL];
#pragma unroll
  for (int e = 0; e < TPL; ++e) acc[e] = 0.f;
  const long base = (long)bh * kv_rows * LPR;
  const int32_t *list = sel_idx + (long)bh * stride;
  const int rows_per_batch = 4 * RPW * ATT_BATCH;
  // Fused prefetch (K_out): the rows read from the pool are also the rows ig_gather_kv would copy.
  // With several slices the row stores of a slice's last batch are held back until the slice has
  // published its softmax state, so that the wait for that publication does not also wait for
  // 64 KiB of row stores to be acknowledged; they then travel while the counter round trip and
  // the final merge are under way.
  const bool fuse_store = INDEXED && K_out != nullptr;
  const bool defer = fuse_store && slices > 1;
  u128 kr[ATT_BATCH], vr[ATT_BATCH];
  int r_keep = -1;                       // first row of the batch whose stores are held back
  auto store_rows = [&](int r0) {
#pragma unroll
    for (int i = 0; i < ATT_BATCH; ++i) {
      const int j = r0 + (i * 4 + w) * RPW + sub;
      if (j < row1 && j < n) {
        const long o = ((long)bh * stride + j) * LPR + li;
        store_stream(K_out + o, kr[i]);
        store_stream(V_out + o, vr[i]);
      }
    }
  };
  for (int r0 = row0; r0 < row1; r0 += rows_per_batch) {
    // Branch-free loads, so that the whole batch is in flight at once: a step past the slice's end
    // re-reads the slice's last row and its logit is masked below; the new-token row is a pointer
    // select, not a branch.
    bool valid[ATT_BATCH];
    long rowoff[ATT_BATCH];
#pragma unroll
    for (int i = 0; i < ATT_BATCH; ++i) {
      // step i of wave w covers rows r0 + (i*4 + w)*RPW + sub
      const int j = r0 + (i * 4 + w) * RPW + sub;
      valid[i] = j < row1;
      const int jc = min(j, row1 - 1);
      const int jl = min(jc, max(n - 1, 0));
      rowoff[i] = INDEXED ? (long)list[jl] : (long)jl;
    }
#pragma unroll
    for (int i = 0; i < ATT_BATCH; ++i) {
      const int j = r0 + (i * 4 + w) * RPW + sub;
      const bool cached = min(j, row1 - 1) < n;
      const u128 *kp = cached ? K + base + rowoff[i] * LPR + li : reinterpret_cast<const u128 *>(k_new + (long)bh * d) + li;
      const u128 *vp = cached ? V + base + rowoff[i] * LPR + li : reinterpret_cast<const u128 *>(v_new + (long)bh * d) + li;
      kr[i] = *kp;
      vr[i] = *vp;
    }
    if (fuse_store) {
      if (defer && r0 + rows_per_batch >= row1) r_keep = r0;
      else store_rows(r0);
    }
    float l[ATT_BATCH];
    float bm = m;
#pragma unroll
    for (int i = 0; i < ATT_BATCH; ++i) {
      float kf[TPL];
      to_float<T>(kr[i], kf);
      float t = 0.f;
#pragma unroll
      for (int e = 0; e < TPL; ++e) t = fmaf(qf[e], kf[e], t);
      if (LPR == 16) {
        t = row16_sum(t);
      } else {
        for (int o = 1; o < LPR; o <<= 1) t += __shfl_xor(t, o, 64);
      }
      l[i] = valid[i] ? t : -INFINITY;
      bm = fmaxf(bm, l[i]);
    }
    if (bm != -INFINITY) {
      const float f = exp_or_zero(m, bm);
      z *= f;
#pragma unroll
      for (int e = 0; e < TPL; ++e) acc[e] *= f;
#pragma unroll
      for (int i = 0; i < ATT_BATCH; ++i) {
        const float p = exp_or_zero(l[i], bm);
        float vf[TPL];
        to_float<T>(vr[i], vf);
        z += p;
#pragma unroll
        for (int e = 0; e < TPL; ++e) acc[e] = fmaf(p, vf[e], acc[e]);
      }
      m = bm;
    }
  }
  // merge the lane groups of the wave (lanes with equal li hold the same slice of V)
  for (int o = LPR; o < 64; o <<= 1) {
    const float m2 = __shfl_xor(m, o, 64), z2 = __shfl_xor(z, o, 64);
    const float M = fmaxf(m, m2);
    const float f1 = exp_or_zero(m, M), f2 = exp_or_zero(m2, M);
    z = z * f1 + z2 * f2;
#pragma unroll
    for (int e = 0; e < TPL; ++e) acc[e] = acc[e] * f1 + __shfl_xor(acc[e], o, 64) * f2;
    m = M;
  }
  if (lane < LPR) {
    if (lane == 0) { sm[w] = m; sz[w] = z; }
#pragma unroll
    for (int e = 0; e < TPL; ++e) sacc[w][lane * TPL + e] = acc[e];
  }
  __syncthreads();
  // merge the four waves: thread c owns output channel c
  const float M = fmaxf(fmaxf(sm[0], sm[1]), fmaxf(sm[2], sm[3]));
  float zc = 0.f;
#pragma unroll
  for (int k = 0; k < 4; ++k) zc += sz[k] * exp_or_zero(sm[k], M);
  if (slices == 1) {
    for (int c = threadIdx.x; c < d; c += 256) {
      float a = 0.f;
#pragma unroll
      for (int k = 0; k < 4; ++k) a += sacc[k][c] * exp_or_zero(sm[k], M);
      out[(long)bh * d + c] = (T)(zc > 0.f ? a / zc : 0.f);
    }
    return;
  }
  // several slices: publish this slice's state; the last arrival merges all of them
  float *mine = part + ((long)bh * max_slices + slice) * (d + 2);
  for (int c = threadIdx.x; c < d; c += 256) {
    float a = 0.f;
#pragma unroll
    for (int k = 0; k < 4; ++k) a += sacc[k][c] * exp_or_zero(sm[k], M);
    coherent_store(mine + 2 + c, a);
  }
  if (threadIdx.x == 0) {
    coherent_store(mine, M);
    coherent_store(mine + 1, zc);
  }
  // wait until this wave's coherent stores have been acknowledged, then meet the other waves
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  // held-back row stores: waves 1..3 issue theirs now; wave 0, which waits for the counter and does
  // the final merge, issues its own only when it has nothing left to wait for
  if (w != 0 && r_keep >= 0) store_rows(r_keep);
  if (threadIdx.x == 0) {
    const int prev = __hip_atomic_fetch_add(&counters[bh], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    s_last = (prev == slices - 1);
    if (s_last) __hip_atomic_store(&counters[bh], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  __syncthreads();
  if (w != 0) return;
  if (s_last) {
    // wave 0 of the last arrival: lane c owns output channels c, c + 64, ...; all loads of a pass
    // (independent, predicated on the slice count) are issued before any is used
    const float *all = part + (long)bh * max_slices * (d + 2);
    float mk[SLICE_MAX], zk[SLICE_MAX];
#pragma unroll
    for (int k = 0; k < SLICE_MAX; ++k) {
      mk[k] = -INFINITY;
      zk[k] = 0.f;
      if (k < slices) {
        mk[k] = coherent_load(all + (long)k * (d + 2));
        zk[k] = coherent_load(all + (long)k * (d + 2) + 1);
      }
    }
    constexpr int CPP = 2;               // channels per lane and pass
    for (int c0 = lane; c0 < d; c0 += 64 * CPP) {
      float ak[CPP][SLICE_MAX];
#pragma unroll
      for (int q = 0; q < CPP; ++q)
#pragma unroll
        for (int k = 0; k < SLICE_MAX; ++k) {
          const int c = c0 + 64 * q;
          ak[q][k] = (k < slices && c < d) ? coherent_load(all + (long)k * (d + 2) + 2 + c) : 0.f;
        }
      float MM = -INFINITY;
#pragma unroll
      for (int k = 0; k < SLICE_MAX; ++k) MM = fmaxf(MM, mk[k]);
      float zz = 0.f;
#pragma unroll
      for (int k = 0; k < SLICE_MAX; ++k) zz += zk[k] * exp_or_zero(mk[k], MM);
#pragma unroll
      for (int q = 0; q < CPP; ++q) {
        const int c = c0 + 64 * q;
        float a = 0.f;
#pragma unroll
        for (int k = 0; k < SLICE_MAX; ++k) a += ak[q][k] * exp_or_zero(mk[k], MM);
        if (c < d) out[(long)bh * d + c] = (T)(zz > 0.f ? a / zz : 0.f);
      }
    }
  }
  if (r_keep >= 0) store_rows(r_keep);
}

__global__ __launch_bounds__(256) void copy_bytes(const u128 *__restrict__ src, u128 *__restrict__ dst,
                                                  long n16) {
  long i = (long)blockIdx.x * 256 + threadIdx.x;
  const long step = (long)gridDim.x * 256;
  for (; i < n16; i += step) dst[i] = src[i];
}

// Plain streaming read: a wave reads 8 consecutive KiB (16 bytes per lane and load) and folds them;
// the result is stored only if it equals a value it practically never takes, so the loads stay.
__global__ __launch_bounds__(256) void read_bytes(const u128 *__restrict__ src, long n16,
                                                  unsigned *__restrict__ sink) {
  const long wave = ((long)blockIdx.x * 256 + threadIdx.x) >> 6;
  const int lane = threadIdx.x & 63;
  const long base = wave * 512 + lane;
  u128 v[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) v[i] = src[min(base + 64L * i, n16 - 1)];
  unsigned x = 0;
#pragma unroll
  for (int i = 0; i < 8; ++i) x ^= v[i].x ^ v[i].y ^ v[i].z ^ v[i].w;
  if (x == 0x9e3779b9u) sink[0] = x;
}

}  // namespace

int ig_launch_read(ig_ctx *ctx, const void *src, size_t bytes, hipStream_t s) {
  const long n16 = (long)(bytes / 16);
  const long waves = (n16 + 511) / 512;
  auto k = read_bytes;
  IG_LAUNCH(ctx, IG_K_READ, k, dim3((unsigned)((waves + 3) / 4)), dim3(256), s, (const u128 *)src, n16,
            (unsigned *)(ctx->status + 8));
  return IG_OK;
}

int ig_launch_slab_build(ig_ctx *ctx, const ig_desc *d, const void *Kpool, const int32_t *idx,
                         void *slab, hipStream_t s) {
  const int tile = ig_tile_tokens(d->dtype);
  const int nTiles = (d->N_cap + tile - 1) / tile;
  if (d->d > 256) return ig_fail(ctx, IG_ESHAPE, "slab build: d = %d exceeds 256", d->d);
  dim3 grid((nTiles * tile + 31) / 32, d->B * d->H), block(256);
  if (d->dtype == IG_F16) {
    auto k = slab_build<half_t>;
    IG_LAUNCH(ctx, IG_K_BUILD, k, grid, block, s, (const half_t *)Kpool, idx, (half_t *)slab,
              (int)d->H, (int)d->d, (int)d->r, (int)d->N, (int)d->N_cap, nTiles);
  } else {
    auto k = slab_build<float>;
    IG_LAUNCH(ctx, IG_K_BUILD, k, grid, block, s, (const float *)Kpool, idx, (float *)slab,
              (int)d->H, (int)d->d, (int)d->r, (int)d->N, (int)d->N_cap, nTiles);
  }
  return IG_OK;
}

int ig_launch_append(ig_ctx *ctx, const ig_desc *d, const void *k_new, const void *v_new,
                     const int32_t *idx, void *slab, void *Kpool, void *Vpool,
                     const int32_t *slots, int32_t *counters, hipStream_t s) {
  const int tile = ig_tile_tokens(d->dtype);
  const int nTiles = (d->N_cap + tile - 1) / tile;
  dim3 grid(d->B * d->H), block(64);
  if (d->dtype == IG_F16) {
    auto k = append_token<half_t>;
    IG_LAUNCH(ctx, IG_K_BUILD, k, grid, block, s, (const half_t *)k_new, (const half_t *)v_new, idx,
              (half_t *)slab, (u128 *)Kpool, (u128 *)Vpool, (int)d->H, (int)d->d, (int)d->r,
              (int)d->N_cap, nTiles, (int)d->N, slots, counters);
  } else {
    auto k = append_token<float>;
    IG_LAUNCH(ctx, IG_K_BUILD, k, grid, block, s, (const float *)k_new, (const float *)v_new, idx,
              (float *)slab, (u128 *)Kpool, (u128 *)Vpool, (int)d->H, (int)d->d, (int)d->r,
              (int)d->N_cap, nTiles, (int)d->N, slots, counters);
  }
  return IG_OK;
}

int ig_launch_pool_touch(ig_ctx *ctx, const ig_desc *d, const int32_t *sel_idx, int32_t sel_stride,
                         const int32_t *sel_cnt, int32_t *counters, int counter_max, hipStream_t s) {
  auto k = pool_touch;
  IG_LAUNCH(ctx, IG_K_BUILD, k, dim3(d->B * d->H), dim3(256), s, sel_idx, sel_cnt, counters,
            (int)sel_stride, (int)d->N, (int)d->N_cap, counter_max);
  return IG_OK;
}

int ig_launch_pool_victim(ig_ctx *ctx, const ig_desc *d, const int32_t *counters, int32_t *victim,
                          hipStream_t s) {
  auto k = pool_victim;
  IG_LAUNCH(ctx, IG_K_BUILD, k, dim3(d->B * d->H), dim3(256), s, counters, victim, (int)d->N,
            (int)d->N_cap);
  return IG_OK;
}

int ig_launch_gather(ig_ctx *ctx, const ig_desc *d, const void *Kpool, const void *Vpool,
                     const int32_t *sel_idx, int32_t sel_stride, const int32_t *sel_cnt,
                     void *K_sel, void *V_sel, int host_pool, hipStream_t s) {
  const int U = d->d * ig_elem_bytes(d->dtype) / 16;
  const int BH = d->B * d->H;
  if (!host_pool) {
    dim3 grid(BH * SLICE_MAX), block(256);
    auto k = gather_rows_sliced;
    IG_LAUNCH(ctx, IG_K_GATHER, k, grid, block, s, (const u128 *)Kpool, (const u128 *)Vpool, sel_idx,
              sel_cnt, (u128 *)K_sel, (u128 *)V_sel, (int)d->N_cap, (int)sel_stride, U, (int)d->H, BH);
    return IG_OK;
  }
  const size_t lds = (size_t)(BH + 1) * sizeof(int);
  if (lds > 60 * 1024) return ig_fail(ctx, IG_ESHAPE, "host gather: B*H = %d exceeds %d", BH, 60 * 256 - 1);
  int wgs = 128, threads = 256, batch = 8;
  dim3 grid(wgs), block(threads);
#define HG_CASE(TH, BA)                                                                              \
  if (threads == TH && batch == BA) {                                                               \
    auto k = gather_rows_flat<TH, BA>;                                                              \
    if (ctx->profiling) {                                                                           \
      hipEvent_t e0, e1;                                                                            \
      ig_prof_events(ctx, IG_K_GATHER, &e0, &e1);                                                   \
      hipExtLaunchKernelGGL(k, grid, block, (unsigned)lds, s, e0, e1, 0, (const u128 *)Kpool,       \
                            (const u128 *)Vpool, sel_idx, sel_cnt, (u128 *)K_sel, (u128 *)V_sel,   \
                            (int)d->N_cap, (int)sel_stride, U, BH);                                 \
    } else {                                                                                        \
      hipLaunchKernelGGL(k, grid, block, (unsigned)lds, s, (const u128 *)Kpool, (const u128 *)Vpool, \
                         sel_idx, sel_cnt, (u128 *)K_sel, (u128 *)V_sel, (int)d->N_cap,             \
                         (int)sel_stride, U, BH);                                                   \
    }                                                                                               \
    hipError_t le = hipGetLastError();                                                              \
    if (le != hipSuccess) return ig_hip_fail(ctx, le, "gather_rows_flat");                          \
    return IG_OK;                                                                                   \
  }
  HG_CASE(256, 8)
#undef HG_CASE
  return ig_fail(ctx, IG_ESHAPE, "host gather: unsupported launch shape");
}

template <typename T>
static int launch_attention_t(ig_ctx *ctx, const ig_desc *d, const void *q, const void *K,
                              const void *V, const int32_t *sel_idx, int32_t sel_stride,
                              const int32_t *sel_cnt, int kv_rows, const void *k_new,
                              const void *v_new, void *out, void *K_out, void *V_out, hipStream_t s) {
  const int LPR = d->d * (int)sizeof(T) / 16;
  const int BH = d->B * d->H;
  int rc = ig_ensure(ctx, (void **)&ctx->attn_part, &ctx->attn_part_bytes,
                     (size_t)BH * SLICE_MAX * (d->d + 2) * sizeof(float));
  if (rc) return rc;
  if ((rc = ig_ensure_zeroed(ctx, (void **)&ctx->attn_cnt, &ctx->attn_cnt_bytes, (size_t)BH * sizeof(int32_t))))
    return rc;
  dim3 grid(BH * SLICE_MAX), block(256);
  if (sel_idx) {
    auto k = sparse_attention<T, true>;
    IG_LAUNCH(ctx, IG_K_ATTENTION, k, grid, block, s, (const T *)q, (const u128 *)K, (const u128 *)V,
              sel_idx, sel_cnt, (int)sel_stride, kv_rows, LPR, (const T *)k_new, (const T *)v_new,
              (T *)out, (float)d->scale, (int)d->d, ctx->attn_part, ctx->attn_cnt, (int)d->H, BH,
              (u128 *)K_out, (u128 *)V_out);
  } else {
    auto k = sparse_attention<T, false>;
    IG_LAUNCH(ctx, IG_K_ATTENTION, k, grid, block, s, (const T *)q, (const u128 *)K, (const u128 *)V,
              sel_idx, sel_cnt, (int)sel_stride, kv_rows, LPR, (const T *)k_new, (const T *)v_new,
              (T *)out, (float)d->scale, (int)d->d, ctx->attn_part, ctx->attn_cnt, (int)d->H, BH,
              (u128 *)nullptr, (u128 *)nullptr);
  }
  return IG_OK;
}

int ig_launch_attention(ig_ctx *ctx, const ig_desc *d, const void *q, const void *K, const void *V,
                        const int32_t *sel_idx, int32_t sel_stride, const int32_t *sel_cnt,
                        int kv_rows_per_bh, const void *k_new, const void *v_new, void *out,
                        void *K_out, void *V_out, hipStream_t s) {
  const int row_bytes = d->d * ig_elem_bytes(d->dtype);
  const int LPR = row_bytes / 16;
  if (row_bytes % 16 || LPR < 1 || LPR > 64 || (LPR & (LPR - 1)))
    return ig_fail(ctx, IG_ESHAPE, "attention: row of %d bytes must be 16 * 2^k bytes, at most 1024",
                   row_bytes);
  return d->dtype == IG_F16
             ? launch_attention_t<half_t>(ctx, d, q, K, V, sel_idx, sel_stride, sel_cnt,
                                          kv_rows_per_bh, k_new, v_new, out, K_out, V_out, s)
             : launch_attention_t<float>(ctx, d, q, K, V, sel_idx, sel_stride, sel_cnt,
                                         kv_rows_per_bh, k_new, v_new, out, K_out, V_out, s);
}

int ig_launch_copy(ig_ctx *ctx, const void *src, void *dst, size_t bytes, hipStream_t s) {
  long n16 = (long)(bytes / 16);
  long blocks = (n16 + 255) / 256;
  if (blocks > 16384) blocks = 16384;
  if (blocks < 1) blocks = 1;
  auto k = copy_bytes;
  IG_LAUNCH(ctx, IG_K_COPY, k, dim3((unsigned)blocks), dim3(256), s, (const u128 *)src, (u128 *)dst,
            n16);
  return IG_OK;
}
