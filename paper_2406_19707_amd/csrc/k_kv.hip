// Partial key cache construction (Section 4.3 "Prefill Stage"), prefetch of the selected K/V rows
// (Section 4.1, Section 4.3) and decode attention over the fetched rows (Section 2.1).
#include "attn_device.h"

namespace {

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
    const int col = min(max(idx[h * r + j], 0), d - 1);     // an index outside the head is clamped, never followed
    slab[((long)bh * nTiles + tile) * r * TILE + (long)j * TILE + tin] = rows[tt * ldr + col];
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
                                                   int32_t *__restrict__ counters, int32_t restart) {
  constexpr int TPL = Elem<T>::TPL;
  constexpr int TILE = IG_WAVE * SlabElem<T>::TPL;
  const int bh = blockIdx.x, h = bh % H;
  // one slot for every pool (append) or the pool's own victim slot (replacement); a slot outside
  // the pool is ignored
  const int slot = slots ? slots[bh] : slot_all;
  if (slot < 0 || slot >= N_cap) return;
  if (counters && threadIdx.x == 0) counters[(long)bh * N_cap + slot] = restart;   // policy state of the new entry
  const int U = d / TPL;
  const u128 *kn = reinterpret_cast<const u128 *>(k_new + (long)bh * d);
  const u128 *vn = reinterpret_cast<const u128 *>(v_new + (long)bh * d);
  for (int c = threadIdx.x; c < U; c += 64) {
    Kpool[((long)bh * N_cap + slot) * U + c] = kn[c];
    Vpool[((long)bh * N_cap + slot) * U + c] = vn[c];
  }
  const int tile = slot / TILE, tin = slot % TILE;
  for (int j = threadIdx.x; j < r; j += 64)
    slab[((long)bh * nTiles + tile) * r * TILE + (long)j * TILE + tin] =
        k_new[(long)bh * d + min(max(idx[h * r + j], 0), d - 1)];
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

// LRU comparison policy (Section 4.4, Table 2): the last-use stamp of every prefetched slot becomes
// `now`; the victim kernel below then names the slot whose last use lies furthest back.
__global__ __launch_bounds__(256) void pool_touch_lru(const int32_t *__restrict__ sel_idx,
                                                      const int32_t *__restrict__ sel_cnt,
                                                      int32_t *__restrict__ stamps, int stride, int N,
                                                      int N_cap, int32_t now) {
  const int bh = blockIdx.x;
  const int n = min(sel_cnt[bh], stride);
  for (int j = threadIdx.x; j < n; j += 256) {
    const int t = sel_idx[(long)bh * stride + j];
    if (t >= 0 && t < N) stamps[(long)bh * N_cap + t] = now;
  }
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
  work_item(blockIdx.x, H, BH, &bh, &slice);
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
      src[i] = src0 + (long)min(max(list[rr], 0), N_cap - 1) * U + c;   // a slot outside the pool is clamped
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
      const long t = min(max(sel_idx[(long)lo * stride + j], 0), N_cap - 1);   // a slot outside the pool is clamped
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

// ---- attention (body in attn_device.h) ----------------------------------------------------------
template <typename T, bool INDEXED>
__global__ __launch_bounds__(256) void sparse_attention(AttnArgs A) {
  sparse_attention_body<T, INDEXED>(A, blockIdx.x);
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
                     const int32_t *slots, int32_t *counters, int32_t restart, hipStream_t s) {
  const int tile = ig_tile_tokens(d->dtype);
  const int nTiles = (d->N_cap + tile - 1) / tile;
  dim3 grid(d->B * d->H), block(64);
  if (d->dtype == IG_F16) {
    auto k = append_token<half_t>;
    IG_LAUNCH(ctx, IG_K_BUILD, k, grid, block, s, (const half_t *)k_new, (const half_t *)v_new, idx,
              (half_t *)slab, (u128 *)Kpool, (u128 *)Vpool, (int)d->H, (int)d->d, (int)d->r,
              (int)d->N_cap, nTiles, (int)d->N, slots, counters, restart);
  } else {
    auto k = append_token<float>;
    IG_LAUNCH(ctx, IG_K_BUILD, k, grid, block, s, (const float *)k_new, (const float *)v_new, idx,
              (float *)slab, (u128 *)Kpool, (u128 *)Vpool, (int)d->H, (int)d->d, (int)d->r,
              (int)d->N_cap, nTiles, (int)d->N, slots, counters, restart);
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

int ig_launch_pool_touch_lru(ig_ctx *ctx, const ig_desc *d, const int32_t *sel_idx, int32_t sel_stride,
                             const int32_t *sel_cnt, int32_t *stamps, int32_t now, hipStream_t s) {
  auto k = pool_touch_lru;
  IG_LAUNCH(ctx, IG_K_BUILD, k, dim3(d->B * d->H), dim3(256), s, sel_idx, sel_cnt, stamps,
            (int)sel_stride, (int)d->N, (int)d->N_cap, now);
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

int ig_attn_fill(ig_ctx *ctx, const ig_desc *d, const void *q, const void *K, const void *V,
                 const int32_t *sel_idx, int32_t sel_stride, const int32_t *sel_cnt, int kv_rows,
                 const void *k_new, const void *v_new, void *out, void *K_out, void *V_out,
                 float *part, int32_t *counters, AttnArgs *A) {
  const int row_bytes = d->d * ig_elem_bytes(d->dtype);
  const int LPR = row_bytes / 16;
  if (row_bytes % 16 || LPR < 1 || LPR > 64 || (LPR & (LPR - 1)))
    return ig_fail(ctx, IG_ESHAPE, "attention: row of %d bytes must be 16 * 2^k bytes, at most 1024",
                   row_bytes);
  A->q = q;
  A->K = (const uint4 *)K;
  A->V = (const uint4 *)V;
  A->sel_idx = sel_idx;
  A->sel_cnt = sel_cnt;
  A->stride = sel_stride;
  A->kv_rows = kv_rows;
  A->LPR = LPR;
  A->k_new = k_new;
  A->v_new = v_new;
  A->out = out;
  A->scale = d->scale;
  A->d = d->d;
  A->part = part;
  A->counters = counters;
  A->H = d->H;
  A->BH = d->B * d->H;
  A->K_out = sel_idx ? (uint4 *)K_out : nullptr;
  A->V_out = sel_idx ? (uint4 *)V_out : nullptr;
  return IG_OK;
}

int ig_attn_args(ig_ctx *ctx, const ig_desc *d, const void *q, const void *K, const void *V,
                 const int32_t *sel_idx, int32_t sel_stride, const int32_t *sel_cnt, int kv_rows,
                 const void *k_new, const void *v_new, void *out, void *K_out, void *V_out, AttnArgs *A) {
  const int BH = d->B * d->H;
  int rc = ig_ensure(ctx, (void **)&ctx->attn_part, &ctx->attn_part_bytes,
                     (size_t)BH * SLICE_MAX * (d->d + 2) * sizeof(float));
  if (rc) return rc;
  if ((rc = ig_ensure_zeroed(ctx, (void **)&ctx->attn_cnt, &ctx->attn_cnt_bytes, (size_t)BH * sizeof(int32_t))))
    return rc;
  return ig_attn_fill(ctx, d, q, K, V, sel_idx, sel_stride, sel_cnt, kv_rows, k_new, v_new, out, K_out,
                      V_out, ctx->attn_part, ctx->attn_cnt, A);
}

int ig_launch_attention(ig_ctx *ctx, const ig_desc *d, const void *q, const void *K, const void *V,
                        const int32_t *sel_idx, int32_t sel_stride, const int32_t *sel_cnt,
                        int kv_rows_per_bh, const void *k_new, const void *v_new, void *out,
                        void *K_out, void *V_out, hipStream_t s) {
  AttnArgs A;
  int rc = ig_attn_args(ctx, d, q, K, V, sel_idx, sel_stride, sel_cnt, kv_rows_per_bh, k_new, v_new, out,
                        K_out, V_out, &A);
  if (rc) return rc;
  dim3 grid(A.BH * SLICE_MAX), block(256);
  if (d->dtype == IG_F16) {
    if (sel_idx) {
      auto k = sparse_attention<half_t, true>;
      IG_LAUNCH(ctx, IG_K_ATTENTION, k, grid, block, s, A);
    } else {
      auto k = sparse_attention<half_t, false>;
      IG_LAUNCH(ctx, IG_K_ATTENTION, k, grid, block, s, A);
    }
  } else {
    if (sel_idx) {
      auto k = sparse_attention<float, true>;
      IG_LAUNCH(ctx, IG_K_ATTENTION, k, grid, block, s, A);
    } else {
      auto k = sparse_attention<float, false>;
      IG_LAUNCH(ctx, IG_K_ATTENTION, k, grid, block, s, A);
    }
  }
  return IG_OK;
}

// ---- attention without any allocation -----------------------------------------------------------
// For callers that cannot allocate (stream capture, serving loops, harnesses that forbid it): the
// per-slice softmax states and the per-(b,h) arrival counters of the attention kernel live in a
// file-scope device array instead of context workspaces.  Every GPU the library runs on holds its
// own copy of the array, at its own address, until the process ends; the address is looked up
// once per context (ig_create, with the context's device current) and host code only ever uses
// that address, never the array's name.  Layout: counters int32 [B*H] (padded to 256 bytes), then
// states float [B*H][SLICE_MAX][d+2].
constexpr size_t STATIC_SCRATCH_BYTES = (size_t)16 << 20;
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];

namespace {
__global__ __launch_bounds__(256) void zero_words(int32_t *p, int n) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < n) p[i] = 0;
}
}  // namespace

int ig_static_scratch_bind(ig_ctx *ctx) {
  void *ptr = nullptr;
  hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
  if (e != hipSuccess || !ptr) {
    ctx->static_scratch = nullptr;
    ctx->static_scratch_bytes = 0;
    return ig_hip_fail(ctx, e, "hipGetSymbolAddress(scratch)");
  }
  ctx->static_scratch = ptr;
  ctx->static_scratch_bytes = STATIC_SCRATCH_BYTES;
  return IG_OK;
}

int ig_launch_attention_static(ig_ctx *ctx, const ig_desc *d, const void *q, const void *K, const void *V,
                               int32_t sel_stride, const int32_t *sel_cnt, const void *k_new,
                               const void *v_new, void *out, hipStream_t s) {
  if (!ctx->static_scratch) return ig_fail(ctx, IG_EHIP, "the static scratch array was not bound on this device");
  const size_t BH = (size_t)d->B * d->H;
  const size_t cnt_bytes = (BH * sizeof(int32_t) + 255) / 256 * 256;
  const size_t need = cnt_bytes + BH * SLICE_MAX * ((size_t)d->d + 2) * sizeof(float);
  if (need > ctx->static_scratch_bytes)
    return ig_fail(ctx, IG_ECAPACITY,
                   "ig_sparse_attention_static: B*H = %zu heads of d = %d need %zu bytes of slice states, "
                   "the static scratch array holds %zu", BH, d->d, need, ctx->static_scratch_bytes);
  int32_t *counters = reinterpret_cast<int32_t *>(ctx->static_scratch);
  float *part = reinterpret_cast<float *>(static_cast<unsigned char *>(ctx->static_scratch) + cnt_bytes);
  AttnArgs A;
  int rc = ig_attn_fill(ctx, d, q, K, V, nullptr, sel_stride, sel_cnt, sel_stride, k_new, v_new, out,
                        nullptr, nullptr, part, counters, &A);
  if (rc) return rc;
  // The array keeps whatever the last call left (a call that was cut short leaves counters
  // behind): the arrival counters start from zero on every call.  A fill kernel, not a memset, so
  // that the sequence can be captured into a graph.
  hipLaunchKernelGGL(zero_words, dim3((unsigned)((BH + 255) / 256)), dim3(256), 0, s, counters, (int)BH);
  dim3 grid((unsigned)(BH * SLICE_MAX)), block(256);
  if (d->dtype == IG_F16) {
    hipLaunchKernelGGL((sparse_attention<half_t, false>), grid, block, 0, s, A);
  } else {
    hipLaunchKernelGGL((sparse_attention<float, false>), grid, block, 0, s, A);
  }
  hipError_t le = hipGetLastError();
  if (le != hipSuccess) return ig_hip_fail(ctx, le, "sparse_attention (static scratch)");
  return IG_OK;
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
