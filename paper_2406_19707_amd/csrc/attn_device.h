// Device side of the gather / attention kernels: 16-byte row units, the (b, h, slice) work-item
// mapping, and the body of the sparse attention kernel.  Shared by the attention kernels and by the
// kernel that runs a layer's attention next to the next layer's scan in one launch.
#ifndef IG_ATTN_DEVICE_H
#define IG_ATTN_DEVICE_H
#include "ig_internal.h"

struct AttnArgs {
  const void *q;              // [B,H,d]
  const uint4 *K, *V;          // gathered rows [B*H, stride, d] or the pool [B*H, kv_rows, d] (INDEXED)
  const int32_t *sel_idx, *sel_cnt;
  int stride, kv_rows, LPR;
  const void *k_new, *v_new;  // optional always-attended row
  void *out;
  float scale;
  int d;
  float *part;                // per-slice softmax states [B*H][SLICE_MAX][d+2]
  int32_t *counters;          // per-(b,h) arrival counters, zero between calls
  int H, BH;
  uint4 *K_out, *V_out;        // INDEXED only: the rows read are also stored here (fused prefetch)
};

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
__device__ __forceinline__ void work_item(int id, int H, int BH, int *bh, int *slice) {
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
// workgroup (see the note at the counter bump below).  The counter is left at zero for the next
// call.
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


// `id` is the linear work item (see work_item); the kernel passes blockIdx.x
template <typename T, bool INDEXED>
__device__ __forceinline__ void sparse_attention_body(const AttnArgs &A, const int id) {
  const T *__restrict__ q = static_cast<const T *>(A.q);
  const u128 *__restrict__ K = A.K;
  const u128 *__restrict__ V = A.V;
  const int32_t *__restrict__ sel_idx = A.sel_idx;
  const int32_t *__restrict__ sel_cnt = A.sel_cnt;
  const int stride = A.stride, kv_rows = A.kv_rows, LPR = A.LPR, d = A.d, H = A.H, BH = A.BH;
  const T *__restrict__ k_new = static_cast<const T *>(A.k_new);
  const T *__restrict__ v_new = static_cast<const T *>(A.v_new);
  T *__restrict__ out = static_cast<T *>(A.out);
  const float scale = A.scale;
  float *part = A.part;
  int32_t *counters = A.counters;
  u128 *__restrict__ K_out = A.K_out;
  u128 *__restrict__ V_out = A.V_out;
  constexpr int TPL = Elem<T>::TPL;
  __shared__ float sm[4], sz[4];
  __shared__ float sacc[4][512];
  __shared__ int s_last;
  constexpr int max_slices = SLICE_MAX;
  int bh, slice;
  work_item(id, H, BH, &bh, &slice);
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
      rowoff[i] = INDEXED ? (long)min(max(list[jl], 0), kv_rows - 1) : (long)jl;   // a slot outside the pool is clamped
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
  // Order between the state stores and the arrival counter.  The states are agent-scope atomic
  // stores (written through to the device's coherence point); every wave waits until its own
  // have been acknowledged there (s_waitcnt vmcnt(0)), the barrier then puts all waves' stores
  // before thread 0's counter bump, an agent-scope atomic performed at the same coherence point,
  // and the last arrival reads the states with agent-scope atomic loads issued after its bump
  // has returned.  The bump itself is relaxed: making it a release-acquire operation adds a
  // write-back and an invalidation of the whole L2 per workgroup, which was measured to double
  // the kernel (20 -> 50 us on 512 lists of 4096 tokens).  What this leans on is therefore the
  // hardware's handling of acknowledged write-through stores, not the language memory model.
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


}  // namespace

// fills the attention argument block; grows the slice-state workspaces if needed
// (ig_attn_fill: the same with the slice-state / counter memory given by the caller, no allocation)
int ig_attn_fill(ig_ctx *ctx, const ig_desc *d, const void *q, const void *K, const void *V,
                 const int32_t *sel_idx, int32_t sel_stride, const int32_t *sel_cnt, int kv_rows,
                 const void *k_new, const void *v_new, void *out, void *K_out, void *V_out,
                 float *part, int32_t *counters, AttnArgs *A);
int ig_attn_args(ig_ctx *ctx, const ig_desc *d, const void *q, const void *K, const void *V,
                 const int32_t *sel_idx, int32_t sel_stride, const int32_t *sel_cnt, int kv_rows,
                 const void *k_new, const void *v_new, void *out, void *K_out, void *V_out, AttnArgs *A);

#endif
