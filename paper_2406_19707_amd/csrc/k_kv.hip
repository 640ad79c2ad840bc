// Partial key cache construction (Section 4.3 "Prefill Stage"), prefetch of the selected K/V rows
// (Section 4.1, Section 4.3) and decode attention over the fetched rows (Section 2.1).
#include "ig_internal.h"

namespace {

typedef uint4 u128;

// ---- slab build ---------------------------------------------------------------------------------
// A workgroup takes 32 consecutive tokens of one (b,h): the full key rows are read coalesced
// (also when the pool is pinned host memory) into LDS, then the r kept channels are written to the
// tile's channel planes, consecutive threads writing consecutive tokens.
template <typename T>
__global__ __launch_bounds__(256) void slab_build(const T *__restrict__ Kpool,
                                                  const int32_t *__restrict__ idx,
                                                  T *__restrict__ slab, int H, int d, int r, int N,
                                                  int N_cap, int nTiles) {
  constexpr int TPL = Elem<T>::TPL;
  constexpr int TILE = IG_WAVE * TPL;
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

// ---- gather -------------------------------------------------------------------------------------
// Row copies in 16-byte units; U units per row.  grid (chunks of ROWS rows, B*H); workgroups whose
// first row lies beyond the list's length leave at once, so the grid can be sized for the worst
// case without the host knowing the counts.
constexpr int GATHER_ROWS = 64;
__global__ __launch_bounds__(256) void gather_rows(const u128 *__restrict__ Kpool,
                                                   const u128 *__restrict__ Vpool,
                                                   const int32_t *__restrict__ sel_idx,
                                                   const int32_t *__restrict__ sel_cnt,
                                                   u128 *__restrict__ K_sel, u128 *__restrict__ V_sel,
                                                   int N_cap, int stride, int U) {
  const int bh = blockIdx.y;
  const int cnt = min(sel_cnt[bh], stride);
  const int row0 = blockIdx.x * GATHER_ROWS;
  if (row0 >= cnt) return;
  const int rows = min(GATHER_ROWS, cnt - row0);
  const int32_t *list = sel_idx + (long)bh * stride + row0;
  const long src0 = (long)bh * N_cap * U, dst0 = ((long)bh * stride + row0) * U;
  const int total = rows * U;
#pragma unroll 4
  for (int u = threadIdx.x; u < total; u += 256) {
    int rr = u / U, c = u - rr * U;
    long src = src0 + (long)list[rr] * U + c;
    u128 kv = Kpool[src];
    u128 vv = Vpool[src];
    K_sel[dst0 + u] = kv;
    V_sel[dst0 + u] = vv;
  }
}

// ---- attention ----------------------------------------------------------------------------------
// One workgroup (4 waves) per (b,h).  A row of d elements is covered by LPR = d*sizeof(T)/16 lanes,
// 16 bytes each; a wave handles 64/LPR rows per step.  Every lane group keeps an online-softmax
// state (running max, normaliser, weighted sum for its 16-byte slice of V); states are merged
// across lane groups with shuffles and across waves through LDS.
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

template <int TPL> struct SoftState {
  float m, z;
  float acc[TPL];
};

template <int TPL>
__device__ __forceinline__ void merge_state(SoftState<TPL> &a, float m2, float z2, const float (&acc2)[TPL]) {
  float M = fmaxf(a.m, m2);
  float f1 = (a.m == -INFINITY) ? 0.f : __expf(a.m - M);
  float f2 = (m2 == -INFINITY) ? 0.f : __expf(m2 - M);
  a.z = a.z * f1 + z2 * f2;
#pragma unroll
  for (int e = 0; e < TPL; ++e) a.acc[e] = a.acc[e] * f1 + acc2[e] * f2;
  a.m = M;
}

template <typename T, bool INDEXED>
__global__ __launch_bounds__(256) void sparse_attention(const T *__restrict__ q,
                                                        const u128 *__restrict__ K,
                                                        const u128 *__restrict__ V,
                                                        const int32_t *__restrict__ sel_idx,
                                                        const int32_t *__restrict__ sel_cnt,
                                                        int stride, int kv_rows, int LPR,
                                                        const T *__restrict__ k_new,
                                                        const T *__restrict__ v_new,
                                                        T *__restrict__ out, float scale, int d) {
  constexpr int TPL = Elem<T>::TPL;
  __shared__ float sm[4], sz[4];
  __shared__ float sacc[4][512];
  const int bh = blockIdx.x;
  const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int RPW = 64 / LPR;            // rows per wave step
  const int sub = lane / LPR, li = lane % LPR;
  const int n = min(sel_cnt[bh], stride);
  const int rows = n + (k_new ? 1 : 0);
  float qf[TPL];
  {
    u128 raw = *reinterpret_cast<const u128 *>(q + (long)bh * d + li * TPL);
    to_float<T>(raw, qf);
#pragma unroll
    for (int e = 0; e < TPL; ++e) qf[e] *= scale;
  }
  SoftState<TPL> st;
  st.m = -INFINITY;
  st.z = 0.f;
#pragma unroll
  for (int e = 0; e < TPL; ++e) st.acc[e] = 0.f;
  const long base = (long)bh * kv_rows * LPR;
  const int32_t *list = sel_idx + (long)bh * stride;
#pragma unroll 2
  for (int j = w * RPW + sub; j < rows; j += 4 * RPW) {
    u128 kr, vr;
    if (j < n) {
      long row = INDEXED ? (long)list[j] : (long)j;
      kr = K[base + row * LPR + li];
      vr = V[base + row * LPR + li];
    } else {
      kr = *reinterpret_cast<const u128 *>(k_new + (long)bh * d + li * TPL);
      vr = *reinterpret_cast<const u128 *>(v_new + (long)bh * d + li * TPL);
    }
    float kf[TPL], vf[TPL];
    to_float<T>(kr, kf);
    to_float<T>(vr, vf);
    float l = 0.f;
#pragma unroll
    for (int e = 0; e < TPL; ++e) l = fmaf(qf[e], kf[e], l);
    for (int o = 1; o < LPR; o <<= 1) l += __shfl_xor(l, o, 64);
    float M = fmaxf(st.m, l);
    float f1 = (st.m == -INFINITY) ? 0.f : __expf(st.m - M);
    float p = __expf(l - M);
    st.z = st.z * f1 + p;
#pragma unroll
    for (int e = 0; e < TPL; ++e) st.acc[e] = st.acc[e] * f1 + p * vf[e];
    st.m = M;
  }
  // merge lane groups of the wave (lanes with equal li hold the same slice of V)
  for (int o = LPR; o < 64; o <<= 1) {
    float m2 = __shfl_xor(st.m, o, 64), z2 = __shfl_xor(st.z, o, 64);
    float a2[TPL];
#pragma unroll
    for (int e = 0; e < TPL; ++e) a2[e] = __shfl_xor(st.acc[e], o, 64);
    merge_state<TPL>(st, m2, z2, a2);
  }
  if (lane < LPR) {
    if (lane == 0) { sm[w] = st.m; sz[w] = st.z; }
#pragma unroll
    for (int e = 0; e < TPL; ++e) sacc[w][lane * TPL + e] = st.acc[e];
  }
  __syncthreads();
  for (int c = threadIdx.x; c < d; c += 256) {
    float M = fmaxf(fmaxf(sm[0], sm[1]), fmaxf(sm[2], sm[3]));
    float z = 0.f, a = 0.f;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      float f = (sm[k] == -INFINITY) ? 0.f : __expf(sm[k] - M);
      z += sz[k] * f;
      a += sacc[k][c] * f;
    }
    out[(long)bh * d + c] = (T)(z > 0.f ? a / z : 0.f);
  }
}

__global__ __launch_bounds__(256) void copy_bytes(const u128 *__restrict__ src, u128 *__restrict__ dst,
                                                  long n16) {
  long i = (long)blockIdx.x * 256 + threadIdx.x;
  const long step = (long)gridDim.x * 256;
  for (; i < n16; i += step) dst[i] = src[i];
}

}  // namespace

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

int ig_launch_gather(ig_ctx *ctx, const ig_desc *d, const void *Kpool, const void *Vpool,
                     const int32_t *sel_idx, int32_t sel_stride, const int32_t *sel_cnt,
                     void *K_sel, void *V_sel, hipStream_t s) {
  const int U = d->d * ig_elem_bytes(d->dtype) / 16;
  dim3 grid((sel_stride + GATHER_ROWS - 1) / GATHER_ROWS, d->B * d->H), block(256);
  auto k = gather_rows;
  IG_LAUNCH(ctx, IG_K_GATHER, k, grid, block, s, (const u128 *)Kpool, (const u128 *)Vpool, sel_idx,
            sel_cnt, (u128 *)K_sel, (u128 *)V_sel, (int)d->N_cap, (int)sel_stride, U);
  return IG_OK;
}

template <typename T>
static int launch_attention_t(ig_ctx *ctx, const ig_desc *d, const void *q, const void *K,
                              const void *V, const int32_t *sel_idx, int32_t sel_stride,
                              const int32_t *sel_cnt, int kv_rows, const void *k_new,
                              const void *v_new, void *out, hipStream_t s) {
  const int LPR = d->d * (int)sizeof(T) / 16;
  dim3 grid(d->B * d->H), block(256);
  if (sel_idx) {
    auto k = sparse_attention<T, true>;
    IG_LAUNCH(ctx, IG_K_ATTENTION, k, grid, block, s, (const T *)q, (const u128 *)K, (const u128 *)V,
              sel_idx, sel_cnt, (int)sel_stride, kv_rows, LPR, (const T *)k_new, (const T *)v_new,
              (T *)out, (float)d->scale, (int)d->d);
  } else {
    auto k = sparse_attention<T, false>;
    IG_LAUNCH(ctx, IG_K_ATTENTION, k, grid, block, s, (const T *)q, (const u128 *)K, (const u128 *)V,
              sel_idx, sel_cnt, (int)sel_stride, kv_rows, LPR, (const T *)k_new, (const T *)v_new,
              (T *)out, (float)d->scale, (int)d->d);
  }
  return IG_OK;
}

int ig_launch_attention(ig_ctx *ctx, const ig_desc *d, const void *q, const void *K, const void *V,
                        const int32_t *sel_idx, int32_t sel_stride, const int32_t *sel_cnt,
                        int kv_rows_per_bh, const void *k_new, const void *v_new, void *out,
                        hipStream_t s) {
  const int row_bytes = d->d * ig_elem_bytes(d->dtype);
  const int LPR = row_bytes / 16;
  if (row_bytes % 16 || LPR < 1 || LPR > 64 || (LPR & (LPR - 1)))
    return ig_fail(ctx, IG_ESHAPE, "attention: row of %d bytes must be 16 * 2^k bytes, at most 1024",
                   row_bytes);
  return d->dtype == IG_F16
             ? launch_attention_t<half_t>(ctx, d, q, K, V, sel_idx, sel_stride, sel_cnt,
                                          kv_rows_per_bh, k_new, v_new, out, s)
             : launch_attention_t<float>(ctx, d, q, K, V, sel_idx, sel_stride, sel_cnt,
                                         kv_rows_per_bh, k_new, v_new, out, s);
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
