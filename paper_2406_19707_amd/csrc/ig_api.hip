// C ABI of libinfinigen_hip: context, argument validation, workspace management, profiling,
// and composition of the kernels into the calls declared in include/infinigen.h.
#include <math.h>
#include <stdarg.h>
#include <string.h>

#include <initializer_list>
#include <new>

#include "ig_internal.h"

int ig_fail(ig_ctx *ctx, int code, const char *fmt, ...) {
  if (ctx) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(ctx->err, sizeof(ctx->err), fmt, ap);
    va_end(ap);
  }
  return code;
}

int ig_hip_fail(ig_ctx *ctx, hipError_t e, const char *what) {
  return ig_fail(ctx, IG_EHIP, "%s: %s", what, hipGetErrorString(e));
}

int ig_ensure(ig_ctx *ctx, void **p, size_t *have, size_t need) {
  if (*have >= need && *p) return IG_OK;
  // Growing means hipMalloc, and for a buffer in use also a device-wide wait and a hipFree: none of
  // them may happen while the call's stream is being captured into a graph (the runtime would
  // invalidate the capture, and a replay would use the freed buffer).  Refuse instead.
  if (ctx->call_stream) {
    hipStreamCaptureStatus st = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(ctx->call_stream, &st) == hipSuccess && st != hipStreamCaptureStatusNone)
      return ig_fail(ctx, IG_EINVAL, "a workspace of %zu bytes would have to be allocated while the stream is being "
                     "captured: call ig_reserve for the largest shape before the capture", need);
  }
  if (*p) {
    IG_HIP(ctx, hipDeviceSynchronize());   // earlier launches may still read the old buffer
    IG_HIP(ctx, hipFree(*p));
    *p = nullptr;
    *have = 0;
  }
  size_t bytes = need < 256 ? 256 : need;
  IG_HIP(ctx, hipMalloc(p, bytes));
  *have = bytes;
  return IG_OK;
}

int ig_ensure_zeroed(ig_ctx *ctx, void **p, size_t *have, size_t need) {
  if (*have >= need && *p) return IG_OK;
  int rc = ig_ensure(ctx, p, have, need);
  if (rc) return rc;
  IG_HIP(ctx, hipMemset(*p, 0, *have));
  IG_HIP(ctx, hipDeviceSynchronize());
  return IG_OK;
}

void ig_prof_events(ig_ctx *ctx, int which, hipEvent_t *e0, hipEvent_t *e1) {
  hipEvent_t ev[2];
  for (int i = 0; i < 2; ++i) {
    if (!ctx->free_events.empty()) {
      ev[i] = ctx->free_events.back();
      ctx->free_events.pop_back();
    } else {
      (void)hipEventCreate(&ev[i]);
    }
  }
  ctx->recs.push_back(ProfRec{which, ev[0], ev[1]});
  *e0 = ev[0];
  *e1 = ev[1];
}

namespace {

int check_desc(ig_ctx *ctx, const ig_desc *d) {
  if (!ctx) return IG_EINVAL;
  if (!d) return ig_fail(ctx, IG_EINVAL, "descriptor is NULL");
  if (d->dtype != IG_F32 && d->dtype != IG_F16) return ig_fail(ctx, IG_EDTYPE, "unknown dtype %d", d->dtype);
  if (d->B < 1 || d->H < 1 || d->d < 1 || d->r < 1 || d->N < 1 || d->N_cap < d->N)
    return ig_fail(ctx, IG_ESHAPE, "bad shape B=%d H=%d d=%d r=%d N=%d N_cap=%d", d->B, d->H, d->d,
                   d->r, d->N, d->N_cap);
  if (d->r > d->d) return ig_fail(ctx, IG_ESHAPE, "r = %d exceeds d = %d", d->r, d->d);
  if (d->r > 256) return ig_fail(ctx, IG_ESHAPE, "r = %d exceeds 256", d->r);
  if ((d->d * ig_elem_bytes(d->dtype)) % 16)
    return ig_fail(ctx, IG_ESHAPE, "a row of d = %d elements must be a multiple of 16 bytes", d->d);
  if (!(d->alpha >= 0.0f)) return ig_fail(ctx, IG_EINVAL, "alpha must be >= 0 (got %g)", (double)d->alpha);
  if (!isfinite(d->scale)) return ig_fail(ctx, IG_EINVAL, "scale must be finite");
  if (d->rope != 0 && d->rope != 1) return ig_fail(ctx, IG_EINVAL, "rope must be 0 or 1");
  if (d->rope && (d->d % 2 || !(d->rope_theta > 0.0f)))
    return ig_fail(ctx, IG_EINVAL, "rope needs an even d and a positive base");
  if ((long)d->B * d->H > 2147483647L / 4) return ig_fail(ctx, IG_ESHAPE, "B*H too large");
  return IG_OK;
}

// the same for a call that enqueues on `stream`; remembers the stream for ig_ensure's capture check
int check_desc(ig_ctx *ctx, const ig_desc *d, void *stream) {
  if (ctx) ctx->call_stream = (hipStream_t)stream;
  return check_desc(ctx, d);
}

// the kernels read rows, queries and inputs in 16-byte units
int check_aligned(ig_ctx *ctx, const char *what, std::initializer_list<const void *> ptrs) {
  for (const void *p : ptrs)
    if (p && (uintptr_t)p % 16) return ig_fail(ctx, IG_EINVAL, "%s: every array must be 16-byte aligned", what);
  return IG_OK;
}

int check_sel(ig_ctx *ctx, const int32_t *sel_idx, int32_t sel_stride, const int32_t *sel_cnt) {
  if (!sel_idx || !sel_cnt) return ig_fail(ctx, IG_EINVAL, "sel_idx or sel_cnt is NULL");
  if (sel_stride < 1) return ig_fail(ctx, IG_ESHAPE, "sel_stride = %d", sel_stride);
  return IG_OK;
}

int set_device(ig_ctx *ctx) {
  IG_HIP(ctx, hipSetDevice(ctx->device));
  return IG_OK;
}

// Device-visible address of a pool: device memory as is; pinned host memory through the mapping.
int resolve_pool(ig_ctx *ctx, const void *p, int space, const void **out) {
  if (space == IG_MEM_DEVICE) {
    *out = p;
    return IG_OK;
  }
  if (space != IG_MEM_HOST_PINNED) return ig_fail(ctx, IG_EINVAL, "unknown pool_space %d", space);
  void *dp = nullptr;
  hipError_t e = hipHostGetDevicePointer(&dp, const_cast<void *>(p), 0);
  if (e != hipSuccess || !dp) {
    (void)hipGetLastError();
    return ig_fail(ctx, IG_EINVAL, "host pool is not pinned, GPU-mapped memory (%s)", hipGetErrorString(e));
  }
  *out = dp;
  return IG_OK;
}

int reserve_for(ig_ctx *ctx, const ig_desc *d, bool scores) {
  ProjGeom g = ig_proj_geom(d);
  int k_per = 0;
  const int ks_cols = d->rope ? 0 : ig_proj_columns_ks(d, &k_per);   // the index-only variant's split
  int rc = ig_ensure(ctx, (void **)&ctx->part, &ctx->part_bytes,
                     (size_t)(g.KS > ks_cols ? g.KS : ks_cols) * g.Bpad * g.Cpad * sizeof(float));
  if (rc) return rc;
  rc = ig_ensure(ctx, (void **)&ctx->qp, &ctx->qp_bytes, (size_t)d->B * d->H * d->r * sizeof(float));
  if (rc) return rc;
  rc = ig_ensure_zeroed(ctx, &ctx->pair_sync, &ctx->pair_sync_bytes, (size_t)d->B * d->H * IG_PAIR_SYNC_BYTES);
  if (rc) return rc;
  rc = ig_ensure_zeroed(ctx, &ctx->seq_sync, &ctx->seq_sync_bytes, (size_t)d->B * (d->H + 1) * sizeof(unsigned long long));
  if (rc) return rc;
  rc = ig_ensure(ctx, (void **)&ctx->eq_cnt, &ctx->eq_cnt_bytes, (size_t)d->B * d->H * sizeof(int32_t));
  if (rc) return rc;
  if (scores) {
    const int tile = ig_tile_tokens(d->dtype);
    const int nTiles = (d->N_cap + tile - 1) / tile;
    rc = ig_ensure(ctx, (void **)&ctx->scores, &ctx->scores_bytes,
                   (size_t)d->B * d->H * d->N_cap * sizeof(float));   // by capacity: N may grow
    if (rc) return rc;
    rc = ig_ensure(ctx, (void **)&ctx->tmax, &ctx->tmax_bytes, (size_t)d->B * d->H * nTiles * sizeof(float));
    if (rc) return rc;
    rc = ig_ensure(ctx, (void **)&ctx->pcount, &ctx->pcount_bytes,
                   (size_t)d->B * d->H * ((d->N_cap + 4095) / 4096) * sizeof(int32_t));
    if (rc) return rc;
    rc = ig_ensure(ctx, (void **)&ctx->attn_part, &ctx->attn_part_bytes,
                   (size_t)d->B * d->H * IG_SLICE_MAX * (d->d + 2) * sizeof(float));
    if (rc) return rc;
    rc = ig_ensure_zeroed(ctx, (void **)&ctx->attn_cnt, &ctx->attn_cnt_bytes,
                          (size_t)d->B * d->H * sizeof(int32_t));
  }
  return rc;
}

}  // namespace

extern "C" {

int ig_create(int device, ig_ctx **out) {
  if (!out) return IG_EINVAL;
  *out = nullptr;
  int n = 0;
  if (hipGetDeviceCount(&n) != hipSuccess || device < 0 || device >= n) return IG_EHIP;
  ig_ctx *ctx = new (std::nothrow) ig_ctx();
  if (!ctx) return IG_ENOMEM;
  ctx->device = device;
  ctx->err[0] = 0;
  ctx->part = ctx->qp = ctx->scores = ctx->tmax = ctx->attn_part = nullptr;
  ctx->attn_cnt = nullptr;
  ctx->pcount = nullptr;
  ctx->pcount_bytes = 0;
  ctx->skew_ws = nullptr;
  ctx->skew_ws_bytes = 0;
  ctx->pair_sync = nullptr;
  ctx->pair_sync_bytes = 0;
  ctx->spin_limit = IG_WAIT_LIMIT_DEFAULT;
  ctx->attn_part_bytes = ctx->attn_cnt_bytes = 0;
  ctx->part_bytes = ctx->qp_bytes = ctx->scores_bytes = ctx->tmax_bytes = 0;
  ctx->status = nullptr;
  ctx->static_scratch = nullptr;
  ctx->static_scratch_bytes = 0;
  ctx->profiling = false;
  memset(ctx->prof_ms, 0, sizeof(ctx->prof_ms));
  memset(ctx->prof_n, 0, sizeof(ctx->prof_n));
  if (hipSetDevice(device) != hipSuccess || hipMalloc((void **)&ctx->status, 256) != hipSuccess ||
      hipMemset(ctx->status, 0, 256) != hipSuccess) {
    delete ctx;
    return IG_EHIP;
  }
  // address of the static scratch array on this device (the device is current here)
  if (ig_static_scratch_bind(ctx) != IG_OK) {
    (void)hipFree(ctx->status);
    delete ctx;
    return IG_EHIP;
  }
  *out = ctx;
  return IG_OK;
}

int ig_destroy(ig_ctx *ctx) {
  if (!ctx) return IG_EINVAL;
  (void)hipSetDevice(ctx->device);
  (void)hipDeviceSynchronize();
  for (auto &r : ctx->recs) {
    (void)hipEventDestroy(r.e0);
    (void)hipEventDestroy(r.e1);
  }
  for (auto &e : ctx->free_events) (void)hipEventDestroy(e);
  for (auto &e : ctx->pipe_events) (void)hipEventDestroy(e);
  if (ctx->side) (void)ig_destroy(ctx->side);
  if (ctx->part) (void)hipFree(ctx->part);
  if (ctx->qp) (void)hipFree(ctx->qp);
  if (ctx->scores) (void)hipFree(ctx->scores);
  if (ctx->tmax) (void)hipFree(ctx->tmax);
  if (ctx->pcount) (void)hipFree(ctx->pcount);
  if (ctx->skew_ws) (void)hipFree(ctx->skew_ws);
  if (ctx->pair_sync) (void)hipFree(ctx->pair_sync);
  if (ctx->seq_sync) (void)hipFree(ctx->seq_sync);
  if (ctx->eq_cnt) (void)hipFree(ctx->eq_cnt);
  if (ctx->attn_part) (void)hipFree(ctx->attn_part);
  if (ctx->attn_cnt) (void)hipFree(ctx->attn_cnt);
  if (ctx->status) (void)hipFree(ctx->status);
  delete ctx;
  return IG_OK;
}

const char *ig_last_error(const ig_ctx *ctx) { return ctx ? ctx->err : "context is NULL"; }

int ig_reserve(ig_ctx *ctx, const ig_desc *desc) {
  int rc = check_desc(ctx, desc);
  if (ctx) ctx->call_stream = nullptr;       // not a stream call: ig_reserve may allocate
  if (rc) return rc;
  if ((rc = set_device(ctx))) return rc;
  return reserve_for(ctx, desc, true);
}

size_t ig_workspace_bytes(const ig_ctx *ctx) {
  if (!ctx) return 0;
  return ctx->part_bytes + ctx->qp_bytes + ctx->scores_bytes + ctx->tmax_bytes + ctx->pcount_bytes +
         ctx->attn_part_bytes + ctx->attn_cnt_bytes + ctx->skew_ws_bytes + ctx->pair_sync_bytes + ctx->seq_sync_bytes + ctx->eq_cnt_bytes;
}

int ig_check_status(ig_ctx *ctx) {
  if (!ctx) return IG_EINVAL;
  int rc = set_device(ctx);
  if (rc) return rc;
  IG_HIP(ctx, hipDeviceSynchronize());
  int32_t st = 0;
  IG_HIP(ctx, hipMemcpy(&st, ctx->status, sizeof(st), hipMemcpyDeviceToHost));
  if (st) IG_HIP(ctx, hipMemset(ctx->status, 0, sizeof(st)));
  if (st & IG_STATUS_CAPACITY)
    return ig_fail(ctx, IG_ECAPACITY, "a selected-token list was longer than sel_stride and was clamped");
  if (st & IG_STATUS_NOCONV)
    return ig_fail(ctx, IG_ENOCONV, "ig_skew_device: the Jacobi sweeps left off-diagonal mass above tolerance");
  return IG_OK;
}

size_t ig_wq_bytes(const ig_desc *d) {
  if (!d || d->H < 1 || d->d < 1 || d->r < 1) return 0;
  ProjGeom g = ig_proj_geom(d);
  const size_t D = (size_t)d->H * d->d;
  return D * g.Cpad * ig_elem_bytes(d->dtype);   // both layouts hold D x Cpad elements
}

int ig_wq_build(ig_ctx *ctx, const ig_desc *d, const void *Wq, const int32_t *idx_dev, void *wq,
                void *stream) {
  int rc = check_desc(ctx, d, stream);
  if (rc) return rc;
  if (!Wq || !wq || (!d->rope && !idx_dev)) return ig_fail(ctx, IG_EINVAL, "ig_wq_build: NULL argument");
  if ((uintptr_t)wq % 16) return ig_fail(ctx, IG_EINVAL, "ig_wq_build: wq must be 16-byte aligned");
  if ((rc = set_device(ctx))) return rc;
  return ig_launch_wq_build(ctx, d, ig_proj_geom(d), Wq, idx_dev, wq, (hipStream_t)stream);
}

int ig_skew_device(ig_ctx *ctx, int D, int H, int n_cal, const float *Qcal, float *A, float *sigma,
                   void *stream) {
  if (!ctx) return IG_EINVAL;
  ctx->call_stream = (hipStream_t)stream;
  if (D < 1 || H < 1 || D % H || n_cal < 1) return ig_fail(ctx, IG_ESHAPE, "ig_skew_device: bad shape");
  const int d = D / H;
  if (d % 2 || d > 256) return ig_fail(ctx, IG_ESHAPE, "ig_skew_device: d = %d must be even and at most 256", d);
  if (!Qcal || !A) return ig_fail(ctx, IG_EINVAL, "ig_skew_device: Qcal or A is NULL");
  int rc = set_device(ctx);
  if (rc) return rc;
  if ((rc = ig_ensure(ctx, (void **)&ctx->skew_ws, &ctx->skew_ws_bytes, ig_skew_workspace(H, d)))) return rc;
  return ig_launch_skew(ctx, D, H, n_cal, Qcal, ctx->skew_ws, A, sigma, (hipStream_t)stream);
}

int ig_partial_index_device(ig_ctx *ctx, int dtype, int H, int d, int n, const void *Qs,
                            const void *Ks, double ratio, int32_t *idx_dev, void *stream) {
  if (!ctx) return IG_EINVAL;
  ctx->call_stream = (hipStream_t)stream;
  if (dtype != IG_F32 && dtype != IG_F16) return ig_fail(ctx, IG_EDTYPE, "unknown dtype %d", dtype);
  if (H < 1 || d < 1 || n < 1) return ig_fail(ctx, IG_ESHAPE, "ig_partial_index_device: bad shape");
  if (d > 256) return ig_fail(ctx, IG_ESHAPE, "ig_partial_index_device: d = %d exceeds 256", d);
  if (!Qs || !idx_dev) return ig_fail(ctx, IG_EINVAL, "ig_partial_index_device: NULL argument");
  if (!(ratio > 0.0) || ratio > 1.0) return ig_fail(ctx, IG_EINVAL, "ratio must be in (0, 1]");
  const int r = (int)floor(ratio * (double)d);
  if (r < 1) return ig_fail(ctx, IG_ESHAPE, "ratio * d < 1");
  int rc = set_device(ctx);
  if (rc) return rc;
  // the partial column sums share the projection's workspace (both are transient)
  if ((rc = ig_ensure(ctx, (void **)&ctx->part, &ctx->part_bytes, ig_partial_index_workspace(H, d)))) return rc;
  return ig_launch_partial_index(ctx, dtype, H, d, n, Qs, Ks, r, ctx->part, idx_dev, (hipStream_t)stream);
}

size_t ig_slab_bytes(const ig_desc *d) {
  if (!d || d->B < 1 || d->H < 1 || d->r < 1 || d->N_cap < 1) return 0;
  const int tile = ig_tile_tokens(d->dtype);
  const size_t nTiles = ((size_t)d->N_cap + tile - 1) / tile;
  return (size_t)d->B * d->H * nTiles * d->r * tile * ig_elem_bytes(d->dtype);
}

int ig_slab_build(ig_ctx *ctx, const ig_desc *d, const void *Kpool, int pool_space,
                  const int32_t *idx_dev, void *slab, void *stream) {
  int rc = check_desc(ctx, d, stream);
  if (rc) return rc;
  if (!Kpool || !idx_dev || !slab) return ig_fail(ctx, IG_EINVAL, "ig_slab_build: NULL argument");
  if ((rc = check_aligned(ctx, "ig_slab_build", {Kpool}))) return rc;
  if ((uintptr_t)slab % 16) return ig_fail(ctx, IG_EINVAL, "ig_slab_build: slab must be 16-byte aligned");
  if ((rc = set_device(ctx))) return rc;
  const void *kp = nullptr;
  if ((rc = resolve_pool(ctx, Kpool, pool_space, &kp))) return rc;
  return ig_launch_slab_build(ctx, d, kp, idx_dev, slab, (hipStream_t)stream);
}

int ig_append_token(ig_ctx *ctx, const ig_desc *d, const void *k_new, const void *v_new,
                    const int32_t *idx_dev, void *slab, void *Kpool, void *Vpool, int pool_space,
                    void *stream) {
  // the descriptor describes the cache before the append: N valid tokens, the new one goes to slot N
  if (!ctx) return IG_EINVAL;
  ctx->call_stream = (hipStream_t)stream;
  if (!d) return ig_fail(ctx, IG_EINVAL, "descriptor is NULL");
  if (d->N == 0 && d->N_cap >= 1) {          // appending to an empty cache is allowed
    ig_desc one = *d;
    one.N = 1;
    int rc0 = check_desc(ctx, &one);
    if (rc0) return rc0;
  } else {
    int rc0 = check_desc(ctx, d);
    if (rc0) return rc0;
  }
  if (d->N >= d->N_cap) return ig_fail(ctx, IG_ECAPACITY, "cache is full: N = %d, N_cap = %d", d->N, d->N_cap);
  if (!k_new || !v_new || !idx_dev || !slab || !Kpool || !Vpool)
    return ig_fail(ctx, IG_EINVAL, "ig_append_token: NULL argument");
  if ((uintptr_t)k_new % 16 || (uintptr_t)v_new % 16)
    return ig_fail(ctx, IG_EINVAL, "ig_append_token: k_new and v_new must be 16-byte aligned");
  int rc = set_device(ctx);
  if (rc) return rc;
  const void *kp = nullptr, *vp = nullptr;
  if ((rc = resolve_pool(ctx, Kpool, pool_space, &kp))) return rc;
  if ((rc = resolve_pool(ctx, Vpool, pool_space, &vp))) return rc;
  return ig_launch_append(ctx, d, k_new, v_new, idx_dev, slab, const_cast<void *>(kp),
                          const_cast<void *>(vp), nullptr, nullptr, 0, (hipStream_t)stream);
}

int ig_pool_touch(ig_ctx *ctx, const ig_desc *d, const int32_t *sel_idx, int32_t sel_stride,
                  const int32_t *sel_cnt, int32_t *counters, int32_t counter_max, void *stream) {
  int rc = check_desc(ctx, d, stream);
  if (rc) return rc;
  if (!counters) return ig_fail(ctx, IG_EINVAL, "ig_pool_touch: counters is NULL");
  if (counter_max < 1) return ig_fail(ctx, IG_EINVAL, "counter_max = %d", counter_max);
  if ((rc = check_sel(ctx, sel_idx, sel_stride, sel_cnt))) return rc;
  if ((rc = set_device(ctx))) return rc;
  return ig_launch_pool_touch(ctx, d, sel_idx, sel_stride, sel_cnt, counters, counter_max,
                              (hipStream_t)stream);
}

int ig_pool_victim(ig_ctx *ctx, const ig_desc *d, const int32_t *counters, int32_t *victim,
                   void *stream) {
  int rc = check_desc(ctx, d, stream);
  if (rc) return rc;
  if (!counters || !victim) return ig_fail(ctx, IG_EINVAL, "ig_pool_victim: NULL argument");
  if ((rc = set_device(ctx))) return rc;
  return ig_launch_pool_victim(ctx, d, counters, victim, (hipStream_t)stream);
}

int ig_pool_replace(ig_ctx *ctx, const ig_desc *d, const int32_t *victim, const void *k_new,
                    const void *v_new, const int32_t *idx_dev, void *slab, void *Kpool, void *Vpool,
                    int pool_space, int32_t *counters, void *stream) {
  int rc = check_desc(ctx, d, stream);
  if (rc) return rc;
  if (!victim || !k_new || !v_new || !idx_dev || !slab || !Kpool || !Vpool)
    return ig_fail(ctx, IG_EINVAL, "ig_pool_replace: NULL argument");
  if ((uintptr_t)k_new % 16 || (uintptr_t)v_new % 16)
    return ig_fail(ctx, IG_EINVAL, "ig_pool_replace: k_new and v_new must be 16-byte aligned");
  if ((rc = set_device(ctx))) return rc;
  const void *kp = nullptr, *vp = nullptr;
  if ((rc = resolve_pool(ctx, Kpool, pool_space, &kp))) return rc;
  if ((rc = resolve_pool(ctx, Vpool, pool_space, &vp))) return rc;
  return ig_launch_append(ctx, d, k_new, v_new, idx_dev, slab, const_cast<void *>(kp),
                          const_cast<void *>(vp), victim, counters, 0, (hipStream_t)stream);
}

int ig_pool_touch_policy(ig_ctx *ctx, const ig_desc *d, int policy, const int32_t *sel_idx,
                         int32_t sel_stride, const int32_t *sel_cnt, int32_t *state, int32_t param,
                         void *stream) {
  if (policy == IG_POLICY_COUNTER)
    return ig_pool_touch(ctx, d, sel_idx, sel_stride, sel_cnt, state, param, stream);
  int rc = check_desc(ctx, d, stream);
  if (rc) return rc;
  if (policy != IG_POLICY_FIFO && policy != IG_POLICY_LRU) return ig_fail(ctx, IG_EINVAL, "unknown pool policy %d", policy);
  if (!state) return ig_fail(ctx, IG_EINVAL, "ig_pool_touch_policy: state is NULL");
  if ((rc = check_sel(ctx, sel_idx, sel_stride, sel_cnt))) return rc;
  if (policy == IG_POLICY_FIFO) return IG_OK;        // being prefetched does not change an entry's age
  if ((rc = set_device(ctx))) return rc;
  return ig_launch_pool_touch_lru(ctx, d, sel_idx, sel_stride, sel_cnt, state, param, (hipStream_t)stream);
}

int ig_pool_replace_policy(ig_ctx *ctx, const ig_desc *d, int policy, const int32_t *victim,
                           const void *k_new, const void *v_new, const int32_t *idx_dev, void *slab,
                           void *Kpool, void *Vpool, int pool_space, int32_t *state, int32_t now,
                           void *stream) {
  int rc = check_desc(ctx, d, stream);
  if (rc) return rc;
  if (policy != IG_POLICY_COUNTER && policy != IG_POLICY_FIFO && policy != IG_POLICY_LRU)
    return ig_fail(ctx, IG_EINVAL, "unknown pool policy %d", policy);
  if (!victim || !k_new || !v_new || !idx_dev || !slab || !Kpool || !Vpool || !state)
    return ig_fail(ctx, IG_EINVAL, "ig_pool_replace_policy: NULL argument");
  if ((uintptr_t)k_new % 16 || (uintptr_t)v_new % 16)
    return ig_fail(ctx, IG_EINVAL, "ig_pool_replace_policy: k_new and v_new must be 16-byte aligned");
  if ((rc = set_device(ctx))) return rc;
  const void *kp = nullptr, *vp = nullptr;
  if ((rc = resolve_pool(ctx, Kpool, pool_space, &kp))) return rc;
  if ((rc = resolve_pool(ctx, Vpool, pool_space, &vp))) return rc;
  return ig_launch_append(ctx, d, k_new, v_new, idx_dev, slab, const_cast<void *>(kp),
                          const_cast<void *>(vp), victim, state, policy == IG_POLICY_COUNTER ? 0 : now,
                          (hipStream_t)stream);
}

static int project_partials(ig_ctx *ctx, const ig_desc *d, const void *x, const void *wq,
                            const float *A_p, const int32_t *pos, ProjGeom *g, hipStream_t s) {
  if (!x || !wq) return ig_fail(ctx, IG_EINVAL, "x or wq is NULL");
  if (int rc0 = check_aligned(ctx, "projection", {x, wq})) return rc0;
  if (d->rope && (!A_p || !pos)) return ig_fail(ctx, IG_EINVAL, "rope mode needs A_p and pos");
  int rc = set_device(ctx);
  if (rc) return rc;
  if ((rc = reserve_for(ctx, d, false))) return rc;
  *g = ig_proj_geom(d);
  return ig_launch_project(ctx, d, *g, x, wq, ctx->part, s);
}

int ig_project(ig_ctx *ctx, const ig_desc *d, const void *x, const void *wq, const float *bias,
               const float *A_p, const int32_t *pos, float *q_p, void *stream) {
  int rc = check_desc(ctx, d, stream);
  if (rc) return rc;
  if (!q_p) return ig_fail(ctx, IG_EINVAL, "q_p is NULL");
  ProjGeom g;
  if ((rc = project_partials(ctx, d, x, wq, A_p, pos, &g, (hipStream_t)stream))) return rc;
  return ig_launch_finalize(ctx, d, g, ctx->part, bias, A_p, pos, q_p, (hipStream_t)stream);
}

// Index-only partial weight: split-K partial sums of x W[:, kept columns] into ctx->part, in the
// geometry `g` of the stored-blob projection but with the split `*ks` of the column kernel.
static int project_columns_partials(ig_ctx *ctx, const ig_desc *d, const void *x, const void *Wq,
                                    const int32_t *idx_dev, ProjGeom *g, int *ks, hipStream_t s) {
  if (!x || !Wq || !idx_dev) return ig_fail(ctx, IG_EINVAL, "x, Wq or idx_dev is NULL");
  if (d->rope) return ig_fail(ctx, IG_EINVAL, "the index-only weight is for rope == 0 (rope == 1 uses the full W_Q already)");
  if ((uintptr_t)Wq % 16 || (uintptr_t)x % 16) return ig_fail(ctx, IG_EINVAL, "x and Wq must be 16-byte aligned");
  int rc = set_device(ctx);
  if (rc) return rc;
  *g = ig_proj_geom(d);
  int k_per = 0;
  *ks = ig_proj_columns_ks(d, &k_per);
  if ((rc = ig_ensure(ctx, (void **)&ctx->part, &ctx->part_bytes,
                      (size_t)(*ks > g->KS ? *ks : g->KS) * g->Bpad * g->Cpad * sizeof(float))))
    return rc;
  if ((rc = ig_ensure(ctx, (void **)&ctx->qp, &ctx->qp_bytes, (size_t)d->B * d->H * d->r * sizeof(float))))
    return rc;
  return ig_launch_project_columns(ctx, d, *g, x, Wq, idx_dev, ctx->part, s);
}

int ig_project_indexed(ig_ctx *ctx, const ig_desc *d, const void *x, const void *Wq,
                       const int32_t *idx_dev, const float *bias, float *q_p, void *stream) {
  int rc = check_desc(ctx, d, stream);
  if (rc) return rc;
  if (!q_p) return ig_fail(ctx, IG_EINVAL, "q_p is NULL");
  ProjGeom g;
  int ks = 0;
  if ((rc = project_columns_partials(ctx, d, x, Wq, idx_dev, &g, &ks, (hipStream_t)stream))) return rc;
  g.KS = ks;
  return ig_launch_finalize(ctx, d, g, ctx->part, bias, nullptr, nullptr, q_p, (hipStream_t)stream);
}

int ig_speculate_indexed(ig_ctx *ctx, const ig_desc *d, const void *x, const void *Wq,
                         const int32_t *idx_dev, const float *bias, const void *slab,
                         int32_t *sel_idx, int32_t sel_stride, int32_t *sel_cnt, float *scores_opt,
                         void *stream) {
  int rc = check_desc(ctx, d, stream);
  if (rc) return rc;
  if (!slab) return ig_fail(ctx, IG_EINVAL, "slab is NULL");
  if ((rc = check_sel(ctx, sel_idx, sel_stride, sel_cnt))) return rc;
  ProjGeom g;
  int ks = 0;
  hipStream_t s = (hipStream_t)stream;
  if ((rc = project_columns_partials(ctx, d, x, Wq, idx_dev, &g, &ks, s))) return rc;
  QSource q{ctx->part, ks, (long)g.Bpad * g.Cpad, (long)g.Cpad, bias};
  return ig_launch_scan_select(ctx, d, q, slab, sel_idx, sel_stride, sel_cnt, scores_opt, s);
}

int ig_scan_select(ig_ctx *ctx, const ig_desc *d, const float *q_p, const void *slab,
                   int32_t *sel_idx, int32_t sel_stride, int32_t *sel_cnt, float *scores_opt,
                   void *stream) {
  int rc = check_desc(ctx, d, stream);
  if (rc) return rc;
  if (!q_p || !slab) return ig_fail(ctx, IG_EINVAL, "q_p or slab is NULL");
  if ((rc = check_sel(ctx, sel_idx, sel_stride, sel_cnt))) return rc;
  if ((rc = set_device(ctx))) return rc;
  QSource q{q_p, 1, 0, (long)d->H * d->r, nullptr};
  return ig_launch_scan_select(ctx, d, q, slab, sel_idx, sel_stride, sel_cnt, scores_opt,
                               (hipStream_t)stream);
}

int ig_speculate(ig_ctx *ctx, const ig_desc *d, const void *x, const void *wq, const float *bias,
                 const float *A_p, const int32_t *pos, const void *slab, int32_t *sel_idx,
                 int32_t sel_stride, int32_t *sel_cnt, float *scores_opt, void *stream) {
  int rc = check_desc(ctx, d, stream);
  if (rc) return rc;
  if (!slab) return ig_fail(ctx, IG_EINVAL, "slab is NULL");
  if ((rc = check_sel(ctx, sel_idx, sel_stride, sel_cnt))) return rc;
  ProjGeom g;
  hipStream_t s = (hipStream_t)stream;
  if ((rc = project_partials(ctx, d, x, wq, A_p, pos, &g, s))) return rc;
  if (d->rope && ig_scan_takes_rope(d)) {
    // rotary embedding and the partial skew sit between the projection and the scan: the scan's
    // workgroups work them out themselves while their first slab loads are in flight
    QSource q{ctx->part, g.KS, (long)g.Bpad * g.Cpad, (long)g.Cpad, bias, A_p, pos};
    return ig_launch_scan_select(ctx, d, q, slab, sel_idx, sel_stride, sel_cnt, scores_opt, s);
  }
  if (d->rope) {
    // other shapes: a small kernel of its own between the two
    if ((rc = ig_launch_finalize(ctx, d, g, ctx->part, bias, A_p, pos, ctx->qp, s))) return rc;
    QSource q{ctx->qp, 1, 0, (long)d->H * d->r, nullptr};
    return ig_launch_scan_select(ctx, d, q, slab, sel_idx, sel_stride, sel_cnt, scores_opt, s);
  }
  // folded: the scan adds the split-K partial sums (and the bias) itself
  QSource q{ctx->part, g.KS, (long)g.Bpad * g.Cpad, (long)g.Cpad, bias};
  return ig_launch_scan_select(ctx, d, q, slab, sel_idx, sel_stride, sel_cnt, scores_opt, s);
}

int ig_speculate_equalized(ig_ctx *ctx, const ig_desc *d, const void *x, const void *wq, const float *bias,
                           const float *A_p, const int32_t *pos, const void *slab, double max_frac,
                           int32_t *sel_idx, int32_t sel_stride, int32_t *sel_cnt, int32_t *thr_cnt_opt,
                           void *stream) {
  int rc = check_desc(ctx, d, stream);
  if (rc) return rc;
  if (!slab) return ig_fail(ctx, IG_EINVAL, "slab is NULL");
  if (!(max_frac > 0.0) || max_frac > 1.0)
    return ig_fail(ctx, IG_EINVAL, "max_frac must be in (0, 1] (got %g)", max_frac);
  if ((rc = check_sel(ctx, sel_idx, sel_stride, sel_cnt))) return rc;
  if (thr_cnt_opt == sel_cnt) return ig_fail(ctx, IG_EINVAL, "ig_speculate_equalized: thr_cnt_opt and sel_cnt must not alias");
  int cap = (int)floor(max_frac * (double)d->N);
  if (cap < 1) cap = 1;
  hipStream_t s = (hipStream_t)stream;
  if (ig_scan_equalizes(d)) {
    // one kernel after the projection: the scan's workgroups exchange their threshold counts and
    // select each head's top n from the scores they still hold in registers
    ProjGeom g;
    if ((rc = project_partials(ctx, d, x, wq, A_p, pos, &g, s))) return rc;
    if (d->rope) {
      QSource q{ctx->part, g.KS, (long)g.Bpad * g.Cpad, (long)g.Cpad, bias, A_p, pos};
      return ig_launch_scan_equalized(ctx, d, q, slab, cap, sel_idx, sel_stride, sel_cnt, thr_cnt_opt, s);
    }
    QSource q{ctx->part, g.KS, (long)g.Bpad * g.Cpad, (long)g.Cpad, bias};
    return ig_launch_scan_equalized(ctx, d, q, slab, cap, sel_idx, sel_stride, sel_cnt, thr_cnt_opt, s);
  }
  // other shapes: the rehearsal with the scores kept, then the stand-alone selection on them
  // (the threshold lists go through sel_idx first and are overwritten by the equalised ones)
  if ((rc = ig_ensure(ctx, (void **)&ctx->scores, &ctx->scores_bytes, (size_t)d->B * d->H * d->N * sizeof(float)))) return rc;
  if ((rc = ig_ensure(ctx, (void **)&ctx->eq_cnt, &ctx->eq_cnt_bytes, (size_t)d->B * d->H * sizeof(int32_t)))) return rc;
  int32_t *thr = thr_cnt_opt ? thr_cnt_opt : ctx->eq_cnt;
  if ((rc = ig_speculate(ctx, d, x, wq, bias, A_p, pos, slab, sel_idx, sel_stride, thr, ctx->scores, stream))) return rc;
  return ig_launch_equalize(ctx, d, ctx->scores, thr, cap, sel_idx, sel_stride, sel_cnt, s);
}

int ig_equalize_heads(ig_ctx *ctx, const ig_desc *d, const float *scores, const int32_t *thr_cnt,
                      double max_frac, int32_t *sel_idx, int32_t sel_stride, int32_t *sel_cnt,
                      void *stream) {
  int rc = check_desc(ctx, d, stream);
  if (rc) return rc;
  if (!scores || !thr_cnt) return ig_fail(ctx, IG_EINVAL, "ig_equalize_heads: NULL argument");
  if (!(max_frac > 0.0) || max_frac > 1.0)
    return ig_fail(ctx, IG_EINVAL, "max_frac must be in (0, 1] (got %g)", max_frac);
  if ((rc = check_sel(ctx, sel_idx, sel_stride, sel_cnt))) return rc;
  if (thr_cnt == sel_cnt) return ig_fail(ctx, IG_EINVAL, "ig_equalize_heads: thr_cnt and sel_cnt must not alias");
  if ((rc = set_device(ctx))) return rc;
  int cap = (int)floor(max_frac * (double)d->N);
  if (cap < 1) cap = 1;
  return ig_launch_equalize(ctx, d, scores, thr_cnt, cap, sel_idx, sel_stride, sel_cnt,
                            (hipStream_t)stream);
}

int ig_gather_kv(ig_ctx *ctx, const ig_desc *d, const void *Kpool, const void *Vpool, int pool_space,
                 const int32_t *sel_idx, int32_t sel_stride, const int32_t *sel_cnt, void *K_sel,
                 void *V_sel, void *stream) {
  int rc = check_desc(ctx, d, stream);
  if (rc) return rc;
  if (!Kpool || !Vpool || !K_sel || !V_sel) return ig_fail(ctx, IG_EINVAL, "ig_gather_kv: NULL argument");
  if ((rc = check_aligned(ctx, "ig_gather_kv", {Kpool, Vpool, K_sel, V_sel}))) return rc;
  if ((rc = check_sel(ctx, sel_idx, sel_stride, sel_cnt))) return rc;
  if ((rc = set_device(ctx))) return rc;
  const void *kp = nullptr, *vp = nullptr;
  if ((rc = resolve_pool(ctx, Kpool, pool_space, &kp))) return rc;
  if ((rc = resolve_pool(ctx, Vpool, pool_space, &vp))) return rc;
  return ig_launch_gather(ctx, d, kp, vp, sel_idx, sel_stride, sel_cnt, K_sel, V_sel,
                          pool_space == IG_MEM_HOST_PINNED, (hipStream_t)stream);
}

int ig_sparse_attention(ig_ctx *ctx, const ig_desc *d, const void *q, const void *K_sel,
                        const void *V_sel, const int32_t *sel_cnt, int32_t sel_stride,
                        const void *k_new, const void *v_new, void *out, void *stream) {
  int rc = check_desc(ctx, d, stream);
  if (rc) return rc;
  if (!q || !K_sel || !V_sel || !sel_cnt || !out) return ig_fail(ctx, IG_EINVAL, "ig_sparse_attention: NULL argument");
  if ((rc = check_aligned(ctx, "ig_sparse_attention", {q, K_sel, V_sel, k_new, v_new}))) return rc;
  if ((k_new == nullptr) != (v_new == nullptr)) return ig_fail(ctx, IG_EINVAL, "k_new and v_new go together");
  if (sel_stride < 1) return ig_fail(ctx, IG_ESHAPE, "sel_stride = %d", sel_stride);
  if ((rc = set_device(ctx))) return rc;
  return ig_launch_attention(ctx, d, q, K_sel, V_sel, nullptr, sel_stride, sel_cnt, sel_stride, k_new,
                             v_new, out, nullptr, nullptr, (hipStream_t)stream);
}

int ig_sparse_attention_static(ig_ctx *ctx, const ig_desc *d, const void *q, const void *K_sel,
                               const void *V_sel, const int32_t *sel_cnt, int32_t sel_stride,
                               const void *k_new, const void *v_new, void *out, void *stream) {
  int rc = check_desc(ctx, d, stream);
  if (rc) return rc;
  if (!q || !K_sel || !V_sel || !sel_cnt || !out)
    return ig_fail(ctx, IG_EINVAL, "ig_sparse_attention_static: NULL argument");
  if ((rc = check_aligned(ctx, "ig_sparse_attention_static", {q, K_sel, V_sel, k_new, v_new}))) return rc;
  if ((k_new == nullptr) != (v_new == nullptr)) return ig_fail(ctx, IG_EINVAL, "k_new and v_new go together");
  if (sel_stride < 1) return ig_fail(ctx, IG_ESHAPE, "sel_stride = %d", sel_stride);
  if ((rc = set_device(ctx))) return rc;
  return ig_launch_attention_static(ctx, d, q, K_sel, V_sel, sel_stride, sel_cnt, k_new, v_new, out,
                                    (hipStream_t)stream);
}

int ig_sparse_attention_indexed(ig_ctx *ctx, const ig_desc *d, const void *q, const void *Kpool,
                                const void *Vpool, const int32_t *sel_idx, int32_t sel_stride,
                                const int32_t *sel_cnt, const void *k_new, const void *v_new,
                                void *out, void *stream) {
  int rc = check_desc(ctx, d, stream);
  if (rc) return rc;
  if (!q || !Kpool || !Vpool || !out) return ig_fail(ctx, IG_EINVAL, "ig_sparse_attention_indexed: NULL argument");
  if ((rc = check_aligned(ctx, "ig_sparse_attention_indexed", {q, Kpool, Vpool, k_new, v_new}))) return rc;
  if ((k_new == nullptr) != (v_new == nullptr)) return ig_fail(ctx, IG_EINVAL, "k_new and v_new go together");
  if ((rc = check_sel(ctx, sel_idx, sel_stride, sel_cnt))) return rc;
  if ((rc = set_device(ctx))) return rc;
  return ig_launch_attention(ctx, d, q, Kpool, Vpool, sel_idx, sel_stride, sel_cnt, d->N_cap, k_new,
                             v_new, out, nullptr, nullptr, (hipStream_t)stream);
}

int ig_gather_attention(ig_ctx *ctx, const ig_desc *d, const void *q, const void *Kpool,
                        const void *Vpool, const int32_t *sel_idx, int32_t sel_stride,
                        const int32_t *sel_cnt, void *K_sel, void *V_sel, const void *k_new,
                        const void *v_new, void *out, void *stream) {
  int rc = check_desc(ctx, d, stream);
  if (rc) return rc;
  if (!q || !Kpool || !Vpool || !K_sel || !V_sel || !out)
    return ig_fail(ctx, IG_EINVAL, "ig_gather_attention: NULL argument");
  if ((rc = check_aligned(ctx, "ig_gather_attention", {q, Kpool, Vpool, K_sel, V_sel, k_new, v_new}))) return rc;
  if ((k_new == nullptr) != (v_new == nullptr)) return ig_fail(ctx, IG_EINVAL, "k_new and v_new go together");
  if ((rc = check_sel(ctx, sel_idx, sel_stride, sel_cnt))) return rc;
  if ((rc = set_device(ctx))) return rc;
  return ig_launch_attention(ctx, d, q, Kpool, Vpool, sel_idx, sel_stride, sel_cnt, d->N_cap, k_new,
                             v_new, out, K_sel, V_sel, (hipStream_t)stream);
}

int ig_layer_step(ig_ctx *ctx, const ig_desc *d, const void *x, const void *wq, const float *bias,
                  const float *A_p, const int32_t *pos, const void *slab, int32_t *sel_idx_next,
                  int32_t *sel_cnt_next, const void *q, const void *Kpool, const void *Vpool,
                  const int32_t *sel_idx, const int32_t *sel_cnt, int32_t sel_stride, void *K_sel,
                  void *V_sel, const void *k_new, const void *v_new, void *out, void *stream) {
  int rc = check_desc(ctx, d, stream);
  if (rc) return rc;
  if (!slab || !q || !Kpool || !Vpool || !K_sel || !V_sel || !out)
    return ig_fail(ctx, IG_EINVAL, "ig_layer_step: NULL argument");
  if ((rc = check_aligned(ctx, "ig_layer_step", {q, Kpool, Vpool, K_sel, V_sel, k_new, v_new}))) return rc;
  if ((k_new == nullptr) != (v_new == nullptr)) return ig_fail(ctx, IG_EINVAL, "k_new and v_new go together");
  if ((rc = check_sel(ctx, sel_idx_next, sel_stride, sel_cnt_next))) return rc;
  if ((rc = check_sel(ctx, sel_idx, sel_stride, sel_cnt))) return rc;
  if (sel_idx_next == sel_idx || sel_cnt_next == sel_cnt)
    return ig_fail(ctx, IG_EINVAL, "ig_layer_step: the next layer's lists must not alias this layer's");
  ProjGeom g;
  hipStream_t s = (hipStream_t)stream;
  if ((rc = project_partials(ctx, d, x, wq, A_p, pos, &g, s))) return rc;
  QSource qs{ctx->part, g.KS, (long)g.Bpad * g.Cpad, (long)g.Cpad, bias};
  if (d->rope && ig_scan_takes_rope(d)) {
    qs.A_p = A_p;
    qs.pos = pos;
  } else if (d->rope) {
    if ((rc = ig_launch_finalize(ctx, d, g, ctx->part, bias, A_p, pos, ctx->qp, s))) return rc;
    qs = QSource{ctx->qp, 1, 0, (long)d->H * d->r, nullptr};
  }
  if (!ig_layer_step_is_joint(d)) {
    // other shapes: the two launches one after the other
    if ((rc = ig_launch_scan_select(ctx, d, qs, slab, sel_idx_next, sel_stride, sel_cnt_next, nullptr, s))) return rc;
    return ig_launch_attention(ctx, d, q, Kpool, Vpool, sel_idx, sel_stride, sel_cnt, d->N_cap, k_new,
                               v_new, out, K_sel, V_sel, s);
  }
  return ig_launch_scan_attend(ctx, d, qs, slab, sel_idx_next, sel_cnt_next, q, Kpool, Vpool, sel_idx,
                               sel_cnt, sel_stride, k_new, v_new, out, K_sel, V_sel, s);
}

int ig_decode_step_overlapped(ig_ctx *ctx, const ig_desc *d, int n_layers, const ig_layer_io *layers,
                              const void *wq, const float *bias, const float *A_p, const int32_t *pos,
                              int pool_space, int n_sets, const ig_buffer_set *sets, int32_t sel_stride,
                              void *main_stream, void *side_stream) {
  int rc = check_desc(ctx, d, main_stream);
  if (rc) return rc;
  if (n_layers < 1 || n_sets < 2 || !layers || !sets)
    return ig_fail(ctx, IG_EINVAL, "ig_decode_step_overlapped: needs layers and at least two buffer sets");
  if (main_stream == side_stream) return ig_fail(ctx, IG_EINVAL, "ig_decode_step_overlapped: the two streams must differ");
  for (int i = 0; i < n_sets; ++i)
    if (!sets[i].sel_idx || !sets[i].sel_cnt || !sets[i].K_sel || !sets[i].V_sel)
      return ig_fail(ctx, IG_EINVAL, "ig_decode_step_overlapped: buffer set %d has a NULL member", i);
  if ((rc = set_device(ctx))) return rc;
  if (!ctx->side) {
    if ((rc = ig_create(ctx->device, &ctx->side))) return ig_fail(ctx, rc, "ig_decode_step_overlapped: no context for the side stream");
  }
  while ((int)ctx->pipe_events.size() < 3 * n_layers) {
    hipEvent_t e;
    IG_HIP(ctx, hipEventCreateWithFlags(&e, hipEventDisableTiming));
    ctx->pipe_events.push_back(e);
  }
  hipStream_t ms = (hipStream_t)main_stream, ss = (hipStream_t)side_stream;
  auto ev_spec = [&](int l) { return ctx->pipe_events[3 * l]; };
  auto ev_gath = [&](int l) { return ctx->pipe_events[3 * l + 1]; };
  auto ev_attn = [&](int l) { return ctx->pipe_events[3 * l + 2]; };
  // Fig. 3(d): iteration l rehearses layer l on the main stream, hands its lists to the side stream
  // for the prefetch, and attends layer l-1 whose rows have arrived meanwhile.  A buffer set is
  // written again only after the attention that read it has been enqueued (lists: same stream) or
  // has finished (rows: the side stream waits for that attention's event).
  for (int l = 0; l <= n_layers; ++l) {
    if (l < n_layers) {
      const ig_layer_io &io = layers[l];
      const ig_buffer_set &st = sets[l % n_sets];
      if ((rc = ig_speculate(ctx, d, io.x, wq, bias, A_p, pos, io.slab, st.sel_idx, sel_stride, st.sel_cnt, nullptr, ms)))
        return rc;
      IG_HIP(ctx, hipEventRecord(ev_spec(l), ms));
      IG_HIP(ctx, hipStreamWaitEvent(ss, ev_spec(l), 0));
      if (l >= n_sets) IG_HIP(ctx, hipStreamWaitEvent(ss, ev_attn(l - n_sets), 0));
      rc = ig_gather_kv(ctx->side, d, io.Kpool, io.Vpool, pool_space, st.sel_idx, sel_stride, st.sel_cnt, st.K_sel,
                        st.V_sel, ss);
      if (rc) return ig_fail(ctx, rc, "prefetch of layer %d: %s", l, ig_last_error(ctx->side));
      IG_HIP(ctx, hipEventRecord(ev_gath(l), ss));
    }
    if (l >= 1) {
      const ig_layer_io &io = layers[l - 1];
      const ig_buffer_set &st = sets[(l - 1) % n_sets];
      IG_HIP(ctx, hipStreamWaitEvent(ms, ev_gath(l - 1), 0));
      if ((rc = ig_sparse_attention(ctx, d, io.q, st.K_sel, st.V_sel, st.sel_cnt, sel_stride, io.k_new, io.v_new, io.out, ms)))
        return rc;
      IG_HIP(ctx, hipEventRecord(ev_attn(l - 1), ms));
    }
  }
  // the side stream's last work is joined to the main stream by the last wait above
  return IG_OK;
}

int ig_set_wait_limit(ig_ctx *ctx, int64_t ticks) {
  if (!ctx) return IG_EINVAL;
  ctx->spin_limit = ticks == 0 ? IG_WAIT_LIMIT_DEFAULT : (long)ticks;
  return IG_OK;
}

int ig_profile_begin(ig_ctx *ctx) {
  if (!ctx) return IG_EINVAL;
  int rc = set_device(ctx);
  if (rc) return rc;
  IG_HIP(ctx, hipDeviceSynchronize());
  for (auto &r : ctx->recs) {
    ctx->free_events.push_back(r.e0);
    ctx->free_events.push_back(r.e1);
  }
  ctx->recs.clear();
  memset(ctx->prof_ms, 0, sizeof(ctx->prof_ms));
  memset(ctx->prof_n, 0, sizeof(ctx->prof_n));
  ctx->profiling = true;
  return IG_OK;
}

int ig_profile_end(ig_ctx *ctx) {
  if (!ctx) return IG_EINVAL;
  int rc = set_device(ctx);
  if (rc) return rc;
  ctx->profiling = false;
  IG_HIP(ctx, hipDeviceSynchronize());
  for (auto &r : ctx->recs) {
    float ms = 0.f;
    IG_HIP(ctx, hipEventElapsedTime(&ms, r.e0, r.e1));
    ctx->prof_ms[r.which] += ms;
    ctx->prof_n[r.which] += 1;
    ctx->free_events.push_back(r.e0);
    ctx->free_events.push_back(r.e1);
  }
  ctx->recs.clear();
  return IG_OK;
}

int ig_profile_read(ig_ctx *ctx, int which, double *total_ms, int32_t *launches) {
  if (!ctx) return IG_EINVAL;
  if (which < 0 || which >= IG_K_COUNT) return ig_fail(ctx, IG_EINVAL, "unknown kernel id %d", which);
  if (total_ms) *total_ms = ctx->prof_ms[which];
  if (launches) *launches = ctx->prof_n[which];
  return IG_OK;
}

int ig_copy_bytes(ig_ctx *ctx, const void *src, void *dst, size_t bytes, void *stream) {
  if (!ctx) return IG_EINVAL;
  if (!src || !dst) return ig_fail(ctx, IG_EINVAL, "ig_copy_bytes: NULL argument");
  if (bytes % 16 || (uintptr_t)src % 16 || (uintptr_t)dst % 16)
    return ig_fail(ctx, IG_EINVAL, "ig_copy_bytes: size and pointers must be multiples of 16");
  int rc = set_device(ctx);
  if (rc) return rc;
  return ig_launch_copy(ctx, src, dst, bytes, (hipStream_t)stream);
}

int ig_read_bytes(ig_ctx *ctx, const void *src, size_t bytes, void *stream) {
  if (!ctx) return IG_EINVAL;
  if (!src) return ig_fail(ctx, IG_EINVAL, "ig_read_bytes: NULL argument");
  if (bytes < 16 || bytes % 16 || (uintptr_t)src % 16)
    return ig_fail(ctx, IG_EINVAL, "ig_read_bytes: size and pointer must be multiples of 16");
  if (bytes / 16 > 2147483647L * 512L) return ig_fail(ctx, IG_ESHAPE, "ig_read_bytes: too large");
  int rc = set_device(ctx);
  if (rc) return rc;
  return ig_launch_read(ctx, src, bytes, (hipStream_t)stream);
}

}  // extern "C"
