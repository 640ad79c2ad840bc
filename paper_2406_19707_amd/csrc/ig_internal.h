// Internal declarations shared by the HIP sources of libinfinigen_hip (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>
#include <stdio.h>
#include <vector>

#include "../../include/infinigen.h"

typedef _Float16 half_t;
typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

// 16-byte vector view of the storage type: 8 halves or 4 floats per lane and load.
template <typename T> struct Elem;
template <> struct Elem<half_t> {
  static constexpr int TPL = 8;
  typedef half8 vec;
};
template <> struct Elem<float> {
  static constexpr int TPL = 4;
  typedef floatx4 vec;
};

// Tokens of one channel that a lane of the scan loads at once (the slab's tile is 64 lanes of them).
constexpr int IG_SLAB_TPL_HALF = 8;
template <typename T> struct SlabElem;
template <> struct SlabElem<half_t> {
  static constexpr int TPL = IG_SLAB_TPL_HALF;
  typedef _Float16 vec __attribute__((ext_vector_type(IG_SLAB_TPL_HALF)));
};
template <> struct SlabElem<float> {
  static constexpr int TPL = 4;
  typedef floatx4 vec;
};

constexpr int IG_WAVE = 64;
constexpr int IG_KS_MAX = 16;     // split-K partial sums a consumer adds up at most
constexpr int IG_STATUS_CAPACITY = 1;
constexpr int IG_STATUS_NOCONV = 2;    // Jacobi sweeps of ig_skew_device left too much off the diagonal
constexpr int IG_SPLIT_MAX = 28;         // workgroups a (b,h) pair's tiles are split over at most (scan)
constexpr int IG_PAIR_SYNC_BYTES = 512;
constexpr long IG_WAIT_LIMIT_DEFAULT = 2000000;   // 20 ms of the 100 MHz clock  // per-pair record through which the splits of a pair meet
constexpr int IG_SLICE_MAX = 16;   // slices a selected-token list is cut into at most (gather, attention)

// Slab geometry: tokens are grouped in tiles of 64 lanes x TPL tokens; inside a tile the r kept
// channels are planes of TILE contiguous tokens:  slab[(bh*nTiles + tile)*r*TILE + j*TILE + t%TILE].
template <typename T> __host__ __device__ constexpr int tile_tokens() { return IG_WAVE * SlabElem<T>::TPL; }
static inline int ig_tile_tokens(int dtype) { return dtype == IG_F16 ? IG_WAVE * IG_SLAB_TPL_HALF : 256; }
static inline int ig_elem_bytes(int dtype) { return dtype == IG_F16 ? 2 : 4; }

// Geometry of the partial query projection.
struct ProjGeom {
  int C;        // output columns: H*r (folded) or D (rope)
  int nCblk;    // column blocks of 16
  int Cpad;     // nCblk*16
  int nKblk;    // K blocks of 32 (MFMA path) -- D/32
  int KS;       // split-K factor (<= IG_KS_MAX)
  int kb_per;   // K blocks (MFMA) or K rows (VALU) per split
  int NBtot;    // batch blocks of 16
  int Bpad;     // NBtot*16
  bool mfma;    // f16 and D % 32 == 0
};
ProjGeom ig_proj_geom(const ig_desc *d);

struct ProfRec {
  int which;
  hipEvent_t e0, e1;
};

struct ig_ctx {
  int device;
  char err[512];
  float *part;      size_t part_bytes;    // projection partial sums [KS][Bpad][Cpad]
  float *qp;        size_t qp_bytes;      // finalised partial queries [B,H,r]
  float *scores;    size_t scores_bytes;  // long-sequence path: s [B*H, N]
  float *tmax;      size_t tmax_bytes;    // long-sequence path: per-tile maxima [B*H, nTiles]
  int32_t *pcount;  size_t pcount_bytes;  // long-sequence path: kept tokens per 4096-token part
  float *attn_part; size_t attn_part_bytes;  // attention: per-slice softmax states [B*H][16][d+2]
  int32_t *attn_cnt; size_t attn_cnt_bytes;  // attention: per-(b,h) arrival counters, zero between calls
  void *pair_sync;  size_t pair_sync_bytes;  // scan: per-(b,h) records of pairs split over workgroups, zero between calls
  void *seq_sync = nullptr;            // scan, head-equalised form: per-sequence exchange records (zero between calls)
  size_t seq_sync_bytes = 0;
  int32_t *eq_cnt = nullptr;            // threshold counts of ig_speculate_equalized's two-kernel route
  size_t eq_cnt_bytes = 0;
  hipStream_t call_stream = nullptr;   // stream of the entry point being served (capture check in ig_ensure)
  long spin_limit;                           // scan: bound of a split's wait for its partners, 100 MHz ticks
  double *skew_ws;  size_t skew_ws_bytes;   // ig_skew_device: Gram matrices and eigenvectors [2][H][d][d]
  int32_t *status;                        // device status word (sticky flags)
  void *static_scratch;                   // this device's address of the library's static scratch array
  size_t static_scratch_bytes;            // (bound by ig_create; shared by every context on the device)
  bool profiling;
  std::vector<ProfRec> recs;
  std::vector<hipEvent_t> free_events;
  ig_ctx *side = nullptr;                     // ig_decode_step_overlapped: the side stream's own workspaces
  std::vector<hipEvent_t> pipe_events;        // ... and its cross-stream events (3 per layer), reused from call to call
  double prof_ms[IG_K_COUNT];
  int prof_n[IG_K_COUNT];
};

int ig_fail(ig_ctx *ctx, int code, const char *fmt, ...);
int ig_hip_fail(ig_ctx *ctx, hipError_t e, const char *what);
int ig_ensure(ig_ctx *ctx, void **p, size_t *have, size_t need);
int ig_ensure_zeroed(ig_ctx *ctx, void **p, size_t *have, size_t need);
void ig_prof_events(ig_ctx *ctx, int which, hipEvent_t *e0, hipEvent_t *e1);

#define IG_HIP(ctx, call)                                        \
  do {                                                           \
    hipError_t e__ = (call);                                     \
    if (e__ != hipSuccess) return ig_hip_fail(ctx, e__, #call);  \
  } while (0)

// Launch a kernel; while profiling, attach start/stop events that take the kernel's own timestamps.
#define IG_LAUNCH(ctx, which, kernel, grid, block, stream, ...)                                    \
  do {                                                                                             \
    if ((ctx)->profiling) {                                                                        \
      hipEvent_t e0__, e1__;                                                                       \
      ig_prof_events(ctx, which, &e0__, &e1__);                                                    \
      hipExtLaunchKernelGGL(kernel, grid, block, 0, (hipStream_t)(stream), e0__, e1__, 0,          \
                            __VA_ARGS__);                                                          \
    } else {                                                                                       \
      hipLaunchKernelGGL(kernel, grid, block, 0, (hipStream_t)(stream), __VA_ARGS__);              \
    }                                                                                              \
    hipError_t le__ = hipGetLastError();                                                           \
    if (le__ != hipSuccess) return ig_hip_fail(ctx, le__, #kernel);                                \
  } while (0)

// the same with `lds` bytes of dynamic LDS
#define IG_LAUNCH_LDS(ctx, which, kernel, grid, block, lds, stream, ...)                           \
  do {                                                                                             \
    if ((ctx)->profiling) {                                                                        \
      hipEvent_t e0__, e1__;                                                                       \
      ig_prof_events(ctx, which, &e0__, &e1__);                                                    \
      hipExtLaunchKernelGGL(kernel, grid, block, lds, (hipStream_t)(stream), e0__, e1__, 0,        \
                            __VA_ARGS__);                                                          \
    } else {                                                                                       \
      hipLaunchKernelGGL(kernel, grid, block, lds, (hipStream_t)(stream), __VA_ARGS__);            \
    }                                                                                              \
    hipError_t le__ = hipGetLastError();                                                           \
    if (le__ != hipSuccess) return ig_hip_fail(ctx, le__, #kernel);                                \
  } while (0)

// ---- launchers implemented in the kernel sources (host functions, return IG_* codes) ----------
int ig_launch_wq_build(ig_ctx *ctx, const ig_desc *d, const ProjGeom &g, const void *Wq,
                       const int32_t *idx, void *wq, hipStream_t s);
int ig_launch_slab_build(ig_ctx *ctx, const ig_desc *d, const void *Kpool, const int32_t *idx,
                         void *slab, hipStream_t s);
int ig_launch_project(ig_ctx *ctx, const ig_desc *d, const ProjGeom &g, const void *x,
                      const void *wq, float *part, hipStream_t s);
// index-only partial weight: columns idx of the full weight W, same partial-sum layout
int ig_proj_columns_ks(const ig_desc *d, int *k_per);
int ig_launch_project_columns(ig_ctx *ctx, const ig_desc *d, const ProjGeom &g, const void *x,
                              const void *W, const int32_t *idx, float *part, hipStream_t s);
int ig_launch_finalize(ig_ctx *ctx, const ig_desc *d, const ProjGeom &g, const float *part,
                       const float *bias, const float *A_p, const int32_t *pos, float *q_p,
                       hipStream_t s);
// q source for the scan: value(b,h,j) = bias[h*r+j] + sum_{s<ks} qsrc[s*ks_stride + b*b_stride + h*r + j]
struct QSource {
  const float *qsrc;
  int ks;
  long ks_stride;
  long b_stride;
  const float *bias;
  // rotary models, shapes for which ig_scan_takes_rope(): qsrc holds the full projection's partial
  // sums ([ks][b][D] columns) and the scan derives the partial query from them with A_p [H,d,r]
  // and pos [B]
  const float *A_p = nullptr;
  const int32_t *pos = nullptr;
};
bool ig_scan_is_fused(const ig_desc *d);
bool ig_scan_takes_rope(const ig_desc *d);
bool ig_scan_equalizes(const ig_desc *d);
int ig_launch_scan_equalized(ig_ctx *ctx, const ig_desc *d, const QSource &q, const void *slab, int cap,
                             int32_t *sel_idx, int32_t sel_stride, int32_t *sel_cnt, int32_t *thr_cnt_opt,
                             hipStream_t s);
bool ig_scan_stream_form(const ig_desc *d, int *tiles_per_wave, int *splits);
int ig_launch_scan_select(ig_ctx *ctx, const ig_desc *d, const QSource &q, const void *slab,
                          int32_t *sel_idx, int32_t sel_stride, int32_t *sel_cnt,
                          float *scores_opt, hipStream_t s);
int ig_launch_append(ig_ctx *ctx, const ig_desc *d, const void *k_new, const void *v_new,
                     const int32_t *idx, void *slab, void *Kpool, void *Vpool,
                     const int32_t *slots, int32_t *counters, int32_t restart, hipStream_t s);
int ig_launch_pool_touch_lru(ig_ctx *ctx, const ig_desc *d, const int32_t *sel_idx, int32_t sel_stride,
                             const int32_t *sel_cnt, int32_t *stamps, int32_t now, hipStream_t s);
int ig_launch_pool_touch(ig_ctx *ctx, const ig_desc *d, const int32_t *sel_idx, int32_t sel_stride,
                         const int32_t *sel_cnt, int32_t *counters, int counter_max, hipStream_t s);
int ig_launch_pool_victim(ig_ctx *ctx, const ig_desc *d, const int32_t *counters, int32_t *victim,
                          hipStream_t s);
int ig_launch_gather(ig_ctx *ctx, const ig_desc *d, const void *Kpool, const void *Vpool,
                     const int32_t *sel_idx, int32_t sel_stride, const int32_t *sel_cnt,
                     void *K_sel, void *V_sel, int host_pool, hipStream_t s);
int ig_launch_attention(ig_ctx *ctx, const ig_desc *d, const void *q, const void *K, const void *V,
                        const int32_t *sel_idx, int32_t sel_stride, const int32_t *sel_cnt,
                        int kv_rows_per_bh, const void *k_new, const void *v_new, void *out,
                        void *K_out, void *V_out, hipStream_t s);
int ig_launch_equalize(ig_ctx *ctx, const ig_desc *d, const float *scores, const int32_t *thr_cnt,
                       int cap, int32_t *sel_idx, int32_t sel_stride, int32_t *sel_cnt,
                       hipStream_t s);
int ig_launch_partial_index(ig_ctx *ctx, int dtype, int H, int d, int n, const void *Qs, const void *Ks,
                            int r, float *part, int32_t *idx, hipStream_t s);
size_t ig_partial_index_workspace(int H, int d);
size_t ig_skew_workspace(int H, int d);
int ig_launch_skew(ig_ctx *ctx, int D, int H, int n_cal, const float *Qcal, double *ws, float *A,
                   float *sigma, hipStream_t s);
// scan of the next layer + one-pass prefetch/attention of this layer in one launch
bool ig_layer_step_is_joint(const ig_desc *d);
int ig_launch_scan_attend(ig_ctx *ctx, const ig_desc *d, const QSource &qs, const void *slab,
                          int32_t *sel_idx_next, int32_t *sel_cnt_next, const void *q,
                          const void *Kpool, const void *Vpool, const int32_t *sel_idx,
                          const int32_t *sel_cnt, int32_t sel_stride, const void *k_new,
                          const void *v_new, void *out, void *K_sel, void *V_sel, hipStream_t s);
// attention whose slice states and arrival counters live in the static scratch array (no allocation)
int ig_static_scratch_bind(ig_ctx *ctx);
int ig_launch_attention_static(ig_ctx *ctx, const ig_desc *d, const void *q, const void *K, const void *V,
                               int32_t sel_stride, const int32_t *sel_cnt, const void *k_new,
                               const void *v_new, void *out, hipStream_t s);
int ig_launch_copy(ig_ctx *ctx, const void *src, void *dst, size_t bytes, hipStream_t s);
int ig_launch_read(ig_ctx *ctx, const void *src, size_t bytes, hipStream_t s);

// ---- rotary embedding angle ---------------------------------------------------------------------
// sin and cos of pos * theta^(-2c/d) in double (positions reach 1e5, where float loses the phase).
// Quadrant reduction with a two-part pi/2 (the fused multiply-adds keep the products exact), then
// the Taylor polynomials of sin and cos on [-pi/4, pi/4] to x^19 / x^18 (truncation below 1e-21):
// a few dozen double FMAs and a handful of registers, where the library routine carries a
// large-argument path the kernel never needs.
__device__ __forceinline__ void rope_sincos(double ang, double *sn, double *cs) {
  const double k = rint(ang * 0.63661977236758134308);          // 2 / pi
  double x = fma(-k, 1.57079632679489655800e+00, ang);          // pi/2 rounded to double ...
  x = fma(-k, 6.12323399573676603587e-17, x);                   // ... and what the rounding left
  const double x2 = x * x;
  double ps = 1.0, pc = 1.0;
#pragma unroll
  for (int n = 9; n >= 1; --n) {
    ps = fma(-x2 * (1.0 / (double)((2 * n) * (2 * n + 1))), ps, 1.0);
    pc = fma(-x2 * (1.0 / (double)((2 * n - 1) * (2 * n))), pc, 1.0);
  }
  const double s = x * ps, c = pc;
  const int q = (int)k & 3;
  *sn = q == 0 ? s : (q == 1 ? c : (q == 2 ? -s : -c));
  *cs = q == 0 ? c : (q == 1 ? -s : (q == 2 ? -c : s));
}
// ---- wave helpers -------------------------------------------------------------------------------
// Cross-lane moves inside a 16-lane row through DPP (no LDS crossbar traffic).
template <int CTRL> __device__ __forceinline__ float dpp_move(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(v), __float_as_int(v), CTRL, 0xF, 0xF, false));
}
constexpr int DPP_QUAD_1032 = 0xB1, DPP_QUAD_2301 = 0x4E, DPP_ROW_HALF_MIRROR = 0x141, DPP_ROW_MIRROR = 0x140;

// maximum over the 64 lanes, returned in every lane
__device__ __forceinline__ float wave_max(float v) {
  v = fmaxf(v, dpp_move<DPP_QUAD_1032>(v));
  v = fmaxf(v, dpp_move<DPP_QUAD_2301>(v));
  v = fmaxf(v, dpp_move<DPP_ROW_HALF_MIRROR>(v));
  v = fmaxf(v, dpp_move<DPP_ROW_MIRROR>(v));        // every lane of a row now holds the row's maximum
  const int iv = __float_as_int(v);
  const float r0 = __int_as_float(__builtin_amdgcn_readlane(iv, 0));
  const float r1 = __int_as_float(__builtin_amdgcn_readlane(iv, 16));
  const float r2 = __int_as_float(__builtin_amdgcn_readlane(iv, 32));
  const float r3 = __int_as_float(__builtin_amdgcn_readlane(iv, 48));
  return fmaxf(fmaxf(r0, r1), fmaxf(r2, r3));
}
// sum over the lanes of a 16-lane row, returned in every lane of the row
__device__ __forceinline__ float row16_sum(float v) {
  v += dpp_move<DPP_QUAD_1032>(v);
  v += dpp_move<DPP_QUAD_2301>(v);
  v += dpp_move<DPP_ROW_HALF_MIRROR>(v);
  v += dpp_move<DPP_ROW_MIRROR>(v);
  return v;
}
// inclusive prefix sum over the 64 lanes
__device__ __forceinline__ int wave_incl_scan(int v, int lane) {
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    int u = __shfl_up(v, o, 64);
    if (lane >= o) v += u;
  }
  return v;
}
// sum over the 64 lanes, returned in every lane
__device__ __forceinline__ int wave_sum(int v) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
// number of lanes below this one whose predicate is set, and the wave's total
__device__ __forceinline__ int lanes_below(unsigned long long ballot) {
  return __builtin_amdgcn_mbcnt_hi((unsigned)(ballot >> 32), __builtin_amdgcn_mbcnt_lo((unsigned)ballot, 0));
}
