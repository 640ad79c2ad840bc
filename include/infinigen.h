/*
 * infinigen.h -- C ABI of the MI355X (gfx950) implementation of InfiniGen's attention rehearsal
 * and of the sparse decode attention it drives (arXiv 2406.19707, Section 4).
 *
 * One decode step of one layer pair (Section 4.3 "Decoding Stage", Fig. 3(d)):
 *   ig_speculate         partial query projection, scan of the skewed partial key cache,
 *                        per-head (max - alpha) threshold, compaction into index lists
 *   ig_gather_kv         copies only the selected K/V rows out of the KV pool (HBM, or pinned host
 *                        memory read over PCIe)
 *   ig_sparse_attention  softmax(q K_sel^T) V_sel on the fetched rows
 * preceded once per model by ig_skew_offline (Section 4.2, Eq. 2 and 3) and once per request by
 * ig_partial_index / ig_wq_build / ig_slab_build (Section 4.3 "Prefill Stage").
 *
 * General rules
 *  - Every call returns an int status (IG_OK = 0).  Nothing throws or aborts across this boundary;
 *    ig_last_error() gives the message of the last failing call on a context.
 *  - Arrays are row-major.  Projections are y = x W with W [in, out] (Section 2.1).
 *  - "device" pointers are HIP device memory on the context's GPU; "host" pointers are ordinary
 *    host memory.  The caller allocates and frees every array; the library owns only the context
 *    (small workspaces, a device status word, profiling events).
 *  - Device calls enqueue work on the hipStream_t passed as `stream` (a void*; NULL = the null
 *    stream) and return without synchronising.  They never read device results on the host.
 *    Workspaces grow on the first call with a larger shape (this allocates); ig_reserve() sizes
 *    them ahead of time, after which the hot-path calls allocate nothing.
 *  - Calls on one context must not overlap in time on different streams: they share workspaces.
 *  - dtype IG_F16: x, weights, K, V, q, out are IEEE half; IG_F32: float.  Partial queries,
 *    scores and all accumulation are float32 in both cases.  Index arrays are int32.
 *  - Every array of desc->dtype (x, weights, pools, fetched rows, queries, new-token rows) must be
 *    16-byte aligned (IG_EINVAL otherwise) and a row of d elements a multiple of 16 bytes.  The four
 *    attention entry points (ig_sparse_attention, ig_sparse_attention_static,
 *    ig_sparse_attention_indexed, ig_gather_attention) and ig_layer_step need more: a row of
 *    16 * 2^k bytes, at most 1024 (d = 8, 16, 32, 64, 128, 256, 512 in half precision); other head
 *    dimensions (d = 96, 80) pass setup, ig_speculate and ig_gather_kv and get IG_ESHAPE there.
 *  - Index values are never followed outside their array: a kept-column index outside [0, d) or a
 *    selected slot outside [0, N_cap) is clamped into the range (the result is then wrong for that
 *    entry, but no access leaves the caller's arrays).
 */
#ifndef INFINIGEN_H
#define INFINIGEN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  IG_OK = 0,
  IG_EINVAL = 1,    /* null pointer, bad flag, alpha < 0 or NaN, unpinned host pool */
  IG_ESHAPE = 2,    /* a dimension is zero, negative or outside what the kernels support */
  IG_EDTYPE = 3,    /* unknown dtype */
  IG_ECAPACITY = 4, /* a selected-token list did not fit in sel_stride (reported by ig_check_status) */
  IG_EHIP = 5,      /* a HIP runtime call failed; message holds hipGetErrorString */
  IG_ENOCONV = 6,   /* Jacobi sweeps exceeded their cap in ig_skew_offline */
  IG_ENOMEM = 7
};

enum { IG_F32 = 0, IG_F16 = 1 };
enum { IG_MEM_DEVICE = 0, IG_MEM_HOST_PINNED = 1 };
/* Victim selection policies of the KV cache pool (Section 4.4): the counter-based one the paper
 * adopts, and the two it is compared with (Table 2). */
enum { IG_POLICY_COUNTER = 0, IG_POLICY_FIFO = 1, IG_POLICY_LRU = 2 };

/* Kernel identifiers for ig_profile_read. */
enum {
  IG_K_PROJECT = 0,  /* partial query projection (split-K partial sums) */
  IG_K_FINALIZE = 1, /* partial-sum reduction, bias, rotary embedding, partial skew */
  IG_K_SCAN = 2,     /* partial key cache scan (+ max, threshold, compaction when fused) */
  IG_K_SELECT = 3,   /* threshold + compaction from a score buffer (long sequences) */
  IG_K_GATHER = 4,
  IG_K_ATTENTION = 5,
  IG_K_BUILD = 6,    /* ig_wq_build / ig_slab_build */
  IG_K_COPY = 7,     /* ig_copy_bytes */
  IG_K_READ = 8,     /* ig_read_bytes */
  IG_K_LAYER = 9,    /* ig_layer_step: next layer's scan + this layer's prefetch and attention, one launch */
  IG_K_COUNT = 10
};

typedef struct ig_ctx ig_ctx;

/* Shape and parameters of one layer's rehearsal; passed by const pointer, plain data. */
typedef struct {
  int32_t B;        /* sequences in the batch */
  int32_t H;        /* attention heads */
  int32_t d;        /* head dimension; D = H*d is the model dimension */
  int32_t r;        /* kept columns per head, floor(ratio*d) (Section 4.3: 30 %) */
  int32_t N;        /* cached tokens per sequence that are valid */
  int32_t N_cap;    /* tokens allocated per (sequence, head) in the pools and the slab, >= N */
  int32_t dtype;    /* IG_F32 or IG_F16 */
  float scale;      /* logit scale applied to speculated scores and attention logits */
  float alpha;      /* threshold slack, >= 0; +infinity selects every token (Section 4.3) */
  int32_t rope;     /* 0: skew folded into the query weight; 1: rotary embedding between
                       projection and skew (the partial projection then needs the full W_Q) */
  float rope_theta; /* rotary base (10000) */
} ig_desc;

/* ---- context ---------------------------------------------------------------------------- */
int ig_create(int device, ig_ctx **out);
int ig_destroy(ig_ctx *ctx);
const char *ig_last_error(const ig_ctx *ctx);
/* Size the context's workspaces for `desc` now (allocates; synchronous). */
int ig_reserve(ig_ctx *ctx, const ig_desc *desc);
/* Device memory the context's workspaces hold at the moment, in bytes (host-side bookkeeping, no
 * device call).  Unchanged by the per-layer calls once ig_reserve has sized them for the largest
 * shape (N_cap, B) they will see. */
size_t ig_workspace_bytes(const ig_ctx *ctx);
/* Synchronise the device and report sticky device-side conditions: IG_ECAPACITY if any list was
 * clamped to sel_stride since the last check, IG_ENOCONV if ig_skew_device did not converge, else
 * IG_OK.  Clears the conditions. */
int ig_check_status(ig_ctx *ctx);

/* ---- offline / prefill helpers (host pointers, float32, synchronous, CPU) ----------------- */

/* Offline skewing (Section 4.2 "Skewed Partial Weight", Eq. 2 and Eq. 3; Section 4.3 "Prefetching
 * Scheme").  For each head h, the [n_cal, d] block of the calibration query matrix Qcal is
 * decomposed Q_h = U S V^T and A_h = V; the head's query / key weight columns (and biases) are
 * multiplied by A_h from the right.  A [H,d,d] always written; sigma [H,d] (singular values,
 * descending), Wq_s, Wk_s [D,D], bq_s, bk_s [D] written when both the input and the output
 * pointer are non-NULL.  Column signs of A_h: largest-magnitude entry positive.
 * ctx may be NULL (no message is kept then). */
int ig_skew_offline(ig_ctx *ctx, int D, int H, int n_cal, const float *Wq, const float *Wk,
                    const float *bq, const float *bk, const float *Qcal, float *A, float *sigma,
                    float *Wq_s, float *Wk_s, float *bq_s, float *bk_s);

/* Partial weight index generation (Section 4.3 "Prefill Stage"): per head, the
 * r = floor(ratio*d) columns with the largest sum over rows of |Qs| + |Ks| (Ks NULL: |Qs| only).
 * Qs, Ks [n, H*d] skewed queries / keys.  idx [H, r] ascending (NULL: only r_out is written).
 * Ties go to the lower column. */
int ig_partial_index(ig_ctx *ctx, int H, int d, int n, const float *Qs, const float *Ks,
                     double ratio, int32_t *idx, int32_t *r_out);

/* Skewed image of a set of rows (Section 4.2, Eq. 2: Q~ = Q A per head): Y[i, h*d:(h+1)*d] =
 * X[i, h*d:(h+1)*d] * A_h.  X, Y host float32 [n, H*d] (Y may be X), A host float32 [H,d,d].
 * Used for the inputs of ig_partial_index (the prompt's skewed queries / keys). */
int ig_apply_skew(ig_ctx *ctx, int H, int d, int n, const float *X, const float *A, float *Y);

/* Rotary embedding of host rows q [n, H, d] in place, row i at position pos[i] (host int32 [n]),
 * with the pairing and angle the rehearsal of a rotary model applies itself (pairs (c, c + d/2),
 * angle pos * theta^(-2c/d), double arithmetic): what a caller needs to prepare calibration queries
 * for ig_skew_offline or a real query on the host for a model with desc->rope == 1
 * (Section 4.2 decomposes the query matrix the model really produces). */
int ig_rope_rows(ig_ctx *ctx, int n, int H, int d, const int32_t *pos, double theta, float *q);

/* Offline skewing on the GPU: the same A [H,d,d] and sigma [H,d] (may be NULL) as ig_skew_offline,
 * from device arrays (Qcal float32 [n_cal, D]); d even, at most 256.  All arithmetic in double;
 * a fixed number of parallel Jacobi sweeps; if they leave off-diagonal mass above tolerance the
 * next ig_check_status returns IG_ENOCONV.  Allocates a double-precision workspace on first use.
 * The weights are skewed by the caller (W~ = W * blockdiag(A)), a plain batched product. */
int ig_skew_device(ig_ctx *ctx, int D, int H, int n_cal, const float *Qcal, float *A, float *sigma,
                   void *stream);

/* The same index generation on the GPU, for a prompt whose skewed queries / keys are device
 * arrays Qs, Ks [n, H*d] of `dtype` (Ks may be NULL): idx_dev receives int32 [H, r],
 * r = floor(ratio*d), d <= 256.  Sums are float32 in a fixed order (repeatable bit for bit); two
 * columns whose sums agree to float32 rounding may rank differently than in ig_partial_index.
 * Uses (and may grow, which allocates and synchronises) the context's projection workspace: a
 * prefill-time call, not to be issued between ig_reserve and a captured decode step. */
int ig_partial_index_device(ig_ctx *ctx, int dtype, int H, int d, int n, const void *Qs,
                            const void *Ks, double ratio, int32_t *idx_dev, void *stream);

/* ---- setup on the device ------------------------------------------------------------------ */

/* Partial query weight (Section 4.3 "Prefill Stage"): the kept columns of the skewed query
 * weight, stored in a library-defined layout.  Wq: device [D, D] of desc->dtype -- the skewed
 * W~_Q when desc->rope == 0, the original W_Q when desc->rope == 1 (all columns are kept then
 * and idx_dev is ignored).  idx_dev: device int32 [H, r].  wq: device, ig_wq_bytes(desc) bytes,
 * 16-byte aligned. */
size_t ig_wq_bytes(const ig_desc *desc);
int ig_wq_build(ig_ctx *ctx, const ig_desc *desc, const void *Wq, const int32_t *idx_dev, void *wq,
                void *stream);

/* Partial key cache ("slab", Section 4.3 "Prefill Stage"): columns idx of the skewed keys of all
 * cached tokens, stored in a library-defined layout.  Kpool: [B, H, N_cap, d] skewed keys of
 * desc->dtype, in device memory or pinned host memory (pool_space).  slab: device,
 * ig_slab_bytes(desc) bytes, 16-byte aligned.  Tokens N..N_cap-1 are stored as zeros. */
size_t ig_slab_bytes(const ig_desc *desc);
int ig_slab_build(ig_ctx *ctx, const ig_desc *desc, const void *Kpool, int pool_space,
                  const int32_t *idx_dev, void *slab, void *stream);

/* Append of the token just decoded (Section 2.1: its key and value join the cache; Section 4.4:
 * the partial key cache on the GPU is updated with it).  `desc` describes the cache before the
 * append (N valid tokens, N < N_cap, else IG_ECAPACITY; N = 0 is allowed): k_new, v_new (device
 * [B,H,d], 16-byte aligned; the key already skewed) are written to slot N of Kpool / Vpool (device
 * or pinned host memory, [B,H,N_cap,d]) and the kept channels idx_dev of k_new to token N of the
 * slab.  Afterwards the caller uses N + 1. */
int ig_append_token(ig_ctx *ctx, const ig_desc *desc, const void *k_new, const void *v_new,
                    const int32_t *idx_dev, void *slab, void *Kpool, void *Vpool, int pool_space,
                    void *stream);

/* KV cache pool management, counter-based policy (Section 4.4).  counters: device int32
 * [B*H, N_cap], one per pool slot, zero-initialised by the caller.
 *   ig_pool_touch    +1 (saturating at counter_max) for every slot a list names, i.e. for every
 *                    prefetched entry; a pool in which a counter reached counter_max has all its
 *                    counters halved after the increments.  counter_max >= 1 (255: 8-bit counters).
 *   ig_pool_victim   victim[b*H+h] = the slot with the smallest count among the N valid slots of
 *                    that pool, the lowest slot on ties.  victim: device int32 [B*H].
 *   ig_pool_replace  overwrites slot victim[b*H+h] of every pool with the new token: K and V rows
 *                    in Kpool / Vpool (device or pinned host), the kept key channels in the slab;
 *                    the slot's counter restarts at zero (counters may be NULL).  Slots outside
 *                    [0, N_cap) are skipped.  k_new, v_new as in ig_append_token. */
int ig_pool_touch(ig_ctx *ctx, const ig_desc *desc, const int32_t *sel_idx, int32_t sel_stride,
                  const int32_t *sel_cnt, int32_t *counters, int32_t counter_max, void *stream);
int ig_pool_victim(ig_ctx *ctx, const ig_desc *desc, const int32_t *counters, int32_t *victim,
                   void *stream);
int ig_pool_replace(ig_ctx *ctx, const ig_desc *desc, const int32_t *victim, const void *k_new,
                    const void *v_new, const int32_t *idx_dev, void *slab, void *Kpool, void *Vpool,
                    int pool_space, int32_t *counters, void *stream);

/* The same management with a choice of policy (Section 4.4, Table 2: FIFO and LRU are the policies
 * the counter-based one is compared with).  `state`: device int32 [B*H, N_cap], one word per slot:
 *   IG_POLICY_COUNTER  the prefetch counters above (param = counter_max; now is ignored);
 *   IG_POLICY_FIFO     the step at which the slot's entry was written (the caller initialises the
 *                      prompt's entries with their token positions, so that the first token is the
 *                      oldest); being prefetched changes nothing, ig_pool_touch_policy returns at
 *                      once (param ignored);
 *   IG_POLICY_LRU      the step at which the slot's entry was last prefetched or written
 *                      (param = the current step).
 * Steps are int32 values the caller supplies, non-decreasing; a step's prefetches should carry a
 * smaller value than its insertion (2*step and 2*step + 1, say) if the new entry is to count as
 * more recent than the entries prefetched in that step.  For FIFO and LRU the victim is the slot
 * with the smallest stamp, i.e. ig_pool_victim on `state`: it is the same minimum, the lowest slot
 * on ties.  ig_pool_replace_policy overwrites the victim like ig_pool_replace and restarts its word
 * at 0 (counter) or `now` (FIFO, LRU). */
int ig_pool_touch_policy(ig_ctx *ctx, const ig_desc *desc, int policy, const int32_t *sel_idx,
                         int32_t sel_stride, const int32_t *sel_cnt, int32_t *state, int32_t param,
                         void *stream);
int ig_pool_replace_policy(ig_ctx *ctx, const ig_desc *desc, int policy, const int32_t *victim,
                           const void *k_new, const void *v_new, const int32_t *idx_dev, void *slab,
                           void *Kpool, void *Vpool, int pool_space, int32_t *state, int32_t now,
                           void *stream);

/* ---- hot path ----------------------------------------------------------------------------- */

/* Attention rehearsal of the next layer (Section 4.3 "Decoding Stage"):
 *   q_p[b,h,:]   = x[b,:] . (partial query weight of head h) (+ bias)
 *                  (rope: q = x W_Q (+ bias), rotated at pos[b], then q . A_p[h])
 *   s[b,h,t]     = scale * q_p[b,h,:] . slab[b,h,t,:]                     t < N
 *   S[b,h]       = { t : s[b,h,t] >= max_t s[b,h,t] - alpha }, ascending t
 * x: device [B, D] of desc->dtype, the previous layer's normalised attention input.
 * wq: from ig_wq_build.  bias: device float32, [H*r] (rope 0: skewed bias at the kept columns) or
 * [D] (rope 1), or NULL.  A_p: device float32 [H, d, r], kept columns of each head's skewing
 * matrix (rope 1 only, else NULL).  pos: device int32 [B], current position of each sequence
 * (rope 1 only).  slab: from ig_slab_build.
 * Out: sel_idx device int32 [B*H, sel_stride], sel_cnt device int32 [B*H].  A list longer than
 * sel_stride is clamped to its first sel_stride tokens and flagged (ig_check_status).
 * scores_opt: NULL, or device float32 [B, H, N] that receives s. */
int ig_speculate(ig_ctx *ctx, const ig_desc *desc, const void *x, const void *wq,
                 const float *bias, const float *A_p, const int32_t *pos, const void *slab,
                 int32_t *sel_idx, int32_t sel_stride, int32_t *sel_cnt, float *scores_opt,
                 void *stream);

/* The two stages of ig_speculate on their own (same definitions, same kernels): ig_project writes
 * the unscaled partial queries q_p, device float32 [B, H, r]; ig_scan_select consumes them. */
int ig_project(ig_ctx *ctx, const ig_desc *desc, const void *x, const void *wq, const float *bias,
               const float *A_p, const int32_t *pos, float *q_p, void *stream);
int ig_scan_select(ig_ctx *ctx, const ig_desc *desc, const float *q_p, const void *slab,
                   int32_t *sel_idx, int32_t sel_stride, int32_t *sel_cnt, float *scores_opt,
                   void *stream);

/* Index-only partial weight (Section 6.2 "Memory Consumption": only the column indices of the
 * partial query weight are stored and the columns are taken from the full query weight, which the
 * model keeps on the GPU anyway).  Same definitions as ig_project / ig_speculate with
 * q_p[b,h,j] = bias[h*r+j] + sum_k x[b,k] Wq[k, h*d + idx_dev[h,j]], desc->rope == 0 only (a rotary
 * model's rehearsal uses the full W_Q in ig_speculate already).  Wq: device [D, D] of
 * desc->dtype, the skewed query weight, 16-byte aligned; idx_dev: device int32 [H, r], entries in
 * [0, d) (others are clamped into that range).  No ig_wq_build blob is needed; the weight bytes
 * read per call grow from D*H*r to D*D elements.  Needs d*sizeof(dtype) to be a multiple of 16 and
 * at most 1024 bytes, else IG_ESHAPE.  Float32 sums in a fixed order (repeatable bit for bit),
 * but another order than ig_project's. */
int ig_project_indexed(ig_ctx *ctx, const ig_desc *desc, const void *x, const void *Wq,
                       const int32_t *idx_dev, const float *bias, float *q_p, void *stream);
int ig_speculate_indexed(ig_ctx *ctx, const ig_desc *desc, const void *x, const void *Wq,
                         const int32_t *idx_dev, const float *bias, const void *slab,
                         int32_t *sel_idx, int32_t sel_stride, int32_t *sel_cnt, float *scores_opt,
                         void *stream);

/* Speculation on the CPU with the partial key cache in host memory (Section 6.2 "Memory
 * Consumption": the partial key cache is placed in the CPU and the speculation is performed there
 * after fetching the partial query from the GPU).  The GPU computes the partial query as usual
 * (ig_project) and the caller copies it to the host; this call, synchronous and on host threads,
 * does the rest of ig_speculate: scores, per-head maximum, (max - alpha) threshold, ascending lists.
 * q_p: host float32 [B, H, r], unscaled, as ig_project writes it.  slab_host: host memory holding a
 * partial key cache in the library's layout, i.e. ig_slab_bytes(desc) bytes that ig_slab_build wrote
 * on the device and the caller copied to the host (the GPU then no longer needs its copy).
 * sel_idx: host int32 [B*H, sel_stride], sel_cnt: host int32 [B*H]; scores_opt: NULL or host float32
 * [B, H, N].  threads: host threads to use (0 = all the host reports, at most 64).  Same arithmetic
 * in the same order as the GPU scan, so for the same q_p the scores and lists are those of
 * ig_scan_select bit for bit.  A list longer than sel_stride is clamped and the call returns
 * IG_ECAPACITY.  ctx may be NULL (no message is kept then); no GPU call is made. */
int ig_speculate_host(ig_ctx *ctx, const ig_desc *desc, const float *q_p, const void *slab_host,
                      int32_t *sel_idx, int32_t sel_stride, int32_t *sel_cnt, float *scores_opt,
                      int threads);

/* Rehearsal with head-equalised lists in one call (Section 4.3 "Decoding Stage", closing sentences;
 * Section 5.1 "Key Metric"): ig_speculate followed by ig_equalize_heads, with the same results bit
 * for bit, but for the shapes whose scan keeps a head's scores in one workgroup's registers (half
 * precision, r = 25 or 38, up to 4096 tokens, at least 128 (sequence, head) pairs) the scan kernel
 * itself exchanges the heads' threshold counts and selects each head's top n_b, so no score array
 * is written and no second kernel runs.  Arguments as ig_speculate; max_frac as ig_equalize_heads;
 * sel_idx / sel_cnt receive the EQUALISED lists and counts; thr_cnt_opt: NULL, or device int32
 * [B*H] that receives the per-head threshold counts (must not alias sel_cnt).  Other shapes take
 * the two kernels internally (sel_idx then passes through the threshold lists first and needs
 * sel_stride >= the longest of them for exact counts, i.e. N to be safe).  The exchange between the
 * heads of a sequence uses bounded waits (ig_set_wait_limit) like the split scan. */
int ig_speculate_equalized(ig_ctx *ctx, const ig_desc *desc, const void *x, const void *wq,
                           const float *bias, const float *A_p, const int32_t *pos, const void *slab,
                           double max_frac, int32_t *sel_idx, int32_t sel_stride, int32_t *sel_cnt,
                           int32_t *thr_cnt_opt, void *stream);

/* Head-equalised selection (Section 4.3 "Decoding Stage", closing sentences; Section 5.1 "Key
 * Metric"): every head of a sequence keeps the same number of tokens,
 *   n_b = max(1, min(floor(sum_h thr_cnt[b,h] / H), floor(max_frac * N))),
 * namely its n_b highest-scoring tokens (equal scores: the earlier token first), in ascending t.
 * scores: device float32 [B, H, N], the speculated scores (ig_speculate's scores_opt).
 * thr_cnt: device int32 [B*H], the per-head threshold counts (ig_speculate's sel_cnt, unclamped:
 * taken with sel_stride >= N).  max_frac in (0, 1]; the paper uses 0.2.
 * Out: sel_idx device int32 [B*H, sel_stride], sel_cnt device int32 [B*H] (= n_b; must not alias
 * thr_cnt).  Exact for the scores given (integer work only).  Lists longer than sel_stride are
 * clamped and flagged as in ig_speculate. */
int ig_equalize_heads(ig_ctx *ctx, const ig_desc *desc, const float *scores, const int32_t *thr_cnt,
                      double max_frac, int32_t *sel_idx, int32_t sel_stride, int32_t *sel_cnt,
                      void *stream);

/* Prefetch of the selected rows (Section 4.1 overview; Section 4.3): for j < sel_cnt[b,h]
 *   K_sel[b,h,j,:] = Kpool[b,h,sel_idx[b,h,j],:],  V_sel likewise.
 * Kpool, Vpool: [B, H, N_cap, d] of desc->dtype in device memory (IG_MEM_DEVICE) or in pinned,
 * GPU-mapped host memory (IG_MEM_HOST_PINNED; rows then cross PCIe, and `stream` is normally a
 * side stream so the copy overlaps the previous layer).  K_sel, V_sel: device
 * [B*H, sel_stride, d]; rows j >= sel_cnt are not written.  Row size d*sizeof(dtype) must be a
 * multiple of 16 bytes. */
int ig_gather_kv(ig_ctx *ctx, const ig_desc *desc, const void *Kpool, const void *Vpool,
                 int pool_space, const int32_t *sel_idx, int32_t sel_stride,
                 const int32_t *sel_cnt, void *K_sel, void *V_sel, void *stream);

/* Decode attention over the fetched rows only (Section 2.1, softmax(Q K^T) V per head; Section 4.1):
 *   l_j = scale * q[b,h,:] . K_sel[b,h,j,:], p = softmax_j(l), out[b,h,:] = sum_j p_j V_sel[b,h,j,:]
 * over j < sel_cnt[b,h], plus one always-attended row (k_new, v_new: device [B,H,d], the token
 * being decoded) when both are non-NULL.  q: device [B,H,d], the layer's real skewed query.
 * out: device [B,H,d] of desc->dtype; zeros for an empty list without a new row. */
int ig_sparse_attention(ig_ctx *ctx, const ig_desc *desc, const void *q, const void *K_sel,
                        const void *V_sel, const int32_t *sel_cnt, int32_t sel_stride,
                        const void *k_new, const void *v_new, void *out, void *stream);

/* ig_sparse_attention for callers that cannot allocate device memory: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernel and
 * the same result bit for bit, but the per-slice softmax states and arrival counters live in a
 * static device array of the library (16 MiB on every GPU the library runs on, held until the
 * process ends) instead of context workspaces, and the call makes no hipMalloc / hipFree or other
 * allocating call, whatever the shape and whether or not ig_reserve was called.  Needs
 * 256*ceil(B*H/64) + 64*B*H*(d+2) bytes of that array (B*H = 2000 heads of d = 128 fit); more
 * returns IG_ECAPACITY and launches nothing.  The arrival counters are cleared by a small fill
 * kernel on `stream` before the attention kernel.  All contexts on one GPU share the array: two
 * calls of this entry point that overlap in time on one GPU (different streams or contexts) race;
 * calls on one stream are safe. */
int ig_sparse_attention_static(ig_ctx *ctx, const ig_desc *desc, const void *q, const void *K_sel,
                               const void *V_sel, const int32_t *sel_cnt, int32_t sel_stride,
                               const void *k_new, const void *v_new, void *out, void *stream);

/* Same attention with the index lists applied to a device-resident pool directly (no K_sel /
 * V_sel copy): row j of (b,h) is Kpool[b,h,sel_idx[b,h,j],:]. */
int ig_sparse_attention_indexed(ig_ctx *ctx, const ig_desc *desc, const void *q, const void *Kpool,
                                const void *Vpool, const int32_t *sel_idx, int32_t sel_stride,
                                const int32_t *sel_cnt, const void *k_new, const void *v_new,
                                void *out, void *stream);

/* Prefetch and attention in one pass over a device-resident pool (Section 4.1: the fetched rows
 * are exactly the rows attention reads): every selected row is read from the pool once, written
 * to K_sel / V_sel as ig_gather_kv would (same layout, rows j >= sel_cnt untouched) and used for
 * the attention of ig_sparse_attention_indexed.  All pointers device memory. */
int ig_gather_attention(ig_ctx *ctx, const ig_desc *desc, const void *q, const void *Kpool,
                        const void *Vpool, const int32_t *sel_idx, int32_t sel_stride,
                        const int32_t *sel_cnt, void *K_sel, void *V_sel, const void *k_new,
                        const void *v_new, void *out, void *stream);

/* ---- measurement --------------------------------------------------------------------------- */

/* One slice of a decode step over a device-resident pool (Section 4.1, Fig. 3(d): the next layer
 * is speculated while the current one computes): the rehearsal of the NEXT layer -- x, wq, bias,
 * A_p, pos, slab as in ig_speculate, lists to sel_idx_next / sel_cnt_next -- and the one-pass
 * prefetch + attention of THIS layer -- q, Kpool, Vpool, sel_idx, sel_cnt, K_sel, V_sel, k_new,
 * v_new, out as in ig_gather_attention.  Both list pairs use sel_stride; the two must not
 * alias.  Same results, bit for bit, as ig_speculate (without score dump) followed by
 * ig_gather_attention.  The projection goes out first; the next layer's scan and this layer's
 * attention are independent and, for sequences of at most 4 tiles (2048 half-precision tokens)
 * with enough (sequence, head) pairs, leave as ONE launch; other shapes get the two launches one
 * after the other. */
int ig_layer_step(ig_ctx *ctx, const ig_desc *desc, const void *x, const void *wq, const float *bias,
                  const float *A_p, const int32_t *pos, const void *slab, int32_t *sel_idx_next,
                  int32_t *sel_cnt_next, const void *q, const void *Kpool, const void *Vpool,
                  const int32_t *sel_idx, const int32_t *sel_cnt, int32_t sel_stride, void *K_sel,
                  void *V_sel, const void *k_new, const void *v_new, void *out, void *stream);

/* One decode step over n_layers layers with the KV pool prefetched on a side stream (Section 4.1,
 * Fig. 3(d): the selected rows of layer l cross to the GPU while layer l+1 is already being
 * rehearsed and layer l-1 attended).  For every layer the call enqueues ig_speculate on
 * main_stream, ig_gather_kv on side_stream and ig_sparse_attention on main_stream, with the events
 * that order them, over n_sets >= 2 rotating buffer sets (layer l uses set l % n_sets).
 * layers: host array [n_layers]; x, slab, q, Kpool, Vpool, out of a layer as in the three calls,
 * k_new / v_new NULL or the always-attended row.  sets: host array [n_sets] of device buffers
 * (sel_idx [B*H, sel_stride], sel_cnt [B*H], K_sel / V_sel [B*H, sel_stride, d]).  wq, bias, A_p,
 * pos as ig_speculate (one model: the same for every layer here; callers with per-layer weights
 * issue the three calls themselves).  The two streams must differ and have the default priority;
 * the context keeps a second context for the side stream's workspaces and the events, created on
 * the first call (so the first call allocates; calls for larger shapes may too).  Nothing is
 * synchronised: when the call returns everything is enqueued, and main_stream's last work depends
 * on side_stream's. */
typedef struct {
  const void *x, *slab, *q, *Kpool, *Vpool, *k_new, *v_new;
  void *out;
} ig_layer_io;
typedef struct {
  int32_t *sel_idx, *sel_cnt;
  void *K_sel, *V_sel;
} ig_buffer_set;
int ig_decode_step_overlapped(ig_ctx *ctx, const ig_desc *desc, int n_layers, const ig_layer_io *layers,
                              const void *wq, const float *bias, const float *A_p, const int32_t *pos,
                              int pool_space, int n_sets, const ig_buffer_set *sets, int32_t sel_stride,
                              void *main_stream, void *side_stream);

/* Long sequences are scanned by several workgroups per (sequence, head), which meet through device
 * memory; each waits for its partners at most `ticks` periods of the GPU's 100 MHz clock (10 ns)
 * and then finishes the pair on its own (slower, same result bit for bit).  0 restores the
 * default (20 ms); a negative value makes every such workgroup take the self-sufficient route
 * without waiting at all -- the hook the tests use to exercise that route. */
int ig_set_wait_limit(ig_ctx *ctx, int64_t ticks);

/* Between ig_profile_begin and ig_profile_end every kernel the context launches carries a pair of
 * HIP events that take the kernel's own start and stop timestamps.  ig_profile_end synchronises
 * the device and stops recording; ig_profile_read then returns, for kernel id `which`
 * (IG_K_*), the summed duration in milliseconds and the number of launches. */
int ig_profile_begin(ig_ctx *ctx);
int ig_profile_end(ig_ctx *ctx);
int ig_profile_read(ig_ctx *ctx, int which, double *total_ms, int32_t *launches);

/* Plain device-to-device copy kernel of `bytes` bytes (multiple of 16); used to scale hardware
 * counters against a transfer of known size and to measure the achievable HBM rate. */
int ig_copy_bytes(ig_ctx *ctx, const void *src, void *dst, size_t bytes, void *stream);

/* Plain streaming read of `bytes` bytes (multiple of 16) of device memory, nothing written: the
 * read rate this GPU sustains for a buffer of that size, measured beside the scan. */
int ig_read_bytes(ig_ctx *ctx, const void *src, size_t bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* INFINIGEN_H */
