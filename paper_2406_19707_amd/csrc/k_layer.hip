// One launch for two independent pieces of a decode step (Section 4.1, Fig. 3(d): the next layer
// is speculated while the current one computes): the scan / threshold / list kernel of the NEXT
// layer's rehearsal and the one-pass prefetch + attention of THIS layer.  The scan needs the next
// layer's projection sums (the launch before this one) and the attention needs this layer's index
// lists (the launch of the previous step), so neither depends on the other, and both are short,
// latency-bound kernels: run as the two halves of one grid they share the launch and overlap fully,
// without streams or events between them.  Workgroups [0, B*H) run the scan body (4 waves, one
// tile each), the remaining B*H*SLICE_MAX run the attention body; the bodies are those of the
// stand-alone kernels, so the results are the same bit for bit.
#include "scan_device.h"
#include "attn_device.h"

namespace {

template <typename T, int CH>
__global__ __launch_bounds__(256) void scan_next_attend_this(ScanArgs sa, AttnArgs aa, int scan_blocks) {
  if ((int)blockIdx.x < scan_blocks)
    scan_select_fused_body<T, CH, 4>(sa, blockIdx.x);
  else
    sparse_attention_body<T, true>(aa, (int)blockIdx.x - scan_blocks);
}

template <typename T>
int launch_t(ig_ctx *ctx, const ScanArgs &sa, const AttnArgs &aa, int BH, int ch, hipStream_t s) {
  dim3 grid(BH + BH * SLICE_MAX), block(256);
#define CASE(CHV)                                                              \
  case CHV: {                                                                  \
    auto k = scan_next_attend_this<T, CHV>;                                    \
    IG_LAUNCH(ctx, IG_K_LAYER, k, grid, block, s, sa, aa, BH);                 \
    return IG_OK;                                                              \
  }
  switch (ch) {
    CASE(4) CASE(8) CASE(12)
    default: break;
  }
#undef CASE
  return ig_fail(ctx, IG_ESHAPE, "layer step: unsupported channel block %d", ch);
}

}  // namespace

// The joint launch takes the shapes whose scan is the 4-wave one-workgroup-per-(b,h) form.
bool ig_layer_step_is_joint(const ig_desc *d) {
  const int tile = ig_tile_tokens(d->dtype);
  return ig_scan_is_fused(d) && (d->N + tile - 1) / tile <= 4;
}

int ig_launch_scan_attend(ig_ctx *ctx, const ig_desc *d, const QSource &qs, const void *slab,
                          int32_t *sel_idx_next, int32_t *sel_cnt_next, const void *q,
                          const void *Kpool, const void *Vpool, const int32_t *sel_idx,
                          const int32_t *sel_cnt, int32_t sel_stride, const void *k_new,
                          const void *v_new, void *out, void *K_sel, void *V_sel, hipStream_t s) {
  ScanArgs sa;
  int rc = ig_scan_args(ctx, d, qs, slab, sel_idx_next, sel_stride, sel_cnt_next, nullptr, &sa);
  if (rc) return rc;
  AttnArgs aa;
  if ((rc = ig_attn_args(ctx, d, q, Kpool, Vpool, sel_idx, sel_stride, sel_cnt, d->N_cap, k_new, v_new, out,
                         K_sel, V_sel, &aa)))
    return rc;
  // at most 12 channel loads in flight per wave: the scan half then needs fewer registers than
  // the attention half, so the joint kernel keeps the attention's occupancy (measured on the
  // B8 H32 N2048 shape: 20.4-20.8 us per launch against 22.2-22.4 us with 20 loads in flight)
  const int ch = ig_pick_ch(d->r, 12);
  const int BH = d->B * d->H;
  return d->dtype == IG_F16 ? launch_t<half_t>(ctx, sa, aa, BH, ch, s) : launch_t<float>(ctx, sa, aa, BH, ch, s);
}
