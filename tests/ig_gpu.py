"""Runs one Case through the HIP library (C ABI via the Python binding) and returns numpy outputs."""
from __future__ import annotations

import numpy as np
import torch

import paper_2406_19707_amd as ig


def desc_of(c, alpha=None, N=None):
    w = c.w
    return ig.IgDesc(B=w.B, H=w.H, d=w.d, r=c.r, N=c.N if N is None else N, N_cap=c.N_cap,
                     dtype=ig.IG_F32 if w.dtype == "f32" else ig.IG_F16, scale=c.scale,
                     alpha=w.alpha if alpha is None else alpha, rope=1 if w.rope else 0)


def dev(a):
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a)).cuda()


class Uploaded:
    """Device-side copies of a Case plus the library-layout buffers built from them."""

    def __init__(self, ctx, c, host_pool=False, alpha=None):
        self.ctx, self.c = ctx, c
        self.desc = desc_of(c, alpha)
        w = c.w
        self.x, self.W = dev(c.x), dev(c.W_in)
        self.idx = dev(c.idx)
        self.bias = dev(c.bias_in)
        self.A_p = dev(c.A_p) if w.rope else None
        self.pos = dev(c.pos) if w.rope else None
        if host_pool:
            self.K = torch.from_numpy(c.Kt).pin_memory()
            self.V = torch.from_numpy(c.V).pin_memory()
            self.space = ig.IG_MEM_HOST_PINNED
        else:
            self.K, self.V = dev(c.Kt), dev(c.V)
            self.space = ig.IG_MEM_DEVICE
        self.q, self.k_new, self.v_new = dev(c.q), dev(c.k_new), dev(c.v_new)
        self.wq = torch.empty(ig.ig_wq_bytes(self.desc), dtype=torch.uint8, device="cuda")
        self.slab = torch.empty(ig.ig_slab_bytes(self.desc), dtype=torch.uint8, device="cuda")
        ctx.ig_wq_build(self.desc, self.W, self.idx, self.wq)
        ctx.ig_slab_build(self.desc, self.K, self.space, self.idx, self.slab)
        torch.cuda.synchronize()


def run_gpu(ctx, c, alpha=None, sel_stride=None, host_pool=False, want_scores=True, up=None):
    w = c.w
    up = up or Uploaded(ctx, c, host_pool, alpha)
    d = up.desc
    BH = w.B * w.H
    stride = c.N if sel_stride is None else sel_stride
    tdt = torch.float32 if w.dtype == "f32" else torch.float16
    q_p = torch.full((w.B, w.H, c.r), float("nan"), device="cuda")
    scores = torch.full((w.B, w.H, c.N), float("nan"), device="cuda") if want_scores else None
    sel_idx = torch.full((BH, stride), -1, dtype=torch.int32, device="cuda")
    sel_cnt = torch.full((BH,), -1, dtype=torch.int32, device="cuda")
    K_sel = torch.zeros((BH, stride, w.d), dtype=tdt, device="cuda")
    V_sel = torch.zeros((BH, stride, w.d), dtype=tdt, device="cuda")
    out = torch.full((w.B, w.H, w.d), float("nan"), dtype=tdt, device="cuda")
    out_new = torch.full_like(out, float("nan"))
    out_idx = torch.full_like(out, float("nan"))
    ctx.ig_project(d, up.x, up.wq, up.bias, up.A_p, up.pos, q_p)
    ctx.ig_speculate(d, up.x, up.wq, up.bias, up.A_p, up.pos, up.slab, sel_idx, stride, sel_cnt, scores)
    ctx.ig_gather_kv(d, up.K, up.V, up.space, sel_idx, stride, sel_cnt, K_sel, V_sel)
    ctx.ig_sparse_attention(d, up.q, K_sel, V_sel, sel_cnt, stride, None, None, out)
    ctx.ig_sparse_attention(d, up.q, K_sel, V_sel, sel_cnt, stride, up.k_new, up.v_new, out_new)
    out_one = torch.full_like(out, float("nan"))
    out_one_new = torch.full_like(out, float("nan"))
    K_one, V_one = torch.zeros_like(K_sel), torch.zeros_like(V_sel)
    if not host_pool:
        ctx.ig_sparse_attention_indexed(d, up.q, up.K, up.V, sel_idx, stride, sel_cnt, None, None, out_idx)
        ctx.ig_gather_attention(d, up.q, up.K, up.V, sel_idx, stride, sel_cnt, K_one, V_one, None, None,
                                out_one)
        ctx.ig_gather_attention(d, up.q, up.K, up.V, sel_idx, stride, sel_cnt, K_one, V_one, up.k_new,
                                up.v_new, out_one_new)
    torch.cuda.synchronize()
    status = ctx.ig_check_status()
    res = dict(q_p=q_p.cpu().numpy(), scores=None if scores is None else scores.cpu().numpy(),
               sel_idx=sel_idx.cpu().numpy(), sel_cnt=sel_cnt.cpu().numpy(),
               K_sel=K_sel.cpu().numpy(), V_sel=V_sel.cpu().numpy(),
               out=out.float().cpu().numpy().reshape(BH, w.d),
               out_new=out_new.float().cpu().numpy().reshape(BH, w.d),
               out_idx=None if host_pool else out_idx.float().cpu().numpy().reshape(BH, w.d),
               out_one=None if host_pool else out_one.float().cpu().numpy().reshape(BH, w.d),
               out_one_new=None if host_pool else out_one_new.float().cpu().numpy().reshape(BH, w.d),
               K_one=None if host_pool else K_one.cpu().numpy(),
               V_one=None if host_pool else V_one.cpu().numpy(),
               status=status, up=up)
    return res


def run_gpu_on_lists(ctx, c, up, sel_idx_host, sel_cnt_host, host_pool=False):
    """Prefetch and attention of the HIP path on index lists given by the caller (the oracle's)."""
    w = c.w
    d = up.desc
    BH = w.B * w.H
    stride = sel_idx_host.shape[1]
    tdt = torch.float32 if w.dtype == "f32" else torch.float16
    sel_idx, sel_cnt = dev(sel_idx_host.astype(np.int32)), dev(sel_cnt_host.astype(np.int32))
    K_sel = torch.zeros((BH, stride, w.d), dtype=tdt, device="cuda")
    V_sel = torch.zeros_like(K_sel)
    out = torch.full((w.B, w.H, w.d), float("nan"), dtype=tdt, device="cuda")
    out_new, out_idx, out_one = torch.full_like(out, float("nan")), None, None
    ctx.ig_gather_kv(d, up.K, up.V, up.space, sel_idx, stride, sel_cnt, K_sel, V_sel)
    ctx.ig_sparse_attention(d, up.q, K_sel, V_sel, sel_cnt, stride, None, None, out)
    ctx.ig_sparse_attention(d, up.q, K_sel, V_sel, sel_cnt, stride, up.k_new, up.v_new, out_new)
    if not host_pool:
        out_idx, out_one = torch.full_like(out, float("nan")), torch.full_like(out, float("nan"))
        K_one, V_one = torch.zeros_like(K_sel), torch.zeros_like(V_sel)
        ctx.ig_sparse_attention_indexed(d, up.q, up.K, up.V, sel_idx, stride, sel_cnt, None, None, out_idx)
        ctx.ig_gather_attention(d, up.q, up.K, up.V, sel_idx, stride, sel_cnt, K_one, V_one, None, None, out_one)
    torch.cuda.synchronize()
    assert ctx.ig_check_status() == 0
    f = lambda t: None if t is None else t.float().cpu().numpy().reshape(BH, w.d)   # noqa: E731
    return dict(K_sel=K_sel.float().cpu().numpy(), V_sel=V_sel.float().cpu().numpy(), out=f(out),
                out_new=f(out_new), out_idx=f(out_idx), out_one=f(out_one))
