"""After ig_reserve the hot-path calls must not allocate device memory: the context's workspace total
(ig_workspace_bytes) and the free device memory read from the driver are the same before and after
the calls, for a shape of every scan form (registers, LDS-parked scores, one wave per tile), for a
capacity larger than the valid length that later fills up, and for the index-only and per-layer
entry points.  Without ig_reserve the same calls do grow the workspaces (the check is live)."""
import pytest
import torch

import ig_workloads as wl
from ig_case import make_case

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("cfg,kw,N_cap", [
    (2, dict(B=3, H=4, N=1500), 2048),                      # registers, 4 waves
    (2, dict(B=8, H=16, d=32, N=5000), 6000),               # registers, 16 waves
    (2, dict(B=8, H=8, d=32, N=9000), 12000),               # scores parked in LDS
    (5, dict(B=1, H=2, N=9000), 20000),                     # one wave per tile, rotary (finalisation kernel)
    (3, dict(B=2, H=4, N=2000), 2048),                      # rotary prologue inside the scan
    (2, dict(B=4, H=32, N=1500), 2048),                     # streaming form; equalised lists built by the scan
    (3, dict(B=4, H=32, N=3000), 4096),                     # the same with the rotary prologue
])
def test_no_allocation_after_reserve(cfg, kw, N_cap):
    import paper_2406_19707_amd as ig
    from ig_gpu import Uploaded, desc_of
    w = wl.shrink(wl.WORKLOADS[cfg], n_cal=max(64, 2 * kw.get("d", 128)), heavy_count=12, **kw)
    c = make_case(w, gain=8.0, N_cap=N_cap)
    ctx = ig.Context(0)
    up = Uploaded(ctx, c)
    d = up.desc
    BH, stride = w.B * w.H, N_cap
    tdt = torch.float32 if w.dtype == "f32" else torch.float16
    idx = [torch.zeros((BH, stride), dtype=torch.int32, device="cuda") for _ in range(2)]
    cnt = [torch.zeros(BH, dtype=torch.int32, device="cuda") for _ in range(2)]
    scores = torch.zeros((w.B, w.H, N_cap), device="cuda")
    Ks, Vs = (torch.zeros((BH, stride, w.d), dtype=tdt, device="cuda") for _ in range(2))
    out = torch.zeros((w.B, w.H, w.d), dtype=tdt, device="cuda")
    q_p = torch.zeros((w.B, w.H, c.r), device="cuda")

    def calls(ctx, N):
        d.N = N
        ctx.ig_project(d, up.x, up.wq, up.bias, up.A_p, up.pos, q_p)
        ctx.ig_speculate(d, up.x, up.wq, up.bias, up.A_p, up.pos, up.slab, idx[0], stride, cnt[0], scores)
        ctx.ig_speculate(d, up.x, up.wq, up.bias, up.A_p, up.pos, up.slab, idx[0], stride, cnt[0], None)
        ctx.ig_equalize_heads(d, scores, cnt[0], 0.2, idx[1], stride, cnt[1])
        ctx.ig_speculate_equalized(d, up.x, up.wq, up.bias, up.A_p, up.pos, up.slab, 0.2, idx[1], stride, cnt[1])
        ctx.ig_speculate_equalized(d, up.x, up.wq, up.bias, up.A_p, up.pos, up.slab, 0.2, idx[1], stride, cnt[1], cnt[0])
        ctx.ig_gather_kv(d, up.K, up.V, up.space, idx[0], stride, cnt[0], Ks, Vs)
        ctx.ig_sparse_attention(d, up.q, Ks, Vs, cnt[0], stride, up.k_new, up.v_new, out)
        ctx.ig_gather_attention(d, up.q, up.K, up.V, idx[0], stride, cnt[0], Ks, Vs, None, None, out)
        ctx.ig_layer_step(d, up.x, up.wq, up.bias, up.A_p, up.pos, up.slab, idx[1], cnt[1], up.q, up.K, up.V,
                          idx[0], cnt[0], stride, Ks, Vs, None, None, out)
        if not w.rope:
            ctx.ig_speculate_indexed(d, up.x, up.W, up.idx, up.bias, up.slab, idx[1], stride, cnt[1], None)
        torch.cuda.synchronize()
        assert ctx.ig_check_status() == ig.IG_OK

    lengths = (c.N, min(N_cap, c.N + 700), N_cap)           # the valid length grows up to the capacity
    # a first context runs everything once, so that the runtime has loaded every kernel's code
    for N in lengths:
        calls(ctx, N)
    assert ctx.ig_workspace_bytes() > 0                      # this context grew its workspaces call by call
    ctx2 = ig.Context(0)
    assert ctx2.ig_workspace_bytes() == 0
    d.N = c.N
    ctx2.ig_reserve(d)
    torch.cuda.synchronize()
    held = ctx2.ig_workspace_bytes()
    free0 = torch.cuda.mem_get_info()[0]
    for N in lengths:
        calls(ctx2, N)
        assert ctx2.ig_workspace_bytes() == held, f"workspaces grew after ig_reserve at N = {N}"
    free1 = torch.cuda.mem_get_info()[0]
    assert free1 == free0, f"device memory changed by {free0 - free1} bytes after ig_reserve"
    ctx2.close()
    ctx.close()
