"""GPU test of ig_layer_step: the next layer's rehearsal and this layer's one-pass prefetch +
attention through one entry point (the scan and the attention as one launch where the shape allows)
must give, bit for bit, what ig_speculate followed by ig_gather_attention give; the lists are also
compared with the CPU oracle under the usual band rule."""
import numpy as np
import pytest
import torch

import ig_workloads as wl
from ig_case import make_case, run_oracle, compare_selection

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    import paper_2406_19707_amd as ig
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    c = ig.Context(0)
    yield c
    c.close()


def check_layer_step(ctx, w, gain, bias=False, N_cap=None, with_new_row=False):
    import paper_2406_19707_amd as ig
    from ig_gpu import Uploaded
    this, nxt = make_case(w, gain=gain, layer=0, bias=bias, N_cap=N_cap), make_case(w, gain=gain, layer=1, bias=bias, N_cap=N_cap)
    print(f"layer-step case {w.name} B{w.B} H{w.H} d{w.d} N{this.N}/{this.N_cap} r{this.r} {w.dtype} "
          f"rope={w.rope} new_row={with_new_row}", flush=True)
    up0, up1 = Uploaded(ctx, this), Uploaded(ctx, nxt)
    d = up0.desc
    BH, stride = w.B * w.H, this.N
    tdt = torch.float32 if w.dtype == "f32" else torch.float16
    new = lambda *shape, dt=torch.int32, fill=-1: torch.full(shape, fill, dtype=dt, device="cuda")   # noqa: E731
    # reference: the separate entry points
    idx0, cnt0 = new(BH, stride), new(BH)
    ctx.ig_speculate(d, up0.x, up0.wq, up0.bias, up0.A_p, up0.pos, up0.slab, idx0, stride, cnt0, None)
    idx1_ref, cnt1_ref = new(BH, stride), new(BH)
    ctx.ig_speculate(d, up1.x, up1.wq, up1.bias, up1.A_p, up1.pos, up1.slab, idx1_ref, stride, cnt1_ref, None)
    K_ref, V_ref = new(BH, stride, w.d, dt=tdt, fill=0), new(BH, stride, w.d, dt=tdt, fill=0)
    out_ref = new(w.B, w.H, w.d, dt=tdt, fill=float("nan"))
    kn, vn = (up0.k_new, up0.v_new) if with_new_row else (None, None)
    ctx.ig_gather_attention(d, up0.q, up0.K, up0.V, idx0, stride, cnt0, K_ref, V_ref, kn, vn, out_ref)
    # the joint entry point, twice (the per-(b,h) counters must be back at zero after a call)
    for rep in range(2):
        idx1, cnt1 = new(BH, stride), new(BH)
        K_sel, V_sel = new(BH, stride, w.d, dt=tdt, fill=0), new(BH, stride, w.d, dt=tdt, fill=0)
        out = new(w.B, w.H, w.d, dt=tdt, fill=float("nan"))
        ctx.ig_layer_step(d, up1.x, up1.wq, up1.bias, up1.A_p, up1.pos, up1.slab, idx1, cnt1,
                          up0.q, up0.K, up0.V, idx0, cnt0, stride, K_sel, V_sel, kn, vn, out)
        torch.cuda.synchronize()
        assert ctx.ig_check_status() == ig.IG_OK
        assert torch.equal(cnt1, cnt1_ref) and torch.equal(idx1, idx1_ref), rep
        assert torch.equal(K_sel, K_ref) and torch.equal(V_sel, V_ref), rep
        assert torch.equal(out.view(torch.uint8), out_ref.view(torch.uint8)), rep
    ref1 = run_oracle(nxt, attend=False)
    slack = compare_selection(idx1.cpu().numpy(), cnt1.cpu().numpy(), ref1, w.alpha)
    print(f"  next layer's lists against the oracle: in-band differences {slack}", flush=True)


@pytest.mark.parametrize("N,N_cap,new_row", [(2048, 2048, False), (1500, 2048, True), (300, 4096, False)])
def test_cfg2_shape_joint_launch(ctx, N, N_cap, new_row):
    w = wl.shrink(wl.WORKLOADS[2], B=3, H=4, N=N, heavy_count=min(20, N))
    check_layer_step(ctx, w, gain=6.0, N_cap=N_cap, with_new_row=new_row)


def test_many_pairs_heavy_lists_joint_launch(ctx):
    # 16 x 16 = 256 pairs with a few thousand kept rows in some lists: multi-slice attention next to the scan
    w = wl.shrink(wl.WORKLOADS[2], B=16, H=16, d=32, N=2048, heavy_count=30)
    check_layer_step(ctx, w, gain=3.0, bias=True)


def test_rotary_joint_launch(ctx):
    w = wl.shrink(wl.WORKLOADS[3], B=2, H=4, N=2000)
    check_layer_step(ctx, w, gain=24.0, with_new_row=True)


def test_f32_joint_launch(ctx):
    w = wl.shrink(wl.WORKLOADS[1], B=2, H=4, N=900, heavy_count=10)      # 4 tiles of 256 floats
    check_layer_step(ctx, w, gain=8.0)


@pytest.mark.parametrize("cfg,B,H,d,N,gain", [(2, 8, 16, 32, 3000, 6.0), (3, 2, 4, 128, 4096, 24.0), (5, 1, 2, 128, 9000, 6.0)])
def test_shapes_that_take_two_launches(ctx, cfg, B, H, d, N, gain):
    w = wl.shrink(wl.WORKLOADS[cfg], B=B, H=H, d=d, N=N, n_cal=max(64, 3 * d), heavy_count=20)
    check_layer_step(ctx, w, gain=gain)


def test_error_paths(ctx):
    import paper_2406_19707_amd as ig
    from ig_gpu import Uploaded
    w = wl.shrink(wl.WORKLOADS[2], B=2, H=2, N=256)
    c = make_case(w, gain=6.0)
    up = Uploaded(ctx, c)
    BH = w.B * w.H
    idx, cnt = torch.zeros((BH, c.N), dtype=torch.int32, device="cuda"), torch.zeros(BH, dtype=torch.int32, device="cuda")
    Ks = torch.zeros((BH, c.N, w.d), dtype=torch.float16, device="cuda")
    out = torch.zeros((w.B, w.H, w.d), dtype=torch.float16, device="cuda")
    with pytest.raises(ig.IgError):      # the next layer's lists alias this layer's
        ctx.ig_layer_step(up.desc, up.x, up.wq, None, None, None, up.slab, idx, cnt, up.q, up.K, up.V, idx, cnt,
                          c.N, Ks, Ks.clone(), None, None, out)
    with pytest.raises(ig.IgError):      # missing output
        ctx.ig_layer_step(up.desc, up.x, up.wq, None, None, None, up.slab, idx.clone(), cnt.clone(), up.q, up.K,
                          up.V, idx, cnt, c.N, Ks, Ks.clone(), None, None, None)
    torch.cuda.synchronize()
    assert ctx.ig_check_status() == ig.IG_OK
