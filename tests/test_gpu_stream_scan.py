"""GPU parity of the streaming scan form (rolling load window; long pairs split over several
workgroups that meet through device memory) against the CPU oracle, through the C ABI.

The form is built for the kept-channel counts of the workloads (r = 38: ratio 0.3 of d = 128, here
0.6 of d = 64; r = 25: ratio 0.2 of d = 128, here 0.4 of d = 64), so the shapes below use those.
Same bars as tests/test_gpu_parity.py (its check_case does the comparison)."""
import numpy as np
import pytest
import torch

import ig_workloads as wl
from ig_case import make_case, run_oracle, compare_selection
from test_gpu_parity import check_case

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    import paper_2406_19707_amd as ig
    c = ig.Context(0)
    yield c
    c.close()


def shape(cfg, B, H, N, ratio, **kw):
    return wl.shrink(wl.WORKLOADS[cfg], B=B, H=H, d=64, N=N, ratio=ratio, n_cal=128, heavy_count=24, **kw)


@pytest.mark.parametrize("cfg,B,H,N,N_cap,ratio,gain,bias", [
    (3, 8, 16, 4096, 4096, 0.6, 30.0, False),     # 8 tiles, 128 pairs: one workgroup per pair, two tiles per wave; rotary
    (2, 8, 16, 2700, 3000, 0.6, 12.0, True),      # 6 tiles, ragged last tile, waves with one valid tile, bias
    (2, 2, 8, 9000, 9000, 0.6, 10.0, False),      # 18 tiles, few pairs: 5 workgroups of 4 tiles per pair
    (5, 4, 40, 32768, 32768, 0.4, 40.0, False),   # the long-context shape: 64 tiles, 8 workgroups of 8 tiles; rotary
    (2, 3, 50, 20000, 24000, 0.4, 14.0, False),   # 40 tiles of 47 allocated, 150 pairs, 5 workgroups per pair
    (2, 1, 2, 60000, 60000, 0.6, 20.0, False),    # 118 tiles: 15 workgroups of 8 tiles (4 per workgroup would need 30)
    (2, 1, 2, 130000, 130000, 0.4, 20.0, False),  # 254 tiles: 16 workgroups of 16 tiles
])
def test_streaming_form_against_the_oracle(ctx, cfg, B, H, N, N_cap, ratio, gain, bias):
    w = shape(cfg, B, H, N, ratio)
    c = make_case(w, gain=gain, bias=bias, N_cap=N_cap)
    assert c.r in (25, 38)
    check_case(ctx, c)


def _speculate(ctx, up, c, stride=None):
    w = c.w
    stride = c.N if stride is None else stride
    sel_idx = torch.full((w.B * w.H, stride), -1, dtype=torch.int32, device="cuda")
    sel_cnt = torch.full((w.B * w.H,), -1, dtype=torch.int32, device="cuda")
    ctx.ig_speculate(up.desc, up.x, up.wq, up.bias, up.A_p, up.pos, up.slab, sel_idx, stride, sel_cnt, None)
    torch.cuda.synchronize()
    return sel_idx.cpu().numpy(), sel_cnt.cpu().numpy()


@pytest.mark.parametrize("cfg,B,H,N,ratio,gain", [
    (2, 2, 8, 9000, 0.6, 10.0),        # 5 workgroups per pair, 4 tiles each
    (5, 2, 40, 32768, 0.4, 40.0),      # 8 workgroups per pair, 8 tiles each, rotary
    (2, 1, 2, 130000, 0.4, 20.0),      # 16 workgroups per pair, 16 tiles each
])
def test_self_sufficient_route_gives_the_same_lists(ctx, cfg, B, H, N, ratio, gain):
    """A negative wait limit makes every workgroup of a split pair give up on its partners at once
    and finish the pair alone; the lists must equal those of the ordinary route bit for bit, and
    the per-pair records must be left clean for the next call."""
    import paper_2406_19707_amd as ig
    from ig_gpu import Uploaded
    c = make_case(shape(cfg, B, H, N, ratio), gain=gain)
    up = Uploaded(ctx, c)
    idx0, cnt0 = _speculate(ctx, up, c)
    ctx.ig_set_wait_limit(-1)
    try:
        idx1, cnt1 = _speculate(ctx, up, c)
        idx2, cnt2 = _speculate(ctx, up, c)
    finally:
        ctx.ig_set_wait_limit(0)
    idx3, cnt3 = _speculate(ctx, up, c)          # ordinary route again, on the records the other left
    assert ctx.ig_check_status() == ig.IG_OK
    for idx, cnt in ((idx1, cnt1), (idx2, cnt2), (idx3, cnt3)):
        assert np.array_equal(cnt, cnt0)
        for i in range(len(cnt0)):
            assert np.array_equal(idx[i, :cnt0[i]], idx0[i, :cnt0[i]])
    ref = run_oracle(c, attend=False)
    compare_selection(idx0, cnt0, ref, c.w.alpha)


def test_split_pairs_clamp_and_flag_long_lists(ctx):
    import paper_2406_19707_amd as ig
    from ig_gpu import Uploaded
    c = make_case(shape(2, 2, 8, 9000, 0.6), gain=1.0)        # gain 1: nearly every token is kept
    up = Uploaded(ctx, c)
    full_idx, full_cnt = _speculate(ctx, up, c)
    assert ctx.ig_check_status() == ig.IG_OK and full_cnt.max() > 5000
    idx, cnt = _speculate(ctx, up, c, stride=3000)
    assert ctx.ig_check_status() == ig.IG_ECAPACITY
    assert ctx.ig_check_status() == ig.IG_OK
    for i in range(len(cnt)):
        assert cnt[i] == min(full_cnt[i], 3000)
        assert np.array_equal(idx[i, :cnt[i]], full_idx[i, :cnt[i]])


def test_split_pairs_are_deterministic(ctx):
    from ig_gpu import Uploaded
    c = make_case(shape(5, 2, 40, 32768, 0.4), gain=40.0)
    up = Uploaded(ctx, c)
    idx0, cnt0 = _speculate(ctx, up, c)
    for _ in range(10):
        idx, cnt = _speculate(ctx, up, c)
        assert np.array_equal(cnt, cnt0) and np.array_equal(idx, idx0)
